"""MI355X-native IO-aware exact attention (forward, backward, causal, dropout, block-sparse).

The compute path is the HIP library under csrc/ reached through the C ABI
declared in include/attn.h; `binding` marshals arguments only.  `inputs`
holds the seeded synthetic-input generators.
"""
__version__ = "0.1.0"
