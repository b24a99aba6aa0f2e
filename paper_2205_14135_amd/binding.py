"""ctypes binding for libattn_gfx950.so: same entry points as include/attn.h.

Argument marshalling only: torch supplies device memory and the current
stream, every step of the computation runs inside the HIP library.  There is
no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_gfx950.so")

ATTN_FP16, ATTN_BF16 = 0, 1

SYMBOLS = (
    "attn_fwd", "attn_bwd_workspace_bytes", "attn_blocksparse_bwd_workspace_bytes", "attn_bwd", "attn_bwd_static", "attn_blocksparse_fwd",
    "attn_blocksparse_bwd", "attn_bwd_timed", "attn_debug_dropout_mask", "attn_debug_mfma_rate", "attn_debug_kernel_choice", "attn_debug_set_variant", "attn_strerror",
    "attn_version",
)


class AttnParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
        ("softmax_scale", ctypes.c_float),
        ("causal", ctypes.c_int32),
        ("dropout_p", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("offset", ctypes.c_uint64),
        ("o_fp32", ctypes.c_int32),
        ("stream", ctypes.c_void_p),
        ("key_lengths", ctypes.c_void_p),
    ]


class AttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def load() -> ctypes.CDLL:
    """Loads the built library (build it first with `python -m paper_2205_14135_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2205_14135_amd.build`; "
            "there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    P = ctypes.POINTER(AttnParams)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    lib.attn_fwd.argtypes = [P, vp, vp, vp, vp, vp]
    lib.attn_fwd.restype = ctypes.c_int
    lib.attn_bwd_workspace_bytes.argtypes = [P]
    lib.attn_bwd_workspace_bytes.restype = sz
    lib.attn_blocksparse_bwd_workspace_bytes.argtypes = [P]
    lib.attn_blocksparse_bwd_workspace_bytes.restype = sz
    lib.attn_bwd.argtypes = [P] + [vp] * 9 + [vp, sz]
    lib.attn_bwd.restype = ctypes.c_int
    lib.attn_bwd_static.argtypes = [P] + [vp] * 9
    lib.attn_bwd_static.restype = ctypes.c_int
    lib.attn_blocksparse_fwd.argtypes = [P, vp, i32, i64, vp, vp, vp, vp, vp]
    lib.attn_blocksparse_fwd.restype = ctypes.c_int
    lib.attn_blocksparse_bwd.argtypes = [P, vp, i32, i64] + [vp] * 9 + [vp, sz]
    lib.attn_blocksparse_bwd.restype = ctypes.c_int
    lib.attn_bwd_timed.argtypes = [P, vp, i32, i64] + [vp] * 9 + [vp, sz, ctypes.POINTER(vp)]
    lib.attn_bwd_timed.restype = ctypes.c_int
    lib.attn_debug_dropout_mask.argtypes = [P, vp]
    lib.attn_debug_dropout_mask.restype = ctypes.c_int
    lib.attn_debug_mfma_rate.argtypes = [i32, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.attn_debug_kernel_choice.argtypes = [P, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.attn_debug_kernel_choice.restype = ctypes.c_int
    lib.attn_debug_mfma_rate.restype = ctypes.c_int
    lib.attn_debug_set_variant.argtypes = [i32, i32]
    lib.attn_debug_set_variant.restype = ctypes.c_int
    lib.attn_strerror.argtypes = [ctypes.c_int]
    lib.attn_strerror.restype = ctypes.c_char_p
    lib.attn_version.argtypes = []
    lib.attn_version.restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().attn_strerror(int(status)).decode()


def version() -> int:
    return int(load().attn_version())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return ATTN_FP16
    if t.dtype == torch.bfloat16:
        return ATTN_BF16
    raise TypeError(f"Q/K/V must be float16 or bfloat16, got {t.dtype}")


def make_params(Q: torch.Tensor, softmax_scale: float, causal: bool = False, dropout_p: float = 0.0,
                seed: int = 0, offset: int = 0, o_fp32: bool = False, stream=None,
                key_lengths: Optional[torch.Tensor] = None) -> AttnParams:
    """Params for [B,H,N,d] tensors laid out like Q (d contiguous)."""
    if Q.dim() != 4 or Q.stride(3) != 1:
        raise ValueError("expected a [B,H,N,d] tensor with contiguous last axis")
    B, H, N, d = Q.shape
    if stream is None:
        stream = torch.cuda.current_stream(Q.device).cuda_stream if Q.is_cuda else 0
    p = AttnParams()
    p.B, p.H, p.N, p.d = B, H, N, d
    p.dtype = _dtype_code(Q)
    p.stride_b, p.stride_h, p.stride_n = Q.stride(0), Q.stride(1), Q.stride(2)
    p.softmax_scale = float(softmax_scale)
    p.causal = int(bool(causal))
    p.dropout_p = float(dropout_p)
    p.seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    p.offset = int(offset) & 0xFFFFFFFFFFFFFFFF
    p.o_fp32 = int(bool(o_fp32))
    p.stream = ctypes.c_void_p(int(stream))
    if key_lengths is not None:
        if key_lengths.dtype != torch.int32 or key_lengths.shape != (B,) or not key_lengths.is_contiguous():
            raise TypeError("key_lengths must be a contiguous int32 tensor of shape [B]")
        p.key_lengths = ctypes.c_void_p(key_lengths.data_ptr())
    return p


def _same_layout(ref: torch.Tensor, *others: torch.Tensor) -> None:
    for t in others:
        if t.shape != ref.shape or t.stride() != ref.stride() or t.device != ref.device:
            raise ValueError("all [B,H,N,d] tensors must share shape, strides and device")


def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _check(status: int, where: str) -> None:
    if status != 0:
        raise AttnError(status, where)


def _mask_args(block_mask: torch.Tensor, H: int):
    if block_mask.dtype != torch.uint8 or not block_mask.is_contiguous():
        raise TypeError("block_mask must be a contiguous uint8 tensor [T,T] or [H,T,T]")
    if block_mask.dim() == 2:
        return 0
    if block_mask.dim() == 3 and block_mask.shape[0] == H:
        return block_mask.stride(0)
    raise ValueError("block_mask must be [T,T] or [H,T,T]")


def attn_fwd(Q, K, V, *, softmax_scale, causal=False, dropout_p=0.0, seed=0, offset=0,
             o_fp32=False, out=None, lse=None, stream=None, key_lengths=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """O, LSE = attention forward.  Outputs are allocated with torch unless given."""
    _same_layout(Q, K, V)
    p = make_params(Q, softmax_scale, causal, dropout_p, seed, offset, o_fp32, stream, key_lengths)
    B, H, N, d = Q.shape
    if out is None:
        out = torch.empty_strided(Q.shape, Q.stride(), dtype=torch.float32 if o_fp32 else Q.dtype,
                                  device=Q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _check(load().attn_fwd(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(out), _ptr(lse)), "attn_fwd")
    return out, lse


def attn_bwd_workspace_bytes(p: AttnParams) -> int:
    return int(load().attn_bwd_workspace_bytes(ctypes.byref(p)))


def attn_blocksparse_bwd_workspace_bytes(p: AttnParams) -> int:
    return int(load().attn_blocksparse_bwd_workspace_bytes(ctypes.byref(p)))


def _workspace(p: AttnParams, device, workspace, sparse=False):
    need = attn_blocksparse_bwd_workspace_bytes(p) if sparse else attn_bwd_workspace_bytes(p)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def attn_bwd(Q, K, V, O, dO, LSE, *, softmax_scale, causal=False, dropout_p=0.0, seed=0, offset=0,
             o_fp32=False, workspace=None, grads=None, stream=None, key_lengths=None):
    """dQ, dK, dV = attention backward (O, LSE from attn_fwd with the same options)."""
    _same_layout(Q, K, V, dO)
    p = make_params(Q, softmax_scale, causal, dropout_p, seed, offset, o_fp32, stream, key_lengths)
    if grads is None:
        grads = tuple(torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
                      for _ in range(3))
    dQ, dK, dV = grads
    workspace, nbytes = _workspace(p, Q.device, workspace)
    _check(load().attn_bwd(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE),
                           _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), nbytes), "attn_bwd")
    return dQ, dK, dV


STATIC_SCRATCH_BYTES = 8 << 20


def attn_bwd_static(Q, K, V, O, dO, LSE, grads, *, softmax_scale, causal=False, dropout_p=0.0, seed=0,
                    offset=0, o_fp32=False, stream=None, key_lengths=None):
    """attn_bwd on the library's built-in scratch: the caller passes the outputs, nothing is allocated."""
    _same_layout(Q, K, V, dO)
    p = make_params(Q, softmax_scale, causal, dropout_p, seed, offset, o_fp32, stream, key_lengths)
    dQ, dK, dV = grads
    _check(load().attn_bwd_static(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE),
                                  _ptr(dQ), _ptr(dK), _ptr(dV)), "attn_bwd_static")
    return dQ, dK, dV


def attn_blocksparse_fwd(Q, K, V, block_mask, *, softmax_scale, mask_block=128, causal=False,
                         dropout_p=0.0, seed=0, offset=0, o_fp32=False, out=None, lse=None, stream=None,
                         key_lengths=None):
    _same_layout(Q, K, V)
    p = make_params(Q, softmax_scale, causal, dropout_p, seed, offset, o_fp32, stream, key_lengths)
    B, H, N, d = Q.shape
    msh = _mask_args(block_mask, H)
    if out is None:
        out = torch.empty_strided(Q.shape, Q.stride(), dtype=torch.float32 if o_fp32 else Q.dtype,
                                  device=Q.device)
    if lse is None:
        lse = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _check(load().attn_blocksparse_fwd(ctypes.byref(p), _ptr(block_mask), int(mask_block), int(msh),
                                       _ptr(Q), _ptr(K), _ptr(V), _ptr(out), _ptr(lse)),
           "attn_blocksparse_fwd")
    return out, lse


def attn_blocksparse_bwd(Q, K, V, O, dO, LSE, block_mask, *, softmax_scale, mask_block=128, causal=False,
                         dropout_p=0.0, seed=0, offset=0, o_fp32=False, workspace=None, grads=None,
                         stream=None, key_lengths=None):
    _same_layout(Q, K, V, dO)
    p = make_params(Q, softmax_scale, causal, dropout_p, seed, offset, o_fp32, stream, key_lengths)
    msh = _mask_args(block_mask, Q.shape[1])
    if grads is None:
        grads = tuple(torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
                      for _ in range(3))
    dQ, dK, dV = grads
    workspace, nbytes = _workspace(p, Q.device, workspace, sparse=True)
    _check(load().attn_blocksparse_bwd(ctypes.byref(p), _ptr(block_mask), int(mask_block), int(msh),
                                       _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE),
                                       _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), nbytes),
           "attn_blocksparse_bwd")
    return dQ, dK, dV


def attn_bwd_timed(Q, K, V, O, dO, LSE, events, *, softmax_scale, block_mask=None, mask_block=128,
                   causal=False, dropout_p=0.0, seed=0, offset=0, o_fp32=False, workspace=None,
                   grads=None, stream=None, key_lengths=None):
    """attn_bwd / attn_blocksparse_bwd that also records four caller-owned hipEvent_t handles
    (ints) on the stream: two before the first launch, one after dQ, one after dK/dV."""
    _same_layout(Q, K, V, dO)
    p = make_params(Q, softmax_scale, causal, dropout_p, seed, offset, o_fp32, stream, key_lengths)
    msh = 0 if block_mask is None else _mask_args(block_mask, Q.shape[1])
    if grads is None:
        grads = tuple(torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
                      for _ in range(3))
    dQ, dK, dV = grads
    workspace, nbytes = _workspace(p, Q.device, workspace, sparse=block_mask is not None)
    ev = (ctypes.c_void_p * 4)(*[ctypes.c_void_p(int(e)) for e in events])
    _check(load().attn_bwd_timed(ctypes.byref(p), _ptr(block_mask), int(mask_block), int(msh),
                                 _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(dO), _ptr(LSE),
                                 _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(workspace), nbytes, ev),
           "attn_bwd_timed")
    return dQ, dK, dV


def attn_debug_dropout_mask(B, H, N, dropout_p, seed, offset, device="cuda") -> torch.Tensor:
    """uint8 [B,H,N,N] keep mask as the kernels generate it (small problems only)."""
    dummy = torch.empty((B, H, N, 64), dtype=torch.float16, device=device)
    p = make_params(dummy, 1.0, False, dropout_p, seed, offset)
    keep = torch.empty((B, H, N, N), dtype=torch.uint8, device=device)
    _check(load().attn_debug_dropout_mask(ctypes.byref(p), _ptr(keep)), "attn_debug_dropout_mask")
    return keep


FWD_KERNELS = ("fwd_kernel", "fwd_pp_kernel")
DKV_KERNELS = ("dkv_rs_kernel", "dkv_fr_kernel", "dkv_fr128_kernel", "dkv_w64_kernel")


def attn_debug_kernel_choice(p: AttnParams, sparse: bool = False) -> Tuple[str, str]:
    """Names of the forward and dK/dV kernels the library would launch for these params."""
    f, k = ctypes.c_int32(), ctypes.c_int32()
    _check(load().attn_debug_kernel_choice(ctypes.byref(p), int(bool(sparse)), ctypes.byref(f), ctypes.byref(k)),
           "attn_debug_kernel_choice")
    return FWD_KERNELS[f.value], DKV_KERNELS[k.value]


def attn_debug_mfma_rate(dtype: str, iters: int, sink: torch.Tensor, operand_sets: int = 1) -> float:
    """Launches the matrix-instruction-only kernel on the current stream; returns the FLOPs launched."""
    fl = ctypes.c_double()
    code = {"fp16": 0, "bf16": 1}[dtype]
    stream = ctypes.c_void_p(int(torch.cuda.current_stream(sink.device).cuda_stream))
    _check(load().attn_debug_mfma_rate(code, int(iters), int(operand_sets), _ptr(sink), stream, ctypes.byref(fl)),
           "attn_debug_mfma_rate")
    return float(fl.value)


FWD_VARIANTS = {"auto": 0, "base": 1, "pp": 2}
DKV_VARIANTS = {"auto": 0, "rs": 1, "fr": 2, "w64": 3}


def attn_debug_set_variant(fwd: Optional[str] = None, dkv: Optional[str] = None) -> None:
    """Overrides the kernel choice for the calls that follow (None leaves a setting unchanged)."""
    f = -1 if fwd is None else FWD_VARIANTS[fwd]
    k = -1 if dkv is None else DKV_VARIANTS[dkv]
    _check(load().attn_debug_set_variant(f, k), "attn_debug_set_variant")
