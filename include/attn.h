/*
 * attn.h -- C ABI of the MI355X (gfx950) exact-attention library.
 *
 * The library computes, for B*H independent problems of N tokens and head
 * dimension d (paper: Section 2.2 and Appendix B.3),
 *
 *     S = tau * Q K^T,  S_masked = MASK(S),  P = softmax(S_masked) row-wise,
 *     P_dropped = dropout(P, p_drop),        O = P_dropped V,
 *
 * without ever writing S or P to memory (tiling with an online softmax,
 * Section 3.1 / Algorithm 1 and 2), and the gradients dQ, dK, dV of a scalar
 * loss given dO by recomputing S and P tile by tile from Q, K, V and the saved
 * per-row statistic (Appendix B.2 and B.4 / Algorithm 4).  A block mask turns
 * both passes into the block-sparse variant (Section 3.3 / Algorithm 5).
 *
 * General conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The
 *     library never allocates, frees, or keeps a pointer after a call returns.
 *   - Q, K, V, O, dO, dQ, dK, dV are [B, H, N, d] arrays of 16-bit floats
 *     (fp16 or bf16, chosen by attn_params.dtype) with d contiguous; the
 *     element strides of the b, h and n axes are given in attn_params and are
 *     shared by all of these tensors (all three 0 = densely packed).
 *   - LSE is a packed [B, H, N] float array: L_i = m_i + ln(l_i), the natural
 *     logsumexp of row i of the scaled, masked logits.  It replaces the pair
 *     (l, m) that Algorithm 2 saves; P_ij = exp(S_ij - L_i).
 *   - Calls are asynchronous on attn_params.stream (a hipStream_t, may be
 *     NULL for the default stream), never synchronise the device, and may be
 *     issued concurrently from several host threads.
 *   - Outputs are fully overwritten; the caller need not clear them.
 *   - A query row that sees no key (through a block mask, or a padded position
 *     under key_lengths) gets O = 0, LSE = -inf and contributes zero gradients.
 *   - All argument checks happen on the host before anything is launched:
 *     sizes, strides (rows 16-byte aligned, non-overlapping: the axes of size
 *     > 1 must nest by stride, as in [B,H,N,d] or a [B,N,H,d] view), tensor
 *     pointers (non-NULL, 16-byte aligned), scale, dropout, mask, workspace.
 *     Functions return ATTN_OK (0) or a negative attn_status; they never
 *     abort, throw, or print.
 *   - Every element of the input tensors must be finite, padded positions
 *     (under key_lengths) included: they enter the matrix products with weight
 *     zero, and 0 * inf is not zero.
 *
 * Supported in this version: d in {16, 32, 64, 128}; any N >= 1 for the dense entry
 * points (a last block of fewer than 128 tokens is handled inside the kernels:
 * nothing outside the [B,H,N,d] tensors is read or written), N a multiple of
 * 128 for the block-sparse ones; tau finite and > 0; 0 <= p_drop < 1;
 * mask_block == 128.
 *
 * Which kernel a call takes depends on head dimension, length, masks and the
 * number of heads; every choice computes the same operation to the same
 * tolerance.  attn_debug_set_variant overrides the choice for comparisons and
 * tests; its initial values come from two environment variables read once, when
 * the first call needs them: ATTN_FWD_VARIANT=base|pp and ATTN_DKV_VARIANT=rs|fr|w64.
 * Unset, the library picks by measurement.
 */
#ifndef ATTN_H_
#define ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ATTN_OK = 0,
  ATTN_ERR_NULL = -1,       /* a required pointer is NULL */
  ATTN_ERR_SHAPE = -2,      /* B, H, N out of range, bad strides, misaligned tensor, block-sparse with N % 128 != 0 */
  ATTN_ERR_DTYPE = -3,      /* dtype is neither ATTN_FP16 nor ATTN_BF16 */
  ATTN_ERR_HEADDIM = -4,    /* d not in {16, 32, 64, 128} */
  ATTN_ERR_DROPOUT_P = -5,  /* p_drop not in [0, 1) or NaN */
  ATTN_ERR_SCALE = -6,      /* softmax_scale not finite or <= 0 */
  ATTN_ERR_WORKSPACE = -7,  /* workspace NULL, misaligned (256 B) or too small */
  ATTN_ERR_MASK = -8,       /* mask_block != 128 or negative mask stride */
  ATTN_ERR_LAUNCH = -9      /* the HIP runtime refused the launch */
} attn_status;

enum { ATTN_FP16 = 0, ATTN_BF16 = 1 };

typedef struct {
  int32_t B, H, N, d;        /* problem sizes */
  int32_t dtype;             /* ATTN_FP16 or ATTN_BF16 */
  int64_t stride_b;          /* element strides of the [B,H,N,d] tensors;    */
  int64_t stride_h;          /*   all three zero means packed                */
  int64_t stride_n;          /*   (stride_n >= d, d itself has stride 1)     */
  float softmax_scale;       /* tau: multiplies Q K^T before mask and softmax */
  int32_t causal;            /* != 0: key j is visible to query i iff j <= i */
  float dropout_p;           /* p_drop in [0,1), applied rounded down to a multiple of 1/256;
                                below 1/256 the generator is switched off      */
  uint64_t seed;             /* Philox key   (the saved generator state R)   */
  uint64_t offset;           /* low 32 bits enter the Philox counter         */
  int32_t o_fp32;            /* != 0: O is read/written as float32 [B,H,N,d] packed
                                with the same strides, instead of dtype      */
  void* stream;              /* hipStream_t, borrowed for the call           */
  const int32_t* key_lengths; /* NULL, or device int32 [B]: key-padding mask (the MASK example of
                                Appendix B.3).  Tokens of batch b at positions >= key_lengths[b]
                                are padding: they are not attended to, their O is 0, their LSE
                                -inf and all gradients at those positions are 0.  Lengths are clamped to [0, N].
                                Sequences of any length are run by padding N up to a multiple
                                of 128 and passing the true lengths here.                    */
} attn_params;

/*
 * Dropout mask (bit-exact contract, shared with nothing but this text):
 * Philox-4x32 with 10 rounds (Salmon et al., SC'11), key = (seed low word,
 * seed high word), counter = (j / 16, i, b * H + h, offset low word) for query
 * row i and key column j of head (b, h); element (i, j) takes the 8-bit
 * field f = j % 16 of the 128-bit output (byte f % 4, i.e. bits [8 (f % 4),
 * 8 (f % 4) + 7], of output word f / 4) and is KEPT iff field >= T, with
 * T = floor((double)dropout_p * 2^8).  The dropout applied is therefore the one
 * with probability T / 256, dropout_p rounded down to a multiple of 1/256
 * (0.1 -> 25/256; below 1/256 nothing is dropped), and kept probabilities are
 * multiplied by 256 / (256 - T), the reciprocal of the keep probability, so
 * that the mask has expectation one.  One generator call decides sixteen
 * consecutive keys of a query.  The mask depends on indices only, so the
 * backward pass regenerates it (Appendix B.4, obs. 1).
 */

/*
 * Forward pass (Algorithm 2; Algorithm 1 when causal = 0 and dropout_p = 0).
 *   Q, K, V : in,  [B,H,N,d] dtype
 *   O       : out, [B,H,N,d] dtype (or float32 when o_fp32)
 *   LSE     : out, [B,H,N] float32, packed
 */
int attn_fwd(const attn_params* p, const void* Q, const void* K, const void* V,
             void* O, float* LSE);

/*
 * Bytes of scratch that attn_bwd needs for these params: two floats per query
 * row (D_i of Eq. (4), Appendix B.2, and the row statistic in base 2), i.e. the
 * O(N) additional memory of Theorem 1; never quadratic in N.  Returns 0 if the
 * params are invalid.
 */
size_t attn_bwd_workspace_bytes(const attn_params* p);

/*
 * Same for attn_blocksparse_bwd (and attn_bwd_timed with a mask): additionally holds the
 * per-column block counts and fp32 dK/dV accumulators used when a mask column keeps so many
 * blocks (a "global token" column) that its work is split over several workgroups.  Still
 * linear in B*H*N*d.  Returns 0 if the params are invalid.
 */
size_t attn_blocksparse_bwd_workspace_bytes(const attn_params* p);

/*
 * Backward pass (Algorithm 4, with D_i = rowsum(dO_i o O_i) from Eq. (4) of
 * Appendix B.2).
 *   Q, K, V, O, dO : in,  [B,H,N,d] (O as written by attn_fwd with the same params)
 *   LSE            : in,  [B,H,N] float32 from attn_fwd
 *   dQ, dK, dV     : out, [B,H,N,d] dtype
 *   workspace      : device scratch, 256-byte aligned, >= attn_bwd_workspace_bytes(p);
 *                    contents on entry are ignored and on exit unspecified
 */
int attn_bwd(const attn_params* p, const void* Q, const void* K, const void* V,
             const void* O, const void* dO, const float* LSE,
             void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes);

/*
 * attn_bwd for callers that can neither allocate device memory nor pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as attn_bwd (bit-identical), except that the two row vectors live in a
 * fixed array inside the library, ATTN_STATIC_SCRATCH_BYTES per GPU, held from the first
 * use on that GPU until the process ends.  The call allocates and frees nothing.  Problems whose
 * attn_bwd_workspace_bytes(p) exceeds ATTN_STATIC_SCRATCH_BYTES (more than 2^20 query rows
 * over all heads, counted in whole blocks of 128 per head) return ATTN_ERR_WORKSPACE.  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 * threads) race and give wrong gradients; calls on one stream, or otherwise ordered, are safe,
 * and no call reads what an earlier one left there.  The device that is current when the call
 * is made must be the one that owns the tensors and the stream.
 */
#define ATTN_STATIC_SCRATCH_BYTES (8u << 20)
int attn_bwd_static(const attn_params* p, const void* Q, const void* K, const void* V,
                    const void* O, const void* dO, const float* LSE,
                    void* dQ, void* dK, void* dV);

/*
 * Block-sparse forward (Section 3.3, Algorithm 5): as attn_fwd, but entry
 * (i, j) is additionally masked out unless
 * block_mask[(i / mask_block) * T + (j / mask_block)] != 0, T = N / mask_block;
 * tiles whose block is zero are skipped, not computed.
 *   block_mask    : in, device uint8 [T, T] row-major (per head if mask_stride_h != 0)
 *   mask_block    : must be 128
 *   mask_stride_h : bytes between the masks of consecutive heads h (0 = one
 *                   mask shared by all heads; batches always share)
 */
int attn_blocksparse_fwd(const attn_params* p, const uint8_t* block_mask, int32_t mask_block,
                         int64_t mask_stride_h, const void* Q, const void* K, const void* V,
                         void* O, float* LSE);

/*
 * Block-sparse backward: Algorithm 4 restricted to the non-zero blocks (the
 * paper states only that the backward skips the same blocks, Section 3.3).
 * Arguments as attn_bwd plus the mask arguments of attn_blocksparse_fwd; the workspace must
 * hold attn_blocksparse_bwd_workspace_bytes(p) bytes.  dK and dV of mask columns that are split
 * over several workgroups are summed with fp32 atomics, so their last bits may differ from run
 * to run; everything else is bit-reproducible.
 */
int attn_blocksparse_bwd(const attn_params* p, const uint8_t* block_mask, int32_t mask_block,
                         int64_t mask_stride_h, const void* Q, const void* K, const void* V,
                         const void* O, const void* dO, const float* LSE,
                         void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes);

/*
 * Profiling aid for the backward pass (Algorithm 4 as attn_bwd / attn_blocksparse_bwd run it):
 * identical to attn_bwd when block_mask is NULL and to attn_blocksparse_bwd otherwise, and in
 * addition records the caller's four hipEvent_t handles on p->stream: events[0] and events[1]
 * before the first launch (two handles for one instant: an earlier version had a preparation
 * launch between them; D = rowsum(dO o O) is now computed inside the dQ kernel), events[2] after
 * the dQ kernel, events[3] after the dK/dV kernel.  The events stay owned by the caller.
 */
int attn_bwd_timed(const attn_params* p, const uint8_t* block_mask, int32_t mask_block,
                   int64_t mask_stride_h, const void* Q, const void* K, const void* V,
                   const void* O, const void* dO, const float* LSE,
                   void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                   void* const* events);

/*
 * Test hook: writes the dropout keep mask the kernels use, keep[b][h][i][j] in
 * {0, 1}, as a packed device uint8 [B,H,N,N] array (N*N bytes per head: only
 * for small problems).  Uses B, H, N, dropout_p, seed, offset, stream of p.
 */
int attn_debug_dropout_mask(const attn_params* p, uint8_t* keep);

/*
 * Measurement aid, outside the paper's operation: launches on `stream` a kernel that
 * only issues 32x32x16 matrix instructions of the given dtype on register operands
 * (2048 workgroups of 4 wavefronts, 4 * iters instructions per wavefront), so a
 * benchmark that times the launch can quote the matrix rate this GPU sustains under
 * load next to the published peak.  operand_sets = 1: every instruction reads the same
 * two registers (fewest bits change between instructions: the highest clock the GPU
 * holds); operand_sets = 4: consecutive instructions read four different pseudo-random
 * operand pairs in turn, as the tile products of a real kernel do.  sink: device pointer
 * to at least one float, never written in practice; *flops (host pointer, may be NULL)
 * receives the number of floating-point operations launched.  iters in [1, 2^20].
 * Asynchronous.
 */
int attn_debug_mfma_rate(int32_t dtype, int32_t iters, int32_t operand_sets, float* sink, void* stream,
                         double* flops);

/*
 * Measurement aid: which kernels attn_fwd / attn_bwd (sparse = 0) or the block-sparse
 * entry points (sparse != 0) would launch for these params, without launching anything.
 * *fwd_kernel: 0 = free-running forward kernel, 1 = two-group forward kernel.
 * *dkv_kernel: 0 = role-split dK/dV kernel, 1 = one-wavefront kernel (d <= 64),
 * 2 = one-wavefront kernel for d = 128 (32 keys per wavefront), 3 = the same with 64 keys
 * per wavefront.  (The dQ kernel is the same for every problem.)
 */
int attn_debug_kernel_choice(const attn_params* p, int32_t sparse, int32_t* fwd_kernel, int32_t* dkv_kernel);

/*
 * Test and comparison hook, outside the paper's operation: which kernel serves the calls that
 * have a choice.  fwd_variant: 0 = by measurement, 1 = free-running forward kernel, 2 = two-group
 * forward kernel (where both exist).  dkv_variant: 0 = by measurement, 1 = role-split dK/dV kernel
 * wherever it exists, 2 = one-wavefront dK/dV kernels with 32 keys per wavefront only, 3 = the
 * 64-keys-per-wavefront dK/dV kernel wherever it exists (d = 128, no dropout, N >= 512, N % 32 == 0).
 * -1 leaves a setting unchanged.  Process-wide and thread-safe; affects calls issued afterwards.
 */
int attn_debug_set_variant(int32_t fwd_variant, int32_t dkv_variant);

/* Static, human-readable text for a status code. */
const char* attn_strerror(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATTN_H_ */
