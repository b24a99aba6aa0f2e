// Forward pass of IO-aware exact attention for gfx950 (MI355X).
//
// What is computed is Algorithm 2 of the paper (Appendix B.3): S = tau Q K^T, mask, online
// softmax with running row max m and row sum l, dropout on the unnormalised probabilities,
// O accumulation with rescaling, and the saved statistic L = m + ln l.  The loop order is
// NOT the paper's: a workgroup owns a 128-row Q tile (4 wavefronts x 32 rows), keeps O, m, l
// in registers for the whole sweep over K/V tiles and writes O and L exactly once, so O, m, l
// never travel to HBM between tiles (the paper's K/V-outer order re-reads and re-writes them
// on every pass).  K/V tiles of 64 keys are staged in LDS.
//
// Online softmax, two departures from the printed recurrence that leave the result the same up
// to rounding.  (1) The reference m of a row is moved (and O, l rescaled) only when a tile's
// maximum exceeds it by more than 2^kLazyRescale: any reference gives the same softmax in exact
// arithmetic, and most tiles then skip the rescaling of the whole O accumulator.  (2) O is divided
// by the sum of the probabilities AS ROUNDED to 16 bits for the second product, not by l: O is
// then a convex combination of V rows with exactly the weights that were used, which is what
// keeps a lagging reference accurate (with the exact l a peaked row would see the rounding of its
// one large weight in full).  The saved statistic L = m + ln l uses the exact fp32 l.
//
// Register layout trick: the kernel computes S^T = K Q^T with 32x32x16 MFMA, so that a lane
// holds 16 keys of ONE query (accumulator register i of key block kb is key
// 32 kb + 8 (i/4) + 4 (lane/32) + i%4, query lane%32).  Row max / row sum are then in-lane
// reductions plus one exchange with lane^32, the rescale factor is a per-lane scalar, and the
// probabilities are already in the B-operand layout of the second product O^T = V^T P^T.
// V^T fragments come from the row-major V tile in LDS through the gfx950 transposing LDS read.
#include "attn_common.h"
#include "attn_tiles.h"

#include <cstdlib>

namespace attn {
namespace {

constexpr int BR = 128;  // query rows per workgroup
constexpr int BC = 64;   // keys per K/V tile
constexpr int NT = 256;  // threads

template <typename T, int D, bool CAUSAL, bool DROPOUT, bool SPARSE>
__global__ __launch_bounds__(NT, D <= 64 ? 3 : 2) void fwd_kernel(const KArgs a) {
  typedef typename Vec<T>::x8 T8;
  typedef typename Vec<T>::x4 T4;
  constexpr int KK = D / 16;        // MFMA k-steps over the head dimension
  constexpr int DB = D / 32;        // 32-row blocks of O^T

  // double buffered, unpadded XOR-swizzled tiles, filled by asynchronous global-to-LDS copies
  __shared__ __attribute__((aligned(16))) T Ks[2][BC * D];
  __shared__ __attribute__((aligned(16))) T Vs[2][BC * D];

  const int item = xcd_item(a.n_items, a.chunk);
  if (item < 0) return;
  const int n_qt = a.T;   // ceil(N / BR): the last block may be ragged
  // Work item = (head, row block), heavy (late) blocks first under a causal mask.  For dense
  // causal d = 64 problems an item is the pair (n_qt - 1 - q, q), one block per pass, so that
  // every workgroup does the same amount of work.
  constexpr bool PAIRED = CAUSAL && !SPARSE && D == 64;
  const int n_per_head = PAIRED ? (n_qt + 1) / 2 : n_qt;
  const int bh = item / n_per_head;
  const int q_item = item % n_per_head;
  const int n_pass = PAIRED && q_item != n_qt - 1 - q_item ? 2 : 1;
#pragma clang loop unroll(disable)
  for (int pass = 0; pass < n_pass; ++pass) {
  if (pass) __syncthreads();   // the tile buffers staged the first block's output rows
  const int qt = PAIRED ? (pass ? q_item : n_qt - 1 - q_item) : (CAUSAL ? n_qt - 1 - q_item : q_item);
  const int b = bh / a.H, h = bh % a.H;
  const int64_t head_off = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const T* __restrict__ Qg = (const T*)a.Q + head_off;
  const T* __restrict__ Kg = (const T*)a.K + head_off;
  const T* __restrict__ Vg = (const T*)a.V + head_off;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int q0 = qt * BR + wave * 32;  // first query row of this wavefront
  // this lane's query row; lanes beyond a ragged end work on a copy of the last row and store nothing
  const bool row_ok = q0 + r < a.N;
  const int qi = min(q0 + r, a.N - 1);

  // Q^T fragments (B operand): lane holds query qi, d = 16 kk + 8 g .. +7
  T8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    if (D == 32 && 16 * kk + 8 * g >= a.dvalid) {   // head dimension 16: the upper columns are zeros
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[kk][e] = (T)0.f;
    } else {
      qf[kk] = *(const T8*)(Qg + (int64_t)qi * a.sn + 16 * kk + 8 * g);
    }
  }

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  float m_run = -INFINITY;  // reference of the row's probabilities, base-2 domain: lags the running
                            // maximum of the scaled logits by at most kLazyRescale
  float l_run = 0.f;        // this lane's share of the exact running row sum (for the saved statistic)
  float lr_run = 0.f;       // its share of the sum of the rounded probabilities (normalises O)

  // key-padding mask: keys >= len are masked, rows >= len produce O = 0, LSE = -inf
  const int len = a.klen ? min(max(a.klen[b], 0), a.N) : a.N;
  TileIter<SPARSE> it;
  {
    int lim;
    if constexpr (SPARSE) lim = min(CAUSAL ? qt + 1 : a.T, (len + 127) / 128);
    else lim = CAUSAL ? min(2 * qt + 2, (len + BC - 1) / BC) : (len + BC - 1) / BC;   // len <= N
    if (qt * BR >= len) lim = 0;
    it.init(SPARSE ? a.mask + (int64_t)h * a.mask_sh + (int64_t)qt * a.T : nullptr, 1, 0, lim);
  }

  TrOffsets<D> tro;
  tro.init();
  TileAsync<T, D, NT / 64> dma;
  dma.init(a.sn, wave, D == 32 ? a.dvalid : D);
  if (D == 32 && a.dvalid < D) {   // the copies leave columns >= 16 of the tile buffers untouched
    zero_tiles(&Ks[0][0], 2 * BC * D);
    zero_tiles(&Vs[0][0], 2 * BC * D);
    __syncthreads();
  }

  const float c = a.scale_log2;
  int jt = it.next();
  int buf = 0;
  if (jt >= 0) {
    dma.copy_rows(Kg, a.sn, jt * BC, a.N, Ks[0]);
    dma.copy_rows(Vg, a.sn, jt * BC, a.N, Vs[0]);
  }
  wait_async_copies();
  __syncthreads();   // tile 0 has landed, and so have the Q fragments
  while (jt >= 0) {
    const int jn = it.next();
    if (jn >= 0) {   // the next tile streams into the other buffer while this one is used
      dma.copy_rows(Kg, a.sn, jn * BC, a.N, Ks[buf ^ 1]);
      dma.copy_rows(Vg, a.sn, jn * BC, a.N, Vs[buf ^ 1]);
    }
    const T* Kt = Ks[buf];
    const T* Vt = Vs[buf];

    const int k0 = jt * BC;
    const bool wave_active = !CAUSAL || k0 <= q0 + 31;
    if (wave_active) {
      // ---- S^T = K Q^T  (64 keys x 32 queries per wavefront); operand reads run PF fragments
      // ahead of their MFMA (the scheduling barriers keep that distance)
      constexpr int PF = 4;
      f32x16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
      {
        auto k_frag = [&](int f) {   // f = 2 kk + kb
          return *(const T8*)(Kt + lds_off<D>(32 * (f & 1) + r, 2 * (f >> 1) + g));
        };
        T8 ring[PF];
#pragma unroll
        for (int f = 0; f < PF; ++f) ring[f] = k_frag(f);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 2 * KK; ++f) {
          const T8 cur = ring[f % PF];
          s[f & 1] = mfma32(cur, qf[f >> 1], s[f & 1]);
          if (f + PF < 2 * KK) ring[f % PF] = k_frag(f + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- masks, online softmax, dropout; P^T fragments (B operand) for the second product
      T8 pf[4];
      softmax_tile_lane_query<T, DB, CAUSAL, DROPOUT>(a, s, o, pf, m_run, l_run, lr_run, c, k0, q0, qi, len, g, bh);
      // ---- O^T += V^T P^T
      {
        auto v_frag = [&](int f) {   // f = DB cc + db: consecutive MFMAs hit different accumulators
          const T* base = Vt + 16 * (f / DB) * D;
          return tr_frag<T8>(base + tro.off[f % DB][0], base + tro.off[f % DB][1]);
        };
        T8 ring[PF];
#pragma unroll
        for (int f = 0; f < PF; ++f) ring[f] = v_frag(f);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 4 * DB; ++f) {
          const T8 cur = ring[f % PF];
          o[f % DB] = mfma32(cur, pf[f / DB], o[f % DB]);
          if (f + PF < 4 * DB) ring[f % PF] = v_frag(f + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    wait_async_copies();
    __syncthreads();   // the next tile has landed, and everyone is done with this buffer
    jt = jn;
    buf ^= 1;
  }

  // ---- epilogue: normalise, apply the dropout scale, write O and L once
  const float l_sum = l_run + xchg32(l_run);
  const float lr_sum = lr_run + xchg32(lr_run);
  const float l_tot = qi < len ? l_sum : 0.f;   // padding rows: O = 0, LSE = -inf
  const float inv = (l_tot > 0.f && lr_sum > 0.f) ? (DROPOUT ? a.keep_scale : 1.f) / lr_sum : 0.f;
  if (g == 0 && row_ok) {
    const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
    a.LSE[(int64_t)bh * a.N + qi] = lse;
  }
  if (a.o_fp32) {
    float* Og = (float*)a.O + head_off + (int64_t)qi * a.sn;
    if (row_ok) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[db][4 * i4 + e] * inv;
          if (D != 32 || 8 * i4 + 4 * g < a.dvalid) *(f32x4*)(Og + 32 * db + 8 * i4 + 4 * g) = v;
        }
    }
  } else {
    // coalesced row stores through the (now idle) tile buffers: two wavefronts per buffer
    T* stage = (wave < 2 ? &Ks[0][0] + wave * 32 * D : &Vs[0][0] + (wave - 2) * 32 * D);
    store_rows_coalesced<T, D>(stage, (T*)a.O + head_off + (int64_t)q0 * a.sn, a.sn, o, inv, a.N - q0,
                               D == 32 ? a.dvalid : D);
  }
  }  // for pass
}

template <typename T, int D>
int launch_fwd_td(const KArgs& a_in, bool causal, bool dropout, bool sparse, hipStream_t s) {
  KArgs a = a_in;
  if (causal && !sparse && D == 64) {   // items are pairs of row blocks
    a.n_items = a.B * a.H * ((a.T + 1) / 2);
    a.chunk = (a.n_items + kXcds - 1) / kXcds;
  }
  const dim3 grid(kXcds * a.chunk), block(NT);
#define ATTN_FWD_CASE(C, P, S)                                                         \
  if (causal == C && dropout == P && sparse == S) {                                    \
    hipLaunchKernelGGL((fwd_kernel<T, D, C, P, S>), grid, block, 0, s, a);             \
    return (int)hipGetLastError();                                                     \
  }
  ATTN_FWD_CASE(false, false, false)
  ATTN_FWD_CASE(true, false, false)
  ATTN_FWD_CASE(false, true, false)
  ATTN_FWD_CASE(true, true, false)
  ATTN_FWD_CASE(false, false, true)
  ATTN_FWD_CASE(true, false, true)
  ATTN_FWD_CASE(false, true, true)
  ATTN_FWD_CASE(true, true, true)
#undef ATTN_FWD_CASE
  return (int)hipErrorInvalidValue;
}

// keep[bh][i][j] for the test hook: one thread per group of sixteen consecutive keys
__global__ void dropout_mask_kernel(const KArgs a, uint8_t* keep) {
  const int64_t ngrp = ((int64_t)a.N + 15) / 16;
  const int64_t total = (int64_t)a.B * a.H * a.N * ngrp;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const uint32_t g16 = (uint32_t)(idx % ngrp);
    const uint32_t i = (uint32_t)((idx / ngrp) % a.N);
    const uint32_t bh = (uint32_t)(idx / (ngrp * a.N));
    const u32x4 w = philox_draw16(g16, i, bh, a.offset_lo, a.seed_lo, a.seed_hi);
    // (when dropout rounds down to nothing the kernels do not draw at all: everything is kept)
    const uint32_t m = a.drop_thr == 0 ? 0xFFFFu : keep_bits16(w, dropout_carry2(a.drop_thr));
    uint8_t* dst = keep + ((int64_t)bh * a.N + i) * a.N + 16 * (int64_t)g16;
    const int n = min(16, a.N - 16 * (int)g16);
    if (n == 16 && a.N % 4 == 0) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {   // four flag bytes at a time
        const uint32_t nib = (m >> (4 * q)) & 0xFu;
        *(uint32_t*)(dst + 4 * q) = (nib & 1u) | ((nib & 2u) << 7) | ((nib & 4u) << 14) | ((nib & 8u) << 21);
      }
    } else {   // rows of N bytes are not 4-byte aligned, or the last group of a row is partial
      for (int f = 0; f < n; ++f) dst[f] = (uint8_t)((m >> f) & 1u);
    }
  }
}

}  // namespace

int choose_fwd(const KArgs& a, int d, bool causal, bool dropout, bool sparse) {
  const int variant = fwd_variant();
  const int n_qt256 = (a.N + 255) / 256;
  const int64_t pp_items = (int64_t)a.B * a.H * (causal ? (n_qt256 + 1) / 2 : n_qt256);
  bool use_pp = d == 128 && pp_items >= kComputeUnits &&
                (dropout ? causal : (a.N >= 1024 || (causal && a.N >= 512)));
  if (variant == 1) use_pp = false;
  if (variant == 2 && d != 32) use_pp = true;
  return !sparse && use_pp ? kFwdTwoGroup : kFwdFreeRunning;   // (the reasons: see launch_fwd)
}

int launch_fwd(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, hipStream_t s) {
  // Which dense d = 128 problems take the two-group ping-pong kernel (attn_fwd_pp.hip), by
  // measurement against this file's kernel (two free-running 4-wave workgroups per compute unit):
  //   no dropout: from N = 1024 on (4-6 % faster from 2048, equal at 1024, 6 % slower at 512), under
  //     the causal mask from N = 512 (its paired work items balance better);
  //   dropout: only under the causal mask (the pairing again: 10-15 % faster); without a mask the
  //     free-running kernel is ~3 % faster at every N (the generator is plain vector ALU work);
  //   and only if its 256-row work items (pairs of them under the causal mask) are at least as
  //     many as the compute units: a problem with few heads would leave half of the chip idle.
  // At d <= 64 the vector ALU work dominates and this file's kernel measured faster at every N;
  // block-sparse problems always take it.  attn_debug_set_variant overrides the choice
  // (comparisons and tests).
  if (choose_fwd(a, d, causal, dropout, sparse) == kFwdTwoGroup) return launch_fwd_pp(a, dtype, d, causal, dropout, s);
  if (dtype == 0 && d == 32) return launch_fwd_td<_Float16, 32>(a, causal, dropout, sparse, s);
  if (dtype == 1 && d == 32) return launch_fwd_td<__bf16, 32>(a, causal, dropout, sparse, s);
  if (dtype == 0 && d == 64) return launch_fwd_td<_Float16, 64>(a, causal, dropout, sparse, s);
  if (dtype == 0 && d == 128) return launch_fwd_td<_Float16, 128>(a, causal, dropout, sparse, s);
  if (dtype == 1 && d == 64) return launch_fwd_td<__bf16, 64>(a, causal, dropout, sparse, s);
  if (dtype == 1 && d == 128) return launch_fwd_td<__bf16, 128>(a, causal, dropout, sparse, s);
  return (int)hipErrorInvalidValue;
}

int launch_dropout_mask(const KArgs& a, uint8_t* keep, hipStream_t s) {
  const int64_t total = (int64_t)a.B * a.H * a.N * ((a.N + 15) / 16);
  const int blocks = (int)((total + 255) / 256 < 65536 ? (total + 255) / 256 : 65536);
  hipLaunchKernelGGL(dropout_mask_kernel, dim3(blocks), dim3(256), 0, s, a, keep);
  return (int)hipGetLastError();
}

}  // namespace attn
