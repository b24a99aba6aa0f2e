// Backward pass of IO-aware exact attention for gfx950 (MI355X).
//
// The arithmetic is Algorithm 4 of the paper (Appendix B.4): S and P are recomputed tile by
// tile from Q, K, V and the saved row statistic, the dropout mask is regenerated from the
// counter-based generator, D_i = rowsum(dO_i o O_i) replaces the row reduction over P o dP
// (Eq. (4), Appendix B.2), and
//     dV = P_dropped^T dO,  dP = (dO V^T) o Z,  dS = P o (dP - D),  dQ = tau dS K,  dK = tau dS^T Q.
// The schedule differs from the paper's single K/V-outer loop with dQ read-modify-written in
// HBM: two launches, neither of which writes a partial result to HBM.
//   1. dq_kernel     : a workgroup owns 128 query rows and sweeps K/V tiles; dQ stays in
//                      registers (S^T, dP^T layout: lane = query, like the forward kernel).  It
//                      also computes D = rowsum(dO o O) of its rows and leaves -D and L in base 2
//                      in the scratch vectors for the second launch.
//   2. dK/dV kernel (attn_bwd_dkv.hip, attn_bwd_dkv_fr.hip): a workgroup owns 128 keys and
//                      sweeps Q/dO tiles; dK, dV stay in registers (S, dP layout: lane = key)
// S and dP are therefore recomputed in both launches (seven tile products per (i, j) instead of
// five) in exchange for no atomics, no fp32 dQ round trip and bit-reproducible gradients.
#include "attn_common.h"
#include "attn_tiles.h"

#include <cstdlib>

namespace attn {
namespace {

constexpr int NT = 256;
constexpr int TILE = 64;  // keys of the streamed tile

// ---------------------------------------------------------------------------------------------
// dQ: workgroup = 128 query rows (4 wavefronts x 32), sweep over 64-key tiles.
template <typename T, int D, bool CAUSAL, bool DROPOUT, bool SPARSE>
__global__ __launch_bounds__(NT, 2) void dq_kernel(const KArgs a) {
  typedef typename Vec<T>::x8 T8;
  constexpr int KK = D / 16, DB = D / 32;
  // K and V tiles, double buffered, filled by async copies.  Without the causal mask they form one
  // LDS block (K tile of buffer b at b TILE D, V tile at (2 + b) TILE D), so that an LDS address
  // is a per-lane register plus an immediate offset once the buffer index is a compile-time
  // constant (see tile_step below); the causal kernels, which cannot afford that unrolling, keep
  // two arrays (the form that the register allocator handles without spilling).
  T* Ks0;
  T* Vs0;
  if constexpr (!CAUSAL) {
    __shared__ __attribute__((aligned(16))) T smem[4 * TILE * D];
    Ks0 = smem;
    Vs0 = smem + 2 * TILE * D;
  } else {
    __shared__ __attribute__((aligned(16))) T Ks[2 * TILE * D];
    __shared__ __attribute__((aligned(16))) T Vs[2 * TILE * D];
    Ks0 = Ks;
    Vs0 = Vs;
  }

  const int item = xcd_item(a.n_items, a.chunk);
  if (item < 0) return;
  const int n_qt = a.T;   // ceil(N / 128): the last block may be ragged
  // Work item = (head, row block).  Under the causal mask row block q sweeps 2 (q + 1) key tiles;
  // for dense d = 64 problems an item is the pair (n_qt - 1 - q, q), one per pass, so that every
  // workgroup does the same amount of work (at d = 128 the loop costs registers the kernel does
  // not have).
  constexpr bool PAIRED = CAUSAL && !SPARSE && D == 64;
  const int n_per_head = PAIRED ? (n_qt + 1) / 2 : n_qt;
  int bh = item / n_per_head;
  int q_item = item % n_per_head;
  if constexpr (CAUSAL && !PAIRED) {
    // unpaired causal items: the row blocks of a.group consecutive heads are dealt out together,
    // heaviest first, so that the items a compute unit receives last are light ones.  The host
    // sizes the group so that the K and V of its heads (the L2 working set of an XCD) stay within
    // 8 MiB: larger groups balance better but thrash L2 on long sequences.
    const int n_heads = a.B * a.H;
    const int grp0 = (bh / a.group) * a.group;             // first head of this group
    const int gsz = min(a.group, n_heads - grp0);          // heads in it (the last group may be short)
    const int within = (bh - grp0) * n_qt + q_item;        // position inside the group's items
    bh = grp0 + within % gsz;
    q_item = within / gsz;                                 // q_item-th heaviest block (see qt below)
  }
  const int n_pass = PAIRED && q_item != n_qt - 1 - q_item ? 2 : 1;
#pragma clang loop unroll(disable)
  for (int pass = 0; pass < n_pass; ++pass) {
  if (pass) __syncthreads();   // the tile buffers staged the first block's output rows
  const int qt = PAIRED ? (pass ? q_item : n_qt - 1 - q_item) : (CAUSAL ? n_qt - 1 - q_item : q_item);
  const int b = bh / a.H, h = bh % a.H;
  const int64_t head_off = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const T* __restrict__ Kg = (const T*)a.K + head_off;
  const T* __restrict__ Vg = (const T*)a.V + head_off;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int q0 = qt * 128 + wave * 32;
  // lanes beyond a ragged end work on a copy of the last row with P = 0 and store nothing
  const bool row_ok = q0 + r < a.N;
  const int qi = min(q0 + r, a.N - 1);

  T8 qf[KK], gf[KK];  // Q^T and dO^T fragments (B operands) of this lane's query
  // -D_i = -sum_d dO[i][d] O[i][d] (Eq. (4), Appendix B.2), from the same 8-element pieces of the row
  // that the dO fragments hold: this lane's half of the sum, completed with the partner lane below
  float d_part = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    const int64_t off = head_off + (int64_t)qi * a.sn + 16 * kk + 8 * g;
    if (D == 32 && 16 * kk + 8 * g >= a.dvalid) {   // head dimension 16: the upper columns are zeros
#pragma unroll
      for (int e = 0; e < 8; ++e) { qf[kk][e] = (T)0.f; gf[kk][e] = (T)0.f; }
      continue;
    }
    qf[kk] = *(const T8*)((const T*)a.Q + off);
    gf[kk] = *(const T8*)((const T*)a.dO + off);
    if (a.o_fp32) {
      const f32x4 o0 = *(const f32x4*)((const float*)a.O + off);
      const f32x4 o1 = *(const f32x4*)((const float*)a.O + off + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) d_part += (float)gf[kk][e] * o0[e] + (float)gf[kk][4 + e] * o1[e];
    } else {
      const T8 o = *(const T8*)((const T*)a.O + off);
#pragma unroll
      for (int e = 0; e < 8; ++e) d_part += (float)gf[kk][e] * (float)o[e];
    }
  }
  const float lse = a.LSE[(int64_t)bh * a.N + qi];
  // base-2 statistic; a row that saw no key (or lies beyond a ragged end) has P = 0 everywhere
  const float l2 = (lse == -INFINITY || !row_ok) ? INFINITY : lse * 1.4426950408889634f;
  const float neg_d = row_ok ? -(d_part + xchg32(d_part)) : 0.f;   // -D_i
  // The dK/dV kernel reads both per 64-row tile from the scratch vectors (padded to whole blocks
  // of 128 rows per head: this workgroup writes all 128 of its block).  The tile kernels start
  // their dP accumulators from -D, so that dP - D needs no instruction of its own.
  if (g == 0) {
    a.Dvec[(int64_t)bh * a.Nr + q0 + r] = neg_d;
    a.L2vec[(int64_t)bh * a.Nr + q0 + r] = l2;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0 && pass == 0 && a.seglist != nullptr) {
    a.seglist[0] = 0;   // block-sparse: empty segment list, no blocks counted (the dK/dV planning
    a.seglist[1] = 0;   // kernels run after this one)
  }

  f32x16 dq[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dq[db][i] = 0.f;

  // key-padding mask: keys >= len contribute nothing (rows >= len have LSE = -inf, hence P = 0)
  const int len = a.klen ? min(max(a.klen[b], 0), a.N) : a.N;
  TileIter<SPARSE> it;
  {
    int lim;
    if constexpr (SPARSE) lim = min(CAUSAL ? qt + 1 : a.T, (len + 127) / 128);
    else lim = CAUSAL ? min(2 * qt + 2, (len + TILE - 1) / TILE) : (len + TILE - 1) / TILE;   // len <= N
    if (qt * 128 >= len) lim = 0;
    it.init(SPARSE ? a.mask + (int64_t)h * a.mask_sh + (int64_t)qt * a.T : nullptr, 1, 0, lim);
  }
  TrOffsets<D> tro;
  tro.init();
  TileAsync<T, D, NT / 64> dma;
  dma.init(a.sn, threadIdx.x >> 6, D == 32 ? a.dvalid : D);
  if (D == 32 && a.dvalid < D) {   // the copies leave columns >= 16 of the tile buffers untouched
    zero_tiles(Ks0, 2 * TILE * D);
    zero_tiles(Vs0, 2 * TILE * D);
    __syncthreads();
  }

  const float c = a.scale_log2;
  int jt = it.next();
  if (jt >= 0) {
    dma.copy_rows(Kg, a.sn, jt * TILE, a.N, Ks0);
    dma.copy_rows(Vg, a.sn, jt * TILE, a.N, Vs0);
  }
  wait_async_copies();
  __syncthreads();   // tile 0 has landed, and so have the Q / dO fragments
  // Without the causal mask the tile loop is unrolled by two, so that the buffer index is a
  // constant in each copy of its body; the causal kernels have no registers for two copies.
  constexpr int UNROLL = CAUSAL ? 1 : 2;
  int buf_rt = 0;
  while (jt >= 0) {
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const int buf = UNROLL == 2 ? u : buf_rt;
    const int jn = it.next();
    if (jn >= 0) {   // next tile streams into the other buffer while this one is used
      dma.copy_rows(Kg, a.sn, jn * TILE, a.N, Ks0 + (buf ^ 1) * TILE * D);
      dma.copy_rows(Vg, a.sn, jn * TILE, a.N, Vs0 + (buf ^ 1) * TILE * D);
    }
    const T* Kt = Ks0 + buf * TILE * D;
    const T* Vt = Vs0 + buf * TILE * D;

    const int k0 = jt * TILE;
    if (!CAUSAL || k0 <= q0 + 31) {
      f32x16 s[2], dp[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          s[kb][i] = 0.f;
          // every accumulator element of a lane belongs to the lane's query: without dropout the
          // product starts from -D_i and ends as dP - D
          dp[kb][i] = DROPOUT ? 0.f : neg_d;
        }
      // S^T = K Q^T and dP^T = V dO^T as one stream of 4 KK MFMAs; operand reads run PF fragments
      // ahead of their MFMA (the scheduling barriers keep that distance)
      constexpr int PF = 4;
      auto kv_frag = [&](int f) {   // f = 4 kk + 2 kb + (0: K, 1: V)
        const int off = lds_off<D>(32 * ((f >> 1) & 1) + r, 2 * (f >> 2) + g);
        return *(const T8*)(((f & 1) ? Vt : Kt) + off);
      };
      {
        T8 ring[PF];
#pragma unroll
        for (int f = 0; f < PF; ++f) ring[f] = kv_frag(f);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 4 * KK; ++f) {
          const T8 cur = ring[f % PF];
          const int kk = f >> 2, kb = (f >> 1) & 1;
          if (f & 1) dp[kb] = mfma32(cur, gf[kk], dp[kb]);
          else s[kb] = mfma32(cur, qf[kk], s[kb]);
          if (f + PF < 4 * KK) ring[f % PF] = kv_frag(f + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (k0 + TILE > len) {   // the tile holds padded keys: their logits become -inf, hence P = 0
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (k0 + 32 * kb + 8 * (i >> 2) + 4 * g + (i & 3) >= len) s[kb][i] = -INFINITY;
      }
      // P = exp(S - L); dS = P o (dP o Z - D)
      KeepLQ kq = {};
      if constexpr (DROPOUT) kq = keep_tile_lane_query(k0, qi, bh, g, a.offset_lo, a.seed_lo, a.seed_hi);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * i4 + e;
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i], c, -l2));
            if (CAUSAL && k0 + 32 * kb + 8 * i4 + 4 * g + e > qi) p = 0.f;
            float dpv = dp[kb][i];
            if constexpr (DROPOUT)   // Z dP - D with Z = keep_scale or 0 by the 8-bit draw of this element
              dpv = dropped(kq.w[kb][i4], e, a.drop_thr) ? neg_d : __builtin_fmaf(dpv, a.keep_scale, neg_d);
            s[kb][i] = p * dpv;
          }
        }
      T8 dsf[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc)
#pragma unroll
        for (int t = 0; t < 8; ++t) dsf[cc][t] = (T)s[cc >> 1][8 * (cc & 1) + t];
      // dQ^T += K^T dS^T
      auto kt_frag = [&](int f) {   // f = DB cc + db: consecutive MFMAs hit different accumulators
        const T* base = Kt + 16 * (f / DB) * D;
        return tr_frag<T8>(base + tro.off[f % DB][0], base + tro.off[f % DB][1]);
      };
      {
        T8 ring[PF];
#pragma unroll
        for (int f = 0; f < PF; ++f) ring[f] = kt_frag(f);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 4 * DB; ++f) {
          const T8 cur = ring[f % PF];
          dq[f % DB] = mfma32(cur, dsf[f / DB], dq[f % DB]);
          if (f + PF < 4 * DB) ring[f % PF] = kt_frag(f + PF);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    wait_async_copies();
    __syncthreads();   // next tile has landed, and everyone is done with this buffer
    jt = jn;
    buf_rt ^= 1;
    if (jt < 0) break;
  }
  }
  // the loop ends on a barrier (or never touched LDS): the tile buffers stage the output rows
  T* stage = (wave < 2 ? Ks0 + wave * 32 * D : Vs0 + (wave - 2) * 32 * D);
  store_rows_coalesced<T, D>(stage, (T*)a.dQ + head_off + (int64_t)q0 * a.sn, a.sn, dq, a.tau, a.N - q0,
                             D == 32 ? a.dvalid : D);
  }  // for pass
}

template <typename T> constexpr int kDtype = 0;
template <> constexpr int kDtype<__bf16> = 1;

template <typename T, int D>
int launch_bwd_td(const KArgs& a, bool causal, bool dropout, bool sparse, hipStream_t s, hipEvent_t* ev) {
  if (ev) (void)hipEventRecord(ev[0], s);
  int e = 0;
  if (ev) (void)hipEventRecord(ev[1], s);   // (there is no separate preparation launch any more)
  const dim3 block(NT);
  // dense causal d = 64 dQ items are pairs of row blocks
  KArgs aq = a;
  if (causal && !sparse && D == 64) {
    aq.n_items = a.B * a.H * ((a.T + 1) / 2);
    aq.chunk = (aq.n_items + kXcds - 1) / kXcds;
  }
  {
    const int64_t kv_bytes = 2 * (int64_t)a.N * D * (int64_t)sizeof(T);
    const int64_t fit = ((int64_t)8 << 20) / kv_bytes;
    aq.group = (int)(fit < 1 ? 1 : (fit > 8 ? 8 : fit));
  }
  const dim3 grid_q(kXcds * aq.chunk);
#define ATTN_BWD_CASE(C, P, S)                                                   \
  if (causal == C && dropout == P && sparse == S) {                              \
    hipLaunchKernelGGL((dq_kernel<T, D, C, P, S>), grid_q, block, 0, s, aq);     \
    e = (int)hipGetLastError();                                                  \
    if (e != 0) return e;                                                        \
    if (ev) (void)hipEventRecord(ev[2], s);                                      \
    e = launch_dkv_rs(a, kDtype<T>, D, C, P, S, s);                              \
    if (ev) (void)hipEventRecord(ev[3], s);                                      \
    return e;                                                                    \
  }
  ATTN_BWD_CASE(false, false, false)
  ATTN_BWD_CASE(true, false, false)
  ATTN_BWD_CASE(false, true, false)
  ATTN_BWD_CASE(true, true, false)
  ATTN_BWD_CASE(false, false, true)
  ATTN_BWD_CASE(true, false, true)
  ATTN_BWD_CASE(false, true, true)
  ATTN_BWD_CASE(true, true, true)
#undef ATTN_BWD_CASE
  return (int)hipErrorInvalidValue;
}

}  // namespace

int launch_bwd(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, hipStream_t s,
               hipEvent_t* ev) {
  if (dtype == 0 && d == 32) return launch_bwd_td<_Float16, 32>(a, causal, dropout, sparse, s, ev);
  if (dtype == 1 && d == 32) return launch_bwd_td<__bf16, 32>(a, causal, dropout, sparse, s, ev);
  if (dtype == 0 && d == 64) return launch_bwd_td<_Float16, 64>(a, causal, dropout, sparse, s, ev);
  if (dtype == 0 && d == 128) return launch_bwd_td<_Float16, 128>(a, causal, dropout, sparse, s, ev);
  if (dtype == 1 && d == 64) return launch_bwd_td<__bf16, 64>(a, causal, dropout, sparse, s, ev);
  if (dtype == 1 && d == 128) return launch_bwd_td<__bf16, 128>(a, causal, dropout, sparse, s, ev);
  return (int)hipErrorInvalidValue;
}

}  // namespace attn
