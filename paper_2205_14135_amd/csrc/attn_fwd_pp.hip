// Forward pass, dense (no block mask) variant with two wavefront groups in ping-pong.
//
// Same arithmetic and register layout as fwd_kernel in attn_fwd.hip (Algorithm 2 of the paper,
// Q-outer, S^T = K Q^T orientation).  What changes is the schedule.  Per 64-key tile a wavefront
// alternates between a matrix block M(j) = { O^T += V(j-1)^T P(j-1)^T ; S(j)^T = K(j) Q^T } and a
// vector block X(j) = { online softmax of tile j }, of roughly equal length.  Two wavefronts that
// share a SIMD and run the same code drift into the same block and then fight for the same
// unit, so here a workgroup has 8 wavefronts = 2 groups x 4 SIMDs, each group owning 128 of the
// workgroup's 256 query rows, and workgroup barriers keep group B exactly one block behind
// group A: while one group issues MFMA the other issues the softmax VALU work.
//
// K and V tiles sit in rings of three LDS buffers (unpadded, XOR-swizzled) shared by both groups.
// In global slot numbers (slot 2j: A in M(j), B in X(j-1); slot 2j+1: A in X(j), B in M(j)) K(t)
// is read in slots 2t, 2t+1 and V(t) in slots 2t+2, 2t+3.  Tiles arrive by asynchronous
// global-to-LDS copies that the compiler does not track; group A copies the K tiles and group B
// the V tiles.  Issuing a tile's copy instructions blocks a wavefront for hundreds of clocks (the
// vector memory path takes 64 bytes per clock), so a wavefront issues tile j + 1 at the END of its
// matrix block M(j), the shorter of the two blocks, where it would otherwise wait at the barrier
// for the other group's vector block, and waits for the copy only at the end of its own X(j): the
// copy has a whole block to land and its latency never shows.  (Measured against issuing at the
// start or at the end of the vector block, or half and half: this placement is the fastest.)  The
// third V buffer is what allows it: when a group B wavefront leaves M(j), its neighbours may still
// be reading V(j-1).
#include "attn_common.h"
#include "attn_tiles.h"

namespace attn {
namespace {

constexpr int BRW = 256;  // query rows per workgroup
constexpr int BC = 64;    // keys per tile
constexpr int NT = 512;

// One block of 256 query rows (row block qt of head bh) against all the keys it sees.
template <typename T, int D, bool CAUSAL, bool DROPOUT>
__device__ __forceinline__ void fwd_pp_rows(const KArgs& a, const int bh, const int qt, T (&Ks)[3][BC * D],
                                            T (&Vs)[3][BC * D]) {
  typedef typename Vec<T>::x8 T8;
  typedef typename Vec<T>::x4 T4;
  constexpr int KK = D / 16, DB = D / 32;
  const int b = bh / a.H, h = bh % a.H;
  const int64_t head_off = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const T* __restrict__ Qg = (const T*)a.Q + head_off;
  const T* __restrict__ Kg = (const T*)a.K + head_off;
  const T* __restrict__ Vg = (const T*)a.V + head_off;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const bool group_b = wave >= 4;
  const int r = lane & 31, g = lane >> 5;
  const int q0 = qt * BRW + wave * 32;
  const bool valid = q0 < a.N;          // wavefronts past the end of the tensor only keep the barriers company
  // lanes beyond a ragged end work on a copy of the last row and store nothing
  const bool row_ok = q0 + r < a.N;
  const int qi = min(q0 + r, a.N - 1);

  T8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    qf[kk] = *(const T8*)(Qg + (int64_t)qi * a.sn + 16 * kk + 8 * g);

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  // m_run: reference of the row's probabilities (base 2; lags the running maximum by at most
  // kLazyRescale); l_run: this lane's share of the exact row sum (for the saved statistic);
  // lr_run: its share of the sum of the rounded probabilities (normalises O)
  float m_run = -INFINITY, l_run = 0.f, lr_run = 0.f;

  // key-padding mask: keys >= len are masked, rows >= len produce O = 0, LSE = -inf
  const int len = a.klen ? min(max(a.klen[b], 0), a.N) : a.N;
  const int n_tiles = (len + BC - 1) / BC;   // len <= N
  const int J = qt * BRW >= len ? 0 : (CAUSAL ? min(n_tiles, 4 * (qt + 1)) : n_tiles);
  if (J == 0) {   // nothing visible for any row of this workgroup: write zeros and leave
    if (row_ok) {
      if (g == 0) a.LSE[(int64_t)bh * a.N + qi] = -INFINITY;
      const int64_t o_off = head_off + (int64_t)qi * a.sn + (D / 2) * g;
      if (a.o_fp32) {
        for (int e = 0; e < D / 2; ++e) ((float*)a.O)[o_off + e] = 0.f;
      } else {
        for (int e = 0; e < D / 2; ++e) ((T*)a.O)[o_off + e] = (T)0.f;
      }
    }
    return;
  }

  typedef TileAsync<T, D, 4> Dma;   // the four wavefronts of a group copy a whole tile
  Dma dma;
  dma.init(a.sn, wave & 3);
  const T* __restrict__ Tg = group_b ? Vg : Kg;   // the tensor this group copies
  TrOffsets<D> tro;
  tro.init();
  const float c = a.scale_log2;

  f32x16 s[2];
  T8 pf[4];

  auto active = [&](int j) { return valid && (!CAUSAL || j * BC <= q0 + 31); };

  // LDS operand reads are issued PF fragments ahead of the MFMA that consumes them, so that the
  // matrix pipe does not idle on LDS latency.
  constexpr int PF = 4;
  auto k_frag = [&](const T* kbuf, int f) {  // f = 2 * kk + kb
    return *(const T8*)(kbuf + lds_off<D>(32 * (f & 1) + r, 2 * (f >> 1) + g));
  };
  auto v_frag = [&](const T* vbuf, int f) {  // f = DB * cc + db: consecutive MFMAs hit different accumulators
    const T* base = vbuf + 16 * (f / DB) * D;
    return tr_frag<T8>(base + tro.off[f % DB][0], base + tro.off[f % DB][1]);
  };

  // M block: O^T += V(jv)^T P^T (if do_pv) followed by S^T = K(js) Q^T (if do_s), as one
  // software-pipelined stream of 4*DB + 2*KK MFMAs.
  auto do_M = [&](bool do_pv, const T* vbuf, bool do_s, const T* kbuf) {
    constexpr int NV = 4 * DB, NK = 2 * KK;
    T8 ring[PF];
    if (do_pv) {
#pragma unroll
      for (int f = 0; f < PF; ++f) ring[f] = v_frag(vbuf, f);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int f = 0; f < NV; ++f) {
        const T8 cur = ring[f % PF];
        o[f % DB] = mfma32(cur, pf[f / DB], o[f % DB]);
        if (f + PF < NV) ring[f % PF] = v_frag(vbuf, f + PF);
        else if (do_s) ring[f % PF] = k_frag(kbuf, f + PF - NV);
        __builtin_amdgcn_sched_barrier(0);   // keep the prefetch distance the source states
      }
    } else if (do_s) {
#pragma unroll
      for (int f = 0; f < PF; ++f) ring[f] = k_frag(kbuf, f);
    }
    if (do_s) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
      for (int f = 0; f < NK; ++f) {
        // ring slot of K fragment f: it was loaded as "fragment NV + f" of the combined stream
        const int slot = do_pv ? (NV + f) % PF : f % PF;
        const T8 cur = ring[slot];
        s[f & 1] = mfma32(cur, qf[f >> 1], s[f & 1]);
        if (f + PF < NK) ring[slot] = k_frag(kbuf, f + PF);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  auto do_softmax = [&](int j) {
    softmax_tile_lane_query<T, DB, CAUSAL, DROPOUT>(a, s, o, pf, m_run, l_run, lr_run, c, j * BC, q0, qi, len, g, bh);
  };

  // ring slot of a tile in this group's ring
  auto ring = [&](int slot) -> T* { return group_b ? Vs[slot] : Ks[slot]; };
  // ---- prologue: tile 0 of this group's tensor.  Group B starts one block later (an extra
  // barrier).  The wait also covers the Q fragment loads issued before.
  dma.copy_rows(Tg, a.sn, 0, a.N, ring(0));
  wait_async_copies();
  __syncthreads();
  if (group_b) {
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();   // B runs one block behind A
  }

  int cur = 0;   // ring slot of tile j: j % 3
  for (int j = 0; j < J; ++j) {
    const int nxt = cur == 2 ? 0 : cur + 1, prv = cur == 0 ? 2 : cur - 1;   // slots of tiles j + 1, j - 1
    // ---- M(j): matrix work, then the copy of this group's tile j + 1 (its slot held tile j - 2)
    do_M(j > 0 && active(j - 1), Vs[prv], active(j), Ks[cur]);
    __builtin_amdgcn_sched_barrier(0);
    if (j + 1 < J) dma.copy_rows(Tg, a.sn, (j + 1) * BC, a.N, ring(nxt));
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    // ---- X(j): the online softmax; then tile j + 1 must have landed
    if (active(j)) do_softmax(j);
    __builtin_amdgcn_sched_barrier(0);
    wait_async_copies();
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
    cur = nxt;
  }
  do_M(active(J - 1), Vs[cur == 0 ? 2 : cur - 1], false, Ks[0]);
  if (!group_b) { __builtin_amdgcn_sched_barrier(0); __syncthreads(); }  // equal barrier counts
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();   // every wavefront is done with the tiles: the buffers become output staging

  if (!valid) return;
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
          *(f32x4*)(Og + 32 * db + 8 * i4 + 4 * g) = v;
        }
    }
  } else {
    T* stage = wave < 4 ? &Ks[0][0] + wave * 32 * D : &Vs[0][0] + (wave - 4) * 32 * D;
    store_rows_coalesced<T, D>(stage, (T*)a.O + head_off + (int64_t)q0 * a.sn, a.sn, o, inv, a.N - q0);
  }
}

// Work item = (head, row block).  Under the causal mask row block q sees 4 (q + 1) key tiles, so
// an item takes the pair (q, n_qt - 1 - q): every workgroup then does the same amount of work
// and the static assignment of items to compute units stays balanced.
template <typename T, int D, bool CAUSAL, bool DROPOUT>
__global__ __launch_bounds__(NT) void fwd_pp_kernel(const KArgs a) {
  __shared__ __attribute__((aligned(16))) T Ks[3][BC * D];
  __shared__ __attribute__((aligned(16))) T Vs[3][BC * D];
  const int item = xcd_item(a.n_items, a.chunk);
  if (item < 0) return;
  const int n_qt = (a.N + BRW - 1) / BRW;
  if constexpr (CAUSAL) {
    const int n_pair = (n_qt + 1) / 2;
    const int bh = item / n_pair, q = item % n_pair;
    fwd_pp_rows<T, D, CAUSAL, DROPOUT>(a, bh, n_qt - 1 - q, Ks, Vs);
    if (q != n_qt - 1 - q) {
      __syncthreads();   // the tile buffers staged the first block's output rows
      fwd_pp_rows<T, D, CAUSAL, DROPOUT>(a, bh, q, Ks, Vs);
    }
  } else {
    fwd_pp_rows<T, D, CAUSAL, DROPOUT>(a, item / n_qt, item % n_qt, Ks, Vs);
  }
}

template <typename T, int D>
int launch_td(KArgs a, bool causal, bool dropout, hipStream_t s) {
  const int n_qt = (a.N + BRW - 1) / BRW;
  a.n_items = a.B * a.H * (causal ? (n_qt + 1) / 2 : n_qt);
  a.chunk = (a.n_items + kXcds - 1) / kXcds;
  const dim3 grid(kXcds * a.chunk), block(NT);
  if (!causal && !dropout) hipLaunchKernelGGL((fwd_pp_kernel<T, D, false, false>), grid, block, 0, s, a);
  else if (causal && !dropout) hipLaunchKernelGGL((fwd_pp_kernel<T, D, true, false>), grid, block, 0, s, a);
  else if (!causal && dropout) hipLaunchKernelGGL((fwd_pp_kernel<T, D, false, true>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((fwd_pp_kernel<T, D, true, true>), grid, block, 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace

int launch_fwd_pp(const KArgs& a, int dtype, int d, bool causal, bool dropout, hipStream_t s) {
  if (dtype == 0 && d == 64) return launch_td<_Float16, 64>(a, causal, dropout, s);
  if (dtype == 0 && d == 128) return launch_td<_Float16, 128>(a, causal, dropout, s);
  if (dtype == 1 && d == 64) return launch_td<__bf16, 64>(a, causal, dropout, s);
  if (dtype == 1 && d == 128) return launch_td<__bf16, 128>(a, causal, dropout, s);
  return (int)hipErrorInvalidValue;
}

}  // namespace attn
