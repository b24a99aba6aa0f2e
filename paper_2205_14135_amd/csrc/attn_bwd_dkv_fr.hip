// dK / dV kernel for head dimensions up to 64 (dense and block-sparse): one wavefront does all
// four tile products of its 32 keys.
//
// Arithmetic: Algorithm 4 of the paper for one block of 128 keys, swept over 64-query tiles:
//     S = Q K^T, P = exp(S - L), dV += (P o Z)^T dO, dP = (dO V^T) o Z, dS = P o (dP - D), dK += tau dS^T Q.
// At d <= 64 both accumulators (dK^T, dV^T), both operand fragment sets (K, V) and the S / dP tiles
// of a wavefront fit in 256 registers, so the work of a key block need not be split over two
// wavefronts of a SIMD as in attn_bwd_dkv.hip: no probabilities travel through LDS, there is one
// workgroup barrier per tile (for the tile buffers only), and a workgroup is 4 wavefronts, so two
// or more independent workgroups share a compute unit and fill each other's stalls.  The vector
// ALU work per tile is the same at every head dimension while the matrix work shrinks with it;
// at d <= 64 that free-running arrangement is faster than the role split (which wins at d = 128,
// where it is also the only one that fits the register file).
// Register layout "lane = key" (S = Q K^T: accumulator rows = queries of the tile, column = the
// lane's key), as in attn_bwd_dkv.hip.
#include "attn_common.h"
#include "attn_tiles.h"

namespace attn {
namespace {

constexpr int NT = 256;
constexpr int TILE = 64;

template <typename T, int D, bool CAUSAL, bool DROPOUT, bool SPARSE>
__global__ __launch_bounds__(NT, 2) void dkv_fr_kernel(const KArgs a) {
  typedef typename Vec<T>::x8 T8;
  constexpr int KK = D / 16, DB = D / 32;
  static_assert(D <= 64, "the accumulators of both gradients must fit one wavefront");
  // Tile buffers, double buffered: Q tiles Qs0 + buf TILE D, dO tiles Gs0 + buf TILE D, base-2 row
  // statistic Ls0 + buf TILE, -D_i Ds0 + buf TILE.  The plain dense kernel (no mask, no dropout)
  // unrolls its tile loop by two, so that the buffer index is a constant, and keeps all of them in
  // one LDS block (row vectors first): every LDS address is then a per-lane register plus an
  // immediate.  The other forms have no registers for two copies of the loop body and keep the
  // separate arrays (the form their register allocation is tuned to).
  constexpr int UNROLL = (!CAUSAL && !DROPOUT && !SPARSE) ? 2 : 1;
  T *Qs0, *Gs0;
  float *Ls0, *Ds0;
  if constexpr (UNROLL == 2) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * TILE * sizeof(float) + 4 * TILE * D * sizeof(T)];
    Ls0 = (float*)smem;
    Ds0 = Ls0 + 2 * TILE;
    Qs0 = (T*)(smem + 4 * TILE * sizeof(float));
    Gs0 = Qs0 + 2 * TILE * D;
  } else {
    __shared__ __attribute__((aligned(16))) T Qs[2 * TILE * D];
    __shared__ __attribute__((aligned(16))) T Gs[2 * TILE * D];
    __shared__ __attribute__((aligned(16))) float Ls[2 * TILE];
    __shared__ __attribute__((aligned(16))) float Ds[2 * TILE];
    Qs0 = Qs; Gs0 = Gs; Ls0 = Ls; Ds0 = Ds;
  }
  // dropout: the keep bits are exchanged along 16-lane rows either through one 64-word LDS slot per
  // wavefront (four 16-byte reads per pass) or by row broadcasts (sixteen per pass, no memory); the
  // forms that are short of registers keep the broadcasts, whose results need no aligned quadruples
  constexpr bool ROW_LDS = DROPOUT && !CAUSAL && !SPARSE;
  __shared__ __attribute__((aligned(16))) uint32_t Kb[ROW_LDS ? NT / 64 : 1][64];

  const int n_kt = a.T;   // ceil(N / 128): the last key block may be ragged
  // Work assignment.  Dense: one key block per workgroup; under the causal mask key block k is
  // visited by N/64 - 2k query tiles, so a workgroup takes the pair (k, n_kt - 1 - k), one per
  // round.  Block-sparse (as in attn_bwd_dkv.hip): the first 8 * chunk workgroups take one mask
  // column each and leave the heavy ones alone; those were cut into segments by
  // sparse_plan_kernel and the remaining workgroups walk that segment list.
  const int n_col_groups = kXcds * a.chunk;
  // (the list workgroups come first in the grid, a multiple of the XCD count of them, so that the
  // long segments start with the launch instead of queueing behind every column)
  const int n_list = SPARSE ? (int)gridDim.x - n_col_groups : 0;
  const bool list_mode = SPARSE && (int)blockIdx.x < n_list;
  constexpr bool PAIRED = CAUSAL && !SPARSE;
  const int n_pair = (n_kt + 1) / 2;
  for (int round = 0;; ++round) {
  int item, skip_blocks = 0, take_blocks = 0x7fffffff;
  bool heavy = false, last_round = true;
  if (!list_mode) {
    item = xcd_item(a.n_items, a.chunk, (int)blockIdx.x - n_list);
    if (item < 0) return;
    if constexpr (SPARSE) {
      if (a.colcnt[item] > a.seglist[2]) return;
    }
    if constexpr (PAIRED) {
      const int q = item % n_pair;
      last_round = round == 1 || q == n_kt - 1 - q;
      item = (item / n_pair) * n_kt + (round == 0 ? q : n_kt - 1 - q);
    }
  } else {
    const int idx = (int)blockIdx.x + round * n_list;
    if (idx >= a.seglist[0]) return;
    const int e = a.seglist[kSegHeader + idx];
    item = e / kMaxSegs;
    const int seg = e % kMaxSegs;
    const int cnt = a.colcnt[item];
    const int nseg = min((int)kMaxSegs, (cnt + kSegBlocks - 1) / kSegBlocks);
    const int seg_len = (cnt + nseg - 1) / nseg;
    skip_blocks = seg * seg_len;
    take_blocks = seg_len;
    heavy = true;
  }
  const int bh = item / n_kt;
  const int kt = item % n_kt;
  const int b = bh / a.H, h = bh % a.H;
  const int64_t head_off = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const T* __restrict__ Qg = (const T*)a.Q + head_off;
  const T* __restrict__ Gg = (const T*)a.dO + head_off;
  // padded to a multiple of 128 rows per head: +inf / 0 beyond a ragged end, so those query rows
  // (whose Q and dO tile rows are copies of the last real row) contribute P = 0 and dS = 0
  const float* __restrict__ Lg = a.L2vec + (int64_t)bh * a.Nr;
  const float* __restrict__ Dg = a.Dvec + (int64_t)bh * a.Nr;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int kw0 = kt * 128 + wave * 32;
  const int kj = kw0 + r;  // this lane's key (>= N beyond a ragged end: masked like a padded key, never stored)

  // loop-invariant B operands: the K and V fragments of this lane's key
  T8 kf[KK], vf[KK];
  {
    const int64_t row_off = head_off + (int64_t)min(kj, a.N - 1) * a.sn;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (D == 32 && 16 * kk + 8 * g >= a.dvalid) {   // head dimension 16: the upper columns are zeros
#pragma unroll
        for (int e = 0; e < 8; ++e) { kf[kk][e] = (T)0.f; vf[kk][e] = (T)0.f; }
        continue;
      }
      kf[kk] = *(const T8*)((const T*)a.K + row_off + 16 * kk + 8 * g);
      vf[kk] = *(const T8*)((const T*)a.V + row_off + 16 * kk + 8 * g);
    }
  }
  // The fragments must have arrived before the tile loop: a wait for them inside the loop would
  // also wait for the asynchronous tile copies in flight there.
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  f32x16 dv[DB], dk[DB];   // dV^T, dK^T (rows d, column = this lane's key)
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dv[db][i] = 0.f; dk[db][i] = 0.f; }

  // key-padding mask: key blocks and query tiles at or beyond the batch's length are not visited
  // (rows >= len inside the last tile have LSE = -inf, hence P = 0); masked keys get P = 0
  const int len = a.klen ? min(max(a.klen[b], 0), a.N) : a.N;
  TileIter<SPARSE> it;
  if constexpr (SPARSE)
    it.init(a.mask + (int64_t)h * a.mask_sh + kt, a.T, CAUSAL ? kt : 0,
            kt * 128 >= len ? 0 : min(a.T, (len + 127) / 128), skip_blocks, take_blocks);
  else
    it.init(nullptr, 0, CAUSAL ? 2 * kt : 0, kt * 128 >= len ? 0 : (len + TILE - 1) / TILE);   // len <= N

  TrOffsets<D> tro;
  tro.init();
  TileAsync<T, D, 4> dma;
  dma.init(a.sn, wave, D == 32 ? a.dvalid : D);
  if (D == 32 && a.dvalid < D) {   // the copies leave columns >= 16 of the tile buffers untouched
    zero_tiles(Qs0, 2 * TILE * D);   // (again in every round: the buffers staged output rows)
    zero_tiles(Gs0, 2 * TILE * D);
    __syncthreads();
  }
  auto fetch_tile = [&](int t, int buf) {
    dma.copy_rows(Qg, a.sn, t * TILE, a.N, Qs0 + buf * TILE * D);
    dma.copy_rows(Gg, a.sn, t * TILE, a.N, Gs0 + buf * TILE * D);
    if (wave == 1) async_copy_b32(Lg + t * TILE + lane, __builtin_amdgcn_readfirstlane(lds_addr(Ls0 + buf * TILE)));
    if (wave == 2) async_copy_b32(Dg + t * TILE + lane, __builtin_amdgcn_readfirstlane(lds_addr(Ds0 + buf * TILE)));
  };
  const float c = a.scale_log2;

  // LDS operand reads run PF fragments ahead of the MFMA that consumes them
  constexpr int PF = 4;
  // out[qb] = Tile[32 qb .. +31][:] . frags, starting from zero or (with_init: a literal at every
  // call, a test of the pointer would be evaluated at run time) from the 64 per-row values at cinit
  auto row_product = [&](const T* tile, const T8 (&bfrag)[KK], const bool with_init, const float* cinit,
                         f32x16 (&out)[2]) {
    auto frag = [&](int f) { return *(const T8*)(tile + lds_off<D>(32 * (f & 1) + r, 2 * (f >> 1) + g)); };  // f = 2 kk + qb
    T8 ring[PF];
#pragma unroll
    for (int f = 0; f < PF; ++f) ring[f] = frag(f);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < 2 * KK; ++f) {
      const T8 cur = ring[f % PF];
      if (f < 2) {
        f32x16 z;
        if (with_init) {
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            const f32x4 c4 = *(const f32x4*)(cinit + 32 * f + 8 * i4 + 4 * g);
#pragma unroll
            for (int e = 0; e < 4; ++e) z[4 * i4 + e] = c4[e];
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) z[i] = 0.f;
        }
        out[f & 1] = mfma32(cur, bfrag[f >> 1], z);
      } else {
        out[f & 1] = mfma32(cur, bfrag[f >> 1], out[f & 1]);
      }
      if (f + PF < 2 * KK) ring[f % PF] = frag(f + PF);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // acc^T += Tile^T . frag   (contraction over the 64 queries of the tile)
  auto col_product = [&](const T* tile, const T8 (&bfrag)[4], f32x16 (&acc)[DB]) {
    auto frag = [&](int f) {   // f = DB cc + db: consecutive MFMAs hit different accumulators
      const T* base = tile + 16 * (f / DB) * D;
      return tr_frag<T8>(base + tro.off[f % DB][0], base + tro.off[f % DB][1]);
    };
    T8 ring[PF];
#pragma unroll
    for (int f = 0; f < PF; ++f) ring[f] = frag(f);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int f = 0; f < 4 * DB; ++f) {
      const T8 cur = ring[f % PF];
      acc[f % DB] = mfma32(cur, bfrag[f / DB], acc[f % DB]);
      if (f + PF < 4 * DB) ring[f % PF] = frag(f + PF);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Dropout bits in this layout: see draw_keep_lane_key() / keep_words_lane_key() in attn_common.h.
  const int kbit = r & 15;   // position of this lane's key in the 16-key group of a draw
  auto draw_keep = [&](int i0) {
    return draw_keep_lane_key(i0, kj, r, g, bh, a.offset_lo, a.seed_lo, a.seed_hi, a.drop_thr);
  };

  // ---- pipeline over the query tiles of this key block: tile t + 1 streams in while t is used
  int buf_rt = 0;
  int t = it.next();
  if (t >= 0) fetch_tile(t, 0);
  wait_async_copies();
  __syncthreads();
  while (t >= 0) {
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    const int buf = UNROLL == 2 ? u : buf_rt;
    const int t_next = it.next();
    if (t_next >= 0) fetch_tile(t_next, buf ^ 1);
    const int i0 = t * TILE;
    if (!CAUSAL || i0 + TILE - 1 >= kw0) {
      f32x16 s[2], dp[2];
      row_product(Qs0 + buf * TILE * D, kf, false, nullptr, s);                // S = Q K^T
      // this lane's packed keep bits; the words of a row group are fetched where they are used
      uint32_t drawn = 0;
      uint32_t* const kslot = Kb[ROW_LDS ? (threadIdx.x >> 6) : 0];
      if constexpr (DROPOUT) drawn = draw_keep(i0);
      if constexpr (ROW_LDS) keep_row_store(kslot, drawn);
      if (kw0 + 32 > len) {   // this wavefront holds padded keys: their logits become -inf, hence P = 0
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (kj >= len) s[qb][i] = -INFINITY;
      }
      // P = exp(S - L), kept in fp32 in s[] for dS; the 16-bit (dropped) copy feeds dV
      T8 pf[4];
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        KeepLK4 kw = {};
        if constexpr (ROW_LDS) kw = keep_row_load(kslot, i4);
        else if constexpr (DROPOUT) kw = keep_words_lane_key(drawn, i4);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          const f32x4 l4 = *(const f32x4*)(Ls0 + buf * TILE + 32 * qb + 8 * i4 + 4 * g);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * i4 + e;
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][i], c, -l4[e]));
            if (CAUSAL && kj > i0 + 32 * qb + 8 * i4 + 4 * g + e) p = 0.f;
            s[qb][i] = p;
            const int cc = 2 * qb + (i4 >> 1), tt = 4 * (i4 & 1) + e;
            if constexpr (DROPOUT) {
              pf[cc][tt] = (T)keep_or_zero(p, keep_mask_lane_key(kw.w[e], kbit + 16 * qb));
            } else {
              pf[cc][tt] = (T)p;
            }
          }
        }
      }
      col_product(Gs0 + buf * TILE * D, pf, dv);                          // dV^T += dO^T P_dropped
      // dP = dO V^T; without dropout it starts from -D, so the result is dP - D
      row_product(Gs0 + buf * TILE * D, vf, !DROPOUT, Ds0 + buf * TILE, dp);
      T8 dsf[4];
      // (the keep words are fetched again here rather than kept from the P pass: sixteen registers
      // held across the dP product would spill; the empty statement keeps the compiler from merging
      // the two sets of broadcasts)
      if constexpr (DROPOUT && !ROW_LDS) asm volatile("" : "+v"(drawn));
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        KeepLK4 kw = {};
        if constexpr (ROW_LDS) kw = keep_row_load(kslot, i4);
        else if constexpr (DROPOUT) kw = keep_words_lane_key(drawn, i4);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          f32x4 d4 = {0.f, 0.f, 0.f, 0.f};
          if constexpr (DROPOUT) d4 = *(const f32x4*)(Ds0 + buf * TILE + 32 * qb + 8 * i4 + 4 * g);   // -D_i
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * i4 + e;
            const int cc = 2 * qb + (i4 >> 1), tt = 4 * (i4 & 1) + e;
            float dpv = dp[qb][i];
            if constexpr (DROPOUT) {
              dpv = dropped_dp_minus_d(dpv, a.keep_scale, keep_mask_lane_key(kw.w[e], kbit + 16 * qb), d4[e]);
            }
            dsf[cc][tt] = (T)(s[qb][i] * dpv);
          }
        }
      }
      col_product(Qs0 + buf * TILE * D, dsf, dk);                         // dK^T += Q^T dS
    }
    wait_async_copies();
    __syncthreads();   // the next tile has landed, and everyone is done with this buffer
    buf_rt ^= 1;
    t = t_next;
    if (t < 0) break;
  }
  }

  if (SPARSE && heavy) {
    // one of several segments of this column: sum in fp32; sparse_finish_kernel converts.  The loop
    // ended on a barrier: the two Q buffers stage the rows of wavefronts 0 and 1, the two dO buffers
    // those of wavefronts 2 and 3 (32 x D floats each), first for dV, then for dK
    float* stage = (float*)(wave < 2 ? Qs0 : Gs0) + (wave & 1) * 32 * D;
    const int64_t acc_row0 = ((int64_t)bh * a.N + kw0) * D;
    atomic_add_rows_coalesced<D>(stage, a.dVacc + acc_row0, dv, DROPOUT ? a.keep_scale : 1.f, D == 32 ? a.dvalid : D);
    atomic_add_rows_coalesced<D>(stage, a.dKacc + acc_row0, dk, a.tau, D == 32 ? a.dvalid : D);
  } else {
    // the loop ends on a barrier (or never touched LDS): the tile buffers stage the output rows
    T* stage_v = Qs0 + wave * 32 * D;   // 4 wavefronts x 32 rows = the two Q buffers
    T* stage_k = Gs0 + wave * 32 * D;
    store_rows_coalesced<T, D>(stage_v, (T*)a.dV + head_off + (int64_t)kw0 * a.sn, a.sn, dv,
                               DROPOUT ? a.keep_scale : 1.f, a.N - kw0, D == 32 ? a.dvalid : D);
    store_rows_coalesced<T, D>(stage_k, (T*)a.dK + head_off + (int64_t)kw0 * a.sn, a.sn, dk, a.tau, a.N - kw0,
                               D == 32 ? a.dvalid : D);
  }
  if (!list_mode && last_round) return;
  __syncthreads();   // LDS is reused by the next key block
  }  // for round
}

template <typename T, int D>
int launch_td(KArgs a, bool causal, bool dropout, bool sparse, int extra_groups, hipStream_t s) {
  if (causal && !sparse) {   // items are pairs of key blocks
    a.n_items = a.B * a.H * ((a.T + 1) / 2);
    a.chunk = (a.n_items + kXcds - 1) / kXcds;
  }
  const dim3 grid(kXcds * a.chunk + (sparse ? extra_groups : 0)), block(NT);
#define ATTN_DKV_FR_CASE(C, P, S)                                                     \
  if (causal == C && dropout == P && sparse == S) {                                   \
    hipLaunchKernelGGL((dkv_fr_kernel<T, D, C, P, S>), grid, block, 0, s, a);         \
    return (int)hipGetLastError();                                                    \
  }
  ATTN_DKV_FR_CASE(false, false, false)
  ATTN_DKV_FR_CASE(true, false, false)
  ATTN_DKV_FR_CASE(false, true, false)
  ATTN_DKV_FR_CASE(true, true, false)
  ATTN_DKV_FR_CASE(false, false, true)
  ATTN_DKV_FR_CASE(true, false, true)
  ATTN_DKV_FR_CASE(false, true, true)
  ATTN_DKV_FR_CASE(true, true, true)
#undef ATTN_DKV_FR_CASE
  return (int)hipErrorInvalidValue;
}

}  // namespace

// sparse: the caller (attn_bwd_dkv.hip) has run the column count / plan kernels and runs the
// finish kernel afterwards; extra_groups workgroups walk the list of heavy-column segments.
int launch_dkv_fr(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, int extra_groups,
                  hipStream_t s) {
  if (dtype == 0 && d == 32) return launch_td<_Float16, 32>(a, causal, dropout, sparse, extra_groups, s);
  if (dtype == 1 && d == 32) return launch_td<__bf16, 32>(a, causal, dropout, sparse, extra_groups, s);
  if (dtype == 0 && d == 64) return launch_td<_Float16, 64>(a, causal, dropout, sparse, extra_groups, s);
  if (dtype == 1 && d == 64) return launch_td<__bf16, 64>(a, causal, dropout, sparse, extra_groups, s);
  return (int)hipErrorInvalidValue;
}

}  // namespace attn
