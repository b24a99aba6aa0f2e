// dK / dV kernel of the backward pass with the work of a key block split by ROLE between two
// wavefronts that share a SIMD.
//
// Arithmetic: Algorithm 4 of the paper for one block of 128 keys, swept over 64-query tiles:
//     S = Q K^T, P = exp(S - L), dV += (P o Z)^T dO, dP = (dO V^T) o Z, dS = P o (dP - D), dK += tau dS^T Q.
// A workgroup is 8 wavefronts.  Wavefronts w and w + 4 (same SIMD) both own keys
// kt*128 + 32 w .. + 31, in the "lane = key" register layout (see attn_bwd.hip), but
//     role A (w < 4):  S tile -> P (exp) -> dV^T += dO^T P_dropped      keeps K fragments, dV accumulator
//     role B (w >= 4): dP tile -> dS = P (dP Z - D) -> dK^T += Q^T dS   keeps V fragments, dK accumulator
// so each wavefront needs half of the accumulators and operand fragments (<= 256 registers, two
// wavefronts per SIMD), the four tile products are done once each, and the two different
// instruction streams on a SIMD overlap MFMA with the exp / dS VALU work.  B needs A's P: A
// leaves it (as fp16 whatever the tensor type, in B's own register layout, plus the dropout keep
// bits) in LDS, and B runs
// its dS / dK part one tile behind, so one workgroup barrier per tile orders everything.
// Tiles arrive by asynchronous global-to-LDS copies (no staging registers, no LDS store
// instructions).  Issuing a tile's 34 copies stalls a wavefront for hundreds of clocks (the
// vector memory path of a compute unit takes 64 bytes per clock), so only the role A wavefronts
// issue them, at the END of their iteration, where they would otherwise idle waiting for role B,
// and for the tile two iterations ahead, so the data has a full iteration to land.
// LDS: Q and D x4 (tile j is read by A in iteration j and by B in iteration j+1, tile j+2 is
// being written), dO and L x3, P exchange x2.
#include "attn_common.h"
#include "attn_tiles.h"

#include <cstdlib>
#include <type_traits>

namespace attn {
namespace {

constexpr int NT = 512;
constexpr int TILE = 64;
constexpr int kListGroups = 512;

template <typename T, int D, bool CAUSAL, bool DROPOUT, bool SPARSE>
__global__ __launch_bounds__(NT) void dkv_rs_kernel(const KArgs a) {
  typedef typename Vec<T>::x8 T8;
  constexpr int KK = D / 16, DB = D / 32;
  __shared__ __attribute__((aligned(16))) T Qs[4][TILE * D];
  __shared__ __attribute__((aligned(16))) T Gs[3][TILE * D];      // dO tiles
  __shared__ __attribute__((aligned(16))) float Ls[3][TILE];      // base-2 row statistic
  __shared__ __attribute__((aligned(16))) float Ds[4][TILE];      // -D_i
  // P exchange [buf][pair][chunk][lane]: always fp16 (11 significant bits, more than bf16 keeps; P <= 1
  // and anything below 2^-24 contributes nothing to dS), because role B can multiply an fp16 half
  // by an fp32 value in one mixed-precision instruction, with no unpacking
  __shared__ __attribute__((aligned(16))) f16x8 Px[2][4][4][64];
  __shared__ __attribute__((aligned(16))) uint32_t Kw[2][4][64];                                // dropout keep words [buf][pair][lane]

  const int n_kt = a.T;   // ceil(N / 128): the last key block may be ragged
  // Work assignment.  Dense: one key block per workgroup; under the causal mask key block k is
  // visited by N/64 - 2k query tiles, so a workgroup takes the pair (k, n_kt - 1 - k), one per
  // round, and all workgroups do the same amount of work.  Block-sparse: the first 8 * chunk
  // workgroups take one mask column each and leave the heavy ones (many kept blocks, e.g. a
  // global-token column) alone; those were cut into segments by sparse_plan_kernel and the
  // remaining workgroups walk that segment list.
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
    const int len = (cnt + nseg - 1) / nseg;
    skip_blocks = seg * len;
    take_blocks = len;
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
  const float* __restrict__ Lg = a.L2vec + (int64_t)bh * a.Nr;   // base 2, +inf for fully masked rows
  const float* __restrict__ Dg = a.Dvec + (int64_t)bh * a.Nr;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool role_b = wave >= 4;
  const int pair = wave & 3;
  const int r = lane & 31, g = lane >> 5;
  const int kw0 = kt * 128 + pair * 32;
  const int kj = kw0 + r;  // this lane's key (>= N beyond a ragged end: masked like a padded key, never stored)

  // loop-invariant B operands: K fragments for role A, V fragments for role B
  T8 kvf[KK];
  {
    const T* src = role_b ? (const T*)a.V : (const T*)a.K;
    const int64_t row_off = head_off + (int64_t)min(kj, a.N - 1) * a.sn;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
      kvf[kk] = *(const T8*)(src + row_off + 16 * kk + 8 * g);
  }
  // The fragments must have arrived before the tile loop: a wait for them inside the loop would
  // also wait for the asynchronous tile copies in flight there.
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  f32x16 acc[DB];  // role A: dV^T, role B: dK^T   (rows d, column = this lane's key)
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;
  f32x16 sd[2];    // role A: S, role B: dP   (rows = queries of the tile, column = key)

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
  TileAsync<T, D, 4> dma;   // the four role A wavefronts copy whole tiles
  dma.init(a.sn, wave & 3);
  // copies per tile issued by this wavefront (role A only): Q and dO shares, plus L (wave 1) or D (wave 2)
  constexpr int kTileCopies = 2 * TileAsync<T, D, 4>::PER_WAVE;
  // starts the copies of tile t into ring slots (q4, g3)
  auto fetch_tile = [&](int t, int q4, int g3) {
    dma.copy_rows(Qg, a.sn, t * TILE, a.N, Qs[q4]);
    dma.copy_rows(Gg, a.sn, t * TILE, a.N, Gs[g3]);
    if (wave == 1) async_copy_b32(Lg + t * TILE + lane, __builtin_amdgcn_readfirstlane(lds_addr(Ls[g3])));
    if (wave == 2) async_copy_b32(Dg + t * TILE + lane, __builtin_amdgcn_readfirstlane(lds_addr(Ds[q4])));
  };

  const float c = a.scale_log2;

  // LDS operand reads run PF fragments ahead of the MFMA that consumes them (the scheduling
  // barriers keep the compiler from shortening that distance), so the matrix pipe does not wait
  // for LDS latency on every instruction.
  constexpr int PF = 4;
  // product of a row-read tile with the register fragments: sd[qb] = Tile[32 qb .. +31][:] . kvf
  // The accumulators start from zero or (with_init: a literal at every call, a test of the pointer
  // would be evaluated at run time) from the 64 per-row values at cinit
  auto row_product = [&](const T* tile, const bool with_init, const float* cinit) {
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
        sd[f & 1] = mfma32(cur, kvf[f >> 1], z);
      } else {
        sd[f & 1] = mfma32(cur, kvf[f >> 1], sd[f & 1]);
      }
      if (f + PF < 2 * KK) ring[f % PF] = frag(f + PF);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // acc^T += Tile^T . frag   (contraction over the 64 queries of the tile)
  auto col_product = [&](const T* tile, const T8 (&bfrag)[4]) {
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

  // ---- role A, tile with first query i0, buffers (q3, p2)
  auto role_a = [&](int i0, int q4, int g3, int p2) {
    row_product(Qs[q4], false, nullptr);                         // S = Q K^T
    KeepLK kw = {};
    if constexpr (DROPOUT) {
      // the drawn bits go to LDS: the lanes of a 16-lane row read each other's words there, and
      // role B regenerates nothing, it reads them too
      keep_row_store(Kw[p2][pair], draw_keep(i0));
      kw = keep_row_load_all(Kw[p2][pair]);
    }
    if (kw0 + 32 > len) {   // this wavefront holds padded keys: their logits become -inf, hence P = 0
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (kj >= len) sd[qb][i] = -INFINITY;
    }
    T8 pf[4], pfull[4];
    f16x8 ph[4];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 l4 = *(const f32x4*)(&Ls[g3][32 * qb + 8 * i4 + 4 * g]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * i4 + e;
          float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sd[qb][i], c, -l4[e]));
          if (CAUSAL && kj > i0 + 32 * qb + 8 * i4 + 4 * g + e) p = 0.f;
          const int cc = 2 * qb + (i4 >> 1), t = 4 * (i4 & 1) + e;
          pfull[cc][t] = (T)p;
          ph[cc][t] = (_Float16)p;
          if constexpr (DROPOUT) {
            pf[cc][t] = (T)keep_or_zero(p, keep_mask_lane_key(kw.w[i4][e], kbit + 16 * qb));
          }
        }
      }
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) Px[p2][pair][cc][lane] = ph[cc];
    if constexpr (DROPOUT) col_product(Gs[g3], pf);        // dV^T += dO^T P_dropped
    else col_product(Gs[g3], pfull);
  };
  // ---- role B, second half for the previous tile: dS from sd (= dP) and A's P, then dK
  auto role_b_ds_dk = [&](int q4, int p2) {
    KeepLK kw = {};
    if constexpr (DROPOUT) kw = keep_row_load_all(Kw[p2][pair]);
    f16x8 pin[4];
    T8 dsf[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) pin[cc] = Px[p2][pair][cc][lane];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        f32x4 d4 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (DROPOUT) d4 = *(const f32x4*)(&Ds[q4][32 * qb + 8 * i4 + 4 * g]);   // -D_i
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * i4 + e;
          const int cc = 2 * qb + (i4 >> 1), t = 4 * (i4 & 1) + e;
          float dpv = sd[qb][i];   // without dropout: already dP - D
          if constexpr (DROPOUT) {
            dpv = dropped_dp_minus_d(dpv, a.keep_scale, keep_mask_lane_key(kw.w[i4][e], kbit + 16 * qb), d4[e]);
          }
          // (an fma with an fp16 operand is one v_fma_mix_f32: the half is widened inside the instruction)
          dsf[cc][t] = (T)__builtin_fmaf((float)pin[cc][t], dpv, 0.f);
        }
      }
    col_product(Qs[q4], dsf);                               // dK^T += Q^T dS
  };

  // ---- pipeline over the tiles of this key block
  int t0 = it.next();
  int t1 = t0 >= 0 ? it.next() : -1;
  if (!role_b) {
    if (t0 >= 0) fetch_tile(t0, 0, 0);
    if (t1 >= 0) fetch_tile(t1, 1, 1);
  }
  int q4 = 0, g3 = 0, p2 = 0;  // ring slots of the current tile: j % 4, j % 3, j % 2
  bool have_prev = false, prev_active = false;
  while (t0 >= 0) {
    if (!role_b) {
      // tile t0 must have landed; the copies of t1, issued after it, may still be in flight
      if (t1 < 0) wait_async_copies();
      else if (wave == 1 || wave == 2) wait_async_copies_but<kTileCopies + 1>();
      else wait_async_copies_but<kTileCopies>();
    }
    __syncthreads();           // tile t0 is visible to everyone; the slots of tile t0 - 2 are free
    const int t2 = t1 >= 0 ? it.next() : -1;
    const int i0 = t0 * TILE;
    const bool active = !CAUSAL || i0 + TILE - 1 >= kw0;
    if (!role_b) {
      if (active) role_a(i0, q4, g3, p2);
      if (t2 >= 0) fetch_tile(t2, (q4 + 2) & 3, g3 == 0 ? 2 : g3 - 1);   // slots (j + 2) % 4, (j + 2) % 3
    } else {
      if (have_prev && prev_active) role_b_ds_dk((q4 + 3) & 3, p2 ^ 1);
      // dP = dO V^T; without dropout it starts from -D, so the result is dP - D
      if (active) row_product(Gs[g3], !DROPOUT, Ds[q4]);
    }
    have_prev = true;
    prev_active = active;
    t0 = t1;
    t1 = t2;
    q4 = (q4 + 1) & 3;
    g3 = g3 == 2 ? 0 : g3 + 1;
    p2 ^= 1;
  }
  __syncthreads();
  if (role_b && have_prev && prev_active) role_b_ds_dk((q4 + 3) & 3, p2 ^ 1);

  const float out_scale = role_b ? a.tau : (DROPOUT ? a.keep_scale : 1.f);
  if (SPARSE && heavy) {
    // one of several segments of this column: sum in fp32; sparse_finish_kernel converts.  The four
    // Q buffers stage 32 x D floats for each of four wavefronts: role A's dV first, then role B's dK
    __syncthreads();   // role B has finished reading the tiles
    float* stage = (float*)&Qs[0][0] + pair * 32 * D;
    const int64_t acc_row0 = ((int64_t)bh * a.N + kw0) * D;
    if (!role_b) atomic_add_rows_coalesced<D>(stage, a.dVacc + acc_row0, acc, out_scale, D == 32 ? a.dvalid : D);
    __syncthreads();
    if (role_b) atomic_add_rows_coalesced<D>(stage, a.dKacc + acc_row0, acc, out_scale, D == 32 ? a.dvalid : D);
  } else {
    __syncthreads();   // role B has finished reading the tiles: they stage the output rows
    T* stage = (role_b ? &Gs[0][0] : &Qs[0][0]) + pair * 32 * D;
    store_rows_coalesced<T, D>(stage, (T*)(role_b ? a.dK : a.dV) + head_off + (int64_t)kw0 * a.sn, a.sn, acc,
                               out_scale, a.N - kw0);
  }
  if (!list_mode && last_round) return;
  __syncthreads();   // LDS is reused by the next segment / key block
  }  // for round
}

// Block-sparse preparation, step 1: kept blocks per mask column (rows >= column under a causal
// mask) and their total.  One 1024-thread group per (bh, 64 consecutive columns): thread = (column,
// one of 16 row groups), so that the 64 lanes of a wavefront read 64 consecutive mask bytes of one
// row (a thread per column entry of one column reads one byte per 64-byte line).
constexpr int kCountRowGroups = 16;
__global__ __launch_bounds__(64 * kCountRowGroups) void sparse_count_kernel(const KArgs a) {
  __shared__ int part[kCountRowGroups][64];
  const int n_kt = a.T;
  const int n_cg = (n_kt + 63) / 64;
  const int bh = blockIdx.x / n_cg, cg = blockIdx.x % n_cg;
  const int h = bh % a.H;
  const int c = threadIdx.x & 63, rg = threadIdx.x >> 6;
  const int kt = cg * 64 + c;
  const int len = a.klen ? min(max(a.klen[bh / a.H], 0), a.N) : a.N;
  int cnt = 0;
  if (kt < n_kt) {
    const uint8_t* col = a.mask + (int64_t)h * a.mask_sh + kt;
    const int first = a.causal ? kt : 0;                                     // same row range as the
    const int limit = kt * 128 >= len ? 0 : min(a.T, (len + 127) / 128);     // tile iterators of the dK/dV kernels
    for (int blk = first + rg; blk < limit; blk += kCountRowGroups) cnt += col[(int64_t)blk * a.T] != 0;
  }
  part[rg][c] = cnt;
  __syncthreads();
  if (rg == 0) {   // one wavefront: the column totals, then their sum as ONE atomic per workgroup
#pragma unroll
    for (int g = 1; g < kCountRowGroups; ++g) cnt += part[g][c];
    if (kt < n_kt) a.colcnt[bh * n_kt + kt] = cnt;
    int sum = kt < n_kt ? cnt : 0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
    if (c == 0 && sum > 0) atomicAdd(a.seglist + 1, sum);
  }
}

// Step 2: the heavy threshold, the segment list of the heavy columns and zeroed fp32
// accumulators for them.  One 256-thread group per kPlanCols consecutive columns (bh, kt): most
// columns are light and need one comparison, so a group per column would be launch overhead only.
constexpr int kPlanCols = 16;
template <int D>
__global__ __launch_bounds__(256) void sparse_plan_kernel(const KArgs a) {
  __shared__ int heavy_col[kPlanCols];
  const int n_kt = a.T;
  const int n_cols = a.B * a.H * n_kt;
  const int first = blockIdx.x * kPlanCols;
  const int thr = max((int)kHeavyBlocks, a.seglist[1] / (2 * kComputeUnits));
  if (blockIdx.x == 0 && threadIdx.x == 0) a.seglist[2] = thr;
  if (threadIdx.x < kPlanCols) {
    const int item = first + (int)threadIdx.x;
    const int cnt = item < n_cols ? a.colcnt[item] : 0;
    heavy_col[threadIdx.x] = cnt > thr;
    if (cnt > thr) {
      const int nseg = min((int)kMaxSegs, (cnt + kSegBlocks - 1) / kSegBlocks);
      const int at = atomicAdd(a.seglist, nseg);
      for (int sgi = 0; sgi < nseg; ++sgi) a.seglist[kSegHeader + at + sgi] = item * kMaxSegs + sgi;
    }
  }
  __syncthreads();
  for (int cidx = 0; cidx < kPlanCols; ++cidx) {
    if (!heavy_col[cidx]) continue;
    const int item = first + cidx;
    const int bh = item / n_kt, kt = item % n_kt;
    const int64_t off = ((int64_t)bh * a.N + (int64_t)kt * 128) * D;
    for (int i = threadIdx.x; i < 128 * D / 4; i += 256) {
      const f32x4 z = {0.f, 0.f, 0.f, 0.f};
      *(f32x4*)(a.dKacc + off + 4 * i) = z;
      *(f32x4*)(a.dVacc + off + 4 * i) = z;
    }
  }
}

// Block-sparse finish: dK, dV of the split columns, fp32 accumulators -> 16-bit outputs (same
// grouping of columns as the plan kernel).
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_finish_kernel(const KArgs a) {
  typedef typename Vec<T>::x4 T4;
  const int n_kt = a.T;
  const int n_cols = a.B * a.H * n_kt;
  const int thr = a.seglist[2];
  for (int cidx = 0; cidx < kPlanCols; ++cidx) {
    const int item = blockIdx.x * kPlanCols + cidx;
    if (item >= n_cols) return;
    if (a.colcnt[item] <= thr) continue;
    const int bh = item / n_kt, kt = item % n_kt;
    const int64_t head_off = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    const int64_t acc_off = ((int64_t)bh * a.N + (int64_t)kt * 128) * D;
    for (int i = threadIdx.x; i < 128 * D / 4; i += 256) {
      const int row = (4 * i) / D, colx = (4 * i) % D;
      const f32x4 k4 = *(const f32x4*)(a.dKacc + acc_off + 4 * i);
      const f32x4 v4 = *(const f32x4*)(a.dVacc + acc_off + 4 * i);
      T4 ko, vo;
#pragma unroll
      for (int e = 0; e < 4; ++e) { ko[e] = (T)k4[e]; vo[e] = (T)v4[e]; }
      const int64_t o = head_off + (int64_t)(kt * 128 + row) * a.sn + colx;
      if (D == 32 && colx >= a.dvalid) continue;   // head dimension 16: the tensors' rows end there
      *(T4*)((T*)a.dK + o) = ko;
      *(T4*)((T*)a.dV + o) = vo;
    }
  }
}

// dK/dV override 1 keeps the role-split kernel at every head dimension (comparisons and tests)
bool force_role_split() { return dkv_variant() == 1; }

template <typename T, int D>
int launch_td(KArgs a, bool causal, bool dropout, bool sparse, hipStream_t s) {
  const int cols = a.B * a.H * a.T;
  if (sparse) {
    a.causal = causal;
    hipLaunchKernelGGL(sparse_count_kernel, dim3(a.B * a.H * ((a.T + 63) / 64)), dim3(64 * kCountRowGroups), 0, s, a);
    hipLaunchKernelGGL((sparse_plan_kernel<D>), dim3((cols + kPlanCols - 1) / kPlanCols), dim3(256), 0, s, a);
    const int e = (int)hipGetLastError();
    if (e != 0) return e;
  }
  // block-sparse: kListGroups extra workgroups walk the list of heavy-column segments
  if (causal && !sparse) {   // items are pairs of key blocks
    a.n_items = a.B * a.H * ((a.T + 1) / 2);
    a.chunk = (a.n_items + kXcds - 1) / kXcds;
  }
  if (sparse && choose_dkv(a, D, causal, dropout, sparse) == kDkvOneWave) {
    // d <= 64: the kernel in which one wavefront does all four products, same work assignment
    int e = launch_dkv_fr(a, std::is_same<T, __bf16>::value ? 1 : 0, D, causal, dropout, true, kListGroups, s);
    if (e == 0) {
      hipLaunchKernelGGL((sparse_finish_kernel<T, D>), dim3((cols + kPlanCols - 1) / kPlanCols), dim3(256), 0, s, a);
      e = (int)hipGetLastError();
    }
    return e;
  }
  const dim3 grid(kXcds * a.chunk + (sparse ? kListGroups : 0)), block(NT);
#define ATTN_DKV_CASE(C, P, S)                                                    \
  if (causal == C && dropout == P && sparse == S) {                               \
    hipLaunchKernelGGL((dkv_rs_kernel<T, D, C, P, S>), grid, block, 0, s, a);     \
    int e = (int)hipGetLastError();                                               \
    if (e == 0 && S) {                                                            \
      hipLaunchKernelGGL((sparse_finish_kernel<T, D>), dim3((cols + kPlanCols - 1) / kPlanCols), dim3(256), 0, s, a); \
      e = (int)hipGetLastError();                                                 \
    }                                                                             \
    return e;                                                                     \
  }
  ATTN_DKV_CASE(false, false, false)
  ATTN_DKV_CASE(true, false, false)
  ATTN_DKV_CASE(false, true, false)
  ATTN_DKV_CASE(true, true, false)
  ATTN_DKV_CASE(false, false, true)
  ATTN_DKV_CASE(true, false, true)
  ATTN_DKV_CASE(false, true, true)
  ATTN_DKV_CASE(true, true, true)
#undef ATTN_DKV_CASE
  return (int)hipErrorInvalidValue;
}

}  // namespace

int choose_dkv(const KArgs& a, int d, bool causal, bool dropout, bool sparse) {
  // Problems with d <= 64 take the kernel in which one wavefront does all four products
  // (attn_bwd_dkv_fr.hip; the block-sparse ones from inside launch_td, between the column
  // planning and the finish kernel).
  // (head dimension 16 exists in that kernel only)
  if (d <= 64 && (!force_role_split() || a.dvalid < d)) return kDkvOneWave;
  // d = 128, dense: the one-wavefront kernel with the V block in LDS (attn_bwd_dkv_fr128.hip)
  // (without dropout, with 64 keys per wavefront where a head has at least two blocks of 256 keys
  // and whole 32-query tiles: attn_bwd_dkv_w64.hip)
  // (dropout under the causal mask keeps the role-split kernel: measured 15 % faster than the
  // one-wavefront kernel at B H = 64, N = 1024 and equal at N = 4096; without a mask the
  // one-wavefront kernel is 1-6 % faster with dropout as well)
  if (!sparse && d == 128 && !force_role_split() && !(dropout && causal && dkv_variant() == 0)) {
    // measured against the 32-key kernel: 1 % faster at N = 2048, 5 % at 4096, 7 % at 16384; slower below,
    // and slower under the causal mask at every length (its 256-key work items balance worse)
    const bool w64 = dkv_variant() == 3 || (dkv_variant() == 0 && !causal && a.N >= 2048);
    return w64 && !dropout && a.N >= 512 && a.N % 32 == 0 ? kDkvOneWave64 : kDkvOneWave128;
  }
  return kDkvRoleSplit;
}

int launch_dkv_rs(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, hipStream_t s) {
  const int choice = choose_dkv(a, d, causal, dropout, sparse);
  if (!sparse && choice == kDkvOneWave) return launch_dkv_fr(a, dtype, d, causal, dropout, false, 0, s);
  if (choice == kDkvOneWave64) return launch_dkv_w64(a, dtype, causal, s);
  if (choice == kDkvOneWave128) return launch_dkv_fr128(a, dtype, causal, dropout, s);
  if (dtype == 0 && d == 32) return launch_td<_Float16, 32>(a, causal, dropout, sparse, s);
  if (dtype == 1 && d == 32) return launch_td<__bf16, 32>(a, causal, dropout, sparse, s);
  if (dtype == 0 && d == 64) return launch_td<_Float16, 64>(a, causal, dropout, sparse, s);
  if (dtype == 0 && d == 128) return launch_td<_Float16, 128>(a, causal, dropout, sparse, s);
  if (dtype == 1 && d == 64) return launch_td<__bf16, 64>(a, causal, dropout, sparse, s);
  if (dtype == 1 && d == 128) return launch_td<__bf16, 128>(a, causal, dropout, sparse, s);
  return (int)hipErrorInvalidValue;
}

}  // namespace attn
