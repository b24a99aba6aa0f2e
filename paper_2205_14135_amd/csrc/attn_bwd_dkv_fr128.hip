// dK / dV kernel for head dimension 128, dense problems, in which one wavefront
// does all four tile products of its 32 keys (the arrangement of
// attn_bwd_dkv_fr.hip carried to d = 128).
//
// Arithmetic: Algorithm 4 of the paper for one block of 128 keys, swept over 32-query tiles:
//     S = Q K^T, P = exp(S - L), dV += P^T dO, dP = dO V^T, dS = P o (dP - D), dK += tau dS^T Q.
// At d = 128 the two accumulators (dK^T, dV^T: 128 registers) and the K fragments (32) leave no
// room for the V fragments and for 64-query S / dP tiles, so here the V rows of the workgroup's 128
// keys stay in LDS (the dP product reads both operands from LDS) and the query tiles are 32 rows:
// Q/dO double buffers 4 x 8 KB + V 32 KB = 64 KB per workgroup, two free-running workgroups of four
// wavefronts per compute unit.  S and dP, and then dV and dK, are issued as alternating MFMA
// streams, so that consecutive instructions write different accumulators.  Measured 6 % faster
// than the role-split kernel of attn_bwd_dkv.hip at N = 4096 and 10 % at N = 1024.  Under the causal
// mask a workgroup takes one key block (not a pair: the loop over a pair costs registers this
// kernel does not have) and the blocks are dealt out heaviest first.  Dropout: a call of the
// generator decides 16 consecutive keys of a query, i.e. the 16 lanes of one row of the wavefront,
// which need the draws of the tile's 16 queries 8 i4 + 4 g + e: every lane draws one of them, packs
// the keep bits and the row exchanges them (draw_keep_lane_key / keep_words_lane_key in
// attn_common.h, here with 32-query tiles: one call per lane and tile).
#include <type_traits>

#include "attn_common.h"
#include "attn_tiles.h"

namespace attn {
namespace {

constexpr int NT = 256;
constexpr int QT = 32;    // queries per streamed tile
constexpr int D = 128;

template <typename T, bool CAUSAL, bool DROPOUT>
__global__ __launch_bounds__(NT, 2) void dkv_fr128_kernel(const KArgs a) {
  typedef typename Vec<T>::x8 T8;
  constexpr int KK = D / 16, DB = D / 32;
  // One LDS block, so that every address is a per-lane register plus a 16-bit immediate: the row
  // vectors first (1 KB), then the Q tiles, the dO tiles and the V rows of this key block.
  constexpr int kVecBytes = 4 * 64 * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kVecBytes + (4 * QT * D + 128 * D) * sizeof(T)];
  float* const Ls0 = (float*)smem;                 // base-2 row statistic: Ls0 + 64 buf (first QT entries used:
  float* const Ds0 = Ls0 + 2 * 64;                 // -D_i:                 Ds0 + 64 buf  a copy moves 64 floats)
  T* const Qs0 = (T*)(smem + kVecBytes);           // Q tiles:  Qs0 + buf QT D
  T* const Gs0 = Qs0 + 2 * QT * D;                 // dO tiles: Gs0 + buf QT D
  T* const Vb = Qs0 + 4 * QT * D;                  // V rows of this key block

  const int n_kt = a.T;   // ceil(N / 128): the last key block may be ragged
  const int item = xcd_item(a.n_items, a.chunk);
  if (item < 0) return;
  int bh = item / n_kt;
  int kt = item % n_kt;
  if constexpr (CAUSAL) {
    // Key block k is visited by the query tiles from the diagonal on, so its work falls with k.
    // The key blocks of a.group consecutive heads are dealt out together, heaviest first, so that
    // the items a compute unit receives last are light ones (the host sizes the group so that the
    // Q and dO of its heads, the L2 working set of an XCD, stay within 8 MiB).
    const int n_heads = a.B * a.H;
    const int grp0 = (bh / a.group) * a.group;             // first head of this group
    const int gsz = min(a.group, n_heads - grp0);          // heads in it (the last group may be short)
    const int within = (bh - grp0) * n_kt + kt;            // position inside the group's items
    bh = grp0 + within % gsz;
    kt = within / gsz;
  }
  const int b = bh / a.H, h = bh % a.H;
  const int64_t head_off = (int64_t)b * a.sb + (int64_t)h * a.sh;
  const T* __restrict__ Qg = (const T*)a.Q + head_off;
  const T* __restrict__ Gg = (const T*)a.dO + head_off;
  const T* __restrict__ Vg = (const T*)a.V + head_off;
  const float* __restrict__ Lg = a.L2vec + (int64_t)bh * a.Nr;
  const float* __restrict__ Dg = a.Dvec + (int64_t)bh * a.Nr;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int kw0 = kt * 128 + wave * 32;
  const int kj = kw0 + r;

  T8 kf[KK];
  {
    const int64_t row_off = head_off + (int64_t)min(kj, a.N - 1) * a.sn;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = *(const T8*)((const T*)a.K + row_off + 16 * kk + 8 * g);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): before any asynchronous copy is in flight
  f32x16 dv[DB], dk[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) { dv[db][i] = 0.f; dk[db][i] = 0.f; }

  const int len = a.klen ? min(max(a.klen[b], 0), a.N) : a.N;
  const int first = CAUSAL ? kt * (128 / QT) : 0;   // causal: the tiles above the diagonal see none of these keys
  const int limit = kt * 128 >= len ? 0 : (len + QT - 1) / QT;

  TrOffsets<D> tro;
  tro.init();
  TileAsync<T, D, 4, QT> dma;      // 32-row tiles: two copy instructions per wavefront
  dma.init(a.sn, wave);
  TileAsync<T, D, 4, 64> dma64;    // the V block: two 64-row pieces
  dma64.init(a.sn, wave);
  auto fetch_tile = [&](int t, int buf) {
    dma.copy_rows(Qg, a.sn, t * QT, a.N, Qs0 + buf * QT * D);
    dma.copy_rows(Gg, a.sn, t * QT, a.N, Gs0 + buf * QT * D);
    const int row = min(t * QT + lane, a.Nr - 1);   // whole-wavefront copies: 64 floats, clamped to the head
    if (wave == 1) async_copy_b32(Lg + row, __builtin_amdgcn_readfirstlane(lds_addr(Ls0 + 64 * buf)));
    if (wave == 2) async_copy_b32(Dg + row, __builtin_amdgcn_readfirstlane(lds_addr(Ds0 + 64 * buf)));
  };
  const float c = a.scale_log2;
  constexpr int PF = 4;

  // V rows of this key block (rows >= N repeat the last one; their keys are masked)
  if (kt * 128 < a.N) dma64.copy_rows(Vg, a.sn, kt * 128, a.N, Vb);
  if (kt * 128 + 64 < a.N) dma64.copy_rows(Vg, a.sn, kt * 128 + 64, a.N, Vb + 64 * D);
  else if (kt * 128 < a.N) dma64.copy_rows(Vg, a.sn, kt * 128, a.N, Vb + 64 * D);   // all of these keys are masked
  if (first < limit) fetch_tile(first, 0);
  wait_async_copies();
  __syncthreads();
  // One query tile.  The buffer index is a compile-time constant (the loop below is unrolled by
  // two), so that every LDS address is a per-lane register plus an immediate offset.
  auto tile_step = [&](int t, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    if (t + 1 < limit) fetch_tile(t + 1, buf ^ 1);
    // causal: of the four tiles on the diagonal of the key block, wavefront w joins from the w-th
    // on, and masks inside that one: query 8 i4 + 4 g + e of the tile sees this lane's key iff
    // that number is >= kj - first query of the tile
    const int i0 = t * QT;
    const int hidden_below = CAUSAL && i0 == kw0 ? r - 4 * g : -(1 << 30);
    if (!CAUSAL || i0 >= kw0) {
      const T* Qt = Qs0 + buf * QT * D;
      const T* Gt = Gs0 + buf * QT * D;
      // ---- S = Q K^T and dP = dO V^T (32 queries x 32 keys each) as one stream of alternating
      // MFMAs: consecutive instructions write different accumulators.  dP starts from -D; its
      // second operand (the V fragments) comes from LDS too.
      f32x16 s, dp;
      {
        auto qfrag = [&](int kk) { return *(const T8*)(Qt + lds_off<D>(r, 2 * kk + g)); };
        auto gfrag = [&](int kk) { return *(const T8*)(Gt + lds_off<D>(r, 2 * kk + g)); };
        auto vfrag = [&](int kk) { return *(const T8*)(Vb + lds_off<D>(wave * 32 + r, 2 * kk + g)); };
        constexpr int PF2 = 2;
        T8 rq[PF2], rg[PF2], rv[PF2];
#pragma unroll
        for (int f = 0; f < PF2; ++f) { rq[f] = qfrag(f); rg[f] = gfrag(f); rv[f] = vfrag(f); }
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          // (with dropout -D joins after the mask: the product starts from zero)
          f32x4 c4 = {0.f, 0.f, 0.f, 0.f};
          if constexpr (!DROPOUT) c4 = *(const f32x4*)(Ds0 + 64 * buf + 8 * i4 + 4 * g);
#pragma unroll
          for (int e = 0; e < 4; ++e) { dp[4 * i4 + e] = c4[e]; s[4 * i4 + e] = 0.f; }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < KK; ++f) {
          const T8 cq = rq[f % PF2], cg = rg[f % PF2], cv = rv[f % PF2];
          s = mfma32(cq, kf[f], s);
          dp = mfma32(cg, cv, dp);
          if (f + PF2 < KK) { rq[f % PF2] = qfrag(f + PF2); rg[f % PF2] = gfrag(f + PF2); rv[f % PF2] = vfrag(f + PF2); }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      if (kw0 + 32 > len) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (kj >= len) s[i] = -INFINITY;
      }
      // dropout: this lane draws the tile's query 8 (u / 4) + 4 g + u % 4 (u = r % 16) for the 16 keys
      // of its row; bit u' of the word of lane u is key u' of that query
      uint32_t drawn = 0;
      if constexpr (DROPOUT) {
        const int u = r & 15;
        const u32x4 w = philox_draw16((uint32_t)kj >> 4, (uint32_t)(i0 + 8 * (u >> 2) + 4 * g + (u & 3)), (uint32_t)bh,
                                      a.offset_lo, a.seed_lo, a.seed_hi);
        drawn = keep_bits16(w, dropout_carry2(a.drop_thr));
      }
      T8 pf[2], dsf[2];
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 l4 = *(const f32x4*)(Ls0 + 64 * buf + 8 * i4 + 4 * g);
        KeepLK4 kw = {};
        f32x4 d4 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (DROPOUT) {
          kw = keep_words_lane_key(drawn, i4);
          d4 = *(const f32x4*)(Ds0 + 64 * buf + 8 * i4 + 4 * g);   // -D_i
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = 4 * i4 + e;
          float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c, -l4[e]));
          if (CAUSAL && 8 * i4 + e < hidden_below) p = 0.f;
          if constexpr (DROPOUT) {
            const uint32_t mask = keep_mask_lane_key(kw.w[e], r & 15);
            pf[i4 >> 1][4 * (i4 & 1) + e] = (T)keep_or_zero(p, mask);
            dsf[i4 >> 1][4 * (i4 & 1) + e] = (T)(p * dropped_dp_minus_d(dp[i], a.keep_scale, mask, d4[e]));
          } else {
            pf[i4 >> 1][4 * (i4 & 1) + e] = (T)p;
            dsf[i4 >> 1][4 * (i4 & 1) + e] = (T)(p * dp[i]);
          }
        }
      }
      // ---- dV^T += dO^T P and dK^T += Q^T dS (contractions over the 32 queries), alternating
      {
        auto gtr = [&](int f) {   // f = DB cc + db
          const T* base = Gt + 16 * (f / DB) * D;
          return tr_frag<T8>(base + tro.off[f % DB][0], base + tro.off[f % DB][1]);
        };
        auto qtr = [&](int f) {
          const T* base = Qt + 16 * (f / DB) * D;
          return tr_frag<T8>(base + tro.off[f % DB][0], base + tro.off[f % DB][1]);
        };
        constexpr int PF2 = 2;
        T8 rg[PF2], rq[PF2];
#pragma unroll
        for (int f = 0; f < PF2; ++f) { rg[f] = gtr(f); rq[f] = qtr(f); }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int f = 0; f < 2 * DB; ++f) {
          const T8 cg = rg[f % PF2], cq = rq[f % PF2];
          dv[f % DB] = mfma32(cg, pf[f / DB], dv[f % DB]);
          dk[f % DB] = mfma32(cq, dsf[f / DB], dk[f % DB]);
          if (f + PF2 < 2 * DB) { rg[f % PF2] = gtr(f + PF2); rq[f % PF2] = qtr(f + PF2); }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    wait_async_copies();
    __syncthreads();
  };
  for (int t = first; t < limit; t += 2) {
    tile_step(t, std::integral_constant<int, 0>());
    if (t + 1 < limit) tile_step(t + 1, std::integral_constant<int, 1>());
  }
  {
    // 4 wavefronts x 32 rows x 128 = 32 KB per gradient: the V block, then the four tile buffers
    T* stage_v = Vb + wave * 32 * D;
    store_rows_coalesced<T, D>(stage_v, (T*)a.dV + head_off + (int64_t)kw0 * a.sn, a.sn, dv,
                               DROPOUT ? a.keep_scale : 1.f, a.N - kw0);
    __builtin_amdgcn_wave_barrier();
    store_rows_coalesced<T, D>(stage_v, (T*)a.dK + head_off + (int64_t)kw0 * a.sn, a.sn, dk, a.tau, a.N - kw0);
  }
}

template <typename T>
int launch_t(const KArgs& a_in, bool causal, bool dropout, hipStream_t s) {
  KArgs a = a_in;
  {
    const int64_t tile_bytes = 2 * (int64_t)a.N * D * (int64_t)sizeof(T);   // Q and dO of one head
    const int64_t fit = ((int64_t)8 << 20) / tile_bytes;
    a.group = (int)(fit < 1 ? 1 : (fit > 8 ? 8 : fit));
  }
  const dim3 grid(kXcds * a.chunk), block(NT);
  if (causal && dropout) hipLaunchKernelGGL((dkv_fr128_kernel<T, true, true>), grid, block, 0, s, a);
  else if (causal) hipLaunchKernelGGL((dkv_fr128_kernel<T, true, false>), grid, block, 0, s, a);
  else if (dropout) hipLaunchKernelGGL((dkv_fr128_kernel<T, false, true>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((dkv_fr128_kernel<T, false, false>), grid, block, 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace

int launch_dkv_fr128(const KArgs& a, int dtype, bool causal, bool dropout, hipStream_t s) {
  return dtype == 0 ? launch_t<_Float16>(a, causal, dropout, s) : launch_t<__bf16>(a, causal, dropout, s);
}

}  // namespace attn
