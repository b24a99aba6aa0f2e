// Tile helpers shared by the backward kernels: staging of [64][D] tiles into swizzled LDS,
// transposing-read offsets, fragment reads and the transposed accumulator store.
#pragma once
#include "attn_common.h"

namespace attn {

// Stages a [64][D] tile: global -> registers -> swizzled LDS.
template <typename T, int D, int NT> struct TileStage {
  typedef typename Vec<T>::x8 T8;
  static constexpr int TILE = 64;
  static constexpr int CPR = D / 8, RPP = NT / CPR, NP = TILE / RPP;
  T8 reg[NP];
  __device__ __forceinline__ void load(const T* g, int64_t sn, int row0) {
    const int lrow = threadIdx.x / CPR, lchunk = threadIdx.x % CPR;
#pragma unroll
    for (int p = 0; p < NP; ++p)
      reg[p] = *(const T8*)(g + (int64_t)(row0 + p * RPP + lrow) * sn + 8 * lchunk);
  }
  __device__ __forceinline__ void store(T* lds) const {
    const int lrow = threadIdx.x / CPR, lchunk = threadIdx.x % CPR;
#pragma unroll
    for (int p = 0; p < NP; ++p) *(T8*)(lds + lds_off<D>(p * RPP + lrow, lchunk)) = reg[p];
  }
};

// Per-lane LDS offsets for the transposing read of a swizzled tile (see attn_fwd.hip for the
// access pattern): off[db][hi] addresses rows 4g + t (+8 if hi) of a 16-row chunk, d block db.
template <int D> struct TrOffsets {
  int off[D / 32][2];
  __device__ __forceinline__ void init() {
    const int lane = threadIdx.x & 63;
    const int g = lane >> 5, i16 = lane & 15, q16 = lane >> 4;
#pragma unroll
    for (int hi = 0; hi < 2; ++hi) {
      const int row = 4 * g + (i16 >> 2) + 8 * hi;
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const int chunk = 4 * db + 2 * (q16 & 1) + ((i16 & 3) >> 1);
        off[db][hi] = lds_off<D>(row, chunk) + 4 * (i16 & 1);
      }
    }
  }
};

template <typename T8>
__device__ __forceinline__ T8 tr_frag(const void* lds_lo, const void* lds_hi) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds_lo));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lds_hi));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(T8, both);
}

// Writes a transposed accumulator (rows = d, column = this lane's token) as a token row.
template <typename T, int D>
__device__ __forceinline__ void store_rows(T* dst_row, const f32x16 (&acc)[D / 32], float scale, int g) {
  typedef typename Vec<T>::x4 T4;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      T4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (T)(acc[db][4 * i4 + e] * scale);
      *(T4*)(dst_row + 32 * db + 8 * i4 + 4 * g) = v;
    }
}


}  // namespace attn
