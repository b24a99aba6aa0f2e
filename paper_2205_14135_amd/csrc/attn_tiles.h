// Tile helpers shared by the tile kernels: asynchronous copies of [64][D] tiles into swizzled
// LDS, transposing-read offsets, fragment reads and the transposed accumulator store.
#pragma once
#include "attn_common.h"

namespace attn {

// Lane index read by an instruction the compiler will not move: address arithmetic of a rarely
// taken path that starts from it stays inside that path instead of being hoisted out of the tile
// loop, where it would occupy registers for the whole kernel.
__device__ __forceinline__ int lane_id_here() {
  int lane = 0;
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
#endif
  return lane;
}

// Asynchronous copy of a [64][D] tile from global memory straight into swizzled LDS (no register
// staging, no LDS store instructions): each global_load_lds_dwordx4 moves 64 lanes x 16 bytes to
// 1 KB of consecutive LDS, so lane l of copy q lands on row q*(64/CPR) + l/CPR, physical chunk
// l%CPR, and therefore fetches the logical chunk (l%CPR) ^ swizzle(row) of that row (TileAsync
// below).  The copy is issued as a raw instruction that the compiler does not track: with the
// builtin form of it the compiler makes every later LDS read that might alias the destination
// wait for the copy, and with run-time buffer indices every read might; a copy issued this way
// stays in flight until the caller waits for it with wait_async_copies() (which it must do,
// followed by a workgroup barrier, before any wavefront reads the tile).  lds_byte_addr must be
// wavefront-uniform.  M0 carries the LDS base of the copy; the statements declare it clobbered, so
// the compiler keeps nothing of its own in it across a copy.
__device__ __forceinline__ void async_copy_b128(const void* gptr_lane, uint32_t lds_byte_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :: "s"(lds_byte_addr), "v"(gptr_lane) : "memory", "m0");
#else
  (void)gptr_lane; (void)lds_byte_addr;
#endif
}
// Same with the address split into a wavefront-uniform base (scalar registers) and a per-lane
// byte offset: no vector ALU work when only the base changes from tile to tile.
__device__ __forceinline__ void async_copy_b128(const void* gbase_uniform, uint32_t byte_off_lane, uint32_t lds_byte_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  // the base must sit in scalar registers whatever the compiler's divergence analysis thinks of it
  const uint64_t bits = (uint64_t)(uintptr_t)gbase_uniform;
  // (readfirstlane returns a signed int: widen through uint32_t, or bit 31 of the low word smears
  // over the high word)
  const uint64_t base = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)bits) |
                        ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(bits >> 32)) << 32);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_byte_addr), "v"(byte_off_lane), "s"(base) : "memory", "m0");
#else
  (void)gbase_uniform; (void)byte_off_lane; (void)lds_byte_addr;
#endif
}
__device__ __forceinline__ void async_copy_b32(const void* gptr_lane, uint32_t lds_byte_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
               :: "s"(lds_byte_addr), "v"(gptr_lane) : "memory", "m0");
#else
  (void)gptr_lane; (void)lds_byte_addr;
#endif
}
// vmcnt(0), as an instruction the compiler sees: it then also knows that its own earlier loads
// have completed and places no second wait for them where copies are in flight.
__device__ __forceinline__ void wait_async_copies() {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  asm volatile("" ::: "memory");
#endif
}
// Waits until at most N of this wavefront's vector-memory operations are outstanding (they
// complete in order, so the N most recent copies may still be in flight).
template <int N> __device__ __forceinline__ void wait_async_copies_but() {
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x0F70 | ((N >> 4) << 14));
  asm volatile("" ::: "memory");
#endif
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

// The tile copy: NW wavefronts (numbered 0..NW-1 by the caller) issue (D/8)/NW copy instructions each.
// ROWS: rows of the tile (64 unless a kernel streams smaller tiles).
// Head dimension 16 runs on the D = 32 kernels: the tensors' rows hold d_valid = 16 elements, the
// lanes whose chunk lies beyond them copy nothing, and the kernel clears the tile buffers once
// (zero_tiles below), so that columns 16..31 read as zeros.
template <typename T, int D, int NW, int ROWS = 64> struct TileAsync {
  static constexpr int CPR = D / 8, RPC = 64 / CPR, NCOPY = ROWS / RPC, PER_WAVE = NCOPY / NW;
  static_assert(NCOPY % NW == 0, "copies must divide evenly over the wavefronts");
  uint32_t goff[PER_WAVE];   // byte offset of this lane's chunk inside a tile whose row 0 is at 0
  int wave;                  // (the host checks that 64 rows of the tensor span less than 2^31 bytes)
  uint32_t beyond;           // D = 32 only: bit p set if this lane's chunk of copy p is beyond d_valid
  __device__ __forceinline__ void init(int64_t sn, int wave_index, int d_valid = D) {
    const int lane = threadIdx.x & 63;
    wave = wave_index;
    beyond = 0;
#pragma unroll
    for (int p = 0; p < PER_WAVE; ++p) {
      const int row = (wave * PER_WAVE + p) * RPC + lane / CPR;
      const int chunk = (lane % CPR) ^ swz_bits<D>(row);
      goff[p] = (uint32_t)(((int64_t)row * sn + 8 * chunk) * (int64_t)sizeof(T));
      if (8 * chunk >= d_valid) beyond |= 1u << p;
    }
  }
  __device__ __forceinline__ bool skip(int p) const {
    if constexpr (D == 32) return (beyond >> p) & 1u;
    return false;
  }
  // g_row0 must be wavefront-uniform
  __device__ __forceinline__ void copy(const T* g_row0, const T* lds_tile) const {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_addr(lds_tile) + (wave * PER_WAVE) * 1024);
#pragma unroll
    for (int p = 0; p < PER_WAVE; ++p)
      if (!skip(p)) async_copy_b128(g_row0, goff[p], base + p * 1024);
  }
  // copy number p (0 .. PER_WAVE - 1) of this wavefront alone, for callers that spread a tile's copies out
  __device__ __forceinline__ void copy_one(const T* g_row0, const T* lds_tile, int p) const {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_addr(lds_tile) + (wave * PER_WAVE) * 1024);
    if (!skip(p)) async_copy_b128(g_row0, goff[p], base + p * 1024);
  }
  // The last tile of a tensor whose row count is not a multiple of 64: only rows_valid (>= 1) rows
  // exist; the LDS rows beyond them receive a copy of the last valid row (finite values that the
  // kernels mask), so that nothing outside the tensor is read.
  __device__ __forceinline__ void copy_tail(const T* g_row0, const T* lds_tile, int64_t sn, int rows_valid) const {
    const int lane_row = lane_id_here() / CPR;
    const uint32_t row_bytes = (uint32_t)sn * (uint32_t)sizeof(T);   // 64 rows span less than 2^31 bytes
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_addr(lds_tile) + (wave * PER_WAVE) * 1024);
#pragma unroll
    for (int p = 0; p < PER_WAVE; ++p) {
      const int excess = max((wave * PER_WAVE + p) * RPC + lane_row - (rows_valid - 1), 0);   // rows past the last one
      if (!skip(p)) async_copy_b128(g_row0, goff[p] - (uint32_t)excess * row_bytes, base + p * 1024);
    }
  }
  // tile whose first row is row0 of a tensor with n_rows rows (row0 < n_rows)
  __device__ __forceinline__ void copy_rows(const T* g, int64_t sn, int row0, int n_rows, const T* lds_tile) const {
    if (row0 + ROWS <= n_rows) copy(g + (int64_t)row0 * sn, lds_tile);
    else copy_tail(g + (int64_t)row0 * sn, lds_tile, sn, n_rows - row0);
  }
};

// Clears n_elems (a multiple of 8 per thread pass) elements of LDS with all threads of the
// workgroup; the caller synchronises before copies land in the buffer.
template <typename T>
__device__ __forceinline__ void zero_tiles(T* lds, int n_elems) {
  typedef typename Vec<T>::x8 T8;
  T8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (T)0.f;
  for (int i = 8 * (int)threadIdx.x; i < n_elems; i += 8 * (int)blockDim.x) *(T8*)(lds + i) = z;
}

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


// Same result as store_rows for the 32 tokens of a wavefront, but through a wavefront-private
// LDS area of 32 * D elements so that global memory sees whole 16-byte-per-lane row segments
// (a token row is written by D/8 consecutive lanes) instead of 8-byte pieces 2*D bytes apart.
// The area is unpadded; the 16-byte chunk index is XORed with the row to spread the banks.
// dst_row0 points at the row of the wavefront's first token; only the first rows_valid of the 32
// rows exist in the destination (fewer than 32 on the last block of a ragged tensor; may be <= 0).
template <typename T, int D>
__device__ __forceinline__ void store_rows_coalesced(T* stage, T* dst_row0, int64_t sn,
                                                     const f32x16 (&acc)[D / 32], float scale,
                                                     int rows_valid = 32, int cols_valid = D) {
  typedef typename Vec<T>::x4 T4;
  typedef typename Vec<T>::x8 T8;
  constexpr int CPR = D / 8;         // 16-byte chunks per row
  constexpr int RPP = 64 / CPR;      // rows per pass of the read-back
  const int lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      T4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = (T)(acc[db][4 * i4 + e] * scale);
      const int chunk = (4 * db + i4) ^ (r & (CPR - 1));
      *(T4*)(stage + r * D + 8 * chunk + 4 * g) = v;
    }
  __builtin_amdgcn_wave_barrier();   // same wavefront: LDS operations complete in program order
#pragma unroll
  for (int p = 0; p < 32 / RPP; ++p) {
    const int row = p * RPP + lane / CPR, ch = lane % CPR;
    const T8 v = *(const T8*)(stage + row * D + 8 * (ch ^ (row & (CPR - 1))));
    if (row < rows_valid && 8 * ch < cols_valid) *(T8*)(dst_row0 + (int64_t)row * sn + 8 * ch) = v;
  }
}

// The same accumulator tile added into an fp32 array (row stride D floats) with atomics, for
// partial results that several workgroups sum: staged in fp32 (32 x D floats per wavefront) so that
// one atomic instruction covers 64 consecutive floats of a row.  Atomics of device scope are
// carried out beyond the XCD's L2, one request per 64-byte line: straight from the accumulator
// layout (a lane holds four consecutive floats of its own row) an instruction touched 32 lines,
// this way four.
template <int D>
__device__ __forceinline__ void atomic_add_rows_coalesced(float* stage, float* dst_row0, const f32x16 (&acc)[D / 32],
                                                          float scale, int cols_valid = D) {
  constexpr int C4 = D / 4;   // 16-byte chunks per row
  const int lane = threadIdx.x & 63, r = lane & 31, g = lane >> 5;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = acc[db][4 * i4 + e] * scale;
      const int chunk = (8 * db + 2 * i4 + g) ^ (r & (C4 - 1));
      *(f32x4*)(stage + r * D + 4 * chunk) = v;
    }
  __builtin_amdgcn_wave_barrier();   // same wavefront: LDS operations complete in program order
#pragma unroll 4
  for (int p = 0; p < D / 2; ++p) {
    const int f = 64 * p + lane, row = f / D, col = f % D;
    const float v = stage[row * D + 4 * ((col >> 2) ^ (row & (C4 - 1))) + (col & 3)];
    if (col < cols_valid) unsafeAtomicAdd(dst_row0 + row * D + col, v);
  }
  __builtin_amdgcn_wave_barrier();
}

}  // namespace attn
