// Internal declarations shared by the gfx950 attention kernels and the C-ABI front end.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attn {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Problem description handed to every kernel (plain data, passed by value).
struct KArgs {
  const void* Q; const void* K; const void* V;
  void* O;                 // fwd: out; bwd: in
  float* LSE;              // fwd: out; bwd: in        [B,H,N]
  const void* dO;          // bwd in
  void* dQ; void* dK; void* dV;   // bwd out
  float* Dvec;             // bwd scratch: -D_i = -rowsum(dO_i o O_i)   [B,H,Nr], 0 for rows >= N
  float* L2vec;            // bwd scratch: L_i * log2(e), +inf where L_i = -inf and for rows >= N   [B,H,Nr]
  int* colcnt;             // block-sparse bwd scratch: kept blocks per mask column   [B*H, T]
  int* seglist;            // block-sparse bwd scratch: [0] = number of entries, [1] = kept blocks in total,
                           // [2] = heavy threshold, from [kSegHeader]: entries (column * kMaxSegs + segment)
  float* dKacc;            // block-sparse bwd scratch: fp32 dK / dV of the columns that are
  float* dVacc;            //   split over several workgroups                         [B,H,N,d]
  int causal;              // causal flag for the kernels that are not specialised on it
  const uint8_t* mask;     // block mask [T,T] (per head if mask_sh != 0) or nullptr
  int64_t mask_sh;
  const int* klen;         // key-padding lengths [B] or nullptr
  int64_t sb, sh, sn;      // element strides of the [B,H,N,d] tensors
  int B, H, N, T;          // T = ceil(N / 128)
  int Nr;                  // 128 T: rows per head of the backward scratch vectors
  int dvalid;              // head dimension of the tensors: 16 with the D = 32 kernels (columns 16..31 are zeros on chip), else D
  float tau;               // softmax scale
  float scale_log2;        // tau * log2(e)
  float keep_scale;        // 1 / (1 - p_drop)
  uint32_t drop_thr;       // T: keep iff 8-bit philox field >= T (1..255 when dropout is on)
  uint32_t seed_lo, seed_hi, offset_lo;
  int o_fp32;
  int n_items;             // work items (B*H*tiles)
  int chunk;               // items per XCD = ceil(n_items / 8)
  int group;               // causal dQ: heads whose row blocks are dealt out together, heaviest first
};

enum { kXcds = 8, kMaskBlock = 128 };
// Block-sparse dK/dV: a mask column is "heavy" when it keeps more than kHeavyBlocks blocks AND
// more than half of a compute unit's fair share of all kept blocks (so a mask whose columns are
// all long, e.g. a dense one, is not split at all).  Heavy columns are cut into segments of about
// kSegBlocks blocks (at most kMaxSegs), one workgroup each, summed with fp32 atomics.
enum { kHeavyBlocks = 24, kSegBlocks = 12, kMaxSegs = 32, kSegHeader = 8, kComputeUnits = 256 };

// Kernel-choice overrides (attn_debug_set_variant; initial values from the environment, read once
// when first needed).  fwd: 0 = by measurement, 1 = free-running kernel, 2 = two-group kernel;
// dkv: 0 = by measurement, 1 = role-split kernel wherever it exists, 2 = the 64-key kernel is not used,
// 3 = the 64-key kernel wherever it exists.
int fwd_variant();
int dkv_variant();

// Which kernel serves a problem (the launchers use these; attn_debug_kernel_choice reports them).
enum { kFwdFreeRunning = 0, kFwdTwoGroup = 1 };
enum { kDkvRoleSplit = 0, kDkvOneWave = 1, kDkvOneWave128 = 2, kDkvOneWave64 = 3 };
int choose_fwd(const KArgs& a, int d, bool causal, bool dropout, bool sparse);
int choose_dkv(const KArgs& a, int d, bool causal, bool dropout, bool sparse);

// Launchers (defined in the .hip files).  dtype: 0 fp16, 1 bf16.  Return hipError_t as int.
int launch_fwd(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, hipStream_t s);
// ev: nullptr, or four events: two recorded before the first launch, one after the dQ kernel, one after dK/dV.
int launch_bwd(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, hipStream_t s,
               hipEvent_t* ev);
int launch_dropout_mask(const KArgs& a, uint8_t* keep, hipStream_t s);
// dK/dV kernel with the S->P->dV and dP->dS->dK halves on two wavefronts of a SIMD (attn_bwd_dkv.hip)
int launch_dkv_rs(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, hipStream_t s);
// dense dK/dV kernel for d <= 64: one wavefront does all four tile products (attn_bwd_dkv_fr.hip)
int launch_dkv_fr(const KArgs& a, int dtype, int d, bool causal, bool dropout, bool sparse, int extra_groups,
                  hipStream_t s);
// the same at d = 128 for dense problems (attn_bwd_dkv_fr128.hip)
int launch_dkv_fr128(const KArgs& a, int dtype, bool causal, bool dropout, hipStream_t s);
// the same with 64 keys per wavefront and the accumulators in the accumulation registers (attn_bwd_dkv_w64.hip)
int launch_dkv_w64(const KArgs& a, int dtype, bool causal, hipStream_t s);
// dense forward with two wavefront groups in ping-pong (attn_fwd_pp.hip); sets its own work items
int launch_fwd_pp(const KArgs& a, int dtype, int d, bool causal, bool dropout, hipStream_t s);
// MFMA-only kernel for measuring the sustained matrix rate (attn_probe.hip); *flops = FLOPs launched
int launch_mfma_rate(int dtype, int iters, int operand_sets, float* sink, hipStream_t s, double* flops);

#if defined(__HIPCC__)
// ---------------------------------------------------------------- device helpers
template <typename T> struct Vec;
template <> struct Vec<_Float16> { typedef f16x8 x8; typedef f16x4 x4; };
template <> struct Vec<__bf16> { typedef bf16x8 x8; typedef bf16x4 x4; };

__device__ __forceinline__ f32x16 mfma32(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// acc + the sum of the eight 16-bit values of v, each widened exactly (four two-element dot products
// with ones: half an instruction per element)
__device__ __forceinline__ float sum8(bf16x8 v, float acc) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const bf16x2 one = {(__bf16)1.f, (__bf16)1.f};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const bf16x2 pr = {v[2 * k], v[2 * k + 1]};
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, one, acc, false);
  }
  return acc;
}
__device__ __forceinline__ float sum8(f16x8 v, float acc) {
  typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
  const f16x2 one = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const f16x2 pr = {v[2 * k], v[2 * k + 1]};
    acc = __builtin_amdgcn_fdot2(pr, one, acc, false);
  }
  return acc;
}

// Online softmax, when the reference of a row is moved: only when the maximum of a new tile
// exceeds the reference by more than this (base-2 exponent units; the first tile always does).
// Probabilities then reach 2^kLazyRescale at most, exactly representable scalings in both 16-bit
// types.  What makes a lagging reference as accurate as the exact running maximum is that O is
// normalised by the sum of the ROUNDED 16-bit probabilities, the very weights the second product
// used: O stays a convex combination of V rows whatever the reference is.
constexpr float kLazyRescale = 8.0f;

// Philox-4x32-10 (Salmon et al., SC'11): counter (c0..c3), key (k0,k1) -> 4 words.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    // the two three-way exclusive ors of a round, one instruction each
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
    c1 = (uint32_t)p1; c3 = (uint32_t)p0; c0 = n0; c2 = n2;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  u32x4 r = {c0, c1, c2, c3};
  return r;
}

// Dropout draw (see the contract in include/attn.h): one Philox call decides the sixteen keys
// 16 g16 .. 16 g16 + 15 of query row i; key 16 g16 + f is KEPT iff byte f % 4 of word f / 4 of the
// result is >= T.
__device__ __forceinline__ u32x4 philox_draw16(uint32_t g16, uint32_t i, uint32_t bh, uint32_t offset_lo,
                                               uint32_t seed_lo, uint32_t seed_hi) {
  return philox4x32_10(g16, i, bh, offset_lo, seed_lo, seed_hi);
}
// The threshold test of the four 8-bit fields of a word, two at a time: field >= T iff
// field + (256 - T) carries out of its eight bits, and in 16-bit lanes the carry of fields 0 / 2
// (even) or 1 / 3 (odd) lands in bit 8 / bit 24, alone in its byte.  carry2 = (256 - T) * 0x00010001.
struct Keep4 { uint32_t even, odd; };
__device__ __forceinline__ uint32_t dropout_carry2(uint32_t thr8) { return (256u - thr8) * 0x00010001u; }
__device__ __forceinline__ Keep4 keep4(uint32_t w, uint32_t carry2) {
  Keep4 k;
  k.even = (w & 0x00FF00FFu) + carry2;
  k.odd = __builtin_amdgcn_perm(0u, w, 0x0C030C01u) + carry2;   // (w >> 8) & 0x00FF00FF in one instruction
  return k;
}
__device__ __forceinline__ float keep_or_zero(float x, uint32_t mask) {
  return __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x) & mask);
}
// true when the 8-bit draw in byte e (a constant, 0..3) of the word is below the threshold: the element is dropped
__device__ __forceinline__ bool dropped(uint32_t w, int e, uint32_t thr8) { return ((w >> (8 * e)) & 0xFFu) < thr8; }
// Dropout on a fragment of eight packed 16-bit values (four registers; element t in half t % 2 of
// register t / 2): element t is zeroed when its 8-bit draw, byte t % 4 of word t / 4 (w_lo, w_hi), is
// below the threshold.  Sub-dword operand addressing does the field extract, the compare and the
// half-register write in two instructions per element, on the values already rounded to 16 bits.
// thr8 and zero are registers holding T and 0.  Written out by hand because the compiler has no
// half-register select; a register written through a sub-dword destination must not be read by the
// next instruction (one wait state), which the order below keeps (the two halves of a register are
// eight instructions apart), and the closing s_nop separates the last writes from whatever follows.
template <typename T8>
__device__ __forceinline__ void drop_fragment8(T8& frag, uint32_t w_lo, uint32_t w_hi, uint32_t thr8, uint32_t zero) {
  const u32x4 p = __builtin_bit_cast(u32x4, frag);
  uint32_t p0 = p[0], p1 = p[1], p2 = p[2], p3 = p[3];
#define ATTN_DROP_HALF(REG, WORD, BYTE, HALF)                                                       \
  "v_cmp_lt_u32_sdwa vcc, " WORD ", %6 src0_sel:BYTE_" #BYTE " src1_sel:DWORD\n\t"                   \
  "v_cndmask_b32_sdwa " REG ", " REG ", %7, vcc dst_sel:WORD_" #HALF                                \
  " dst_unused:UNUSED_PRESERVE src0_sel:WORD_" #HALF " src1_sel:DWORD\n\t"
  asm volatile(
      ATTN_DROP_HALF("%0", "%4", 0, 0) ATTN_DROP_HALF("%1", "%4", 2, 0)
      ATTN_DROP_HALF("%2", "%5", 0, 0) ATTN_DROP_HALF("%3", "%5", 2, 0)
      ATTN_DROP_HALF("%0", "%4", 1, 1) ATTN_DROP_HALF("%1", "%4", 3, 1)
      ATTN_DROP_HALF("%2", "%5", 1, 1) ATTN_DROP_HALF("%3", "%5", 3, 1)
      "s_nop 1"
      : "+v"(p0), "+v"(p1), "+v"(p2), "+v"(p3)
      : "v"(w_lo), "v"(w_hi), "v"(thr8), "v"(zero)
      : "vcc");
#undef ATTN_DROP_HALF
  const u32x4 q = {p0, p1, p2, p3};
  frag = __builtin_bit_cast(T8, q);
}
// the sixteen keep bits of a call: bit f set iff key 16 g16 + f is kept
__device__ __forceinline__ uint32_t keep_bits16(const u32x4& w, uint32_t carry2) {
  uint32_t bits = 0;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const Keep4 k = keep4(w[t], carry2);
    // the four flag bytes (0 or 1) of the word side by side: fields 0, 1, 2, 3
    const uint32_t flags = __builtin_amdgcn_perm(k.odd, k.even, 0x07030501u);
    const uint32_t nib = (flags | (flags >> 7) | (flags >> 14) | (flags >> 21)) & 0xFu;
    bits |= nib << (4 * t);
  }
  return bits;
}

// value of the lane 32 positions away (wave64)
__device__ __forceinline__ float xchg32(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0] = {lo half, lo half}, r[1] = {hi half, hi half}
  const uint32_t other = (threadIdx.x & 32) ? r[0] : r[1];
  return __builtin_bit_cast(float, other);
}

// Dropout words of a 64-key tile in the "lane = query" layout (forward, dQ).  A call decides 16
// consecutive keys of the lane's query: the four calls of a tile are key block kb = 0, 1 times half
// 0, 1 of its 32 keys, and word w of a call holds keys 4 w .. 4 w + 3 of that half, which belong to
// lane g' = w % 2 of the query's two lanes, row group i4 = 2 half + w / 2.  Lane g draws half g of
// both key blocks, and the pair exchanges the words that belong to the other lane (four swaps serve
// both directions).  Result: byte e of w[kb][i4] decides element (kb, i4, e) of THIS lane.
struct KeepLQ { uint32_t w[2][4]; };
__device__ __forceinline__ KeepLQ keep_tile_lane_query(int k0, int qi, int bh, int g, uint32_t offset_lo,
                                                       uint32_t seed_lo, uint32_t seed_hi) {
  KeepLQ k;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const u32x4 r = philox_draw16((uint32_t)(k0 >> 4) + 2 * kb + g, (uint32_t)qi, (uint32_t)bh, offset_lo, seed_lo, seed_hi);
    // v_permlane32_swap(x, y): the upper 32 lanes' x and the lower 32 lanes' y change places
    auto s01 = __builtin_amdgcn_permlane32_swap(r[0], r[1], false, false);
    auto s23 = __builtin_amdgcn_permlane32_swap(r[2], r[3], false, false);
    // lane 0 now holds (own word 0, lane 1's word 0, own word 2, lane 1's word 2) = row groups 0, 2, 1, 3;
    // lane 1 holds (lane 0's word 1, own word 1, lane 0's word 3, own word 3) = row groups 0, 2, 1, 3
    k.w[kb][0] = s01[0]; k.w[kb][2] = s01[1]; k.w[kb][1] = s23[0]; k.w[kb][3] = s23[1];
  }
  return k;
}

// Dropout in the "lane = key" layout (dK / dV kernels): a wavefront holds 32 keys (lane r, twice:
// g = 0, 1) times 64 queries; lane (r, g) holds its key for the queries i0 + 32 qb + 8 i4 + 4 g + e.
// A call decides 16 consecutive keys of one query, i.e. the 16 lanes of one row of the wavefront
// (same g, same r / 16), which all need the draws of the same 32 queries.  Lane u = r % 16 of a row
// draws the two queries (qb = 0, 1; i4 = u / 4, e = u % 4) and packs their keep bits into one word,
// bit 16 qb + key.  Every lane then needs the words of all 16 lanes of its row: word 4 i4 + e,
// bit (r % 16) + 16 qb, is this lane's key for query (qb, i4, e).  Two ways to hand them round:
// keep_words_lane_key() (row broadcasts through the LDS crossbar, no memory involved, a row group
// of four words at a time) and keep_row_store() / keep_row_load*() (through an LDS slot).
__device__ __forceinline__ uint32_t draw_keep_lane_key(int i0, int kj, int r, int g, int bh, uint32_t offset_lo,
                                                       uint32_t seed_lo, uint32_t seed_hi, uint32_t thr8) {
  const int u = r & 15;
  const uint32_t carry2 = dropout_carry2(thr8);
  uint32_t mine = 0;
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const uint32_t qrow = (uint32_t)(i0 + 32 * qb + 8 * (u >> 2) + 4 * g + (u & 3));
    const u32x4 w = philox_draw16((uint32_t)kj >> 4, qrow, (uint32_t)bh, offset_lo, seed_lo, seed_hi);
    mine |= keep_bits16(w, carry2) << (16 * qb);
  }
  return mine;
}
struct KeepLK { uint32_t w[4][4]; };
template <int SRC> __device__ __forceinline__ uint32_t row16_broadcast(uint32_t x) {
  // ds_swizzle, bit mode within 32 lanes: source lane = (lane & 0x10) | SRC
  return (uint32_t)__builtin_amdgcn_ds_swizzle((int)x, 0x10 | (SRC << 5));
}
// The exchange through LDS: every lane stores its packed word into its wavefront's 64-word slot, and
// the four words of row group i4 of a lane's 16-lane row are one 16-byte read (all lanes of the row
// read the same address).  No barrier: one wavefront's LDS instructions execute in order.
struct KeepLK4 { uint32_t w[4]; };
__device__ __forceinline__ void keep_row_store(uint32_t* slot64, uint32_t mine) { slot64[threadIdx.x & 63] = mine; }
__device__ __forceinline__ KeepLK4 keep_row_load(const uint32_t* slot64, int i4) {
  const u32x4 v = *(const u32x4*)(slot64 + (threadIdx.x & 48) + 4 * i4);
  KeepLK4 k;
  k.w[0] = v[0]; k.w[1] = v[1]; k.w[2] = v[2]; k.w[3] = v[3];
  return k;
}
// all sixteen words of the lane's row (row groups i4 = 0..3), for kernels that hold them
__device__ __forceinline__ KeepLK keep_row_load_all(const uint32_t* slot64) {
  KeepLK k;
#pragma unroll
  for (int i4 = 0; i4 < 4; ++i4) {
    const u32x4 v = *(const u32x4*)(slot64 + (threadIdx.x & 48) + 4 * i4);
    k.w[i4][0] = v[0]; k.w[i4][1] = v[1]; k.w[i4][2] = v[2]; k.w[i4][3] = v[3];
  }
  return k;
}
// Z dP - D for one element: dP times keep_scale where the key was kept (mask all ones), times zero
// where it was dropped, plus -D, as one multiply-add with a masked factor
__device__ __forceinline__ float dropped_dp_minus_d(float dp, float keep_scale, uint32_t mask, float neg_d) {
  return __builtin_fmaf(dp, __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, keep_scale) & mask), neg_d);
}
// The row broadcasts: the four words of row group i4 (a constant after unrolling), fetched where
// they are used by kernels that cannot afford to hold all sixteen.
__device__ __forceinline__ KeepLK4 keep_words_lane_key(uint32_t mine, int i4) {
  KeepLK4 k;
  switch (i4) {
    case 0: k.w[0] = row16_broadcast<0>(mine); k.w[1] = row16_broadcast<1>(mine); k.w[2] = row16_broadcast<2>(mine); k.w[3] = row16_broadcast<3>(mine); break;
    case 1: k.w[0] = row16_broadcast<4>(mine); k.w[1] = row16_broadcast<5>(mine); k.w[2] = row16_broadcast<6>(mine); k.w[3] = row16_broadcast<7>(mine); break;
    case 2: k.w[0] = row16_broadcast<8>(mine); k.w[1] = row16_broadcast<9>(mine); k.w[2] = row16_broadcast<10>(mine); k.w[3] = row16_broadcast<11>(mine); break;
    default: k.w[0] = row16_broadcast<12>(mine); k.w[1] = row16_broadcast<13>(mine); k.w[2] = row16_broadcast<14>(mine); k.w[3] = row16_broadcast<15>(mine); break;
  }
  return k;
}
// all ones if this lane's key is kept for query (qb, i4, e); bit = (r % 16) + 16 qb
__device__ __forceinline__ uint32_t keep_mask_lane_key(uint32_t word, int bit) {
  return (uint32_t)__builtin_amdgcn_sbfe((int)word, bit, 1);
}

// Online softmax of one 64-key tile in the "lane = query" layout of the forward kernels (Algorithm 2
// of the paper's follow-up formulation of Algorithm 1's inner loop, base 2): s holds the raw logits
// S^T (two 32-key blocks; lane (r, g) has query row q0 + r and keys 32 kb + 8 (i / 4) + 4 g + i % 4)
// and is left holding the unnormalised probabilities; pf receives them rounded to T as the four
// 16-key B-operand fragments of O^T += V^T P^T, with dropout applied.  Masks keys beyond `last`
// on tiles that cross the causal diagonal or the end of the sequence, moves the running reference
// m_run (and rescales o, l_run, lr_run) only when a row of the wavefront outgrew it by more than
// kLazyRescale, and keeps two row sums per lane: l_run of the exact probabilities (for the saved
// statistic) and lr_run of the rounded ones (the normaliser of O), both before dropout.
template <typename T, int DB, bool CAUSAL, bool DROPOUT>
__device__ __forceinline__ void softmax_tile_lane_query(const KArgs& a, f32x16 (&s)[2], f32x16 (&o)[DB],
                                                        typename Vec<T>::x8 (&pf)[4], float& m_run, float& l_run,
                                                        float& lr_run, float c, int k0, int q0, int qi, int len, int g,
                                                        int bh) {
  if ((CAUSAL && k0 + 63 > q0) || k0 + 64 > len) {   // diagonal tiles, and the padded last tile
    const int last = CAUSAL ? min(qi, len - 1) : len - 1;   // last visible key of this row
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = k0 + 32 * kb + 8 * (i >> 2) + 4 * g + (i & 3);
        if (key > last) s[kb][i] = -INFINITY;
      }
  }
  float mx = s[0][0];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
  mx = fmaxf(mx, xchg32(mx)) * c;
  if (__builtin_amdgcn_ballot_w64(mx > m_run + kLazyRescale) != 0) {   // wavefront-uniform: rare after the first tiles
    const float m_new = fmaxf(m_run, mx);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_safe);
    m_run = m_new;
    l_run *= alpha;
    lr_run *= alpha;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
  }
  const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
  float psum = 0.f;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i], c, -m_use));
      s[kb][i] = p;
      psum += p;
    }
  l_run += psum;
  // P^T fragments: 16-key chunk cc = 2 kb + half
#pragma unroll
  for (int cc = 0; cc < 4; ++cc)
#pragma unroll
    for (int t = 0; t < 8; ++t) pf[cc][t] = (T)s[cc >> 1][8 * (cc & 1) + t];
  float part[4];
#pragma unroll
  for (int cc = 0; cc < 4; ++cc) part[cc] = sum8(pf[cc], 0.f);
  lr_run += (part[0] + part[1]) + (part[2] + part[3]);
  if constexpr (DROPOUT) {   // element t of chunk cc has field t % 4 of word 2 (cc & 1) + t / 4 of its block
    const KeepLQ kq = keep_tile_lane_query(k0, qi, bh, g, a.offset_lo, a.seed_lo, a.seed_hi);
#pragma unroll
    for (int cc = 0; cc < 4; ++cc)
      drop_fragment8(pf[cc], kq.w[cc >> 1][2 * (cc & 1)], kq.w[cc >> 1][2 * (cc & 1) + 1], a.drop_thr, 0u);
  }
}

// Work-item index for this workgroup: consecutive items share an XCD (workgroups are
// dealt round-robin to the 8 XCDs, each with its own L2).  Returns -1 for padding groups.
__device__ __forceinline__ int xcd_item(int n_items, int chunk, int id = (int)blockIdx.x) {
  const int item = (id % kXcds) * chunk + id / kXcds;
  return item < n_items && (id / kXcds) < chunk ? item : -1;
}
// XOR swizzle of the 16-byte chunk index inside an unpadded [rows][D] LDS tile.  It makes both
// access patterns used on the tiles conflict-free on a 64-bank LDS: 16 consecutive rows at one
// chunk (row-wise 16-byte operand reads) and 4 consecutive rows x 64 bytes (transposing reads).
template <int D> __device__ __forceinline__ int swz_bits(int row) {
  if constexpr (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  else if constexpr (D == 64) return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
  else return (row >> 2) & 3;   // D == 32: four chunks per row, four rows per 256 bytes
}
template <int D> __device__ __forceinline__ int lds_off(int row, int chunk) {
  return row * D + ((chunk ^ swz_bits<D>(row)) << 3);
}

// Iterates, in increasing order, over the 64-wide tiles a workgroup must visit.
// Dense: first .. limit-1 (in tiles).  Sparse: the two 64-wide halves of every 128-block b in
// [first, limit) with mask[b * stride] != 0.  All state is wavefront-uniform.
// Sparse only: the first `skip` kept blocks are passed over and at most `take` are delivered.
template <bool SPARSE> struct TileIter {
  const uint8_t* mask;
  int64_t stride;
  int limit, pos, base, half, skip, take;
  uint64_t bits;
  __device__ __forceinline__ void init(const uint8_t* m, int64_t st, int first, int lim,
                                       int skip_blocks = 0, int take_blocks = 0x7fffffff) {
    mask = m; stride = st; limit = lim; pos = first; bits = 0; base = 0; half = -1;
    skip = skip_blocks; take = take_blocks;
  }
  __device__ __forceinline__ int next() {
    if constexpr (!SPARSE) {
      return pos < limit ? pos++ : -1;
    } else {
      if (half >= 0) { const int t = half; half = -1; return t; }
      if (take <= 0) return -1;
      while (true) {
        while (bits == 0) {
          if (pos >= limit) return -1;
          const int blk = pos + (int)(threadIdx.x & 63);
          const bool on = blk < limit && mask[(int64_t)blk * stride] != 0;
          bits = __ballot(on);
          base = pos;
          pos += 64;
          const int n = __builtin_popcountll(bits);
          if (n <= skip) { skip -= n; bits = 0; }   // the whole chunk is before this segment
        }
        const int b = __builtin_ctzll(bits);
        bits &= bits - 1;
        if (skip > 0) { --skip; continue; }
        --take;
        half = 2 * (base + b) + 1;
        return 2 * (base + b);
      }
    }
  }
};
#endif  // __HIPCC__

}  // namespace attn
