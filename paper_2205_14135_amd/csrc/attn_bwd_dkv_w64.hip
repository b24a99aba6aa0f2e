// dK / dV kernel for head dimension 128, dense problems without dropout, register-blocked: one
// wavefront owns 64 keys (two blocks of 32) and has a SIMD's whole register file to itself.
//
// Arithmetic: Algorithm 4 of the paper for one block of 256 keys, swept over 32-query tiles:
//     S = Q K^T, P = exp(S - L), dV += P^T dO, dP = dO V^T, dS = P o (dP - D), dK += tau dS^T Q.
// Why this shape: with 32 keys per wavefront every MFMA takes a fresh 1 KB operand fragment from
// LDS, which is as much as LDS delivers while the matrix pipe runs the instruction, so LDS and the
// matrix pipe each sit at about two thirds.  With 64 keys per wavefront every Q / dO fragment read
// from LDS feeds two MFMAs.  That needs dK^T and dV^T accumulators of 256 registers per lane: they
// live in the 256 accumulation registers (AGPRs), everything else in the 256 architectural ones,
// one wavefront per SIMD, four wavefronts (256 keys) per workgroup and compute unit.
//
// Register files.  The accumulation registers are addressed BY NAME in raw MFMA instructions
// (accumulator tile t = a[16 t : 16 t + 15]); no C++ variable ever holds an accumulator, so the
// register allocator has nothing to move, split or spill there.  S and dP are ordinary builtin
// MFMAs whose results the compiler keeps in architectural registers; that needs the file to be
// compiled with -mllvm -amdgpu-mfma-vgpr-form=1 (otherwise every builtin MFMA result of a kernel
// that may use 512 registers is placed in AGPRs, on top of the accumulators).  The build checks the
// generated code: no instruction outside the raw statements of this file may name an AGPR, and
// nothing may be spilled.
//
// With no second wavefront on the SIMD to overlap with, the vector arithmetic of a tile is issued
// between the MFMAs: a wavefront's own independent vector instructions issue while its MFMA
// occupies the matrix pipe.  The 64 MFMAs of a tile run as six streams
//     S (16) | dP (16) | dV, first 16 queries (8) | dK, first 16 queries (8) | dV, rest (8) | dK, rest (8)
// with one ring of operand fragments read ahead from LDS across the stream boundaries; the exp /
// convert work and the dS products are dealt out over the MFMA slots by the tables below, and
// scheduling fences keep the order the source states.
//
// Hazards of the raw MFMAs (the compiler does not see inside them): an accumulator tile is only
// ever read by the next MFMA on the same tile (hardware-interlocked) and, after the loop, by
// v_accvgpr_read behind explicit idle cycles; their A/B operands are architectural registers
// written by LDS loads and vector instructions that the compiler tracks as operands.
//
// Key-padding mask and ragged ends: lane = key in every product of this kernel, so a padded key
// only ever affects its own dK / dV rows; those rows are cleared (or not stored) at the end
// instead of masking S in the loop.  Padded queries have a row statistic of +inf, hence P = 0.
#include <type_traits>
#include <utility>

#include "attn_common.h"
#include "attn_tiles.h"

namespace attn {
namespace {

constexpr int NT = 256;
constexpr int QT = 32;     // queries per streamed tile
constexpr int D = 128;
constexpr int KB = 256;    // keys per workgroup

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>()), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>());
}

// The work that a wavefront issues between the MFMAs of a tile, per MFMA slot (up to three items
// per slot, 0 = none).  The S stream is slots 0..15, dP 16..31, then dV / dK of the first 16
// queries of the tile 32..39 / 40..47 and of the rest 48..55 / 56..63.
//   400 + k  copy piece k of tile t + 2 (k = 0, 1: Q; 2, 3: dO; 4: a row vector).  A copy
//            instruction holds the wavefront up for 10-20 clocks; one at a time hides in the shadow
//            of an MFMA, several in a row do not.
//   300 + i  -D of row group i into both dP accumulators
//   310 + h  row statistics of row groups 2 h, 2 h + 1 from LDS
//   100 + u  P unit u: one value exp(S - L) (v_exp_f32 occupies the vector ALU for 16 clocks, so
//            a slot takes one of them: 16 + 4 + 4 clocks fit under the 32 of the MFMA, two do
//            not), every second unit converts a pair to 16 bits.  u = 16 cc + 8 kb + 4 (i4 % 2) + e:
//            half cc of the queries, key block kb, row group i4 = 2 cc + .., value e.
//   200 + v  dS unit v: two products P o (dP - D) and their conversion, v = 8 cc + 4 kb + 2 (i4 % 2) + pair.
// Deadlines: P needs S complete (key block 0 finishes at slot 12, key block 1 at 15, results two
// slots later), dS needs dP complete (slot 31); a 16-bit operand written by vector instructions is
// read by a raw MFMA two slots later at the earliest (the compiler places no wait states in front of
// a raw instruction; a whole slot in between is far more than the hardware asks for): P units of
// half 0 by slot 30, of half 1 by 46, dS units of half 0 by 38, of half 1 by 54.
constexpr int kPlan[64][3] = {
    {400, 0, 0}, {300, 0, 0}, {401, 0, 0}, {301, 0, 0},
    {402, 0, 0}, {302, 0, 0}, {403, 0, 0}, {303, 0, 0},
    {404, 0, 0}, {310, 0, 0}, {0, 0, 0}, {0, 0, 0},
    {0, 0, 0}, {0, 0, 0}, {100, 0, 0}, {101, 0, 0},
    {102, 0, 0}, {103, 0, 0}, {104, 0, 0}, {105, 0, 0},
    {106, 0, 0}, {107, 0, 0}, {108, 0, 0}, {109, 0, 0},
    {110, 0, 0}, {111, 0, 0}, {112, 0, 0}, {113, 0, 0},
    {114, 0, 0}, {115, 311, 0}, {116, 0, 0}, {117, 0, 0},
    {118, 0, 0}, {200, 201, 119}, {202, 120, 0}, {203, 121, 0},
    {204, 122, 0}, {205, 123, 0}, {206, 207, 0}, {124, 0, 0},
    {125, 0, 0}, {126, 0, 0}, {127, 0, 0}, {128, 0, 0},
    {129, 0, 0}, {130, 0, 0}, {131, 0, 0}, {208, 0, 0},
    {209, 0, 0}, {210, 0, 0}, {211, 0, 0}, {212, 0, 0},
    {213, 0, 0}, {214, 0, 0}, {215, 0, 0}, {0, 0, 0},
    {0, 0, 0}, {0, 0, 0}, {0, 0, 0}, {0, 0, 0},
    {0, 0, 0}, {0, 0, 0}, {0, 0, 0}, {0, 0, 0},
};
constexpr int plan_slot(int item) {
  for (int s = 0; s < 64; ++s)
    for (int k = 0; k < 3; ++k)
      if (kPlan[s][k] == item) return 4 * s + k;   // slot and position: orders items of one slot too
  return -1;
}
constexpr bool plan_ok() {
  for (int u = 0; u < 32; ++u) {
    const int at = plan_slot(100 + u), cc = u >> 4, kb = (u >> 3) & 1;
    if (at < 0 || at / 4 < (kb ? 17 : 14) || at / 4 > (cc ? 46 : 30)) return false;
    if ((u & 1) && plan_slot(100 + u - 1) > at) return false;            // the pair is converted together
    if (at < plan_slot(310 + cc)) return false;                          // its row statistics are there
    if (cc == 0 && at > plan_slot(311)) return false;                    // and not yet replaced
  }
  for (int v = 0; v < 16; ++v) {
    const int at = plan_slot(200 + v), cc = v >> 3;
    if (at < 0 || at / 4 < 33 || at / 4 > (cc ? 54 : 38)) return false;
    const int u0 = 16 * cc + 8 * ((v >> 2) & 1) + 4 * ((v >> 1) & 1) + 2 * (v & 1);
    if (plan_slot(100 + u0) > at || plan_slot(100 + u0 + 1) > at) return false;
  }
  for (int i = 0; i < 4; ++i)
    if (plan_slot(300 + i) < 0 || plan_slot(300 + i) / 4 > 14) return false;
  for (int k = 0; k < 5; ++k)
    if (plan_slot(400 + k) < 0) return false;
  return true;
}
static_assert(plan_ok(), "slot plan violates a deadline");
// The S stream takes the Q fragments 0..4 for both key blocks in turn and the last three (the
// depth of the fragment ring) for key block 0 first, so that its logits are complete three slots
// earlier and the exp work can start there.
constexpr int slot_frag(int slot) { return slot >= 10 && slot < 16 ? 5 + (slot - 10) % 3 : slot >> 1; }
constexpr int slot_kb(int slot) { return slot >= 10 && slot < 16 ? (slot - 10) / 3 : slot & 1; }
constexpr int last_user(int n) { return n >= 5 && n < 8 ? 8 + n : 2 * n + 1; }   // slot of the second MFMA on fragment n

template <typename T> struct Raw;
template <> struct Raw<__bf16> {
  // a[16 TILE ..] += A B
  template <int TILE> static __device__ __forceinline__ void mfma_acc(bf16x8 a, bf16x8 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3]"
                 :: "v"(a), "v"(b), "n"(16 * TILE), "n"(16 * TILE + 15));
  }
};
template <> struct Raw<_Float16> {
  template <int TILE> static __device__ __forceinline__ void mfma_acc(f16x8 a, f16x8 b) {
    asm volatile("v_mfma_f32_32x32x16_f16 a[%2:%3], %0, %1, a[%2:%3]"
                 :: "v"(a), "v"(b), "n"(16 * TILE), "n"(16 * TILE + 15));
  }
};

// The value is computed by this point of the instruction stream and not later: the compiler may
// otherwise sink the vector instructions that produce an operand down to its first use, which for
// an operand of a raw MFMA would put them right in front of an instruction it does not protect.
template <typename V> __device__ __forceinline__ void pin_here(V& v) { asm volatile("" : "+v"(v)); }

#define ATTN_A8(n) "a" #n "0", "a" #n "1", "a" #n "2", "a" #n "3", "a" #n "4", "a" #n "5", "a" #n "6", "a" #n "7", "a" #n "8", "a" #n "9"
// Clears all 256 accumulation registers.  The clobber list is what tells the compiler that this
// kernel uses them at all (the register counts of the kernel descriptor come from it).
__device__ __forceinline__ void acc_clear_all() {
#define ATTN_Z4(b) "v_accvgpr_write_b32 a[" #b "+0], 0\n\tv_accvgpr_write_b32 a[" #b "+1], 0\n\tv_accvgpr_write_b32 a[" #b "+2], 0\n\tv_accvgpr_write_b32 a[" #b "+3], 0\n\t"
#define ATTN_Z16(b) ATTN_Z4(b) ATTN_Z4(b+4) ATTN_Z4(b+8) ATTN_Z4(b+12)
#define ATTN_Z64(b) ATTN_Z16(b) ATTN_Z16(b+16) ATTN_Z16(b+32) ATTN_Z16(b+48)
  asm volatile(ATTN_Z64(0) ATTN_Z64(64) ATTN_Z64(128) ATTN_Z64(192)
               ::: "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9",
                   ATTN_A8(1), ATTN_A8(2), ATTN_A8(3), ATTN_A8(4), ATTN_A8(5), ATTN_A8(6), ATTN_A8(7), ATTN_A8(8), ATTN_A8(9),
                   ATTN_A8(10), ATTN_A8(11), ATTN_A8(12), ATTN_A8(13), ATTN_A8(14), ATTN_A8(15), ATTN_A8(16), ATTN_A8(17),
                   ATTN_A8(18), ATTN_A8(19), ATTN_A8(20), ATTN_A8(21), ATTN_A8(22), ATTN_A8(23), ATTN_A8(24),
                   "a250", "a251", "a252", "a253", "a254", "a255");
#undef ATTN_Z64
#undef ATTN_Z16
#undef ATTN_Z4
}
#undef ATTN_A8

// One accumulator tile out of the accumulation registers (after the MFMAs have drained).
template <int TILE> __device__ __forceinline__ f32x16 acc_read() {
  f32x16 v;
#define ATTN_RD(i) asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v[i]) : "n"(16 * TILE + i));
  ATTN_RD(0) ATTN_RD(1) ATTN_RD(2) ATTN_RD(3) ATTN_RD(4) ATTN_RD(5) ATTN_RD(6) ATTN_RD(7)
  ATTN_RD(8) ATTN_RD(9) ATTN_RD(10) ATTN_RD(11) ATTN_RD(12) ATTN_RD(13) ATTN_RD(14) ATTN_RD(15)
#undef ATTN_RD
  return v;
}

// Accumulator tiles: dV^T of key block kb, d block db = tile 4 kb + db; dK^T = tile 8 + 4 kb + db.
template <typename T, bool CAUSAL>
__global__ __launch_bounds__(NT, 1) void dkv_w64_kernel(const KArgs a) {
  typedef typename Vec<T>::x8 T8;
  typedef Raw<T> M;
  constexpr int KK = D / 16, DB = D / 32;
  // One LDS block, so that every address is a per-lane register plus an immediate: the row
  // vectors first, then the Q tiles, the dO tiles (three buffers each) and the V rows of this key block.
  constexpr int NBUF = 3;
  constexpr int kVecBytes = 2 * NBUF * 64 * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[kVecBytes + (2 * NBUF * QT * D + KB * D) * sizeof(T)];
  float* const Ls0 = (float*)smem;                 // base-2 row statistic: Ls0 + 64 buf (first QT entries used:
  float* const Ds0 = Ls0 + NBUF * 64;              // -D_i:                 Ds0 + 64 buf  a copy moves 64 floats)
  T* const Qs0 = (T*)(smem + kVecBytes);           // Q tiles:  Qs0 + buf QT D
  T* const Gs0 = Qs0 + NBUF * QT * D;              // dO tiles: Gs0 + buf QT D
  T* const Vb = Qs0 + 2 * NBUF * QT * D;           // V rows of this key block

  const int n_kt = (a.N + KB - 1) / KB;   // the last key block may be ragged
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

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // in a scalar register: branches on it are scalar
  const int r = lane & 31, g = lane >> 5;
  const int kw0 = kt * KB + wave * 64;   // this wavefront's keys: kw0 + 32 kb + r, kb = 0, 1

  // loop-invariant B operands: the K fragments of this lane's two keys (rows beyond a ragged end
  // repeat the last one; they are never stored).  The V rows of the key block stay in LDS.
  T8 kf[2][KK];
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const int64_t row_off = head_off + (int64_t)min(kw0 + 32 * kb + r, a.N - 1) * a.sn;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kb][kk] = *(const T8*)((const T*)a.K + row_off + 16 * kk + 8 * g);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): before any asynchronous copy is in flight
  acc_clear_all();

  const int len = __builtin_amdgcn_readfirstlane(a.klen ? min(max(a.klen[b], 0), a.N) : a.N);
  const int first = CAUSAL ? kt * (KB / QT) : 0;   // causal: the tiles above the diagonal see none of these keys
  const int limit = kt * KB >= len ? 0 : (len + QT - 1) / QT;   // query tiles (rows >= len have P = 0)

  TrOffsets<D> tro;
  tro.init();
  TileAsync<T, D, 4, QT> dma;      // 32-row tiles: two copy instructions per wavefront and tensor
  dma.init(a.sn, wave);
  TileAsync<T, D, 4, 64> dma64;    // the V block: four 64-row pieces
  dma64.init(a.sn, wave);
  // This wavefront's share of the copy of query tile t into buffer buf, in five pieces: two copy
  // instructions per tensor, and one row vector for wavefronts 0 and 1.
  // (N is a multiple of the tile height here: the launcher sends other lengths to the 32-key kernel)
  auto fetch_piece = [&](int t, int buf, int k) {
    if (k < 2) dma.copy_one(Qg + (int64_t)t * QT * a.sn, Qs0 + buf * QT * D, k);
    else if (k < 4) dma.copy_one(Gg + (int64_t)t * QT * a.sn, Gs0 + buf * QT * D, k - 2);
    else {
      const int row = min(t * QT + lane, a.Nr - 1);   // whole-wavefront copies: 64 floats, clamped to the head
      if (wave == 0) async_copy_b32(Lg + row, __builtin_amdgcn_readfirstlane(lds_addr(Ls0 + 64 * buf)));
      if (wave == 1) async_copy_b32(Dg + row, __builtin_amdgcn_readfirstlane(lds_addr(Ds0 + 64 * buf)));
    }
  };
  auto fetch_tile = [&](int t, int buf) {
#pragma unroll
    for (int k = 0; k < 5; ++k) fetch_piece(t, buf, k);
  };
  const float c = a.scale_log2;

  // V rows of this key block (pieces beyond the end of the tensor repeat the last rows that exist:
  // those keys are never stored)
#pragma unroll
  for (int piece = 0; piece < KB / 64; ++piece) {
    const int row0 = min(kt * KB + 64 * piece, ((a.N - 1) / 64) * 64);
    dma64.copy_rows(Vg, a.sn, row0, a.N, Vb + 64 * piece * D);
  }
  if (first < limit) fetch_tile(first, 0);
  if (first + 1 < limit) fetch_tile(first + 1, 1);
  wait_async_copies();
  __syncthreads();

  // One query tile.  Tiles are copied two ahead into a ring of three buffers; the buffer index is
  // a compile-time constant (the loop below is unrolled by three), so that every LDS address is a
  // per-lane register plus an immediate offset.  The copy instructions of tile t + 2 are issued
  // one at a time between the MFMAs of the S stream of tile t (slot plan above).
  auto tile_step = [&](int t, auto buf_c) {
    constexpr int buf = decltype(buf_c)::value;
    constexpr int buf_next2 = (buf + 2) % NBUF;
    const bool more = t + 2 < limit;
    const int i0 = t * QT;

    // causal: a wavefront joins from the tile that holds its first key on; in the two tiles on
    // its diagonal, query i0 + 8 i4 + 4 g + e sees key kw0 + 32 kb + r iff key <= query
    const bool diag = CAUSAL && i0 < kw0 + 64;
    if (!CAUSAL || i0 >= kw0) {
      const T* Qt = Qs0 + buf * QT * D;
      const T* Gt = Gs0 + buf * QT * D;
      const float* Lt = Ls0 + 64 * buf;
      const float* Dt = Ds0 + 64 * buf;
      // ---- operand fragments, in the order the MFMA slots use them.  A fragments (one per two
      // slots): 0..7 Q rows (S), 8..15 dO rows (dP), then per half cc of the queries: 4 dO^T (dV)
      // and 4 Q^T (dK) fragments by transposing reads.
      auto a_frag = [&](int n) -> T8 {
        if (n < KK) return *(const T8*)(Qt + lds_off<D>(r, 2 * n + g));
        if (n < 2 * KK) return *(const T8*)(Gt + lds_off<D>(r, 2 * (n - KK) + g));
        const int m = n - 2 * KK, cc = m >> 3, db = m & 3;
        const T* base = (((m >> 2) & 1) ? Qt : Gt) + 16 * cc * D;
        return tr_frag<T8>(base + tro.off[db][0], base + tro.off[db][1]);
      };
      auto v_frag = [&](int n) -> T8 {   // n = 2 kk + kb: B operands of the dP stream
        return *(const T8*)(Vb + lds_off<D>(wave * 64 + 32 * (n & 1) + r, 2 * (n >> 1) + g));
      };
      constexpr int NA = 2 * KK + 4 * DB, PFA = 3;   // 32 A fragments, read 3 ahead
      constexpr int NV = 2 * KK, PFV = 3;            // 16 V fragments, read 3 ahead
      T8 ra[PFA], rv[PFV];
      f32x16 s[2], dp[2];
      T8 pf[2][2], dsf[2][2];
      f32x4 lr[2];
      // ---- the work items of the slot plan
      auto seed_dp = [&](int i4) {
        const f32x4 c4 = *(const f32x4*)(Dt + 8 * i4 + 4 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) { dp[0][4 * i4 + e] = c4[e]; dp[1][4 * i4 + e] = c4[e]; }
      };
      auto lrow = [&](int i4) { return *(const f32x4*)(Lt + 8 * i4 + 4 * g); };
      // P = exp(S - L), kept as fp32 in place; pairs go to the 16-bit operands of dV
      auto p_unit = [&](auto uc) __attribute__((always_inline)) {
        constexpr int u = decltype(uc)::value;
        constexpr int cc = u >> 4, kb = (u >> 3) & 1, i4 = 2 * cc + ((u >> 2) & 1), e = u & 3, x = 4 * i4 + e;
        float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][x], c, -lr[i4 & 1][e]));
        if (CAUSAL && diag && kw0 + 32 * kb + r > i0 + 8 * i4 + 4 * g + e) p = 0.f;
        pin_here(p);
        s[kb][x] = p;
        if constexpr (e & 1) {
          pf[kb][cc][4 * (i4 & 1) + e - 1] = (T)s[kb][x - 1];
          pf[kb][cc][4 * (i4 & 1) + e] = (T)p;
          pin_here(pf[kb][cc]);
        }
      };
      // dS = P o (dP - D) for a pair of values (dP started from -D)
      auto ds_unit = [&](auto vc) __attribute__((always_inline)) {
        constexpr int v = decltype(vc)::value;
        constexpr int cc = v >> 3, kb = (v >> 2) & 1, i4 = 2 * cc + ((v >> 1) & 1), e0 = 2 * (v & 1), x = 4 * i4 + e0;
        dsf[kb][cc][4 * (i4 & 1) + e0] = (T)(s[kb][x] * dp[kb][x]);
        dsf[kb][cc][4 * (i4 & 1) + e0 + 1] = (T)(s[kb][x + 1] * dp[kb][x + 1]);
        pin_here(dsf[kb][cc]);
      };
      auto plan_item = [&](auto item_c) __attribute__((always_inline)) {
        constexpr int item = decltype(item_c)::value;
        if constexpr (item >= 400) { if (more) fetch_piece(t + 2, buf_next2, item - 400); }
        else if constexpr (item >= 310) { lr[0] = lrow(2 * (item - 310)); lr[1] = lrow(2 * (item - 310) + 1); }
        else if constexpr (item >= 300) seed_dp(item - 300);
        else if constexpr (item >= 200) ds_unit(std::integral_constant<int, item - 200>());
        else if constexpr (item >= 100) p_unit(std::integral_constant<int, item - 100>());
      };
#pragma unroll
      for (int n = 0; n < PFA; ++n) ra[n] = a_frag(n);
      __builtin_amdgcn_sched_barrier(0);
      // One MFMA slot: the instruction, the operand reads that keep the rings full, the slot's
      // items of the plan.  The slot number is a compile-time constant.
      auto slot_body = [&](auto slot_c) __attribute__((always_inline)) {
        constexpr int slot = decltype(slot_c)::value;
        constexpr int n = slot_frag(slot), kb = slot_kb(slot);   // A fragment of this slot, key block
        const T8 cur = ra[n % PFA];
        if constexpr (slot < 16) {
          if constexpr (slot < 2) {
            f32x16 z;
#pragma unroll
            for (int i = 0; i < 16; ++i) z[i] = 0.f;
            s[kb] = mfma32(cur, kf[kb][n], z);
          } else {
            s[kb] = mfma32(cur, kf[kb][n], s[kb]);
          }
          // the V ring starts filling while S runs
          if constexpr (slot >= 16 - PFV) rv[(slot - (16 - PFV)) % PFV] = v_frag(slot - (16 - PFV));
        } else if constexpr (slot < 32) {
          constexpr int nv = slot - 16;
          const T8 cv = rv[nv % PFV];
          dp[kb] = mfma32(cur, cv, dp[kb]);
          if constexpr (nv + PFV < NV) rv[nv % PFV] = v_frag(nv + PFV);
        } else {
          // accumulator tiles: dV^T (kb, db) = 4 kb + db, dK^T = 8 + 4 kb + db
          constexpr int m = n - 2 * KK, cc = m >> 3, db = m & 3;
          constexpr bool is_dk = (m >> 2) & 1;
          constexpr int tile = (is_dk ? 8 : 0) + 4 * kb + db;
          if constexpr (is_dk) M::template mfma_acc<tile>(cur, dsf[kb][cc]);
          else M::template mfma_acc<tile>(cur, pf[kb][cc]);
        }
        if constexpr (slot == last_user(n) && n + PFA < NA) ra[n % PFA] = a_frag(n + PFA);   // both users of the fragment have issued
        plan_item(std::integral_constant<int, kPlan[slot][0]>());
        plan_item(std::integral_constant<int, kPlan[slot][1]>());
        plan_item(std::integral_constant<int, kPlan[slot][2]>());
        __builtin_amdgcn_sched_barrier(0);
      };
      static_for<64>(slot_body);
    } else {
      if (more) fetch_tile(t + 2, buf_next2);   // (causal) this wavefront sits the tile out
    }
    // Tile t + 1 (copied during the previous step) must have landed; the copies of tile t + 2
    // that this wavefront has just issued (5 for wavefronts 0 and 1, else 4) may stay in flight.
    if (more) {
      if (wave < 2) wait_async_copies_but<5>(); else wait_async_copies_but<4>();
    } else {
      wait_async_copies();
    }
    __syncthreads();
  };
  for (int t = first; t < limit; t += 3) {
    tile_step(t, std::integral_constant<int, 0>());
    if (t + 1 < limit) tile_step(t + 1, std::integral_constant<int, 1>());
    if (t + 2 < limit) tile_step(t + 2, std::integral_constant<int, 2>());
  }
  // The last MFMAs have left the pipe long before a wavefront gets here (the loop ends on a
  // workgroup barrier); the idle cycles make the accumulator reads safe whatever came before.
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");
  // The loop ended on a barrier (or never touched LDS): this wavefront's 64 V rows (16 KB of LDS)
  // stage its output rows, 32 rows x 128 at a time.  Rows of padded keys (lane = key) are
  // cleared, whatever their P was.
  T* stage = Vb + wave * 64 * D;
  auto put = [&](auto kb_c, auto which_c) {
    constexpr int kb = decltype(kb_c)::value, which = decltype(which_c)::value;   // which: 0 dV, 1 dK
    const int k0 = kw0 + 32 * kb;
    const bool padded = k0 + r >= len;
    f32x16 out[DB];
    out[0] = acc_read<8 * which + 4 * kb + 0>();
    out[1] = acc_read<8 * which + 4 * kb + 1>();
    out[2] = acc_read<8 * which + 4 * kb + 2>();
    out[3] = acc_read<8 * which + 4 * kb + 3>();
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) out[db][i] = padded ? 0.f : out[db][i];
    T* dst = which ? (T*)a.dK : (T*)a.dV;
    store_rows_coalesced<T, D>(stage + 32 * D * kb, dst + head_off + (int64_t)k0 * a.sn, a.sn, out,
                               which ? a.tau : 1.f, a.N - k0);
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  put(std::integral_constant<int, 0>(), std::integral_constant<int, 0>());
  put(std::integral_constant<int, 1>(), std::integral_constant<int, 0>());
  put(std::integral_constant<int, 0>(), std::integral_constant<int, 1>());
  put(std::integral_constant<int, 1>(), std::integral_constant<int, 1>());
}

template <typename T>
int launch_t(const KArgs& a_in, bool causal, hipStream_t s) {
  KArgs a = a_in;
  const int n_kt = (a.N + KB - 1) / KB;
  a.n_items = a.B * a.H * n_kt;
  a.chunk = (a.n_items + kXcds - 1) / kXcds;
  {
    const int64_t tile_bytes = 2 * (int64_t)a.N * D * (int64_t)sizeof(T);   // Q and dO of one head
    const int64_t fit = ((int64_t)8 << 20) / tile_bytes;
    a.group = (int)(fit < 1 ? 1 : (fit > 8 ? 8 : fit));
  }
  const dim3 grid(kXcds * a.chunk), block(NT);
  if (causal) hipLaunchKernelGGL((dkv_w64_kernel<T, true>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((dkv_w64_kernel<T, false>), grid, block, 0, s, a);
  return (int)hipGetLastError();
}

}  // namespace

int launch_dkv_w64(const KArgs& a, int dtype, bool causal, hipStream_t s) {
  return dtype == 0 ? launch_t<_Float16>(a, causal, s) : launch_t<__bf16>(a, causal, s);
}

}  // namespace attn
