// C-ABI front end: argument checks (host only, before any launch) and kernel dispatch.
#include "../../include/attn.h"
#include "attn_common.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <mutex>

// Scratch of attn_bwd_static: every GPU that runs the library holds its own copy of this array, at
// its own address, until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[ATTN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kVersion = 100;  // 0.1.0

static_assert(sizeof(attn_params) == 104, "attn_params layout is part of the ABI");

struct Checked {
  attn::KArgs k;
  int dtype, d;
  bool causal, dropout;
  hipStream_t stream;
};

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Validates everything that does not involve tensor pointers and fills the kernel arguments.
int check_params(const attn_params* p, Checked* out) {
  if (p == nullptr) return ATTN_ERR_NULL;
  if (p->dtype != ATTN_FP16 && p->dtype != ATTN_BF16) return ATTN_ERR_DTYPE;
  if (p->d != 16 && p->d != 32 && p->d != 64 && p->d != 128) return ATTN_ERR_HEADDIM;
  if (p->B <= 0 || p->H <= 0 || p->N <= 0) return ATTN_ERR_SHAPE;
  if (p->N > (1 << 30)) return ATTN_ERR_SHAPE;
  const int T = (p->N + attn::kMaskBlock - 1) / attn::kMaskBlock;   // a ragged last block is allowed (dense entry points)
  if ((int64_t)p->B * p->H > (int64_t)1 << 24) return ATTN_ERR_SHAPE;
  if ((int64_t)p->B * p->H * T > (int64_t)1 << 28) return ATTN_ERR_SHAPE;
  int64_t sb = p->stride_b, sh = p->stride_h, sn = p->stride_n;
  if (sb == 0 && sh == 0 && sn == 0) {
    sn = p->d;
    sh = (int64_t)p->N * p->d;
    sb = (int64_t)p->H * sh;
  }
  // rows must start on 16-byte boundaries for the vector loads
  if (sn < p->d || sn % 8 != 0 || sh % 8 != 0 || sb % 8 != 0 || sh < 0 || sb < 0) return ATTN_ERR_SHAPE;
  if (sn > ((int64_t)1 << 23)) return ATTN_ERR_SHAPE;   // the tile copies address 64 rows with 32-bit byte offsets
  // Output rows must not alias: the axes of size > 1, taken by increasing stride, must nest (each
  // stride at least the extent of the axis below it; the innermost at least one row).  This admits
  // head-major [B,H,N,d], token-major [B,N,H,d] views and padded rows, and rejects zero strides.
  {
    int64_t st[3] = {sn, sh, sb};
    int64_t sz[3] = {p->N, p->H, p->B};
    for (int i = 0; i < 3; ++i)
      for (int j = i + 1; j < 3; ++j)
        if (st[j] < st[i]) { std::swap(st[i], st[j]); std::swap(sz[i], sz[j]); }
    int64_t extent = p->d;
    for (int i = 0; i < 3; ++i) {
      if (sz[i] == 1) continue;
      if (st[i] < extent) return ATTN_ERR_SHAPE;
      if (st[i] > ((int64_t)1 << 50) / sz[i]) return ATTN_ERR_SHAPE;
      extent = st[i] * sz[i];
    }
  }
  if (!(p->dropout_p >= 0.0f && p->dropout_p < 1.0f)) return ATTN_ERR_DROPOUT_P;
  if (!std::isfinite(p->softmax_scale) || !(p->softmax_scale > 0.0f)) return ATTN_ERR_SCALE;

  attn::KArgs& k = out->k;
  std::memset(&k, 0, sizeof(k));
  k.sb = sb; k.sh = sh; k.sn = sn;
  k.B = p->B; k.H = p->H; k.N = p->N; k.T = T; k.Nr = T * attn::kMaskBlock;
  k.dvalid = p->d;
  k.tau = p->softmax_scale;
  k.scale_log2 = (float)((double)p->softmax_scale * 1.4426950408889634);
  // 8-bit fields: the dropout applied has probability T / 256, and kept entries are scaled by the
  // reciprocal of the matching keep probability
  k.drop_thr = (uint32_t)std::floor((double)p->dropout_p * 256.0);
  k.keep_scale = 256.0f / (256.0f - (float)k.drop_thr);
  k.seed_lo = (uint32_t)(p->seed & 0xFFFFFFFFu);
  k.seed_hi = (uint32_t)(p->seed >> 32);
  k.offset_lo = (uint32_t)(p->offset & 0xFFFFFFFFu);
  k.o_fp32 = p->o_fp32 != 0;
  k.klen = p->key_lengths;
  out->dtype = p->dtype;
  out->d = p->d == 16 ? 32 : p->d;   // head dimension 16 runs on the d = 32 kernels (zero upper half on chip)
  out->causal = p->causal != 0;
  out->dropout = k.drop_thr > 0;   // below 1/256 nothing is dropped: the generator stays off
  out->stream = (hipStream_t)p->stream;
  return ATTN_OK;
}

int check_mask(const uint8_t* block_mask, int32_t mask_block, int64_t mask_stride_h, const attn_params* p) {
  if (block_mask == nullptr) return ATTN_ERR_NULL;
  if (mask_block != attn::kMaskBlock) return ATTN_ERR_MASK;
  if (p->N % attn::kMaskBlock != 0) return ATTN_ERR_SHAPE;   // the block mask covers whole 128 x 128 blocks
  const int64_t T = p->N / attn::kMaskBlock;
  if (mask_stride_h < 0 || (mask_stride_h != 0 && mask_stride_h < T * T)) return ATTN_ERR_MASK;
  return ATTN_OK;
}

void set_items(attn::KArgs& k, int tiles_per_head) {
  k.n_items = k.B * k.H * tiles_per_head;
  k.chunk = (k.n_items + attn::kXcds - 1) / attn::kXcds;
}

// Backward scratch layout: D vector, base-2 row statistic | (block-sparse only) column counts |
// fp32 dK | fp32 dV.
struct WsLayout { size_t d_bytes, cnt_bytes, acc_bytes; };
WsLayout ws_layout(const attn_params* p) {
  WsLayout w;
  const size_t T = ((size_t)p->N + attn::kMaskBlock - 1) / attn::kMaskBlock;
  // two floats per row, rows padded to whole 128-blocks per head
  w.d_bytes = align_up(2 * (size_t)p->B * p->H * T * attn::kMaskBlock * sizeof(float), 256);
  // column counts, then the segment list: one counter plus at most kMaxSegs entries per column
  w.cnt_bytes = align_up(((size_t)p->B * p->H * T * (1 + attn::kMaxSegs) + 64) * sizeof(int), 256);
  const size_t d_kernel = p->d == 16 ? 32 : p->d;   // the fp32 accumulators have the kernels' row length
  w.acc_bytes = align_up((size_t)p->B * p->H * p->N * d_kernel * sizeof(float), 256);
  return w;
}

// every [B,H,N,d] tensor is read and written in 16-byte pieces
bool aligned16(std::initializer_list<const void*> ptrs) {
  for (const void* q : ptrs)
    if (((uintptr_t)q & 15u) != 0) return false;
  return true;
}

int fwd_common(const attn_params* p, const uint8_t* mask, int64_t mask_sh, bool sparse,
               const void* Q, const void* K, const void* V, void* O, float* LSE) {
  Checked c;
  const int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  if (!Q || !K || !V || !O || !LSE) return ATTN_ERR_NULL;
  if (!aligned16({Q, K, V, O}) || ((uintptr_t)LSE & 3u) != 0) return ATTN_ERR_SHAPE;
  c.k.Q = Q; c.k.K = K; c.k.V = V; c.k.O = O; c.k.LSE = LSE;
  c.k.mask = mask; c.k.mask_sh = mask_sh;
  set_items(c.k, c.k.T);
  const int e = attn::launch_fwd(c.k, c.dtype, c.d, c.causal, c.dropout, sparse, c.stream);
  return e == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int bwd_common(const attn_params* p, const uint8_t* mask, int64_t mask_sh, bool sparse,
               const void* Q, const void* K, const void* V, const void* O, const void* dO,
               const float* LSE, void* dQ, void* dK, void* dV, void* ws, size_t ws_bytes,
               void* const* events = nullptr) {
  Checked c;
  const int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return ATTN_ERR_NULL;
  if (!aligned16({Q, K, V, O, dO, dQ, dK, dV}) || ((uintptr_t)LSE & 3u) != 0) return ATTN_ERR_SHAPE;
  const size_t need = sparse ? attn_blocksparse_bwd_workspace_bytes(p) : attn_bwd_workspace_bytes(p);
  if (ws == nullptr || ((uintptr_t)ws & 255u) != 0 || ws_bytes < need) return ATTN_ERR_WORKSPACE;
  c.k.Q = Q; c.k.K = K; c.k.V = V; c.k.O = const_cast<void*>(O); c.k.LSE = const_cast<float*>(LSE);
  c.k.dO = dO; c.k.dQ = dQ; c.k.dK = dK; c.k.dV = dV;
  c.k.Dvec = (float*)ws;
  c.k.L2vec = c.k.Dvec + (size_t)p->B * p->H * c.k.Nr;
  if (sparse) {
    const WsLayout w = ws_layout(p);
    c.k.seglist = (int*)((char*)ws + w.d_bytes);
    c.k.colcnt = c.k.seglist + 64 + (size_t)p->B * p->H * (p->N / attn::kMaskBlock) * attn::kMaxSegs;
    c.k.dKacc = (float*)((char*)ws + w.d_bytes + w.cnt_bytes);
    c.k.dVacc = (float*)((char*)ws + w.d_bytes + w.cnt_bytes + w.acc_bytes);
  }
  c.k.mask = mask; c.k.mask_sh = mask_sh;
  set_items(c.k, c.k.T);
  hipEvent_t ev[4];
  if (events) {
    for (int i = 0; i < 4; ++i) {
      if (events[i] == nullptr) return ATTN_ERR_NULL;
      ev[i] = (hipEvent_t)events[i];
    }
  }
  const int e = attn::launch_bwd(c.k, c.dtype, c.d, c.causal, c.dropout, sparse, c.stream,
                                 events ? ev : nullptr);
  return e == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

// Device address of the current GPU's copy of `scratch`: looked up once per device, with that
// device current, and kept; nullptr if the runtime cannot tell.  Allocates nothing.
void* static_scratch() {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> ptr[kMaxDevices];
  static std::mutex mu;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* q = ptr[dev].load(std::memory_order_acquire);
  if (q != nullptr) return q;
  std::lock_guard<std::mutex> lock(mu);
  q = ptr[dev].load(std::memory_order_relaxed);
  if (q != nullptr) return q;
  void* addr = nullptr;
  if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || addr == nullptr) return nullptr;
  ptr[dev].store(addr, std::memory_order_release);
  return addr;
}

// Kernel-choice overrides: set through attn_debug_set_variant; until then the values of
// ATTN_FWD_VARIANT (base | pp) and ATTN_DKV_VARIANT (rs | fr | w64), read once.
std::atomic<int> g_fwd_variant{-1}, g_dkv_variant{-1};
int env_choice(const char* name, char c1, char c2, char c3 = 0) {
  const char* v = std::getenv(name);
  if (v == nullptr) return 0;
  return v[0] == c1 ? 1 : (v[0] == c2 ? 2 : (c3 != 0 && v[0] == c3 ? 3 : 0));
}

}  // namespace

namespace attn {
int fwd_variant() {
  int v = g_fwd_variant.load(std::memory_order_relaxed);
  if (v < 0) {
    v = env_choice("ATTN_FWD_VARIANT", 'b', 'p');
    int expected = -1;
    if (!g_fwd_variant.compare_exchange_strong(expected, v)) v = expected;
  }
  return v;
}
int dkv_variant() {
  int v = g_dkv_variant.load(std::memory_order_relaxed);
  if (v < 0) {
    v = env_choice("ATTN_DKV_VARIANT", 'r', 'f', 'w');
    int expected = -1;
    if (!g_dkv_variant.compare_exchange_strong(expected, v)) v = expected;
  }
  return v;
}
}  // namespace attn

extern "C" {

int attn_fwd(const attn_params* p, const void* Q, const void* K, const void* V, void* O, float* LSE) {
  return fwd_common(p, nullptr, 0, false, Q, K, V, O, LSE);
}

size_t attn_bwd_workspace_bytes(const attn_params* p) {
  Checked c;
  if (check_params(p, &c) != ATTN_OK) return 0;
  // D_i = rowsum(dO_i o O_i) and the base-2 row statistic: two floats per row
  return ws_layout(p).d_bytes;
}

size_t attn_blocksparse_bwd_workspace_bytes(const attn_params* p) {
  Checked c;
  if (check_params(p, &c) != ATTN_OK || p->N % attn::kMaskBlock != 0) return 0;
  const WsLayout w = ws_layout(p);
  return w.d_bytes + w.cnt_bytes + 2 * w.acc_bytes;
}

int attn_bwd(const attn_params* p, const void* Q, const void* K, const void* V, const void* O,
             const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
             size_t workspace_bytes) {
  return bwd_common(p, nullptr, 0, false, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes);
}

int attn_bwd_static(const attn_params* p, const void* Q, const void* K, const void* V, const void* O,
                    const void* dO, const float* LSE, void* dQ, void* dK, void* dV) {
  Checked c;
  const int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  if (ws_layout(p).d_bytes > (size_t)ATTN_STATIC_SCRATCH_BYTES) return ATTN_ERR_WORKSPACE;
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return ATTN_ERR_NULL;
  void* ws = static_scratch();
  if (ws == nullptr) return ATTN_ERR_LAUNCH;
  // the two row vectors are written in full by the first launch before the second reads them:
  // nothing of an earlier call's contents is ever read, nothing needs clearing
  return bwd_common(p, nullptr, 0, false, Q, K, V, O, dO, LSE, dQ, dK, dV, ws, ATTN_STATIC_SCRATCH_BYTES);
}

int attn_blocksparse_fwd(const attn_params* p, const uint8_t* block_mask, int32_t mask_block,
                         int64_t mask_stride_h, const void* Q, const void* K, const void* V, void* O,
                         float* LSE) {
  Checked c;
  int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  st = check_mask(block_mask, mask_block, mask_stride_h, p);
  if (st != ATTN_OK) return st;
  return fwd_common(p, block_mask, mask_stride_h, true, Q, K, V, O, LSE);
}

int attn_blocksparse_bwd(const attn_params* p, const uint8_t* block_mask, int32_t mask_block,
                         int64_t mask_stride_h, const void* Q, const void* K, const void* V,
                         const void* O, const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                         void* workspace, size_t workspace_bytes) {
  Checked c;
  int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  st = check_mask(block_mask, mask_block, mask_stride_h, p);
  if (st != ATTN_OK) return st;
  return bwd_common(p, block_mask, mask_stride_h, true, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace,
                    workspace_bytes);
}

int attn_bwd_timed(const attn_params* p, const uint8_t* block_mask, int32_t mask_block,
                   int64_t mask_stride_h, const void* Q, const void* K, const void* V, const void* O,
                   const void* dO, const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                   size_t workspace_bytes, void* const* events) {
  if (events == nullptr) return ATTN_ERR_NULL;
  if (block_mask != nullptr) {
    Checked c;
    int st = check_params(p, &c);
    if (st != ATTN_OK) return st;
    st = check_mask(block_mask, mask_block, mask_stride_h, p);
    if (st != ATTN_OK) return st;
  }
  return bwd_common(p, block_mask, mask_stride_h, block_mask != nullptr, Q, K, V, O, dO, LSE, dQ, dK, dV,
                    workspace, workspace_bytes, events);
}

int attn_debug_dropout_mask(const attn_params* p, uint8_t* keep) {
  Checked c;
  const int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  if (keep == nullptr) return ATTN_ERR_NULL;
  const int e = attn::launch_dropout_mask(c.k, keep, c.stream);
  return e == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int attn_debug_mfma_rate(int32_t dtype, int32_t iters, int32_t operand_sets, float* sink, void* stream,
                         double* flops) {
  if (sink == nullptr) return ATTN_ERR_NULL;
  if (dtype != ATTN_FP16 && dtype != ATTN_BF16) return ATTN_ERR_DTYPE;
  if (iters < 1 || iters > (1 << 20)) return ATTN_ERR_SHAPE;
  if (operand_sets != 1 && operand_sets != 4) return ATTN_ERR_SHAPE;
  const int e = attn::launch_mfma_rate(dtype, iters, operand_sets, sink, (hipStream_t)stream, flops);
  return e == 0 ? ATTN_OK : ATTN_ERR_LAUNCH;
}

int attn_debug_kernel_choice(const attn_params* p, int32_t sparse, int32_t* fwd_kernel, int32_t* dkv_kernel) {
  Checked c;
  const int st = check_params(p, &c);
  if (st != ATTN_OK) return st;
  if (fwd_kernel == nullptr || dkv_kernel == nullptr) return ATTN_ERR_NULL;
  if (sparse != 0 && p->N % attn::kMaskBlock != 0) return ATTN_ERR_SHAPE;
  *fwd_kernel = attn::choose_fwd(c.k, c.d, c.causal, c.dropout, sparse != 0);
  *dkv_kernel = attn::choose_dkv(c.k, c.d, c.causal, c.dropout, sparse != 0);
  return ATTN_OK;
}

int attn_debug_set_variant(int32_t fwd_variant, int32_t dkv_variant) {
  if (fwd_variant < -1 || fwd_variant > 2 || dkv_variant < -1 || dkv_variant > 3) return ATTN_ERR_SHAPE;
  if (fwd_variant >= 0) g_fwd_variant.store(fwd_variant);
  if (dkv_variant >= 0) g_dkv_variant.store(dkv_variant);
  return ATTN_OK;
}

const char* attn_strerror(int status) {
  switch (status) {
    case ATTN_OK: return "ok";
    case ATTN_ERR_NULL: return "a required pointer is NULL";
    case ATTN_ERR_SHAPE: return "unsupported shape, strides or tensor alignment (16 bytes; block-sparse: N must be a multiple of 128)";
    case ATTN_ERR_DTYPE: return "dtype must be ATTN_FP16 or ATTN_BF16";
    case ATTN_ERR_HEADDIM: return "head dimension must be 16, 32, 64 or 128";
    case ATTN_ERR_DROPOUT_P: return "dropout_p must be in [0, 1)";
    case ATTN_ERR_SCALE: return "softmax_scale must be finite and positive";
    case ATTN_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or too small (attn_bwd_static: problem beyond the built-in scratch)";
    case ATTN_ERR_MASK: return "mask_block must be 128 and mask_stride_h 0 or >= T*T";
    case ATTN_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

int attn_version(void) { return kVersion; }

}  // extern "C"
