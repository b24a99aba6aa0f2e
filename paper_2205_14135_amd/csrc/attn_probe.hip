// Measurement aid, not part of the attention path: a kernel that does nothing but issue
// 32x32x16 MFMA instructions on register operands, so that a benchmark can state what dense
// matrix rate this particular GPU sustains (clock under load included) next to the published peak.
// The clock a GPU holds under matrix load depends on how many operand bits change from one
// instruction to the next: with SETS = 1 every MFMA reads the same two registers (the most
// favourable case), with SETS = 4 consecutive MFMAs read four different pseudo-random operand
// pairs in turn, as the products of a real kernel do.
#include "attn_common.h"

namespace attn {
namespace {

constexpr int kProbeGroups = 2048;   // 8 workgroups of 4 wavefronts per compute unit
constexpr int kProbeThreads = 256;
constexpr int kProbeChain = 4;       // independent accumulators per wavefront

__device__ __forceinline__ float probe_value(uint32_t x) {   // integer hash -> [-2, 2)
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return (float)(int)(x >> 8) * (1.0f / 4194304.0f) - 2.0f;
}

template <typename T, int SETS>
__global__ __launch_bounds__(kProbeThreads) void mfma_rate_kernel(int iters, float* sink) {
  typedef typename Vec<T>::x8 x8;
  const int lane = threadIdx.x & 63;
  x8 a[SETS], b[SETS];
#pragma unroll
  for (int s = 0; s < SETS; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[s][i] = (T)probe_value((uint32_t)(lane * 64 + s * 16 + i));
      b[s][i] = (T)probe_value((uint32_t)(lane * 64 + s * 16 + 8 + i + 4096));
    }
  f32x16 c[kProbeChain];
#pragma unroll
  for (int j = 0; j < kProbeChain; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kProbeChain; ++j) c[j] = mfma32(a[j % SETS], b[j % SETS], c[j]);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kProbeChain; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c[j][i];
  // never true for finite sums of these operands; keeps the loop from being removed
  if (s == 1.2345678e30f) sink[0] = s;
}

}  // namespace

int launch_mfma_rate(int dtype, int iters, int operand_sets, float* sink, hipStream_t s, double* flops) {
  const dim3 grid(kProbeGroups), block(kProbeThreads);
  if (dtype == 0 && operand_sets == 1) hipLaunchKernelGGL((mfma_rate_kernel<_Float16, 1>), grid, block, 0, s, iters, sink);
  else if (dtype == 0) hipLaunchKernelGGL((mfma_rate_kernel<_Float16, 4>), grid, block, 0, s, iters, sink);
  else if (operand_sets == 1) hipLaunchKernelGGL((mfma_rate_kernel<__bf16, 1>), grid, block, 0, s, iters, sink);
  else hipLaunchKernelGGL((mfma_rate_kernel<__bf16, 4>), grid, block, 0, s, iters, sink);
  if (flops != nullptr)
    *flops = 2.0 * 32 * 32 * 16 * kProbeChain * (double)iters * (kProbeThreads / 64) * kProbeGroups;
  return (int)hipGetLastError();
}

}  // namespace attn
