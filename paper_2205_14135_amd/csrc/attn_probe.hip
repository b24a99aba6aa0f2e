// Measurement aid, not part of the attention path: a kernel that does nothing but issue
// 32x32x16 MFMA instructions on register operands, so that a benchmark can state what dense
// matrix rate this particular GPU sustains (clock under load included) next to the published peak.
#include "attn_common.h"

namespace attn {
namespace {

constexpr int kProbeGroups = 2048;   // 8 workgroups of 4 wavefronts per compute unit
constexpr int kProbeThreads = 256;
constexpr int kProbeChain = 4;       // independent accumulators per wavefront

template <typename T>
__global__ __launch_bounds__(kProbeThreads) void mfma_rate_kernel(int iters, float* sink) {
  typedef typename Vec<T>::x8 x8;
  const int lane = threadIdx.x & 63;
  x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (T)(0.125f * (float)((lane * 7 + i * 3) % 13 - 6));
    b[i] = (T)(0.125f * (float)((lane * 5 + i * 11) % 13 - 6));
  }
  f32x16 c[kProbeChain];
#pragma unroll
  for (int j = 0; j < kProbeChain; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kProbeChain; ++j) c[j] = mfma32(a, b, c[j]);
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

int launch_mfma_rate(int dtype, int iters, float* sink, hipStream_t s, double* flops) {
  if (dtype == 0) hipLaunchKernelGGL(mfma_rate_kernel<_Float16>, dim3(kProbeGroups), dim3(kProbeThreads), 0, s, iters, sink);
  else hipLaunchKernelGGL(mfma_rate_kernel<__bf16>, dim3(kProbeGroups), dim3(kProbeThreads), 0, s, iters, sink);
  if (flops != nullptr)
    *flops = 2.0 * 32 * 32 * 16 * kProbeChain * (double)iters * (kProbeThreads / 64) * kProbeGroups;
  return (int)hipGetLastError();
}

}  // namespace attn
