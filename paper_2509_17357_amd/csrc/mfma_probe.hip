// Measurement aid, not part of the attention path: the rate of v_mfma_f32_32x32x16_bf16 that
// this GPU sustains when nothing else runs.  The published dense bf16 peak assumes the matrix
// pipes busy every cycle at the nominal clock; under a chip-wide MFMA load the clock follows
// the power drawn, and that follows the switching activity of the operands.  The probe runs
// the same instruction stream with operand registers that hold small constants or random
// bf16 values, so the difference is the data's.
#include <hip/hip_runtime.h>

#include "cronus_internal.h"

namespace cronus {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 512;     // 8 wavefronts, two per SIMD, like the attention kernel
constexpr int kProbeMfmaPerIter = 32;  // per wavefront

template <bool RANDOM>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(float* sink, int iters) {
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  u32x4 a[8], b[8];
  unsigned h = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
  auto next = [&]() {
    h ^= h << 13;
    h ^= h >> 17;
    h ^= h << 5;
    // two bf16 values: random sign and mantissa, exponent 0x7b .. 0x7e (magnitude 1/16 .. 1)
    return (h & 0x81ff81ffu) | 0x3d803d80u | ((h >> 3) & 0x01000100u);
  };
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a[i][j] = RANDOM ? next() : (unsigned)(i + j);
      b[i][j] = RANDOM ? next() : (unsigned)(2 * i + j);
    }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < kProbeMfmaPerIter; ++s)
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[s & 3]) : "v"(a[s & 7]), "v"(b[(s >> 2) & 7]));
  }
  float r = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[j][i];
  sink[(size_t)blockIdx.x * kProbeThreads + threadIdx.x] = r;
}

}  // namespace

int launch_mfma_probe(int random_operands, int iters, int n_cus, float* sink, void* stream, double* flops) {
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (random_operands)
    hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)n_cus), dim3(kProbeThreads), 0, s, sink, iters);
  else
    hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)n_cus), dim3(kProbeThreads), 0, s, sink, iters);
  if (hipGetLastError() != hipSuccess) return CRONUS_ERR_HIP;
  *flops = 2.0 * 32 * 32 * 16 * (double)kProbeMfmaPerIter * (double)iters * (kProbeThreads / 64) * (double)n_cus;
  return CRONUS_OK;
}

int mfma_probe_sink_floats(int n_cus) { return n_cus * kProbeThreads; }

}  // namespace cronus
