// Benchmark hook: what the matrix cores of this GPU sustain on a loop of nothing but fp16 MFMAs with operands in
// registers (no memory traffic, no LDS) - the achievable figure beside the published dense peak that prefill rooflines
// are quoted against.  Operands are pseudo-random fp16 values: with constant data the same loop clocks higher.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/www.h"

#define WWW_EXPORT extern "C" __attribute__((visibility("default")))

void set_error(const char* fmt, ...);

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int MFMA_PER_ITER = 8;  // independent accumulators per wavefront: the 32x32x16 MFMA never waits for its own result

__global__ __launch_bounds__(256, 2) void mfma_loop_kernel(int iters, float* __restrict__ sink) {
  // operands: a different small value per lane and element, sign and magnitude varying (integer hash of the lane)
  f16x8 a[2], b[2];
  uint32_t h = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u;
      a[s][e] = (_Float16)(((int)(h >> 20) - 2048) * (1.0f / 4096.0f));
      h = h * 1664525u + 1013904223u;
      b[s][e] = (_Float16)(((int)(h >> 20) - 2048) * (1.0f / 4096.0f));
    }
  f32x16 acc[MFMA_PER_ITER];
#pragma unroll
  for (int i = 0; i < MFMA_PER_ITER; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < MFMA_PER_ITER; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i & 1], b[(i >> 1) & 1], acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MFMA_PER_ITER; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = s;
}

}  // namespace

WWW_EXPORT int www_debug_mfma_loop(int32_t workgroups, int32_t iters, float* sink_dev, double* flops_out, void* hip_stream) {
  if (workgroups < 1 || workgroups > (1 << 20) || iters < 1 || !sink_dev) { set_error("bad argument"); return WWW_E_INVALID_ARG; }
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, sink_dev);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("launch failed: %s", hipGetErrorString(e)); return WWW_E_HIP; }
  if (flops_out) *flops_out = (double)workgroups * 4.0 * (double)iters * MFMA_PER_ITER * (2.0 * 32 * 32 * 16);
  return WWW_OK;
}
