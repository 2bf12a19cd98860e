// Load-time kernels: repack a row-major weight matrix into MFMA fragment order (see common.h),
// and the block-table slot probe used by the indexing tests.
#include "common.h"

// packed row -> source row
__device__ __forceinline__ int source_row(int p, int mode, int hd, int n_rot_rows, int F) {
  if (mode == 1) {  // q and k heads: rotary pairs (i, i + hd/2) become neighbours (2i, 2i+1)
    if (p >= n_rot_rows) return p;
    int head = p / hd, w = p % hd, i = w >> 1;
    return head * hd + ((w & 1) ? i + hd / 2 : i);
  }
  if (mode == 2) {  // gate and up rows alternate in groups of 16
    int j = p >> 5, w = p & 31;
    return w < 16 ? 16 * j + w : F + 16 * j + (w - 16);
  }
  return p;
}

// one thread = one lane's 8 elements of one fragment
template <typename SRC>
__global__ void pack_matrix_kernel(const SRC* __restrict__ src, int N, int K, int KB, int mode, int hd, int n_rot_rows, int F,
                                   uint16_t* __restrict__ hi, uint16_t* __restrict__ lo) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t total = (int64_t)(N / 16) * KB * 64;
  if (idx >= total) return;
  int lane = (int)(idx & 63);
  int64_t frag = idx >> 6;
  const int NRG = N / 16;
  int rg = (int)(frag % NRG);
  int kb = (int)(frag / NRG);
  int p = rg * 16 + (lane & 15);
  int k0 = kb * 32 + (lane >> 4) * 8;
  int64_t srow = source_row(p, mode, hd, n_rot_rows, F);
  union { uint16_t s[8]; uint4 v; } h, l;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    int k = k0 + e;
    float x = 0.f;
    if (k < K) {
      if constexpr (sizeof(SRC) == 4) x = (float)src[srow * K + k];
      else x = bf16_bits_to_float(((const uint16_t*)src)[srow * K + k]);
    }
    split_f16(x, h.s[e], l.s[e]);
  }
  *reinterpret_cast<uint4*>(hi + idx * 8) = h.v;
  if (lo) *reinterpret_cast<uint4*>(lo + idx * 8) = l.v;
}

int launch_pack_matrix(const void* src, int src_dtype, int N, int K, int KB, int mode, int hd, int n_rot_rows, int F, uint16_t* hi, uint16_t* lo,
                       hipStream_t st) {
  int64_t total = (int64_t)(N / 16) * KB * 64;
  int threads = 256;
  int64_t blocks = (total + threads - 1) / threads;
  if (src_dtype == (int)WWW_DTYPE_F32)
    hipLaunchKernelGGL(pack_matrix_kernel<float>, dim3((unsigned)blocks), dim3(threads), 0, st, (const float*)src, N, K, KB, mode, hd,
                       n_rot_rows, F, (uint16_t*)hi, (uint16_t*)lo);
  else
    hipLaunchKernelGGL(pack_matrix_kernel<uint16_t>, dim3((unsigned)blocks), dim3(threads), 0, st, (const uint16_t*)src, N, K, KB, mode,
                       hd, n_rot_rows, F, (uint16_t*)hi, (uint16_t*)nullptr);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

__global__ void debug_slots_kernel(const int32_t* __restrict__ row, const int32_t* __restrict__ pos, int n, int64_t* __restrict__ out) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = kv_slot(row, pos[i]);
}

int launch_debug_slots(const int32_t* row, const int32_t* pos, int n, int64_t* out, hipStream_t st) {
  if (n == 0) return 0;
  hipLaunchKernelGGL(debug_slots_kernel, dim3((n + 255) / 256), dim3(256), 0, st, row, pos, n, out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}
