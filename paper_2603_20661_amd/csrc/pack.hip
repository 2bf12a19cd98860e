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

// Value of an FP8 E4M3 code (OCP: bias 7, subnormals at exponent 0, no infinities), exact in fp16: the seven magnitude
// bits, moved to fp16's exponent / mantissa position, read as fp16 give the value divided by 2^8 (bias 15 instead of 7).
__device__ __forceinline__ float e4m3_to_float(uint8_t c) {
  const uint16_t h = (uint16_t)(((c & 0x80u) << 8) | ((c & 0x7Fu) << 7));
  return f16_bits_to_float(h) * 256.f;
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
      else if constexpr (sizeof(SRC) == 1) x = e4m3_to_float(((const uint8_t*)src)[srow * K + k]);  // exact in the hi plane
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
  if (src_dtype == (int)WWW_DTYPE_FP8WO)
    hipLaunchKernelGGL(pack_matrix_kernel<uint8_t>, dim3((unsigned)blocks), dim3(threads), 0, st, (const uint8_t*)src, N, K, KB, mode, hd,
                       n_rot_rows, F, (uint16_t*)hi, (uint16_t*)nullptr);
  else if (src_dtype == (int)WWW_DTYPE_F32)
    hipLaunchKernelGGL(pack_matrix_kernel<float>, dim3((unsigned)blocks), dim3(threads), 0, st, (const float*)src, N, K, KB, mode, hd,
                       n_rot_rows, F, (uint16_t*)hi, (uint16_t*)lo);
  else
    hipLaunchKernelGGL(pack_matrix_kernel<uint16_t>, dim3((unsigned)blocks), dim3(threads), 0, st, (const uint16_t*)src, N, K, KB, mode,
                       hd, n_rot_rows, F, (uint16_t*)hi, (uint16_t*)nullptr);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Gains of the query / key head normalisation, [2][hd], in the row order of a packed head (rotary pairs adjacent).
__global__ void pack_qk_gain_kernel(const float* __restrict__ q_src, const float* __restrict__ k_src, int hd, float* __restrict__ out) {
  const int p = threadIdx.x;
  if (p >= hd) return;
  const int s = source_row(p, 1, hd, hd, 0);
  out[p] = q_src[s];
  out[hd + p] = k_src[s];
}

int launch_pack_qk_gain(const float* q_src, const float* k_src, int hd, float* out, hipStream_t st) {
  hipLaunchKernelGGL(pack_qk_gain_kernel, dim3(1), dim3(128), 0, st, q_src, k_src, hd, out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// FP8 codes in the order the decode GEMM streams them: 16-byte unit ((pair of k blocks j, row group rg), lane) holds the
// lane's 8 codes of k block 2j followed by its 8 codes of k block 2j + 1 (rows and k positions as in the fp16 layout);
// positions past K, and the second half of a last odd block, are zero codes.
__global__ void pack_fp8_kernel(const uint8_t* __restrict__ src, int N, int K, int KB, int mode, int hd, int n_rot_rows, int F,
                                uint8_t* __restrict__ out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int NRG = N / 16, KB2 = (KB + 1) / 2;
  if (idx >= (int64_t)NRG * KB2 * 64) return;
  const int lane = (int)(idx & 63);
  const int64_t unit = idx >> 6;
  const int rg = (int)(unit % NRG), kb2 = (int)(unit / NRG);
  const int64_t srow = source_row(rg * 16 + (lane & 15), mode, hd, n_rot_rows, F);
  union { uint8_t b[16]; uint4 v; } o;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int k0 = (kb2 * 2 + half) * 32 + (lane >> 4) * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.b[half * 8 + e] = (k0 + e < K) ? src[srow * K + k0 + e] : (uint8_t)0;
  }
  *reinterpret_cast<uint4*>(out + idx * 16) = o.v;
}

int launch_pack_fp8(const void* src, int N, int K, int KB, int mode, int hd, int n_rot_rows, int F, uint8_t* out, hipStream_t st) {
  const int64_t total = (int64_t)(N / 16) * ((KB + 1) / 2) * 64;
  hipLaunchKernelGGL(pack_fp8_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint8_t*)src, N, K, KB, mode, hd,
                     n_rot_rows, F, out);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// int4 weight-only sources: codes[N][K/2] (two per byte, even column low), scales[N][K/group] in bf16.
__device__ __forceinline__ int int4_code(const uint8_t* __restrict__ codes, int64_t row, int K, int k) {
  const uint8_t b = codes[(row * K + k) >> 1];
  return (k & 1) ? (b >> 4) : (b & 0xF);
}

// fp16 plane for the prefill GEMMs, in the usual fragment order: (c - 8) * scale (a 4-bit integer times a bf16: exact in
// fp16 unless the scale is below fp16's normal range)
__global__ void pack_int4_f16_kernel(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales, int N, int K, int KB, int group,
                                     int mode, int hd, int n_rot_rows, int F, uint16_t* __restrict__ hi) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)(N / 16) * KB * 64) return;
  const int lane = (int)(idx & 63);
  const int64_t frag = idx >> 6;
  const int NRG = N / 16;
  const int rg = (int)(frag % NRG), kb = (int)(frag / NRG);
  const int64_t srow = source_row(rg * 16 + (lane & 15), mode, hd, n_rot_rows, F);
  const int k0 = kb * 32 + (lane >> 4) * 8;
  union { uint16_t s[8]; uint4 v; } h;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k = k0 + e;
    float x = 0.f;
    if (k < K) x = (float)(int4_code(codes, srow, K, k) - 8) * bf16_bits_to_float(scales[srow * (K / group) + k / group]);
    h.s[e] = f32_to_f16_sat(x);
  }
  *reinterpret_cast<uint4*>(hi + idx * 8) = h.v;
}

// Decode order: 16-byte unit ((chunk j of 4 k blocks, row group rg), lane) holds the lane's 8 codes of k blocks 4j .. 4j+3,
// one 32-bit word per k block, the code of the lane's e-th column in nibble e; zero weights (code 8) past K.
// Group scales for the decode GEMM: fp16, [chunk][packed row][4] = the scale of each of the chunk's 4 k blocks.
__global__ void pack_int4_kernel(const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scales, int N, int K, int KB, int group,
                                 int mode, int hd, int n_rot_rows, int F, uint8_t* __restrict__ out, uint16_t* __restrict__ sc_out) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int NRG = N / 16, KB4 = (KB + 3) / 4;
  if (idx >= (int64_t)NRG * KB4 * 64) return;
  const int lane = (int)(idx & 63);
  const int64_t unit = idx >> 6;
  const int rg = (int)(unit % NRG), kb4 = (int)(unit / NRG);
  const int p = rg * 16 + (lane & 15);
  const int64_t srow = source_row(p, mode, hd, n_rot_rows, F);
  uint32_t w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int k0 = (kb4 * 4 + j) * 32 + (lane >> 4) * 8;
    uint32_t v = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) v |= (uint32_t)((k0 + e < K) ? int4_code(codes, srow, K, k0 + e) : 8) << (4 * e);
    w[j] = v;
  }
  *reinterpret_cast<uint4*>(out + idx * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  if (lane < 16) {
    union { uint16_t s[4]; uint2 v; } sc;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = (kb4 * 4 + j) * 32;
      sc.s[j] = k < K ? f32_to_f16_sat(bf16_bits_to_float(scales[srow * (K / group) + k / group])) : (uint16_t)0;
    }
    *reinterpret_cast<uint2*>(sc_out + ((int64_t)kb4 * N + p) * 4) = sc.v;
  }
}

int launch_pack_int4(const void* codes, const void* scales_bf16, int N, int K, int KB, int group, int mode, int hd, int n_rot_rows, int F,
                     uint16_t* f16_plane, uint8_t* codes_out, void* scales_out, hipStream_t st) {
  if (f16_plane) {
    const int64_t total = (int64_t)(N / 16) * KB * 64;
    hipLaunchKernelGGL(pack_int4_f16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint8_t*)codes,
                       (const uint16_t*)scales_bf16, N, K, KB, group, mode, hd, n_rot_rows, F, f16_plane);
  }
  const int64_t total = (int64_t)(N / 16) * ((KB + 3) / 4) * 64;
  hipLaunchKernelGGL(pack_int4_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const uint8_t*)codes,
                     (const uint16_t*)scales_bf16, N, K, KB, group, mode, hd, n_rot_rows, F, codes_out, (uint16_t*)scales_out);
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
