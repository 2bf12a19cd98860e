// Temperature / nucleus (top-p) sampling from next-token logits (App. C of the paper lists temperature and top-p among
// the generation parameters; its own runs use temperature 0, i.e. the greedy argmax of the decode path).
//
// Per row: z_i = logit_i / T, e_i = exp(z_i - max z).  The nucleus is {i : e_i >= tau}, tau being the largest of the e
// values for which the members' sum reaches top_p * sum of all e (elements equal to tau are all in).  The token is drawn
// by the inverse CDF over the nucleus taken in index order: the first member whose running sum exceeds u * (nucleus sum),
// u in [0, 1) supplied by the caller.  No sort: tau is found by bisection on the bit pattern of a non-negative float
// (31 passes over the row's e values, which stay in L2), every sum has a fixed order, so a call is reproducible.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/www.h"

#define WWW_EXPORT extern "C" __attribute__((visibility("default")))

void set_error(const char* fmt, ...);

namespace {

constexpr int TPB = 1024;

// sum of v over the workgroup, added in a fixed order (lanes by halving, then wavefronts in index order); all threads get it
__device__ float block_sum(float v, float* red) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();  // red may still be read from the previous call
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < TPB / 64; ++w) t += red[w];
  return t;
}

__device__ float block_max(float v, float* red) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v = fmaxf(v, __shfl_xor(v, s));
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int w = 1; w < TPB / 64; ++w) t = fmaxf(t, red[w]);
  return t;
}

__global__ __launch_bounds__(TPB) void sample_top_p_kernel(const float* __restrict__ logits, int V, float inv_T, float top_p,
                                                           const float* __restrict__ u01, float* __restrict__ scratch,
                                                           int32_t* __restrict__ tokens) {
  __shared__ float red[TPB / 64];
  __shared__ float part[TPB];
  __shared__ int s_owner;
  __shared__ float s_before;
  const int row = blockIdx.x, tid = threadIdx.x;
  const float* lg = logits + (int64_t)row * V;
  float* e = scratch + (int64_t)row * V;

  float m = -INFINITY;
  for (int i = tid; i < V; i += TPB) m = fmaxf(m, lg[i] * inv_T);
  m = block_max(m, red);
  float acc = 0.f;
  for (int i = tid; i < V; i += TPB) {
    const float x = exp2f((lg[i] * inv_T - m) * 1.4426950408889634f);
    e[i] = x;
    acc += x;
  }
  const float total = block_sum(acc, red);  // the barriers inside also make every thread's e[] visible to the workgroup
  const float need = top_p * total;

  // largest threshold (as a bit pattern; non-negative floats order like their bits) whose members' sum still reaches `need`
  uint32_t lo = 0u, hi = 0x3F800001u;  // sum(e >= 0) = total >= need;  no e exceeds 1
  while (hi - lo > 1u) {
    const uint32_t mid = lo + (hi - lo) / 2u;
    const float thr = __uint_as_float(mid);
    float s = 0.f;
    for (int i = tid; i < V; i += TPB) {
      const float x = e[i];
      s += x >= thr ? x : 0.f;
    }
    s = block_sum(s, red);
    if (s >= need) lo = mid; else hi = mid;  // the same value in every thread
  }
  const float tau = __uint_as_float(lo);

  // inverse CDF over the nucleus in index order: contiguous segment per thread, running sums across threads by thread 0
  const int seg = (V + TPB - 1) / TPB;
  const int i0 = min(tid * seg, V), i1 = min(i0 + seg, V);
  float mine = 0.f;
  for (int i = i0; i < i1; ++i) {
    const float x = e[i];
    mine += x >= tau ? x : 0.f;
  }
  part[tid] = mine;
  __syncthreads();
  if (tid == 0) {
    float nuc = 0.f;
    for (int t = 0; t < TPB; ++t) nuc += part[t];
    const float target = u01[row] * nuc;
    float run = 0.f;
    int owner = -1;
    for (int t = 0; t < TPB && owner < 0; ++t) {
      if (part[t] > 0.f && target < run + part[t]) { owner = t; s_before = run; }
      else run += part[t];
    }
    if (owner < 0) {  // rounding at the very end of the range: the last thread that holds a member
      for (int t = TPB - 1; t >= 0 && owner < 0; --t)
        if (part[t] > 0.f) owner = t;
      s_before = -INFINITY;  // marks the fallback: take the owner's last member
    }
    s_owner = owner;
    part[0] = target;
  }
  __syncthreads();
  if (tid == s_owner) {
    const float target = part[0];
    float run = s_before;
    int pick = -1, last = -1;
    for (int i = i0; i < i1 && pick < 0; ++i) {
      const float x = e[i];
      if (!(x >= tau)) continue;
      last = i;
      if (s_before != -INFINITY) {
        run += x;
        if (target < run) pick = i;
      }
    }
    tokens[row] = pick >= 0 ? pick : last;
  }
}

}  // namespace

WWW_EXPORT int www_sample_top_p(const float* logits_dev, int32_t batch, int32_t vocab, float temperature, float top_p,
                                const float* u01_dev, float* scratch_dev, int32_t* tokens_dev, void* hip_stream) {
  if (batch < 0 || vocab <= 0) { set_error("negative batch or non-positive vocab"); return WWW_E_INVALID_ARG; }
  if (!(temperature > 0.f) || !(top_p > 0.f && top_p <= 1.f)) {
    set_error("temperature must be positive (temperature 0 is the greedy token of www_decode_step) and top_p in (0, 1]");
    return WWW_E_INVALID_ARG;
  }
  if (batch == 0) return WWW_OK;
  if (!logits_dev || !u01_dev || !scratch_dev || !tokens_dev) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  hipLaunchKernelGGL(sample_top_p_kernel, dim3(batch), dim3(TPB), 0, (hipStream_t)hip_stream, logits_dev, vocab, 1.f / temperature, top_p,
                     u01_dev, scratch_dev, tokens_dev);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) { set_error("sampling kernel launch failed: %s", hipGetErrorString(err)); return WWW_E_HIP; }
  return WWW_OK;
}

// ------------------------------------------------------------------------------------------------
// The same sampling for callers that cannot allocate device memory (code under HIP graph capture, serving loops and
// harnesses that forbid hipMalloc): the [batch][vocab] buffer of unnormalised probabilities lives in a file-scope
// device array instead of a caller-provided one.  Every GPU holds its own copy of the array at its own address until
// the process ends; the address is looked up once per device and kept.  All calls on one GPU share the array: calls
// that overlap on one GPU (different streams, different host threads) race.  Nothing in it has to start at zero - the
// kernel writes every element it later reads.
static __device__ __align__(256) float scratch[WWW_SAMPLE_STATIC_MAX_FLOATS];

namespace {
constexpr int MAX_DEVICES = 64;
float* g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on each device, once looked up
std::mutex g_scratch_mutex;

// device address of this device's copy of `scratch` (the array's name itself is only a host-side stand-in)
int static_scratch(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { set_error("hipGetDevice failed: %s", hipGetErrorString(e)); return WWW_E_HIP; }
  if (dev < 0 || dev >= MAX_DEVICES) { set_error("device index %d out of range", dev); return WWW_E_HIP; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    float* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) { set_error("hipGetSymbolAddress failed: %s", hipGetErrorString(e)); return WWW_E_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return WWW_OK;
}
}  // namespace

WWW_EXPORT int www_sample_top_p_static(const float* logits_dev, int32_t batch, int32_t vocab, float temperature, float top_p,
                                       const float* u01_dev, int32_t* tokens_dev, void* hip_stream) {
  if (batch < 0 || vocab <= 0) { set_error("negative batch or non-positive vocab"); return WWW_E_INVALID_ARG; }
  if ((uint64_t)batch * (uint64_t)vocab > (uint64_t)WWW_SAMPLE_STATIC_MAX_FLOATS) {
    set_error("batch * vocab = %llu exceeds the %llu floats of the built-in scratch array; use www_sample_top_p with a buffer of your own",
              (unsigned long long)((uint64_t)batch * (uint64_t)vocab), (unsigned long long)WWW_SAMPLE_STATIC_MAX_FLOATS);
    return WWW_E_CAPACITY;
  }
  if (batch == 0) {  // still validate, as www_sample_top_p does
    if (!(temperature > 0.f) || !(top_p > 0.f && top_p <= 1.f)) { set_error("temperature must be positive and top_p in (0, 1]"); return WWW_E_INVALID_ARG; }
    return WWW_OK;
  }
  float* ptr = nullptr;
  if (int rc = static_scratch(&ptr)) return rc;
  return www_sample_top_p(logits_dev, batch, vocab, temperature, top_p, u01_dev, ptr, tokens_dev, hip_stream);
}
