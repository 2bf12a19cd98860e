// Duel bookkeeping on the device (Sec. 4.2 of the paper): the verdict of a judge pass read off the last-position
// logits.  The credit ledger the verdicts are settled in is host code (ledger.cpp).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/www.h"

#define WWW_EXPORT extern "C" __attribute__((visibility("default")))

void set_error(const char* fmt, ...);

// ------------------------------------------------------------------------------------------------
// Verdict: one thread per judged sequence reads the two designated logits of its row.
__global__ __launch_bounds__(256) void judge_verdict_kernel(const float* __restrict__ logits, int batch, int64_t vocab, int token_a,
                                                            int token_b, int32_t* __restrict__ verdict, float* __restrict__ margin) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b >= batch) return;
  const float la = logits[(int64_t)b * vocab + token_a], lb = logits[(int64_t)b * vocab + token_b];
  verdict[b] = (la >= lb) ? 0 : 1;  // a tie goes to the first answer, as the lowest index wins the greedy argmax
  if (margin) margin[b] = la - lb;
}

WWW_EXPORT int www_judge_verdict(const float* logits_dev, int32_t batch, int32_t vocab, int32_t token_a, int32_t token_b,
                                 int32_t* verdict_dev, float* margin_dev, void* hip_stream) {
  if (batch < 0 || vocab <= 0) { set_error("negative batch or non-positive vocab"); return WWW_E_INVALID_ARG; }
  if (token_a < 0 || token_a >= vocab || token_b < 0 || token_b >= vocab || token_a == token_b) {
    set_error("verdict tokens %d, %d must be distinct ids below vocab %d", token_a, token_b, vocab);
    return WWW_E_INVALID_ARG;
  }
  if (batch == 0) return WWW_OK;
  if (!logits_dev || !verdict_dev) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  hipLaunchKernelGGL(judge_verdict_kernel, dim3((batch + 255) / 256), dim3(256), 0, (hipStream_t)hip_stream, logits_dev, batch,
                     (int64_t)vocab, token_a, token_b, verdict_dev, margin_dev);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("verdict kernel launch failed: %s", hipGetErrorString(e)); return WWW_E_HIP; }
  return WWW_OK;
}
