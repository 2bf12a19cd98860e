/* Seeded synthetic-input generator shared by the CPU oracle's tests and the GPU path's tests.
 *
 * This file holds no transformer arithmetic: it only produces reproducible pseudo-random
 * numbers (weights, token ids, lengths, permutations) from a counter-based hash, so that both
 * sides of a parity test can be handed bit-identical inputs.
 *
 * Definition of the stream (seed, stream_id):
 *   key      = mix(seed ^ mix(stream_id))
 *   word(c)  = mix(key + c * 0x9E3779B97F4A7C15)          c = 0, 1, 2, ...
 * where mix is the 64-bit finaliser of the SplitMix64 generator (Steele, Lea, Flood 2014).
 * Normal deviates use the Box-Muller transform on the two 32-bit halves of word(i / 2):
 * element i takes the cosine branch when i is even and the sine branch when i is odd.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

static inline uint64_t mix(uint64_t z) {
  z += 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

static inline uint64_t stream_key(uint64_t seed, uint64_t stream_id) { return mix(seed ^ mix(stream_id)); }
static inline uint64_t word(uint64_t key, uint64_t c) { return mix(key + c * 0x9E3779B97F4A7C15ULL); }

static inline double normal_at(uint64_t key, uint64_t i) {
  uint64_t r = word(key, i >> 1);
  double u1 = ((double)(r >> 32) + 0.5) * (1.0 / 4294967296.0);
  double u2 = ((double)(r & 0xFFFFFFFFULL) + 0.5) * (1.0 / 4294967296.0);
  double rad = sqrt(-2.0 * log(u1));
  double ang = 6.283185307179586476925286766559 * u2;
  return (i & 1) ? rad * sin(ang) : rad * cos(ang);
}

/* round-to-nearest-even fp32 -> bf16 bit pattern (inputs are finite) */
static inline uint16_t f32_to_bf16_bits(float f) {
  union { float f; uint32_t u; } v; v.f = f;
  uint32_t lsb = (v.u >> 16) & 1u;
  return (uint16_t)((v.u + 0x7FFFu + lsb) >> 16);
}

/* out[i] = mean + std * N(0,1), i in [0,n), element counter starts at first */
void wwwsynth_normal_f32(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, double mean, double std, float* out) {
  uint64_t key = stream_key(seed, stream_id);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i) out[i] = (float)(mean + std * normal_at(key, first + (uint64_t)i));
}

/* as above, rounded fp32 -> bf16 (nearest even), stored as 16-bit patterns */
void wwwsynth_normal_bf16(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, double mean, double std, uint16_t* out) {
  uint64_t key = stream_key(seed, stream_id);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = f32_to_bf16_bits((float)(mean + std * normal_at(key, first + (uint64_t)i)));
}

/* fp32 -> OCP FP8 E4M3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, largest finite value
 * 448 = 0x7E, 0x7F is NaN and never produced), round to nearest even, saturating.  Part of the input recipe of the
 * fp8 weight-only configuration: the blob stores these codes, code = e4m3(value * inv_scale). */
static inline uint8_t f32_to_e4m3(float x) {
  uint8_t sign = signbit(x) ? 0x80 : 0x00;
  float a = fabsf(x);
  if (!(a < 448.f)) return sign | 0x7E; /* also catches NaN */
  int ex;
  (void)frexpf(a, &ex); /* a = m * 2^ex, m in [0.5, 1) */
  int e = ex - 1;
  if (a == 0.f || e < -6) { /* subnormal range: multiples of 2^-9; 8 of them make the smallest normal, code 0x08 */
    return sign | (uint8_t)rintf(a * 512.f);
  }
  float q = rintf(ldexpf(a, 3 - e)); /* 8 .. 16 */
  if (q == 16.f) { q = 8.f; e += 1; }
  return sign | (uint8_t)(((e + 7) << 3) | ((int)q - 8));
}

void wwwsynth_encode_e4m3(const float* src, uint64_t n, double inv_scale, uint8_t* out) {
  const float f = (float)inv_scale;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i) out[i] = f32_to_e4m3(src[i] * f);
}

/* Group-wise 4-bit codes of a [rows][cols] fp32 matrix (input recipe of the int4 weight-only configurations): for
 * every run of `group` consecutive elements of a row, scale = bf16(max|w| / 7) (1 if the run is all zero),
 * code = clamp(rint(w / scale) + 8, 0, 15); two codes per byte, the element with the even column in the low nibble.
 * codes: rows * cols / 2 bytes; scales: rows * (cols / group) bf16 patterns, row-major. */
void wwwsynth_encode_int4(const float* src, uint64_t rows, uint64_t cols, uint64_t group, uint8_t* codes, uint16_t* scales) {
  const uint64_t ng = cols / group;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < (int64_t)rows; ++r)
    for (uint64_t g = 0; g < ng; ++g) {
      const float* w = src + (uint64_t)r * cols + g * group;
      float amax = 0.f;
      for (uint64_t i = 0; i < group; ++i) amax = fmaxf(amax, fabsf(w[i]));
      uint16_t sb = amax > 0.f ? f32_to_bf16_bits(amax / 7.f) : (uint16_t)0x3F80;
      union { uint32_t u; float f; } sv; sv.u = (uint32_t)sb << 16;
      scales[(uint64_t)r * ng + g] = sb;
      uint8_t* out = codes + ((uint64_t)r * cols + g * group) / 2;
      for (uint64_t i = 0; i < group; i += 2) {
        int q0 = (int)rintf(w[i] / sv.f) + 8, q1 = (int)rintf(w[i + 1] / sv.f) + 8;
        q0 = q0 < 0 ? 0 : q0 > 15 ? 15 : q0;
        q1 = q1 < 0 ? 0 : q1 > 15 ? 15 : q1;
        out[i / 2] = (uint8_t)(q0 | (q1 << 4));
      }
    }
}

/* the bare mixing function, exported so that tests can check it against SplitMix64's published outputs */
uint64_t wwwsynth_mix(uint64_t z) { return mix(z); }

/* raw 64-bit words of the stream */
void wwwsynth_words(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, uint64_t* out) {
  uint64_t key = stream_key(seed, stream_id);
  for (uint64_t i = 0; i < n; ++i) out[i] = word(key, first + i);
}

/* integers uniform on [0, bound): high 32 bits of word scaled by bound (bound < 2^31) */
void wwwsynth_uniform_i32(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, uint32_t bound, int32_t* out) {
  uint64_t key = stream_key(seed, stream_id);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < (int64_t)n; ++i)
    out[i] = (int32_t)(((word(key, first + (uint64_t)i) >> 32) * (uint64_t)bound) >> 32);
}
