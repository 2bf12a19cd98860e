// Decode path (one new token per sequence): embedding, weight-streaming MFMA GEMMs with fused
// RMSNorm scale / rotary + KV-cache write / SwiGLU / residual epilogues, split-KV paged attention,
// argmax.  Activations travel between kernels as hi/lo fp16 pairs already laid out as MFMA B
// operands, so every GEMM's inner loop is loads and MFMAs only.
#include <stdlib.h>

#include <vector>

#include "common.h"

#define NEG_INF (-__builtin_inff())

__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }

// Cross-workgroup hand-over of partial results inside one kernel.  Partial tiles are written and read with
// device-scope (sc1) 16-byte accesses; every wavefront of the producer waits for its stores, the workgroup syncs, one
// thread bumps a device-scope counter (after a device-scope release fence when the splits of a tile are not known to
// share an L2); the workgroup that sees the last count reads the tiles back.  Only that one thread per workgroup
// fences: a device-scope fence in every wavefront (write-back of the whole L2) costs tens of microseconds per kernel.
// 16-byte accesses with device scope (cache-policy bit 4 = sc1 on gfx942/gfx950) through a raw buffer descriptor
__device__ __forceinline__ __amdgpu_buffer_rsrc_t shared_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
__device__ __forceinline__ void store_shared_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off, f32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, byte_off, 0, 16);
}
__device__ __forceinline__ f32x4 load_shared_f32x4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 16));
}
__device__ __forceinline__ void store_shared_f32(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float load_shared_f32(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// All of this wavefront's earlier vector memory operations have completed (stores: acknowledged by L2).  Written as the
// wait itself: a workgroup-scope release fence compiles to no vector-memory wait here (the wavefronts of a workgroup
// share one L1, so for ordering inside the workgroup none is needed), and then the partial-tile stores of a slow
// wavefront could still be on their way when the arrival counter moved: once in some ten thousand launches the last
// workgroup read the previous launch's values of a few cache lines.
__device__ __forceinline__ void wait_own_memory_ops() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
}

// offset (in elements) of column k of token t in a packed activation buffer with MT token groups
__device__ __forceinline__ int64_t packed_x_offset(int k, int t, int MT, int hl) {
  int kb = k >> 5, g = (k & 31) >> 3, e = k & 7;
  return ((((int64_t)kb * MT + (t >> 4)) * 2 + hl) * 64 + g * 16 + (t & 15)) * 8 + e;
}

// ------------------------------------------------------------------------------------------------
// Embedding gather: h = E[token]; sum of squares; packed (h * gain) for the first QKV GEMM.
template <typename ET>
__global__ __launch_bounds__(256) void embed_pack_kernel(const int32_t* __restrict__ tokens, const ET* __restrict__ embed, int d,
                                                          const float* __restrict__ gain, float* __restrict__ h,
                                                          float* __restrict__ ssq, uint16_t* __restrict__ xq, int MT) {
  int t = blockIdx.x;
  const ET* row = embed + (int64_t)tokens[t] * d;
  float local = 0.f;
  for (int o = threadIdx.x; o < d / 8; o += blockDim.x) {
    int k = o * 8;
    union { uint16_t s[8]; u32x4 v; } hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x;
      if constexpr (sizeof(ET) == 4) x = (float)row[k + e];
      else x = bf16_bits_to_float(((const uint16_t*)row)[k + e]);
      h[(int64_t)t * d + k + e] = x;
      local += x * x;
      split_f16(x * gain[k + e], hi.s[e], lo.s[e]);
    }
    *reinterpret_cast<u32x4*>(xq + packed_x_offset(k, t, MT, 0)) = hi.v;
    *reinterpret_cast<u32x4*>(xq + packed_x_offset(k, t, MT, 1)) = lo.v;
  }
  __shared__ float red[256];
  red[threadIdx.x] = local;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) ssq[(int64_t)t * SSQ_TILES] = red[0];  // row t of the [token][row tile] table; one entry in use
}

// ------------------------------------------------------------------------------------------------
// Skinny GEMM: Y^T[n][t] = sum_k W[n][k] X[t][k] for up to 64 tokens per workgroup pass.
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct GemmP {
  const u32x4* W;    // packed weights, 16-byte units (fp16 fragments, or FP8 codes of two k blocks)
  const u32x4* Wlo;  // low-order plane (fp32 sources) or null
  float wfactor;     // FP8 weights: the matrix's scale, applied to the result
  const u32x2* Wscale;  // int4 weights: four fp16 group scales per (chunk of 4 k blocks, row)
  int NRG, KB;       // row groups of 16, k blocks of 32
  const u32x4* X;    // packed activations
  int MT, M;         // token groups in X, valid tokens
  int kb_per_split, ksplit;
  int row_tiles, zbs;  // grid: 8 * ceil(row_tiles / 8) * ksplit * zbs workgroups
  int fence_handover;  // 1: workgroups of one row tile may sit behind different L2s
  float* partial;    // [ksplit][zbs][row_tiles] tiles of 128 rows x 64 tokens
  unsigned long long* counters;  // [zbs][row_tiles]: arrivals in bits 0-7, arrivals per XCD in eight 5-bit fields above
  int* fault_flag;   // host-visible; set when the splits of a row tile turn out to sit on different XCDs
  const float* ssq_in;  // [token][SSQ_TILES]; row scale = rsqrt(sum of the first n_ssq_in entries / dim + eps); null: no scale
  int n_ssq_in;
  float inv_dim, eps;
  // QKV epilogue
  uint16_t *q_hi, *q_lo;
  float qscale;
  uint16_t *kplane, *vplane;  // this layer's K and V planes of the pool (16-bit codes)
  float* kvscale;             // and its plane of scales
  const int32_t *seq_lens, *table;
  int mbs, hd, Hq, Hkv;
  const float2* rope;
  const float* qk_gain;  // models with normalised query / key heads: [2][hd] gains in packed row order; null otherwise
  // residual epilogue
  float* h;
  const float* gain_next;
  uint16_t* xnext;
  float* ssq_out;
  int d;
  // SwiGLU epilogue
  uint16_t* xa;
  int F;
  // logits epilogue
  float* logits;
  int V;
};

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

// 8 FP8 E4M3 codes (two 32-bit words, lowest byte first) -> 8 fp16 values, exact (|value| <= 448); the conversion
// instruction widens two codes at a time.
__device__ __forceinline__ f16x8 fp8x8_to_f16x8(uint32_t lo, uint32_t hi) {
  const f16x2 a = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lo, 1.0f, false), b = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(lo, 1.0f, true);
  const f16x2 c = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hi, 1.0f, false), d = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(hi, 1.0f, true);
  return __builtin_shufflevector(__builtin_shufflevector(a, b, 0, 1, 2, 3), __builtin_shufflevector(c, d, 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
}

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

// 8 four-bit codes (one 32-bit word, the code of column e in nibble e) -> 8 fp16 values (code - 8) * scale.  A code n
// is planted in the mantissa of the fp16 number 1024 (0x6400 | n = 1024 + n, exact), 1032 is subtracted and the result
// multiplied by the group's scale, two values per instruction; with a scale of 8 significant bits (bf16) the product
// is exact.
__device__ __forceinline__ f16x8 int4x8_to_f16x8(uint32_t w, f16x2 scale) {
  const uint32_t even = w & 0x0F0F0F0Fu, odd = (w >> 4) & 0x0F0F0F0Fu;  // codes of columns 0,2,4,6 / 1,3,5,7, one per byte
  const f16x2 off = {(_Float16)1032.f, (_Float16)1032.f};
  f16x2 v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // low half: byte i of `even`, high half: byte i of `odd`
    const uint32_t pair = __builtin_amdgcn_perm(odd, even, 0x0C040C00u + 0x00010001u * i) | 0x64006400u;
    v[i] = (__builtin_bit_cast(f16x2, pair) - off) * scale;
  }
  return __builtin_shufflevector(__builtin_shufflevector(v[0], v[1], 0, 1, 2, 3), __builtin_shufflevector(v[2], v[3], 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
}

// WMODE: 0 = fp16 weights; 1 = fp16 hi + lo planes (fp32 sources); 2 = FP8 codes, two k blocks per 16-byte unit, widened
// to fp16 in registers just before the MFMAs (the matrix's scale multiplies the result in the epilogue); 3 = int4 codes,
// four k blocks (one chunk) per 16-byte unit, widened and multiplied by their group's scale in registers
enum { WMODE_F16 = 0, WMODE_SPLIT = 1, WMODE_FP8 = 2, WMODE_INT4 = 3 };

// KH = 1: four wavefronts, each multiplies its two row groups with all four k blocks of a chunk.  KH = 2: eight
// wavefronts (two per SIMD); wavefront w and w + 4 own the same two row groups and take k blocks 0,1 / 2,3 of every
// chunk, so each issues half of the MFMAs and one can issue while its SIMD partner waits for memory; the two partial
// tiles are added through LDS behind the loop and wavefronts 4..7 retire.
template <int MTK, int WMODE, int EPI, int KH>
__global__ __launch_bounds__(256 * KH, 2 / KH) void skinny_gemm_kernel(const GemmP p) {
  constexpr bool WSPLIT = WMODE == WMODE_SPLIT, W8 = WMODE == WMODE_FP8, W4 = WMODE == WMODE_INT4;
  constexpr int R = 2, KC = 4, WP = WSPLIT ? 2 : 1;
  constexpr int NT = 256 * KH;                     // threads
  constexpr int KPW = KC / KH;                     // k blocks of a chunk per wavefront
  static_assert(KH == 1 || (KH == 2 && !W4), "the int4 unit spans the whole chunk");
  constexpr int CHUNK_UNITS = KC * MTK * 128;      // 16-byte units of activations per k chunk
  constexpr int NSTG = (CHUNK_UNITS + NT - 1) / NT;
  __shared__ u32x4 lds[2][CHUNK_UNITS];
  __shared__ float s_scale[64];
  // after the main loop the staging buffers are dead and are reused for the epilogue's small reductions
  float(*red)[64] = reinterpret_cast<float(*)[64]>(&lds[0][0]);
  volatile int* s_last = reinterpret_cast<volatile int*>(&lds[1][0]);

  const int tid = threadIdx.x, wave = (tid >> 6) & 3, khalf = KH == 1 ? 0 : tid >> 8, lane = tid & 63;
  const int k_first = khalf * KPW;                 // first k block of a chunk this wavefront multiplies
  // Workgroup id -> work item.  Consecutive workgroup ids are dealt round-robin to the XCDs (8 here; any power of two
  // up to 8 divides 8), so ids that are equal modulo 8 run behind the same L2.  All k splits of a row tile get such
  // ids: id = c + 8 * ((zb * tiles_per_xcd + lt) * ksplit + split) for row tile c + 8 * lt.  Their partial tiles then
  // meet in one L2 and the split-K hand-over needs no L2 write-back.  The host checks this placement rule with a probe
  // kernel when a model is loaded and sets fence_handover when it does not hold.
  const int tiles_per_xcd = (p.row_tiles + 7) / 8;
  const int slot = blockIdx.x >> 3;
  const int split = slot % p.ksplit;
  const int lt = (slot / p.ksplit) % tiles_per_xcd, zb = slot / (p.ksplit * tiles_per_xcd);
  const int tile = (blockIdx.x & 7) + 8 * lt;
  if (tile >= p.row_tiles) return;  // grid padding when the row tiles are not a multiple of 8
  const int tb0 = zb * 4;
  const int rg0 = tile * 8 + wave * R;
  const int kb_begin = split * p.kb_per_split;
  const int kb_end = min(p.KB, kb_begin + p.kb_per_split);
  const int nchunks = (kb_end - kb_begin + KC - 1) / KC;

  int rgc[R];  // clamped row group (loads stay in bounds; stores are masked)
#pragma unroll
  for (int r = 0; r < R; ++r) rgc[r] = min(rg0 + r, p.NRG - 1);

  f32x4 acc[R][MTK];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb) acc[r][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Inputs of the epilogue that hang off dependent loads (RMSNorm scale; position and KV block of each token) are
  // requested at kernel entry together with the first weights and activations, and only touched once that first chunk
  // has arrived, so they never put a memory round trip in front of the streaming loop.
  // Sum of squares of a token: wavefront w owns token group w (every workgroup of the grid reads the same small table,
  // so each reads it once, not once per wavefront).  Lane group g = lane/16 reads entries 16g .. 16g+15 of the token's
  // row (four 16-byte loads, always in bounds; entries past n_ssq_in are masked), adds them in index order, and the
  // four groups are combined by two cross-lane exchanges: a fixed order, so the scale is the same in every workgroup.
  f32x4 ssq_raw[4];
  int pos_pre[MTK];
  int tok_c[MTK];
#pragma unroll
  for (int tb = 0; tb < MTK; ++tb) {
    tok_c[tb] = min((tb0 + tb) * 16 + (lane & 15), p.M - 1);
    pos_pre[tb] = 0;
    if constexpr (EPI == EPI_QKV) pos_pre[tb] = p.seq_lens[tok_c[tb]] - 1;
  }
  if (p.ssq_in && wave < MTK && khalf == 0) {
    const int t = min((tb0 + wave) * 16 + (lane & 15), p.M - 1);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      ssq_raw[c] = *reinterpret_cast<const f32x4*>(p.ssq_in + (int64_t)t * SSQ_TILES + (lane >> 4) * 16 + c * 4);
  }
  float scale_pre[MTK];
  int blk_pre[MTK];
  // before the first barrier: reduce the sums and publish the scales; table loads for the KV slots go out
  auto finish_prefetch = [&]() __attribute__((always_inline)) {
    if (p.ssq_in && wave < MTK && khalf == 0) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) s += ((lane >> 4) * 16 + c * 4 + e < p.n_ssq_in) ? ssq_raw[c][e] : 0.f;
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (lane < 16) s_scale[wave * 16 + lane] = rsqrtf(s * p.inv_dim + p.eps);
    }
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb) {
      blk_pre[tb] = 0;
      if constexpr (EPI == EPI_QKV) blk_pre[tb] = kv_block_id(p.table + (int64_t)tok_c[tb] * p.mbs, pos_pre[tb]);
    }
  };
  // after that barrier
  auto read_scales = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb) {
      scale_pre[tb] = p.ssq_in ? s_scale[tb * 16 + (lane & 15)] : 1.f;
      if constexpr (W8) scale_pre[tb] *= p.wfactor;
    }
  };

  u32x4 wA[KC][R][WP], wB[KC][R][WP], stg[NSTG];

  // Loads past the end of this split's k range are redirected to its last valid block (in bounds) and the
  // matching MFMAs are skipped in compute(): no per-element selects in the streaming loop.
  auto load_w = [&](u32x4(&w)[KC][R][WP], int c) {
    if constexpr (W4) {
      // one 16-byte unit carries the whole chunk (entry 0 of the set); entry 1 takes the four group scales (8 bytes)
      const int chunk = min((kb_begin + c * KC) >> 2, (kb_end - 1) >> 2);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        w[0][r][0] = p.W[((int64_t)chunk * p.NRG + rgc[r]) * 64 + lane];
        const u32x2 sc = p.Wscale[((int64_t)chunk * p.NRG + rgc[r]) * 16 + (lane & 15)];
        w[1][r][0] = u32x4{sc.x, sc.y, 0u, 0u};
      }
      return;
    }
    if constexpr (W8) {
      // one 16-byte unit carries two k blocks: entries 0 and 2 of the set hold the chunk's two units, 1 and 3 stay unused
      // (kb_begin is a multiple of 4, so a chunk starts on a pair)
#pragma unroll
      for (int j = 0; j < KPW; j += 2) {
        const int pair = min((kb_begin + c * KC + k_first + j) >> 1, (kb_end - 1) >> 1);
#pragma unroll
        for (int r = 0; r < R; ++r) w[j][r][0] = p.W[((int64_t)pair * p.NRG + rgc[r]) * 64 + lane];
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < KPW; ++j) {  // register slot j holds k block k_first + j of the chunk
      const int kbc = min(kb_begin + c * KC + k_first + j, kb_end - 1);
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int64_t idx = ((int64_t)kbc * p.NRG + rgc[r]) * 64 + lane;
        w[j][r][0] = p.W[idx];
        if constexpr (WSPLIT) w[j][r][1] = p.Wlo[idx];
      }
    }
  };
  auto load_stage = [&](int c) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NSTG; ++i) {
      const int u = min(tid + i * NT, CHUNK_UNITS - 1);  // (more threads than units when MTK = 1 and KH = 2)
      const int kk = u / (MTK * 128), within = u % (MTK * 128);
      const int kbc = min(kb_begin + c * KC + kk, kb_end - 1);
      stg[i] = p.X[((int64_t)kbc * p.MT + tb0) * 128 + within];
    }
  };
  auto store_stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NSTG; ++i) lds[buf][min(tid + i * NT, CHUNK_UNITS - 1)] = stg[i];
  };
  // nvalid = k blocks of the chunk that lie inside the range: KC for every chunk but possibly the last.
  // The B fragments (activations) of k block kk+1 are fetched from LDS while the MFMAs of k block kk run.
  auto compute = [&](u32x4(&w)[KC][R][WP], int buf, int nvalid) __attribute__((always_inline)) {
    u32x4 bq[2][MTK][2];
    auto fetch = [&](int set, int kk) __attribute__((always_inline)) {
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        bq[set][tb][0] = lds[buf][(kk * MTK + tb) * 128 + lane];
        bq[set][tb][1] = lds[buf][(kk * MTK + tb) * 128 + 64 + lane];
      }
    };
    fetch(0, k_first);
#pragma unroll
    for (int j = 0; j < KPW; ++j) {  // k block k_first + j of the chunk, operands in register slot j
      if (k_first + j >= nvalid) break;
      if (j + 1 < KPW) fetch((j + 1) & 1, k_first + j + 1);
      __builtin_amdgcn_sched_barrier(0);
      f16x8 a8[R];
      if constexpr (W8) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const u32x4 raw = w[j & ~1][r][0];
          a8[r] = (j & 1) ? fp8x8_to_f16x8(raw.z, raw.w) : fp8x8_to_f16x8(raw.x, raw.y);
        }
      }
      if constexpr (W4) {  // (KH = 1: j is the k block)
#pragma unroll
        for (int r = 0; r < R; ++r) {
          const u32x4 raw = w[0][r][0], sc = w[1][r][0];
          const uint32_t word = j == 0 ? raw.x : j == 1 ? raw.y : j == 2 ? raw.z : raw.w;
          const uint32_t s2 = j < 2 ? sc.x : sc.y;
          const uint32_t s16 = (j & 1) ? (s2 >> 16) : (s2 & 0xFFFFu);
          a8[r] = int4x8_to_f16x8(word, __builtin_bit_cast(f16x2, s16 | (s16 << 16)));
        }
      }
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        const f16x8 bhi = as_f16x8(bq[j & 1][tb][0]), blo = as_f16x8(bq[j & 1][tb][1]);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          f16x8 a;
          if constexpr (W8 || W4) a = a8[r];
          else a = as_f16x8(w[j][r][0]);
          acc[r][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bhi, acc[r][tb], 0, 0, 0);
          acc[r][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, blo, acc[r][tb], 0, 0, 0);
          if constexpr (WSPLIT) acc[r][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(w[j][r][1]), bhi, acc[r][tb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // Software pipeline: while chunk c is multiplied out of LDS buffer c&1 and register set A/B, chunk c+1 is
  // already on its way from HBM.  The steady-state loop has no conditional loads, so the new loads can stay
  // in flight across the MFMAs of the current chunk; the last one or two chunks are peeled.
  if (nchunks > 0) {
    const int last_valid = (kb_end - kb_begin) - (nchunks - 1) * KC;  // k blocks in the final chunk
    load_stage(0);
    load_w(wA, 0);
    __builtin_amdgcn_sched_barrier(0);
    store_stage(0);
    finish_prefetch();
    __syncthreads();
    read_scales();
    int c = 0;
    for (; c + 2 < nchunks; c += 2) {
      load_stage(c + 1);
      load_w(wB, c + 1);
      __builtin_amdgcn_sched_barrier(0);  // keep the prefetch in front of the MFMAs it overlaps with
      compute(wA, 0, KC);
      __builtin_amdgcn_sched_barrier(0);
      store_stage(1);
      __syncthreads();
      load_stage(c + 2);
      load_w(wA, c + 2);
      __builtin_amdgcn_sched_barrier(0);
      compute(wB, 1, KC);
      __builtin_amdgcn_sched_barrier(0);
      store_stage(0);
      __syncthreads();
    }
    if (c + 1 < nchunks) {
      load_stage(c + 1);
      load_w(wB, c + 1);
      __builtin_amdgcn_sched_barrier(0);
      compute(wA, 0, KC);
      __builtin_amdgcn_sched_barrier(0);
      store_stage(1);
      __syncthreads();
      compute(wB, 1, last_valid);
    } else {
      compute(wA, 0, last_valid);
    }
    __syncthreads();
  } else {
    finish_prefetch();
    __syncthreads();
    read_scales();
  }

  if constexpr (KH == 2) {
    // the staging buffers are dead: wavefronts 4..7 hand their partial tile to wavefronts 0..3 (same rows) and retire;
    // the barriers further down then only count the wavefronts that are left
    u32x4* xch = &lds[0][0];  // [wavefront 0..3][r][tb][lane]
    if (khalf == 1) {
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int tb = 0; tb < MTK; ++tb) xch[((wave * R + r) * MTK + tb) * 64 + lane] = __builtin_bit_cast(u32x4, acc[r][tb]);
    }
    __syncthreads();
    if (khalf == 1) return;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) acc[r][tb] += __builtin_bit_cast(f32x4, xch[((wave * R + r) * MTK + tb) * 64 + lane]);
    __syncthreads();  // `red` and `s_last` below reuse the same LDS
  }

  // accumulator layout: acc[r][tb][i] = Y^T[row][token], row = (rg0+r)*16 + (lane/16)*4 + i, token = (tb0+tb)*16 + lane%16
  const int rsub = (lane >> 4) * 4;
  const int tsub = lane & 15;

  // Operands of the epilogue that live in memory (residual stream and next norm's gain; rotary factors) are requested
  // before the split-K partial tiles, so the last workgroup pays one memory round trip for everything it needs.
  // Addresses are clamped into range; values of invalid rows / tokens are never used.
  f32x4 hv_pre[R][MTK], gv_pre[R], cs_pre[R][MTK];
  auto request_epilogue_inputs = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int n0 = rgc[r] * 16 + rsub;
      if constexpr (EPI == EPI_RESID) gv_pre[r] = *reinterpret_cast<const f32x4*>(p.gain_next + n0);
      if constexpr (EPI == EPI_QKV) {  // gains of the head normalisation (value rows read the key gains and ignore them)
        if (p.qk_gain) gv_pre[r] = *reinterpret_cast<const f32x4*>(p.qk_gain + (n0 / p.hd < p.Hq ? 0 : p.hd) + n0 % p.hd);
      }
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        if constexpr (EPI == EPI_RESID) hv_pre[r][tb] = *reinterpret_cast<const f32x4*>(p.h + (int64_t)tok_c[tb] * p.d + n0);
        if constexpr (EPI == EPI_QKV)
          cs_pre[r][tb] = *reinterpret_cast<const f32x4*>(p.rope + (int64_t)pos_pre[tb] * (p.hd / 2) + ((n0 % p.hd) >> 1));
      }
    }
  };

  if (p.ksplit <= 1) request_epilogue_inputs();
  if (p.ksplit > 1) {
    // split-K: park the partial tile, and let the workgroup that arrives last add all partial tiles in split order
    // parked as a register image: unit ((((split, zb, tile), wave), r), tb), lane -> one 16-byte store per lane,
    // 1 KiB contiguous per instruction; the last workgroup reads it back with the same thread mapping
    const __amdgpu_buffer_rsrc_t prs = shared_rsrc(p.partial);
    auto punit = [&](int sp, int r, int tb) __attribute__((always_inline)) {
      return (uint32_t)((((((sp * p.zbs + zb) * p.row_tiles + tile) * 4 + wave) * R + r) * MTK + tb) * 64 + lane) * 16u;
    };
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) store_shared_f32x4(prs, punit(split, r, tb), acc[r][tb]);
    wait_own_memory_ops();
    __syncthreads();
    if (tid == 0) {
      // Conservative path for partial tiles that may have to cross to another XCD: a device-scope release (L2
      // write-back) before the counter moves.  The barrier above orders every wavefront's completed stores before
      // this thread's fence.
      if (p.fence_handover) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      // the counter also records on which XCD each split ran, so that the last workgroup can tell whether the
      // placement rule held for this tile (the unfenced hand-over is only sound if it did)
      const unsigned xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u;  // HW_REG_XCC_ID
      const unsigned long long mine = 1ull + (xcc < 8 ? 1ull << (8 + 5 * xcc) : 0ull);
      const unsigned long long old = __hip_atomic_fetch_add(&p.counters[zb * p.row_tiles + tile], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const bool last = (int)(old & 0xff) == p.ksplit - 1;
      *s_last = last;
      if (last && !p.fence_handover) {
        const unsigned same = xcc < 8 ? (unsigned)(((old + mine) >> (8 + 5 * xcc)) & 31u) : 0u;
        if ((int)same != p.ksplit) *p.fault_flag = 1;
      }
    }
    __syncthreads();
    if (!*s_last) return;
    // the fenced hand-over's other half: the partial tiles may come from another L2, so everything this workgroup has
    // cached is dropped before they are read (acquire side of the producers' release fences)
    if (p.fence_handover) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    if (tid == 0) __hip_atomic_store(&p.counters[zb * p.row_tiles + tile], 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    request_epilogue_inputs();
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) acc[r][tb] = f32x4{0.f, 0.f, 0.f, 0.f};
    // partial tiles are added in split order (reproducible); loads are issued four splits at a time so that
    // the reduction is not one memory round trip per split
    for (int s0 = 0; s0 < p.ksplit; s0 += 4) {
      f32x4 pv[4][R][MTK];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int sidx = min(s0 + u, p.ksplit - 1);
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int tb = 0; tb < MTK; ++tb) pv[u][r][tb] = load_shared_f32x4(prs, punit(sidx, r, tb));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (s0 + u >= p.ksplit) break;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int tb = 0; tb < MTK; ++tb) acc[r][tb] += pv[u][r][tb];
      }
    }
  }

  float ssq_local[MTK];
#pragma unroll
  for (int tb = 0; tb < MTK; ++tb) ssq_local[tb] = 0.f;

  // Normalised query / key heads: 1 / rms of each token's head vector.  A row tile holds whole heads (128 rows: one head
  // of 128, or two of 64 owned by wavefronts 0,1 and 2,3); a wavefront adds the squares of its 32 rows per token (lanes,
  // then two cross-lane exchanges) and the wavefronts of a head are added through LDS in index order.  Row groups past
  // the end of the matrix only ever fall into a head that does not exist.
  float head_rs[MTK];
  if constexpr (EPI == EPI_QKV) {
    if (p.qk_gain) {
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        float s = 0.f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float v = acc[r][tb][i] * scale_pre[tb];
            s += v * v;
          }
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (lane < 16) red[wave][tb * 16 + lane] = s;
      }
      __syncthreads();
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        const int at = tb * 16 + tsub;
        const float tot = p.hd == 128 ? (red[0][at] + red[1][at]) + (red[2][at] + red[3][at]) : red[wave & 2][at] + red[(wave & 2) + 1][at];
        head_rs[tb] = rsqrtf(tot / (float)p.hd + p.eps);
      }
    }
  }

  // QKV: finish the values in place (RMSNorm factor, head normalisation, rotation), then take, per token, the largest
  // magnitude of every head's vector (lanes, two cross-lane exchanges, the head's wavefronts through LDS): the scale of
  // the key / value codes.  (Query heads get one too and ignore it.)
  float head_amax[MTK];
  if constexpr (EPI == EPI_QKV) {
    const int rot_rows = (p.Hq + p.Hkv) * p.hd;
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb) {
      float am = 0.f;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int n0 = (rg0 + r) * 16 + rsub;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = acc[r][tb][i] * scale_pre[tb];
        if (n0 < rot_rows) {
          if (p.qk_gain) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] *= head_rs[tb] * gv_pre[r][i];
          }
          // rows arrive with the rotary pair (i, i + hd/2) at neighbouring positions (2i, 2i+1)
#pragma unroll
          for (int pr = 0; pr < 2; ++pr) {
            const float cs_x = cs_pre[r][tb][2 * pr], cs_y = cs_pre[r][tb][2 * pr + 1];
            float a = v[2 * pr], b = v[2 * pr + 1];
            v[2 * pr] = a * cs_x - b * cs_y;
            v[2 * pr + 1] = b * cs_x + a * cs_y;
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          acc[r][tb][i] = v[i];
          am = fmaxf(am, __builtin_fabsf(v[i]));  // (a NaN element is dropped by fmaxf; its code is 0)
        }
      }
      am = fmaxf(am, __shfl_xor(am, 16));
      am = fmaxf(am, __shfl_xor(am, 32));
      head_amax[tb] = am;
    }
    if (p.qk_gain) __syncthreads();  // `red` may still be read by the head normalisation above
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb)
      if (lane < 16) red[wave][tb * 16 + lane] = head_amax[tb];
    __syncthreads();
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb) {
      const int at = tb * 16 + tsub;
      head_amax[tb] = p.hd == 128 ? fmaxf(fmaxf(red[0][at], red[1][at]), fmaxf(red[2][at], red[3][at]))
                                  : fmaxf(red[wave & 2][at], red[(wave & 2) + 1][at]);
    }
  }

#pragma unroll
  for (int tb = 0; tb < MTK; ++tb) {
    const int t = (tb0 + tb) * 16 + tsub;
    const bool tok_ok = t < p.M;
    const float scale = scale_pre[tb];

    if constexpr (EPI == EPI_SWIGLU) {
      if (tok_ok && rg0 + 1 < p.NRG) {
        int f0 = (rg0 >> 1) * 16 + rsub;
        union { uint16_t s[4]; u32x2 v; } hi, lo;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float g = acc[0][tb][i] * scale, u = acc[1][tb][i] * scale;
          float a = g / (1.f + __expf(-g)) * u;
          split_f16(a, hi.s[i], lo.s[i]);
        }
        *reinterpret_cast<u32x2*>(p.xa + packed_x_offset(f0, t, p.MT, 0)) = hi.v;
        *reinterpret_cast<u32x2*>(p.xa + packed_x_offset(f0, t, p.MT, 1)) = lo.v;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (!tok_ok || rg0 + r >= p.NRG) continue;
        const int n0 = (rg0 + r) * 16 + rsub;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = acc[r][tb][i] * scale;  // (QKV: overwritten below, the values are already final)

        if constexpr (EPI == EPI_LOGITS) {
          *reinterpret_cast<float4*>(p.logits + (int64_t)t * p.V + n0) = make_float4(v[0], v[1], v[2], v[3]);
        } else if constexpr (EPI == EPI_RESID) {
          const f32x4 hv = hv_pre[r][tb], gv = gv_pre[r];
          float hn[4] = {hv[0] + v[0], hv[1] + v[1], hv[2] + v[2], hv[3] + v[3]};
          float gn[4] = {gv[0], gv[1], gv[2], gv[3]};
          *reinterpret_cast<float4*>(p.h + (int64_t)t * p.d + n0) = make_float4(hn[0], hn[1], hn[2], hn[3]);
          union { uint16_t s[4]; u32x2 v; } hi, lo;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            ssq_local[tb] += hn[i] * hn[i];
            split_f16(hn[i] * gn[i], hi.s[i], lo.s[i]);
          }
          *reinterpret_cast<u32x2*>(p.xnext + packed_x_offset(n0, t, p.MT, 0)) = hi.v;
          *reinterpret_cast<u32x2*>(p.xnext + packed_x_offset(n0, t, p.MT, 1)) = lo.v;
        } else {  // EPI_QKV: the values were finished (scaled, normalised, rotated) in place above
          const int head = n0 / p.hd, c0 = n0 % p.hd;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = acc[r][tb][i];
          if (head < p.Hq) {
            // queries leave as fp16 hi + lo, already multiplied by log2(e)/sqrt(hd), in the order the attention kernel loads them
            union { uint16_t s[4]; u32x2 v; } qh, ql;
#pragma unroll
            for (int i = 0; i < 4; ++i) split_f16(v[i] * p.qscale, qh.s[i], ql.s[i]);
            *reinterpret_cast<u32x2*>(p.q_hi + (int64_t)t * (p.Hq * p.hd) + n0) = qh.v;
            *reinterpret_cast<u32x2*>(p.q_lo + (int64_t)t * (p.Hq * p.hd) + n0) = ql.v;
          } else {
            // keys and values go to the cache as 16-bit codes with the scale of their (token, head) vector
            const int64_t slot = kv_slot_in_block(blk_pre[tb], pos_pre[tb]);
            const int64_t blk = slot / KV_BS;
            const int tok = (int)(slot % KV_BS);
            const bool is_v = head >= p.Hq + p.Hkv;
            const int j = head - p.Hq - (is_v ? p.Hkv : 0);
            const float inv = kv_code_inv(head_amax[tb]);
            union { uint16_t s[4]; u32x2 v; } code;
#pragma unroll
            for (int i = 0; i < 4; ++i) code.s[i] = kv_code(v[i], inv);
            if (!is_v) {
              *reinterpret_cast<u32x2*>(p.kplane + (blk * p.Hkv + j) * (int64_t)(KV_BS * p.hd) + k_cache_offset(tok, c0)) = code.v;
            } else {
              uint16_t* dst = p.vplane + (blk * p.Hkv + j) * (int64_t)(KV_BS * p.hd);
#pragma unroll
              for (int i = 0; i < 4; ++i) dst[v_cache_offset(tok, c0 + i)] = code.s[i];
            }
            if (c0 == 0 && rsub == 0)  // one lane per (token, head): first row of the head
              p.kvscale[kv_scale_offset(blk, p.Hkv, j) + (is_v ? 16 : 0) + tok] = kv_code_scale(head_amax[tb]);
          }
        }
      }
    }
  }

  if constexpr (EPI == EPI_RESID) {
    // per (row tile, token) sum of squares of the new residual, reduced in a fixed order
#pragma unroll
    for (int tb = 0; tb < MTK; ++tb) {
      float s = ssq_local[tb];
      s += __shfl_xor(s, 16);
      s += __shfl_xor(s, 32);
      if (lane < 16) red[wave][tb * 16 + lane] = s;
    }
    __syncthreads();
    if (tid < MTK * 16) {
      int t = tb0 * 16 + tid;
      if (t < p.M) p.ssq_out[(int64_t)t * SSQ_TILES + tile] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Plan of the decode attention, built once per step and used by every layer.
//
// The keys of the batch are counted in pairs of 16-key blocks.  All (sequence b, kv head j, pair) triples, in that
// order, form one long list of T = Hkv * sum_b P_b entries (P_b = pairs of sequence b); the attention kernel runs W
// wavefronts and wavefront w takes the entries [w*C, (w+1)*C), C = max(16, ceil(T / W)).  Every wavefront therefore
// streams the same number of bytes and all of them finish together, whatever the mix of sequence lengths.  A chunk may
// end inside a (b, j) sequence and continue into the next one; each piece is a segment with its own softmax state,
// parked as a record and merged afterwards (a sequence of P pairs is cut into at most P/C + 2 <= P/16 + 2 segments).
// The cut points depend on the lengths of all sequences of the batch: results are reproducible for a given batch
// but the rounding of a sequence's attention output may differ between batches of different composition.
//   hdr[0] = T, hdr[1] = C;  start[w] = (b, j, first pair) of wavefront w, b = -1 if it has no work;
//   pref[b] = sum of P over the sequences before b
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t* __restrict__ seq_lens, int batch, int Hkv, int W,
                                                        int32_t* __restrict__ hdr, int32_t* __restrict__ start,
                                                        int32_t* __restrict__ pref_out) {
  extern __shared__ int pref[];  // [batch + 1]
  const int tid = threadIdx.x, lane = tid & 63;
  if (tid < 64) {
    int carry = 0;
    if (lane == 0) pref[0] = 0;
    for (int c = 0; c < batch; c += 64) {
      const int bb = c + lane;
      const int P = bb < batch ? max(0, (seq_lens[bb] + 31) / 32) : 0;
      int inc = P;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(inc, o);
        if (lane >= o) inc += up;
      }
      if (bb < batch) pref[bb + 1] = carry + inc;
      carry += __shfl(inc, 63);
    }
  }
  __syncthreads();
  const int T = pref[batch] * Hkv;
  const int C = max(16, (T + W - 1) / W);
  if (tid == 0) { hdr[0] = T; hdr[1] = C; }
  for (int i = tid; i <= batch; i += 256) pref_out[i] = pref[i];
  for (int w = tid; w < W; w += 256) {
    const int64_t x0 = (int64_t)w * C;
    int sb = -1, sj = 0, sp = 0;
    if (x0 < T) {
      int lo = 0, hi = batch - 1;  // largest b with Hkv * pref[b] <= x0
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)pref[mid] * Hkv <= x0) lo = mid; else hi = mid - 1;
      }
      const int P = max(1, pref[lo + 1] - pref[lo]);  // (never 0 for the sequence that holds entry x0 < T)
      const int r = (int)(x0 - (int64_t)pref[lo] * Hkv);
      sb = lo; sj = r / P; sp = r % P;
    }
    start[4 * w] = sb; start[4 * w + 1] = sj; start[4 * w + 2] = sp; start[4 * w + 3] = 0;
  }
}

// Two 16-bit codes (one 32-bit word, offset binary u = x + 32768) as two pairs of fp16 numbers a, b with x = 256 a + b,
// a in [-128, 127], b in [0, 255] - both exact in fp16, so the matrix cores multiply the codes without losing a bit.
// The high and low bytes of u are planted in the mantissa of the fp16 number 1024 (0x6400 | n = 1024 + n) and
// 1024 + 128, resp. 1024, is subtracted, two values per instruction.
__device__ __forceinline__ void split_codes(uint32_t u, uint32_t& hi, uint32_t& lo) {
  const f16x2 off_hi = {(_Float16)1152.f, (_Float16)1152.f}, off_lo = {(_Float16)1024.f, (_Float16)1024.f};
  const uint32_t ph = __builtin_amdgcn_perm(0x64646464u, u, 0x04030401u);  // bytes: u.b1, 0x64, u.b3, 0x64
  const uint32_t pl = __builtin_amdgcn_perm(0x64646464u, u, 0x04020400u);  // bytes: u.b0, 0x64, u.b2, 0x64
  hi = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, ph) - off_hi);
  lo = __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, pl) - off_lo);
}
__device__ __forceinline__ void split_codes4(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t w3, f16x8& hi, f16x8& lo) {
  uint32_t h0, h1, h2, h3, l0, l1, l2, l3;
  split_codes(w0, h0, l0);
  split_codes(w1, h1, l1);
  split_codes(w2, h2, l2);
  split_codes(w3, h3, l3);
  hi = as_f16x8(u32x4{h0, h1, h2, h3});
  lo = as_f16x8(u32x4{l0, l1, l2, l3});
}
__device__ __forceinline__ void split_codes8(u32x4 w, f16x8& hi, f16x8& lo) { split_codes4(w.x, w.y, w.z, w.w, hi, lo); }

// ------------------------------------------------------------------------------------------------
// Decode attention.  Each wavefront walks its chunk of the plan above, segment by segment:
//   S^T = K Q^T (keys x heads), online softmax per head along the key axis with cross-lane shuffles,
//   O^T = V^T P^T (head_dim x heads).  The G query heads of the group share every K/V byte.
// A segment that covers its whole (sequence, kv head) writes the packed hi/lo operand of the O projection itself;
// otherwise it parks (m, l, unnormalised o) as record number (w - first wavefront of that sequence).
template <int HD, int G>
__global__ __launch_bounds__(256) void decode_attn_kernel(const uint16_t* __restrict__ q_hi, const uint16_t* __restrict__ q_lo,
                                                           const uint16_t* __restrict__ kplane,
                                                           const uint16_t* __restrict__ vplane, const float* __restrict__ kvscale,
                                                           const int32_t* __restrict__ seq_lens,
                                                           const int32_t* __restrict__ table, int batch, int mbs, int Hq, int Hkv,
                                                           const int32_t* __restrict__ hdr, const int32_t* __restrict__ start,
                                                           int maxrec, float* __restrict__ part, uint16_t* __restrict__ xo, int MT) {
  constexpr int NKF = HD / 32;  // K fragments per block
  constexpr int NVF = HD / 16;  // V fragments per block
  constexpr int PSTRIDE = HD + 4;  // floats per (record, head): o[HD], m, l, pad
  const int w = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int n = lane & 15, g = lane >> 4;
  const int T = hdr[0], C = hdr[1];
  int b = __builtin_amdgcn_readfirstlane(start[4 * w]);
  if (b < 0) return;
  int j = __builtin_amdgcn_readfirstlane(start[4 * w + 1]);
  int p = __builtin_amdgcn_readfirstlane(start[4 * w + 2]);
  int x = w * C;                      // position in the list of the next entry
  int remaining = min(C, T - x);
  const int64_t blk_elems = (int64_t)KV_BS * HD;

  while (remaining > 0 && b < batch) {  // (the second test only guards against a plan that does not match the lengths)
    const int ctx = __builtin_amdgcn_readfirstlane(seq_lens[b]);
    const int P = (ctx + 31) / 32;
    if (P <= 0) {  // an empty sequence has no entries in the list
      ++b;
      continue;
    }
    const int np = min(P - p, remaining);
    const int kend = min(ctx, (p + np) * 32);
    const int32_t* trow = table + (int64_t)b * mbs;
    // Q^T operand: lane (head n, group g) holds dims f*32 + g*8 .. +7 of head n, as fp16 hi + lo (pre-scaled by the producer)
    f16x8 qhi[NKF], qlo[NKF];
    {
      const int64_t qoff = ((int64_t)b * Hq + j * G + min(n, G - 1)) * HD + g * 8;
#pragma unroll
      for (int f = 0; f < NKF; ++f) {
        u32x4 h = *reinterpret_cast<const u32x4*>(q_hi + qoff + f * 32);
        u32x4 l = *reinterpret_cast<const u32x4*>(q_lo + qoff + f * 32);
        if (n >= G) { h = u32x4{0, 0, 0, 0}; l = u32x4{0, 0, 0, 0}; }
        qhi[f] = as_f16x8(h);
        qlo[f] = as_f16x8(l);
      }
    }
    f32x4 oacc[NVF];
#pragma unroll
    for (int f = 0; f < NVF; ++f) oacc[f] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = NEG_INF, l_run = 0.f;
    // The value scales ride on the probabilities (fp16 operands of the second product).  To keep those operands in
    // fp16's normal range whatever the magnitude of the model's values, they are multiplied by a power of two taken
    // from the first key's scale (2^-4 / 2^exponent, so p * scale * vnorm is about p / 16) and the accumulator is
    // divided by it at the end of the segment.  Scales more than 2^11 times the first one would saturate.
    float vnorm = 0.f, vnorm_inv = 0.f;

    // the segment in runs of at most 32 pairs = 64 blocks, whose ids are held one per lane
    for (int sp = 0; sp < np; sp += 32) {
      const int npairs = min(32, np - sp);
      const int k0 = (p + sp) * 32;
      const int blk0 = k0 / KV_BS;
      const int my_blk = trow[min(blk0 + lane, mbs - 1)];
      const int last_blk_local = min(63, (kend - 1) / KV_BS - blk0);  // index, within this run, of its last valid block

      struct KV {
        u32x4 k0[NKF], k1[NKF];
        u32x2 v0[NVF], v1[NVF];
        f32x4 ks0, ks1, vs0, vs1;  // scales of this lane's keys 4g .. 4g+3 of the two blocks
      };
      auto load_pair = [&](KV& r, int pr) __attribute__((always_inline)) {
        const int id0 = __shfl(my_blk, min(2 * pr, last_blk_local));
        const int id1 = __shfl(my_blk, min(2 * pr + 1, last_blk_local));  // past the end: the last block again (masked)
        const int64_t off0 = ((int64_t)id0 * Hkv + j) * blk_elems;
        const int64_t off1 = ((int64_t)id1 * Hkv + j) * blk_elems;
        const float* sc0 = kvscale + kv_scale_offset(id0, Hkv, j) + 4 * g;
        const float* sc1 = kvscale + kv_scale_offset(id1, Hkv, j) + 4 * g;
        r.ks0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(sc0));
        r.vs0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(sc0 + 16));
        r.ks1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(sc1));
        r.vs1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(sc1 + 16));
#pragma unroll
        for (int f = 0; f < NKF; ++f) {
          r.k0[f] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kplane + off0 + (f * 64 + lane) * 8));
          r.k1[f] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kplane + off1 + (f * 64 + lane) * 8));
        }
#pragma unroll
        for (int f = 0; f < NVF; ++f) {
          r.v0[f] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vplane + off0 + (f * 64 + lane) * 4));
          r.v1[f] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(vplane + off1 + (f * 64 + lane) * 4));
        }
      };
      auto process = [&](KV& r, int pr) __attribute__((always_inline)) {
        const int base = k0 + pr * 32;
        // scores (already in log2 units): lane (head n, g) gets keys base + 4g + i (block 0) and base + 16 + 4g + i (block 1).
        // Codes x = 256 a + b: the a plane meets both query planes, the b plane the hi plane (b q_lo is below 2^-19 of the score).
        f32x4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = {0.f, 0.f, 0.f, 0.f}, b0 = {0.f, 0.f, 0.f, 0.f}, b1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int f = 0; f < NKF; ++f) {
          f16x8 ka, kb;
          split_codes8(r.k0[f], ka, kb);
          a0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qhi[f], a0, 0, 0, 0);
          a0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qlo[f], a0, 0, 0, 0);
          b0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb, qhi[f], b0, 0, 0, 0);
          split_codes8(r.k1[f], ka, kb);
          a1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qhi[f], a1, 0, 0, 0);
          a1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qlo[f], a1, 0, 0, 0);
          b1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb, qhi[f], b1, 0, 0, 0);
        }
        if (vnorm == 0.f) {  // first pair of the segment: its first key is valid, its scale sets the normaliser
          const uint32_t bits = __builtin_amdgcn_readfirstlane(__float_as_uint(r.vs0[0]));
          int e = (int)((bits >> 23) & 0xffu);
          e = e < 8 ? 114 : min(e, 240);  // an all-zero first value vector: take 2^-13; (NaN / inf: anything finite)
          vnorm = __uint_as_float((uint32_t)(250 - e) << 23);           // 2^(123 - e): scale * vnorm lies in [1/16, 1/8)
          vnorm_inv = __uint_as_float((uint32_t)(e + 4) << 23);         // 2^(e - 123)
        }
        float sc[8], pvs[8];
        float mx = NEG_INF;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool ok0 = base + 4 * g + i < kend, ok1 = base + 16 + 4 * g + i < kend;
          sc[i] = ok0 ? (a0[i] * 256.f + b0[i]) * r.ks0[i] : NEG_INF;
          sc[4 + i] = ok1 ? (a1[i] * 256.f + b1[i]) * r.ks1[i] : NEG_INF;
          pvs[i] = ok0 ? r.vs0[i] * vnorm : 0.f;      // slots past the end may hold anything: their scale never enters
          pvs[4 + i] = ok1 ? r.vs1[i] * vnorm : 0.f;
          mx = fmaxf(mx, fmaxf(sc[i], sc[4 + i]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        // the probabilities times the value scales go to the matrix cores as fp16 hi + lo, like every other operand of the
        // single-token path (for the a plane of the value codes with the factor 256; the b plane, 2^-8 of the value, takes
        // the hi part alone); non-negative, so one bound keeps a wild scale from overflowing
        union { _Float16 s[8]; f16x8 v; } pa, pl, pb;
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float pv = __builtin_amdgcn_exp2f(sc[i] - m_new);
          psum += pv;
          const float w = fminf(pv * pvs[i], 255.f), w256 = w * 256.f;
          pa.s[i] = (_Float16)w256;
          pl.s[i] = (_Float16)(w256 - (float)pa.s[i]);
          pb.s[i] = (_Float16)w;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__any(alpha != 1.f)) {  // the running maximum moved for some head of the wavefront (rare after the first pairs)
#pragma unroll
          for (int f = 0; f < NVF; ++f) {
            oacc[f][0] *= alpha; oacc[f][1] *= alpha; oacc[f][2] *= alpha; oacc[f][3] *= alpha;
          }
        }
#pragma unroll
        for (int f = 0; f < NVF; ++f) {
          f16x8 va, vb;
          split_codes4(r.v0[f].x, r.v0[f].y, r.v1[f].x, r.v1[f].y, va, vb);
          oacc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pa.v, oacc[f], 0, 0, 0);
          oacc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, pl.v, oacc[f], 0, 0, 0);
          oacc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vb, pb.v, oacc[f], 0, 0, 0);
        }
      };

      // two register sets: the keys and values of pair pr+1 travel while pair pr is processed
      KV ra, rb;
      load_pair(ra, 0);
      int pr = 0;
      bool done = false;
      while (pr + 1 < npairs) {
        load_pair(rb, pr + 1);
        __builtin_amdgcn_sched_barrier(0);
        process(ra, pr);
        ++pr;
        if (pr + 1 >= npairs) {
          process(rb, pr);
          done = true;
          break;
        }
        load_pair(ra, pr + 1);
        __builtin_amdgcn_sched_barrier(0);
        process(rb, pr);
        ++pr;
      }
      if (!done) process(ra, pr);
    }

    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
#pragma unroll
    for (int f = 0; f < NVF; ++f) {
      oacc[f][0] *= vnorm_inv; oacc[f][1] *= vnorm_inv; oacc[f][2] *= vnorm_inv; oacc[f][3] *= vnorm_inv;
    }

    const int S = x - p;                // list position of this (b, j) sequence's first pair
    const int first_w = S / C;
    const int nrec = (S + P - 1) / C - first_w + 1;
    if (nrec == 1) {
      // this segment is the whole sequence: normalise and emit the packed O-projection operand directly
      if (n < G) {
        const float inv = 1.f / l_run;
#pragma unroll
        for (int f = 0; f < NVF; ++f) {
          union { uint16_t s[4]; u32x2 v; } hi, lo;
#pragma unroll
          for (int i = 0; i < 4; ++i) split_f16(oacc[f][i] * inv, hi.s[i], lo.s[i]);
          const int k = (j * G + n) * HD + f * 16 + g * 4;
          *reinterpret_cast<u32x2*>(xo + packed_x_offset(k, b, MT, 0)) = hi.v;
          *reinterpret_cast<u32x2*>(xo + packed_x_offset(k, b, MT, 1)) = lo.v;
        }
      }
    } else {
      // park the record [b][j][w - first_w][head n][o(HD), m, l]; a separate small kernel merges the records (a kernel
      // boundary is a far cheaper hand-over here than in-kernel device-scope signalling)
      float* rec = part + ((((int64_t)b * Hkv + j) * maxrec + (w - first_w)) * G) * PSTRIDE;
      if (n < G) {
#pragma unroll
        for (int f = 0; f < NVF; ++f)
          *reinterpret_cast<float4*>(rec + n * PSTRIDE + f * 16 + g * 4) = make_float4(oacc[f][0], oacc[f][1], oacc[f][2], oacc[f][3]);
        if (g == 0) {
          rec[n * PSTRIDE + HD] = m_run;
          rec[n * PSTRIDE + HD + 1] = l_run;
        }
      }
    }
    x += np;
    remaining -= np;
    p = 0;
    if (++j == Hkv) { j = 0; ++b; }
  }
}

// Merges the records of one (sequence, kv head) in key order and writes the packed hi/lo operand of the O
// projection.  One wavefront per (kv head, sequence); sequences that were a single segment were finished by the
// attention kernel itself.
template <int HD, int G>
__global__ __launch_bounds__(64) void decode_attn_merge_kernel(const int32_t* __restrict__ seq_lens, int Hkv,
                                                                const int32_t* __restrict__ hdr, const int32_t* __restrict__ pref,
                                                                int nsplit_max, const float* __restrict__ part,
                                                                uint16_t* __restrict__ xo, int MT) {
  constexpr int PSTRIDE = HD + 4;
  const int j = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const int C = hdr[1];
  const int P = max(0, (seq_lens[b] + 31) / 32);
  const int S = pref[b] * Hkv + j * P;  // list position of this sequence's first pair
  const int nsplit_act = (S + P - 1) / C - S / C + 1;
  if (nsplit_act <= 1) return;
  // Lane owns head-dim elements lane + 64*i of every head; records are read four splits at a time so the merge is
  // not one memory round trip per split.
  const float* recs = part + (((int64_t)b * Hkv + j) * nsplit_max) * G * PSTRIDE;
  constexpr int NE = HD / 64;
  float Mh[G], Lh[G], oh[G][NE];
#pragma unroll
  for (int hh = 0; hh < G; ++hh) {
    Mh[hh] = NEG_INF;
    Lh[hh] = 0.f;
#pragma unroll
    for (int i = 0; i < NE; ++i) oh[hh][i] = 0.f;
  }
  for (int s0 = 0; s0 < nsplit_act; s0 += 4) {
    float mv[4][G], lv[4][G], ov[4][G][NE];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int sidx = min(s0 + u, nsplit_act - 1);
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        const float* r = recs + ((int64_t)sidx * G + hh) * PSTRIDE;
        mv[u][hh] = r[HD];
        lv[u][hh] = r[HD + 1];
#pragma unroll
        for (int i = 0; i < NE; ++i) ov[u][hh][i] = r[lane + 64 * i];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (s0 + u >= nsplit_act) break;
#pragma unroll
      for (int hh = 0; hh < G; ++hh) {
        const float Mn = fmaxf(Mh[hh], mv[u][hh]);
        const float a = __builtin_amdgcn_exp2f(Mh[hh] - Mn), w = __builtin_amdgcn_exp2f(mv[u][hh] - Mn);
        Lh[hh] = Lh[hh] * a + lv[u][hh] * w;
#pragma unroll
        for (int i = 0; i < NE; ++i) oh[hh][i] = oh[hh][i] * a + ov[u][hh][i] * w;
        Mh[hh] = Mn;
      }
    }
  }
#pragma unroll
  for (int hh = 0; hh < G; ++hh) {
    const float inv = 1.f / Lh[hh];
#pragma unroll
    for (int i = 0; i < NE; ++i) {
      const int k = (j * G + hh) * HD + lane + 64 * i;
      uint16_t hi, lo;
      split_f16(oh[hh][i] * inv, hi, lo);
      xo[packed_x_offset(k, b, MT, 0)] = hi;
      xo[packed_x_offset(k, b, MT, 1)] = lo;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Greedy next token: index of the largest logit, the lowest index winning ties.  Two stages: ARGMAX_CHUNKS
// workgroups per row each scan a contiguous slice with 16-byte loads, then one wavefront per row combines them.
#define ARGMAX_CHUNKS 32
__device__ __forceinline__ void argmax_take(float& best, int& bi, float v, int i) {
  if (v > best || (v == best && i < bi)) { best = v; bi = i; }
}
__global__ __launch_bounds__(256) void argmax_partial_kernel(const float* __restrict__ logits, int V, float* __restrict__ pval,
                                                             int* __restrict__ pidx) {
  const float* row = logits + (int64_t)blockIdx.y * V;
  const int nq = V / 4, per = (nq + ARGMAX_CHUNKS - 1) / ARGMAX_CHUNKS;
  const int q0 = blockIdx.x * per, q1 = min(nq, q0 + per);
  float best = NEG_INF;
  int bi = 0x7fffffff;
  for (int q = q0 + threadIdx.x; q < q1; q += 256) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(row + 4 * q);
#pragma unroll
    for (int e = 0; e < 4; ++e) argmax_take(best, bi, v[e], 4 * q + e);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) argmax_take(best, bi, __shfl_xor(best, o), __shfl_xor(bi, o));
  __shared__ float sv[4];
  __shared__ int si[4];
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = best; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < 4; ++w) argmax_take(best, bi, sv[w], si[w]);
    pval[blockIdx.y * ARGMAX_CHUNKS + blockIdx.x] = best;
    pidx[blockIdx.y * ARGMAX_CHUNKS + blockIdx.x] = bi;
  }
}
__global__ __launch_bounds__(64) void argmax_final_kernel(const float* __restrict__ pval, const int* __restrict__ pidx,
                                                          int32_t* __restrict__ out) {
  const int lane = threadIdx.x;
  float best = lane < ARGMAX_CHUNKS ? pval[blockIdx.x * ARGMAX_CHUNKS + lane] : NEG_INF;
  int bi = lane < ARGMAX_CHUNKS ? pidx[blockIdx.x * ARGMAX_CHUNKS + lane] : 0x7fffffff;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) argmax_take(best, bi, __shfl_xor(best, o), __shfl_xor(bi, o));
  // a row without any ordered value (all NaN) has no largest element: token 0, never an index outside the vocabulary
  if (lane == 0) out[blockIdx.x] = bi == 0x7fffffff ? 0 : bi;
}

// ------------------------------------------------------------------------------------------------
// Host side

// Workgroups a skinny GEMM should spread over (split-K is used when the row tiles alone are fewer): one per compute
// unit, so that no compute unit carries two of a kernel's workgroups while others carry one.  Tunable through the
// environment variable WWW_GEMM_WG_TARGET, read once.
static int wg_target() {
  static int v = 0;
  if (!v) {
    const char* e = getenv("WWW_GEMM_WG_TARGET");
    if (e) {
      v = atoi(e);
    } else {
      int dev = 0, cus = 0;
      if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess) v = cus;
      else (void)hipGetLastError();
      if (v < 1) v = 256;
    }
    if (v < 1) v = 1;
  }
  return v;
}

static void choose_split(int row_tiles, int zb, int KB, int* ksplit, int* kb_per_split) {
  int want = wg_target() / (row_tiles * zb);
  if (want < 1) want = 1;
  if (want > MAX_KSPLIT) want = MAX_KSPLIT;
  int per = (KB + want - 1) / want;
  per = (per + 3) / 4 * 4;
  if (per < 8) per = 8;  // at least two k chunks per workgroup, so the load pipeline has something to overlap
  *kb_per_split = per;
  *ksplit = (KB + per - 1) / per;
}

// split factor the decode path will use for a GEMM with NRG row groups and KB k blocks (for workspace sizing)
int decode_gemm_ksplit(int NRG, int KB, int MT) {
  int zb = MT > 4 ? MT / 4 : 1, ks, per;
  choose_split((NRG + 7) / 8, zb, KB, &ks, &per);
  return ks;
}

template <int EPI>
static void launch_gemm(www_model* m, GemmP& p, int MT, hipStream_t st) {
  const int row_tiles = (p.NRG + 7) / 8;
  const int zb = MT > 4 ? MT / 4 : 1;
  const int mtk = MT > 4 ? 4 : MT;
  choose_split(row_tiles, zb, p.KB, &p.ksplit, &p.kb_per_split);
  p.MT = MT;
  p.partial = m->partial;
  p.counters = m->counters;
  p.fault_flag = m->fault_dev;
  p.row_tiles = row_tiles;
  p.zbs = zb;
  p.fence_handover = m->handover_fence;
  if (p.wfactor == 0.f) p.wfactor = 1.f;  // not set: an unscaled matrix
  dim3 grid(8 * ((row_tiles + 7) / 8) * p.ksplit * zb);
#define LAUNCH(MTK_, WM_, KH_) hipLaunchKernelGGL((skinny_gemm_kernel<MTK_, WM_, EPI, KH_>), grid, dim3(256 * KH_), 0, st, p);
  // With more than 32 tokens the MFMAs of a chunk take a third of a wavefront's time; in the gate/up GEMM (no split-K,
  // 32 chunks per workgroup) two wavefronts per SIMD (KH = 2) hide them behind each other's waits: 53 -> 49.5 us at 64
  // tokens of the 8B shape.  The split-K GEMMs walk 4 - 14 chunks and are bound by their fixed costs; the hand-over
  // between the wavefront halves costs them as much as it saves, so they stay at KH = 1.
  constexpr int kh4 = EPI == EPI_SWIGLU ? 2 : 1;
  if (m->int4_group) {
    if (mtk == 1) LAUNCH(1, WMODE_INT4, 1) else if (mtk == 2) LAUNCH(2, WMODE_INT4, 1) else LAUNCH(4, WMODE_INT4, 1)
  } else if (m->fp8) {
    if (mtk == 1) LAUNCH(1, WMODE_FP8, 1) else if (mtk == 2) LAUNCH(2, WMODE_FP8, 1) else LAUNCH(4, WMODE_FP8, kh4)
  } else if (m->wsplit) {
    if (mtk == 1) LAUNCH(1, WMODE_SPLIT, 1) else if (mtk == 2) LAUNCH(2, WMODE_SPLIT, 1) else LAUNCH(4, WMODE_SPLIT, 1)
  } else {
    if (mtk == 1) LAUNCH(1, WMODE_F16, 1) else if (mtk == 2) LAUNCH(2, WMODE_F16, 1) else LAUNCH(4, WMODE_F16, kh4)
  }
#undef LAUNCH
}

// wavefronts the decode attention kernel keeps resident on the whole device (its grid), a multiple of 4
int decode_attn_resident_waves(int hd, int G) {
  int dev = 0, cus = 0, per_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    (void)hipGetLastError();
    return 1024;
  }
  hipError_t e = hipErrorInvalidValue;
#define OCC(HD_, G_) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_attn_kernel<HD_, G_>, 256, 0)
  if (hd == 128) {
    if (G == 1) OCC(128, 1); else if (G == 2) OCC(128, 2); else if (G == 4) OCC(128, 4); else OCC(128, 8);
  } else {
    if (G == 1) OCC(64, 1); else if (G == 2) OCC(64, 2); else if (G == 4) OCC(64, 4); else OCC(64, 8);
  }
#undef OCC
  if (e != hipSuccess || per_cu < 1) { (void)hipGetLastError(); per_cu = 1; }
  return per_cu * cus * 4;
}

// Placement probe: every workgroup records the id of the XCD it runs on.
__global__ __launch_bounds__(256) void xcc_probe_kernel(int32_t* __restrict__ out) {
  const int xcc = __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15;  // HW_REG_XCC_ID, bits 3:0
  if (threadIdx.x == 0) out[blockIdx.x] = xcc;
}

// 1 if workgroups whose ids are equal modulo 8 were all placed on the same XCD in a probe launch of n workgroups
// (scratch_dev: n ints of device memory), 0 if not, -1 on a HIP error.
int decode_probe_placement(int32_t* scratch_dev, int n, hipStream_t st) {
  std::vector<int32_t> h(n);
  hipLaunchKernelGGL(xcc_probe_kernel, dim3(n), dim3(256), 0, st, scratch_dev);
  if (hipMemcpyAsync(h.data(), scratch_dev, (size_t)n * 4, hipMemcpyDeviceToHost, st) != hipSuccess) return -1;
  if (hipStreamSynchronize(st) != hipSuccess) return -1;
  for (int i = 8; i < n; ++i)
    if (h[i] != h[i & 7]) return 0;
  return 1;
}

int decode_MT(int batch) { return batch <= 16 ? 1 : batch <= 32 ? 2 : ((batch + 63) / 64) * 4; }

int run_decode(www_model* m, const int32_t* tok, const int32_t* lens, const int32_t* table, int batch, float* logits, int32_t* next,
               hipStream_t st) {
  const int MT = decode_MT(batch);
  const int d = m->d;
  prof_mark(m, PK_EMBED, st);
  if (m->cfg.weight_dtype == WWW_DTYPE_F32)
    hipLaunchKernelGGL(embed_pack_kernel<float>, dim3(batch), dim3(256), 0, st, tok, (const float*)m->embed, d, m->layers[0].attn_norm,
                       m->h, m->ssq, (uint16_t*)m->xq, MT);
  else
    hipLaunchKernelGGL(embed_pack_kernel<uint16_t>, dim3(batch), dim3(256), 0, st, tok, (const uint16_t*)m->embed, d,
                       m->layers[0].attn_norm, m->h, m->ssq, (uint16_t*)m->xq, MT);
  hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(256), (size_t)(batch + 1) * 4, st, lens, batch, m->Hkv, m->attn_waves, m->attn_hdr,
                     m->attn_start, m->attn_pref);
  int n_ssq = 1;
  const float qscale = 1.4426950408889634f / sqrtf((float)m->hd);
  for (int l = 0; l < m->L; ++l) {
    const LayerW& w = m->layers[l];
    uint16_t* kplane = (uint16_t*)m->kv + (int64_t)(2 * l) * m->kv_plane;
    uint16_t* vplane = (uint16_t*)m->kv + (int64_t)(2 * l + 1) * m->kv_plane;
    float* kvscale = m->kv_scales + (int64_t)l * m->kv_scale_plane;
    {
      GemmP p = {};
      p.W = (const u32x4*)(w.wqkv8 ? (const void*)w.wqkv8 : (const void*)w.wqkv); p.Wlo = (const u32x4*)w.wqkv_lo; p.wfactor = w.sqkv; p.Wscale = (const u32x2*)w.gqkv;
      p.NRG = m->QKVN / 16; p.KB = d / 32;
      p.X = (const u32x4*)m->xq; p.M = batch;
      p.ssq_in = m->ssq; p.n_ssq_in = n_ssq; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
      p.q_hi = m->q_hi; p.q_lo = m->q_lo; p.qscale = qscale; p.kplane = kplane; p.vplane = vplane; p.kvscale = kvscale; p.seq_lens = lens; p.table = table; p.mbs = m->cfg.max_blocks_per_seq;
      p.hd = m->hd; p.Hq = m->Hq; p.Hkv = m->Hkv; p.rope = m->rope; p.qk_gain = w.qk_gain;
      prof_mark(m, PK_QKV, st);
      launch_gemm<EPI_QKV>(m, p, MT, st);
    }
    {
      prof_mark(m, PK_ATTN, st);
#define ATTN(HD_, G_)                                                                                                              \
  {                                                                                                                                \
    hipLaunchKernelGGL((decode_attn_kernel<HD_, G_>), dim3(m->attn_waves / 4), dim3(256), 0, st, m->q_hi, m->q_lo, kplane, vplane,  \
                       kvscale, lens, table, batch, (int)m->cfg.max_blocks_per_seq, m->Hq, m->Hkv, m->attn_hdr, m->attn_start,            \
                       m->attn_maxrec,                                                                                             \
                       m->attn_part, (uint16_t*)m->xo, MT);                                                                        \
    hipLaunchKernelGGL((decode_attn_merge_kernel<HD_, G_>), dim3(m->Hkv, batch), dim3(64), 0, st, lens, m->Hkv, m->attn_hdr,        \
                       m->attn_pref, m->attn_maxrec, m->attn_part, (uint16_t*)m->xo, MT);                                          \
  }
      if (m->hd == 128) {
        if (m->G == 1) ATTN(128, 1) else if (m->G == 2) ATTN(128, 2) else if (m->G == 4) ATTN(128, 4) else ATTN(128, 8)
      } else {
        if (m->G == 1) ATTN(64, 1) else if (m->G == 2) ATTN(64, 2) else if (m->G == 4) ATTN(64, 4) else ATTN(64, 8)
      }
#undef ATTN
    }
    {
      GemmP p = {};
      p.W = (const u32x4*)(w.wo8 ? (const void*)w.wo8 : (const void*)w.wo); p.Wlo = (const u32x4*)w.wo_lo; p.wfactor = w.so; p.Wscale = (const u32x2*)w.go;
      p.NRG = d / 16; p.KB = m->QD / 32;
      p.X = (const u32x4*)m->xo; p.M = batch;
      p.h = m->h; p.gain_next = w.ffn_norm; p.xnext = (uint16_t*)m->xq; p.ssq_out = m->ssq; p.d = d;
      prof_mark(m, PK_OPROJ, st);
      launch_gemm<EPI_RESID>(m, p, MT, st);
      n_ssq = (d / 16 + 7) / 8;
    }
    {
      GemmP p = {};
      p.W = (const u32x4*)(w.wgu8 ? (const void*)w.wgu8 : (const void*)w.wgu); p.Wlo = (const u32x4*)w.wgu_lo; p.wfactor = w.sgu; p.Wscale = (const u32x2*)w.ggu;
      p.NRG = 2 * m->F / 16; p.KB = d / 32;
      p.X = (const u32x4*)m->xq; p.M = batch;
      p.ssq_in = m->ssq; p.n_ssq_in = n_ssq; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
      p.xa = (uint16_t*)m->xa; p.F = m->F;
      prof_mark(m, PK_GATEUP, st);
      launch_gemm<EPI_SWIGLU>(m, p, MT, st);
    }
    {
      GemmP p = {};
      p.W = (const u32x4*)(w.wd8 ? (const void*)w.wd8 : (const void*)w.wd); p.Wlo = (const u32x4*)w.wd_lo; p.wfactor = w.sd; p.Wscale = (const u32x2*)w.gd;
      p.NRG = d / 16; p.KB = m->Fp / 32;
      p.X = (const u32x4*)m->xa; p.M = batch;
      p.h = m->h; p.gain_next = (l + 1 < m->L) ? m->layers[l + 1].attn_norm : m->final_norm;
      p.xnext = (uint16_t*)m->xq; p.ssq_out = m->ssq; p.d = d;
      prof_mark(m, PK_DOWN, st);
      launch_gemm<EPI_RESID>(m, p, MT, st);
    }
  }
  float* lg = logits ? logits : m->logits_buf;
  {
    GemmP p = {};
    p.W = (const u32x4*)(m->lm_head8 ? (const void*)m->lm_head8 : (const void*)m->lm_head); p.Wlo = (const u32x4*)m->lm_head_lo; p.wfactor = m->s_lm; p.Wscale = (const u32x2*)m->g_lm;
    p.NRG = m->V / 16; p.KB = d / 32;
    p.X = (const u32x4*)m->xq; p.M = batch;
    p.ssq_in = m->ssq; p.n_ssq_in = n_ssq; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
    p.logits = lg; p.V = m->V;
    prof_mark(m, PK_LMHEAD, st);
    launch_gemm<EPI_LOGITS>(m, p, MT, st);
  }
  if (next) prof_mark(m, PK_ARGMAX, st);
  if (next) {
    hipLaunchKernelGGL(argmax_partial_kernel, dim3(ARGMAX_CHUNKS, batch), dim3(256), 0, st, lg, m->V, m->argmax_val, m->argmax_idx);
    hipLaunchKernelGGL(argmax_final_kernel, dim3(batch), dim3(64), 0, st, m->argmax_val, m->argmax_idx, next);
  }
  prof_mark(m, -1, st);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("decode launch failed: %s", hipGetErrorString(e));
    return WWW_E_HIP;
  }
  return WWW_OK;
}
