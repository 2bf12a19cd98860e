// Decode path (one new token per sequence): embedding, weight-streaming MFMA GEMMs with fused
// RMSNorm scale / rotary + KV-cache write / SwiGLU / residual epilogues, split-KV paged attention,
// argmax.  Activations travel between kernels as hi/lo fp16 pairs already laid out as MFMA B
// operands, so every GEMM's inner loop is loads and MFMAs only.
#include "common.h"

#define NEG_INF (-__builtin_inff())

__device__ __forceinline__ f16x8 as_f16x8(uint4 v) { return __builtin_bit_cast(f16x8, v); }

__device__ __forceinline__ float rstd_of(const float* __restrict__ ssq, int n_tiles, int stride, int t, float inv_dim, float eps) {
  float s = 0.f;
  for (int i = 0; i < n_tiles; ++i) s += ssq[i * stride + t];  // fixed order: reproducible
  return rsqrtf(s * inv_dim + eps);
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
    union { uint16_t s[8]; uint4 v; } hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x;
      if constexpr (sizeof(ET) == 4) x = (float)row[k + e];
      else x = bf16_bits_to_float(((const uint16_t*)row)[k + e]);
      h[(int64_t)t * d + k + e] = x;
      local += x * x;
      split_f16(x * gain[k + e], hi.s[e], lo.s[e]);
    }
    *reinterpret_cast<uint4*>(xq + packed_x_offset(k, t, MT, 0)) = hi.v;
    *reinterpret_cast<uint4*>(xq + packed_x_offset(k, t, MT, 1)) = lo.v;
  }
  __shared__ float red[256];
  red[threadIdx.x] = local;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) ssq[t] = red[0];
}

// ------------------------------------------------------------------------------------------------
// Skinny GEMM: Y^T[n][t] = sum_k W[n][k] X[t][k] for up to 64 tokens per workgroup pass.
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LOGITS = 3 };

struct GemmP {
  const uint4* W;    // packed weights, 16-byte units
  const uint4* Wlo;  // low-order plane (fp32 sources) or null
  int NRG, KB;       // row groups of 16, k blocks of 32
  const uint4* X;    // packed activations
  int MT, M;         // token groups in X, valid tokens
  int kb_per_split, ksplit;
  float* partial;    // [ksplit][MT*16][NRG*16]
  int* counters;     // [gridDim.z][gridDim.x]
  const float* ssq_in;  // row scale = rsqrt(sum(ssq_in)/dim + eps), or null for no scale
  int n_ssq_in, ssq_stride;
  float inv_dim, eps;
  // QKV epilogue
  float* q;
  uint16_t *kplane, *vplane;  // this layer's K and V planes of the pool
  const int32_t *seq_lens, *table;
  int mbs, hd, Hq, Hkv;
  const float2* rope;
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

template <int MTK, bool WSPLIT, int EPI>
__global__ __launch_bounds__(256, 2) void skinny_gemm_kernel(const GemmP p) {
  constexpr int R = 2, KC = 4, WP = WSPLIT ? 2 : 1;
  constexpr int CHUNK_UNITS = KC * MTK * 128;      // 16-byte units of activations per k chunk
  constexpr int NSTG = CHUNK_UNITS / 256;
  __shared__ uint4 lds[2][CHUNK_UNITS];
  // after the main loop the staging buffers are dead and are reused for the epilogue's small reductions
  float(*red)[64] = reinterpret_cast<float(*)[64]>(&lds[0][0]);
  volatile int* s_last = reinterpret_cast<volatile int*>(&lds[1][0]);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int tile = blockIdx.x, split = blockIdx.y, zb = blockIdx.z;
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

  uint4 wA[KC][R][WP], wB[KC][R][WP], stg[NSTG];
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  auto load_w = [&](uint4(&w)[KC][R][WP], int c) {
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
      int kb = kb_begin + c * KC + kk;
      bool ok = kb < kb_end;
      int kbc = ok ? kb : kb_end - 1;
#pragma unroll
      for (int r = 0; r < R; ++r) {
        int64_t idx = ((int64_t)rgc[r] * p.KB + kbc) * 64 + lane;
        uint4 v = p.W[idx];
        w[kk][r][0] = ok ? v : zero4;
        if constexpr (WSPLIT) {
          uint4 v2 = p.Wlo[idx];
          w[kk][r][1] = ok ? v2 : zero4;
        }
      }
    }
  };
  auto load_stage = [&](int c) {
#pragma unroll
    for (int i = 0; i < NSTG; ++i) {
      int u = tid + i * 256;
      int kk = u / (MTK * 128), within = u % (MTK * 128);
      int kb = kb_begin + c * KC + kk;
      bool ok = kb < kb_end;
      int kbc = ok ? kb : kb_end - 1;
      uint4 v = p.X[((int64_t)kbc * p.MT + tb0) * 128 + within];
      stg[i] = ok ? v : zero4;
    }
  };
  auto store_stage = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NSTG; ++i) lds[buf][tid + i * 256] = stg[i];
  };
  auto compute = [&](uint4(&w)[KC][R][WP], int buf) {
#pragma unroll
    for (int kk = 0; kk < KC; ++kk) {
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        f16x8 bhi = as_f16x8(lds[buf][(kk * MTK + tb) * 128 + lane]);
        f16x8 blo = as_f16x8(lds[buf][(kk * MTK + tb) * 128 + 64 + lane]);
#pragma unroll
        for (int r = 0; r < R; ++r) {
          f16x8 a = as_f16x8(w[kk][r][0]);
          acc[r][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bhi, acc[r][tb], 0, 0, 0);
          acc[r][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, blo, acc[r][tb], 0, 0, 0);
          if constexpr (WSPLIT) acc[r][tb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(w[kk][r][1]), bhi, acc[r][tb], 0, 0, 0);
        }
      }
    }
  };

  if (nchunks > 0) {
    load_stage(0);
    load_w(wA, 0);
    store_stage(0);
    __syncthreads();
    for (int c = 0; c < nchunks; c += 2) {
      bool has1 = c + 1 < nchunks;
      if (has1) { load_stage(c + 1); load_w(wB, c + 1); }
      compute(wA, 0);
      if (has1) store_stage(1);
      __syncthreads();
      if (!has1) break;
      bool has2 = c + 2 < nchunks;
      if (has2) { load_stage(c + 2); load_w(wA, c + 2); }
      compute(wB, 1);
      if (has2) store_stage(0);
      __syncthreads();
    }
  }

  // accumulator layout: acc[r][tb][i] = Y^T[row][token], row = (rg0+r)*16 + (lane/16)*4 + i, token = (tb0+tb)*16 + lane%16
  const int Npad = p.NRG * 16;
  const int rsub = (lane >> 4) * 4;
  const int tsub = lane & 15;

  if (p.ksplit > 1) {
    // split-K: park the partial tile, and let the workgroup that arrives last add all partial tiles in split order
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (rg0 + r >= p.NRG) continue;
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        int t = (tb0 + tb) * 16 + tsub;
        float4 v = make_float4(acc[r][tb][0], acc[r][tb][1], acc[r][tb][2], acc[r][tb][3]);
        *reinterpret_cast<float4*>(p.partial + ((int64_t)split * (p.MT * 16) + t) * Npad + (rg0 + r) * 16 + rsub) = v;
      }
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      int old = atomicAdd(&p.counters[zb * gridDim.x + tile], 1);
      *s_last = (old == p.ksplit - 1);
    }
    __syncthreads();
    if (!*s_last) return;
    __threadfence();
    if (tid == 0) p.counters[zb * gridDim.x + tile] = 0;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int tb = 0; tb < MTK; ++tb) {
        acc[r][tb] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (rg0 + r >= p.NRG) continue;
        int t = (tb0 + tb) * 16 + tsub;
        for (int s = 0; s < p.ksplit; ++s) {
          float4 v = *reinterpret_cast<const float4*>(p.partial + ((int64_t)s * (p.MT * 16) + t) * Npad + (rg0 + r) * 16 + rsub);
          acc[r][tb][0] += v.x; acc[r][tb][1] += v.y; acc[r][tb][2] += v.z; acc[r][tb][3] += v.w;
        }
      }
  }

  float ssq_local[MTK];
#pragma unroll
  for (int tb = 0; tb < MTK; ++tb) ssq_local[tb] = 0.f;

#pragma unroll
  for (int tb = 0; tb < MTK; ++tb) {
    const int t = (tb0 + tb) * 16 + tsub;
    const bool tok_ok = t < p.M;
    float scale = 1.f;
    if (p.ssq_in && tok_ok) scale = rstd_of(p.ssq_in, p.n_ssq_in, p.ssq_stride, t, p.inv_dim, p.eps);

    if constexpr (EPI == EPI_SWIGLU) {
      if (tok_ok && rg0 + 1 < p.NRG) {
        int f0 = (rg0 >> 1) * 16 + rsub;
        union { uint16_t s[4]; uint2 v; } hi, lo;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float g = acc[0][tb][i] * scale, u = acc[1][tb][i] * scale;
          float a = g / (1.f + __expf(-g)) * u;
          split_f16(a, hi.s[i], lo.s[i]);
        }
        *reinterpret_cast<uint2*>(p.xa + packed_x_offset(f0, t, p.MT, 0)) = hi.v;
        *reinterpret_cast<uint2*>(p.xa + packed_x_offset(f0, t, p.MT, 1)) = lo.v;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (!tok_ok || rg0 + r >= p.NRG) continue;
        const int n0 = (rg0 + r) * 16 + rsub;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = acc[r][tb][i] * scale;

        if constexpr (EPI == EPI_LOGITS) {
          *reinterpret_cast<float4*>(p.logits + (int64_t)t * p.V + n0) = make_float4(v[0], v[1], v[2], v[3]);
        } else if constexpr (EPI == EPI_RESID) {
          float4 hv = *reinterpret_cast<const float4*>(p.h + (int64_t)t * p.d + n0);
          float4 gv = *reinterpret_cast<const float4*>(p.gain_next + n0);
          float hn[4] = {hv.x + v[0], hv.y + v[1], hv.z + v[2], hv.w + v[3]};
          float gn[4] = {gv.x, gv.y, gv.z, gv.w};
          *reinterpret_cast<float4*>(p.h + (int64_t)t * p.d + n0) = make_float4(hn[0], hn[1], hn[2], hn[3]);
          union { uint16_t s[4]; uint2 v; } hi, lo;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            ssq_local[tb] += hn[i] * hn[i];
            split_f16(hn[i] * gn[i], hi.s[i], lo.s[i]);
          }
          *reinterpret_cast<uint2*>(p.xnext + packed_x_offset(n0, t, p.MT, 0)) = hi.v;
          *reinterpret_cast<uint2*>(p.xnext + packed_x_offset(n0, t, p.MT, 1)) = lo.v;
        } else {  // EPI_QKV
          const int pos = p.seq_lens[t] - 1;
          const int rot_rows = (p.Hq + p.Hkv) * p.hd;
          const int head = n0 / p.hd, c0 = n0 % p.hd;
          if (n0 < rot_rows) {
            // rows arrive with the rotary pair (i, i + hd/2) at neighbouring positions (2i, 2i+1)
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
              float2 cs = p.rope[(int64_t)pos * (p.hd / 2) + (c0 >> 1) + pr];
              float a = v[2 * pr], b = v[2 * pr + 1];
              v[2 * pr] = a * cs.x - b * cs.y;
              v[2 * pr + 1] = b * cs.x + a * cs.y;
            }
          }
          if (head < p.Hq) {
            *reinterpret_cast<float4*>(p.q + (int64_t)t * (p.Hq * p.hd) + n0) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            const int64_t slot = kv_slot(p.table + (int64_t)t * p.mbs, pos);
            const int64_t blk = slot / KV_BS;
            const int tok = (int)(slot % KV_BS);
            if (head < p.Hq + p.Hkv) {
              const int j = head - p.Hq;
              union { uint16_t s[4]; uint2 v; } kb16;
#pragma unroll
              for (int i = 0; i < 4; ++i) kb16.s[i] = f32_to_f16_sat(v[i]);
              *reinterpret_cast<uint2*>(p.kplane + (blk * p.Hkv + j) * (int64_t)(KV_BS * p.hd) + k_cache_offset(tok, c0)) = kb16.v;
            } else {
              const int j = head - p.Hq - p.Hkv;
              uint16_t* dst = p.vplane + (blk * p.Hkv + j) * (int64_t)(KV_BS * p.hd);
#pragma unroll
              for (int i = 0; i < 4; ++i) dst[v_cache_offset(tok, c0 + i)] = f32_to_f16_sat(v[i]);
            }
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
      if (t < p.M) p.ssq_out[tile * p.ssq_stride + t] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Decode attention, one wavefront per (key split, kv head, sequence).
//   S^T = K Q^T (keys x heads), online softmax per head along the key axis with cross-lane shuffles,
//   O^T = V^T P^T (head_dim x heads).  The G query heads of the group share every K/V byte.
// Partial results (m, l, unnormalised o) of all splits of a (sequence, kv head) are merged by the
// wavefront that finishes last, which also writes the packed hi/lo operand of the O projection.
template <int HD>
__global__ __launch_bounds__(64) void decode_attn_kernel(const float* __restrict__ q, const uint16_t* __restrict__ kplane,
                                                          const uint16_t* __restrict__ vplane, const int32_t* __restrict__ seq_lens,
                                                          const int32_t* __restrict__ table, int mbs, int G, int Hq, int Hkv, int kps,
                                                          float qscale, float* __restrict__ part, int* __restrict__ counters,
                                                          uint16_t* __restrict__ xo, int MT) {
  constexpr int NKF = HD / 32;  // K fragments per block
  constexpr int NVF = HD / 16;  // V fragments per block
  constexpr int PSTRIDE = HD + 4;  // floats per (split, head) partial record: o[HD], m, l, pad
  const int split = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x;
  const int n = lane & 15, g = lane >> 4;
  const int ctx = seq_lens[b];
  const int k0 = split * kps;
  if (k0 >= ctx) return;
  const int nsplit_act = (ctx + kps - 1) / kps;
  const int nsplit_max = gridDim.x;
  const int kend = min(ctx, k0 + kps);
  const int npairs = (kend - k0 + 31) / 32;
  const int32_t* trow = table + (int64_t)b * mbs;
  const int last_blk = (ctx - 1) / KV_BS;

  // Q^T operand: lane (head n, group g) holds dims f*32 + g*8 .. +7 of head n, as hi + lo
  f16x8 qhi[NKF], qlo[NKF];
#pragma unroll
  for (int f = 0; f < NKF; ++f) {
    union { uint16_t s[8]; f16x8 v; } hi, lo;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = 0.f;
      if (n < G) x = q[((int64_t)b * Hq + j * G + n) * HD + f * 32 + g * 8 + e] * qscale;
      split_f16(x, hi.s[e], lo.s[e]);
    }
    qhi[f] = hi.v;
    qlo[f] = lo.v;
  }

  f32x4 oacc[NVF];
#pragma unroll
  for (int f = 0; f < NVF; ++f) oacc[f] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = NEG_INF, l_run = 0.f;

  const int64_t blk_elems = (int64_t)KV_BS * HD;
  for (int pr = 0; pr < npairs; ++pr) {
    const int base = k0 + pr * 32;
    const int bi0 = base / KV_BS;
    const int bi1 = min(bi0 + 1, last_blk);
    const int64_t off0 = ((int64_t)trow[bi0] * Hkv + j) * blk_elems;
    const int64_t off1 = ((int64_t)trow[bi1] * Hkv + j) * blk_elems;
    uint4 kf0[NKF], kf1[NKF];
    uint2 vf0[NVF], vf1[NVF];
#pragma unroll
    for (int f = 0; f < NKF; ++f) {
      kf0[f] = *reinterpret_cast<const uint4*>(kplane + off0 + (f * 64 + lane) * 8);
      kf1[f] = *reinterpret_cast<const uint4*>(kplane + off1 + (f * 64 + lane) * 8);
    }
#pragma unroll
    for (int f = 0; f < NVF; ++f) {
      vf0[f] = *reinterpret_cast<const uint2*>(vplane + off0 + (f * 64 + lane) * 4);
      vf1[f] = *reinterpret_cast<const uint2*>(vplane + off1 + (f * 64 + lane) * 4);
    }
    // scores (already in log2 units): lane (head n, g) gets keys base + 4g + i (block 0) and base + 16 + 4g + i (block 1)
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int f = 0; f < NKF; ++f) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(kf0[f]), qhi[f], s0, 0, 0, 0);
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(kf0[f]), qlo[f], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(kf1[f]), qhi[f], s1, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(kf1[f]), qlo[f], s1, 0, 0, 0);
    }
    float sc[8];
    float mx = NEG_INF;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      sc[i] = (base + 4 * g + i < kend) ? s0[i] : NEG_INF;
      sc[4 + i] = (base + 16 + 4 * g + i < kend) ? s1[i] : NEG_INF;
      mx = fmaxf(mx, fmaxf(sc[i], sc[4 + i]));
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    union { uint16_t s[8]; f16x8 v; } pb;
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float pv = __builtin_amdgcn_exp2f(sc[i] - m_new);
      psum += pv;
      pb.s[i] = f32_to_f16_sat(pv);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    // values of masked keys must not reach the MFMA (0 * NaN): clear them in the tail pair
    if (base + 32 > kend) {
      const int ka = base + 4 * g, kb2 = base + 16 + 4 * g;
      const uint32_t a01 = (ka + 0 < kend ? 0xFFFFu : 0u) | (ka + 1 < kend ? 0xFFFF0000u : 0u);
      const uint32_t a23 = (ka + 2 < kend ? 0xFFFFu : 0u) | (ka + 3 < kend ? 0xFFFF0000u : 0u);
      const uint32_t b01 = (kb2 + 0 < kend ? 0xFFFFu : 0u) | (kb2 + 1 < kend ? 0xFFFF0000u : 0u);
      const uint32_t b23 = (kb2 + 2 < kend ? 0xFFFFu : 0u) | (kb2 + 3 < kend ? 0xFFFF0000u : 0u);
#pragma unroll
      for (int f = 0; f < NVF; ++f) {
        vf0[f].x &= a01; vf0[f].y &= a23;
        vf1[f].x &= b01; vf1[f].y &= b23;
      }
    }
#pragma unroll
    for (int f = 0; f < NVF; ++f) {
      uint4 a = make_uint4(vf0[f].x, vf0[f].y, vf1[f].x, vf1[f].y);
      oacc[f][0] *= alpha; oacc[f][1] *= alpha; oacc[f][2] *= alpha; oacc[f][3] *= alpha;
      oacc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), pb.v, oacc[f], 0, 0, 0);
    }
  }
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);

  // park this split's record: [b][j][split][head n][o(HD), m, l]
  float* rec = part + ((((int64_t)b * Hkv + j) * nsplit_max + split) * G) * PSTRIDE;
  if (n < G) {
#pragma unroll
    for (int f = 0; f < NVF; ++f)
      *reinterpret_cast<float4*>(rec + n * PSTRIDE + f * 16 + g * 4) = make_float4(oacc[f][0], oacc[f][1], oacc[f][2], oacc[f][3]);
    if (g == 0) {
      rec[n * PSTRIDE + HD] = m_run;
      rec[n * PSTRIDE + HD + 1] = l_run;
    }
  }
  __threadfence();
  int old = 0;
  if (lane == 0) old = atomicAdd(&counters[b * Hkv + j], 1);
  old = __shfl(old, 0);
  if (old != nsplit_act - 1) return;
  __threadfence();
  if (lane == 0) counters[b * Hkv + j] = 0;

  // merge all splits (in split order) and emit the packed O-projection operand
  const float* recs = part + (((int64_t)b * Hkv + j) * nsplit_max) * G * PSTRIDE;
  for (int hh = 0; hh < G; ++hh) {
    float M = NEG_INF;
    for (int s = 0; s < nsplit_act; ++s) M = fmaxf(M, recs[((int64_t)s * G + hh) * PSTRIDE + HD]);
    float Lsum = 0.f;
    float o[HD / 64];
#pragma unroll
    for (int i = 0; i < HD / 64; ++i) o[i] = 0.f;
    for (int s = 0; s < nsplit_act; ++s) {
      const float* r = recs + ((int64_t)s * G + hh) * PSTRIDE;
      float w = __builtin_amdgcn_exp2f(r[HD] - M);
      Lsum += r[HD + 1] * w;
#pragma unroll
      for (int i = 0; i < HD / 64; ++i) o[i] += r[lane + 64 * i] * w;
    }
    const float inv = 1.f / Lsum;
#pragma unroll
    for (int i = 0; i < HD / 64; ++i) {
      int k = (j * G + hh) * HD + lane + 64 * i;
      uint16_t hi, lo;
      split_f16(o[i] * inv, hi, lo);
      xo[packed_x_offset(k, b, MT, 0)] = hi;
      xo[packed_x_offset(k, b, MT, 1)] = lo;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Greedy next token: index of the largest logit, the lowest index winning ties.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int V, int32_t* __restrict__ out) {
  const float* row = logits + (int64_t)blockIdx.x * V;
  float best = NEG_INF;
  int bi = 0x7fffffff;
  for (int i = threadIdx.x; i < V; i += blockDim.x) {
    float v = row[i];
    if (v > best || (v == best && i < bi)) { best = v; bi = i; }
  }
  __shared__ float sv[1024];
  __shared__ int si[1024];
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int s = 512; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) {
      float ov = sv[threadIdx.x + s];
      int oi = si[threadIdx.x + s];
      if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) { sv[threadIdx.x] = ov; si[threadIdx.x] = oi; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = si[0];
}

// ------------------------------------------------------------------------------------------------
// Host side

static void choose_split(int row_tiles, int zb, int KB, int* ksplit, int* kb_per_split) {
  int want = 384 / (row_tiles * zb);
  if (want < 1) want = 1;
  if (want > MAX_KSPLIT) want = MAX_KSPLIT;
  int per = (KB + want - 1) / want;
  per = (per + 3) / 4 * 4;
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
  dim3 grid(row_tiles, p.ksplit, zb), block(256);
#define LAUNCH(MTK_, WS_) hipLaunchKernelGGL((skinny_gemm_kernel<MTK_, WS_, EPI>), grid, block, 0, st, p)
  if (m->wsplit) {
    if (mtk == 1) LAUNCH(1, true); else if (mtk == 2) LAUNCH(2, true); else LAUNCH(4, true);
  } else {
    if (mtk == 1) LAUNCH(1, false); else if (mtk == 2) LAUNCH(2, false); else LAUNCH(4, false);
  }
#undef LAUNCH
}

int decode_MT(int batch) { return batch <= 16 ? 1 : batch <= 32 ? 2 : ((batch + 63) / 64) * 4; }

int run_decode(www_model* m, const int32_t* tok, const int32_t* lens, const int32_t* table, int batch, float* logits, int32_t* next,
               hipStream_t st) {
  const int MT = decode_MT(batch);
  const int d = m->d;
  if (m->cfg.weight_dtype == WWW_DTYPE_F32)
    hipLaunchKernelGGL(embed_pack_kernel<float>, dim3(batch), dim3(256), 0, st, tok, (const float*)m->embed, d, m->layers[0].attn_norm,
                       m->h, m->ssq, (uint16_t*)m->xq, MT);
  else
    hipLaunchKernelGGL(embed_pack_kernel<uint16_t>, dim3(batch), dim3(256), 0, st, tok, (const uint16_t*)m->embed, d,
                       m->layers[0].attn_norm, m->h, m->ssq, (uint16_t*)m->xq, MT);
  int n_ssq = 1;
  const int stride = m->maxB;
  const float qscale = 1.4426950408889634f / sqrtf((float)m->hd);
  for (int l = 0; l < m->L; ++l) {
    const LayerW& w = m->layers[l];
    uint16_t* kplane = (uint16_t*)m->kv + (int64_t)(2 * l) * m->kv_plane;
    uint16_t* vplane = (uint16_t*)m->kv + (int64_t)(2 * l + 1) * m->kv_plane;
    {
      GemmP p = {};
      p.W = (const uint4*)w.wqkv; p.Wlo = (const uint4*)w.wqkv_lo; p.NRG = m->QKVN / 16; p.KB = d / 32;
      p.X = (const uint4*)m->xq; p.M = batch;
      p.ssq_in = m->ssq; p.n_ssq_in = n_ssq; p.ssq_stride = stride; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
      p.q = m->q; p.kplane = kplane; p.vplane = vplane; p.seq_lens = lens; p.table = table; p.mbs = m->cfg.max_blocks_per_seq;
      p.hd = m->hd; p.Hq = m->Hq; p.Hkv = m->Hkv; p.rope = m->rope;
      launch_gemm<EPI_QKV>(m, p, MT, st);
    }
    {
      dim3 grid(m->attn_splits, m->Hkv, batch);
      if (m->hd == 128)
        hipLaunchKernelGGL(decode_attn_kernel<128>, grid, dim3(64), 0, st, m->q, kplane, vplane, lens, table, (int)m->cfg.max_blocks_per_seq,
                           m->G, m->Hq, m->Hkv, m->attn_kps, qscale, m->attn_part, m->counters + 65536, (uint16_t*)m->xo, MT);
      else
        hipLaunchKernelGGL(decode_attn_kernel<64>, grid, dim3(64), 0, st, m->q, kplane, vplane, lens, table, (int)m->cfg.max_blocks_per_seq,
                           m->G, m->Hq, m->Hkv, m->attn_kps, qscale, m->attn_part, m->counters + 65536, (uint16_t*)m->xo, MT);
    }
    {
      GemmP p = {};
      p.W = (const uint4*)w.wo; p.Wlo = (const uint4*)w.wo_lo; p.NRG = d / 16; p.KB = m->QD / 32;
      p.X = (const uint4*)m->xo; p.M = batch;
      p.h = m->h; p.gain_next = w.ffn_norm; p.xnext = (uint16_t*)m->xq; p.ssq_out = m->ssq; p.ssq_stride = stride; p.d = d;
      launch_gemm<EPI_RESID>(m, p, MT, st);
      n_ssq = (d / 16 + 7) / 8;
    }
    {
      GemmP p = {};
      p.W = (const uint4*)w.wgu; p.Wlo = (const uint4*)w.wgu_lo; p.NRG = 2 * m->F / 16; p.KB = d / 32;
      p.X = (const uint4*)m->xq; p.M = batch;
      p.ssq_in = m->ssq; p.n_ssq_in = n_ssq; p.ssq_stride = stride; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
      p.xa = (uint16_t*)m->xa; p.F = m->F;
      launch_gemm<EPI_SWIGLU>(m, p, MT, st);
    }
    {
      GemmP p = {};
      p.W = (const uint4*)w.wd; p.Wlo = (const uint4*)w.wd_lo; p.NRG = d / 16; p.KB = m->Fp / 32;
      p.X = (const uint4*)m->xa; p.M = batch;
      p.h = m->h; p.gain_next = (l + 1 < m->L) ? m->layers[l + 1].attn_norm : m->final_norm;
      p.xnext = (uint16_t*)m->xq; p.ssq_out = m->ssq; p.ssq_stride = stride; p.d = d;
      launch_gemm<EPI_RESID>(m, p, MT, st);
    }
  }
  float* lg = logits ? logits : m->logits_buf;
  {
    GemmP p = {};
    p.W = (const uint4*)m->lm_head; p.Wlo = (const uint4*)m->lm_head_lo; p.NRG = m->V / 16; p.KB = d / 32;
    p.X = (const uint4*)m->xq; p.M = batch;
    p.ssq_in = m->ssq; p.n_ssq_in = n_ssq; p.ssq_stride = stride; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
    p.logits = lg; p.V = m->V;
    launch_gemm<EPI_LOGITS>(m, p, MT, st);
  }
  if (next) hipLaunchKernelGGL(argmax_kernel, dim3(batch), dim3(1024), 0, st, lg, m->V, next);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("decode launch failed: %s", hipGetErrorString(e));
    return WWW_E_HIP;
  }
  return WWW_OK;
}
