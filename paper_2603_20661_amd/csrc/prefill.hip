// Prefill path (many new tokens per sequence): ragged-batch bookkeeping, embedding, RMSNorm,
// LDS-tiled fp16 MFMA GEMM with rotary + KV-cache write / residual / SwiGLU epilogues, and causal
// paged flash attention over cached prefix + new tokens.  This pass fills the KV cache; the logits
// of each sequence's last position are produced afterwards by the decode path, which keeps the
// activations of that one row in hi/lo precision.
#include "common.h"

#define NEG_INF (-__builtin_inff())

__device__ __forceinline__ f16x8 as_f16x8(u32x4 v) { return __builtin_bit_cast(f16x8, v); }

#define ATTN_TQ 64  // query rows per attention workgroup

// ------------------------------------------------------------------------------------------------
// Ragged batch bookkeeping (one workgroup).  meta[0] = number of attention tiles.
__global__ __launch_bounds__(1024) void prefill_meta_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ q_lens,
                                                             const int32_t* __restrict__ seq_lens, int batch, int T,
                                                             int32_t* __restrict__ row_seq, int32_t* __restrict__ row_pos,
                                                             int32_t* __restrict__ tile_seq, int32_t* __restrict__ tile_q0,
                                                             int32_t* __restrict__ meta, int32_t* __restrict__ last_tok,
                                                             int32_t* __restrict__ cum /* [2*(batch+1)] scratch */) {
  int32_t* cum_rows = cum;
  int32_t* cum_tiles = cum + batch + 1;
  if (threadIdx.x == 0) {
    int r = 0, tl = 0;
    for (int b = 0; b < batch; ++b) {
      cum_rows[b] = r;
      cum_tiles[b] = tl;
      r += q_lens[b];
      tl += (q_lens[b] + ATTN_TQ - 1) / ATTN_TQ;
    }
    cum_rows[batch] = r;
    cum_tiles[batch] = tl;
    meta[0] = tl;
  }
  __syncthreads();
  for (int r = threadIdx.x; r < T; r += blockDim.x) {
    int lo = 0, hi = batch - 1;  // last b with cum_rows[b] <= r
    while (lo < hi) {
      int mid = (lo + hi + 1) >> 1;
      if (cum_rows[mid] <= r) lo = mid; else hi = mid - 1;
    }
    row_seq[r] = lo;
    row_pos[r] = seq_lens[lo] - q_lens[lo] + (r - cum_rows[lo]);
  }
  for (int b = threadIdx.x; b < batch; b += blockDim.x) {
    int nt = cum_tiles[b + 1] - cum_tiles[b];
    for (int i = 0; i < nt; ++i) {
      tile_seq[cum_tiles[b] + i] = b;
      tile_q0[cum_tiles[b] + i] = i * ATTN_TQ;
    }
    last_tok[b] = tokens[cum_rows[b + 1] - 1];
  }
}

// The residual stream of the prefill path is only ever touched by the embedding kernel and by the residual epilogues of
// the O and down projections, which both tile it 256 tokens x 256 rows with the same accumulator layout.  It is
// therefore kept in that layout ("register image"): block (token tile tt, row tile rt) holds 64 Ki floats ordered
// [wavefront wn*2+wt][rb][tb][q4][lane][4], element = the lane's four consecutive rows
//   row   = rt*256 + wn*128 + rb*32 + q4*8 + (lane/32)*4 + e,   token = tt*256 + wt*128 + tb*32 + lane%32,
// so that every load and store of an epilogue is one contiguous KiB per wavefront instead of 64 pieces of 16 bytes
// that lie a whole token row apart.
__device__ __forceinline__ int64_t hp_image_offset(int tt, int rt, int n_rt, int wave, int rb, int tb, int q4, int lane) {
  return (((((((int64_t)tt * n_rt + rt) * 4 + wave) * 4 + rb) * 4 + tb) * 4 + q4) * 64 + lane) * 4;
}
// the same for token t and row n (a multiple of 4)
__device__ __forceinline__ int64_t hp_image_offset_of(int64_t t, int n, int n_rt) {
  const int w256 = (int)(t & 255), c = n & 255;
  const int wave = (c >> 7) * 2 + (w256 >> 7), rb = (c & 127) >> 5, tb = (w256 & 127) >> 5, q4 = (c & 31) >> 3;
  const int lane = ((c & 7) >> 2) * 32 + (w256 & 31);
  return hp_image_offset((int)(t >> 8), n >> 8, n_rt, wave, rb, tb, q4, lane);
}

// Embedding rows: residual stream h = E[token] (fp32), the first GEMM operand fp16(h * gain) in the packed prefill
// layout, and the row's sum of squares.  RMSNorm's 1/rms factor is applied by the consuming GEMM's epilogue.
template <typename ET>
__global__ __launch_bounds__(256) void embed_rows_kernel(const int32_t* __restrict__ tokens, const ET* __restrict__ embed, int d,
                                                          const float* __restrict__ gain, float* __restrict__ hp,
                                                          uint16_t* __restrict__ xn, float* __restrict__ ssq) {
  int64_t r = blockIdx.x;
  const ET* row = embed + (int64_t)tokens[r] * d;
  float local = 0.f;
  for (int k = threadIdx.x * 4; k < d; k += blockDim.x * 4) {
    union { uint16_t s[4]; u32x2 v; } o;
    float x[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if constexpr (sizeof(ET) == 4) x[e] = (float)row[k + e];
      else x[e] = bf16_bits_to_float(((const uint16_t*)row)[k + e]);
      local += x[e] * x[e];
      o.s[e] = f32_to_f16_sat(x[e] * gain[k + e]);
    }
    *reinterpret_cast<float4*>(hp + hp_image_offset_of(r, k, (d + 255) >> 8)) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<u32x2*>(xn + packed_p_offset(r, k, d >> 4)) = o.v;
  }
  __shared__ float red[256];
  red[threadIdx.x] = local;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) ssq[(int64_t)r * PSSQ] = red[0];  // row r of the [token][PSSQ] table, one entry in use
}

// ------------------------------------------------------------------------------------------------
// Tiled GEMM  Y^T[n][t] = sum_k W[n][k] X[t][k]:  256 weight rows x 256 tokens per workgroup, four
// wavefronts each owning 128 x 128 as 4 x 4 MFMA 32x32x16 tiles.  Both operands arrive already in MFMA
// fragment order (packed weights, packed activations), so a K step of 32 is a straight 32 KiB copy into
// LDS (16 weight fragments + 16 activation fragments) and every LDS read is a conflict-free 16-byte read.
enum { PEPI_QKV = 0, PEPI_RESID = 1, PEPI_SWIGLU = 2 };
#define PGEMM_NB 4  // stage buffers of the prefill GEMM (32 KiB each)
#define PGEMM_LDS_BYTES (PGEMM_NB * 2048 * 16)

struct PGemmP {
  const u32x4* W;  // packed weights
  float wfactor;   // scale of the matrix (FP8 weight-only sources; 1 otherwise), applied to the result
  int NRG, KB;
  const u32x4* X;  // packed activations
  int T;
  int n_tt, n_rt;  // token tiles, row tiles
  // QKV epilogue
  const float* qk_gain;  // models with normalised query / key heads: [2][hd] gains in packed row order; null otherwise
  uint16_t* qp;
  uint16_t *kplane, *vplane;  // this layer's key / value planes of the pool (16-bit codes)
  float* kvscale;             // and its plane of scales
  const int32_t *row_seq, *row_pos, *table;
  int mbs, hd, Hq, Hkv;
  const float2* rope;
  // RMSNorm scale of the input rows (QKV and SwiGLU GEMMs): rsqrt(sum_i ssq_in[i][t] / dim + eps) multiplies the result
  const float* ssq_in;
  int n_ssq_in;
  float inv_dim, eps;
  // residual epilogue: h += result; also emits the next GEMM's operand fp16(h * gain_next) and partial sums of squares
  float* hp;
  int d;
  const float* gain_next;
  uint16_t* xn_out;
  float* ssq_out;
  // SwiGLU epilogue
  uint16_t* ap;
  int Fp;
};

// Workgroup id -> tile of the prefill GEMM.  Workgroup ids are dealt round-robin to the 8 XCDs and dispatched in order,
// so a round of 256 workgroups gives every XCD 32 consecutive local indices.  Token tiles are taken in super-groups of
// 8 x GT: XCD x owns GT of them and walks the row tiles 8 at a time (32 workgroups = GT token tiles x 8 row tiles: its
// L2 sees GT + 8 operand panels per round), and all XCDs walk the row tiles in step, so a weight panel is fetched from
// memory once per super-group and found in the memory-side cache by the other seven.  The token tiles that do not
// fill a super-group follow in groups of GT with the ids' order simply transposed over the XCDs.  The map is a
// bijection from [0, n_tt * n_rt) onto the tiles (checked on the host for many shapes through www_debug_prefill_tile).
__host__ __device__ __forceinline__ void pgemm_tile_of(int id, int n_tt, int n_rt, int* tt_out, int* rt_out) {
  constexpr int GT = 4;
  const int total = n_tt * n_rt;
  const int n_sg = n_tt / (8 * GT);            // full super-groups
  const int total_sg = n_sg * 8 * GT * n_rt;   // tiles in them (a multiple of 8)
  if (id < total_sg) {
    const int x = id & 7, li = id >> 3;
    const int per_sg = GT * n_rt;              // tiles of one XCD in one super-group
    const int sg = li / per_sg, within = li % per_sg;
    *tt_out = (sg * 8 + x) * GT + within % GT;
    *rt_out = within / GT;
  } else {
    int v = id - total_sg;
    const int rest = total - total_sg, tt0 = n_sg * 8 * GT;
    if (rest % 8 == 0) v = (v % 8) * (rest / 8) + v / 8;
    const int per_group = GT * n_rt;
    const int group = v / per_group, first_tt = tt0 + group * GT;
    const int left = n_tt - first_tt;
    const int gsz = left < GT ? left : GT;
    *tt_out = first_tt + (v % per_group) % gsz;
    *rt_out = (v % per_group) / gsz;
  }
}

// QKN: the QKV epilogue also normalises the query and key heads (an instantiation of its own, so that the plain model's
// kernel carries none of its registers)
template <int EPI, bool QKN = false>
__global__ __launch_bounds__(256) void prefill_gemm_kernel(const PGemmP p) {
  // PGEMM_NB stage buffers of 2048 sixteen-byte units: 0..1023 weights [16 row groups][64], 1024..2047 activations [8 token groups][2 k16][64]
  extern __shared__ u32x4 smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wn = wave >> 1, wt = wave & 1;

  int tt, rt;
  pgemm_tile_of((int)blockIdx.x, p.n_tt, p.n_rt, &tt, &rt);

  const int rg_tile = rt * 16;
  const int t_tile = tt * 256;
  const int K16 = p.KB * 2;

  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

  // Stage copies go from memory straight into LDS, without a register stage and without LDS store instructions: one
  // global_load_lds_dwordx4 moves 64 lanes x 16 bytes to 1 KiB of LDS in lane order (M0 = LDS byte address), which is
  // the layout of a packed fragment unit.  The copies are written as inline assembly so that the waits for them can be
  // placed by hand: the compiler would wait for all of them at every LDS barrier.  They count in vmcnt like any load
  // and complete in order; the kernel issues no other vector memory instruction before the end of the main loop.
  // NB stage buffers: while k block s is multiplied, blocks s+1 .. s+NB-2 are in flight or have landed and block
  // s+NB-1 is being requested.
  constexpr int NB = PGEMM_NB;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const u32x4* srcA[4];
  const u32x4* srcB[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int f = wave_u + 4 * i;  // fragment unit 0..15 handled by this wavefront
    srcA[i] = p.W + (int64_t)min(rg_tile + f, p.NRG - 1) * 64;
    srcB[i] = p.X + ((int64_t)(tt * 8 + (f >> 1)) * K16 + (f & 1)) * 64;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
  const uint32_t voff = lane * 16;
  u32x4 fa0[4], fb0[4], fa1[4], fb1[4];
  const int fm = lane & 31, fh = lane >> 5;
  auto dma16 = [&](const u32x4* g, uint32_t lds_addr) __attribute__((always_inline)) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(g), "s"(lds_addr) : "memory", "m0");
  };
  // unit i = 0..7 of this wavefront's share of a k block: even = weights, odd = activations
  auto stage1 = [&](int kbc, int buf, int i) __attribute__((always_inline)) {
    const int q = i >> 1;
    if (i & 1) dma16(srcB[q] + (int64_t)kbc * 128, lds0 + (uint32_t)(buf * 2048 + 1024 + (wave_u + 4 * q) * 64) * 16u);
    else dma16(srcA[q] + (int64_t)kbc * p.NRG * 64, lds0 + (uint32_t)(buf * 2048 + (wave_u + 4 * q) * 64) * 16u);
  };
  auto stage = [&](int kb, int buf) __attribute__((always_inline)) {
    const int kbc = min(kb, p.KB - 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) stage1(kbc, buf, i);
  };
  // fragment read i = 0..7 of a 16-column half: 0..3 weights (row blocks), 4..7 activations (token blocks)
  auto fetch1 = [&](u32x4(&fa)[4], u32x4(&fb)[4], int buf, int k16, int i) __attribute__((always_inline)) {
    if (i < 4) fa[i] = smem[buf * 2048 + (wn * 8 + i * 2 + (fm >> 4)) * 64 + ((k16 * 2 + fh) << 4) + (fm & 15)];
    else fb[i - 4] = smem[buf * 2048 + 1024 + ((wt * 4 + (i - 4)) * 2 + k16) * 64 + lane];
  };
  auto fetch = [&](u32x4(&fa)[4], u32x4(&fb)[4], int buf, int k16) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) fetch1(fa, fb, buf, k16, i);
  };
  auto mfma1 = [&](u32x4(&fa)[4], u32x4(&fb)[4], int i) __attribute__((always_inline)) {
    const int rb = i >> 2, tb = i & 3;
    acc[rb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(fa[rb]), as_f16x8(fb[tb]), acc[rb][tb], 0, 0, 0);
  };
  auto lds_barrier = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  };
  // k block s sits in buffer r = s mod NB; two fragment sets carry the LDS reads of its two 16-column halves.  The
  // instruction order is fixed by hand: one LDS read behind each of the first eight MFMAs of a half (half 1 of block s
  // in the first half, half 0 of block s+1 in the second, each 8 to 16 MFMAs before its data is needed) and one stage
  // copy behind every fourth MFMA, so that the requests of the four wavefronts reach the memory pipeline evenly spread.
  // The copies of block s+NB-1 go to the buffer of block s-1, which nobody reads any more once the barrier of block
  // s-1 has been passed.  One barrier per k block, in the middle: in front of it a wavefront waits until its own units
  // of block s+1 have landed (at most (NB-3) blocks of 8 units and the 4 units of block s+NB-1 requested so far may
  // still be outstanding); behind it everybody's have.  Past the last k block the copies are redirected to the last
  // block; nobody reads them.
  // s_waitcnt immediates for "at most n memory requests outstanding": a 6-bit count split over bits 3:0 and 15:14, the
  // other counters unconstrained
  constexpr int VM_MID = (NB - 3) * 8 + 4;
  constexpr int WAIT_MID = 0x0F70 | (VM_MID & 15) | ((VM_MID >> 4) << 14);
  constexpr int VM_PRO = (NB - 2) * 8;
  constexpr int WAIT_PRO = 0x0F70 | (VM_PRO & 15) | ((VM_PRO >> 4) << 14);
  auto k_block = [&](int s, int r) __attribute__((always_inline)) {
    const int buf1 = r == NB - 1 ? 0 : r + 1, bufp = r == 0 ? NB - 1 : r - 1;
    const int kbc = min(s + NB - 1, p.KB - 1);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      mfma1(fa0, fb0, i);
      if (i < 8) fetch1(fa1, fb1, r, 1, i);
      if ((i & 3) == 3) stage1(kbc, bufp, i >> 2);
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(WAIT_MID);  // this wavefront's units of block s+1 have landed
    lds_barrier();                         // ... everybody's
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      mfma1(fa1, fb1, i);
      if (i < 8) fetch1(fa0, fb0, buf1, 0, i);
      if ((i & 3) == 3) stage1(kbc, bufp, 4 + (i >> 2));
      __builtin_amdgcn_sched_barrier(0);
    }
  };

#pragma unroll
  for (int b = 0; b < NB - 1; ++b) stage(b, b);
  __builtin_amdgcn_s_waitcnt(WAIT_PRO);
  lds_barrier();
  fetch(fa0, fb0, 0, 0);
  {
    int s = 0;
    for (; s + NB - 1 < p.KB; s += NB) {
#pragma unroll
      for (int r = 0; r < NB; ++r) k_block(s + r, r);
    }
#pragma unroll
    for (int r = 0; r < NB - 1; ++r)
      if (s + r < p.KB) k_block(s + r, r);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // the redirected copies past the last k block have landed too
  __syncthreads();  // the staging buffers are dead from here on; the residual epilogue reuses them
  float(*red_ssq)[256] = reinterpret_cast<float(*)[256]>(smem);
  (void)red_ssq;

  // acc[rb][tb][i] = Y^T[row][token]: row = (rg_tile + wn*8 + rb*2)*16 + (i/4)*8 + (lane/32)*4 + i%4, token = t_tile + wt*128 + tb*32 + lane%32
  const int hsel = lane >> 5;
  // Everything the epilogue needs from memory per token is requested up front for all four token groups (one memory
  // round trip, two for the KV block ids), and the per-element operands of a token group (residual rows, rotary
  // factors) in one batch per group: a wavefront has no partner on its SIMD to hide a chain of dependent loads behind.
  // Addresses of tokens past the end are clamped; their results are dropped.
  int tcl[4];
  bool tok_ok[4];
  float scale[4];
  int pos[4], blk[4];
#pragma unroll
  for (int tb = 0; tb < 4; ++tb) {
    const int t = t_tile + wt * 128 + tb * 32 + (lane & 31);
    tok_ok[tb] = t < p.T;
    tcl[tb] = min(t, p.T - 1);
    scale[tb] = p.wfactor;
    pos[tb] = 0;
    blk[tb] = 0;
  }
  if constexpr (EPI != PEPI_RESID) {
    if constexpr (EPI == PEPI_QKV) {
      int seq[4];
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) {
        pos[tb] = p.row_pos[tcl[tb]];
        seq[tb] = p.row_seq[tcl[tb]];
      }
#pragma unroll
      for (int tb = 0; tb < 4; ++tb) blk[tb] = kv_block_id(p.table + (int64_t)seq[tb] * p.mbs, pos[tb]);
    }
    // the tokens' rows of the sum-of-squares table, [token][PSSQ], two token groups at a time (64 registers);
    // entries past n_ssq_in are masked, the rest is added in tile order
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      if (!p.ssq_in) break;  // no normalisation requested: the scales stay 1
      f32x4 sq[2][PSSQ / 4];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int c = 0; c < PSSQ / 4; ++c)
          sq[u][c] = *reinterpret_cast<const f32x4*>(p.ssq_in + (int64_t)tcl[half * 2 + u] * PSSQ + c * 4);
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float ss = 0.f;
#pragma unroll
        for (int c = 0; c < PSSQ / 4; ++c)
#pragma unroll
          for (int e = 0; e < 4; ++e) ss += (c * 4 + e < p.n_ssq_in) ? sq[u][c][e] : 0.f;
        scale[half * 2 + u] = rsqrtf(ss * p.inv_dim + p.eps) * p.wfactor;
      }
    }
  }
  f32x4 gv[4][4];  // next norm's gain for this lane's 16 x 4 rows (residual epilogue); gains of the head normalisation (QKV)
  if constexpr (EPI == PEPI_QKV && QKN) {
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int rg = min(rg_tile + wn * 8 + rb * 2 + (q4 >> 1), p.NRG - 1);
        const int n0 = rg * 16 + (q4 & 1) * 8 + hsel * 4;
        gv[rb][q4] = *reinterpret_cast<const f32x4*>(p.qk_gain + (n0 / p.hd < p.Hq ? 0 : p.hd) + n0 % p.hd);  // (value rows: unused)
      }
  }
  if constexpr (EPI == PEPI_RESID) {
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int rg = min(rg_tile + wn * 8 + rb * 2 + (q4 >> 1), p.NRG - 1);
        gv[rb][q4] = *reinterpret_cast<const f32x4*>(p.gain_next + rg * 16 + (q4 & 1) * 8 + hsel * 4);
      }
  }
#pragma unroll
  for (int tb = 0; tb < 4; ++tb) {
    __builtin_amdgcn_sched_barrier(0);  // one token group at a time: keeps the accumulator copies of the others out of the way
    const int t = tcl[tb];
    const bool ok = tok_ok[tb];
    const int64_t slot = kv_slot_in_block(blk[tb], pos[tb]);
    const int64_t kvbase = (slot / KV_BS) * p.Hkv;
    const int tok = (int)(slot % KV_BS);
    // one batch of loads for this token group: residual rows (RESID) or rotary factors (QKV)
    f32x4 pre[4][4];
    if constexpr (EPI != PEPI_SWIGLU) {
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int rg = min(rg_tile + wn * 8 + rb * 2 + (q4 >> 1), p.NRG - 1);
          const int n0 = rg * 16 + (q4 & 1) * 8 + hsel * 4;
          if constexpr (EPI == PEPI_RESID)  // (whole tiles are allocated: in bounds also for tokens and rows past the end)
            pre[rb][q4] = *reinterpret_cast<const f32x4*>(p.hp + hp_image_offset(tt, rt, p.n_rt, wave, rb, tb, q4, lane));
          else pre[rb][q4] = *reinterpret_cast<const f32x4*>(p.rope + (int64_t)pos[tb] * (p.hd / 2) + ((n0 % p.hd) >> 1));
        }
    }
    float ssq_tok = 0.f;
    // Normalised query / key heads: a wavefront's 128 rows are one head of 128 or two heads of 64 (row blocks 0,1 and
    // 2,3), and a token's values of these rows sit in the two lanes l, l + 32: 1 / rms per head from the lane's own
    // squares and one cross-lane exchange.
    float head_rs[2] = {1.f, 1.f};
    if constexpr (EPI == PEPI_QKV && QKN) {
      float ss[2] = {0.f, 0.f};
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float v = acc[rb][tb][i] * scale[tb];
          ss[rb >> 1] += v * v;
        }
      if (p.hd == 128) ss[0] = ss[1] = ss[0] + ss[1];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        ss[hh] += __shfl_xor(ss[hh], 32);
        head_rs[hh] = rsqrtf(ss[hh] / (float)p.hd + p.eps);
      }
    }
    // QKV: finish the values in place (RMSNorm factor, head normalisation, rotation) and take the largest magnitude of
    // each head's vector for this token: the scale of its key / value codes.  A wavefront's 128 rows are one head of
    // 128 or two of 64 (row blocks 0,1 and 2,3); the token's values sit in the lanes l and l + 32.
    float head_amax[2] = {0.f, 0.f};
    if constexpr (EPI == PEPI_QKV) {
      const int rot_rows = (p.Hq + p.Hkv) * p.hd;
#pragma unroll
      for (int rb = 0; rb < 4; ++rb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int rg = rg_tile + wn * 8 + rb * 2 + (q4 >> 1);
          const int n0 = rg * 16 + (q4 & 1) * 8 + hsel * 4;
          float v4[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) v4[i] = acc[rb][tb][q4 * 4 + i] * scale[tb];
          if (n0 < rot_rows) {
            if constexpr (QKN) {
#pragma unroll
              for (int i = 0; i < 4; ++i) v4[i] *= head_rs[rb >> 1] * gv[rb][q4][i];
            }
            const f32x4 cs = pre[rb][q4];  // (cos, sin) of the two rotary pairs held here
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
              float a = v4[2 * pr], b = v4[2 * pr + 1];
              v4[2 * pr] = a * cs[2 * pr] - b * cs[2 * pr + 1];
              v4[2 * pr + 1] = b * cs[2 * pr] + a * cs[2 * pr + 1];
            }
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            acc[rb][tb][q4 * 4 + i] = v4[i];
            head_amax[rb >> 1] = fmaxf(head_amax[rb >> 1], __builtin_fabsf(v4[i]));
          }
        }
      if (p.hd == 128) head_amax[0] = head_amax[1] = fmaxf(head_amax[0], head_amax[1]);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) head_amax[hh] = fmaxf(head_amax[hh], __shfl_xor(head_amax[hh], 32));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
      const int rgb = rg_tile + wn * 8 + rb * 2;  // first of the two row groups of this 32-row block
      if constexpr (EPI == PEPI_SWIGLU) {
        if (!ok || rgb + 1 >= p.NRG) continue;
#pragma unroll
        for (int q4 = 0; q4 < 2; ++q4) {
          int f0 = (rgb >> 1) * 16 + q4 * 8 + hsel * 4;
          union { uint16_t s[4]; u32x2 v; } o;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float g = acc[rb][tb][q4 * 4 + i] * scale[tb], u = acc[rb][tb][(q4 + 2) * 4 + i] * scale[tb];
            // (hardware reciprocal, 1 ulp: the result is rounded to fp16 right away; a correctly rounded fp32 division
            // costs ten instructions per element of the widest GEMM's epilogue)
            o.s[i] = f32_to_f16_sat(g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u);
          }
          *reinterpret_cast<u32x2*>(p.ap + packed_p_offset(t, f0, p.Fp >> 4)) = o.v;
        }
      } else {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int rg = rgb + (q4 >> 1);
          if (!ok || rg >= p.NRG) continue;
          const int n0 = rg * 16 + (q4 & 1) * 8 + hsel * 4;
          float v4[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) v4[i] = acc[rb][tb][q4 * 4 + i] * scale[tb];
          if constexpr (EPI == PEPI_RESID) {
            const f32x4 hv = pre[rb][q4], g4 = gv[rb][q4];
            const float hn[4] = {hv[0] + v4[0], hv[1] + v4[1], hv[2] + v4[2], hv[3] + v4[3]};
            *reinterpret_cast<float4*>(p.hp + hp_image_offset(tt, rt, p.n_rt, wave, rb, tb, q4, lane)) = make_float4(hn[0], hn[1], hn[2], hn[3]);
            union { uint16_t s[4]; u32x2 v; } o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              ssq_tok += hn[i] * hn[i];
              o.s[i] = f32_to_f16_sat(hn[i] * g4[i]);
            }
            *reinterpret_cast<u32x2*>(p.xn_out + packed_p_offset(t, n0, p.d >> 4)) = o.v;
          } else {  // PEPI_QKV: the values were finished in place above
            const int head = n0 / p.hd, c0 = n0 % p.hd;
#pragma unroll
            for (int i = 0; i < 4; ++i) v4[i] = acc[rb][tb][q4 * 4 + i];
            union { uint16_t s[4]; u32x2 v; } o;
            if (head < p.Hq) {
#pragma unroll
              for (int i = 0; i < 4; ++i) o.s[i] = f32_to_f16_sat(v4[i]);  // queries feed the fp16 attention kernel
              *reinterpret_cast<u32x2*>(p.qp + (int64_t)t * (p.Hq * p.hd) + n0) = o.v;
            } else {
              // keys and values go to the cache as 16-bit codes with the scale of their (token, head) vector
              const bool is_v = head >= p.Hq + p.Hkv;
              const int j = head - p.Hq - (is_v ? p.Hkv : 0);
              const float amax = head_amax[rb >> 1], inv = kv_code_inv(amax);
#pragma unroll
              for (int i = 0; i < 4; ++i) o.s[i] = kv_code(v4[i], inv);
              if (!is_v) {
                *reinterpret_cast<u32x2*>(p.kplane + (kvbase + j) * (int64_t)(KV_BS * p.hd) + k_cache_offset(tok, c0)) = o.v;
              } else {
                uint16_t* dst = p.vplane + (kvbase + j) * (int64_t)(KV_BS * p.hd);
#pragma unroll
                for (int i = 0; i < 4; ++i) dst[v_cache_offset(tok, c0 + i)] = o.s[i];
              }
              if (c0 == 0) p.kvscale[kv_scale_offset(slot / KV_BS, p.Hkv, j) + (is_v ? 16 : 0) + tok] = kv_code_scale(amax);
            }
          }
        }
      }
    }
    if constexpr (EPI == PEPI_RESID) {
      ssq_tok += __shfl_xor(ssq_tok, 32);  // the two lane halves hold different rows of the same token
      if (lane < 32) red_ssq[wn][wt * 128 + tb * 32 + lane] = ssq_tok;  // (slots of tokens past the end are never read)
    }
  }
  if constexpr (EPI == PEPI_RESID) {
    // per (row tile, token) sum of squares of the new residual, the two row halves added in a fixed order
    __syncthreads();
    const int t = t_tile + tid;
    if (t < p.T) p.ssq_out[(int64_t)t * PSSQ + rt] = red_ssq[0][tid] + red_ssq[1][tid];
  }
}

// ------------------------------------------------------------------------------------------------
// Causal paged flash attention for new tokens.  One workgroup = 64 consecutive new tokens of one
// sequence x one kv head (x GH of its query heads); each wavefront owns 16 query positions and keeps
// S^T = K Q^T / O^T = V^T P^T for its GH heads.  The keys and values of a pair of blocks (32 keys) are
// copied into LDS once per workgroup and read from there by the four wavefronts (the cache already stores them
// in MFMA operand order; the copy turns the 16-bit codes into fp16 values, code * scale of its token, rounded once - the
// precision an fp16 cache would give this pass, which only needs the keys and values of other positions to matrix-core
// accuracy); the next pair travels from memory while this one is used.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int HD, int GH, int HG>
__global__ __launch_bounds__(256 * HG, 2 / HG) void prefill_attn_kernel(const uint16_t* __restrict__ qp, const uint16_t* __restrict__ kplane,
                                                            const uint16_t* __restrict__ vplane, const float* __restrict__ kvscale,
                                                            const int32_t* __restrict__ q_lens,
                                                            const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ table,
                                                            int mbs, int Hq, int Hkv, int G, const int32_t* __restrict__ tile_seq,
                                                            const int32_t* __restrict__ tile_q0, const int32_t* __restrict__ meta,
                                                            const int32_t* __restrict__ cum_rows, float scale_log2,
                                                            uint16_t* __restrict__ op, int max_tiles) {
  constexpr int NKF = HD / 32, NVF = HD / 16;
  constexpr int CH = NKF * 64;         // 16-byte units of one block's keys (and of one block's values)
  constexpr int NT = 256 * HG;         // threads: HG groups of four wavefronts, each group with its own GH query heads
  constexpr int NLD = 4 * CH / NT;     // units each thread moves per pair
  __shared__ u32x4 kv[2][4 * CH];      // per pair: keys of block 0, keys of block 1, values of block 0, values of block 1
  // Work items in the order (head group, kv head, tile), tiles fastest; workgroup ids are dealt round-robin to the 8
  // XCDs, so the ids are transposed: XCD x gets the x-th eighth of that order, i.e. the consecutive tiles of a
  // sequence and kv head run behind one L2 and fetch its keys and values into it once (with 8 kv heads: one per XCD).
  int item = blockIdx.x;
  const int n_items = gridDim.x;
  if (n_items % 8 == 0) item = (item & 7) * (n_items >> 3) + (item >> 3);
  const int tile = item % max_tiles;
  if (tile >= meta[0]) return;
  const int j = (item / max_tiles) % Hkv;
  const int tid = threadIdx.x, wave = (tid >> 6) & 3, lane = tid & 63;
  const int h0 = j * G + ((item / (max_tiles * Hkv)) * HG + (tid >> 8)) * GH;  // first query head handled by this wavefront
  const int n = lane & 15, g = lane >> 4;
  const int b = tile_seq[tile];
  const int qlen = q_lens[b], ctx = seq_lens[b];
  const int prefix = ctx - qlen;
  const int tq0 = tile_q0[tile];
  const int qw0 = tq0 + wave * 16;        // first query (index among the new tokens) of this wavefront
  const bool active = qw0 < qlen;         // a wavefront past the end of the sequence only helps with the copies
  const int nq = active ? min(16, qlen - qw0) : 1;
  const int64_t row0 = (int64_t)cum_rows[b] + (active ? qw0 : 0);
  const int my_q = min(n, nq - 1);        // lanes past the end repeat the last query; their output is dropped
  const int qpos = prefix + qw0 + my_q;   // this lane's query position
  const int kmax = active ? prefix + qw0 + nq : 0;  // keys 0 .. kmax-1 are visible to some query of the wavefront
  const int npairs = (kmax + 31) / 32;
  const int npairs_wg = (prefix + min(qlen, tq0 + 64) + 31) / 32;  // pairs the workgroup walks through
  const int last_blk = (ctx - 1) / KV_BS;
  const int32_t* trow = table + (int64_t)b * mbs;
  const int QD = Hq * HD;

  f16x8 qf[GH][NKF];
#pragma unroll
  for (int hh = 0; hh < GH; ++hh)
#pragma unroll
    for (int f = 0; f < NKF; ++f)
      qf[hh][f] = as_f16x8(*reinterpret_cast<const u32x4*>(qp + (row0 + my_q) * QD + (h0 + hh) * HD + f * 32 + g * 8));

  f32x4 oacc[GH][NVF];
  float m_run[GH], l_run[GH];
#pragma unroll
  for (int hh = 0; hh < GH; ++hh) {
    m_run[hh] = NEG_INF;
    l_run[hh] = 0.f;
#pragma unroll
    for (int f = 0; f < NVF; ++f) oacc[hh][f] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int64_t blk_elems = (int64_t)KV_BS * HD;
  u32x4 stg[NLD];
  // units 0 .. NLD/2-1 of a thread are keys (one token per unit: one scale), the others values (four tokens per unit)
  static_assert(NLD % 2 == 0 && (NLD / 2) * NT == 2 * CH, "the first half of a thread's units are keys");
  float ksc[NLD / 2];
  f32x4 vsc[NLD / 2];
  // Block ids are fetched one pair ahead of the request that uses them, so the request never waits for the table.
  // A pair past the workgroup's last one is redirected to the last one (in bounds, never used).
  int id0 = 0, id1 = 0;
  auto fetch_ids = [&](int pr) __attribute__((always_inline)) {
    const int prc = min(pr, npairs_wg - 1);
    id0 = trow[min(prc * 2, last_blk)];
    id1 = trow[min(prc * 2 + 1, last_blk)];
  };
  auto request = [&]() __attribute__((always_inline)) {
    const int64_t off0 = ((int64_t)id0 * Hkv + j) * blk_elems;
    const int64_t off1 = ((int64_t)id1 * Hkv + j) * blk_elems;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int u = tid + i * NT, c = u / CH, within = u % CH;
      const uint16_t* src = (c < 2 ? kplane : vplane) + ((c & 1) ? off1 : off0) + within * 8;
      stg[i] = *reinterpret_cast<const u32x4*>(src);
      const float* sc = kvscale + kv_scale_offset((c & 1) ? id1 : id0, Hkv, j);
      if (i < NLD / 2) ksc[i] = sc[within & 15];                                        // key unit: token = unit % 16
      else vsc[i - NLD / 2] = *reinterpret_cast<const f32x4*>(sc + 16 + ((within >> 3) & 3) * 4);  // value unit: tokens 4t .. 4t+3
    }
  };
  auto copy_in = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const uint32_t w[4] = {stg[i].x, stg[i].y, stg[i].z, stg[i].w};
      u32x4 out;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        // word d holds elements 2d, 2d+1 of the unit; a value unit's element e belongs to token e % 4
        const float s0 = i < NLD / 2 ? ksc[i < NLD / 2 ? i : 0] : vsc[i < NLD / 2 ? 0 : i - NLD / 2][(2 * d) & 3];
        const float s1 = i < NLD / 2 ? ksc[i < NLD / 2 ? i : 0] : vsc[i < NLD / 2 ? 0 : i - NLD / 2][(2 * d + 1) & 3];
        // offset-binary codes u = q + 32768:  value = (u - 32768) * scale
        const float x0 = __builtin_fmaf((float)(w[d] & 0xffffu), s0, -32768.f * s0), x1 = __builtin_fmaf((float)(w[d] >> 16), s1, -32768.f * s1);
        const f16x2 h = __builtin_convertvector((f32x2){x0, x1}, f16x2);
        out[d] = __builtin_bit_cast(uint32_t, h);
      }
      kv[buf][tid + i * NT] = out;
    }
  };
  // masked = false: every key of the pair is visible to every query of the wavefront (the pair ends at or before its
  // first query position), so neither the scores nor the values need a mask; that is the case for all pairs but the
  // last one to three of a wavefront.  The argument is a literal at both call sites.
  auto compute = [&](int buf, int pr, const bool masked) __attribute__((always_inline)) {
    const int base = pr * 32;
    u32x4 kf0[NKF], kf1[NKF];
    u32x2 vf0[NVF], vf1[NVF];
    const u32x2* v0p = reinterpret_cast<const u32x2*>(&kv[buf][2 * CH]);
    const u32x2* v1p = reinterpret_cast<const u32x2*>(&kv[buf][3 * CH]);
#pragma unroll
    for (int f = 0; f < NKF; ++f) {
      kf0[f] = kv[buf][f * 64 + lane];
      kf1[f] = kv[buf][CH + f * 64 + lane];
    }
#pragma unroll
    for (int f = 0; f < NVF; ++f) {
      vf0[f] = v0p[f * 64 + lane];
      vf1[f] = v1p[f * 64 + lane];
    }
    // three passes over the GH heads (scores, softmax, values) rather than one head after the other: the heads are
    // independent, so each pass is a run of independent MFMAs or of independent cross-lane exchanges
    f32x4 s0[GH], s1[GH];
#pragma unroll
    for (int hh = 0; hh < GH; ++hh) {
      s0[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
      s1[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int f = 0; f < NKF; ++f)
#pragma unroll
      for (int hh = 0; hh < GH; ++hh) {
        s0[hh] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(kf0[f]), qf[hh][f], s0[hh], 0, 0, 0);
        s1[hh] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(kf1[f]), qf[hh][f], s1[hh], 0, 0, 0);
      }
    // Softmax numerators p = 2^(score * log2(e)/sqrt(hd) - m) with a per-query reference point m (m_run) that is not
    // necessarily the running maximum: the result o / l does not depend on it.  The common case takes no maximum at
    // all: the exponentials are formed against the current reference, and only if some lane's sum of its eight
    // numerators exceeds 256 (so a numerator might not fit fp16 comfortably; also true for a NaN or an infinity) or
    // on the first pair (no reference yet) the wavefront takes the exact maxima, moves the reference up, rescales o
    // and l and forms the exponentials again.  After the first pairs of a sequence that is rare, and the 4 * NVF
    // accumulator registers per head are then left alone.  Hidden keys (later than the query, or slots past the end
    // of the sequence, which may hold anything) enter as -inf and get p = 0.
    f16x8 pbv[GH];
#pragma unroll
    for (int hh = 0; hh < GH; ++hh) {
      float sr[8];  // raw scores
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sr[i] = (!masked || base + 4 * g + i <= qpos) ? s0[hh][i] : NEG_INF;
        sr[4 + i] = (!masked || base + 16 + 4 * g + i <= qpos) ? s1[hh][i] : NEG_INF;
      }
      float neg_m = (m_run[hh] == NEG_INF) ? 0.f : -m_run[hh];
      float pv[8];
      float psum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        pv[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sr[i], scale_log2, neg_m));
        psum += pv[i];
      }
      if (pr == 0 || __any(!(psum <= 256.f))) {
        float scl[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) scl[i] = sr[i] * scale_log2;
        float mx = fmaxf(fmaxf(fmaxf(scl[0], scl[1]), fmaxf(scl[2], scl[3])), fmaxf(fmaxf(scl[4], scl[5]), fmaxf(scl[6], scl[7])));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run[hh], mx);
        // a query whose visible keys all lie in later pairs has m_new = -inf here: keep its state untouched
        const float alpha = __builtin_amdgcn_exp2f(m_run[hh] - ((m_new == NEG_INF) ? 0.f : m_new));
        l_run[hh] *= alpha;
        m_run[hh] = m_new;
#pragma unroll
        for (int f = 0; f < NVF; ++f) {
          oacc[hh][f][0] *= alpha; oacc[hh][f][1] *= alpha; oacc[hh][f][2] *= alpha; oacc[hh][f][3] *= alpha;
        }
        neg_m = (m_new == NEG_INF) ? 0.f : -m_new;
        psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          pv[i] = __builtin_amdgcn_exp2f(scl[i] + neg_m);
          psum += pv[i];
        }
      }
      l_run[hh] += psum;
      // two values per conversion instruction, round to nearest even
      const f16x2 h01 = __builtin_convertvector((f32x2){pv[0], pv[1]}, f16x2), h23 = __builtin_convertvector((f32x2){pv[2], pv[3]}, f16x2);
      const f16x2 h45 = __builtin_convertvector((f32x2){pv[4], pv[5]}, f16x2), h67 = __builtin_convertvector((f32x2){pv[6], pv[7]}, f16x2);
      pbv[hh] = __builtin_shufflevector(__builtin_shufflevector(h01, h23, 0, 1, 2, 3), __builtin_shufflevector(h45, h67, 0, 1, 2, 3), 0, 1, 2, 3, 4, 5, 6, 7);
    }
    // slots past the end of the sequence may hold anything: keep them out of the MFMA (masks are all-ones elsewhere)
    uint32_t a01 = 0xFFFFFFFFu, a23 = 0xFFFFFFFFu, b01 = 0xFFFFFFFFu, b23 = 0xFFFFFFFFu;
    if (masked) {
      const int ka = base + 4 * g, kb2 = base + 16 + 4 * g;
      a01 = (ka + 0 < ctx ? 0xFFFFu : 0u) | (ka + 1 < ctx ? 0xFFFF0000u : 0u);
      a23 = (ka + 2 < ctx ? 0xFFFFu : 0u) | (ka + 3 < ctx ? 0xFFFF0000u : 0u);
      b01 = (kb2 + 0 < ctx ? 0xFFFFu : 0u) | (kb2 + 1 < ctx ? 0xFFFF0000u : 0u);
      b23 = (kb2 + 2 < ctx ? 0xFFFFu : 0u) | (kb2 + 3 < ctx ? 0xFFFF0000u : 0u);
    }
#pragma unroll
    for (int f = 0; f < NVF; ++f) {
      const u32x4 a = masked ? u32x4{vf0[f].x & a01, vf0[f].y & a23, vf1[f].x & b01, vf1[f].y & b23}
                             : u32x4{vf0[f].x, vf0[f].y, vf1[f].x, vf1[f].y};
#pragma unroll
      for (int hh = 0; hh < GH; ++hh)
        oacc[hh][f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_f16x8(a), pbv[hh], oacc[hh][f], 0, 0, 0);
    }
  };

  fetch_ids(0);
  request();
  fetch_ids(1);
  copy_in(0);
  __syncthreads();
  for (int pr = 0; pr < npairs_wg; ++pr) {
    request();          // pair pr + 1
    fetch_ids(pr + 2);
    __builtin_amdgcn_sched_barrier(0);
    if (pr < npairs) {
      if (pr * 32 + 31 <= prefix + qw0) compute(pr & 1, pr, false);
      else compute(pr & 1, pr, true);
    }
    __builtin_amdgcn_sched_barrier(0);
    copy_in((pr + 1) & 1);
    __syncthreads();
  }
  if (!active || n >= nq) return;
#pragma unroll
  for (int hh = 0; hh < GH; ++hh) {
    float l = l_run[hh];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const float inv = 1.f / l;
#pragma unroll
    for (int f = 0; f < NVF; ++f) {
      union { uint16_t s[4]; u32x2 v; } o;
#pragma unroll
      for (int i = 0; i < 4; ++i) o.s[i] = f32_to_f16_sat(oacc[hh][f][i] * inv);
      *reinterpret_cast<u32x2*>(op + packed_p_offset(row0 + n, (h0 + hh) * HD + f * 16 + g * 4, QD >> 4)) = o.v;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Host side

template <int EPI, bool QKN = false>
static void launch_pgemm(PGemmP& p, hipStream_t st) {
  if constexpr (EPI == PEPI_QKV && !QKN) {
    if (p.qk_gain) return launch_pgemm<EPI, true>(p, st);
  }
  p.n_tt = (p.T + 255) / 256;
  p.n_rt = (p.NRG + 15) / 16;
  if (p.wfactor == 0.f) p.wfactor = 1.f;  // not set: an unscaled matrix
  static bool lds_enabled = false;  // per instantiation: allow 128 KiB of dynamic LDS
  if (!lds_enabled) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_gemm_kernel<EPI, QKN>), hipFuncAttributeMaxDynamicSharedMemorySize,
                              PGEMM_LDS_BYTES);
    lds_enabled = true;
  }
  hipLaunchKernelGGL((prefill_gemm_kernel<EPI, QKN>), dim3(p.n_tt * p.n_rt), dim3(256), PGEMM_LDS_BYTES, st, p);
}

template <int HD>
static void launch_pattn(www_model* m, const uint16_t* kplane, const uint16_t* vplane, const float* kvscale, const int32_t* qlens, const int32_t* lens,
                         const int32_t* table, int max_tiles, hipStream_t st) {
  const int G = m->G;
  // two query heads per workgroup pass: their accumulators and operands fit 256 registers, so two workgroups share a
  // compute unit and one hides the other's softmax and LDS latencies (four heads per pass at one workgroup per unit: 1.5x slower)
  const int GH = (G % 2 == 0) ? 2 : 1;
  // with 128-wide heads two such head groups form one workgroup of eight wavefronts (still two per SIMD) and share
  // the copy of the keys and values into LDS, which halves the code-to-fp16 conversions per query head
  const int HG = (HD == 128 && (G / GH) % 2 == 0) ? 2 : 1;
  dim3 grid(max_tiles * m->Hkv * (G / GH / HG)), block(256 * HG);
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
  const int32_t* cum_rows = m->meta + 16;
#define PATTN(GH_, HG_)                                                                                                            \
  hipLaunchKernelGGL((prefill_attn_kernel<HD, GH_, HG_>), grid, block, 0, st, (const uint16_t*)m->qp, kplane, vplane, kvscale, qlens, lens, \
                     table,                                                                                                        \
                     (int)m->cfg.max_blocks_per_seq, m->Hq, m->Hkv, G, m->tile_seq, m->tile_q0, m->meta, cum_rows, scale_log2,      \
                     (uint16_t*)m->op, max_tiles)
  if constexpr (HD == 128) {
    if (HG == 2) { PATTN(2, 2); return; }
  }
  if (GH == 2) PATTN(2, 1); else PATTN(1, 1);
#undef PATTN
}

int run_prefill(www_model* m, const int32_t* tok, const int32_t* qlens, const int32_t* lens, const int32_t* table, int batch, int T,
                hipStream_t st) {
  const int d = m->d;
  int32_t* cum = m->meta + 16;
  hipLaunchKernelGGL(prefill_meta_kernel, dim3(1), dim3(1024), 0, st, tok, qlens, lens, batch, T, m->row_seq, m->row_pos, m->tile_seq,
                     m->tile_q0, m->meta, m->last_tok, cum);
  if (m->cfg.weight_dtype == WWW_DTYPE_F32)
    hipLaunchKernelGGL(embed_rows_kernel<float>, dim3(T), dim3(256), 0, st, tok, (const float*)m->embed, d, m->layers[0].attn_norm, m->hp,
                       (uint16_t*)m->xn, m->ssq_p);
  else
    hipLaunchKernelGGL(embed_rows_kernel<uint16_t>, dim3(T), dim3(256), 0, st, tok, (const uint16_t*)m->embed, d, m->layers[0].attn_norm,
                       m->hp, (uint16_t*)m->xn, m->ssq_p);
  int n_ssq = 1;
  const int n_rt_d = (d / 16 + 15) / 16;  // row tiles of a GEMM with d output rows
  const int max_tiles = T / ATTN_TQ + batch;
  for (int l = 0; l < m->L; ++l) {
    const LayerW& w = m->layers[l];
    uint16_t* kplane = (uint16_t*)m->kv + (int64_t)(2 * l) * m->kv_plane;
    uint16_t* vplane = (uint16_t*)m->kv + (int64_t)(2 * l + 1) * m->kv_plane;
    float* kvscale = m->kv_scales + (int64_t)l * m->kv_scale_plane;
    {
      PGemmP p = {};
      p.W = (const u32x4*)w.wqkv; p.wfactor = w.sqkv; p.NRG = m->QKVN / 16; p.KB = d / 32; p.X = (const u32x4*)m->xn; p.T = T;
      p.ssq_in = m->ssq_p; p.n_ssq_in = n_ssq; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
      p.qp = (uint16_t*)m->qp; p.kplane = kplane; p.vplane = vplane; p.kvscale = kvscale; p.row_seq = m->row_seq; p.row_pos = m->row_pos; p.table = table;
      p.mbs = m->cfg.max_blocks_per_seq; p.hd = m->hd; p.Hq = m->Hq; p.Hkv = m->Hkv; p.rope = m->rope; p.qk_gain = w.qk_gain;
      launch_pgemm<PEPI_QKV>(p, st);
    }
    if (l == m->L - 1) break;  // only this layer's keys and values are still needed
    if (m->hd == 128) launch_pattn<128>(m, kplane, vplane, kvscale, qlens, lens, table, max_tiles, st);
    else launch_pattn<64>(m, kplane, vplane, kvscale, qlens, lens, table, max_tiles, st);
    {
      PGemmP p = {};
      p.W = (const u32x4*)w.wo; p.wfactor = w.so; p.NRG = d / 16; p.KB = m->QD / 32; p.X = (const u32x4*)m->op; p.T = T;
      p.hp = m->hp; p.d = d; p.gain_next = w.ffn_norm; p.xn_out = (uint16_t*)m->xn; p.ssq_out = m->ssq_p;
      launch_pgemm<PEPI_RESID>(p, st);
      n_ssq = n_rt_d;
    }
    {
      PGemmP p = {};
      p.W = (const u32x4*)w.wgu; p.wfactor = w.sgu; p.NRG = 2 * m->F / 16; p.KB = d / 32; p.X = (const u32x4*)m->xn; p.T = T;
      p.ssq_in = m->ssq_p; p.n_ssq_in = n_ssq; p.inv_dim = 1.f / d; p.eps = m->cfg.rms_eps;
      p.ap = (uint16_t*)m->ap; p.Fp = m->Fp;
      launch_pgemm<PEPI_SWIGLU>(p, st);
    }
    {
      PGemmP p = {};
      p.W = (const u32x4*)w.wd; p.wfactor = w.sd; p.NRG = d / 16; p.KB = m->Fp / 32; p.X = (const u32x4*)m->ap; p.T = T;
      p.hp = m->hp; p.d = d; p.gain_next = m->layers[l + 1].attn_norm; p.xn_out = (uint16_t*)m->xn; p.ssq_out = m->ssq_p;
      launch_pgemm<PEPI_RESID>(p, st);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("prefill launch failed: %s", hipGetErrorString(e));
    return WWW_E_HIP;
  }
  return WWW_OK;
}

// Host-side view of the prefill GEMM's workgroup -> tile map (tests).
extern "C" __attribute__((visibility("default"))) int www_debug_prefill_tile(int32_t workgroup, int32_t token_tiles, int32_t row_tiles, int32_t* token_tile_out,
                                      int32_t* row_tile_out) {
  if (!token_tile_out || !row_tile_out || token_tiles < 1 || row_tiles < 1 || workgroup < 0 ||
      (int64_t)workgroup >= (int64_t)token_tiles * row_tiles || (int64_t)token_tiles * row_tiles > 0x7fffffff) {
    set_error("www_debug_prefill_tile: arguments out of range");
    return WWW_E_INVALID_ARG;
  }
  int tt, rt;
  pgemm_tile_of(workgroup, token_tiles, row_tiles, &tt, &rt);
  *token_tile_out = tt;
  *row_tile_out = rt;
  return WWW_OK;
}
