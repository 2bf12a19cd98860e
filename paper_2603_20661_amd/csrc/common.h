// Shared declarations of the gfx950 inference library: vector types, fp16 helpers, the layouts of
// packed weights / packed activations / KV-cache blocks, and the model handle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/www.h"

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // 16 raw bytes (native vector: stays in registers)
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

#define KV_BS 16  // tokens per KV block

// ------------------------------------------------------------------------------------------------
// Number format.  Every MFMA operand is IEEE fp16, stored as 16-bit patterns (uint16_t).  Weights that
// arrive in bf16 have 8 significant bits and convert to fp16 exactly for |w| >= 2^-17 (below that the
// absolute error is at most 2^-25); activations keep 11 significant bits instead of bf16's 8, which
// is what holds the logit error inside the tolerance; values are clamped to +-65504 on conversion.
// Where one fp16 is not enough (decode-path activations, fp32 weights) a value is carried as hi + lo.
//
// Layouts
//
// Packed weight matrix W[N][K] (out x in), K padded with zeros to KB*32:
//   fragment (rg, kb) = rows rg*16..+15, columns kb*32..+31, 1 KiB, stored lane-major for the
//   16x16x32 MFMA A operand: lane l holds row rg*16 + l%16, columns kb*32 + (l/16)*8 .. +7.
//   Fragments are ordered k block first: element offset = ((kb*NRG + rg)*64 + l)*8 + e (NRG = N/16), so the
//   workgroups of a GEMM, which walk K in step, read one contiguous region per k block - no HBM channel sees a
//   power-of-two stride.
//   Rows may be permuted at pack time (packed row p <-> source row, see pack.hip):
//     QKV: inside each q and k head, p = 2i -> i, p = 2i+1 -> i + hd/2  (rotary pairs adjacent)
//     gate/up: row-group 2j = gate rows 16j..16j+15, row-group 2j+1 = up rows 16j..16j+15
//
// Packed activations X[M][K] for the decode path, tokens in groups of 16 (MT groups), hi/lo split:
//   fragment (kb, tb, hl) = tokens tb*16..+15, columns kb*32..+31 as the MFMA B operand:
//   lane l holds token tb*16 + l%16, columns kb*32 + (l/16)*8 .. +7; x = hi + lo with hi = fp16(x).
//   element offset = (((kb*MT + tb)*2 + hl)*64 + l)*8 + e.
//
// Packed activations X[T][K] for the prefill path (fp16, no hi/lo), tokens in groups of 32, columns in steps of 16:
//   fragment (tb, ks) = tokens tb*32..+31, columns ks*16..+15 = B operand of the 32x32x16 MFMA:
//   lane l holds token tb*32 + l%32, columns ks*16 + (l/32)*8 .. +7;  element offset = ((tb*(K/16) + ks)*64 + l)*8 + e.
//   Buffers are sized for the token count rounded up to 256.
//
// KV pool: [layer][K|V][block][kv head][16 tokens x hd] 16-bit codes, then [layer][block][kv head][K|V][16 tokens] fp32
// scales.  A key or value vector (one token, one kv head) is stored as hd 16-bit integers q with one fp32 scale
// s = max|x| / 32767:  x ~ q * s,  q = round(x / s), kept in offset-binary form u = q + 32768 (1 .. 65535), whose two
// bytes feed the matrix cores without a sign fix-up.  Against an fp16 copy of the same size (11 significant bits
// everywhere) the uniform step of s is 4-5 times finer on the elements that matter, which is what holds the greedy
// agreement of deep models: measured with the oracle alone, rounding the cache to fp16 after every call moves the
// logits of the 32-layer 8B-shaped model by 1.4e-2 (mean of the row maxima), these codes by 1.5e-3.
// Inside one (block, head) the codes sit where the matrix-core operands want them:
//   K (head-dim in rotary-interleaved order c): offset = ((c/32)*64 + ((c%32)/8)*16 + tok)*8 + c%8
//        -> fragment c/32 is the A operand of S^T = K Q^T for those 32 dims.
//   V (head-dim in natural order c):           offset = ((c/16)*64 + (tok/4)*16 + c%16)*4 + tok%4
//        -> fragment c/16 is the A operand (V^T rows c, 4 keys per lane) of O^T = V^T P^T.
// ------------------------------------------------------------------------------------------------

__host__ __device__ inline int64_t packed_w_elems(int64_t N, int64_t KB) { return N * KB * 32; }

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// fp32 -> fp16 bit pattern, round to nearest even, saturating instead of overflowing to infinity
__device__ __forceinline__ uint16_t f32_to_f16_sat(float f) {
  f = fminf(fmaxf(f, -65504.f), 65504.f);
  return __builtin_bit_cast(uint16_t, (_Float16)f);
}
__device__ __forceinline__ float f16_bits_to_float(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
// x = hi + lo, about 22 significant bits
__device__ __forceinline__ void split_f16(float x, uint16_t& hi, uint16_t& lo) {
  hi = f32_to_f16_sat(x);
  lo = f32_to_f16_sat(x - f16_bits_to_float(hi));
}

__device__ __forceinline__ int64_t packed_p_offset(int64_t t, int k, int K16) {
  return (((t >> 5) * K16 + (k >> 4)) * 64 + ((k & 15) >> 3) * 32 + (t & 31)) * 8 + (k & 7);
}

__device__ __forceinline__ int k_cache_offset(int tok, int c) { return ((c >> 5) * 64 + ((c & 31) >> 3) * 16 + tok) * 8 + (c & 7); }
__device__ __forceinline__ int v_cache_offset(int tok, int c) { return ((c >> 4) * 64 + (tok >> 2) * 16 + (c & 15)) * 4 + (tok & 3); }

// 16-bit code of x for a vector whose largest magnitude is amax: inv = 32767 / amax (0 for an all-zero vector)
__device__ __forceinline__ float kv_code_inv(float amax) { return amax > 0.f ? 32767.f / amax : 0.f; }
__device__ __forceinline__ float kv_code_scale(float amax) { return amax * (1.f / 32767.f); }  // (NaN stays NaN: it poisons what reads it)
__device__ __forceinline__ uint16_t kv_code(float x, float inv) {
  const float q = fminf(fmaxf(rintf(x * inv), -32767.f), 32767.f);
  return (uint16_t)((int)q + 32768);  // offset binary
}
// scales of (block blk, kv head j): K scales of the 16 tokens at +0, V scales at +16
__device__ __forceinline__ int64_t kv_scale_offset(int64_t blk, int Hkv, int j) { return (blk * Hkv + j) * 32; }

// physical token slot of logical position pos of a sequence with block-table row `row`
// (split in two so that a kernel can issue the table load early and finish the arithmetic where the slot is used)
__device__ __forceinline__ int32_t kv_block_id(const int32_t* __restrict__ row, int pos) { return row[pos / KV_BS]; }
__device__ __forceinline__ int64_t kv_slot_in_block(int32_t block_id, int pos) { return (int64_t)block_id * KV_BS + (pos % KV_BS); }
__device__ __forceinline__ int64_t kv_slot(const int32_t* __restrict__ row, int pos) {
  return kv_slot_in_block(kv_block_id(row, pos), pos);
}

// ------------------------------------------------------------------------------------------------
struct LayerW {
  const uint16_t *wqkv, *wqkv_lo, *wo, *wo_lo, *wgu, *wgu_lo, *wd, *wd_lo;  // packed fp16 (lo planes only for fp32 sources)
  const uint8_t *wqkv8, *wo8, *wgu8, *wd8;  // weight-only quantised models: packed codes for the decode path ...
  float sqkv, so, sgu, sd;                  // ... FP8: the matrices' scales (1 otherwise)
  const void *gqkv, *go, *ggu, *gd;         // ... int4: group scales as fp16, [chunk of 4 k blocks][packed row][4]
  const float *attn_norm, *ffn_norm;
  const float* qk_gain;  // models with normalised query / key heads: [2][hd] gains (q, then k) in packed row order, else null
};

struct GraphEntry {
  const void *tok, *lens, *table, *logits, *next;
  int batch;
  hipStream_t stream;
  hipGraphExec_t exec;
};

struct www_model {
  www_config cfg;
  int L, d, Hq, Hkv, hd, G, F, Fp, V, QKVN, QD, KD, max_pos, maxB, MTmax, maxT;
  bool wsplit;
  bool fp8;  // FP8 weight-only source
  int int4_group;  // 128 or 32 for an int4 weight-only source, else 0
  const uint8_t* lm_head8;
  float s_lm;
  const void* g_lm;
  // weights (inside the workspace)
  LayerW* layers;  // host array
  const void* embed;  // [V][d] in the source dtype
  const uint16_t *lm_head, *lm_head_lo;
  const float* final_norm;
  const float2* rope;  // [max_pos][hd/2] (cos, sin)
  // KV pool
  uint16_t* kv;  // 16-bit codes
  int64_t kv_plane;  // elements per (layer, K|V) plane = num_blocks * Hkv * 16 * hd
  float* kv_scales;  // behind the code planes: [layer][block][kv head][K|V][16] fp32
  int64_t kv_scale_plane;  // floats per layer = num_blocks * Hkv * 32
  // decode-path buffers
  float* h;        // [maxB][d] residual stream
  float* ssq;      // [maxB][SSQ_TILES] partial sums of squares of h, one per row tile of the producing GEMM
  uint16_t *q_hi, *q_lo;  // [maxB][QD] rotated, pre-scaled queries as fp16 hi + lo
  uint16_t* xq;        // packed activations feeding the QKV / gate-up / lm_head GEMMs (K = d)
  uint16_t* xo;        // packed attention output feeding the O projection (K = QD)
  uint16_t* xa;        // packed SwiGLU output feeding the down projection (K = Fp)
  float* partial;  // split-K partial tiles
  float* attn_part;
  int *attn_hdr, *attn_start, *attn_pref;  // per-step plan of the decode attention: totals, per-wavefront start, prefix of pair counts
  float* argmax_val;  // [maxB][32] per-slice maxima of the logits and
  int* argmax_idx;    // their indices
  unsigned long long* counters;  // split-K arrival counters
  int* fault_host;  // pinned host words: [0] set by the kernels when the placement rule of the split-K hand-over is violated,
  int* fault_dev;   // (its device address); [1], [2] receive the result words of the argument validation
  int validate;     // 1: every call first checks its device-resident arguments (WWW_VALIDATE=1 at load)
  int* val_words;   // device: [0] flags of what the check found, [1] sum of the new-token counts
  unsigned* val_bitmap;  // device: one bit per KV block, to find a block that is named twice
  uint64_t val_bitmap_bytes;
  float* logits_buf;  // used when the caller passes no logits buffer
  int* last_tok;      // [maxB] tokens of the last prompt position (prefill)
  // prefill-path buffers
  float* hp;       // residual stream of the prefill path in 256 x 256 blocks of accumulator order (see prefill.hip)
  float* ssq_p;    // [d/256][maxT rounded to 256] partial sums of squares of hp
  uint16_t* xn;        // packed [maxT][d] normalised activations
  uint16_t* qp;    // [maxT][QD] rotated queries, fp16 (interleaved head-dim order)
  uint16_t* op;        // packed [maxT][QD] attention output
  uint16_t* ap;        // packed [maxT][Fp] SwiGLU output
  int *row_seq, *row_pos, *tile_seq, *tile_q0, *meta;  // ragged-batch bookkeeping
  int attn_waves;  // wavefronts of the decode attention grid (all resident at once)
  int handover_fence;  // 1: split-K partial tiles get a device-scope release fence (placement rule not confirmed)
  int attn_maxrec; // most partial records per (sequence, kv head)
  GraphEntry* graphs;
  int n_graphs;
  int use_graph;
  struct DecodeProfiler* prof;  // per-kernel-class timing of eager decode steps (benchmark hook), or null
};

#define MAX_ATTN_WAVES 8192  // upper bound of the decode attention grid, in wavefronts (sizes its plan buffer)
#define PSSQ 32            // entries per token of the prefill path's sum-of-squares table (d_model / 256 row tiles at most)
#define SSQ_TILES 64       // most row tiles of a residual-producing GEMM (d_model / 128)
#define GEMM_TILE_ROWS 128 // rows of W per workgroup of the skinny GEMM
#define MAX_KSPLIT 16

// decode kernel classes reported by the profiling hook
enum { PK_EMBED = 0, PK_QKV, PK_ATTN, PK_OPROJ, PK_GATEUP, PK_DOWN, PK_LMHEAD, PK_ARGMAX, PK_COUNT };
void prof_mark(www_model* m, int cls, hipStream_t st);  // records an event in front of the next launch when profiling is on

// host-side launchers (decode.hip / prefill.hip / pack.hip)
void set_error(const char* fmt, ...);
int launch_pack_int4(const void* codes, const void* scales_bf16, int N, int K, int KB, int group, int mode, int hd, int n_rot_rows, int F,
                     uint16_t* f16_plane, uint8_t* codes_out, void* scales_out, hipStream_t st);
int launch_pack_qk_gain(const float* q_src, const float* k_src, int hd, float* out, hipStream_t st);
int launch_pack_fp8(const void* src, int N, int K, int KB, int mode, int hd, int n_rot_rows, int F, uint8_t* out, hipStream_t st);
int decode_attn_resident_waves(int hd, int G);
int decode_probe_placement(int32_t* scratch_dev, int n, hipStream_t st);
int run_decode(www_model* m, const int32_t* tok, const int32_t* lens, const int32_t* table, int batch, float* logits, int32_t* next,
               hipStream_t st);
int run_prefill(www_model* m, const int32_t* tok, const int32_t* qlens, const int32_t* lens, const int32_t* table, int batch, int T,
                hipStream_t st);
int launch_pack_matrix(const void* src, int src_dtype, int N, int K, int KB, int mode, int hd, int n_rot_rows, int F, uint16_t* hi, uint16_t* lo,
                       hipStream_t st);
int launch_debug_slots(const int32_t* row, const int32_t* pos, int n, int64_t* out, hipStream_t st);
