// C ABI (include/www.h): argument checks, workspace plan, weight packing at load, prefill,
// graph-captured decode step.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "common.h"

// the library is built with hidden visibility; only the C ABI is exported
#define WWW_EXPORT extern "C" __attribute__((visibility("default")))

int decode_gemm_ksplit(int NRG, int KB, int MT);
int decode_MT(int batch);

static thread_local char g_err[512] = "";

// Captured decode steps kept per model, one per (batch, argument pointers, stream); a serving loop whose batch grows and
// shrinks one sequence at a time passes through about a hundred batch sizes.
static const int MAX_GRAPHS = 128;

// Benchmark hook: while enabled, decode steps run eagerly and an event is recorded in front of every
// kernel; the elapsed time between consecutive events is charged to the class of the kernel in between.
struct DecodeProfiler {
  bool on = false;
  std::vector<hipEvent_t> ev;
  std::vector<int> cls;
  size_t used = 0;
};

void prof_mark(www_model* m, int cls, hipStream_t st) {
  DecodeProfiler* p = m->prof;
  if (!p || !p->on) return;
  if (p->used == p->ev.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    p->ev.push_back(e);
    p->cls.push_back(cls);
  }
  p->cls[p->used] = cls;
  (void)hipEventRecord(p->ev[p->used], st);
  ++p->used;
}

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

#define HIP_TRY(x)                                                       \
  do {                                                                   \
    hipError_t e_ = (x);                                                 \
    if (e_ != hipSuccess) {                                              \
      set_error("%s failed: %s", #x, hipGetErrorString(e_));             \
      return WWW_E_HIP;                                                  \
    }                                                                    \
  } while (0)

static int check_config(const www_config* c) {
  if (!c) { set_error("config is NULL"); return WWW_E_INVALID_ARG; }
  if (c->abi_version != WWW_ABI_VERSION) { set_error("abi_version %u, library has %u", c->abi_version, WWW_ABI_VERSION); return WWW_E_ABI_MISMATCH; }
  const char* why = nullptr;
  if (c->n_layers == 0 || c->d_model == 0 || c->vocab == 0 || c->ffn_dim == 0 || c->n_kv_heads == 0) why = "zero dimension";
  else if (c->head_dim != 64 && c->head_dim != 128) why = "head_dim must be 64 or 128";
  else if (c->d_model % 128 || c->d_model > 128 * SSQ_TILES) why = "d_model must be a multiple of 128, at most 8192";
  else if (c->ffn_dim % 16) why = "ffn_dim must be a multiple of 16";
  else if (c->vocab % 16) why = "vocab must be a multiple of 16";
  else if (c->n_q_heads % c->n_kv_heads) why = "n_q_heads must be a multiple of n_kv_heads";
  else if (int g = c->n_q_heads / c->n_kv_heads; g != 1 && g != 2 && g != 4 && g != 8) why = "query heads per kv head must be 1, 2, 4 or 8";
  else if (c->kv_block_size != KV_BS) why = "kv_block_size must be 16";
  else if (c->weight_dtype > 4) why = "weight_dtype must be 0 (fp32), 1 (bf16), 2 (FP8 weight-only), 3 or 4 (int4 weight-only, groups of 128 / 32)";

  else if (c->max_batch == 0 || c->max_batch > 1024) why = "max_batch must be in 1..1024";
  else if (c->max_blocks_per_seq == 0 || c->num_kv_blocks == 0) why = "empty KV pool";
  else if (c->num_kv_blocks > 0x7fffffffull) why = "num_kv_blocks must fit int32";
  else if (c->max_prefill_tokens == 0) why = "max_prefill_tokens must be positive";
  else if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) why = "bad rms_eps / rope_theta";
  else if (c->flags & ~WWW_FLAG_QK_NORM) why = "unknown bits in flags";
  if (!why && c->weight_dtype >= WWW_DTYPE_INT4WO_128) {
    const uint32_t g = c->weight_dtype == WWW_DTYPE_INT4WO_128 ? 128u : 32u;
    if (c->d_model % g || (c->n_q_heads * c->head_dim) % g || c->ffn_dim % g)
      why = "int4 weight-only: d_model, n_q_heads * head_dim and ffn_dim must be multiples of the group size";
  }
  if (why) { set_error("unsupported configuration: %s", why); return WWW_E_BAD_CONFIG; }
  return WWW_OK;
}

// The unfenced split-K hand-over relies on a placement rule that is probed at load and re-checked by the kernels.  If
// a kernel has reported a violation, results since the last check are unreliable: switch the model to the fenced
// hand-over (cached graphs hold the old kernel arguments and are dropped) and tell the caller.
static int check_placement_fault(www_model* m) {
  if (!m->fault_host || !*m->fault_host) return WWW_OK;
  *m->fault_host = 0;
  m->handover_fence = 1;
  for (int i = 0; i < m->n_graphs; ++i) (void)hipGraphExecDestroy(m->graphs[i].exec);
  m->n_graphs = 0;
  set_error("split-K partners ran on different XCDs: results of the calls since the last successful one are unreliable; "
            "the model now uses the fenced hand-over, repeat those calls");
  return WWW_E_STALE;
}

static uint64_t align256(uint64_t n) { return (n + 255) / 256 * 256; }

// byte offsets of everything inside the workspace
struct Plan {
  uint64_t total;
  uint64_t embed, final_norm, lm_head, lm_head_lo, rope;
  std::vector<uint64_t> attn_norm, ffn_norm, wqkv, wqkv_lo, wo, wo_lo, wgu, wgu_lo, wd, wd_lo;
  std::vector<uint64_t> wqkv8, wo8, wgu8, wd8;  // weight-only quantised models: packed codes for the decode path
  std::vector<uint64_t> gqkv, go, ggu, gd;      // int4: group scales for the decode path
  std::vector<uint64_t> qk_gain;                // gains of the query / key head normalisation, in packed row order
  uint64_t lm_head8, g_lm;
  uint64_t zero_begin, zero_end;  // region cleared at load (counters, padded activation buffers)
  uint64_t h, ssq, q, xq, xo, xa, partial, attn_part, counters, logits, last_tok, argmax_val, argmax_idx, attn_hdr, attn_start, attn_pref;
  uint64_t hp, ssq_p, xn, qp, op, ap, row_seq, row_pos, tile_seq, tile_q0, meta;
  uint64_t val_words, val_bitmap, val_bitmap_bytes;  // argument validation (WWW_VALIDATE=1): result words, one bit per KV block
  int attn_maxrec;
};

struct Dims {
  int L, d, Hq, Hkv, hd, G, F, Fp, V, QKVN, QD, KD, maxB, MTmax, maxT, max_pos;
  bool wsplit, fp8, qk_norm;
  int int4_group;  // 0: not an int4 source
};

static Dims dims_of(const www_config* c) {
  Dims s;
  s.L = c->n_layers; s.d = c->d_model; s.Hq = c->n_q_heads; s.Hkv = c->n_kv_heads; s.hd = c->head_dim; s.G = s.Hq / s.Hkv;
  s.F = c->ffn_dim; s.Fp = (s.F + 31) / 32 * 32; s.V = c->vocab;
  s.QD = s.Hq * s.hd; s.KD = s.Hkv * s.hd; s.QKVN = s.QD + 2 * s.KD;
  s.maxB = c->max_batch; s.MTmax = decode_MT(s.maxB); s.maxT = c->max_prefill_tokens;
  s.max_pos = c->max_blocks_per_seq * KV_BS;
  s.wsplit = c->weight_dtype == WWW_DTYPE_F32;
  s.fp8 = c->weight_dtype == WWW_DTYPE_FP8WO;
  s.qk_norm = (c->flags & WWW_FLAG_QK_NORM) != 0;
  s.int4_group = c->weight_dtype == WWW_DTYPE_INT4WO_128 ? 128 : c->weight_dtype == WWW_DTYPE_INT4WO_32 ? 32 : 0;
  return s;
}

static void make_plan(const www_config* c, Plan& p) {
  const Dims s = dims_of(c);
  uint64_t off = 0;
  auto take = [&](uint64_t bytes) { uint64_t o = off; off += align256(bytes); return o; };
  const uint64_t wb = s.wsplit ? 4 : 2;
  p.embed = take((uint64_t)s.V * s.d * wb);
  p.final_norm = take((uint64_t)s.d * 4);
  // FP8 codes in decode order: N rows x ceil(KB / 2) pairs of k blocks x 64 bytes
  // int4 codes in decode order: N rows x ceil(KB / 4) chunks x 64 bytes; their scales: 8 bytes per row and chunk
  const bool quant = s.fp8 || s.int4_group;
  auto fp8_bytes = [&](uint64_t N, uint64_t K) {
    const uint64_t KB = (K + 31) / 32;
    return s.int4_group ? N * ((KB + 3) / 4) * 64 : N * ((KB + 1) / 2) * 64;
  };
  auto gscale_bytes = [&](uint64_t N, uint64_t K) { return N * (((K + 31) / 32 + 3) / 4) * 8; };
  p.lm_head = quant ? 0 : take((uint64_t)s.V * s.d * 2);  // the output head is only ever streamed by the decode path
  p.lm_head_lo = s.wsplit ? take((uint64_t)s.V * s.d * 2) : 0;
  p.lm_head8 = quant ? take(fp8_bytes(s.V, s.d)) : 0;
  p.g_lm = s.int4_group ? take(gscale_bytes(s.V, s.d)) : 0;
  p.rope = take((uint64_t)s.max_pos * (s.hd / 2) * 8);
  for (int l = 0; l < s.L; ++l) {
    p.attn_norm.push_back(take((uint64_t)s.d * 4));
    p.ffn_norm.push_back(take((uint64_t)s.d * 4));
    p.wqkv.push_back(take((uint64_t)s.QKVN * s.d * 2));
    p.wqkv_lo.push_back(s.wsplit ? take((uint64_t)s.QKVN * s.d * 2) : 0);
    p.wo.push_back(take((uint64_t)s.d * s.QD * 2));
    p.wo_lo.push_back(s.wsplit ? take((uint64_t)s.d * s.QD * 2) : 0);
    p.wgu.push_back(take((uint64_t)2 * s.F * s.d * 2));
    p.wgu_lo.push_back(s.wsplit ? take((uint64_t)2 * s.F * s.d * 2) : 0);
    p.wd.push_back(take((uint64_t)s.d * s.Fp * 2));
    p.wd_lo.push_back(s.wsplit ? take((uint64_t)s.d * s.Fp * 2) : 0);
    p.wqkv8.push_back(quant ? take(fp8_bytes(s.QKVN, s.d)) : 0);
    p.wo8.push_back(quant ? take(fp8_bytes(s.d, s.QD)) : 0);
    p.wgu8.push_back(quant ? take(fp8_bytes(2 * (uint64_t)s.F, s.d)) : 0);
    p.wd8.push_back(quant ? take(fp8_bytes(s.d, s.Fp)) : 0);
    p.gqkv.push_back(s.int4_group ? take(gscale_bytes(s.QKVN, s.d)) : 0);
    p.go.push_back(s.int4_group ? take(gscale_bytes(s.d, s.QD)) : 0);
    p.ggu.push_back(s.int4_group ? take(gscale_bytes(2 * (uint64_t)s.F, s.d)) : 0);
    p.gd.push_back(s.int4_group ? take(gscale_bytes(s.d, s.Fp)) : 0);
    p.qk_gain.push_back(s.qk_norm ? take((uint64_t)2 * s.hd * 4) : 0);
  }
  p.zero_begin = off;
  const uint64_t Mpad = (uint64_t)s.MTmax * 16;
  p.counters = take((uint64_t)65536 * 8);
  p.h = take(Mpad * s.d * 4);
  p.ssq = take((uint64_t)SSQ_TILES * s.maxB * 4);
  p.q = take(Mpad * s.QD * 4);
  p.xq = take(Mpad * s.d * 4);
  p.xo = take(Mpad * s.QD * 4);
  p.xa = take(Mpad * s.Fp * 4);
  uint64_t part = 0;
  {
    const int N[5] = {s.QKVN, s.d, 2 * s.F, s.d, s.V};
    const int K[5] = {s.d, s.QD, s.d, s.Fp, s.d};
    for (int i = 0; i < 5; ++i)
      for (int mt = 1; mt <= s.MTmax; mt = mt < 4 ? mt * 2 : mt + 4) {  // every token-group count a batch can produce
        uint64_t ks = decode_gemm_ksplit(N[i] / 16, K[i] / 32, mt);
        uint64_t bytes = ks * mt * 16 * (((uint64_t)N[i] + 127) / 128 * 128) * 4;  // whole 128-row tiles are parked
        if (ks > 1 && bytes > part) part = bytes;
      }
  }
  p.partial = take(part ? part : 256);
  // a wavefront of the decode attention takes at least 16 key pairs (512 keys) of the batch's work list, so a sequence
  // is cut into at most max_pos / 512 + 2 segments
  p.attn_maxrec = s.max_pos / 512 + 2;
  p.attn_part = take((uint64_t)s.maxB * s.Hkv * p.attn_maxrec * s.G * (s.hd + 4) * 4);
  p.logits = take((uint64_t)s.maxB * s.V * 4);
  p.last_tok = take((uint64_t)s.maxB * 4);
  p.attn_hdr = take(16);
  p.attn_start = take((uint64_t)MAX_ATTN_WAVES * 16);
  p.attn_pref = take(((uint64_t)s.maxB + 1) * 4);
  p.argmax_val = take((uint64_t)s.maxB * 32 * 4);
  p.argmax_idx = take((uint64_t)s.maxB * 32 * 4);
  const uint64_t Tpad = ((uint64_t)s.maxT + 255) / 256 * 256;  // packed activation buffers hold whole 256-token tiles
  p.hp = take(Tpad * (((uint64_t)s.d + 255) / 256 * 256) * 4);  // residual stream in whole 256 x 256 blocks (accumulator order)
  p.ssq_p = take(Tpad * (uint64_t)PSSQ * 4);
  p.xn = take(Tpad * s.d * 2);
  p.qp = take((uint64_t)s.maxT * s.QD * 2);
  p.op = take(Tpad * s.QD * 2);
  p.ap = take(Tpad * s.Fp * 2);
  p.row_seq = take((uint64_t)s.maxT * 4);
  p.row_pos = take((uint64_t)s.maxT * 4);
  const uint64_t max_tiles = (uint64_t)s.maxT / 64 + s.maxB + 1;
  p.tile_seq = take(max_tiles * 4);
  p.tile_q0 = take(max_tiles * 4);
  p.meta = take((16 + 2 * ((uint64_t)s.maxB + 1)) * 4);
  p.val_words = take(256);
  p.val_bitmap_bytes = ((uint64_t)c->num_kv_blocks + 31) / 32 * 4;
  p.val_bitmap = take(p.val_bitmap_bytes);
  p.zero_end = off;
  p.total = off;
}

// bytes of one matrix in the source blob (an FP8 matrix is followed by a 256-byte slot with its scale)
static uint64_t blob_matrix_bytes(const Dims& s, uint64_t N, uint64_t K) {
  if (s.int4_group) return align256(N * K / 2) + align256(N * (K / s.int4_group) * 2);  // codes, then bf16 group scales
  return s.fp8 ? align256(N * K) + 256 : align256(N * K * (s.wsplit ? 4 : 2));
}

static uint64_t blob_bytes(const www_config* c) {
  const Dims s = dims_of(c);
  const uint64_t wb_embed = s.wsplit ? 4 : 2;  // the embedding of an FP8 weight-only model is bf16
  uint64_t off = align256((uint64_t)s.V * s.d * wb_embed);
  for (int l = 0; l < s.L; ++l)
    off += align256((uint64_t)s.d * 4) * 2 + blob_matrix_bytes(s, s.QKVN, s.d) + blob_matrix_bytes(s, s.d, s.QD) +
           blob_matrix_bytes(s, 2 * (uint64_t)s.F, s.d) + blob_matrix_bytes(s, s.d, s.F) +
           (s.qk_norm ? 2 * align256((uint64_t)s.hd * 4) : 0);
  off += align256((uint64_t)s.d * 4) + blob_matrix_bytes(s, s.V, s.d);
  return off;
}

// ------------------------------------------------------------------------------------------------
// Opt-in validation of the device-resident arguments of a call (environment variable WWW_VALIDATE=1, read when a model
// is loaded).  One small kernel checks every token id, every length and every block id the call would use and marks
// each block in a bitmap (a block named twice is an error); the host waits for it and launches nothing else if
// anything is out of range.
enum { VAL_TOKEN = 1, VAL_LENGTH = 2, VAL_BLOCK = 4, VAL_DUPLICATE = 8, VAL_TOTAL = 16 };

__global__ __launch_bounds__(256) void validate_args_kernel(const int32_t* __restrict__ tokens, int n_tokens, const int32_t* __restrict__ q_lens,
                                                            const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ table,
                                                            int batch, int mbs, int vocab, int64_t num_blocks,
                                                            unsigned* __restrict__ bitmap, int* __restrict__ out) {
  const int stride = gridDim.x * 256, first = blockIdx.x * 256 + threadIdx.x;
  unsigned bad = 0;
  long long qsum = 0;
  for (int i = first; i < n_tokens; i += stride)
    if (tokens[i] < 0 || tokens[i] >= vocab) bad |= VAL_TOKEN;
  for (int b = first; b < batch; b += stride) {
    const int q = q_lens ? q_lens[b] : 1, n = seq_lens[b];
    if (q < 1 || n < q || n > mbs * KV_BS) bad |= VAL_LENGTH;
    qsum += q;
  }
  // block-table entries in use: entry j of row b for j < ceil(seq_lens[b] / 16) (rows with a bad length are skipped)
  for (long long e = first; e < (long long)batch * mbs; e += stride) {
    const int b = (int)(e / mbs), j = (int)(e % mbs), n = seq_lens[b];
    if (n < 1 || n > mbs * KV_BS || j >= (n + KV_BS - 1) / KV_BS) continue;
    const int id = table[e];
    if (id < 0 || id >= num_blocks) { bad |= VAL_BLOCK; continue; }
    const unsigned bit = 1u << (id & 31);
    if (atomicOr(&bitmap[id >> 5], bit) & bit) bad |= VAL_DUPLICATE;
  }
  if (bad) atomicOr((unsigned*)&out[0], bad);
  if (qsum) atomicAdd(&out[1], (int)qsum);
}

// Runs the check on `st` and waits for it.  WWW_OK, or WWW_E_INVALID_ARG with a message naming what was found.
static int validate_device_args(www_model* m, const int32_t* tokens, int n_tokens, const int32_t* q_lens, const int32_t* seq_lens,
                                const int32_t* table, int batch, hipStream_t st) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone) {
    set_error("WWW_VALIDATE=1 waits for the stream and cannot run on a stream that is being captured");
    return WWW_E_INVALID_ARG;
  }
  HIP_TRY(hipMemsetAsync(m->val_words, 0, 256, st));
  HIP_TRY(hipMemsetAsync(m->val_bitmap, 0, m->val_bitmap_bytes, st));
  const long long work = (long long)batch * m->cfg.max_blocks_per_seq > n_tokens ? (long long)batch * m->cfg.max_blocks_per_seq : n_tokens;
  int grid = (int)((work + 255) / 256);
  if (grid < 1) grid = 1;
  if (grid > 1024) grid = 1024;
  hipLaunchKernelGGL(validate_args_kernel, dim3(grid), dim3(256), 0, st, tokens, n_tokens, q_lens, seq_lens, table, batch,
                     (int)m->cfg.max_blocks_per_seq, m->V, (int64_t)m->cfg.num_kv_blocks, m->val_bitmap, m->val_words);
  HIP_TRY(hipGetLastError());
  HIP_TRY(hipMemcpyAsync(m->fault_host + 1, m->val_words, 8, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  const int flags = m->fault_host[1], qsum = m->fault_host[2];
  int bad = flags | (!(flags & VAL_LENGTH) && qsum != n_tokens ? VAL_TOTAL : 0);
  if (!bad) return WWW_OK;
  set_error("device arguments rejected (WWW_VALIDATE=1):%s%s%s%s%s; nothing was launched",
            bad & VAL_TOKEN ? " token id outside [0, vocab)" : "", bad & VAL_LENGTH ? " lengths violate 1 <= q_len <= seq_len <= 16 * max_blocks_per_seq" : "",
            bad & VAL_BLOCK ? " block id outside [0, num_kv_blocks)" : "", bad & VAL_DUPLICATE ? " a block id is used twice in the call" : "",
            bad & VAL_TOTAL ? " the lengths of the new tokens do not add up to total_q_tokens" : "");
  return WWW_E_INVALID_ARG;
}

WWW_EXPORT int www_query_sizes(const www_config* cfg, uint64_t* weight_blob_bytes, uint64_t* kv_pool_bytes, uint64_t* workspace_bytes) {
  int rc = check_config(cfg);
  if (rc) return rc;
  const Dims s = dims_of(cfg);
  Plan p;
  make_plan(cfg, p);
  if (weight_blob_bytes) *weight_blob_bytes = blob_bytes(cfg);
  // 16-bit codes of every key and value element, then one fp32 scale per (token, kv head, K|V)
  if (kv_pool_bytes) *kv_pool_bytes = (uint64_t)cfg->num_kv_blocks * s.L * 2 * s.Hkv * KV_BS * (s.hd * 2 + 4);
  if (workspace_bytes) *workspace_bytes = p.total;
  return WWW_OK;
}

WWW_EXPORT int www_model_load(const www_config* cfg, const void* weights_dev, void* kv_pool_dev, void* workspace_dev, void* hip_stream,
                              www_model** out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!weights_dev || !kv_pool_dev || !workspace_dev || !out) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  if (((uintptr_t)weights_dev | (uintptr_t)kv_pool_dev | (uintptr_t)workspace_dev) & 255) { set_error("device buffers must be 256-byte aligned"); return WWW_E_INVALID_ARG; }
  hipStream_t st = (hipStream_t)hip_stream;
  const Dims s = dims_of(cfg);
  Plan p;
  make_plan(cfg, p);
  char* ws = (char*)workspace_dev;
  const char* blob = (const char*)weights_dev;
  const uint64_t wb = s.wsplit ? 4 : 2;
  const int dt = (int)cfg->weight_dtype;

  HIP_TRY(hipMemsetAsync(ws + p.zero_begin, 0, p.zero_end - p.zero_begin, st));

  www_model* m = new www_model();
  memset(m, 0, sizeof(*m));
  m->cfg = *cfg;
  m->L = s.L; m->d = s.d; m->Hq = s.Hq; m->Hkv = s.Hkv; m->hd = s.hd; m->G = s.G; m->F = s.F; m->Fp = s.Fp; m->V = s.V;
  m->QKVN = s.QKVN; m->QD = s.QD; m->KD = s.KD; m->max_pos = s.max_pos; m->maxB = s.maxB; m->MTmax = s.MTmax; m->maxT = s.maxT;
  m->wsplit = s.wsplit;
  m->fp8 = s.fp8;
  m->int4_group = s.int4_group;
  m->layers = new LayerW[s.L];
  memset(m->layers, 0, sizeof(LayerW) * s.L);
  m->graphs = new GraphEntry[MAX_GRAPHS];
  m->n_graphs = 0;
  const char* env = getenv("WWW_NO_GRAPH");
  m->use_graph = !(env && env[0] == '1');

  auto fail = [&](int code) { delete[] m->layers; delete[] m->graphs; delete m; return code; };
#define LOAD_TRY(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { set_error("%s failed: %s", #x, hipGetErrorString(e_)); return fail(WWW_E_HIP); } } while (0)

  uint64_t src = 0;
  std::vector<float*> scale_dst;   // host destinations of the FP8 matrices' scales, in blob order, and
  std::vector<uint64_t> scale_src; // their byte offsets in the blob
  // hi (and lo): the fp16 planes of the matrix in the workspace; codes8: its FP8 codes in decode order (FP8 sources).
  // hi == 0 with an FP8 source: no fp16 copy is made.
  auto pack = [&](int N, int K, int mode, uint64_t hi, uint64_t lo, uint64_t codes8, float* scale_out, uint64_t gscales) {
    int KB = (K + 31) / 32;
    int r = 0;
    if (s.int4_group) {
      *scale_out = 1.f;
      r = launch_pack_int4(blob + src, blob + src + align256((uint64_t)N * K / 2), N, K, KB, s.int4_group, mode, s.hd, (s.Hq + s.Hkv) * s.hd,
                           s.F, hi ? (uint16_t*)(ws + hi) : nullptr, (uint8_t*)(ws + codes8), ws + gscales, st);
      src += blob_matrix_bytes(s, N, K);
      return r;
    }
    if (!s.fp8 || hi)
      r = launch_pack_matrix(blob + src, dt, N, K, KB, mode, s.hd, (s.Hq + s.Hkv) * s.hd, s.F, (uint16_t*)(ws + hi), s.wsplit ? (uint16_t*)(ws + lo) : nullptr, st);
    if (s.fp8) {
      if (!r) r = launch_pack_fp8(blob + src, N, K, KB, mode, s.hd, (s.Hq + s.Hkv) * s.hd, s.F, (uint8_t*)(ws + codes8), st);
      scale_dst.push_back(scale_out);
      scale_src.push_back(src + align256((uint64_t)N * K));
    } else {
      *scale_out = 1.f;
    }
    src += blob_matrix_bytes(s, N, K);
    return r;
  };
  // embed
  LOAD_TRY(hipMemcpyAsync(ws + p.embed, blob + src, (uint64_t)s.V * s.d * wb, hipMemcpyDeviceToDevice, st));
  src += align256((uint64_t)s.V * s.d * wb);  // (an FP8 weight-only model's embedding is bf16: wb = 2)
  for (int l = 0; l < s.L; ++l) {
    LayerW& w = m->layers[l];
    LOAD_TRY(hipMemcpyAsync(ws + p.attn_norm[l], blob + src, (uint64_t)s.d * 4, hipMemcpyDeviceToDevice, st));
    src += align256((uint64_t)s.d * 4);
    if (pack(s.QKVN, s.d, 1, p.wqkv[l], p.wqkv_lo[l], p.wqkv8[l], &w.sqkv, p.gqkv[l])) { set_error("pack launch failed"); return fail(WWW_E_HIP); }
    if (s.qk_norm) {  // q_norm[hd], k_norm[hd]: stored in the row order of the packed heads
      const uint64_t slot = align256((uint64_t)s.hd * 4);
      if (launch_pack_qk_gain((const float*)(blob + src), (const float*)(blob + src + slot), s.hd, (float*)(ws + p.qk_gain[l]), st)) {
        set_error("pack launch failed");
        return fail(WWW_E_HIP);
      }
      src += 2 * slot;
      w.qk_gain = (const float*)(ws + p.qk_gain[l]);
    }
    if (pack(s.d, s.QD, 0, p.wo[l], p.wo_lo[l], p.wo8[l], &w.so, p.go[l])) { set_error("pack launch failed"); return fail(WWW_E_HIP); }
    LOAD_TRY(hipMemcpyAsync(ws + p.ffn_norm[l], blob + src, (uint64_t)s.d * 4, hipMemcpyDeviceToDevice, st));
    src += align256((uint64_t)s.d * 4);
    if (pack(2 * s.F, s.d, 2, p.wgu[l], p.wgu_lo[l], p.wgu8[l], &w.sgu, p.ggu[l])) { set_error("pack launch failed"); return fail(WWW_E_HIP); }
    if (pack(s.d, s.F, 0, p.wd[l], p.wd_lo[l], p.wd8[l], &w.sd, p.gd[l])) { set_error("pack launch failed"); return fail(WWW_E_HIP); }
    if (s.fp8 || s.int4_group) {
      w.wqkv8 = (const uint8_t*)(ws + p.wqkv8[l]); w.wo8 = (const uint8_t*)(ws + p.wo8[l]);
      w.wgu8 = (const uint8_t*)(ws + p.wgu8[l]); w.wd8 = (const uint8_t*)(ws + p.wd8[l]);
    }
    if (s.int4_group) { w.gqkv = ws + p.gqkv[l]; w.go = ws + p.go[l]; w.ggu = ws + p.ggu[l]; w.gd = ws + p.gd[l]; }
    w.wqkv = (const uint16_t*)(ws + p.wqkv[l]); w.wo = (const uint16_t*)(ws + p.wo[l]);
    w.wgu = (const uint16_t*)(ws + p.wgu[l]); w.wd = (const uint16_t*)(ws + p.wd[l]);
    w.wqkv_lo = s.wsplit ? (const uint16_t*)(ws + p.wqkv_lo[l]) : nullptr; w.wo_lo = s.wsplit ? (const uint16_t*)(ws + p.wo_lo[l]) : nullptr;
    w.wgu_lo = s.wsplit ? (const uint16_t*)(ws + p.wgu_lo[l]) : nullptr; w.wd_lo = s.wsplit ? (const uint16_t*)(ws + p.wd_lo[l]) : nullptr;
    w.attn_norm = (const float*)(ws + p.attn_norm[l]); w.ffn_norm = (const float*)(ws + p.ffn_norm[l]);
  }
  LOAD_TRY(hipMemcpyAsync(ws + p.final_norm, blob + src, (uint64_t)s.d * 4, hipMemcpyDeviceToDevice, st));
  src += align256((uint64_t)s.d * 4);
  if (pack(s.V, s.d, 0, p.lm_head, p.lm_head_lo, p.lm_head8, &m->s_lm, p.g_lm)) { set_error("pack launch failed"); return fail(WWW_E_HIP); }
  for (size_t i = 0; i < scale_dst.size(); ++i)  // the scales travel to the host: they are kernel arguments
    LOAD_TRY(hipMemcpyAsync(scale_dst[i], blob + scale_src[i], 4, hipMemcpyDeviceToHost, st));

  // rotary table: angle = pos * theta^(-2i/hd) evaluated in double, stored as (cos, sin) in fp32
  {
    std::vector<float> tab((size_t)s.max_pos * (s.hd / 2) * 2);
    for (int i = 0; i < s.hd / 2; ++i) {
      double freq = pow((double)cfg->rope_theta, -2.0 * i / s.hd);
      for (int pos = 0; pos < s.max_pos; ++pos) {
        double a = pos * freq;
        tab[((size_t)pos * (s.hd / 2) + i) * 2] = (float)cos(a);
        tab[((size_t)pos * (s.hd / 2) + i) * 2 + 1] = (float)sin(a);
      }
    }
    LOAD_TRY(hipMemcpyAsync(ws + p.rope, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, st));
    LOAD_TRY(hipStreamSynchronize(st));  // tab is about to go out of scope; also fences the packing kernels
  }
#undef LOAD_TRY

  m->embed = ws + p.embed;
  m->lm_head = (s.fp8 || s.int4_group) ? nullptr : (const uint16_t*)(ws + p.lm_head);
  m->lm_head8 = (s.fp8 || s.int4_group) ? (const uint8_t*)(ws + p.lm_head8) : nullptr;
  m->g_lm = s.int4_group ? ws + p.g_lm : nullptr;
  m->lm_head_lo = s.wsplit ? (const uint16_t*)(ws + p.lm_head_lo) : nullptr;
  m->final_norm = (const float*)(ws + p.final_norm);
  m->rope = (const float2*)(ws + p.rope);
  m->kv = (uint16_t*)kv_pool_dev;
  m->kv_plane = (int64_t)cfg->num_kv_blocks * s.Hkv * KV_BS * s.hd;
  m->kv_scales = (float*)(m->kv + (int64_t)2 * s.L * m->kv_plane);
  m->kv_scale_plane = (int64_t)cfg->num_kv_blocks * s.Hkv * 32;
  m->h = (float*)(ws + p.h); m->ssq = (float*)(ws + p.ssq); m->q_hi = (uint16_t*)(ws + p.q); m->q_lo = m->q_hi + (size_t)s.MTmax * 16 * s.QD;
  m->xq = (uint16_t*)(ws + p.xq); m->xo = (uint16_t*)(ws + p.xo); m->xa = (uint16_t*)(ws + p.xa);
  m->partial = (float*)(ws + p.partial); m->attn_part = (float*)(ws + p.attn_part); m->counters = (unsigned long long*)(ws + p.counters);
  m->logits_buf = (float*)(ws + p.logits); m->last_tok = (int*)(ws + p.last_tok);
  m->attn_hdr = (int*)(ws + p.attn_hdr); m->attn_start = (int*)(ws + p.attn_start); m->attn_pref = (int*)(ws + p.attn_pref);
  m->argmax_val = (float*)(ws + p.argmax_val); m->argmax_idx = (int*)(ws + p.argmax_idx);
  m->hp = (float*)(ws + p.hp); m->ssq_p = (float*)(ws + p.ssq_p); m->xn = (uint16_t*)(ws + p.xn); m->qp = (uint16_t*)(ws + p.qp); m->op = (uint16_t*)(ws + p.op); m->ap = (uint16_t*)(ws + p.ap);
  m->row_seq = (int*)(ws + p.row_seq); m->row_pos = (int*)(ws + p.row_pos); m->tile_seq = (int*)(ws + p.tile_seq);
  m->tile_q0 = (int*)(ws + p.tile_q0); m->meta = (int*)(ws + p.meta);
  m->attn_maxrec = p.attn_maxrec;
  m->attn_waves = decode_attn_resident_waves(s.hd, s.G);
  if (m->attn_waves > MAX_ATTN_WAVES) m->attn_waves = MAX_ATTN_WAVES;
  {
    // the split-K hand-over may skip its L2 write-back only if workgroup ids equal modulo 8 share an XCD: probe it
    // (4096 workgroups, results in the attention plan buffer, which is rewritten by every decode step)
    const char* force = getenv("WWW_HANDOVER_FENCE");
    const int ok = decode_probe_placement(m->attn_start, 4096, st);
    if (ok < 0) { set_error("placement probe failed: %s", hipGetErrorString(hipGetLastError())); return fail(WWW_E_HIP); }
    m->handover_fence = (ok == 0) || (force && atoi(force) != 0);
    // a pinned host word the kernels set if, against the probe, the splits of a row tile ever run on different XCDs
    if (hipHostMalloc((void**)&m->fault_host, 4 * sizeof(int), hipHostMallocMapped) != hipSuccess ||
        hipHostGetDevicePointer((void**)&m->fault_dev, m->fault_host, 0) != hipSuccess) {
      set_error("pinned flag allocation failed: %s", hipGetErrorString(hipGetLastError()));
      if (m->fault_host) (void)hipHostFree(m->fault_host);
      return fail(WWW_E_HIP);
    }
    *m->fault_host = 0;
  }
  {
    const char* v = getenv("WWW_VALIDATE");
    m->validate = v && atoi(v) != 0;
    m->val_words = (int*)(ws + p.val_words);
    m->val_bitmap = (unsigned*)(ws + p.val_bitmap);
    m->val_bitmap_bytes = p.val_bitmap_bytes;
  }
  *out = m;
  return WWW_OK;
}

WWW_EXPORT int www_prefill(www_model* m, const int32_t* tokens_dev, const int32_t* q_lens_dev, const int32_t* seq_lens_dev,
                           const int32_t* block_table_dev, int32_t batch, int32_t total_q_tokens, float* logits_dev,
                           int32_t* next_tokens_dev, void* hip_stream) {
  if (!m) { set_error("NULL model"); return WWW_E_INVALID_ARG; }
  if (batch < 0 || total_q_tokens < 0 || total_q_tokens < batch) { set_error("bad batch / total_q_tokens"); return WWW_E_INVALID_ARG; }
  if (int rcp = check_placement_fault(m)) return rcp;
  if (batch == 0) return WWW_OK;  // nothing to do; the pointers of empty arrays may be NULL
  if (!tokens_dev || !q_lens_dev || !seq_lens_dev || !block_table_dev) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  if (batch > m->maxB) { set_error("batch %d exceeds max_batch %d", batch, m->maxB); return WWW_E_CAPACITY; }
  if (total_q_tokens > m->maxT) { set_error("total_q_tokens %d exceeds max_prefill_tokens %d", total_q_tokens, m->maxT); return WWW_E_CAPACITY; }
  hipStream_t st = (hipStream_t)hip_stream;
  if (m->validate)
    if (int rcv = validate_device_args(m, tokens_dev, total_q_tokens, q_lens_dev, seq_lens_dev, block_table_dev, batch, st)) return rcv;
  int rc = run_prefill(m, tokens_dev, q_lens_dev, seq_lens_dev, block_table_dev, batch, total_q_tokens, st);
  if (rc) return rc;
  // the last new position of every sequence goes through the decode path (hi/lo activations), which also yields the logits
  return run_decode(m, m->last_tok, seq_lens_dev, block_table_dev, batch, logits_dev, next_tokens_dev, st);
}

WWW_EXPORT int www_decode_step(www_model* m, const int32_t* last_tokens_dev, const int32_t* seq_lens_dev, const int32_t* block_table_dev,
                               int32_t batch, float* logits_dev, int32_t* next_tokens_dev, void* hip_stream) {
  if (!m) { set_error("NULL model"); return WWW_E_INVALID_ARG; }
  if (batch < 0) { set_error("negative batch"); return WWW_E_INVALID_ARG; }
  if (int rcp = check_placement_fault(m)) return rcp;
  if (batch == 0) return WWW_OK;  // nothing to do; the pointers of empty arrays may be NULL
  if (!last_tokens_dev || !seq_lens_dev || !block_table_dev) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  if (batch > m->maxB) { set_error("batch %d exceeds max_batch %d", batch, m->maxB); return WWW_E_CAPACITY; }
  hipStream_t st = (hipStream_t)hip_stream;
  if (m->validate)
    if (int rcv = validate_device_args(m, last_tokens_dev, batch, nullptr, seq_lens_dev, block_table_dev, batch, st)) return rcv;
  if (!m->use_graph || st == nullptr || (m->prof && m->prof->on))  // the legacy default stream cannot be captured
    return run_decode(m, last_tokens_dev, seq_lens_dev, block_table_dev, batch, logits_dev, next_tokens_dev, st);

  for (int i = 0; i < m->n_graphs; ++i) {
    GraphEntry& g = m->graphs[i];
    if (g.batch == batch && g.tok == last_tokens_dev && g.lens == seq_lens_dev && g.table == block_table_dev && g.logits == logits_dev &&
        g.next == next_tokens_dev && g.stream == st) {
      HIP_TRY(hipGraphLaunch(g.exec, st));
      return WWW_OK;
    }
  }
  // capture one step; pointers and grid sizes are frozen, lengths / tables / tokens are read from device memory at replay
  hipGraph_t graph = nullptr;
  HIP_TRY(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
  int rc = run_decode(m, last_tokens_dev, seq_lens_dev, block_table_dev, batch, logits_dev, next_tokens_dev, st);
  hipError_t ec = hipStreamEndCapture(st, &graph);
  if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
  if (ec != hipSuccess) { set_error("hipStreamEndCapture failed: %s", hipGetErrorString(ec)); return WWW_E_HIP; }
  hipGraphExec_t exec = nullptr;
  hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (ei != hipSuccess) { set_error("hipGraphInstantiate failed: %s", hipGetErrorString(ei)); return WWW_E_HIP; }
  if (m->n_graphs == MAX_GRAPHS) {  // evict the oldest
    (void)hipGraphExecDestroy(m->graphs[0].exec);
    memmove(&m->graphs[0], &m->graphs[1], (MAX_GRAPHS - 1) * sizeof(GraphEntry));
    m->n_graphs = MAX_GRAPHS - 1;
  }
  GraphEntry& g = m->graphs[m->n_graphs++];
  g.batch = batch; g.tok = last_tokens_dev; g.lens = seq_lens_dev; g.table = block_table_dev; g.logits = logits_dev; g.next = next_tokens_dev;
  g.stream = st; g.exec = exec;
  HIP_TRY(hipGraphLaunch(exec, st));
  return WWW_OK;
}

WWW_EXPORT void www_model_free(www_model* m) {
  if (!m) return;
  for (int i = 0; i < m->n_graphs; ++i) (void)hipGraphExecDestroy(m->graphs[i].exec);
  if (m->fault_host) (void)hipHostFree(m->fault_host);
  if (m->prof) {
    for (hipEvent_t e : m->prof->ev) (void)hipEventDestroy(e);
    delete m->prof;
  }
  delete[] m->graphs;
  delete[] m->layers;
  delete m;
}

WWW_EXPORT const char* www_last_error(void) { return g_err; }

WWW_EXPORT int www_check(www_model* m, void* hip_stream) {
  if (!m) { set_error("NULL model"); return WWW_E_INVALID_ARG; }
  HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
  return check_placement_fault(m);
}

WWW_EXPORT int www_debug_slots(const int32_t* table_row_dev, const int32_t* positions_dev, int32_t n, int64_t* slots_dev, void* hip_stream) {
  if (!table_row_dev || !positions_dev || !slots_dev || n < 0) { set_error("bad argument"); return WWW_E_INVALID_ARG; }
  if (launch_debug_slots(table_row_dev, positions_dev, n, slots_dev, (hipStream_t)hip_stream)) { set_error("launch failed"); return WWW_E_HIP; }
  return WWW_OK;
}

WWW_EXPORT int www_debug_read(www_model* m, int32_t which, float* dst_host, uint64_t n_floats, void* hip_stream) {
  if (!m || !dst_host) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  const float* src = nullptr;
  uint64_t cap = 0;
  if (which == 0) { src = m->h; cap = (uint64_t)m->MTmax * 16 * m->d; }
  else if (which == 1) { src = (const float*)m->q_hi; cap = (uint64_t)m->MTmax * 16 * m->QD; }  // raw fp16 hi then lo planes
  else if (which == 2) { src = (const float*)m->xo; cap = (uint64_t)m->MTmax * 16 * m->QD; }    // raw packed attention output
  else { set_error("unknown buffer %d", which); return WWW_E_INVALID_ARG; }
  if (n_floats > cap) { set_error("buffer holds %llu floats", (unsigned long long)cap); return WWW_E_INVALID_ARG; }
  HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
  HIP_TRY(hipMemcpy(dst_host, src, n_floats * 4, hipMemcpyDeviceToHost));
  return check_placement_fault(m);  // the work is complete: a violation found by its kernels is reported now, not by the next call
}

WWW_EXPORT int www_debug_profile(www_model* m, int32_t enable) {
  if (!m) { set_error("NULL model"); return WWW_E_INVALID_ARG; }
  if (!m->prof) m->prof = new DecodeProfiler();
  m->prof->on = enable != 0;
  m->prof->used = 0;
  return WWW_OK;
}

WWW_EXPORT int www_debug_profile_read(www_model* m, float* ms_host, int32_t* launches_host, void* hip_stream) {
  if (!m || !m->prof || !ms_host || !launches_host) { set_error("profiling was never enabled, or NULL argument"); return WWW_E_INVALID_ARG; }
  HIP_TRY(hipStreamSynchronize((hipStream_t)hip_stream));
  for (int i = 0; i < PK_COUNT; ++i) { ms_host[i] = 0.f; launches_host[i] = 0; }
  DecodeProfiler* p = m->prof;
  for (size_t i = 0; i + 1 < p->used; ++i) {
    int c = p->cls[i];
    if (c < 0 || c >= PK_COUNT) continue;  // -1 marks the end of a step
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, p->ev[i], p->ev[i + 1]));
    ms_host[c] += ms;
    launches_host[c] += 1;
  }
  p->used = 0;
  return WWW_OK;
}
