/* www_oracle.c -- plain CPU oracle for batched decoder inference with a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is checked against; it is
 * used by tests/, by the smoke check and by the CPU-baseline leg of the benchmark and by nothing
 * else.  It shares no code, header, table or helper with the GPU path.
 *
 * What it computes.  The paper (WWW.Serve) treats the engine behind each provider as a black box
 * that executes requests locally (Sec. 3.2, "Model Manager"; App. A.1 "Local execution") with
 * greedy decoding (App. C: temperature 0), and a judge that reads two responses in one pass
 * (Sec. 4.2).  It gives no equations for the model, so the definition implemented here is the
 * standard pre-norm decoder that the served model families share and that the repository's
 * synthetic configurations name: RMSNorm -> grouped-query attention with rotary position embedding
 * -> residual -> RMSNorm -> SwiGLU -> residual, final RMSNorm, untied output head, argmax.
 * For a token at position p (0-based) of a sequence:
 *
 *   x  = E[token]
 *   for each layer:  u = rmsnorm(x, g1);  q,k,v = u Wq^T, u Wk^T, u Wv^T  (per head)
 *                    [qk_norm models: q_h = rmsnorm(q_h, gq); k_j = rmsnorm(k_j, gk), over the head's hd values,
 *                     gains gq, gk [hd] shared by the heads of the layer -- the per-head query / key
 *                     normalisation of the Qwen3 family the paper serves (Sec. 6.3, App. C)]
 *                    q_h = rope(q_h, p); k_j = rope(k_j, p); cache (k, v) at position p
 *                    o_h = sum_i softmax_i( q_h . k_{j,i} / sqrt(hd) ) v_{j,i},  i = 0..p, j = h / G
 *                    x  += concat(o) Wo^T
 *                    u = rmsnorm(x, g2);  x += ( silu(u Wg^T) * (u Wu^T) ) Wd^T
 *   logits = rmsnorm(x, gf) Wlm^T    (last position of each sequence only);  next = argmax(logits)
 *
 *   rmsnorm(x,g)_i = x_i g_i / sqrt(mean_j x_j^2 + eps)         silu(z) = z / (1 + exp(-z))
 *   rope(x,p): theta_i = theta^(-2i/hd), i < hd/2; the pair (x_i, x_{i+hd/2}) is rotated by p*theta_i
 *
 * Arithmetic.  Values are stored in fp32 between operations.  Inside one operation (a dot product,
 * a sum of squares, a softmax, a rotation) everything is carried in fp64 and rounded to fp32 once.
 * Weights given in bf16 are widened exactly.  Every output element is produced by the same routine
 * whatever the batch, chunking or cache layout, which is what makes the layout/chunking invariants
 * bit-exact.
 *
 * KV cache.  Kept twice: per-sequence contiguous arrays and a paged pool addressed through a block
 * table (slot(b,pos) = table[b][pos / bs] * bs + pos % bs).  kv_mode selects which copy attention
 * reads; both are always written.
 *
 * Pins (tests/test_oracle_*.py): softmax/RoPE/RMSNorm closed forms and invariants, single-key
 * attention, library-routine cross-checks (PyTorch CPU ops), fp64 dense brute force on tiny
 * inputs, paged == contiguous, chunked == unchunked == token-by-token, GQA == MHA with repeated
 * heads, causality, batch independence.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
  float rms_eps, rope_theta;
  int32_t kv_block_size;
  int32_t weight_dtype; /* 0 = fp32, 1 = bf16 */
  int32_t qk_norm;      /* 1: query and key heads are RMS-normalised before the rotation */
} orc_config;

typedef struct {
  size_t attn_norm, wqkv, q_norm, k_norm, wo, ffn_norm, wgu, wd;
} orc_layer_off;

typedef struct orc_model {
  orc_config c;
  const uint8_t* blob; /* borrowed from the caller */
  size_t off_embed, off_final_norm, off_lm_head;
  orc_layer_off* lo;
  int32_t max_seqs, max_ctx;
  int64_t num_blocks;
  float* kv_contig; /* [max_seqs][L][2][max_ctx][Hkv*hd] or NULL */
  float* kv_paged;  /* [num_blocks][L][2][bs][Hkv*hd] or NULL */
  int32_t kv_mode;  /* 0: attention reads the contiguous copy, 1: the paged copy */
} orc_model;

/* ------------------------------------------------------------------ elementary operations */

static inline float bf16_to_f32(uint16_t b) {
  union { uint32_t u; float f; } v;
  v.u = (uint32_t)b << 16;
  return v.f;
}

static inline double weight_at(const void* w, int wdtype, size_t i) {
  return wdtype == 0 ? (double)((const float*)w)[i] : (double)bf16_to_f32(((const uint16_t*)w)[i]);
}

/* y[t][n] = sum_k x[t][k] * w[n][k]; w is [N][K] row-major in fp32 or bf16 */
void orc_matmul(float* y, const float* x, const void* w, int wdtype, int64_t T, int64_t N, int64_t K) {
#pragma omp parallel
  {
    double* wrow = (double*)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
      for (int64_t k = 0; k < K; ++k) wrow[k] = weight_at(w, wdtype, (size_t)n * (size_t)K + (size_t)k);
      for (int64_t t = 0; t < T; ++t) {
        const float* xr = x + t * K;
        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
        for (int64_t k = 0; k < K; ++k) acc += (double)xr[k] * wrow[k];
        y[t * N + n] = (float)acc;
      }
    }
    free(wrow);
  }
}

/* out_i = x_i * g_i / sqrt(mean(x^2) + eps) */
void orc_rmsnorm(float* out, const float* x, const float* g, int64_t d, double eps) {
  double ss = 0.0;
  for (int64_t i = 0; i < d; ++i) ss += (double)x[i] * (double)x[i];
  double r = 1.0 / sqrt(ss / (double)d + eps);
  for (int64_t i = 0; i < d; ++i) out[i] = (float)((double)x[i] * r * (double)g[i]);
}

/* rotary embedding of one head vector at position pos; pairs are (i, i + hd/2) */
void orc_rope(float* out, const float* x, int hd, int64_t pos, double theta) {
  int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    double freq = pow(theta, -2.0 * (double)i / (double)hd);
    double ang = (double)pos * freq;
    double c = cos(ang), s = sin(ang);
    double a = (double)x[i], b = (double)x[i + half];
    out[i] = (float)(a * c - b * s);
    out[i + half] = (float)(b * c + a * s);
  }
}

/* p = softmax(s) in fp64 (max-subtracted) */
static void softmax_f64(double* p, const double* s, int64_t n) {
  double m = s[0];
  for (int64_t i = 1; i < n; ++i)
    if (s[i] > m) m = s[i];
  double z = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    p[i] = exp(s[i] - m);
    z += p[i];
  }
  for (int64_t i = 0; i < n; ++i) p[i] /= z;
}

void orc_softmax(float* p, const float* s, int64_t n) {
  if (n <= 0) return; /* nothing to normalise */
  double* a = (double*)malloc(sizeof(double) * (size_t)n * 2);
  for (int64_t i = 0; i < n; ++i) a[i] = (double)s[i];
  softmax_f64(a + n, a, n);
  for (int64_t i = 0; i < n; ++i) p[i] = (float)a[n + i];
  free(a);
}

/* One query vector against n keys/values. Key i is at kbase[i], value i at vbase[i] (hd floats each).
 * o = sum_i softmax_i(q.k_i / sqrt(hd)) v_i.  scratch holds 2n doubles. */
static void attend(float* o, const float* q, const float* const* kbase, const float* const* vbase, int64_t n, int hd,
                   double* scratch) {
  double* s = scratch;
  double* p = scratch + n;
  double scale = 1.0 / sqrt((double)hd);
  for (int64_t i = 0; i < n; ++i) {
    const float* k = kbase[i];
    double acc = 0.0;
    for (int e = 0; e < hd; ++e) acc += (double)q[e] * (double)k[e];
    s[i] = acc * scale;
  }
  softmax_f64(p, s, n);
  for (int e = 0; e < hd; ++e) {
    double acc = 0.0;
    for (int64_t i = 0; i < n; ++i) acc += p[i] * (double)vbase[i][e];
    o[e] = (float)acc;
  }
}

/* Contiguous-array form of the above for unit tests: K, V are [n][hd]. */
void orc_attend(float* o, const float* q, const float* K, const float* V, int64_t n, int hd) {
  const float** kb = (const float**)malloc(sizeof(float*) * (size_t)n * 2);
  const float** vb = kb + n;
  for (int64_t i = 0; i < n; ++i) {
    kb[i] = K + i * hd;
    vb[i] = V + i * hd;
  }
  double* scratch = (double*)malloc(sizeof(double) * (size_t)n * 2);
  attend(o, q, kb, vb, n, hd, scratch);
  free(scratch);
  free((void*)kb);
}

/* a_i = silu(g_i) * u_i */
void orc_silu_mul(float* a, const float* g, const float* u, int64_t n) {
  for (int64_t i = 0; i < n; ++i) {
    double z = (double)g[i];
    a[i] = (float)(z / (1.0 + exp(-z)) * (double)u[i]);
  }
}

/* index of the largest element; the lowest index wins a tie */
int32_t orc_argmax(const float* x, int64_t n) {
  int64_t best = 0;
  for (int64_t i = 1; i < n; ++i)
    if (x[i] > x[best]) best = i;
  return (int32_t)best;
}

/* physical token slot of logical position pos of a sequence whose block-table row is given */
int64_t orc_slot(const int32_t* table_row, int64_t pos, int bs) {
  return (int64_t)table_row[pos / bs] * (int64_t)bs + pos % bs;
}

/* ------------------------------------------------------------------ model */

static size_t align_up(size_t n) { return (n + 255) / 256 * 256; }

orc_model* orc_create(const orc_config* c, const void* blob, int32_t max_seqs, int32_t max_ctx, int64_t num_blocks) {
  if (!c || !blob || c->head_dim % 2 || c->n_q_heads % c->n_kv_heads || c->kv_block_size <= 0) return NULL;
  orc_model* m = (orc_model*)calloc(1, sizeof(orc_model));
  m->c = *c;
  m->blob = (const uint8_t*)blob;
  m->lo = (orc_layer_off*)calloc((size_t)c->n_layers, sizeof(orc_layer_off));
  size_t wb = c->weight_dtype == 0 ? 4 : 2;
  size_t d = (size_t)c->d_model, F = (size_t)c->ffn_dim, V = (size_t)c->vocab;
  size_t qkv = (size_t)(c->n_q_heads + 2 * c->n_kv_heads) * (size_t)c->head_dim;
  size_t qd = (size_t)c->n_q_heads * (size_t)c->head_dim;
  size_t off = 0;
  m->off_embed = off; off += align_up(V * d * wb);
  for (int l = 0; l < c->n_layers; ++l) {
    m->lo[l].attn_norm = off; off += align_up(d * 4);
    m->lo[l].wqkv = off;      off += align_up(qkv * d * wb);
    if (c->qk_norm) {
      m->lo[l].q_norm = off;  off += align_up((size_t)c->head_dim * 4);
      m->lo[l].k_norm = off;  off += align_up((size_t)c->head_dim * 4);
    }
    m->lo[l].wo = off;        off += align_up(d * qd * wb);
    m->lo[l].ffn_norm = off;  off += align_up(d * 4);
    m->lo[l].wgu = off;       off += align_up(2 * F * d * wb);
    m->lo[l].wd = off;        off += align_up(d * F * wb);
  }
  m->off_final_norm = off; off += align_up(d * 4);
  m->off_lm_head = off;
  m->max_seqs = max_seqs;
  m->max_ctx = max_ctx;
  m->num_blocks = num_blocks;
  size_t row = (size_t)c->n_kv_heads * (size_t)c->head_dim;
  if (max_seqs > 0 && max_ctx > 0)
    m->kv_contig = (float*)calloc((size_t)max_seqs * (size_t)c->n_layers * 2 * (size_t)max_ctx * row, sizeof(float));
  if (num_blocks > 0)
    m->kv_paged = (float*)calloc((size_t)num_blocks * (size_t)c->n_layers * 2 * (size_t)c->kv_block_size * row, sizeof(float));
  m->kv_mode = m->kv_paged ? 1 : 0;
  return m;
}

void orc_free(orc_model* m) {
  if (!m) return;
  free(m->kv_contig);
  free(m->kv_paged);
  free(m->lo);
  free(m);
}

void orc_set_kv_mode(orc_model* m, int32_t mode) { m->kv_mode = mode; }
float* orc_kv_paged_ptr(orc_model* m) { return m->kv_paged; }
float* orc_kv_contig_ptr(orc_model* m) { return m->kv_contig; }
size_t orc_blob_bytes(const orc_model* m) {
  size_t wb = m->c.weight_dtype == 0 ? 4 : 2;
  return m->off_lm_head + align_up((size_t)m->c.vocab * (size_t)m->c.d_model * wb);
}

static inline float* contig_at(const orc_model* m, int64_t seq, int l, int kv, int64_t pos) {
  size_t row = (size_t)m->c.n_kv_heads * (size_t)m->c.head_dim;
  return m->kv_contig + ((((size_t)seq * (size_t)m->c.n_layers + (size_t)l) * 2 + (size_t)kv) * (size_t)m->max_ctx + (size_t)pos) * row;
}

static inline float* paged_at(const orc_model* m, const int32_t* table_row, int l, int kv, int64_t pos) {
  size_t row = (size_t)m->c.n_kv_heads * (size_t)m->c.head_dim;
  int bs = m->c.kv_block_size;
  int64_t slot = orc_slot(table_row, pos, bs);
  size_t blk = (size_t)(slot / bs), in = (size_t)(slot % bs);
  return m->kv_paged + ((((blk * (size_t)m->c.n_layers + (size_t)l) * 2 + (size_t)kv) * (size_t)bs) + in) * row;
}

/* One call = prefill, chunked prefill or decode, depending only on q_lens:
 *   tokens      packed new tokens, sum(q_lens) of them, sequence after sequence
 *   q_lens[b]   number of new tokens of sequence b (1 for a decode step)
 *   seq_lens[b] length of sequence b AFTER this call; positions seq_lens-q_lens .. seq_lens-1 are new
 *   seq_ids[b]  which contiguous cache this sequence owns (may be NULL if there is no contiguous copy)
 *   block_table [batch][max_blocks_per_seq] physical block ids (may be NULL if there is no paged copy)
 *   logits      [batch][vocab] at the last new position of each sequence (may be NULL)
 *   next_tokens [batch] argmax of logits (may be NULL)
 *   trace       optional [L+1][T][d]: residual stream after the embedding and after each layer
 * Returns 0, or a negative code on a bad argument. */
int orc_forward(orc_model* m, const int32_t* tokens, const int32_t* q_lens, const int32_t* seq_lens, const int32_t* seq_ids,
                const int32_t* block_table, int32_t max_blocks_per_seq, int32_t batch, float* logits, int32_t* next_tokens,
                float* trace) {
  const orc_config* c = &m->c;
  const int L = c->n_layers, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim, bs = c->kv_block_size;
  const int G = Hq / Hkv;
  const int64_t d = c->d_model, F = c->ffn_dim, V = c->vocab;
  const int64_t QD = (int64_t)Hq * hd, KD = (int64_t)Hkv * hd, QKV = QD + 2 * KD;
  const int wdt = c->weight_dtype;
  const size_t wb = wdt == 0 ? 4 : 2;

  int64_t T = 0, max_len = 0;
  for (int b = 0; b < batch; ++b) {
    if (q_lens[b] < 0 || seq_lens[b] < q_lens[b]) return -1;
    if (m->kv_contig && (!seq_ids || seq_ids[b] < 0 || seq_ids[b] >= m->max_seqs || seq_lens[b] > m->max_ctx)) return -2;
    if (m->kv_paged && (!block_table || (seq_lens[b] + bs - 1) / bs > max_blocks_per_seq)) return -3;
    T += q_lens[b];
    if (seq_lens[b] > max_len) max_len = seq_lens[b];
  }
  if (m->kv_paged)
    for (int b = 0; b < batch; ++b)
      for (int64_t j = 0; j < (seq_lens[b] + bs - 1) / bs; ++j) {
        int32_t id = block_table[(size_t)b * max_blocks_per_seq + j];
        if (id < 0 || id >= m->num_blocks) return -4;
      }
  if (T == 0) return 0;

  int32_t* row_seq = (int32_t*)malloc(sizeof(int32_t) * (size_t)T);
  int64_t* row_pos = (int64_t*)malloc(sizeof(int64_t) * (size_t)T);
  int64_t* last_row = (int64_t*)malloc(sizeof(int64_t) * (size_t)batch);
  {
    int64_t r = 0;
    for (int b = 0; b < batch; ++b) {
      for (int i = 0; i < q_lens[b]; ++i, ++r) {
        row_seq[r] = b;
        row_pos[r] = (int64_t)seq_lens[b] - q_lens[b] + i;
      }
      last_row[b] = q_lens[b] > 0 ? r - 1 : -1;
    }
  }
  for (int64_t r = 0; r < T; ++r)
    if (tokens[r] < 0 || tokens[r] >= V) { free(row_seq); free(row_pos); free(last_row); return -5; }

  float* x = (float*)malloc(sizeof(float) * (size_t)(T * d));
  float* u = (float*)malloc(sizeof(float) * (size_t)(T * d));
  float* qkv = (float*)malloc(sizeof(float) * (size_t)(T * QKV));
  float* att = (float*)malloc(sizeof(float) * (size_t)(T * QD));
  float* y = (float*)malloc(sizeof(float) * (size_t)(T * d));
  float* gu = (float*)malloc(sizeof(float) * (size_t)(T * 2 * F));
  float* act = (float*)malloc(sizeof(float) * (size_t)(T * F));

  /* embedding */
  for (int64_t r = 0; r < T; ++r)
    for (int64_t i = 0; i < d; ++i)
      x[r * d + i] = (float)weight_at(m->blob + m->off_embed, wdt, (size_t)tokens[r] * (size_t)d + (size_t)i);
  if (trace) memcpy(trace, x, sizeof(float) * (size_t)(T * d));

  for (int l = 0; l < L; ++l) {
    const orc_layer_off* o = &m->lo[l];
    const float* g1 = (const float*)(m->blob + o->attn_norm);
    const float* g2 = (const float*)(m->blob + o->ffn_norm);

    /* attention block */
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < T; ++r) orc_rmsnorm(u + r * d, x + r * d, g1, d, (double)c->rms_eps);
    orc_matmul(qkv, u, m->blob + o->wqkv, wdt, T, QKV, d);

    /* rotary embedding on every q and k head, then append k, v to the cache(s) at the row's position */
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < T; ++r) {
      float* row = qkv + r * QKV;
      if (c->qk_norm)
        for (int h = 0; h < Hq + Hkv; ++h)
          orc_rmsnorm(row + (int64_t)h * hd, row + (int64_t)h * hd, (const float*)(m->blob + (h < Hq ? o->q_norm : o->k_norm)), hd,
                      (double)c->rms_eps);
      for (int h = 0; h < Hq + Hkv; ++h) orc_rope(row + (int64_t)h * hd, row + (int64_t)h * hd, hd, row_pos[r], (double)c->rope_theta);
      int b = row_seq[r];
      if (m->kv_contig) {
        memcpy(contig_at(m, seq_ids[b], l, 0, row_pos[r]), row + QD, sizeof(float) * (size_t)KD);
        memcpy(contig_at(m, seq_ids[b], l, 1, row_pos[r]), row + QD + KD, sizeof(float) * (size_t)KD);
      }
      if (m->kv_paged) {
        const int32_t* tr = block_table + (size_t)b * max_blocks_per_seq;
        memcpy(paged_at(m, tr, l, 0, row_pos[r]), row + QD, sizeof(float) * (size_t)KD);
        memcpy(paged_at(m, tr, l, 1, row_pos[r]), row + QD + KD, sizeof(float) * (size_t)KD);
      }
    }

    /* causal attention: the query at position p sees keys 0..p of its own sequence, read from the cache */
#pragma omp parallel
    {
      const float** kb = (const float**)malloc(sizeof(float*) * (size_t)max_len * 2);
      const float** vb = kb + max_len;
      double* scratch = (double*)malloc(sizeof(double) * (size_t)max_len * 2);
#pragma omp for schedule(dynamic, 1) collapse(2)
      for (int64_t r = 0; r < T; ++r)
        for (int h = 0; h < Hq; ++h) {
          int b = row_seq[r];
          int j = h / G; /* query head h uses KV head h / G */
          int64_t n = row_pos[r] + 1;
          const int32_t* tr = block_table ? block_table + (size_t)b * max_blocks_per_seq : NULL;
          for (int64_t i = 0; i < n; ++i) {
            if (m->kv_mode == 1) {
              kb[i] = paged_at(m, tr, l, 0, i) + (int64_t)j * hd;
              vb[i] = paged_at(m, tr, l, 1, i) + (int64_t)j * hd;
            } else {
              kb[i] = contig_at(m, seq_ids[b], l, 0, i) + (int64_t)j * hd;
              vb[i] = contig_at(m, seq_ids[b], l, 1, i) + (int64_t)j * hd;
            }
          }
          attend(att + r * QD + (int64_t)h * hd, qkv + r * QKV + (int64_t)h * hd, kb, vb, n, hd, scratch);
        }
      free(scratch);
      free((void*)kb);
    }
    orc_matmul(y, att, m->blob + o->wo, wdt, T, d, QD);
    for (int64_t i = 0; i < T * d; ++i) x[i] = x[i] + y[i];

    /* feed-forward block: gate rows 0..F-1 and up rows F..2F-1 of wgu */
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < T; ++r) orc_rmsnorm(u + r * d, x + r * d, g2, d, (double)c->rms_eps);
    orc_matmul(gu, u, m->blob + o->wgu, wdt, T, 2 * F, d);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < T; ++r) orc_silu_mul(act + r * F, gu + r * 2 * F, gu + r * 2 * F + F, F);
    orc_matmul(y, act, m->blob + o->wd, wdt, T, d, F);
    for (int64_t i = 0; i < T * d; ++i) x[i] = x[i] + y[i];
    if (trace) memcpy(trace + (size_t)(l + 1) * (size_t)(T * d), x, sizeof(float) * (size_t)(T * d));
  }

  /* output head on the last new position of each sequence */
  if (logits || next_tokens) {
    float* xl = (float*)calloc((size_t)batch * (size_t)d, sizeof(float));
    float* lg = logits ? logits : (float*)malloc(sizeof(float) * (size_t)batch * (size_t)V);
    const float* gf = (const float*)(m->blob + m->off_final_norm);
    for (int b = 0; b < batch; ++b)
      if (last_row[b] >= 0) orc_rmsnorm(xl + (int64_t)b * d, x + last_row[b] * d, gf, d, (double)c->rms_eps);
    orc_matmul(lg, xl, m->blob + m->off_lm_head, wdt, batch, V, d);
    if (next_tokens)
      for (int b = 0; b < batch; ++b) next_tokens[b] = orc_argmax(lg + (int64_t)b * V, V);
    if (!logits) free(lg);
    free(xl);
  }
  (void)wb;
  free(x); free(u); free(qkv); free(att); free(y); free(gu); free(act);
  free(row_seq); free(row_pos); free(last_row);
  return 0;
}
