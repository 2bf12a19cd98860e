// Exercises the CPU oracle, the input generator and the host-side C++ of the library (scheduler, credit ledger) in one
// executable that tests/test_sanitizers.py builds with -fsanitize=address,undefined and runs: any out-of-bounds access,
// use after free, leak, signed overflow or misaligned access in those sources ends the run with a non-zero status.
// The checks of the results themselves live in the other tests; this driver only has to walk the code paths.
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/www.h"

extern "C" {
// oracle/www_oracle.c
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
  float rms_eps, rope_theta;
  int32_t kv_block_size, weight_dtype, qk_norm;
} orc_config;
struct orc_model;
orc_model* orc_create(const orc_config* c, const void* blob, int32_t max_seqs, int32_t max_ctx, int64_t num_blocks);
void orc_free(orc_model* m);
size_t orc_blob_bytes(const orc_model* m);
void orc_set_kv_mode(orc_model* m, int32_t mode);
int orc_forward(orc_model* m, const int32_t* tokens, const int32_t* q_lens, const int32_t* seq_lens, const int32_t* seq_ids,
                const int32_t* block_table, int32_t max_blocks_per_seq, int32_t batch, float* logits, int32_t* next_tokens, float* trace);
void orc_softmax(float* p, const float* s, int64_t n);
void orc_attend(float* o, const float* q, const float* K, const float* V, int64_t n, int hd);
// synth/wwwsynth.c
void wwwsynth_normal_f32(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, double mean, double std, float* out);
void wwwsynth_normal_bf16(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, double mean, double std, uint16_t* out);
void wwwsynth_uniform_i32(uint64_t seed, uint64_t stream_id, uint64_t first, uint64_t n, uint32_t bound, int32_t* out);
void wwwsynth_encode_e4m3(const float* src, uint64_t n, double inv_scale, uint8_t* out);
void wwwsynth_encode_int4(const float* src, uint64_t rows, uint64_t cols, uint64_t group, uint8_t* codes, uint16_t* scales);
}

// the library's error sink (api.hip in the real build)
void set_error(const char* fmt, ...) {
  char buf[256];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
}

#define REQUIRE(x) do { if (!(x)) { fprintf(stderr, "driver: %s failed (line %d)\n", #x, __LINE__); return 1; } } while (0)

static int run_oracle(int wdtype, int qk_norm) {
  orc_config c = {2, 64, 4, 2, 16, 96, 128, 1e-5f, 1e4f, 16, wdtype, qk_norm};
  // a blob that is large enough for any layout of this shape: gains of 1, everything else small normal numbers
  orc_model* probe = orc_create(&c, "", 0, 0, 0);
  REQUIRE(probe);
  const size_t bytes = orc_blob_bytes(probe);
  orc_free(probe);
  std::vector<uint8_t> blob(bytes);
  if (wdtype == 0) wwwsynth_normal_f32(1, 2, 0, bytes / 4, 0.0, 0.05, (float*)blob.data());
  else wwwsynth_normal_bf16(1, 2, 0, bytes / 2, 0.0, 0.05, (uint16_t*)blob.data());
  const int nb = 12, mbs = 4;
  orc_model* m = orc_create(&c, blob.data(), 3, mbs * 16, nb);
  REQUIRE(m && orc_blob_bytes(m) == bytes);
  // note: the gains are read as fp32 wherever the layout puts them; random bit patterns there are still finite numbers
  int32_t table[3 * mbs] = {7, 2, 9, 0, 5, 11, 1, 3, 4, 6, 8, 10};
  int32_t seq_ids[3] = {0, 1, 2};
  std::vector<int32_t> tok(64);
  wwwsynth_uniform_i32(3, 4, 0, tok.size(), (uint32_t)c.vocab, tok.data());
  std::vector<float> logits(3 * (size_t)c.vocab), trace((size_t)(c.n_layers + 1) * 40 * c.d_model);
  int32_t next[3];
  int32_t q1[3] = {17, 1, 22}, s1[3] = {17, 1, 22};
  REQUIRE(orc_forward(m, tok.data(), q1, s1, seq_ids, table, mbs, 3, logits.data(), next, trace.data()) == 0);
  int32_t q2[3] = {15, 1, 1}, s2[3] = {32, 2, 23};  // a second chunk, two decode steps
  REQUIRE(orc_forward(m, tok.data() + 40, q2, s2, seq_ids, table, mbs, 3, logits.data(), next, nullptr) == 0);
  orc_set_kv_mode(m, 0);
  int32_t q3[3] = {1, 1, 1}, s3[3] = {33, 3, 24};
  REQUIRE(orc_forward(m, next, q3, s3, seq_ids, table, mbs, 3, nullptr, next, nullptr) == 0);
  int32_t s4[3] = {65, 3, 24};  // beyond the capacity: must be refused, not written
  REQUIRE(orc_forward(m, next, q3, s4, seq_ids, table, mbs, 3, nullptr, next, nullptr) != 0);
  int32_t bad_table[3 * mbs];
  memcpy(bad_table, table, sizeof(table));
  bad_table[0] = nb;
  REQUIRE(orc_forward(m, next, q3, s3, seq_ids, bad_table, mbs, 3, nullptr, next, nullptr) != 0);
  int32_t bad_tok[3] = {next[0], c.vocab, next[2]};
  REQUIRE(orc_forward(m, bad_tok, q3, s3, seq_ids, table, mbs, 3, nullptr, next, nullptr) != 0);
  orc_free(m);
  float s[5] = {0.f, 1.f, -2.f, 3.f, 0.5f}, p[5];
  orc_softmax(p, s, 5);
  orc_softmax(p, s, 0);
  float q[16], K[3 * 16], V[3 * 16], o[16];
  wwwsynth_normal_f32(5, 6, 0, 16, 0, 1, q);
  wwwsynth_normal_f32(5, 7, 0, 48, 0, 1, K);
  wwwsynth_normal_f32(5, 8, 0, 48, 0, 1, V);
  orc_attend(o, q, K, V, 3, 16);
  return 0;
}

static int run_generator() {
  std::vector<float> w(4 * 256);
  wwwsynth_normal_f32(9, 1, 0, w.size(), 0.0, 0.02, w.data());
  std::vector<uint8_t> codes(w.size()), c4(w.size() / 2);
  std::vector<uint16_t> scales(4 * 256 / 32);
  wwwsynth_encode_e4m3(w.data(), w.size(), 448.0 / 0.1, codes.data());
  wwwsynth_encode_int4(w.data(), 4, 256, 32, c4.data(), scales.data());
  wwwsynth_encode_int4(w.data(), 4, 256, 128, c4.data(), scales.data());
  return 0;
}

static int run_scheduler() {
  www_sched_config cfg = {4, 8, 64, 24, 16, 0, 40, 0.8};
  www_sched* s = nullptr;
  REQUIRE(www_sched_create(&cfg, &s) == WWW_OK && s);
  www_sched_config bad = cfg;
  bad.chunk_tokens = 65;
  www_sched* none = nullptr;
  REQUIRE(www_sched_create(&bad, &none) == WWW_E_BAD_CONFIG && !none);
  const int plen[9] = {50, 7, 100, 24, 1, 90, 33, 16, 64};
  for (int r = 0; r < 9; ++r) REQUIRE(www_sched_submit(s, 100 + r, plen[r], 1 + r % 4) == WWW_OK);
  REQUIRE(www_sched_submit(s, 1, 0, 1) == WWW_E_INVALID_ARG);
  REQUIRE(www_sched_submit(s, 2, 1000, 1) == WWW_E_CAPACITY);
  std::vector<int32_t> a(4), b(4), c(4), d(4), e(4), f(4), row(8);
  std::vector<uint64_t> ra(4), rb(4), fin(4);
  www_stats st;
  for (int it = 0; it < 500; ++it) {
    www_sched_step step;
    REQUIRE(www_sched_plan(s, &step, a.data(), b.data(), c.data(), d.data(), ra.data(), e.data(), f.data(), rb.data()) == WWW_OK);
    REQUIRE(www_sched_plan(s, &step, a.data(), b.data(), c.data(), d.data(), ra.data(), e.data(), f.data(), rb.data()) != WWW_OK);
    for (int i = 0; i < 4; ++i) REQUIRE(www_sched_table_row(s, i, row.data()) == WWW_OK);
    REQUIRE(www_sched_table_row(s, 4, row.data()) != WWW_OK);
    int32_t nfin = 0;
    REQUIRE(www_sched_commit(s, &nfin, fin.data()) == WWW_OK);
    REQUIRE(www_get_stats(s, &st) == WWW_OK);
    if (st.active == 0 && st.queued == 0) break;
  }
  REQUIRE(st.finished == 9);
  www_sched_free(s);
  www_sched_free(nullptr);
  return 0;
}

static int run_ledger() {
  const double stakes[5] = {10.0, 0.0, 5.0, 0.25, 30.0};
  www_credit_params par = {1.0, 0.5, 0.5, 0.1};
  www_ledger* l = nullptr;
  REQUIRE(www_ledger_create(5, stakes, &par, &l) == WWW_OK && l);
  const double u[3] = {0.0, 0.5, 0.999999};
  int32_t chosen[3], excl[1] = {4};
  REQUIRE(www_pos_sample(l, u, 3, excl, 1, chosen) == WWW_OK);
  REQUIRE(www_pos_sample(l, u, 3, nullptr, 0, chosen) == WWW_OK);
  const double u4[4] = {0.1, 0.2, 0.3, 0.4};
  int32_t c4[4];
  REQUIRE(www_pos_sample(l, u4, 4, excl, 1, c4) == WWW_E_CAPACITY);  // only three staked nodes are left in play
  REQUIRE(www_ledger_serve(l, 1, 0) == WWW_OK && www_ledger_serve(l, 1, 9) == WWW_E_INVALID_ARG);
  int32_t judges[2] = {2, 4}, votes[2] = {1, 1}, winner = -9;
  REQUIRE(www_ledger_duel(l, 1, 0, 3, judges, votes, 2, &winner) == WWW_OK && winner == 3);
  votes[1] = 0;
  REQUIRE(www_ledger_duel(l, 2, 0, 3, judges, votes, 2, &winner) == WWW_OK && winner == -1);
  REQUIRE(www_ledger_duel(l, 3, 0, 3, nullptr, nullptr, 0, nullptr) == WWW_OK);
  judges[0] = 0;
  REQUIRE(www_ledger_duel(l, 4, 0, 3, judges, votes, 2, &winner) == WWW_E_INVALID_ARG);  // an executor cannot judge its own duel
  double now[5];
  REQUIRE(www_ledger_stakes(l, now) == WWW_OK);
  const int64_t n = www_ledger_num_ops(l);
  std::vector<www_ledger_op> ops((size_t)n);
  REQUIRE(www_ledger_read_ops(l, 0, n, ops.data()) == WWW_OK);
  REQUIRE(www_ledger_read_ops(l, 1, n, ops.data()) != WWW_OK);
  www_ledger_free(l);
  www_ledger_free(nullptr);
  return 0;
}

int main() {
  if (run_oracle(0, 0) || run_oracle(1, 1) || run_generator() || run_scheduler() || run_ledger()) return 1;
  puts("sanitize driver: all paths walked");
  return 0;
}
