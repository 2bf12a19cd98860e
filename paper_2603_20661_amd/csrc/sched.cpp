// Continuous-batching scheduler of a provider's serving loop (host only): admission queue, KV-block allocator with a
// free list, chunked prefill under a per-iteration token budget, and the load figures a Model Manager polls (App. B
// of the paper: active and queued requests, memory utilisation; App. C: target utilisation).
#include <stddef.h>
#include <stdint.h>

#include <deque>
#include <new>
#include <vector>

#include "../../include/www.h"

#define WWW_EXPORT extern "C" __attribute__((visibility("default")))

void set_error(const char* fmt, ...);

namespace {

struct Sequence {
  uint64_t request = 0;
  int32_t prompt_len = 0, max_new = 0;
  int32_t prefilled = 0;   // prompt tokens in the cache
  int32_t generated = 0;   // tokens produced so far (the prefill that completes the prompt produces the first)
  bool active = false;
  std::vector<int32_t> blocks;
};

struct Pending {
  uint64_t request;
  int32_t prompt_len, max_new;
};

}  // namespace

struct www_sched {
  www_sched_config cfg;
  std::vector<Sequence> slot;        // max_batch rows of the block table
  std::vector<int32_t> free_blocks;  // stack; block ids are handed out in increasing order from a fresh pool
  std::deque<Pending> queue;
  uint64_t blocks_reserved = 0, block_limit = 0;
  int32_t rr = 0;  // slot after the last one that received a prefill chunk
  // the planned, not yet committed iteration
  bool planned = false;
  std::vector<int32_t> plan_prefill_slot, plan_prefill_q, plan_decode_slot;
  // counters
  uint64_t finished = 0, iterations = 0, prompt_tokens_done = 0, tokens_generated = 0;
};

static uint64_t blocks_for(const www_sched* s, int64_t tokens) { return (uint64_t)((tokens + s->cfg.kv_block_size - 1) / s->cfg.kv_block_size); }

WWW_EXPORT int www_sched_create(const www_sched_config* cfg, www_sched** out) {
  if (!out) { set_error("NULL out pointer"); return WWW_E_INVALID_ARG; }
  *out = nullptr;
  if (!cfg) { set_error("NULL scheduler configuration"); return WWW_E_INVALID_ARG; }
  if (cfg->max_batch == 0 || cfg->max_blocks_per_seq == 0 || cfg->token_budget == 0 || cfg->chunk_tokens == 0 ||
      cfg->kv_block_size != 16 || cfg->reserved != 0 || cfg->num_kv_blocks == 0 || cfg->num_kv_blocks > 0x7fffffffull ||
      !(cfg->target_utilisation > 0.0 && cfg->target_utilisation <= 1.0)) {
    set_error("scheduler configuration: counts must be positive, kv_block_size 16, 0 < target_utilisation <= 1");
    return WWW_E_BAD_CONFIG;
  }
  if (cfg->chunk_tokens > cfg->token_budget) {  // a full chunk would never fit an iteration: its sequence could not progress
    set_error("scheduler configuration: chunk_tokens %u exceeds token_budget %u", cfg->chunk_tokens, cfg->token_budget);
    return WWW_E_BAD_CONFIG;
  }
  www_sched* s = new (std::nothrow) www_sched;
  if (!s) { set_error("out of host memory"); return WWW_E_INVALID_ARG; }
  s->cfg = *cfg;
  s->slot.resize(cfg->max_batch);
  s->free_blocks.resize(cfg->num_kv_blocks);
  for (uint64_t i = 0; i < cfg->num_kv_blocks; ++i) s->free_blocks[i] = (int32_t)(cfg->num_kv_blocks - 1 - i);  // pop_back() yields 0, 1, 2, ...
  s->block_limit = (uint64_t)(cfg->target_utilisation * (double)cfg->num_kv_blocks);
  *out = s;
  return WWW_OK;
}

WWW_EXPORT void www_sched_free(www_sched* s) { delete s; }

WWW_EXPORT int www_sched_submit(www_sched* s, uint64_t request_id, int32_t prompt_len, int32_t max_new_tokens) {
  if (!s) { set_error("NULL scheduler"); return WWW_E_INVALID_ARG; }
  if (prompt_len < 1 || max_new_tokens < 1) { set_error("a request needs at least one prompt token and one new token"); return WWW_E_INVALID_ARG; }
  // the cache must hold the prompt and every generated token but the last (which is never fed back)
  const uint64_t need = blocks_for(s, (int64_t)prompt_len + max_new_tokens - 1);
  if (need > s->cfg.max_blocks_per_seq || need > s->block_limit) {
    set_error("request of %d + %d tokens needs %llu blocks: more than a sequence (%u) or the pool's target share (%llu) holds", prompt_len,
              max_new_tokens, (unsigned long long)need, s->cfg.max_blocks_per_seq, (unsigned long long)s->block_limit);
    return WWW_E_CAPACITY;
  }
  s->queue.push_back(Pending{request_id, prompt_len, max_new_tokens});
  return WWW_OK;
}

WWW_EXPORT int www_sched_plan(www_sched* s, www_sched_step* step, int32_t* prefill_slot, int32_t* prefill_q_len, int32_t* prefill_seq_len,
                              int32_t* prefill_prompt_offset, uint64_t* prefill_request, int32_t* decode_slot, int32_t* decode_seq_len,
                              uint64_t* decode_request) {
  if (!s || !step || !prefill_slot || !prefill_q_len || !prefill_seq_len || !prefill_prompt_offset || !prefill_request || !decode_slot ||
      !decode_seq_len || !decode_request) {
    set_error("NULL pointer argument");
    return WWW_E_INVALID_ARG;
  }
  if (s->planned) { set_error("the previous iteration has not been committed"); return WWW_E_INVALID_ARG; }
  const int32_t nslot = (int32_t)s->slot.size();
  // 1. admission, first come first served: the head of the queue enters when a slot is free and its blocks fit under the
  //    target share of the pool; nobody overtakes it
  while (!s->queue.empty()) {
    const Pending& p = s->queue.front();
    const uint64_t need = blocks_for(s, (int64_t)p.prompt_len + p.max_new - 1);
    if (s->blocks_reserved + need > s->block_limit) break;
    int32_t free_slot = -1;
    for (int32_t i = 0; i < nslot && free_slot < 0; ++i)
      if (!s->slot[i].active) free_slot = i;
    if (free_slot < 0) break;
    Sequence& q = s->slot[free_slot];
    q = Sequence();
    q.request = p.request; q.prompt_len = p.prompt_len; q.max_new = p.max_new; q.active = true;
    q.blocks.resize(need);
    for (uint64_t b = 0; b < need; ++b) { q.blocks[b] = s->free_blocks.back(); s->free_blocks.pop_back(); }
    s->blocks_reserved += need;
    s->queue.pop_front();
  }
  // 2. prefill chunks, round-robin from the slot after the last one served, until the first chunk that does not fit
  s->plan_prefill_slot.clear(); s->plan_prefill_q.clear(); s->plan_decode_slot.clear();
  int32_t left = (int32_t)s->cfg.token_budget, n_tok = 0;
  for (int32_t k = 0; k < nslot; ++k) {
    const int32_t i = (s->rr + k) % nslot;
    const Sequence& q = s->slot[i];
    if (!q.active || q.prefilled >= q.prompt_len) continue;
    const int32_t rest = q.prompt_len - q.prefilled;
    const int32_t chunk = rest < (int32_t)s->cfg.chunk_tokens ? rest : (int32_t)s->cfg.chunk_tokens;
    if (chunk > left) break;
    const int32_t at = (int32_t)s->plan_prefill_slot.size();
    prefill_slot[at] = i; prefill_q_len[at] = chunk; prefill_seq_len[at] = q.prefilled + chunk; prefill_prompt_offset[at] = q.prefilled;
    prefill_request[at] = q.request;
    s->plan_prefill_slot.push_back(i); s->plan_prefill_q.push_back(chunk);
    left -= chunk; n_tok += chunk;
  }
  // 3. one decode step over the sequences whose prompt is complete once this iteration's chunks are in and that still
  //    owe tokens (a sequence that completes its prompt now has produced its first token by then)
  for (int32_t i = 0; i < nslot; ++i) {
    const Sequence& q = s->slot[i];
    if (!q.active) continue;
    int32_t prefilled = q.prefilled, generated = q.generated;
    for (size_t a = 0; a < s->plan_prefill_slot.size(); ++a)
      if (s->plan_prefill_slot[a] == i) { prefilled += s->plan_prefill_q[a]; if (prefilled == q.prompt_len) generated = 1; }
    if (prefilled < q.prompt_len || generated >= q.max_new) continue;
    const int32_t at = (int32_t)s->plan_decode_slot.size();
    decode_slot[at] = i; decode_seq_len[at] = q.prompt_len + generated;  // length once the token fed to this step is appended
    decode_request[at] = q.request;
    s->plan_decode_slot.push_back(i);
  }
  step->n_prefill = (int32_t)s->plan_prefill_slot.size();
  step->n_prefill_tokens = n_tok;
  step->n_decode = (int32_t)s->plan_decode_slot.size();
  s->planned = true;
  return WWW_OK;
}

WWW_EXPORT int www_sched_table_row(const www_sched* s, int32_t slot, int32_t* row) {
  if (!s || !row || slot < 0 || slot >= (int32_t)s->slot.size()) { set_error("bad scheduler, slot or row pointer"); return WWW_E_INVALID_ARG; }
  const Sequence& q = s->slot[slot];
  for (uint32_t b = 0; b < s->cfg.max_blocks_per_seq; ++b) row[b] = (q.active && b < q.blocks.size()) ? q.blocks[b] : -1;
  return WWW_OK;
}

WWW_EXPORT int www_sched_commit(www_sched* s, int32_t* n_finished, uint64_t* finished_requests) {
  if (!s || !n_finished || !finished_requests) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  if (!s->planned) { set_error("no planned iteration to commit"); return WWW_E_INVALID_ARG; }
  for (size_t a = 0; a < s->plan_prefill_slot.size(); ++a) {
    Sequence& q = s->slot[s->plan_prefill_slot[a]];
    q.prefilled += s->plan_prefill_q[a];
    s->prompt_tokens_done += (uint64_t)s->plan_prefill_q[a];
    if (q.prefilled == q.prompt_len) { q.generated = 1; ++s->tokens_generated; }
  }
  if (!s->plan_prefill_slot.empty()) s->rr = (s->plan_prefill_slot.back() + 1) % (int32_t)s->slot.size();
  for (size_t a = 0; a < s->plan_decode_slot.size(); ++a) { ++s->slot[s->plan_decode_slot[a]].generated; ++s->tokens_generated; }
  int32_t nf = 0;
  for (size_t i = 0; i < s->slot.size(); ++i) {
    Sequence& q = s->slot[i];
    if (!q.active || q.prefilled < q.prompt_len || q.generated < q.max_new) continue;
    finished_requests[nf++] = q.request;
    for (size_t b = q.blocks.size(); b-- > 0;) s->free_blocks.push_back(q.blocks[b]);  // its first block is the next one handed out
    s->blocks_reserved -= q.blocks.size();
    q = Sequence();
    ++s->finished;
  }
  *n_finished = nf;
  ++s->iterations;
  s->planned = false;
  return WWW_OK;
}

WWW_EXPORT int www_get_stats(const www_sched* s, www_stats* out) {
  if (!s || !out) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  uint32_t active = 0;
  for (const Sequence& q : s->slot) active += q.active ? 1u : 0u;
  out->active = active;
  out->queued = (uint32_t)s->queue.size();
  out->finished = s->finished;
  out->kv_blocks_reserved = s->blocks_reserved;
  out->kv_blocks_total = s->cfg.num_kv_blocks;
  out->kv_utilisation = (double)s->blocks_reserved / (double)s->cfg.num_kv_blocks;
  out->iterations = s->iterations;
  out->prompt_tokens_done = s->prompt_tokens_done;
  out->tokens_generated = s->tokens_generated;
  return WWW_OK;
}
