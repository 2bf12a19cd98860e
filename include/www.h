/* www.h -- C ABI of the MI355X (gfx950) inference library behind a WWW.Serve provider node.
 *
 * In the paper a provider's Model Manager hands each dispatched request to a local serving backend
 * and only sees its completions and load figures (Sec. 3.2 "Model Manager"; App. A.1 "Local
 * execution"; App. B).  Executors generate greedily (App. C, temperature 0); a duel runs the same
 * request on two executors and each judge reads both answers in one pass (Sec. 4.2).  This library
 * is that backend's compute path: batched decoder inference with a paged KV cache.
 *
 *   www_model_load   bind a weight blob, a KV pool and a workspace; repack weights for the matrix cores
 *   www_prefill      run new prompt tokens (whole prompts or chunks) and fill the KV cache
 *   www_decode_step  append one token per sequence and return next-token logits
 *
 * The function computed is the standard pre-norm decoder (RMSNorm, grouped-query attention with
 * rotary embedding on half-split pairs, SwiGLU, untied output head, greedy argmax with the lowest
 * index winning ties); the paper itself gives no model equations.
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; the library borrows it and
 *    never allocates or frees device memory.  Pointers without the suffix are host memory.
 *  - `hip_stream` is a hipStream_t passed as void*; all work of a call is enqueued on it and the
 *    call returns without synchronising (except www_model_load, which waits for its own packing).
 *    Calls on one model must not overlap: they share the model's workspace.
 *  - Return value: 0 on success, a negative WWW_E_* code otherwise; www_last_error() then gives
 *    a message for the calling thread.  Argument checks run on the host before anything is
 *    launched.  Contents of device arrays (token ids, block ids, lengths) are by default NOT
 *    checked: the caller guarantees  0 <= token < vocab,  0 <= block id < num_kv_blocks for every
 *    block a sequence uses, distinct blocks for distinct (sequence, position/16) of a call, and
 *    1 <= q_lens <= seq_lens <= max_blocks_per_seq * 16.
 *  - Validation mode: with the environment variable WWW_VALIDATE=1 set when www_model_load runs,
 *    every www_prefill / www_decode_step of that model first checks exactly those conditions with a
 *    small kernel, WAITS for it on the stream, and returns WWW_E_INVALID_ARG without launching
 *    anything else if one is violated (the message names which).  The mode costs a stream
 *    synchronisation per call and cannot be used on a stream the caller is capturing.
 *
 * Weight blob (source format, device memory, may be released after www_model_load returns).
 * Tensors in this order, each starting on a 256-byte boundary, every matrix row-major
 * [out_features][in_features] in `weight_dtype`, gains in fp32:
 *     embed[vocab][d]
 *     per layer: attn_norm[d], wqkv[(Hq+2Hkv)*hd][d] (q heads, then k heads, then v heads),
 *                [WWW_FLAG_QK_NORM models: q_norm[hd], k_norm[hd],]
 *                wo[d][Hq*hd], ffn_norm[d], wgu[2F][d] (gate rows, then up rows), wd[d][F]
 *     final_norm[d], lm_head[vocab][d]
 *
 * KV pool (device, caller-owned, contents opaque to the caller): 16-bit codes plus one fp32 scale per (token, kv head)
 * vector of keys / values, i.e. 2 * head_dim + 4 bytes per vector (size from www_query_sizes), num_kv_blocks blocks of
 * kv_block_size = 16 token slots.  Logical position p of sequence b lives in block
 * block_table[b][p / 16], slot p % 16.
 */
#ifndef WWW_H
#define WWW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WWW_ABI_VERSION 1u

#define WWW_OK 0
#define WWW_E_INVALID_ARG (-1)  /* null pointer, negative count, misaligned buffer */
#define WWW_E_BAD_CONFIG (-2)   /* unsupported shape (see www_config) */
#define WWW_E_ABI_MISMATCH (-3) /* config.abi_version != WWW_ABI_VERSION */
#define WWW_E_CAPACITY (-4)     /* batch > max_batch, tokens > max_prefill_tokens, ... */
#define WWW_E_HIP (-5)          /* a HIP runtime call failed; message holds hipGetErrorString */
#define WWW_E_STALE (-6)        /* a kernel of an earlier call on this model found the workgroup placement rule of its
                                   split-K hand-over violated: results since the last successful call are unreliable; the
                                   model has switched to the fenced hand-over, repeat those calls (never seen so far) */

#define WWW_DTYPE_F32 0u  /* weights given in fp32: kept as two fp16 terms (hi + lo) */
#define WWW_DTYPE_BF16 1u /* weights given in bf16: converted to fp16 (exact for |w| >= 2^-17) */
#define WWW_DTYPE_FP8WO 2u /* weight-only FP8 (the paper's quantisation experiment, Sec. 6.3, names "fp8wo"; the format is
                              this library's reading): every projection matrix and the output head as OCP FP8 E4M3 codes
                              (1 byte each, row-major), each followed, on the next 256-byte boundary, by one fp32 scale in a
                              256-byte slot; weight = value(code) * scale.  The embedding stays bf16, gains fp32, and
                              activations and arithmetic are those of the unquantised model.  The decode path streams the
                              codes (half the bytes) and widens them to fp16 in registers; prefill uses an fp16 copy. */
#define WWW_DTYPE_INT4WO_128 3u /* weight-only int4, groups of 128 ("int4wo-128" of the same experiment; format again this
                              library's reading): every projection matrix and the output head as 4-bit codes c in 0..15,
                              two per byte (even column in the low nibble), row-major, followed, on the next 256-byte
                              boundary, by bf16 scales [rows][cols / 128]; weight = (c - 8) * scale of its run of 128
                              consecutive columns.  d_model, n_q_heads * head_dim and ffn_dim must be multiples of 128.
                              Everything else as for WWW_DTYPE_FP8WO. */
#define WWW_DTYPE_INT4WO_32 4u  /* the same with runs of 32 columns ("int4wo-32"); the three sizes must be multiples of 32 */

/* www_config.flags */
#define WWW_FLAG_QK_NORM 1u /* every query head and every key head is RMS-normalised over its head_dim values, with the gains
                               q_norm / k_norm of its layer (shared by the heads) and rms_eps, before the rotary embedding; the
                               value heads are not.  This is the per-head normalisation of the Qwen3 family that the paper's
                               nodes serve (Sec. 6.3, App. C); the paper itself gives no model equations. */

typedef struct www_model www_model; /* opaque handle */

/* Model shape and capacities.  Supported: head_dim in {64, 128}; d_model % 128 == 0 and <= 8192; ffn_dim % 16 == 0;
 * vocab % 16 == 0; n_q_heads / n_kv_heads in {1, 2, 4, 8}; kv_block_size == 16. */
typedef struct {
  uint32_t abi_version; /* WWW_ABI_VERSION */
  uint32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
  float rms_eps, rope_theta;
  uint32_t kv_block_size;      /* 16 */
  uint32_t weight_dtype;       /* WWW_DTYPE_* of the source blob */
  uint32_t max_batch;          /* most sequences in one call */
  uint32_t max_blocks_per_seq; /* row length of block tables; longest sequence = 16 * this */
  uint32_t max_prefill_tokens; /* most new tokens in one www_prefill call (sum of q_lens) */
  uint32_t flags;              /* WWW_FLAG_* bits, 0 for the plain decoder */
  uint64_t num_kv_blocks;      /* blocks in the KV pool */
} www_config;

/* Sizes in bytes of the three caller-provided device buffers for this configuration.
 * Any out pointer may be NULL.  Errors: INVALID_ARG, ABI_MISMATCH, BAD_CONFIG. */
int www_query_sizes(const www_config* cfg, uint64_t* weight_blob_bytes, uint64_t* kv_pool_bytes, uint64_t* workspace_bytes);

/* Creates a model.  Repacks the blob into the workspace (matrix-core fragment order), builds the
 * rotary table, zeroes the workspace's counters and waits for that work on `hip_stream`.
 * weights_dev is only read during this call.  kv_pool_dev and workspace_dev (256-byte aligned, sizes
 * from www_query_sizes) stay borrowed until www_model_free.  The KV pool is not cleared.
 * Errors: INVALID_ARG, ABI_MISMATCH, BAD_CONFIG, HIP. */
int www_model_load(const www_config* cfg, const void* weights_dev, void* kv_pool_dev, void* workspace_dev, void* hip_stream,
                   www_model** out);

/* Prefill: processes q_lens[b] new tokens of each of `batch` sequences and writes their keys and
 * values into the KV pool.  Sequence b's new tokens occupy positions seq_lens[b]-q_lens[b] ..
 * seq_lens[b]-1; earlier positions must already be cached (chunked prefill) and are attended to.
 *   tokens_dev       int32 [total_q_tokens], sequences packed back to back
 *   q_lens_dev       int32 [batch], each >= 1
 *   seq_lens_dev     int32 [batch], length after this call
 *   block_table_dev  int32 [batch][max_blocks_per_seq]; unused entries are ignored
 *   logits_dev       fp32 [batch][vocab], logits at the LAST new position of each sequence; may be NULL
 *   next_tokens_dev  int32 [batch], argmax of those logits; may be NULL
 * batch == 0 is a no-op.  Errors: INVALID_ARG, CAPACITY (batch > max_batch, total_q_tokens > max_prefill_tokens), HIP, STALE. */
int www_prefill(www_model* m, const int32_t* tokens_dev, const int32_t* q_lens_dev, const int32_t* seq_lens_dev,
                const int32_t* block_table_dev, int32_t batch, int32_t total_q_tokens, float* logits_dev, int32_t* next_tokens_dev,
                void* hip_stream);

/* One decode step: sequence b appends last_tokens[b] at position seq_lens[b]-1 (so seq_lens is the
 * length AFTER the append) and attends to positions 0 .. seq_lens[b]-1.
 *   last_tokens_dev  int32 [batch];  seq_lens_dev int32 [batch];  block_table_dev as above
 *   logits_dev       fp32 [batch][vocab]; may be NULL
 *   next_tokens_dev  int32 [batch] greedy next token; may be NULL
 * The step is replayed from a captured HIP graph keyed on (batch, pointers, stream); lengths, tables
 * and tokens are read from device memory at run time, so the same arrays can be updated in place
 * between steps.  A model keeps up to 128 captured steps (the oldest is dropped); a caller whose batch
 * changes from step to step should pass the same staging arrays every time so that each batch size is
 * captured once.  batch == 0 is a no-op.  Errors: INVALID_ARG, CAPACITY, HIP, STALE. */
int www_decode_step(www_model* m, const int32_t* last_tokens_dev, const int32_t* seq_lens_dev, const int32_t* block_table_dev,
                    int32_t batch, float* logits_dev, int32_t* next_tokens_dev, void* hip_stream);

/* Releases the handle and its HIP graphs.  Device buffers remain the caller's.  NULL is allowed. */
void www_model_free(www_model* m);

/* Message of the last error on this thread ("" if none); storage is thread-local and static. */
const char* www_last_error(void);

/* Waits for the work enqueued on hip_stream and reports what its kernels found: WWW_E_STALE if a split-K hand-over
 * saw its placement rule violated since the last check (see WWW_E_STALE; the model switches to the fenced hand-over),
 * else WWW_OK.  www_prefill / www_decode_step make the same check on entry, i.e. for the calls BEFORE them; a caller
 * that wants the verdict on the last call's results before using them calls this.  Errors: INVALID_ARG, HIP, STALE. */
int www_check(www_model* m, void* hip_stream);

/* Test hook: physical token slot of (block-table row, position), computed on the device by the same
 * routine the cache-writing kernels use.  table_row_dev int32 [n_blocks]; positions_dev int32 [n];
 * slots_dev int64 [n] receives block * 16 + position % 16.  Errors: INVALID_ARG, HIP. */
int www_debug_slots(const int32_t* table_row_dev, const int32_t* positions_dev, int32_t n, int64_t* slots_dev, void* hip_stream);

/* Test hook: copies an internal fp32 buffer of the last call to host memory after synchronising the
 * stream.  which: 0 = residual stream of the decode path [batch][d_model]; 1 = the decode path's query buffer and
 * 2 = its packed attention output, both as raw 32-bit words.  Ends with the check of www_check.
 * Errors: INVALID_ARG, HIP, STALE. */
int www_debug_read(www_model* m, int32_t which, float* dst_host, uint64_t n_floats, void* hip_stream);

/* Benchmark hook: per-kernel timing of decode steps.  While enabled, www_decode_step launches its
 * kernels one by one (no graph replay) with a HIP event in front of each; www_debug_profile_read
 * synchronises the stream and returns, for the 8 kernel classes
 *   0 embedding, 1 QKV GEMM, 2 decode attention, 3 O-projection GEMM, 4 gate/up GEMM, 5 down GEMM,
 *   6 output-head GEMM, 7 argmax,
 * the accumulated milliseconds (ms_host[8]) and number of launches (launches_host[8]) since the last
 * read, then clears them.  Errors: INVALID_ARG, HIP. */
int www_debug_profile(www_model* m, int32_t enable);
int www_debug_profile_read(www_model* m, float* ms_host, int32_t* launches_host, void* hip_stream);

/* Benchmark hook: launches a kernel of `workgroups` workgroups of four wavefronts that does nothing but `iters` rounds of
 * eight independent fp16 32x32x16 MFMAs per wavefront on pseudo-random register operands (no memory traffic), and
 * writes one float per wavefront to sink_dev [workgroups * 4] so that the work cannot be dropped.  *flops_out (host,
 * may be NULL) receives the floating-point operations of the launch; the caller times it.  This is the measured
 * matrix-core rate of the GPU at hand, to set beside the published dense peak.  Errors: INVALID_ARG, HIP. */
int www_debug_mfma_loop(int32_t workgroups, int32_t iters, float* sink_dev, double* flops_out, void* hip_stream);

/* Test hook, host only (no GPU call): the tile that workgroup `workgroup` of a prefill projection GEMM over token_tiles x
 * row_tiles tiles of 256 x 256 works on.  The order is laid out for the 8 L2 caches of the GPU (Sec. 3.2 names no kernel
 * design; this is the library's own); what a test can check is that it visits every tile exactly once.  Outputs are
 * host pointers.  Errors: INVALID_ARG (null pointers, counts below 1, workgroup outside [0, token_tiles * row_tiles)). */
int www_debug_prefill_tile(int32_t workgroup, int32_t token_tiles, int32_t row_tiles, int32_t* token_tile_out, int32_t* row_tile_out);

/* ------------------------------------------------------------------------------------------------
 * Duel bookkeeping (Sec. 4.2 "Duel-and-Judge Mechanism"; Sec. 5, Assumptions 2 and 3).
 *
 * A duel sends one request to two executors drawn by Proof-of-Stake; k judges, drawn the same way, compare the two
 * answers; the loser forfeits part of its stake, the winner and the judges earn credit, and the outcome is recorded in
 * the credit ledger.  The paper fixes the selection law p_i = s_i / sum_j s_j and the parameters R (base reward of a
 * served request), R_add (reward for winning a duel) and P (penalty for losing one); how a judge's output becomes a
 * vote, how k votes are combined, and the size of the judges' reward are not in the paper.  Chosen here:
 *   - a judge's vote is read off its last-position logits: answer A wins iff logit[token_a] >= logit[token_b];
 *   - the executor with more votes wins; with equal votes there is no winner and no stake moves between executors;
 *   - the loser pays min(P, its stake) (stakes stay >= 0, Assumption 1); every judge of the duel earns judge_reward;
 *   - draws are without replacement among nodes with a positive stake; the random numbers are the caller's.
 * The ledger is host memory owned by the library; it is not thread-safe. */

/* Votes of a judge pass.  logits_dev fp32 [batch][vocab] (as written by www_prefill); verdict_dev int32 [batch]
 * receives 0 (answer A) or 1 (answer B); margin_dev fp32 [batch] receives logit[token_a] - logit[token_b], may be
 * NULL.  batch == 0 is a no-op.  Errors: INVALID_ARG (tokens out of range or equal, NULL), HIP. */
int www_judge_verdict(const float* logits_dev, int32_t batch, int32_t vocab, int32_t token_a, int32_t token_b,
                      int32_t* verdict_dev, float* margin_dev, void* hip_stream);

typedef struct www_credit_params {
  double base_reward;  /* R: credited to an executor for every delegated request it serves */
  double duel_reward;  /* R_add: credited to the winner of a duel */
  double duel_penalty; /* P: taken from the loser of a duel */
  double judge_reward; /* credited to every judge of a duel */
} www_credit_params;

#define WWW_OP_BASE_REWARD 0
#define WWW_OP_DUEL_REWARD 1
#define WWW_OP_DUEL_PENALTY 2
#define WWW_OP_JUDGE_REWARD 3

typedef struct www_ledger_op {
  uint64_t request_id;
  int32_t kind; /* WWW_OP_* */
  int32_t node;
  double amount;      /* signed change of the node's stake */
  double stake_after; /* the node's stake once the operation is applied */
} www_ledger_op;

typedef struct www_ledger www_ledger;

/* New ledger over n_nodes nodes with the given stakes (host array, copied; each >= 0).  Errors: INVALID_ARG. */
int www_ledger_create(int32_t n_nodes, const double* initial_stake, const www_credit_params* params, www_ledger** out);
void www_ledger_free(www_ledger* ledger); /* NULL is allowed */
/* Copies the current stakes into out[n_nodes] (host). */
int www_ledger_stakes(const www_ledger* ledger, double* out);

/* k Proof-of-Stake draws without replacement (Sec. 3.2 "Executor selection"; Assumption 3: p_i = s_i / sum_j s_j
 * over the nodes still in play).  u01[k]: the caller's uniform numbers in [0, 1); draw d picks the first node, in node
 * order, whose running stake sum exceeds u01[d] times the total still in play; nodes in exclude[n_exclude], nodes
 * already drawn and nodes without stake are out of play.  chosen[k] receives the node ids.  Errors: INVALID_ARG,
 * CAPACITY (fewer staked nodes in play than draws). */
int www_pos_sample(const www_ledger* ledger, const double* u01, int32_t k, const int32_t* exclude, int32_t n_exclude,
                   int32_t* chosen);

/* Records that `executor` served delegated request `request_id`: + base_reward. */
int www_ledger_serve(www_ledger* ledger, uint64_t request_id, int32_t executor);

/* Settles a duel: verdicts[j] in {0, 1} is judge judges[j]'s vote for executor_a (0) or executor_b (1); judges are
 * distinct nodes other than the executors; k may be 0.  Appends, in this order: winner + duel_reward and loser
 * - min(duel_penalty, stake) if there is a winner, then + judge_reward for every judge in the given order.
 * *winner_out (may be NULL) receives the winning node or -1.  Errors: INVALID_ARG (nothing is applied). */
int www_ledger_duel(www_ledger* ledger, uint64_t request_id, int32_t executor_a, int32_t executor_b, const int32_t* judges,
                    const int32_t* verdicts, int32_t k, int32_t* winner_out);

/* Number of operations recorded so far, and a copy of operations [first, first + count) into out (host). */
int64_t www_ledger_num_ops(const www_ledger* ledger);
int www_ledger_read_ops(const www_ledger* ledger, int64_t first, int64_t count, www_ledger_op* out);

/* ------------------------------------------------------------------------------------------------
 * Serving loop of one provider (App. B "Model Manager": the node polls its backend for the number of active and
 * queued requests and the memory utilisation; App. C: target utilisation 70 %).  Host-side only; it plans which
 * sequences go into the next www_prefill / www_decode_step calls and owns the KV blocks.  The paper treats the backend
 * as a black box, so the policy is this library's: requests are admitted first come first served (nobody overtakes
 * the head of the queue) while a block-table row is free and the blocks they can ever need, ceil((prompt +
 * max_new_tokens - 1) / 16), fit under target_utilisation * num_kv_blocks (reserved at admission, so a running
 * sequence is never evicted); each iteration feeds prompt chunks of at most chunk_tokens, round-robin over the
 * sequences still prefilling and starting behind the last one served, until the first chunk that would exceed
 * token_budget, and then runs one decode step over every sequence whose prompt is complete (the prefill call that
 * completes a prompt yields the sequence's first token).  A request ends after max_new_tokens tokens; its blocks go
 * back to the free list (last freed, first reused).  Not thread-safe. */
typedef struct www_sched_config {
  uint32_t max_batch;          /* sequences resident at once = rows ("slots") of the block table */
  uint32_t max_blocks_per_seq; /* columns of the block table */
  uint32_t token_budget;       /* new prompt tokens per iteration (<= the model's max_prefill_tokens) */
  uint32_t chunk_tokens;       /* longest prompt chunk of one sequence per iteration */
  uint32_t kv_block_size;      /* 16 */
  uint32_t reserved;           /* 0 */
  uint64_t num_kv_blocks;      /* blocks of the model's KV pool */
  double target_utilisation;   /* in (0, 1]: share of the pool that admitted sequences may reserve */
} www_sched_config;

typedef struct www_sched_step {
  int32_t n_prefill;        /* sequences in this iteration's www_prefill call (0: no call) */
  int32_t n_prefill_tokens; /* sum of their chunk lengths */
  int32_t n_decode;         /* sequences in this iteration's www_decode_step call (0: no call) */
} www_sched_step;

typedef struct www_stats {
  uint32_t active, queued;     /* sequences holding a slot / requests waiting */
  uint64_t finished;           /* requests completed so far */
  uint64_t kv_blocks_reserved, kv_blocks_total;
  double kv_utilisation;       /* reserved / total */
  uint64_t iterations, prompt_tokens_done, tokens_generated;
} www_stats;

typedef struct www_sched www_sched;

/* Errors: INVALID_ARG, BAD_CONFIG. */
int www_sched_create(const www_sched_config* cfg, www_sched** out);
void www_sched_free(www_sched* sched); /* NULL is allowed */

/* Queues a request.  Errors: INVALID_ARG (lengths < 1), CAPACITY (it could never be admitted). */
int www_sched_submit(www_sched* sched, uint64_t request_id, int32_t prompt_len, int32_t max_new_tokens);

/* Admits what fits and plans one iteration.  All arrays are host memory with room for max_batch entries.
 * Prefill call, entry i < n_prefill: block-table row prefill_slot[i], chunk of prefill_q_len[i] tokens taken from
 * position prefill_prompt_offset[i] of request prefill_request[i]'s prompt, sequence length afterwards
 * prefill_seq_len[i].  Decode call, entry i < n_decode: row decode_slot[i], length decode_seq_len[i] once the token
 * fed to the step is appended; that token is the sequence's latest one (from this iteration's prefill call if the
 * prompt was completed there).  The plan must be executed and committed before the next one.  Errors: INVALID_ARG. */
int www_sched_plan(www_sched* sched, www_sched_step* step, int32_t* prefill_slot, int32_t* prefill_q_len, int32_t* prefill_seq_len,
                   int32_t* prefill_prompt_offset, uint64_t* prefill_request, int32_t* decode_slot, int32_t* decode_seq_len,
                   uint64_t* decode_request);

/* Block-table row of a slot: row_host[max_blocks_per_seq], -1 beyond the sequence's reservation. */
int www_sched_table_row(const www_sched* sched, int32_t slot, int32_t* row_host);

/* Marks the planned iteration as executed: counters advance, requests that have all their tokens leave and are listed
 * in finished_requests[max_batch] (*n_finished of them, in slot order).  Errors: INVALID_ARG (nothing planned). */
int www_sched_commit(www_sched* sched, int32_t* n_finished, uint64_t* finished_requests);

/* The figures a Model Manager polls. */
int www_get_stats(const www_sched* sched, www_stats* out);

/* ------------------------------------------------------------------------------------------------
 * Sampling beyond greedy (App. C lists temperature and top-p among the generation parameters; the paper's own runs
 * use temperature 0, which is the greedy token www_decode_step already returns).  Definition used here, per row:
 * p = softmax(logits / temperature); the nucleus is {i : p_i >= tau} for the largest tau among the probabilities whose
 * members' mass reaches top_p (equal probabilities enter together); the token is the first member, in index order,
 * whose running mass exceeds u01[row] times the nucleus mass.  No sort is involved and every sum has a fixed order, so
 * a call is reproducible; against an exact evaluation the choice can differ only where a sum lies within fp32
 * rounding of a decision point.
 *   logits_dev fp32 [batch][vocab]; u01_dev fp32 [batch], the caller's uniform numbers in [0, 1);
 *   scratch_dev fp32 [batch][vocab], overwritten (unnormalised probabilities); tokens_dev int32 [batch].
 * temperature > 0, 0 < top_p <= 1; batch == 0 is a no-op.  Errors: INVALID_ARG, HIP. */
int www_sample_top_p(const float* logits_dev, int32_t batch, int32_t vocab, float temperature, float top_p, const float* u01_dev,
                     float* scratch_dev, int32_t* tokens_dev, void* hip_stream);

/* www_sample_top_p for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernel and the same results, with the [batch][vocab] buffer of
 * unnormalised probabilities in an array built into the library (WWW_SAMPLE_STATIC_MAX_FLOATS floats = 32 MiB of
 * device memory on every GPU the library runs on, held until the process ends) instead of scratch_dev.  The call
 * allocates and frees nothing.  batch * vocab must not exceed WWW_SAMPLE_STATIC_MAX_FLOATS (enough for 64 rows of a
 * 128 256-token vocabulary).  All calls on one GPU share the array: calls that overlap on one GPU race; calls on one
 * stream are ordered.  The first call on a device looks the array's address up (no allocation; make it outside a
 * capture).  Errors: INVALID_ARG, CAPACITY (batch * vocab too large), HIP. */
#define WWW_SAMPLE_STATIC_MAX_FLOATS (8u << 20)
int www_sample_top_p_static(const float* logits_dev, int32_t batch, int32_t vocab, float temperature, float top_p,
                            const float* u01_dev, int32_t* tokens_dev, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* WWW_H */
