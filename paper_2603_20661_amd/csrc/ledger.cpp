// Credit ledger of the duel-and-judge mechanism (host only; Sec. 4.2, Sec. 5 Assumptions 2-3 of the paper): stakes,
// Proof-of-Stake sampling, the credit changes of served requests and settled duels.
#include <stddef.h>
#include <stdint.h>

#include <new>
#include <vector>

#include "../../include/www.h"

#define WWW_EXPORT extern "C" __attribute__((visibility("default")))

void set_error(const char* fmt, ...);

// ------------------------------------------------------------------------------------------------
// Ledger: stakes of n nodes and an append-only list of the operations that changed them.
struct www_ledger {
  std::vector<double> stake;
  www_credit_params par;
  std::vector<www_ledger_op> ops;
};

static bool node_ok(const www_ledger* l, int32_t i) { return i >= 0 && i < (int32_t)l->stake.size(); }

static void append(www_ledger* l, uint64_t request_id, int32_t kind, int32_t node, double amount) {
  l->stake[node] += amount;
  www_ledger_op op;
  op.request_id = request_id;
  op.kind = kind;
  op.node = node;
  op.amount = amount;
  op.stake_after = l->stake[node];
  l->ops.push_back(op);
}

WWW_EXPORT int www_ledger_create(int32_t n_nodes, const double* initial_stake, const www_credit_params* params, www_ledger** out) {
  if (!out) { set_error("NULL out pointer"); return WWW_E_INVALID_ARG; }
  *out = nullptr;
  if (n_nodes <= 0 || !initial_stake || !params) { set_error("ledger needs at least one node, its stakes and the parameters"); return WWW_E_INVALID_ARG; }
  if (!(params->base_reward >= 0.0) || !(params->duel_reward >= 0.0) || !(params->duel_penalty >= 0.0) || !(params->judge_reward >= 0.0)) {
    set_error("credit parameters must be non-negative numbers");
    return WWW_E_INVALID_ARG;
  }
  for (int32_t i = 0; i < n_nodes; ++i)
    if (!(initial_stake[i] >= 0.0)) { set_error("stake of node %d is negative or not a number", i); return WWW_E_INVALID_ARG; }
  www_ledger* l = new (std::nothrow) www_ledger;
  if (!l) { set_error("out of host memory"); return WWW_E_INVALID_ARG; }
  l->stake.assign(initial_stake, initial_stake + n_nodes);
  l->par = *params;
  *out = l;
  return WWW_OK;
}

WWW_EXPORT void www_ledger_free(www_ledger* l) { delete l; }

WWW_EXPORT int www_ledger_stakes(const www_ledger* l, double* out) {
  if (!l || !out) { set_error("NULL pointer argument"); return WWW_E_INVALID_ARG; }
  for (size_t i = 0; i < l->stake.size(); ++i) out[i] = l->stake[i];
  return WWW_OK;
}

WWW_EXPORT int www_pos_sample(const www_ledger* l, const double* u01, int32_t k, const int32_t* exclude, int32_t n_exclude,
                              int32_t* chosen) {
  if (!l || k < 0 || n_exclude < 0 || (k > 0 && (!u01 || !chosen)) || (n_exclude > 0 && !exclude)) {
    set_error("bad arguments to www_pos_sample");
    return WWW_E_INVALID_ARG;
  }
  const int32_t n = (int32_t)l->stake.size();
  std::vector<char> out_of_play(n, 0);
  for (int32_t e = 0; e < n_exclude; ++e) {
    if (!node_ok(l, exclude[e])) { set_error("excluded node %d does not exist", exclude[e]); return WWW_E_INVALID_ARG; }
    out_of_play[exclude[e]] = 1;
  }
  for (int32_t d = 0; d < k; ++d) {
    if (!(u01[d] >= 0.0 && u01[d] < 1.0)) { set_error("draw %d is not in [0, 1)", d); return WWW_E_INVALID_ARG; }
    double total = 0.0;  // stakes still in play, added in node order
    for (int32_t i = 0; i < n; ++i)
      if (!out_of_play[i]) total += l->stake[i];
    if (!(total > 0.0)) { set_error("no staked node left for draw %d", d); return WWW_E_CAPACITY; }
    const double target = u01[d] * total;
    double cum = 0.0;
    int32_t pick = -1, last = -1;
    for (int32_t i = 0; i < n && pick < 0; ++i) {
      if (out_of_play[i] || !(l->stake[i] > 0.0)) continue;
      cum += l->stake[i];
      last = i;
      if (target < cum) pick = i;
    }
    if (pick < 0) pick = last;  // rounding of the running sum against the total at the very end of the range
    chosen[d] = pick;
    out_of_play[pick] = 1;
  }
  return WWW_OK;
}

WWW_EXPORT int www_ledger_serve(www_ledger* l, uint64_t request_id, int32_t executor) {
  if (!l || !node_ok(l, executor)) { set_error("bad ledger or node"); return WWW_E_INVALID_ARG; }
  append(l, request_id, WWW_OP_BASE_REWARD, executor, l->par.base_reward);
  return WWW_OK;
}

WWW_EXPORT int www_ledger_duel(www_ledger* l, uint64_t request_id, int32_t executor_a, int32_t executor_b, const int32_t* judges,
                               const int32_t* verdicts, int32_t k, int32_t* winner_out) {
  if (!l || !node_ok(l, executor_a) || !node_ok(l, executor_b) || executor_a == executor_b || k < 0 || (k > 0 && (!judges || !verdicts))) {
    set_error("bad arguments to www_ledger_duel");
    return WWW_E_INVALID_ARG;
  }
  int32_t votes_b = 0;
  for (int32_t j = 0; j < k; ++j) {
    if (!node_ok(l, judges[j]) || judges[j] == executor_a || judges[j] == executor_b) { set_error("judge %d is not an eligible node", j); return WWW_E_INVALID_ARG; }
    for (int32_t i = 0; i < j; ++i)
      if (judges[i] == judges[j]) { set_error("judge %d appears twice", judges[j]); return WWW_E_INVALID_ARG; }
    if (verdicts[j] != 0 && verdicts[j] != 1) { set_error("verdict %d is neither 0 nor 1", j); return WWW_E_INVALID_ARG; }
    votes_b += verdicts[j];
  }
  const int32_t votes_a = k - votes_b;
  const int32_t winner = votes_a > votes_b ? executor_a : votes_b > votes_a ? executor_b : -1;
  if (winner >= 0) {
    const int32_t loser = winner == executor_a ? executor_b : executor_a;
    append(l, request_id, WWW_OP_DUEL_REWARD, winner, l->par.duel_reward);
    const double fine = l->stake[loser] < l->par.duel_penalty ? l->stake[loser] : l->par.duel_penalty;  // a stake never goes below zero
    append(l, request_id, WWW_OP_DUEL_PENALTY, loser, -fine);
  }
  for (int32_t j = 0; j < k; ++j) append(l, request_id, WWW_OP_JUDGE_REWARD, judges[j], l->par.judge_reward);
  if (winner_out) *winner_out = winner;
  return WWW_OK;
}

WWW_EXPORT int64_t www_ledger_num_ops(const www_ledger* l) { return l ? (int64_t)l->ops.size() : 0; }

WWW_EXPORT int www_ledger_read_ops(const www_ledger* l, int64_t first, int64_t count, www_ledger_op* out) {
  if (!l || first < 0 || count < 0 || first + count > (int64_t)l->ops.size() || (count > 0 && !out)) {
    set_error("operation range outside the ledger");
    return WWW_E_INVALID_ARG;
  }
  for (int64_t i = 0; i < count; ++i) out[i] = l->ops[first + i];
  return WWW_OK;
}
