"""CPU oracle of the duel bookkeeping (test infrastructure only; nothing outside tests/ may import it).

Written from the paper's description (Sec. 3.2 "Executor selection": a candidate is drawn with probability proportional
to its staked credit; Sec. 4.2: two executors and k judges drawn that way, the inferior executor loses part of its
stake, the superior one and the judges earn credit, the outcome is recorded; Sec. 5, Assumption 2: base reward R, duel
reward R_add, penalty P; Assumption 3: p_i = s_i / sum_j s_j).  Where the paper is silent (how a judge's output
becomes a vote, how k votes combine, what a judge earns, what happens when the stake is smaller than the penalty)
the readings are the ones stated in include/www.h.  Plain Python floats (fp64), one operation after the other."""
from __future__ import annotations

BASE_REWARD, DUEL_REWARD, DUEL_PENALTY, JUDGE_REWARD = 0, 1, 2, 3


def verdicts(logits, token_a: int, token_b: int):
    """logits: [batch][vocab] array-like of fp32 values.  Vote of each row: 0 if answer A's token scores at least as
    high as answer B's (a tie goes to the first answer), else 1; and the margin logit[a] - logit[b] in fp32."""
    import numpy as np
    lg = np.asarray(logits, dtype=np.float32)
    la, lb = lg[:, token_a], lg[:, token_b]
    return (la < lb).astype(np.int32), (la - lb).astype(np.float32)


class Ledger:
    def __init__(self, stakes, base_reward, duel_reward, duel_penalty, judge_reward):
        self.stake = [float(s) for s in stakes]
        self.R, self.R_add, self.P, self.R_judge = float(base_reward), float(duel_reward), float(duel_penalty), float(judge_reward)
        self.ops = []

    def _apply(self, request_id, kind, node, amount):
        self.stake[node] += amount
        self.ops.append((request_id, kind, node, amount, self.stake[node]))

    def pos_sample(self, u01, exclude=()):
        """Draws without replacement; draw d takes the first node (in node order, among those still in play with a
        positive stake) whose running stake sum exceeds u01[d] * (total stake in play)."""
        out_of_play = set(exclude)
        chosen = []
        for u in u01:
            total = 0.0
            for i, s in enumerate(self.stake):
                if i not in out_of_play:
                    total += s
            if not total > 0.0:
                raise ValueError("no staked node left")
            target, cum, pick, last = u * total, 0.0, None, None
            for i, s in enumerate(self.stake):
                if i in out_of_play or not s > 0.0:
                    continue
                cum += s
                last = i
                if target < cum:
                    pick = i
                    break
            if pick is None:
                pick = last
            chosen.append(pick)
            out_of_play.add(pick)
        return chosen

    def serve(self, request_id, executor):
        self._apply(request_id, BASE_REWARD, executor, self.R)

    def duel(self, request_id, executor_a, executor_b, judges, votes):
        votes_b = sum(votes)
        votes_a = len(votes) - votes_b
        winner = executor_a if votes_a > votes_b else executor_b if votes_b > votes_a else -1
        if winner >= 0:
            loser = executor_b if winner == executor_a else executor_a
            self._apply(request_id, DUEL_REWARD, winner, self.R_add)
            self._apply(request_id, DUEL_PENALTY, loser, -min(self.P, self.stake[loser]))
        for j in judges:
            self._apply(request_id, JUDGE_REWARD, j, self.R_judge)
        return winner
