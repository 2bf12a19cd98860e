"""CPU oracle of the serving loop's scheduler (test infrastructure only; nothing outside tests/ may import it).

The paper treats a provider's backend as a black box that reports active and queued requests and memory utilisation
and is configured with a target utilisation (App. B "Model Manager", App. C); the policy is therefore the one stated
in include/www.h, restated here step by step in plain Python: first-come-first-served admission with the blocks of a
whole request reserved up front under the target share of the pool, chunked prefill dealt round-robin under a token
budget, one decode step over the sequences whose prompt is complete, blocks recycled last-freed-first."""
from __future__ import annotations


class Scheduler:
    def __init__(self, max_batch, max_blocks_per_seq, token_budget, chunk_tokens, num_kv_blocks, target_utilisation=0.7):
        self.nslot, self.mbs, self.budget, self.chunk = max_batch, max_blocks_per_seq, token_budget, chunk_tokens
        self.total = num_kv_blocks
        self.limit = int(target_utilisation * num_kv_blocks)
        self.free = list(range(num_kv_blocks - 1, -1, -1))      # pop() hands out 0, 1, 2, ...
        self.slots = [None] * max_batch
        self.queue = []
        self.reserved = 0
        self.rr = 0
        self.planned = None
        self.finished = self.iterations = self.prompt_tokens_done = self.tokens_generated = 0

    @staticmethod
    def blocks_needed(prompt_len, max_new):
        return (prompt_len + max_new - 1 + 15) // 16            # the last generated token is never fed back

    def submit(self, request, prompt_len, max_new):
        if prompt_len < 1 or max_new < 1:
            raise ValueError("lengths")
        need = self.blocks_needed(prompt_len, max_new)
        if need > self.mbs or need > self.limit:
            raise OverflowError("request can never be admitted")
        self.queue.append((request, prompt_len, max_new))

    def plan(self):
        assert self.planned is None
        while self.queue:
            request, plen, max_new = self.queue[0]
            need = self.blocks_needed(plen, max_new)
            if self.reserved + need > self.limit or None not in self.slots:
                break
            i = self.slots.index(None)
            self.slots[i] = {"request": request, "plen": plen, "max_new": max_new, "prefilled": 0, "generated": 0,
                             "blocks": [self.free.pop() for _ in range(need)]}
            self.reserved += need
            self.queue.pop(0)
        pre, left = [], self.budget
        for k in range(self.nslot):
            i = (self.rr + k) % self.nslot
            q = self.slots[i]
            if q is None or q["prefilled"] >= q["plen"]:
                continue
            c = min(self.chunk, q["plen"] - q["prefilled"])
            if c > left:
                break
            pre.append((i, c, q["prefilled"] + c, q["prefilled"], q["request"]))
            left -= c
        dec = []
        for i, q in enumerate(self.slots):
            if q is None:
                continue
            prefilled, generated = q["prefilled"], q["generated"]
            for e in pre:
                if e[0] == i:
                    prefilled += e[1]
                    if prefilled == q["plen"]:
                        generated = 1
            if prefilled == q["plen"] and generated < q["max_new"]:
                dec.append((i, q["plen"] + generated, q["request"]))
        self.planned = (pre, dec)
        return pre, dec

    def table_row(self, i):
        q = self.slots[i]
        blocks = q["blocks"] if q else []
        return blocks + [-1] * (self.mbs - len(blocks))

    def commit(self):
        pre, dec = self.planned
        for i, c, _, _, _ in pre:
            q = self.slots[i]
            q["prefilled"] += c
            self.prompt_tokens_done += c
            if q["prefilled"] == q["plen"]:
                q["generated"] = 1
                self.tokens_generated += 1
        if pre:
            self.rr = (pre[-1][0] + 1) % self.nslot
        for i, _, _ in dec:
            self.slots[i]["generated"] += 1
            self.tokens_generated += 1
        done = []
        for i, q in enumerate(self.slots):
            if q is not None and q["prefilled"] == q["plen"] and q["generated"] >= q["max_new"]:
                done.append(q["request"])
                self.free.extend(reversed(q["blocks"]))
                self.reserved -= len(q["blocks"])
                self.slots[i] = None
                self.finished += 1
        self.iterations += 1
        self.planned = None
        return done

    def stats(self):
        return {"active": sum(q is not None for q in self.slots), "queued": len(self.queue), "finished": self.finished,
                "kv_blocks_reserved": self.reserved, "kv_blocks_total": self.total, "kv_utilisation": self.reserved / self.total,
                "iterations": self.iterations, "prompt_tokens_done": self.prompt_tokens_done, "tokens_generated": self.tokens_generated}
