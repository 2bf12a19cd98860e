"""Recipes of the full-depth parity cases (32-layer 8B-shaped and 16-layer 1B-shaped models) and the format of their
stored oracle results.

The CPU oracle needs minutes to hours for one sequence of these models, so its results are computed once by
``tests/golden/make_full_depth.py`` (which calls only the oracle and the seeded input generators) and stored under
``tests/golden/``; the GPU tests replay the same seeded jobs, teacher-forced with the stored oracle tokens, and compare
their logits with the stored values.  Per sampled sequence a file holds, for every logit row (row 0: after the prompt,
row s: after s greedy tokens):

  tokens   [rows]        the oracle's greedy token of the row (= its argmax)
  cols     [C]           a seeded sample of vocabulary columns, the same for all rows
  vals     [rows, C]     the oracle's logits at those columns
  top_idx / top_val [rows, 8]   its eight largest logits (value, then lowest index, first)
  full_rows, full [n, V] complete logit rows (the first and the last row)

Nothing here performs model arithmetic.
"""
from __future__ import annotations

import os

import numpy as np

from paper_2603_20661_amd import synth

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
N_COLS = 1024
N_TOP = 8


def golden_path(case: str) -> str:
    return os.path.join(GOLDEN_DIR, f"full_depth_{case}.npz")


def sample_columns(vocab: int, salt: int) -> np.ndarray:
    return np.sort(synth.permutation(777 + salt, synth.STREAM_MISC, vocab)[:N_COLS]).astype(np.int64)


# ------------------------------------------------------------------ the cases
def bench_case(name: str):
    """The 8B / 1B workloads of bench.py: (workload, sampled sequence ids: shortest, median, longest)."""
    wl = synth.workload(name)
    order = np.argsort(wl.prompt_lens, kind="stable")
    return wl, [int(order[0]), int(order[len(order) // 2]), int(order[-1])]


# which of the sampled sequences of a bench workload a golden file covers
BENCH_FILES = {"1b": ("1b", [0, 1, 2]), "8b": ("8b", [0, 1]), "8b-long": ("8b", [2])}

DUEL = dict(n_seq=32, plen=768, steps=256, sample=0, vote_tokens=(32, 33))


def duel_prompts():
    return synth.tokens(12345, DUEL["n_seq"] * DUEL["plen"], 32000).reshape(DUEL["n_seq"], DUEL["plen"])


MIXED = dict(n_seq=128, chunk=512, budget=8192, dec_steps=64, zipf_seed=2, sample_lens=(525, 546))


def mixed_case():
    """(lens, prompts, sampled sequence ids) of the long-context mixed batch: the sampled sequences are the ones of 525
    and 546 tokens, whose prompts are fed in two chunks."""
    m = MIXED
    lens = synth.lengths_zipf(m["zipf_seed"], m["n_seq"], 1.2, 256, 16384).astype(np.int64)
    prompts = [synth.tokens(1000 + b, int(lens[b]), synth.M8B.vocab) for b in range(m["n_seq"])]
    ids = [int(np.nonzero(lens == n)[0][0]) for n in m["sample_lens"]]
    return lens, prompts, ids


# ------------------------------------------------------------------ stored results
def pack_rows(prefix: str, logits: np.ndarray, cols: np.ndarray, out: dict):
    """logits [rows, V] fp32 of one sequence -> entries of the npz"""
    rows = logits.shape[0]
    order = np.argsort(-logits, axis=-1, kind="stable")[:, :N_TOP]     # equal values stay in index order
    out[f"{prefix}.tokens"] = order[:, 0].astype(np.int32)
    out[f"{prefix}.vals"] = np.ascontiguousarray(logits[:, cols])
    out[f"{prefix}.top_idx"] = order.astype(np.int32)
    out[f"{prefix}.top_val"] = np.take_along_axis(logits, order, axis=-1)
    full_rows = np.unique(np.array([0, rows - 1]))
    out[f"{prefix}.full_rows"] = full_rows.astype(np.int32)
    out[f"{prefix}.full"] = np.ascontiguousarray(logits[full_rows])


class Stored:
    """One sequence's stored oracle rows."""

    def __init__(self, z, prefix, cols_key="cols"):
        self.tokens = z[f"{prefix}.tokens"]
        self.vals = z[f"{prefix}.vals"]
        self.top_idx, self.top_val = z[f"{prefix}.top_idx"], z[f"{prefix}.top_val"]
        self.full_rows, self.full = z[f"{prefix}.full_rows"], z[f"{prefix}.full"]
        self.cols = z[cols_key]
        self.rows = len(self.tokens)

    def compare(self, gpu_logits: np.ndarray):
        """gpu_logits [rows, V] -> (max |dlogit| over the stored entries, per-row maxima, number of rows whose argmax is
        the oracle's token, number of rows that agree or whose oracle top-2 gap is below twice the row's error)"""
        assert gpu_logits.shape[0] == self.rows
        assert np.isfinite(gpu_logits).all(), "non-finite logits from the GPU path"
        per_row = np.abs(gpu_logits[:, self.cols] - self.vals).max(-1)
        per_row = np.maximum(per_row, np.abs(np.take_along_axis(gpu_logits, self.top_idx.astype(np.int64), -1) - self.top_val).max(-1))
        per_row[self.full_rows] = np.maximum(per_row[self.full_rows], np.abs(gpu_logits[self.full_rows] - self.full).max(-1))
        hit = gpu_logits.argmax(-1) == self.tokens
        gap = self.top_val[:, 0] - self.top_val[:, 1]
        return float(per_row.max()), per_row, int(hit.sum()), int((hit | (gap < 2 * per_row)).sum())


class LiveRows:
    """The same interface over oracle rows computed on the spot (every column of every row is compared)."""

    def __init__(self, logits: np.ndarray):
        self.logits = logits
        order = np.argsort(-logits, axis=-1, kind="stable")[:, :2]
        self.tokens = order[:, 0].astype(np.int32)
        self.gap = np.take_along_axis(logits, order[:, :1], -1)[:, 0] - np.take_along_axis(logits, order[:, 1:2], -1)[:, 0]
        self.rows = len(self.tokens)
        self.full = logits

    def compare(self, gpu_logits: np.ndarray):
        assert gpu_logits.shape == self.logits.shape
        assert np.isfinite(gpu_logits).all(), "non-finite logits from the GPU path"
        per_row = np.abs(gpu_logits - self.logits).max(-1)
        hit = gpu_logits.argmax(-1) == self.tokens
        return float(per_row.max()), per_row, int(hit.sum()), int((hit | (self.gap < 2 * per_row)).sum())
