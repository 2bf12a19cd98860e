"""ctypes binding of the C ABI declared in include/www.h.

Argument marshalling only: every function takes torch CUDA tensors (used purely as device memory)
and passes their raw pointers on; every step of the computation runs in the HIP kernels of
libwww.so.  There is no CPU fallback: importing this module fails if the library has not been built.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwww.so")

ABI_VERSION = 1
E_INVALID_ARG, E_BAD_CONFIG, E_ABI_MISMATCH, E_CAPACITY, E_HIP, E_STALE = -1, -2, -3, -4, -5, -6
EXPORTS = ("www_query_sizes", "www_model_load", "www_prefill", "www_decode_step", "www_model_free", "www_last_error",
           "www_debug_slots", "www_debug_read", "www_debug_profile", "www_debug_profile_read",
           "www_judge_verdict", "www_ledger_create", "www_ledger_free", "www_ledger_stakes", "www_pos_sample", "www_ledger_serve",
           "www_ledger_duel", "www_ledger_num_ops", "www_ledger_read_ops",
           "www_sched_create", "www_sched_free", "www_sched_submit", "www_sched_plan", "www_sched_table_row", "www_sched_commit",
           "www_get_stats", "www_sample_top_p", "www_sample_top_p_static", "www_check", "www_debug_mfma_loop", "www_debug_prefill_tile")
FLAG_QK_NORM = 1
OP_BASE_REWARD, OP_DUEL_REWARD, OP_DUEL_PENALTY, OP_JUDGE_REWARD = 0, 1, 2, 3


class WwwConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("abi_version", "n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab")] + \
               [("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float)] + \
               [(n, ctypes.c_uint32) for n in ("kv_block_size", "weight_dtype", "max_batch", "max_blocks_per_seq",
                                               "max_prefill_tokens", "flags")] + \
               [("num_kv_blocks", ctypes.c_uint64)]


class WwwCreditParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("base_reward", "duel_reward", "duel_penalty", "judge_reward")]


class WwwLedgerOp(ctypes.Structure):
    _fields_ = [("request_id", ctypes.c_uint64), ("kind", ctypes.c_int32), ("node", ctypes.c_int32),
                ("amount", ctypes.c_double), ("stake_after", ctypes.c_double)]


class WwwSchedConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("max_batch", "max_blocks_per_seq", "token_budget", "chunk_tokens", "kv_block_size",
                                               "reserved")] + [("num_kv_blocks", ctypes.c_uint64), ("target_utilisation", ctypes.c_double)]


class WwwSchedStep(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_prefill", "n_prefill_tokens", "n_decode")]


class WwwStats(ctypes.Structure):
    _fields_ = [("active", ctypes.c_uint32), ("queued", ctypes.c_uint32), ("finished", ctypes.c_uint64),
                ("kv_blocks_reserved", ctypes.c_uint64), ("kv_blocks_total", ctypes.c_uint64), ("kv_utilisation", ctypes.c_double),
                ("iterations", ctypes.c_uint64), ("prompt_tokens_done", ctypes.c_uint64), ("tokens_generated", ctypes.c_uint64)]


class WwwError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"www error {code}: {msg}")
        self.code = code


def _load_library():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2603_20661_amd.build)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, u64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_uint64)
    cfgp = ctypes.POINTER(WwwConfig)
    L.www_query_sizes.argtypes = [cfgp, u64p, u64p, u64p]
    L.www_model_load.argtypes = [cfgp, vp, vp, vp, vp, ctypes.POINTER(vp)]
    L.www_prefill.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]
    L.www_decode_step.argtypes = [vp, vp, vp, vp, i32, vp, vp, vp]
    L.www_model_free.argtypes = [vp]
    L.www_model_free.restype = None
    L.www_last_error.argtypes = []
    L.www_last_error.restype = ctypes.c_char_p
    L.www_debug_mfma_loop.argtypes = [i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    L.www_debug_mfma_loop.restype = ctypes.c_int
    L.www_debug_prefill_tile.argtypes = [i32, i32, i32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    L.www_debug_prefill_tile.restype = ctypes.c_int
    L.www_check.argtypes = [vp, vp]
    L.www_check.restype = ctypes.c_int
    L.www_debug_slots.argtypes = [vp, vp, i32, vp, vp]
    L.www_debug_read.argtypes = [vp, i32, vp, ctypes.c_uint64, vp]
    L.www_debug_profile.argtypes = [vp, i32]
    L.www_debug_profile_read.argtypes = [vp, vp, vp, vp]
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
    L.www_judge_verdict.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp]
    L.www_ledger_create.argtypes = [i32, dp, ctypes.POINTER(WwwCreditParams), ctypes.POINTER(vp)]
    L.www_ledger_free.argtypes = [vp]
    L.www_ledger_free.restype = None
    L.www_ledger_stakes.argtypes = [vp, dp]
    L.www_pos_sample.argtypes = [vp, dp, i32, ip, i32, ip]
    L.www_ledger_serve.argtypes = [vp, ctypes.c_uint64, i32]
    L.www_ledger_duel.argtypes = [vp, ctypes.c_uint64, i32, i32, ip, ip, i32, ip]
    L.www_ledger_num_ops.argtypes = [vp]
    L.www_ledger_num_ops.restype = ctypes.c_int64
    L.www_ledger_read_ops.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, ctypes.POINTER(WwwLedgerOp)]
    u64a = ctypes.POINTER(ctypes.c_uint64)
    L.www_sched_create.argtypes = [ctypes.POINTER(WwwSchedConfig), ctypes.POINTER(vp)]
    L.www_sched_free.argtypes = [vp]
    L.www_sched_free.restype = None
    L.www_sched_submit.argtypes = [vp, ctypes.c_uint64, i32, i32]
    L.www_sched_plan.argtypes = [vp, ctypes.POINTER(WwwSchedStep), ip, ip, ip, ip, u64a, ip, ip, u64a]
    L.www_sched_table_row.argtypes = [vp, i32, ip]
    L.www_sched_commit.argtypes = [vp, ip, u64a]
    L.www_get_stats.argtypes = [vp, ctypes.POINTER(WwwStats)]
    L.www_sample_top_p.argtypes = [vp, i32, i32, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp]
    L.www_sample_top_p.restype = ctypes.c_int
    L.www_sample_top_p_static.argtypes = [vp, i32, i32, ctypes.c_float, ctypes.c_float, vp, vp, vp]
    L.www_sample_top_p_static.restype = ctypes.c_int
    for name in ("www_query_sizes", "www_model_load", "www_prefill", "www_decode_step", "www_debug_slots", "www_debug_read",
                 "www_debug_profile", "www_debug_profile_read", "www_judge_verdict", "www_ledger_create", "www_ledger_stakes",
                 "www_pos_sample", "www_ledger_serve", "www_ledger_duel", "www_ledger_read_ops", "www_sched_create", "www_sched_submit",
                 "www_sched_plan", "www_sched_table_row", "www_sched_commit", "www_get_stats"):
        getattr(L, name).restype = ctypes.c_int
    return L


lib = _load_library()


def _check(rc):
    if rc != 0:
        raise WwwError(rc, lib.www_last_error().decode())


def make_config(shape, max_batch, max_blocks_per_seq, max_prefill_tokens, num_kv_blocks) -> WwwConfig:
    """shape: object with the model-shape attribute names (n_layers, d_model, ...)."""
    return WwwConfig(ABI_VERSION, shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                     shape.ffn_dim, shape.vocab, shape.rms_eps, shape.rope_theta, shape.kv_block_size, shape.weight_dtype,
                     max_batch, max_blocks_per_seq, max_prefill_tokens, FLAG_QK_NORM if getattr(shape, "qk_norm", 0) else 0,
                     num_kv_blocks)


def www_query_sizes(cfg: WwwConfig):
    """-> (weight_blob_bytes, kv_pool_bytes, workspace_bytes)"""
    a, b, c = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib.www_query_sizes(ctypes.byref(cfg), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def _ptr(t, dtype=None):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return t.data_ptr()


def _stream(stream):
    return (stream if stream is not None else torch.cuda.current_stream()).cuda_stream


class Model:
    """Owns the device buffers (torch allocations) the library borrows, and the opaque handle."""

    def __init__(self, cfg: WwwConfig, blob_dev: torch.Tensor, stream=None, kv_fill=None):
        wbytes, kvbytes, wsbytes = www_query_sizes(cfg)
        assert blob_dev.dtype == torch.uint8 and blob_dev.numel() == wbytes, (blob_dev.numel(), wbytes)
        self.cfg = cfg
        self.kv_pool = torch.empty(kvbytes, dtype=torch.uint8, device=blob_dev.device)
        if kv_fill is not None:
            self.kv_pool.view(torch.int16).fill_(kv_fill)
        self.workspace = torch.empty(wsbytes, dtype=torch.uint8, device=blob_dev.device)
        h = ctypes.c_void_p()
        _check(lib.www_model_load(ctypes.byref(cfg), _ptr(blob_dev), _ptr(self.kv_pool), _ptr(self.workspace), _stream(stream),
                                  ctypes.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib.www_model_free(self._h)
            self._h = None

    def __del__(self):
        self.close()


def www_prefill(model: Model, tokens, q_lens, seq_lens, block_table, logits=None, next_tokens=None, stream=None):
    i32 = torch.int32
    batch, total = q_lens.numel(), tokens.numel()
    if logits is not None:
        assert logits.shape == (batch, model.cfg.vocab)
    _check(lib.www_prefill(model._h, _ptr(tokens, i32), _ptr(q_lens, i32), _ptr(seq_lens, i32), _ptr(block_table, i32), batch, total,
                           _ptr(logits, torch.float32), _ptr(next_tokens, i32), _stream(stream)))


def www_decode_step(model: Model, last_tokens, seq_lens, block_table, logits=None, next_tokens=None, stream=None):
    i32 = torch.int32
    batch = last_tokens.numel()
    if logits is not None:
        assert logits.shape == (batch, model.cfg.vocab)
    _check(lib.www_decode_step(model._h, _ptr(last_tokens, i32), _ptr(seq_lens, i32), _ptr(block_table, i32), batch,
                               _ptr(logits, torch.float32), _ptr(next_tokens, i32), _stream(stream)))


def www_debug_mfma_loop(workgroups: int, iters: int, sink, stream=None) -> float:
    """launches the pure-MFMA loop; sink fp32 [workgroups * 4]; -> floating-point operations of the launch"""
    assert sink.numel() >= workgroups * 4
    flops = ctypes.c_double()
    _check(lib.www_debug_mfma_loop(workgroups, iters, _ptr(sink, torch.float32), ctypes.byref(flops), _stream(stream)))
    return flops.value


def www_debug_prefill_tile(workgroup: int, token_tiles: int, row_tiles: int):
    """(token tile, row tile) that a workgroup of the prefill GEMM works on; host only"""
    tt, rt = ctypes.c_int32(), ctypes.c_int32()
    _check(lib.www_debug_prefill_tile(workgroup, token_tiles, row_tiles, ctypes.byref(tt), ctypes.byref(rt)))
    return tt.value, rt.value


def www_check(model: Model, stream=None):
    """waits for the stream; raises WwwError(E_STALE) if a kernel of the finished work reported a hand-over violation"""
    _check(lib.www_check(model._h, _stream(stream)))


def www_debug_slots(table_row, positions, stream=None):
    out = torch.empty(positions.numel(), dtype=torch.int64, device=positions.device)
    _check(lib.www_debug_slots(_ptr(table_row, torch.int32), _ptr(positions, torch.int32), positions.numel(), _ptr(out), _stream(stream)))
    return out


def www_debug_read(model: Model, which: int, n_floats: int, stream=None):
    out = torch.empty(n_floats, dtype=torch.float32)
    _check(lib.www_debug_read(model._h, which, out.data_ptr(), n_floats, _stream(stream)))
    return out


KERNEL_CLASSES = ("embed", "qkv_gemm", "decode_attention", "o_gemm", "gate_up_gemm", "down_gemm", "lm_head_gemm", "argmax")


def www_debug_profile(model: Model, enable: bool):
    _check(lib.www_debug_profile(model._h, 1 if enable else 0))


def www_debug_profile_read(model: Model, stream=None):
    """-> {class name: (total ms, launches)} since the last read"""
    ms = (ctypes.c_float * 8)()
    n = (ctypes.c_int32 * 8)()
    _check(lib.www_debug_profile_read(model._h, ms, n, _stream(stream)))
    return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(KERNEL_CLASSES)}


def www_judge_verdict(logits, token_a: int, token_b: int, verdict, margin=None, stream=None):
    """logits fp32 [batch, vocab] -> verdict int32 [batch] (0: answer A, 1: answer B), margin fp32 [batch] (optional)"""
    batch, vocab = logits.shape
    _check(lib.www_judge_verdict(_ptr(logits, torch.float32), batch, vocab, token_a, token_b, _ptr(verdict, torch.int32),
                                 _ptr(margin, torch.float32), _stream(stream)))


def www_sample_top_p(logits, temperature: float, top_p: float, u01, scratch, tokens, stream=None):
    """logits fp32 [batch, vocab], u01 fp32 [batch], scratch fp32 [batch, vocab] (overwritten) -> tokens int32 [batch]"""
    batch, vocab = logits.shape
    assert scratch.numel() >= batch * vocab
    _check(lib.www_sample_top_p(_ptr(logits, torch.float32), batch, vocab, temperature, top_p, _ptr(u01, torch.float32),
                                _ptr(scratch, torch.float32), _ptr(tokens, torch.int32), _stream(stream)))


SAMPLE_STATIC_MAX_FLOATS = 8 << 20


def www_sample_top_p_static(logits, temperature: float, top_p: float, u01, tokens, stream=None):
    """www_sample_top_p with the library's built-in scratch array (no device allocation anywhere in the call)"""
    batch, vocab = logits.shape
    _check(lib.www_sample_top_p_static(_ptr(logits, torch.float32), batch, vocab, temperature, top_p, _ptr(u01, torch.float32),
                                       _ptr(tokens, torch.int32), _stream(stream)))


class Ledger:
    """Handle of a host-side credit ledger (argument marshalling only)."""

    def __init__(self, stakes, base_reward, duel_reward, duel_penalty, judge_reward):
        n = len(stakes)
        self.n = n
        par = WwwCreditParams(base_reward, duel_reward, duel_penalty, judge_reward)
        h = ctypes.c_void_p()
        _check(lib.www_ledger_create(n, (ctypes.c_double * n)(*[float(x) for x in stakes]), ctypes.byref(par), ctypes.byref(h)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            lib.www_ledger_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def stakes(self):
        out = (ctypes.c_double * self.n)()
        _check(lib.www_ledger_stakes(self._h, out))
        return list(out)

    def pos_sample(self, u01, exclude=()):
        k, ne = len(u01), len(exclude)
        chosen = (ctypes.c_int32 * max(k, 1))()
        _check(lib.www_pos_sample(self._h, (ctypes.c_double * max(k, 1))(*[float(u) for u in u01]), k,
                                  (ctypes.c_int32 * max(ne, 1))(*[int(e) for e in exclude]), ne, chosen))
        return list(chosen)[:k]

    def serve(self, request_id: int, executor: int):
        _check(lib.www_ledger_serve(self._h, request_id, executor))

    def duel(self, request_id: int, executor_a: int, executor_b: int, judges, verdicts) -> int:
        k = len(judges)
        assert len(verdicts) == k
        winner = ctypes.c_int32(-2)
        _check(lib.www_ledger_duel(self._h, request_id, executor_a, executor_b, (ctypes.c_int32 * max(k, 1))(*[int(j) for j in judges]),
                                   (ctypes.c_int32 * max(k, 1))(*[int(v) for v in verdicts]), k, ctypes.byref(winner)))
        return winner.value

    def ops(self):
        n = lib.www_ledger_num_ops(self._h)
        out = (WwwLedgerOp * max(n, 1))()
        _check(lib.www_ledger_read_ops(self._h, 0, n, out))
        return [(o.request_id, o.kind, o.node, o.amount, o.stake_after) for o in out[:n]]


class Scheduler:
    """Handle of a host-side continuous-batching scheduler (argument marshalling only)."""

    def __init__(self, max_batch, max_blocks_per_seq, token_budget, chunk_tokens, num_kv_blocks, target_utilisation=0.7):
        self.cfg = WwwSchedConfig(max_batch, max_blocks_per_seq, token_budget, chunk_tokens, 16, 0, num_kv_blocks, target_utilisation)
        h = ctypes.c_void_p()
        _check(lib.www_sched_create(ctypes.byref(self.cfg), ctypes.byref(h)))
        self._h = h
        n = max_batch
        self._i = [(ctypes.c_int32 * n)() for _ in range(6)]
        self._r = [(ctypes.c_uint64 * n)() for _ in range(3)]
        self._row = (ctypes.c_int32 * max_blocks_per_seq)()

    def close(self):
        if getattr(self, "_h", None):
            lib.www_sched_free(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def submit(self, request_id: int, prompt_len: int, max_new_tokens: int):
        _check(lib.www_sched_submit(self._h, request_id, prompt_len, max_new_tokens))

    def plan(self):
        """-> (prefill entries [(slot, q_len, seq_len, prompt_offset, request)], decode entries [(slot, seq_len, request)])"""
        st = WwwSchedStep()
        ps, pq, pl, po, ds, dl = self._i
        pr, dr, _ = self._r
        _check(lib.www_sched_plan(self._h, ctypes.byref(st), ps, pq, pl, po, pr, ds, dl, dr))
        pre = [(ps[i], pq[i], pl[i], po[i], pr[i]) for i in range(st.n_prefill)]
        assert sum(e[1] for e in pre) == st.n_prefill_tokens
        return pre, [(ds[i], dl[i], dr[i]) for i in range(st.n_decode)]

    def table_row(self, slot: int):
        _check(lib.www_sched_table_row(self._h, slot, self._row))
        return list(self._row)

    def commit(self):
        """-> requests that finished with this iteration"""
        n = ctypes.c_int32()
        _check(lib.www_sched_commit(self._h, ctypes.byref(n), self._r[2]))
        return list(self._r[2][:n.value])

    def stats(self) -> dict:
        st = WwwStats()
        _check(lib.www_get_stats(self._h, ctypes.byref(st)))
        return {f: getattr(st, f) for f, _ in WwwStats._fields_}
