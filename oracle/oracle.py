"""ctypes wrapper around www_oracle.c -- TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the CPU-baseline leg of the benchmark may import this module;
the GPU library never does.  The wrapper marshals numpy arrays and does no arithmetic of its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwww_oracle.so")
_lib = None


class OrcConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab")] + \
               [("rms_eps", ctypes.c_float), ("rope_theta", ctypes.c_float),
                ("kv_block_size", ctypes.c_int32), ("weight_dtype", ctypes.c_int32), ("qk_norm", ctypes.c_int32)]


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "www_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-march=x86-64-v3", "-std=c11",
                               "-Wall", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        L.orc_matmul.argtypes = [vp, vp, vp, ctypes.c_int, i64, i64, i64]; L.orc_matmul.restype = None
        L.orc_rmsnorm.argtypes = [vp, vp, vp, i64, dbl]; L.orc_rmsnorm.restype = None
        L.orc_rope.argtypes = [vp, vp, ctypes.c_int, i64, dbl]; L.orc_rope.restype = None
        L.orc_softmax.argtypes = [vp, vp, i64]; L.orc_softmax.restype = None
        L.orc_attend.argtypes = [vp, vp, vp, vp, i64, ctypes.c_int]; L.orc_attend.restype = None
        L.orc_silu_mul.argtypes = [vp, vp, vp, i64]; L.orc_silu_mul.restype = None
        L.orc_argmax.argtypes = [vp, i64]; L.orc_argmax.restype = i32
        L.orc_slot.argtypes = [vp, i64, ctypes.c_int]; L.orc_slot.restype = i64
        L.orc_create.argtypes = [ctypes.POINTER(OrcConfig), vp, i32, i32, i64]; L.orc_create.restype = vp
        L.orc_free.argtypes = [vp]; L.orc_free.restype = None
        L.orc_set_kv_mode.argtypes = [vp, i32]; L.orc_set_kv_mode.restype = None
        L.orc_kv_paged_ptr.argtypes = [vp]; L.orc_kv_paged_ptr.restype = vp
        L.orc_kv_contig_ptr.argtypes = [vp]; L.orc_kv_contig_ptr.restype = vp
        L.orc_blob_bytes.argtypes = [vp]; L.orc_blob_bytes.restype = ctypes.c_size_t
        L.orc_forward.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]; L.orc_forward.restype = ctypes.c_int
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


# ------------------------------------------------------------------ elementary operations
def matmul(x, w, wdtype=0):
    """x [T,K] fp32; w [N,K] fp32 (wdtype 0) or bf16 bit patterns uint16 (wdtype 1) -> [T,N]"""
    x = _f32(x)
    w = np.ascontiguousarray(w, dtype=np.float32 if wdtype == 0 else np.uint16)
    T, K = x.shape
    N = w.shape[0]
    assert w.shape[1] == K
    y = np.empty((T, N), dtype=np.float32)
    lib().orc_matmul(y.ctypes.data, x.ctypes.data, w.ctypes.data, wdtype, T, N, K)
    return y


def rmsnorm(x, g, eps):
    x, g = _f32(x), _f32(g)
    out = np.empty_like(x)
    lib().orc_rmsnorm(out.ctypes.data, x.ctypes.data, g.ctypes.data, x.size, float(eps))
    return out


def rope(x, pos, theta):
    x = _f32(x)
    out = np.empty_like(x)
    lib().orc_rope(out.ctypes.data, x.ctypes.data, x.size, int(pos), float(theta))
    return out


def softmax(s):
    s = _f32(s)
    p = np.empty_like(s)
    lib().orc_softmax(p.ctypes.data, s.ctypes.data, s.size)
    return p


def attend(q, K, V):
    q, K, V = _f32(q), _f32(K), _f32(V)
    n, hd = K.shape
    o = np.empty(hd, dtype=np.float32)
    lib().orc_attend(o.ctypes.data, q.ctypes.data, K.ctypes.data, V.ctypes.data, n, hd)
    return o


def silu_mul(g, u):
    g, u = _f32(g), _f32(u)
    a = np.empty_like(g)
    lib().orc_silu_mul(a.ctypes.data, g.ctypes.data, u.ctypes.data, g.size)
    return a


def argmax(x):
    x = _f32(x)
    return int(lib().orc_argmax(x.ctypes.data, x.size))


def slot(table_row, pos, bs=16):
    t = _i32(table_row)
    return int(lib().orc_slot(t.ctypes.data, int(pos), bs))


# ------------------------------------------------------------------ model
class OracleModel:
    """shape: any object with the ModelShape attribute names; blob: uint8 numpy array (kept alive here)."""

    def __init__(self, shape, blob, max_seqs=0, max_ctx=0, num_blocks=0):
        self.shape = shape
        self.blob = np.ascontiguousarray(blob, dtype=np.uint8)
        cfg = OrcConfig(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                        shape.ffn_dim, shape.vocab, shape.rms_eps, shape.rope_theta, shape.kv_block_size,
                        shape.weight_dtype, int(getattr(shape, "qk_norm", 0)))
        self._h = lib().orc_create(ctypes.byref(cfg), self.blob.ctypes.data, max_seqs, max_ctx, num_blocks)
        if not self._h:
            raise ValueError("orc_create rejected the configuration")
        assert lib().orc_blob_bytes(self._h) == self.blob.size, "blob size does not match the layout"
        self.max_seqs, self.max_ctx, self.num_blocks = max_seqs, max_ctx, num_blocks

    def close(self):
        if getattr(self, "_h", None):
            lib().orc_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: the module globals may already be gone
            pass

    def set_kv_mode(self, paged: bool):
        lib().orc_set_kv_mode(self._h, 1 if paged else 0)

    def kv_paged(self) -> np.ndarray:
        """view [num_blocks, L, 2, bs, Hkv*hd] fp32 of the paged pool"""
        s = self.shape
        n = self.num_blocks * s.n_layers * 2 * s.kv_block_size * s.n_kv_heads * s.head_dim
        buf = (ctypes.c_float * n).from_address(lib().orc_kv_paged_ptr(self._h))
        return np.frombuffer(buf, dtype=np.float32).reshape(self.num_blocks, s.n_layers, 2, s.kv_block_size,
                                                            s.n_kv_heads * s.head_dim)

    def forward(self, tokens, q_lens, seq_lens, seq_ids=None, block_table=None, want_logits=True, trace=False):
        """Returns (logits [B,V] fp32 or None, next_tokens [B] int32, trace [L+1,T,d] or None)."""
        tokens, q_lens, seq_lens = _i32(tokens), _i32(q_lens), _i32(seq_lens)
        B = len(q_lens)
        T = int(q_lens.sum())
        assert tokens.size == T
        sid = _i32(seq_ids) if seq_ids is not None else None
        bt = _i32(block_table) if block_table is not None else None
        mbs = bt.shape[1] if bt is not None else 0
        logits = np.empty((B, self.shape.vocab), dtype=np.float32) if want_logits else None
        nxt = np.empty(B, dtype=np.int32)
        tr = np.empty((self.shape.n_layers + 1, T, self.shape.d_model), dtype=np.float32) if trace else None
        rc = lib().orc_forward(self._h, tokens.ctypes.data, q_lens.ctypes.data, seq_lens.ctypes.data,
                               sid.ctypes.data if sid is not None else None,
                               bt.ctypes.data if bt is not None else None, mbs, B,
                               logits.ctypes.data if logits is not None else None, nxt.ctypes.data,
                               tr.ctypes.data if tr is not None else None)
        if rc != 0:
            raise ValueError(f"orc_forward failed with code {rc}")
        return logits, nxt, tr
