"""Seeded synthetic inputs (weights, tokens, lengths, block tables) for tests and benchmarks.

Nothing here performs any step of transformer inference: the module only draws reproducible
pseudo-random numbers (from the counter-based generator in ``wwwsynth.c``) and arranges them in
the documented weight-blob format.  Both the CPU oracle and the GPU library are handed the
buffers produced here, which is what makes their outputs comparable element by element.

Workload recipes (shapes, length distributions, seeds) follow the five synthetic
configurations this repository is measured on; they stand in for the trained checkpoints and
the prompt dataset of the paper's experiments (App. C), none of which are reproduced.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field, asdict

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libwwwsynth.so")
_lib = None

WDTYPE_F32 = 0
WDTYPE_BF16 = 1
WDTYPE_FP8WO = 2   # matrices as FP8 E4M3 codes with one fp32 scale per matrix; embedding bf16
WDTYPE_INT4WO_128 = 3   # matrices as 4-bit codes with one bf16 scale per 128 consecutive weights of a row; embedding bf16
WDTYPE_INT4WO_32 = 4    # the same with groups of 32
INT4_GROUP = {WDTYPE_INT4WO_128: 128, WDTYPE_INT4WO_32: 32}
KV_BLOCK = 16
ALIGN = 256  # every tensor of the weight blob starts on a 256-byte boundary


def build(force: bool = False) -> str:
    """Compile the generator with gcc (host only)."""
    src = os.path.join(_HERE, "wwwsynth.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-march=x86-64-v2",
                               "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        u64, dbl, vp = ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
        lib.wwwsynth_normal_f32.argtypes = [u64, u64, u64, u64, dbl, dbl, vp]
        lib.wwwsynth_normal_bf16.argtypes = [u64, u64, u64, u64, dbl, dbl, vp]
        lib.wwwsynth_words.argtypes = [u64, u64, u64, u64, vp]
        lib.wwwsynth_uniform_i32.argtypes = [u64, u64, u64, u64, ctypes.c_uint32, vp]
        lib.wwwsynth_encode_e4m3.argtypes = [vp, u64, dbl, vp]
        lib.wwwsynth_encode_e4m3.restype = None
        lib.wwwsynth_encode_int4.argtypes = [vp, u64, u64, u64, vp, vp]
        lib.wwwsynth_encode_int4.restype = None
        lib.wwwsynth_mix.argtypes = [u64]
        lib.wwwsynth_mix.restype = u64
        for f in (lib.wwwsynth_normal_f32, lib.wwwsynth_normal_bf16, lib.wwwsynth_words, lib.wwwsynth_uniform_i32):
            f.restype = None
        _lib = lib
    return _lib


# ----------------------------------------------------------------------------- raw draws
def normal_f32(seed: int, stream: int, n: int, std: float = 1.0, mean: float = 0.0, out=None) -> np.ndarray:
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
    _load().wwwsynth_normal_f32(seed, stream, 0, n, mean, std, out.ctypes.data)
    return out


def normal_bf16(seed: int, stream: int, n: int, std: float = 1.0, mean: float = 0.0, out=None) -> np.ndarray:
    """bf16 bit patterns (uint16) of round-to-nearest-even(fp32 draw)."""
    if out is None:
        out = np.empty(n, dtype=np.uint16)
    assert out.dtype == np.uint16 and out.size == n and out.flags.c_contiguous
    _load().wwwsynth_normal_bf16(seed, stream, 0, n, mean, std, out.ctypes.data)
    return out


def words(seed: int, stream: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    _load().wwwsynth_words(seed, stream, 0, n, out.ctypes.data)
    return out


def mix(z: int) -> int:
    return int(_load().wwwsynth_mix(z & 0xFFFFFFFFFFFFFFFF))


def uniform_i32(seed: int, stream: int, n: int, bound: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _load().wwwsynth_uniform_i32(seed, stream, 0, n, bound, out.ctypes.data)
    return out


def uniform01(seed: int, stream: int, n: int) -> np.ndarray:
    """doubles in (0,1) from the top 53 bits of each word."""
    return ((words(seed, stream, n) >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def permutation(seed: int, stream: int, n: int) -> np.ndarray:
    """A permutation of 0..n-1: stable argsort of n stream words."""
    return np.argsort(words(seed, stream, n), kind="stable").astype(np.int64)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------- model shapes
@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab: int
    rms_eps: float = 1e-5
    rope_theta: float = 1e4
    weight_dtype: int = WDTYPE_BF16
    seed: int = 0
    kv_block_size: int = KV_BLOCK
    qk_norm: int = 0   # 1: every query and key head is RMS-normalised (own gains, shared by the heads of a layer) before the rotation

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def wbytes(self) -> int:
        return 4 if self.weight_dtype == WDTYPE_F32 else 2

    def n_params(self) -> int:
        d, F, V = self.d_model, self.ffn_dim, self.vocab
        per_layer = 2 * d + self.qkv_rows * d + d * self.n_q_heads * self.head_dim + 2 * F * d + d * F
        per_layer += 2 * self.head_dim if self.qk_norm else 0
        return 2 * V * d + d + self.n_layers * per_layer


TINY = ModelShape("tiny", 2, 256, 4, 2, 64, 688, 1024, 1e-5, 1e4, WDTYPE_F32, seed=0)
M1B = ModelShape("1b", 16, 2048, 32, 8, 64, 8192, 32000, 1e-5, 1e4, WDTYPE_BF16, seed=1)
M8B = ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, 1e-5, 5e5, WDTYPE_BF16, seed=2)
SHAPES = {s.name: s for s in (TINY, M1B, M8B)}


def blob_layout(shape: ModelShape):
    """Tensor table of the weight blob: list of (name, byte offset, rows, cols, dtype code).

    Every matrix is stored [out_features, in_features] row-major, i.e. the weights that produce
    one output feature are contiguous.  Norm gains are always fp32 (dtype code WDTYPE_F32).
    """
    d, F, V = shape.d_model, shape.ffn_dim, shape.vocab
    entries = []
    off = 0

    def add(name, rows, cols, dt):
        nonlocal off
        entries.append((name, off, rows, cols, dt))
        if dt in INT4_GROUP:
            assert cols % INT4_GROUP[dt] == 0, f"{name}: {cols} columns are not a multiple of the group size"
            nbytes = rows * cols // 2
        else:
            nbytes = rows * cols * {WDTYPE_F32: 4, WDTYPE_BF16: 2, WDTYPE_FP8WO: 1}[dt]
        off += (nbytes + ALIGN - 1) // ALIGN * ALIGN
        if dt == WDTYPE_FP8WO:      # the matrix's scale follows it in a slot of its own
            entries.append((name + ".scale", off, 1, 1, WDTYPE_F32))
            off += ALIGN
        if dt in INT4_GROUP:        # bf16 scales [rows][cols / group] follow the codes
            ng = cols // INT4_GROUP[dt]
            entries.append((name + ".scale", off, rows, ng, WDTYPE_BF16))
            off += (rows * ng * 2 + ALIGN - 1) // ALIGN * ALIGN

    wd = shape.weight_dtype
    add("embed", V, d, WDTYPE_BF16 if wd in (WDTYPE_FP8WO, WDTYPE_INT4WO_128, WDTYPE_INT4WO_32) else wd)
    for l in range(shape.n_layers):
        add(f"l{l}.attn_norm", 1, d, WDTYPE_F32)
        add(f"l{l}.wqkv", shape.qkv_rows, d, wd)
        if shape.qk_norm:
            add(f"l{l}.q_norm", 1, shape.head_dim, WDTYPE_F32)
            add(f"l{l}.k_norm", 1, shape.head_dim, WDTYPE_F32)
        add(f"l{l}.wo", d, shape.n_q_heads * shape.head_dim, wd)
        add(f"l{l}.ffn_norm", 1, d, WDTYPE_F32)
        add(f"l{l}.wgu", 2 * F, d, wd)
        add(f"l{l}.wd", d, F, wd)
    add("final_norm", 1, d, WDTYPE_F32)
    add("lm_head", V, d, wd)
    return entries, off


def make_blob(shape: ModelShape, std: float = 0.02, gain_std: float = 0.0, seed=None) -> np.ndarray:
    """Random-init weight blob (uint8 array).  Matrices ~ N(0, std^2); gains = 1 + N(0, gain_std^2).

    Tensor t of the table is drawn from stream id t of the model's seed.  In the fp8 weight-only format a matrix is
    drawn in fp32, its scale is max|w| / 448 (fp32) and each element is stored as the E4M3 code nearest to w / scale
    (`wwwsynth_encode_e4m3`): the codes and scales ARE the model, both sides read them as given.
    """
    seed = shape.seed if seed is None else seed
    entries, total = blob_layout(shape)
    blob = np.zeros(total, dtype=np.uint8)
    for t, (name, off, rows, cols, dt) in enumerate(entries):
        n = rows * cols
        if name.endswith(".scale"):
            continue                                  # written together with its matrix
        if dt == WDTYPE_FP8WO:
            w = normal_f32(seed, t, n, std=std)
            scale = np.float32(np.abs(w).max() / 448.0)
            codes = blob[off:off + n]
            _load().wwwsynth_encode_e4m3(w.ctypes.data, n, 1.0 / float(scale), codes.ctypes.data)
            soff = entries[t + 1][1]
            blob[soff:soff + 4].view(np.float32)[0] = scale
            del w
            continue
        if dt in INT4_GROUP and not name.endswith(".scale"):
            w = normal_f32(seed, t, n, std=std)
            soff, ng = entries[t + 1][1], cols // INT4_GROUP[dt]
            _load().wwwsynth_encode_int4(w.ctypes.data, rows, cols, INT4_GROUP[dt], blob[off:off + n // 2].ctypes.data,
                                         blob[soff:soff + rows * ng * 2].ctypes.data)
            del w
            continue
        if name.endswith("norm"):
            view = blob[off:off + 4 * n].view(np.float32)
            if gain_std > 0:
                normal_f32(seed, t, n, std=gain_std, mean=1.0, out=view)
            else:
                view[:] = 1.0
        elif dt == WDTYPE_F32:
            normal_f32(seed, t, n, std=std, out=blob[off:off + 4 * n].view(np.float32))
        else:
            normal_bf16(seed, t, n, std=std, out=blob[off:off + 2 * n].view(np.uint16))
    return blob


def blob_tensor(shape: ModelShape, blob: np.ndarray, name: str) -> np.ndarray:
    """fp32 copy of one tensor of the blob, shape [rows, cols] (gains: [cols])."""
    entries, _ = blob_layout(shape)
    for (nm, off, rows, cols, dt) in entries:
        if nm == name:
            n = rows * cols
            if dt == WDTYPE_FP8WO or dt in INT4_GROUP:
                raise ValueError("quantised matrices are not decoded here (the generators hold none of the method's arithmetic)")
            if dt == WDTYPE_F32:
                a = blob[off:off + 4 * n].view(np.float32).copy()
            else:
                a = bf16_bits_to_f32(blob[off:off + 2 * n].view(np.uint16))
            return a.reshape(cols) if nm.endswith("norm") else a.reshape(rows, cols)
    raise KeyError(name)


# ----------------------------------------------------------------------------- workloads
STREAM_TOKENS = 1_000_001
STREAM_LENGTHS = 1_000_002
STREAM_BLOCKS = 1_000_003
STREAM_MISC = 1_000_004


def tokens(seed: int, n: int, vocab: int, stream: int = STREAM_TOKENS) -> np.ndarray:
    return uniform_i32(seed, stream, n, vocab)


def lengths_uniform(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """integers uniform on [lo, hi] inclusive"""
    return (lo + uniform_i32(seed, STREAM_LENGTHS, n, hi - lo + 1)).astype(np.int32)


def lengths_lognormal(seed: int, n: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    z = normal_f32(seed, STREAM_LENGTHS, n).astype(np.float64)
    return np.clip(np.rint(np.exp(math.log(median) + sigma * z)), lo, hi).astype(np.int32)


def lengths_zipf(seed: int, n: int, s: float, lo: int, hi: int) -> np.ndarray:
    """P(len = l) proportional to l^-s for integer l in [lo, hi] (inverse-CDF sampling)."""
    support = np.arange(lo, hi + 1, dtype=np.float64)
    cdf = np.cumsum(support ** (-s))
    cdf /= cdf[-1]
    u = uniform01(seed, STREAM_LENGTHS, n)
    return (lo + np.searchsorted(cdf, u, side="left")).astype(np.int32)


def block_tables(seed: int, capacities, num_blocks: int, max_blocks_per_seq: int, permute: bool = True) -> np.ndarray:
    """int32 [B, max_blocks_per_seq]; row b holds ceil(capacities[b]/16) distinct physical block ids, rest -1.

    permute=True scatters the sequences' blocks over the whole pool by a seeded permutation of all
    block ids; permute=False hands them out in increasing order (identity layout).
    """
    need = [(int(c) + KV_BLOCK - 1) // KV_BLOCK for c in capacities]
    assert sum(need) <= num_blocks, "KV pool too small"
    assert max(need) <= max_blocks_per_seq
    ids = permutation(seed, STREAM_BLOCKS, num_blocks) if permute else np.arange(num_blocks, dtype=np.int64)
    table = np.full((len(need), max_blocks_per_seq), -1, dtype=np.int32)
    at = 0
    for b, nb in enumerate(need):
        table[b, :nb] = ids[at:at + nb]
        at += nb
    return table


@dataclass
class Workload:
    """One synthetic serving job: a model shape, B prompts and a number of greedy decode steps."""
    name: str
    shape: ModelShape
    prompt_lens: np.ndarray
    prompt_tokens: np.ndarray          # packed, sum(prompt_lens)
    decode_steps: int
    extra: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return len(self.prompt_lens)


def workload(name: str) -> Workload:
    """The synthetic configurations ("tiny", "1b", "8b", "duel_1b", "duel_8b"; "1b-fp8wo" / "8b-fp8wo": the same jobs
    with the matrices stored as FP8 codes; "-int4wo128" / "-int4wo32": as 4-bit codes with group-wise scales)."""
    if name.endswith("-qknorm"):     # the same job on a model whose query and key heads are normalised
        import dataclasses
        w = workload(name[:-len("-qknorm")])
        return Workload(name, dataclasses.replace(w.shape, name=w.shape.name + "-qknorm", qk_norm=1), w.prompt_lens,
                        w.prompt_tokens, w.decode_steps)
    for suffix, dt in (("-fp8wo", WDTYPE_FP8WO), ("-int4wo128", WDTYPE_INT4WO_128), ("-int4wo32", WDTYPE_INT4WO_32)):
        if name.endswith(suffix):
            import dataclasses
            w = workload(name[:-len(suffix)])
            return Workload(name, dataclasses.replace(w.shape, name=w.shape.name + suffix, weight_dtype=dt), w.prompt_lens,
                            w.prompt_tokens, w.decode_steps)
    if name == "tiny":
        sh = TINY
        lens = np.full(4, 128, dtype=np.int32)
        steps = 16
    elif name == "1b":
        sh = M1B
        lens = lengths_uniform(sh.seed, 32, 512, 2048)
        steps = 128
    elif name == "8b":
        sh = M8B
        lens = lengths_lognormal(sh.seed, 64, 1024.0, 0.6, 16, 4096)
        steps = 256
    elif name in ("duel_1b", "duel_8b"):
        sh = M1B if name == "duel_1b" else M8B
        lens = np.full(32, 768, dtype=np.int32)
        steps = 256
        toks = tokens(12345, int(lens.sum()), 32000)   # identical prompts for both duelists
        return Workload(name, sh, lens, toks, steps)
    else:
        raise KeyError(name)
    toks = tokens(sh.seed, int(lens.sum()), sh.vocab)
    return Workload(name, sh, lens, toks, steps)
