"""CPU oracle of the weight-only quantised formats (test infrastructure only; nothing outside tests/, smoke() and the
CPU baseline may import it).

The paper's quantisation experiment serves the same model with weight-only quantised weights (Sec. 6.3, "fp8wo");
it gives no format details.  The reading taken (stated in include/www.h): every projection matrix is stored as OCP
FP8 E4M3 codes -- 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits, subnormals at exponent 0, no infinities,
0x7F / 0xFF are NaN -- together with one fp32 scale per matrix; the weight is value(code) * scale; activations,
embedding, norms and all arithmetic stay as in the unquantised model.  The same section names "int4wo-128" and
"int4wo-32"; reading: 4-bit codes c in 0..15, two per byte (even column in the low nibble), with one bf16 scale per run
of 128 (or 32) consecutive weights of a row, stored [rows][cols / group] after the codes; the weight is (c - 8) * scale.
This module decodes such a blob into the plain fp32 blob of the same model, which the model oracle then runs
unchanged."""
from __future__ import annotations

import dataclasses

import numpy as np

ALIGN = 256


def e4m3_value(code: int) -> float:
    """Value of one E4M3 code, from the format definition."""
    sign = -1.0 if code & 0x80 else 1.0
    e, m = (code >> 3) & 0xF, code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return sign * (m / 8.0) * 2.0 ** -6
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


TABLE = np.array([e4m3_value(c) for c in range(256)], dtype=np.float32)   # every finite value is exact in fp32


INT4_GROUP = {3: 128, 4: 32}   # weight_dtype code -> group size


def dequantize_blob(shape, blob):
    """(shape, weight-only quantised blob) -> (the same shape with fp32 weights, its fp32 blob).  Layout of the source:
    embed [V][d] bf16; per layer attn_norm[d] fp32, wqkv codes + scale(s), wo codes + scale(s), ffn_norm[d] fp32, wgu
    codes + scale(s), wd codes + scale(s); final_norm[d] fp32; lm_head codes + scale(s); every tensor and every scale
    array on a 256-byte boundary."""
    d, F, V, L = shape.d_model, shape.ffn_dim, shape.vocab, shape.n_layers
    qkv = (shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim
    qd = shape.n_q_heads * shape.head_dim
    src = np.ascontiguousarray(blob, dtype=np.uint8)
    pad = lambda n: (n + ALIGN - 1) // ALIGN * ALIGN
    out, at = [], 0

    def emit(a):
        raw = np.ascontiguousarray(a, dtype=np.float32).view(np.uint8).reshape(-1)
        out.append(raw)
        if pad(raw.size) != raw.size:
            out.append(np.zeros(pad(raw.size) - raw.size, np.uint8))

    def gains(n):
        nonlocal at
        emit(src[at:at + 4 * n].view(np.float32))
        at += pad(4 * n)

    def matrix_int4(rows, cols, group):
        nonlocal at
        packed = src[at:at + rows * cols // 2].reshape(rows, cols // 2)
        at += pad(rows * cols // 2)
        ng = cols // group
        sc = (src[at:at + rows * ng * 2].view(np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(rows, ng)
        at += pad(rows * ng * 2)
        c = np.empty((rows, cols), np.int32)
        c[:, 0::2] = packed & 0xF
        c[:, 1::2] = packed >> 4
        emit((c - 8).astype(np.float32) * np.repeat(sc, group, axis=1))    # exact: a 4-bit integer times a bf16

    def matrix(rows, cols):
        nonlocal at
        if shape.weight_dtype in INT4_GROUP:
            return matrix_int4(rows, cols, INT4_GROUP[shape.weight_dtype])
        codes = src[at:at + rows * cols]
        at += pad(rows * cols)
        scale = src[at:at + 4].view(np.float32)[0]
        at += ALIGN
        emit(TABLE[codes] * scale)                      # fp32 product, one rounding

    emb = src[at:at + 2 * V * d].view(np.uint16)
    at += pad(2 * V * d)
    emit((emb.astype(np.uint32) << np.uint32(16)).view(np.float32))   # bf16 widened exactly
    for _ in range(L):
        gains(d); matrix(qkv, d)
        if getattr(shape, "qk_norm", 0):                # gains of the query / key head normalisation follow wqkv
            gains(shape.head_dim); gains(shape.head_dim)
        matrix(d, qd); gains(d); matrix(2 * F, d); matrix(d, F)
    gains(d); matrix(V, d)
    assert at == src.size, "blob size does not match the quantised layout"
    return dataclasses.replace(shape, weight_dtype=0), np.concatenate(out)
