"""fp64 CPU oracle for the MatKV hot path: ctypes front end.  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in ``matkv_oracle.c`` (plain double-precision loops).  This
module compiles it with gcc, loads it, and offers numpy-level wrappers plus the
trivial glue the definition needs: concatenating chunk KVs and the tail into one
flat key list (the paper's cache assembly, Section IV "Avoiding Prefill Using KV
in SSD": loaded chunk KVs combined with the query's KVs as the past cache).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module; it imports nothing from the HIP package and the HIP package never
imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "matkv_oracle.c")
_LIB = os.environ.get("MATKV_ORACLE_LIB") or os.path.join(_HERE, "libmatkv_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math: summation order is the source's).
    MATKV_ORACLE_LIB (used only by the mutation test of the pins) names a prebuilt library."""
    if os.environ.get("MATKV_ORACLE_LIB"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        lib.oracle_threads.restype = ctypes.c_int
        lib.oracle_rope.argtypes = [dp, ctypes.c_int, ctypes.c_double, ctypes.c_double]
        lib.oracle_rope.restype = None
        lib.oracle_materialize.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_int, ctypes.c_double, ctypes.c_double, dp, dp]
        lib.oracle_materialize.restype = None
        lib.oracle_attn.argtypes = [dp, dp, dp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    ctypes.c_double, dp, dp, dp]
        lib.oracle_attn.restype = None
        _lib = lib
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def threads() -> int:
    """Number of OpenMP threads the oracle's parallel loops use."""
    return int(_load().oracle_threads())


def rope(x, pos: float, base: float):
    """Rotate one head vector x[D] to position ``pos`` (half-split pairing)."""
    x = _f64(x).copy()
    assert x.ndim == 1 and x.shape[0] % 2 == 0
    _load().oracle_rope(_p(x), x.shape[0], float(pos), float(base))
    return x


def materialize(X, Wk, Wv, n_kv_heads: int, head_dim: int, pos0: float, base: float):
    """K = RoPE(X Wk^T, pos0 + i), V = X Wv^T for one layer.

    X [T, Hd]; Wk, Wv [Hkv*D, Hd].  Returns K, V as [Hkv, T, D] float64.
    A chunk uses pos0 = 0 (Section III-B: every document starts at the first
    input position)."""
    X, Wk, Wv = _f64(X), _f64(Wk), _f64(Wv)
    T, Hd = X.shape
    assert Wk.shape == (n_kv_heads * head_dim, Hd) and Wv.shape == Wk.shape
    K = np.empty((n_kv_heads, T, head_dim), dtype=np.float64)
    V = np.empty_like(K)
    _load().oracle_materialize(_p(X), _p(Wk), _p(Wv), T, Hd, n_kv_heads, head_dim,
                               float(pos0), float(base), _p(K), _p(V))
    return K, V


def attn(Q, K, V, n_ctx: int, row0: int, scale: float | None = None,
         want_lse: bool = False, want_probs: bool = False):
    """Attention of R rows over a flat key list (see ``oracle_attn`` in the C file).

    Q [R, Hq, D]; K, V [Hkv, Nk, D]; first n_ctx keys unmasked, the rest causal
    with row r seeing tail keys j <= row0 + r.  Returns O [R, Hq, D] (and lse
    [R, Hq], probs [R, Hq, Nk] when asked)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    R, Hq, D = Q.shape
    Hkv, Nk, D2 = K.shape
    assert D2 == D and V.shape == K.shape and Hq % Hkv == 0
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    O = np.empty((R, Hq, D), dtype=np.float64)
    lse = np.empty((R, Hq), dtype=np.float64) if want_lse else None
    probs = np.empty((R, Hq, Nk), dtype=np.float64) if want_probs else None
    _load().oracle_attn(_p(Q), _p(K), _p(V), R, Hq, Hkv, D, Nk, int(n_ctx), int(row0),
                        float(scale), _p(O), _p(lse), _p(probs))
    out = [O]
    if want_lse:
        out.append(lse)
    if want_probs:
        out.append(probs)
    return out[0] if len(out) == 1 else tuple(out)


def store_round(a, dtype: str):
    """Storage rounding of materialized K/V (the paper stores the KV tensors as raw
    16-bit values; here bf16): one round-to-nearest-even of the fp64 value to the
    storage type, returned widened to float64.  "f32" rounds to single precision."""
    a = _f64(a)
    if dtype == "f32":
        return a.astype(np.float32).astype(np.float64)
    assert dtype == "bf16"
    # bf16 keeps the sign, the exponent and the top 7 of fp64's 52 mantissa bits: drop the low
    # 45 bits with round-to-nearest-even on the integer pattern (a carry moves into the
    # exponent as it should).  Magnitudes below bf16's normal range (2^-126) do not occur here.
    u = a.view(np.uint64)
    bias = np.uint64((1 << 44) - 1) + ((u >> np.uint64(45)) & np.uint64(1))
    r = (u + bias) & ~np.uint64((1 << 45) - 1)
    return r.view(np.float64)


def assemble(chunks, tail_k, tail_v):
    """Flat key list of one instance and one layer: chunk KVs in the given order,
    then the tail (question tokens, then generated tokens).

    chunks: list of (K, V) each [Hkv, L_c, D]; tail_k/tail_v [Hkv, T_tail, D].
    Returns K, V [Hkv, N + T_tail, D] and n_ctx = N."""
    ks = [_f64(k) for k, _ in chunks] + [_f64(tail_k)]
    vs = [_f64(v) for _, v in chunks] + [_f64(tail_v)]
    K = np.concatenate(ks, axis=1)
    V = np.concatenate(vs, axis=1)
    n_ctx = int(sum(k.shape[1] for k, _ in chunks))
    return K, V, n_ctx


def prefill_attn(Q, chunks, tail_k, tail_v, scale=None):
    """Question sub-prefill (Section V-A "Prefill time"): row i of the Lq-token
    question attends to every chunk token and to question tokens j <= i.
    tail_k/tail_v hold exactly the Lq question tokens."""
    K, V, n_ctx = assemble(chunks, tail_k, tail_v)
    assert np.asarray(Q).shape[0] == np.asarray(tail_k).shape[1]
    return attn(Q, K, V, n_ctx, 0, scale)


def chunk_attn(Q, K, V, scale=None):
    """Self-attention of one chunk during its materialization (Section III-B, steps
    2-3: the chunk runs through the model's prefill alone, from the first input
    position): token i attends to the chunk's own tokens j <= i and to nothing else.
    Q [L, Hq, D]; K, V [Hkv, L, D], all at positions 0..L-1.  Returns O [L, Hq, D]."""
    assert np.asarray(Q).shape[0] == np.asarray(K).shape[1]
    return attn(Q, K, V, 0, 0, scale)


def decode_attn(q, chunks, tail_k, tail_v, scale=None):
    """One decode step: the newest token (last tail row) attends to every chunk
    token and to the whole tail including itself.  q [Hq, D] -> o [Hq, D]."""
    K, V, n_ctx = assemble(chunks, tail_k, tail_v)
    t_tail = np.asarray(tail_k).shape[1]
    o = attn(np.asarray(q)[None], K, V, n_ctx, t_tail - 1, scale)
    return o[0]


# ------------------------------------------------------------------ compressed KV blobs ----
# The paper names KV compression as the lever on storage cost and load time (Section III-C,
# "Discussion"; related work on KV-size reduction) without fixing a scheme.  The scheme here is
# the simplest one a loader can undo for free: 8-bit floating point codes (OCP FP8 E4M3, the
# "fn" variant: no infinities, S.1111.111 is NaN, largest finite value 448) with one
# power-of-two scale per (layer, K or V, KV head).

def e4m3_decode(codes):
    """Value of every E4M3 code, by the format's definition: 1 sign, 4 exponent (bias 7),
    3 mantissa bits; exponent 0 = subnormal m/8 * 2^-6; S.1111.111 = NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c >> 7, -1.0, 1.0)
    e, m = (c >> 3) & 15, c & 7
    val = np.where(e == 0, (m / 8.0) * 2.0 ** -6, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


def e4m3_encode(y):
    """Nearest E4M3 code of every element, ties to the even mantissa, magnitudes beyond 448
    saturate to 448.  Below 2^-6 the codes step by 2^-9 (subnormals)."""
    y = _f64(y)
    a = np.minimum(np.abs(y), 448.0)
    sub = a < 2.0 ** -6
    q_sub = np.rint(a * 2.0 ** 9)                       # 0..8; 8 is the first normal code
    an = np.where(sub, 1.0, a)                          # keep log2 away from 0
    e = np.floor(np.log2(an))
    q = np.rint((an / np.exp2(e) - 1.0) * 8.0)          # numpy rounds halves to even
    e = np.where(q == 8, e + 1, e)
    q = np.where(q == 8, 0, q)
    code = np.where(sub, q_sub, (e + 7) * 8 + q).astype(np.int64)
    code = np.minimum(code, 0x7E)
    return (code | np.where(np.signbit(y), 0x80, 0)).astype(np.uint8)


def kv_scale(amax):
    """Smallest power of two s with amax <= 448 s; 1 when amax is 0; never below 2^-60
    (heads that small keep that scale and lose precision instead)."""
    amax = _f64(amax)
    m, e = np.frexp(np.where(amax > 0, amax, 1.0))      # amax = m 2^e, m in [0.5, 1)
    k = np.maximum(np.where(2.0 * m <= 1.75, e - 1 - 8, e - 1 - 7), -60)
    return np.where(amax > 0, np.exp2(k.astype(np.float64)), 1.0)


def compress(K, V):
    """K, V [Hkv, L, D] (the stored values) -> codes [2, Hkv, L, D] uint8 and power-of-two
    scales [2, Hkv]: code = e4m3(x / scale of its head), scale from the head's largest
    magnitude over all tokens and dims."""
    X = np.stack([_f64(K), _f64(V)])
    scales = kv_scale(np.abs(X).max(axis=(2, 3)))
    return e4m3_encode(X / scales[:, :, None, None]), scales


def decompress(codes, scales):
    """What a reader of a compressed blob sees: value(code) * scale.  Returns K, V."""
    X = e4m3_decode(codes) * _f64(scales)[:, :, None, None]
    return X[0], X[1]
