"""Pins of the fp64 oracle against what the paper and the mathematics fix.

The paper prints no worked numerical example of this path, so the pins are
definitions written a second, structurally different way (explicit masked score
matrix over the flattened prompt), closed forms, invariants that follow from
Section III-B (chunks independent, each starting at position 0, placed before the
query), special cases that reduce to a library routine, and hand-computable
values stored under tests/golden/.
"""
import os

import numpy as np
import pytest

import oracle

RNG = np.random.default_rng(20251222)
HERE = os.path.dirname(os.path.abspath(__file__))


# --------------------------------------------------------------------------- helpers
def brute_attention(Q, K, V, n_ctx, row0, scale):
    """Second definition: full score tensor, additive -inf mask, exp, divide (numpy)."""
    R, Hq, D = Q.shape
    Hkv, Nk, _ = K.shape
    G = Hq // Hkv
    Kq = np.repeat(K, G, axis=0)                      # [Hq, Nk, D]
    Vq = np.repeat(V, G, axis=0)
    S = np.einsum("rhd,hnd->rhn", Q, Kq) * scale
    key = np.arange(Nk)[None, :]
    row = np.arange(R)[:, None]
    allowed = (key < n_ctx) | (key - n_ctx <= row0 + row)
    S = np.where(allowed[:, None, :], S, -np.inf)
    E = np.exp(S - S.max(axis=-1, keepdims=True))
    P = E / E.sum(axis=-1, keepdims=True)
    return np.einsum("rhn,hnd->rhd", P, Vq), P


def rand(*shape, s=1.0):
    return RNG.standard_normal(shape) * s


# --------------------------------------------------------------------------- P1 / P10
@pytest.mark.parametrize("Hq,Hkv,D,n_ctx,tail,R,row0", [
    (4, 2, 8, 5, 3, 3, 0),      # prefill, GQA
    (4, 4, 4, 0, 4, 4, 0),      # no chunks: plain causal MHA
    (6, 2, 16, 11, 6, 1, 5),    # decode row
    (8, 1, 8, 7, 5, 2, 3),      # MQA, rows in the middle of the tail
])
def test_attn_equals_brute_force(Hq, Hkv, D, n_ctx, tail, R, row0):
    Nk = n_ctx + tail
    Q, K, V = rand(R, Hq, D), rand(Hkv, Nk, D), rand(Hkv, Nk, D)
    scale = 0.37
    O, lse, P = oracle.attn(Q, K, V, n_ctx, row0, scale, want_lse=True, want_probs=True)
    Ob, Pb = brute_attention(Q, K, V, n_ctx, row0, scale)
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-12)
    np.testing.assert_allclose(P, Pb, rtol=0, atol=1e-12)


def test_default_scale_is_inv_sqrt_d():
    Q, K, V = rand(2, 2, 16), rand(2, 6, 16), rand(2, 6, 16)
    O = oracle.attn(Q, K, V, 4, 0)
    Ob, _ = brute_attention(Q, K, V, 4, 0, 1.0 / 4.0)
    np.testing.assert_allclose(O, Ob, atol=1e-12)


# --------------------------------------------------------------------------- P2
def test_softmax_rows_sum_to_one_and_convex_hull():
    Q, K, V = rand(5, 4, 8, s=3.0), rand(2, 20, 8, s=3.0), rand(2, 20, 8)
    O, P = oracle.attn(Q, K, V, 15, 0, want_probs=True)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-12)
    assert (P >= 0).all()
    for r in range(5):
        vis = 15 + r + 1
        assert (P[r, :, vis:] == 0).all()
        for h in range(4):
            v = V[h // 2, :vis]
            assert (O[r, h] <= v.max(0) + 1e-12).all() and (O[r, h] >= v.min(0) - 1e-12).all()


# --------------------------------------------------------------------------- golden (hand-computed)
def test_golden_hand_computed_case():
    """tests/golden/attn_2keys.txt: D=2, one head, two keys, scores 0 and ln 3 ->
    probabilities 1/4 and 3/4 (closed form), values (1,0) and (0,1)."""
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "attn_2keys.txt"))
            if l.strip() and not l.startswith("#")]
    vals = {r[0]: np.array([float(x) for x in r[1:]]) for r in rows}
    Q = vals["q"].reshape(1, 1, 2)
    K = np.stack([vals["k0"], vals["k1"]]).reshape(1, 2, 2)
    V = np.stack([vals["v0"], vals["v1"]]).reshape(1, 2, 2)
    O, lse = oracle.attn(Q, K, V, 2, 0, float(vals["scale"][0]), want_lse=True)
    np.testing.assert_allclose(O.ravel(), vals["o"], atol=1e-15)
    np.testing.assert_allclose(lse.ravel(), vals["lse"], atol=1e-15)


def test_golden_rope_quarter_turn():
    """tests/golden/rope_quarter_turn.txt: D=4, base 10000 -> theta = (1, 0.01).
    Position pi/2 turns pair (x0,x2) by 90 degrees and pair (x1,x3) by pi/200."""
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "rope_quarter_turn.txt"))
            if l.strip() and not l.startswith("#")]
    vals = {r[0]: np.array([float(x) for x in r[1:]]) for r in rows}
    y = oracle.rope(vals["x"], float(vals["pos"][0]), float(vals["base"][0]))
    np.testing.assert_allclose(y, vals["y"], atol=1e-15)


# --------------------------------------------------------------------------- P5 rotary closed forms
def test_rope_identity_norm_and_2x2():
    x = rand(64)
    np.testing.assert_array_equal(oracle.rope(x, 0.0, 10000.0), x)
    for pos in (1.0, 17.0, 9999.0):
        y = oracle.rope(x, pos, 10000.0)
        assert abs(np.linalg.norm(y) - np.linalg.norm(x)) < 1e-12
        # each (j, j+D/2) pair keeps its own norm
        np.testing.assert_allclose(y[:32] ** 2 + y[32:] ** 2, x[:32] ** 2 + x[32:] ** 2, atol=1e-12)
    # D = 2: theta_0 = 1, counter-clockwise rotation by pos radians
    p = 0.7
    y = oracle.rope(np.array([1.0, 0.0]), p, 500000.0)
    np.testing.assert_allclose(y, [np.cos(p), np.sin(p)], atol=1e-15)
    y = oracle.rope(np.array([0.0, 1.0]), p, 500000.0)
    np.testing.assert_allclose(y, [-np.sin(p), np.cos(p)], atol=1e-15)


def test_rope_matches_complex_exponential():
    D, base, pos = 32, 10000.0, 123.0
    x = rand(D)
    z = (x[:D // 2] + 1j * x[D // 2:]) * np.exp(1j * pos * base ** (-np.arange(D // 2) / (D / 2)))
    y = oracle.rope(x, pos, base)
    np.testing.assert_allclose(y, np.concatenate([z.real, z.imag]), atol=1e-12)


def test_rope_scores_depend_on_relative_position_only():
    q, k = rand(64), rand(64)
    base = 10000.0
    s0 = oracle.rope(q, 40.0, base) @ oracle.rope(k, 13.0, base)
    s1 = oracle.rope(q, 1040.0, base) @ oracle.rope(k, 1013.0, base)
    assert abs(s0 - s1) < 1e-10
    s2 = oracle.rope(q, 41.0, base) @ oracle.rope(k, 13.0, base)
    assert abs(s0 - s2) > 1e-6          # and it does depend on the difference


# --------------------------------------------------------------------------- materialize
def test_materialize_at_position_zero_is_plain_matmul():
    """Token 0 of a chunk is not rotated: K = X Wk^T there; V = X Wv^T everywhere."""
    T, Hd, Hkv, D = 5, 24, 3, 8
    X, Wk, Wv = rand(T, Hd), rand(Hkv * D, Hd), rand(Hkv * D, Hd)
    K, V = oracle.materialize(X, Wk, Wv, Hkv, D, 0.0, 10000.0)
    Kp = (X @ Wk.T).reshape(T, Hkv, D).transpose(1, 0, 2)
    Vp = (X @ Wv.T).reshape(T, Hkv, D).transpose(1, 0, 2)
    np.testing.assert_allclose(V, Vp, atol=1e-12)
    np.testing.assert_allclose(K[:, 0], Kp[:, 0], atol=1e-12)
    # token i is the plain projection rotated to position pos0 + i
    K7, _ = oracle.materialize(X, Wk, Wv, Hkv, D, 7.0, 10000.0)
    for g in range(Hkv):
        for i in range(T):
            np.testing.assert_allclose(K7[g, i], oracle.rope(Kp[g, i], 7.0 + i, 10000.0), atol=1e-12)
            np.testing.assert_allclose(K[g, i], oracle.rope(Kp[g, i], float(i), 10000.0), atol=1e-12)


def test_materialize_rows_are_independent_of_other_rows():
    """K/V of a token depend on that token's hidden state and position only
    (what lets chunks be precomputed independently of the query)."""
    T, Hd, Hkv, D = 6, 16, 2, 8
    X, Wk, Wv = rand(T, Hd), rand(Hkv * D, Hd), rand(Hkv * D, Hd)
    K, V = oracle.materialize(X, Wk, Wv, Hkv, D, 0.0, 10000.0)
    K2, V2 = oracle.materialize(X[2:4], Wk, Wv, Hkv, D, 2.0, 10000.0)
    np.testing.assert_allclose(K[:, 2:4], K2, atol=1e-13)
    np.testing.assert_allclose(V[:, 2:4], V2, atol=1e-13)


# --------------------------------------------------------------------------- P3
def test_single_chunk_equals_full_causal_computation():
    """One chunk (C=1), first question position = chunk length: the MatKV result on
    the question rows equals ordinary causal attention over [chunk; question] run
    as one sequence at positions 0..L+Lq-1."""
    L, Lq, Hd, Hq, Hkv, D = 9, 4, 32, 4, 2, 8
    base = 10000.0
    Xc, Xq = rand(L, Hd), rand(Lq, Hd)
    Wk, Wv, Wq = rand(Hkv * D, Hd, s=.3), rand(Hkv * D, Hd, s=.3), rand(Hq * D, Hd, s=.3)

    def queries(X, pos0):
        q = (X @ Wq.T).reshape(-1, Hq, D)
        return np.stack([[oracle.rope(q[i, h], pos0 + i, base) for h in range(Hq)]
                         for i in range(q.shape[0])])

    # MatKV: chunk materialized alone at positions 0.., question at L..
    Kc, Vc = oracle.materialize(Xc, Wk, Wv, Hkv, D, 0.0, base)
    Kt, Vt = oracle.materialize(Xq, Wk, Wv, Hkv, D, float(L), base)
    O_mat = oracle.prefill_attn(queries(Xq, L), [(Kc, Vc)], Kt, Vt)

    # direct: one sequence, plain causal attention over everything (n_ctx = 0)
    Xall = np.concatenate([Xc, Xq])
    Ka, Va = oracle.materialize(Xall, Wk, Wv, Hkv, D, 0.0, base)
    O_full = oracle.attn(queries(Xall, 0), Ka, Va, 0, 0)
    np.testing.assert_allclose(O_mat, O_full[L:], atol=1e-12)
    # against the numpy brute force as well (flattened causal mask)
    Ob, _ = brute_attention(queries(Xall, 0), Ka, Va, 0, 0, 1 / np.sqrt(D))
    np.testing.assert_allclose(O_mat, Ob[L:], atol=1e-12)


def test_chunk_attn_is_library_causal_attention():
    """A chunk's own prefill attention is ordinary causal attention: equal to the
    library routine (torch CPU, fp64, KV heads repeated for the groups), its first
    row is V[0], and a chunk's prefix gives the same rows as the whole chunk."""
    import torch
    import torch.nn.functional as F
    L, Hq, Hkv, D = 13, 6, 2, 16
    Q, K, V = rand(L, Hq, D), rand(Hkv, L, D), rand(Hkv, L, D)
    scale = 0.21
    O = oracle.chunk_attn(Q, K, V, scale)
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]                       # [1, Hq, L, D]
    k = torch.from_numpy(K).repeat_interleave(Hq // Hkv, dim=0)[None]
    v = torch.from_numpy(V).repeat_interleave(Hq // Hkv, dim=0)[None]
    ref = F.scaled_dot_product_attention(q, k, v, is_causal=True, scale=scale)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
    for h in range(Hq):
        np.testing.assert_allclose(O[0, h], V[h // (Hq // Hkv), 0], atol=1e-14)
    O7 = oracle.chunk_attn(Q[:7], K[:, :7], V[:, :7], scale)
    np.testing.assert_allclose(O7, O[:7], rtol=0, atol=1e-13)


def test_two_chunks_differ_from_concatenated_prefill():
    """With two chunks the MatKV cache is NOT the vanilla one: the second chunk
    restarts at position 0 (Section III-B), so keys differ from the concatenation."""
    L, Hd, Hkv, D = 5, 16, 1, 8
    X1, X2 = rand(L, Hd), rand(L, Hd)
    Wk, Wv = rand(Hkv * D, Hd), rand(Hkv * D, Hd)
    K2, _ = oracle.materialize(X2, Wk, Wv, Hkv, D, 0.0, 10000.0)
    Kcat, _ = oracle.materialize(np.concatenate([X1, X2]), Wk, Wv, Hkv, D, 0.0, 10000.0)
    assert np.abs(K2[:, 1:] - Kcat[:, L + 1:]).max() > 1e-3
    np.testing.assert_allclose(K2[:, 0], oracle.materialize(X2[:1], Wk, Wv, Hkv, D, 0.0, 10000.0)[0][:, 0])


# --------------------------------------------------------------------------- P4
def test_chunk_order_invariance():
    Hq, Hkv, D, Lq = 4, 2, 8, 3
    chunks = [(rand(Hkv, n, D), rand(Hkv, n, D)) for n in (5, 7, 3)]
    Kt, Vt, Q = rand(Hkv, Lq, D), rand(Hkv, Lq, D), rand(Lq, Hq, D)
    O0 = oracle.prefill_attn(Q, chunks, Kt, Vt)
    O1 = oracle.prefill_attn(Q, [chunks[2], chunks[0], chunks[1]], Kt, Vt)
    np.testing.assert_allclose(O0, O1, atol=1e-12)
    o0 = oracle.decode_attn(Q[0], chunks, Kt, Vt)
    o1 = oracle.decode_attn(Q[0], chunks[::-1], Kt, Vt)
    np.testing.assert_allclose(o0, o1, atol=1e-12)


# --------------------------------------------------------------------------- P6
def test_degenerate_attention_cases():
    Hq, Hkv, D, N, T = 2, 1, 4, 6, 2
    Q = rand(T, Hq, D)
    V = rand(Hkv, N + T, D)
    # all keys zero -> arithmetic mean of the visible values
    O = oracle.attn(Q, np.zeros((Hkv, N + T, D)), V, N, 0)
    for r in range(T):
        np.testing.assert_allclose(O[r, 0], V[0, :N + r + 1].mean(0), atol=1e-12)
    # all value rows equal -> that row
    v0 = rand(D)
    O = oracle.attn(Q, rand(Hkv, N + T, D), np.broadcast_to(v0, (Hkv, N + T, D)).copy(), N, 0)
    np.testing.assert_allclose(O, np.broadcast_to(v0, O.shape), atol=1e-12)
    # one key far above the rest -> its value row
    K = rand(Hkv, N + T, D, s=0.01)
    q = np.zeros((1, Hq, D)); q[:, :, 0] = 1.0
    K[0, 3, 0] = 200.0
    O = oracle.attn(q, K, V, N, T - 1, 1.0)
    np.testing.assert_allclose(O[0, 0], V[0, 3], atol=1e-10)
    # a masked key never contributes, however large its score
    K[0, N + 1, 0] = 1e6
    O2 = oracle.attn(q, K, V, N, 0, 1.0)
    np.testing.assert_allclose(O2[0, 0], V[0, 3], atol=1e-10)


# --------------------------------------------------------------------------- P7
def test_gqa_equals_mha_on_replicated_heads():
    Hq, Hkv, D, N, T = 6, 2, 8, 7, 3
    Q, K, V = rand(T, Hq, D), rand(Hkv, N + T, D), rand(Hkv, N + T, D)
    O = oracle.attn(Q, K, V, N, 0)
    O_mha = oracle.attn(Q, np.repeat(K, 3, axis=0), np.repeat(V, 3, axis=0), N, 0)
    np.testing.assert_allclose(O, O_mha, atol=1e-13)
    # contiguous groups: heads 0..2 read KV head 0 -> changing KV head 1 leaves them alone
    K2 = K.copy(); K2[1] += rand(N + T, D)
    O2 = oracle.attn(Q, K2, V, N, 0)
    np.testing.assert_allclose(O2[:, :3], O[:, :3], atol=1e-13)
    assert np.abs(O2[:, 3:] - O[:, 3:]).max() > 1e-3


# --------------------------------------------------------------------------- P8
def test_split_merge_by_log_sum_exp():
    """Attention over a union of key segments equals the LSE-weighted mix of the
    per-segment results (what a split-KV kernel and a paged cache rely on)."""
    Hq, Hkv, D = 4, 2, 8
    segs = [(rand(Hkv, n, D), rand(Hkv, n, D)) for n in (6, 1, 9)]
    q = rand(1, Hq, D)
    Kall = np.concatenate([k for k, _ in segs], axis=1)
    Vall = np.concatenate([v for _, v in segs], axis=1)
    O = oracle.attn(q, Kall, Vall, Kall.shape[1], 0)
    parts = [oracle.attn(q, k, v, k.shape[1], 0, want_lse=True) for k, v in segs]
    lses = np.stack([p[1] for p in parts])                    # [S, 1, Hq]
    w = np.exp(lses - lses.max(0))
    w = w / w.sum(0)
    merged = sum(w[i][..., None] * parts[i][0] for i in range(len(segs)))
    np.testing.assert_allclose(O, merged, atol=1e-12)


# --------------------------------------------------------------------------- P9
def test_decode_row_equals_prefill_row():
    Hq, Hkv, D, Lq, steps = 4, 2, 8, 3, 4
    chunks = [(rand(Hkv, 6, D), rand(Hkv, 6, D)), (rand(Hkv, 4, D), rand(Hkv, 4, D))]
    T = Lq + steps
    Kt, Vt, Q = rand(Hkv, T, D), rand(Hkv, T, D), rand(T, Hq, D)
    O_long = oracle.prefill_attn(Q, chunks, Kt, Vt)           # all T rows as one prefill
    for t in range(steps):
        n = Lq + t + 1
        o = oracle.decode_attn(Q[n - 1], chunks, Kt[:, :n], Vt[:, :n])
        np.testing.assert_allclose(o, O_long[n - 1], atol=1e-12)


def test_oracle_reports_threads():
    assert oracle.threads() >= 1


# --------------------------------------------------------------------------- storage rounding
def test_store_round_bf16_is_round_to_nearest_even():
    from oracle.matkv_oracle import store_round
    # representable values stay; exact ties go to the even neighbour; sign symmetric
    x = np.array([1.0, 1.0 + 2 ** -7, -3.5, 0.0, 2.0 ** -20])
    np.testing.assert_array_equal(store_round(x, "bf16"), x)
    ties = np.array([1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -(1.0 + 2 ** -8), 2.0 - 2 ** -8])
    np.testing.assert_array_equal(store_round(ties, "bf16"), [1.0, 1.0 + 2 ** -6, -1.0, 2.0])
    # just above a tie goes up even though a first rounding to fp32 would land on the tie
    np.testing.assert_array_equal(store_round(np.array([1.0 + 2 ** -8 + 2 ** -40]), "bf16"), [1.0 + 2 ** -7])
    a = RNG.standard_normal(10000) * 3
    r = store_round(a, "bf16")
    assert (np.abs(r - a) <= 2.0 ** -8 * np.abs(a)).all()    # half an ulp: unit roundoff 2^-8
    assert ((r.view(np.uint64) & np.uint64((1 << 45) - 1)) == 0).all()           # 7 mantissa bits
    np.testing.assert_array_equal(store_round(a, "f32"), a.astype(np.float32).astype(np.float64))


# --------------------------------------------------------------------------- compressed blobs
def test_e4m3_matches_library_cast_and_closed_forms():
    """The 8-bit code of the compressed blobs against the library's cast (torch CPU,
    float8_e4m3fn) on every code, on a dense grid with all midpoints, and on random values;
    plus the values the format fixes."""
    import torch
    codes = np.arange(256, dtype=np.uint8)
    lib_vals = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = oracle.e4m3_decode(codes)
    assert np.array_equal(np.isnan(mine), np.isnan(lib_vals)) and np.isnan(mine).sum() == 2
    ok = ~np.isnan(mine)
    assert np.array_equal(mine[ok], lib_vals[ok])
    # the format's fixed points
    assert oracle.e4m3_decode([0x7E])[0] == 448.0 and oracle.e4m3_decode([0x01])[0] == 2.0 ** -9
    assert oracle.e4m3_decode([0x38])[0] == 1.0 and oracle.e4m3_decode([0x08])[0] == 2.0 ** -6
    assert np.array_equal(oracle.e4m3_encode(mine[ok]), codes[ok])          # every value is its own nearest
    # ties go to the even mantissa; beyond the largest value the code saturates
    assert oracle.e4m3_encode([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 1e4, -1e4]).tolist() == \
        [0x38, 0x3A, 0x00, 0x02, 0x7E, 0xFE]
    # every representable value, every midpoint between neighbours, and a step either side
    pos = np.sort(mine[ok & (codes < 0x80)])
    mids = (pos[1:] + pos[:-1]) / 2
    grid = np.concatenate([pos, mids, mids * (1 + 2.0 ** -20), mids * (1 - 2.0 ** -20), RNG.uniform(0, 448, 4000)])
    grid = np.concatenate([grid, -grid]).astype(np.float32)                 # all exactly fp32
    lib = torch.from_numpy(grid).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = oracle.e4m3_encode(grid)
    zero = grid == 0                                                         # the sign of zero is the input's
    assert np.array_equal(got[~zero], lib[~zero])
    # rounding error: half a step, i.e. 2^-4 relative for normals, 2^-10 absolute below 2^-6
    back = oracle.e4m3_decode(got)
    assert (np.abs(back - grid) <= np.maximum(2.0 ** -4 * np.abs(grid), 2.0 ** -10) * (1 + 1e-12)).all()


def test_kv_scale_and_compress_roundtrip():
    """Scale rule: the smallest power of two that brings the head's largest magnitude to at
    most 448 (so it lands in (224, 448]); exact powers of two and the 1.75 boundary; a blob of
    representable values survives compress -> decompress unchanged."""
    amax = np.array([0.0, 448.0, 448.0001, 224.0, 224.0001, 1.0, 3.5, 3.50001, 1e-3, 7e4])
    s = oracle.kv_scale(amax)
    assert s[0] == 1.0
    nz = amax > 0
    assert (np.log2(s[nz]) == np.round(np.log2(s[nz]))).all()
    r = amax[nz] / s[nz]
    assert (r <= 448.0).all() and (r > 224.0).all()
    assert s[1] == 1.0 and s[2] == 2.0 and s[3] == 0.5 and s[4] == 1.0 and s[6] == 2.0 ** -7 and s[7] == 2.0 ** -6
    assert oracle.kv_scale([1e-30])[0] == 2.0 ** -60 and oracle.kv_scale([448 * 2.0 ** -60])[0] == 2.0 ** -60
    Hkv, L, D = 3, 11, 8
    K, V = rand(Hkv, L, D, s=5.0), rand(Hkv, L, D, s=0.01)
    codes, scales = oracle.compress(K, V)
    assert codes.shape == (2, Hkv, L, D) and codes.dtype == np.uint8 and scales.shape == (2, Hkv)
    Kd, Vd = oracle.decompress(codes, scales)
    for X, Xd, sc in ((K, Kd, scales[0]), (V, Vd, scales[1])):
        amax_h = np.abs(X).max(axis=(1, 2))
        assert (amax_h / sc <= 448).all() and (amax_h / sc > 224).all()
        # half a step of the head's grid: 2^-4 relative, or half a subnormal step of the scaled grid
        assert (np.abs(Xd - X) <= np.maximum(2.0 ** -4 * np.abs(X), 2.0 ** -10 * sc[:, None, None]) * (1 + 1e-12)).all()
    Kd2, Vd2 = oracle.decompress(*oracle.compress(Kd, Vd))                   # already on a grid: kept exactly
    assert np.array_equal(Kd2, Kd) and np.array_equal(Vd2, Vd)              # (the scale may halve, the values stay)
    # a head of zeros keeps scale 1 and code 0
    c0, s0 = oracle.compress(np.zeros((1, 2, 4)), np.zeros((1, 2, 4)))
    assert (c0 == 0).all() and (s0 == 1.0).all()
