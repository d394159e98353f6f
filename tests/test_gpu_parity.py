"""GPU parity: libmatkv (through the C-ABI) against the fp64 oracle, element by element.

Bars (written in tests/chain.py): attention outputs max-abs <= 1e-5 (fp32 path) or
<= 1e-2 (bf16 inputs, fp32 accumulation), plus a gate relative to the rms of the oracle's
output (1e-4 / 2e-2); stored K/V within half an ulp of the storage type plus fp32
accumulation error of the unrounded fp64 value.
"""
import numpy as np
import pytest
import torch

from tests import chain
from tests.chain import Case

pytestmark = pytest.mark.gpu


def _attention_parity(case, use_graph=False, layers=None, steps=None, instances=None):
    inp = chain.make_attention_inputs(case)
    o_pre, o_dec = chain.run_gpu_attention(case, inp, use_graph=use_graph)
    pre, dec = chain.run_oracle_attention(case, inp, layers=layers, steps=steps, instances=instances)
    return chain.compare_attention(case, o_pre, o_dec, pre, dec)


# ------------------------------------------------------------------ configuration 1: chain --
def test_config1_full_chain_fp32():
    err = chain.run_chain_case(1)
    assert err <= 1e-5


def test_bf16_chain_ragged_chunks():
    case = Case("bf16-chain", n_layers=2, Hq=8, Hkv=2, D=128, hidden=512, dtype="bf16",
                chunk_lens={0: 200, 1: 137, 2: 64}, retrieved=[[0, 1], [2, 0, 1]], q_lens=[9, 21],
                steps=5, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0)
    inp = chain.make_chain_inputs(case)
    gpu = chain.run_gpu_chain(case, inp)
    ref = chain.run_oracle_chain(case, inp)
    for cid in case.chunk_lens:
        for l in range(case.n_layers):
            chain.compare_materialized(case, gpu["blobs"][cid][l, 0], ref["blobs"][cid][l][0], f"chunk {cid} K")
            chain.compare_materialized(case, gpu["blobs"][cid][l, 1], ref["blobs"][cid][l][1], f"chunk {cid} V")
    for (l, b), (Kt, Vt) in ref["tails"].items():
        n = Kt.shape[1]
        chain.compare_materialized(case, gpu["tail"][l, 0, b, :, :n], Kt, "tail K")
        chain.compare_materialized(case, gpu["tail"][l, 1, b, :, :n], Vt, "tail V")
    chain.compare_attention(case, gpu["o_pre"], gpu["o_dec"], ref["pre"], ref["dec"])


def _chain_parity(case, fused=False, use_graph=False):
    inp = chain.make_chain_inputs(case)
    gpu = chain.run_gpu_chain(case, inp, fused=fused, use_graph=use_graph)
    ref = chain.run_oracle_chain(case, inp)
    for cid in case.chunk_lens:
        for l in range(case.n_layers):
            chain.compare_materialized(case, gpu["blobs"][cid][l, 0], ref["blobs"][cid][l][0], f"chunk {cid} K")
            chain.compare_materialized(case, gpu["blobs"][cid][l, 1], ref["blobs"][cid][l][1], f"chunk {cid} V")
    for (l, b), (Kt, Vt) in ref["tails"].items():
        n = Kt.shape[1]
        chain.compare_materialized(case, gpu["tail"][l, 0, b, :, :n], Kt, "tail K")
        chain.compare_materialized(case, gpu["tail"][l, 1, b, :, :n], Vt, "tail V")
    chain.compare_attention(case, gpu["o_pre"], gpu["o_dec"], ref["pre"], ref["dec"])


@pytest.mark.parametrize("batch", [1, 2, 5])
def test_bf16_chain_hidden_4096(batch):
    """Llama-3-8B hidden size: the chunk and question projections run on the matrix-core GEMM
    (token counts that are not tile multiples), the decode-token projection on the GEMV form
    with 1, 2 and 5 rows."""
    retrieved = [[0], [1, 0], [0, 1], [1], [0]][:batch]
    case = Case(f"bf16-chain-4096-{batch}", n_layers=1, Hq=8, Hkv=2, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: 150, 1: 40}, retrieved=retrieved, q_lens=[3, 17, 1, 8, 20][:batch],
                steps=2, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case)


@pytest.mark.parametrize("batch,Hq,use_graph", [(1, 8, False), (2, 8, False), (4, 8, True), (5, 8, False),
                                                (1, 16, False), (6, 16, False)])
def test_fused_decode_step_chain(batch, Hq, use_graph):
    """matkv_decode_step, full chain against the oracle (bf16, head_dim 128, hidden 4096): the
    new token's K/V land in the tail cache and the attention includes them.  Batches 1, 2 and 4
    at group size 4 take the single-launch form (one row per projection task; a partly and a
    fully used group of four rows; once recorded and replayed); batch 5 and group size 8 take
    the two launches it stands for."""
    retrieved = [[0], [1, 0], [0, 1], [1], [0], [1, 1]][:batch]
    case = Case(f"fused-step-{batch}-{Hq}", n_layers=2, Hq=Hq, Hkv=2, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: 150, 1: 40}, retrieved=retrieved, q_lens=[3, 17, 1, 8, 20, 2][:batch],
                steps=3, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case, fused=True, use_graph=use_graph)


def test_fused_decode_step_degenerate_caches():
    """Single-launch decode step on degenerate caches: an instance without pages (its first
    decode token sees only the question and itself), a one-token question, a tail that ends
    exactly at its capacity on the last step, and a three-instance batch (a partly used group
    of four rows per projection task)."""
    case = Case("fused-degenerate", n_layers=1, Hq=8, Hkv=2, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: 70, 1: 9}, retrieved=[[], [0, 1], [1]], q_lens=[1, 5, 3],
                steps=3, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0, max_tail=8)
    assert case.tail_cap == 8 and max(case.q_lens) + case.steps == 8
    _chain_parity(case, fused=True)


def test_decode_step_rejects_bad_arguments():
    from paper_2512_22195_amd import binding as mk
    case = Case("step-args", n_layers=1, Hq=8, Hkv=2, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: 32}, retrieved=[[0]], q_lens=[4], steps=2)
    ctx = chain.make_context(case)
    try:
        slot = ctx.new_slot(32)
        table, tail = ctx.new_table(), ctx.new_tail()
        x = torch.zeros((1, 4096), dtype=torch.bfloat16, device="cuda")
        w = torch.zeros((2 * 128, 4096), dtype=torch.bfloat16, device="cuda")
        q = torch.zeros((1, 8, 128), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(mk.MatKVError) as e:      # table never assembled
            ctx.decode_step(0, x, w, w, q, table, tail[0, 0], tail[0, 1], q)
        assert e.value.status == mk.EINVAL
        host = torch.zeros(mk.blob_bytes(ctx.cfg, 32), dtype=torch.uint8).pin_memory()
        ctx.wait(ctx.load(host, 32, slot))
        ctx.assemble([[(slot, 32)]], [4], table)
        with pytest.raises(mk.MatKVError) as e:      # layer out of range
            ctx.decode_step(3, x, w, w, q, table, tail[0, 0], tail[0, 1], q)
        assert e.value.status == mk.EINVAL
        with pytest.raises(mk.MatKVError) as e:      # misaligned hidden pointer
            ctx.decode_step(0, x.view(-1)[1:], w, w, q, table, tail[0, 0], tail[0, 1], q)
        assert e.value.status == mk.EINVAL
        ctx.advance(table, 1)
        ctx.decode_step(0, x, w, w, q, table, tail[0, 0], tail[0, 1], q)   # still works afterwards
        ctx.compute_stream.synchronize()
        assert torch.isfinite(q.float()).all()
    finally:
        ctx.close()


def test_decode_step_other_shapes_run_two_launches():
    """Same entry point where the single-launch form does not apply (hidden 512; fp32)."""
    case = Case("step-fallback-bf16", n_layers=1, Hq=8, Hkv=2, D=128, hidden=512, dtype="bf16",
                chunk_lens={0: 90}, retrieved=[[0], [0]], q_lens=[4, 2], steps=2, scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case, fused=True)
    case = Case("step-fallback-f32", n_layers=1, Hq=4, Hkv=2, D=64, hidden=256, dtype="f32",
                chunk_lens={0: 70}, retrieved=[[0]], q_lens=[5], steps=2, scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case, fused=True)


@pytest.mark.parametrize("T", [16, 37, 64, 150, 255, 300, 1000, 1100, 2100])
def test_materialize_row_count_forms_bf16(T):
    """The bf16 projection picks its kernel by row count: skinny split-hidden form (16..255 rows;
    one, two and four 16-row blocks, several row tiles, ragged ends), tiled GEMM with two
    workgroups per 128 x 128 tile, each over half of the hidden axis (300, 1000: ragged last
    tiles) and with one (1100, 2100).  Each against the oracle, K with rotary positions starting
    at 1000; run twice, the second time into fresh outputs: the arrival counters of the split
    form must be back at zero."""
    case = Case("bf16-rows", n_layers=1, Hq=16, Hkv=8, D=128, hidden=512, dtype="bf16",
                chunk_lens={0: 8}, retrieved=[[0]], q_lens=[1], steps=0, rope_base=500000.0, scale=1.0 / 4.0)
    from workload import normal, to_f64
    import oracle
    ctx = chain.make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            w = normal(("rows", "w"), (2, 8 * 128, 512), 0.25, torch.bfloat16).cuda()
            x = normal(("rows", "x", T), (T, 512), 0.25, torch.bfloat16).cuda()
            outs = []
            for _ in range(2):
                k = torch.zeros((8, T, 128), dtype=torch.bfloat16, device="cuda")
                v = torch.zeros_like(k)
                ctx.materialize(x, w[0], w[1], T, 1000, k, v, T)
                outs.append((k, v))
            ctx.compute_stream.synchronize()
        K, V = oracle.materialize(to_f64(x), to_f64(w[0]), to_f64(w[1]), 8, 128, 1000.0, 500000.0)
        for r, (k, v) in enumerate(outs):
            chain.compare_materialized(case, k.cpu(), K, f"K, {T} rows, run {r}")
            chain.compare_materialized(case, v.cpu(), V, f"V, {T} rows, run {r}")
    finally:
        ctx.close()


@pytest.mark.parametrize("hidden,T", [(3072, 1), (3072, 3), (3072, 9), (6144, 2), (6144, 5), (3072, 40), (3072, 300), (4096, 7),
                                      (8192, 1), (8192, 2), (8192, 4), (8192, 9),
                                      (4096, 64), (4096, 100), (4096, 448), (8192, 37), (8192, 500), (6144, 70),
                                      (2048, 130), (1024, 20), (1536, 50), (4096, 1000), (8192, 700), (3072, 1300), (192, 300),
                                      (4096, 8), (4096, 13), (2048, 16), (8192, 16), (6144, 12), (8192, 6)])
def test_materialize_hidden_sizes_bf16(hidden, T):
    """Hidden sizes of the paper's models: 3072 (the 3B model; passes of six loads in the GEMV
    form) and a multiple of it, 4096, and 8192 (the 70B model: in the GEMV form two waves share
    a rotary pair, each with half of the hidden axis), at row counts that take the GEMV form,
    the skinny forms and the tiled GEMM.  Multiples of 1024 take the skinny form that stages rows
    through LDS (16-row tiles to 64 rows, 32-row tiles beyond, ragged last tiles; one, two, three,
    four, six and eight rounds per wave); 1536 the one with direct operand loads.  Up to 16 rows
    (from 8 rows on, at hidden 8192 from one) the staged form cut into 256 workgroups of four rotary
    pairs x 4, 8 or 16 token rows."""
    case = Case(f"bf16-hidden-{hidden}", n_layers=1, Hq=6, Hkv=2, D=128, hidden=hidden, dtype="bf16",
                chunk_lens={0: 8}, retrieved=[[0]], q_lens=[1], steps=0, rope_base=500000.0, scale=1.0 / 8.0)
    from workload import normal, to_f64
    import oracle
    ctx = chain.make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            w = normal(("hidden", hidden, "w"), (2, 2 * 128, hidden), 1.0 / 8.0, torch.bfloat16).cuda()
            x = normal(("hidden", hidden, "x", T), (T, hidden), 1.0 / 8.0, torch.bfloat16).cuda()
            k = torch.zeros((2, T, 128), dtype=torch.bfloat16, device="cuda")
            v = torch.zeros_like(k)
            ctx.materialize(x, w[0], w[1], T, 77, k, v, T)
            ctx.compute_stream.synchronize()
        K, V = oracle.materialize(to_f64(x), to_f64(w[0]), to_f64(w[1]), 2, 128, 77.0, 500000.0)
        chain.compare_materialized(case, k.cpu(), K, f"K, hidden {hidden}, {T} rows")
        chain.compare_materialized(case, v.cpu(), V, f"V, hidden {hidden}, {T} rows")
    finally:
        ctx.close()


def test_bf16_chain_batch17_decode_rows_on_matrix_cores():
    """Seventeen instances: the decode-token projection has 17 rows (skinny form, ragged second
    16-row block), the question projection 17 ragged groups of rows."""
    B = 17
    case = Case("bf16-chain-b17", n_layers=1, Hq=8, Hkv=2, D=128, hidden=512, dtype="bf16",
                chunk_lens={0: 33, 1: 20}, retrieved=[[i % 2] for i in range(B)],
                q_lens=[1 + (i % 3) for i in range(B)], steps=2, rope_base=500000.0,
                scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case)


@pytest.mark.parametrize("hidden,q_lens", [(512, [150, 90, 128, 130, 110]), (512, [300, 290, 310, 280]),
                                           (1024, [100, 37, 64, 90]), (1024, [20, 30, 25, 1, 9, 40, 33, 16, 28, 30, 17, 5, 31, 29, 30, 22, 19])])
def test_bf16_chain_long_questions_take_the_tiled_and_staged_projections(hidden, q_lens):
    """Question rows of a whole batch through the tail form of the projection (rows of several
    instances in one launch, each row looked up in the table): 608 rows on 128 x 128 tiles with
    two workgroups per tile, 1180 rows with one, 291 rows on the staged skinny form with 32-row
    tiles; then decode steps of 17 instances, whose 17 new rows take the staged form too."""
    B = len(q_lens)
    case = Case(f"bf16-chain-longq-{hidden}-{B}", n_layers=1, Hq=8, Hkv=2, D=128, hidden=hidden, dtype="bf16",
                chunk_lens={0: 40, 1: 25}, retrieved=[[i % 2] for i in range(B)], q_lens=q_lens, steps=2,
                rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case)


def test_materialize_large_positions_bf16():
    """Question/decode tokens sit at positions ~20 000: rotary angles must stay accurate."""
    case = Case("bf16-farpos", n_layers=1, Hq=4, Hkv=1, D=128, hidden=256, dtype="bf16",
                chunk_lens={0: 8}, retrieved=[[0]], q_lens=[16], steps=2, rope_base=500000.0,
                scale=1.0 / 4.0)
    from workload import normal, to_f64
    import oracle
    ctx = chain.make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            w = normal(("farpos", "w"), (2, 128, 256), 0.25, torch.bfloat16).cuda()
            x = normal(("farpos", "x"), (40, 256), 0.25, torch.bfloat16).cuda()
            k = torch.zeros((1, 40, 128), dtype=torch.bfloat16, device="cuda")
            v = torch.zeros_like(k)
            ctx.materialize(x, w[0], w[1], 40, 20123, k, v, 40)
            ctx.compute_stream.synchronize()
        K, V = oracle.materialize(to_f64(x), to_f64(w[0]), to_f64(w[1]), 1, 128, 20123.0, 500000.0)
        chain.compare_materialized(case, k.cpu(), K, "far K")
        chain.compare_materialized(case, v.cpu(), V, "far V")
    finally:
        ctx.close()


# ------------------------------------------------------------------ attention-only parity ---
@pytest.mark.parametrize("dtype,D,Hq,Hkv", [
    ("f32", 64, 4, 2), ("f32", 128, 2, 2), ("f32", 64, 8, 1),
    ("bf16", 128, 8, 2), ("bf16", 128, 8, 1), ("bf16", 64, 4, 4), ("bf16", 128, 4, 2),
])
def test_attention_shapes(dtype, D, Hq, Hkv):
    """Several tiles and ragged ends: chunk lengths not multiples of anything, a 1-token chunk,
    batch of 3 with shared chunks and different question lengths, a forced number of decode units."""
    case = Case(f"attn-{dtype}-{D}-{Hq}-{Hkv}", n_layers=2, Hq=Hq, Hkv=Hkv, D=D, hidden=64, dtype=dtype,
                chunk_lens={0: 300, 1: 77, 2: 1, 3: 129}, retrieved=[[0, 1], [2], [3, 0, 2]],
                q_lens=[5, 1, 17], steps=3, scale=1.0, q_scale=1.0, decode_units=7)
    _attention_parity(case)


@pytest.mark.parametrize("variant", [404, 408, 802, 804, 9024, 9034, 9028, 9022])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (16, 2)])
def test_decode_kernel_variants(variant, Hq, Hkv):
    """Every decode kernel shape that can be selected (plain-ALU: waves*100 + loads in flight;
    matrix-core: 9000 + 10*blocks in flight + waves) against the oracle, group sizes 4 and 8."""
    case = Case(f"attn-variant-{Hq}-{Hkv}", n_layers=1, Hq=Hq, Hkv=Hkv, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 300, 1: 77, 2: 1, 3: 129}, retrieved=[[0, 1], [2], [3, 0, 2]],
                q_lens=[5, 1, 17], steps=3, scale=1.0, q_scale=1.0, decode_units=3, decode_variant=variant)
    _attention_parity(case)


def test_attention_baseline_distribution_auto_units():
    """The stated value distribution (N(0,1)/sqrt(128): near-uniform softmax) with the
    library's own choice of work units."""
    case = Case("attn-baseline", n_layers=1, Hq=32, Hkv=8, D=128, hidden=64, dtype="bf16",
                chunk_lens={i: 1000 for i in range(3)}, retrieved=[[0, 1, 2]], q_lens=[64], steps=4,
                scale=128 ** -0.5)
    _attention_parity(case)


def test_attention_peaked_and_needle():
    """Q scaled up (peaked softmax) and one planted dominant key."""
    case = Case("attn-peaked", n_layers=1, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 500, 1: 260}, retrieved=[[0, 1], [1, 0]], q_lens=[8, 3], steps=2,
                scale=1.0, q_scale=8.0, decode_units=5)
    _attention_parity(case)
    case = Case("attn-needle", n_layers=1, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 500, 1: 260}, retrieved=[[0, 1], [1, 0]], q_lens=[8, 3], steps=2,
                scale=1.0, q_scale=1.0, decode_units=5, needle=True)
    _attention_parity(case)
    case = Case("attn-needle-f32", n_layers=1, Hq=4, Hkv=2, D=64, hidden=64, dtype="f32",
                chunk_lens={0: 300}, retrieved=[[0]], q_lens=[4], steps=2,
                scale=1.0, q_scale=1.0, decode_units=6, needle=True)
    _attention_parity(case)


def test_prefill_mixed_unit_counts_and_row_tiles():
    """Matrix-core prefill with a batch whose instances are cut differently: a long cache
    (several units, folded by the second launch), a short one (one unit, output written
    directly) and one without pages; question lengths that give one partly filled 128-row tile,
    two tiles, and a single row; chunk lengths that leave ragged 32-token blocks."""
    case = Case("prefill-mixed", n_layers=2, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 1203, 1: 997, 2: 85}, retrieved=[[0, 1, 0], [2], []],
                q_lens=[41, 19, 1], steps=1, scale=0.5)
    _attention_parity(case)


def test_prefill_group8_two_row_tiles():
    """Group of 8 query heads per KV head: 23 question rows make 184 (row, head) rows, i.e. one
    full 128-row tile and one ragged one, over a cache cut into several units."""
    case = Case("prefill-g8", n_layers=1, Hq=16, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 700, 1: 333}, retrieved=[[0, 1]], q_lens=[23], steps=1, scale=0.5)
    _attention_parity(case)


@pytest.mark.parametrize("compressed", [False, True])
def test_prefill_many_small_pages_takes_the_other_kernel(compressed):
    """More pages in one unit than the item list of the row-parallel prefill kernel holds
    (64): the launch falls back to the token-parallel matrix-core kernel (plain and compressed
    pages; every page has its own scales, and blocks never reach across two pages)."""
    lens = {i: 3 + (i % 4) for i in range(90)}
    case = Case("prefill-small-pages", n_layers=1, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens=lens, retrieved=[list(range(90))], q_lens=[9], steps=1, scale=0.5,
                compressed=compressed)
    _attention_parity(case)


@pytest.mark.parametrize("compressed", [False, True])
def test_prefill_mixed_unit_counts_compressed_and_question_of_one_page(compressed):
    """The mixed batch of test_prefill_mixed_unit_counts_and_row_tiles with a fourth instance
    whose question is longer than its one short page, both page formats."""
    case = Case("prefill-mixed-f8", n_layers=2, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 1203, 1: 997, 2: 85, 3: 8}, retrieved=[[0, 1, 0], [2], [], [3]],
                q_lens=[41, 19, 1, 70], steps=2, scale=0.5, compressed=compressed)
    _attention_parity(case)


def test_attention_no_pages_and_full_tail():
    """Degenerate caches: an instance that retrieved nothing (plain causal attention over its
    own tokens) and a tail filled to its capacity."""
    case = Case("attn-nopages", n_layers=1, Hq=4, Hkv=2, D=64, hidden=64, dtype="f32",
                chunk_lens={0: 40}, retrieved=[[], [0]], q_lens=[13, 2], steps=3, scale=1.0,
                max_tail=16)
    assert case.tail_cap == 16 and max(case.q_lens) + case.steps == 16
    _attention_parity(case)


def test_chunk_order_invariance_on_gpu():
    """Permuting the page list leaves the result unchanged up to summation order."""
    base = dict(n_layers=1, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 300, 1: 200, 2: 100}, q_lens=[6], steps=2, scale=1.0, decode_units=6)
    c1 = Case("attn-perm", retrieved=[[0, 1, 2]], **base)
    c2 = Case("attn-perm", retrieved=[[2, 0, 1]], **base)
    inp = chain.make_attention_inputs(c1)
    a_pre, a_dec = chain.run_gpu_attention(c1, inp)
    b_pre, b_dec = chain.run_gpu_attention(c2, inp)
    # two summation orders, each output rounded once to bf16: one ulp (2^-7 relative) apart at
    # most, on top of the noise of the bf16-rounded weights, which differ between the two orders
    # (each run alone is held to 2e-2 rms of the oracle; the two are held to that of each other)
    for a, b in ((a_pre.float(), b_pre.float()), (a_dec.float(), b_dec.float())):
        bound = 2.0 ** -7 * a.abs() + 2e-2 * a.pow(2).mean().sqrt()
        assert ((a - b).abs() <= bound).all()
    pre, dec = chain.run_oracle_attention(c1, inp)
    chain.compare_attention(c1, a_pre, a_dec, pre, dec)
    chain.compare_attention(c1, b_pre, b_dec, pre, dec)


def test_graph_replay_matches_eager():
    """A recorded decode step replayed for every step (tail lengths read on the device) gives
    what the eager calls give, on every replay, with eager work and syncs in between."""
    case = Case("attn-graph", n_layers=3, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 400, 1: 333}, retrieved=[[0, 1], [1]], q_lens=[7, 12], steps=6,
                scale=1.0, decode_units=9)
    inp = chain.make_attention_inputs(case)
    e_pre, e_dec = chain.run_gpu_attention(case, inp, use_graph=False)
    g_pre, g_dec = chain.run_gpu_attention(case, inp, use_graph=True)
    assert torch.equal(e_pre, g_pre)
    for t in range(case.steps):
        assert torch.equal(e_dec[t], g_dec[t]), f"replay {t} differs from the eager step"
    pre, dec = chain.run_oracle_attention(case, inp)
    chain.compare_attention(case, g_pre, g_dec, pre, dec)


# ------------------------------------------------------------------ full-size, sampled ------
def test_config2_full_size_sampled():
    """Llama-3-8B layer shape, 10 chunks x 1000 tokens, all 32 layers resident, the launch
    configuration the benchmark times; the oracle checks layers {0, 16, 31} and decode
    steps {0, 3, 7} of 8 (every head, every row of the question)."""
    case = chain.case_from_config(2)
    case.steps = 8
    inp = chain.make_attention_inputs(case)
    o_pre, o_dec = chain.run_gpu_attention(case, inp)
    pre, dec = chain.run_oracle_attention(case, inp, layers=[0, 16, 31], steps=[0, 3, 7])
    chain.compare_attention(case, o_pre, o_dec, pre, dec)
    # layers the oracle did not sample: finite and of the right size everywhere
    assert torch.isfinite(o_pre.float()).all() and torch.isfinite(o_dec.float()).all()


def test_config2_full_size_fused_step_sampled():
    """The launch configuration bench.py times: Llama-3-8B layer shape, 10 x 1000 cached tokens,
    all 32 layers resident, decode steps through matkv_decode_step recorded once and replayed;
    the new token's K/V are projected from hidden states of size 4096 inside the same launch.
    The oracle checks layers {0, 31} at decode steps {0, 5} (all heads)."""
    from workload import normal
    case = chain.case_from_config(2)
    case.steps = 6
    inp = chain.make_attention_inputs(case)
    proj = dict(w=normal((case.name, "w"), (case.n_layers, 2, case.Hkv * case.D, case.hidden), case.scale, case.tdtype),
                x_dec=normal((case.name, "x_dec"), (case.steps, case.n_layers, case.batch, case.hidden), 1.0, case.tdtype))
    o_pre, o_dec = chain.run_gpu_attention(case, inp, proj=proj)
    pre, dec = chain.run_oracle_attention(case, inp, layers=[0, 31], steps=[0, 5], proj=proj)
    chain.compare_attention(case, o_pre, o_dec, pre, dec)
    assert torch.isfinite(o_dec.float()).all()


def test_config3_batch16_shared_pages_sampled():
    """Config 3 shape: batch 16, five 1000-token chunks each, drawn from a pool of 200 so that
    instances share pages, question lengths uniform in 32..128.  Two layers resident; the oracle
    checks instances {0, 7, 15}: three decode steps (all heads) and four question rows."""
    case = chain.case_from_config(3, n_layers=2)
    case.steps = 6
    assert case.batch == 16 and len({c for r in case.retrieved for c in r}) < 80
    inp = chain.make_attention_inputs(case)
    o_pre, o_dec = chain.run_gpu_attention(case, inp)
    pre, dec = chain.run_oracle_attention(case, inp, layers=[1], steps=[0, 2, 5], instances=[0, 7, 15],
                                          prefill_rows=[0, 9, 31, 127])
    chain.compare_attention(case, o_pre, o_dec, pre, dec)
    assert torch.isfinite(o_pre.float()).all() and torch.isfinite(o_dec.float()).all()


def test_config4_70b_shape_sampled():
    """Config 4 shape: 64 query / 8 KV heads (group 8), 20 chunks x 1000 tokens, batch 4,
    128-token questions.  Two layers resident; the oracle checks instances {0, 3}."""
    case = chain.case_from_config(4, n_layers=2)
    case.steps = 5
    inp = chain.make_attention_inputs(case)
    o_pre, o_dec = chain.run_gpu_attention(case, inp)
    pre, dec = chain.run_oracle_attention(case, inp, layers=[0], steps=[0, 4], instances=[0, 3],
                                          prefill_rows=[0, 64, 127])
    chain.compare_attention(case, o_pre, o_dec, pre, dec)
    assert torch.isfinite(o_pre.float()).all() and torch.isfinite(o_dec.float()).all()


def _full_size_resident(config_id, layers, instances, steps, prefill_rows):
    """A BASELINE configuration at its stated size with EVERY layer resident in HBM, inputs drawn
    on the GPU (the bench's recipe), pushed through the launch configuration bench.py times:
    question projection + prefill attention per layer, then decode steps replayed from one
    recorded graph of matkv_decode_step calls.  The oracle reads back and checks the sampled
    (layer, instance, step / question row) outputs."""
    from workload import normal
    case = chain.case_from_config(config_id)
    case.steps = max(steps) + 1
    c, dev = case, "cuda:0"
    ctx = chain.make_context(case)
    cs = ctx.compute_stream
    try:
        with torch.cuda.stream(cs):
            blobs = {cid: normal((c.name, "blob", cid), (c.n_layers, 2, c.Hkv, n, c.D), c.scale, c.tdtype, dev)
                     for cid, n in c.chunk_lens.items()}
            total_q = sum(c.q_lens)
            w = normal((c.name, "w"), (c.n_layers, 2, c.Hkv * c.D, c.hidden), c.scale, c.tdtype, dev)
            x_q = normal((c.name, "x_q"), (c.n_layers, total_q, c.hidden), c.scale, c.tdtype, dev)
            x_dec = normal((c.name, "x_dec"), (c.steps, c.n_layers, c.batch, c.hidden), c.scale, c.tdtype, dev)
            q_pre = normal((c.name, "q_pre"), (c.n_layers, total_q, c.Hq, c.D), c.scale, c.tdtype, dev)
            q_dec = normal((c.name, "q_dec"), (c.steps, c.n_layers, c.batch, c.Hq, c.D), c.scale, c.tdtype, dev)
            tail = ctx.new_tail()
            table = ctx.new_table()
            ctx.assemble([[(blobs[cid], c.chunk_lens[cid]) for cid in r] for r in c.retrieved], c.q_lens, table)
            o_pre = torch.full_like(q_pre, float("nan"))
            o_dec = torch.full_like(q_dec, float("nan"))
            for l in range(c.n_layers):
                ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
                ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
            x_cur, q_cur, o_cur = torch.empty_like(x_dec[0]), torch.empty_like(q_dec[0]), torch.empty_like(o_dec[0])
            ctx.graph_begin()
            ctx.advance(table, 1)
            for l in range(c.n_layers):
                ctx.decode_step(l, x_cur[l], w[l, 0], w[l, 1], q_cur[l], table, tail[l, 0], tail[l, 1], o_cur[l])
            g = ctx.graph_end()
            for t in range(c.steps):
                x_cur.copy_(x_dec[t]); q_cur.copy_(q_dec[t])
                ctx.graph_launch(g)
                o_dec[t].copy_(o_cur)
            cs.synchronize()
            ctx.graph_destroy(g)
        assert torch.isfinite(o_pre.float()).all() and torch.isfinite(o_dec.float()).all()
        # the oracle's tail rows: the question rows as the GPU projected them are checked against
        # the oracle's own projection first (sampled layers), then both sides attend over the
        # oracle's rounded rows
        import oracle
        from workload import to_f64
        from oracle.matkv_oracle import store_round
        cu = chain.cu_q(c)
        tail_ref = torch.zeros_like(tail)
        for l in layers:
            for b in instances:
                p0 = float(sum(c.chunk_lens[cid] for cid in c.retrieved[b]))
                K, V = oracle.materialize(to_f64(x_q[l, cu[b]:cu[b + 1]]), to_f64(w[l, 0]), to_f64(w[l, 1]), c.Hkv, c.D, p0, c.rope_base)
                lq = c.q_lens[b]
                chain.compare_materialized(c, tail[l, 0, b, :, :lq].cpu(), K, f"question K layer {l} inst {b}")
                chain.compare_materialized(c, tail[l, 1, b, :, :lq].cpu(), V, f"question V layer {l} inst {b}")
                tail_ref[l, 0, b, :, :lq] = torch.from_numpy(store_round(K, c.dtype)).to(tail.dtype)
                tail_ref[l, 1, b, :, :lq] = torch.from_numpy(store_round(V, c.dtype)).to(tail.dtype)
        inp = dict(blobs=blobs, tail=tail_ref, q_pre=q_pre, q_dec=q_dec)
        pre, dec = chain.run_oracle_attention(c, inp, layers=layers, steps=steps, instances=instances,
                                              prefill_rows=prefill_rows, proj=dict(w=w, x_dec=x_dec))
        return chain.compare_attention(c, o_pre.cpu(), o_dec.cpu(), pre, dec)
    finally:
        ctx.close()


def test_config3_full_size_all_layers_resident():
    """Config 3 as stated: batch 16, five 1000-token chunks each out of a pool of 200 (shared
    pages), questions of 32..128 tokens, all 32 layers resident (8.5 GB of chunk KV)."""
    _full_size_resident(3, layers=[0, 15, 31], instances=[0, 9, 15], steps=[0, 3], prefill_rows=[0, 17, 127])


def test_config4_full_size_all_layers_resident():
    """Config 4 as stated: 70B layer shape (64 / 8 heads, hidden 8192), batch 4, twenty 1000-token
    chunks each, 128-token questions, all 80 layers resident (26 GB of chunk KV)."""
    _full_size_resident(4, layers=[0, 41, 79], instances=[0, 3], steps=[0, 2], prefill_rows=[0, 64, 127])


# ------------------------------------------- float outputs: the stated bars, no rounding slack --
@pytest.mark.parametrize("kind", ["attention", "graph", "shared", "compressed", "rows-kernel", "fused-chain", "chunk"])
def test_float_outputs_meet_the_stated_bars(kind):
    """config.out_f32: a bf16 configuration writes its attention outputs as float, so the bars as
    stated - max-abs 1e-2 for bf16 inputs with fp32 accumulation, and the 2e-2-of-rms gate - are
    asserted without the half ulp of a bf16 output: every kernel that writes outputs (row-parallel
    prefill with and without the unit fold, decode with its last-arrival merge, the shared
    partition's merge, compressed pages, the plain-ALU kernel, the fused step, a chunk's own
    attention)."""
    lens = {0: 700, 1: 333, 2: 64, 3: 2100}
    base = dict(n_layers=2, Hq=8, Hkv=2, D=128, hidden=256, dtype="bf16", chunk_lens=lens,
                retrieved=[[0, 1], [2, 0, 1], [3, 0]], q_lens=[37, 150, 5], steps=3, scale=0.5, q_scale=1.0,
                out_f32=True)
    if kind in ("attention", "graph"):
        _attention_parity(Case(f"f32out-{kind}", **base), use_graph=kind == "graph")
    elif kind == "shared":
        case = Case("f32out-shared", **{**base, "retrieved": [[0, 1], [0, 1], [1, 0], [0, 1], [0]], "q_lens": [3, 9, 1, 20, 6]})
        inp = chain.make_attention_inputs(case)
        info = {}
        o_pre, o_dec = chain.run_gpu_attention(case, inp, info=info)
        assert info["shared_units"] > 0
        pre, dec = chain.run_oracle_attention(case, inp)
        chain.compare_attention(case, o_pre, o_dec, pre, dec)
    elif kind == "compressed":
        _attention_parity(Case("f32out-f8", **{**base, "compressed": True}))
    elif kind == "rows-kernel":
        _attention_parity(Case("f32out-rows", **{**base, "decode_variant": 404}))
    elif kind == "fused-chain":
        case = Case("f32out-fused", n_layers=1, Hq=8, Hkv=2, D=128, hidden=4096, dtype="bf16",
                    chunk_lens={0: 300, 1: 77}, retrieved=[[0, 1], [1]], q_lens=[9, 30], steps=3,
                    rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0, out_f32=True)
        _chain_parity(case, fused=True, use_graph=True)
    else:
        case = Case("f32out-chunk", n_layers=2, Hq=8, Hkv=2, D=128, hidden=256, dtype="bf16",
                    chunk_lens={0: 64, 1: 200, 2: 1024}, retrieved=[[0]], q_lens=[1], steps=0,
                    scale=1.0 / 4.0, q_scale=1.0, out_f32=True)
        inp = chain.make_chain_inputs(case)
        q_chunk = chain.make_chunk_queries(case)
        blobs, outs = chain.run_gpu_chunk_prefill(case, inp, q_chunk)
        assert all(o.dtype == torch.float32 for o in outs.values())
        chain.compare_chunk_prefill(case, outs, chain.run_oracle_chunk_prefill(case, inp, q_chunk))


# ------------------------------------------------------------------ boundary behaviour ------
def test_load_is_byte_exact_and_validates():
    from paper_2512_22195_amd import binding as mk
    case = Case("load", n_layers=2, Hq=4, Hkv=2, D=64, hidden=64, dtype="bf16",
                chunk_lens={0: 50}, retrieved=[[0]], q_lens=[1], steps=0)
    ctx = chain.make_context(case)
    try:
        n = mk.blob_bytes(ctx.cfg, 50)
        host = torch.randint(0, 256, (n,), dtype=torch.uint8).pin_memory()
        slot = ctx.new_slot(50)
        t = ctx.load(host, 50, slot)
        ctx.sync(t)
        assert ctx.query(t)
        assert torch.equal(slot.cpu(), host)
        with pytest.raises(mk.MatKVError) as e:      # wrong byte count
            ctx.load(host[:-16], 50, slot)
        assert e.value.status == mk.EINVAL
        with pytest.raises(mk.MatKVError) as e:      # pageable host memory
            ctx.load(torch.zeros(n, dtype=torch.uint8), 50, slot)
        assert e.value.status == mk.EINVAL
        with pytest.raises(mk.MatKVError) as e:      # slot too small
            ctx.load(host, 50, slot[: n // 2])
        assert e.value.status == mk.EINVAL
        # the context still works after rejected calls
        t = ctx.load(host, 50, slot)
        ctx.sync(t)
    finally:
        ctx.close()


def test_chain_through_files(tmp_path):
    """The paper's round trip (Section IV): chunks are materialized on the device, written to a file
    (matkv_store_file), read back into slots (matkv_load_file), and the question and the decode
    steps attend over them; file bytes equal the device blobs, outputs match the oracle."""
    case = Case("chain-files", n_layers=2, Hq=8, Hkv=2, D=128, hidden=512, dtype="bf16",
                chunk_lens={0: 200, 1: 137, 2: 64}, retrieved=[[0, 1], [2, 0, 1]], q_lens=[9, 21],
                steps=3, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0)
    inp = chain.make_chain_inputs(case)
    gpu = chain.run_gpu_chain(case, inp, blob_dir=str(tmp_path))
    ref = chain.run_oracle_chain(case, inp)
    for cid in case.chunk_lens:
        for l in range(case.n_layers):
            chain.compare_materialized(case, gpu["blobs"][cid][l, 0], ref["blobs"][cid][l][0], f"chunk {cid} K")
            chain.compare_materialized(case, gpu["blobs"][cid][l, 1], ref["blobs"][cid][l][1], f"chunk {cid} V")
    chain.compare_attention(case, gpu["o_pre"], gpu["o_dec"], ref["pre"], ref["dec"])


def test_load_file_is_byte_exact(tmp_path):
    """matkv_load_file: blobs read from a file at nonzero offsets by the context's reader threads,
    through the bounce buffers (a blob of several 8 MiB pieces with a ragged last one, and a small
    one), land byte-exact in their slots; the call returns once the request is queued and the
    ticket completes when the last piece's copy does; the loaded pages then serve an attention
    call; a file that ends early makes the ticket fail with MATKV_EIO, and a table over that slot
    is refused; O_DIRECT is used when the filesystem allows it."""
    import os
    from paper_2512_22195_amd import binding as mk
    case = Case("load-file", n_layers=3, Hq=8, Hkv=4, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 3000, 1: 40}, retrieved=[[0, 1]], q_lens=[2], steps=0)
    ctx = chain.make_context(case)
    path = str(tmp_path / "blobs.bin")
    try:
        n0, n1 = mk.blob_bytes(ctx.cfg, 3000), mk.blob_bytes(ctx.cfg, 40)      # 18 432 000 and 245 760 bytes
        assert n0 > 2 * (8 << 20) and n0 % (8 << 20) != 0
        g = torch.Generator().manual_seed(5)
        b0 = torch.randint(0, 256, (n0,), dtype=torch.uint8, generator=g)
        b1 = torch.randint(0, 256, (n1,), dtype=torch.uint8, generator=g)
        off0, off1 = 4096, 4096 + n0 + 8192
        with open(path, "wb") as f:
            f.write(b"\0" * off0); f.write(b0.numpy().tobytes())
            f.write(b"\0" * 8192); f.write(b1.numpy().tobytes())
            f.flush(); os.fsync(f.fileno())
        ran = 0
        for flags in (os.O_RDONLY | getattr(os, "O_DIRECT", 0), os.O_RDONLY):
            try:
                fd = os.open(path, flags)
            except OSError:
                continue                                    # no O_DIRECT on this filesystem
            try:
                s0, s1 = ctx.new_slot(3000), ctx.new_slot(40)
                t0 = ctx.load_file(fd, off0, n0, 3000, s0)
                t1 = ctx.load_file(fd, off1, n1, 40, s1)
                try:
                    ctx.sync(t0)
                except mk.MatKVError as e:
                    if flags & getattr(os, "O_DIRECT", 0) and e.status == mk.EIO:
                        continue                            # direct reads refused by this filesystem
                    raise
                ctx.sync(t1)
                assert ctx.query(t0) and ctx.query(t1)
                assert torch.equal(s0.cpu(), b0) and torch.equal(s1.cpu(), b1)
                ran += 1
                # the file ends inside the blob: the request is accepted, its ticket fails
                t_bad = ctx.load_file(fd, off1 + 4096, n1, 40, s1)
                for fn in (ctx.sync, ctx.wait, ctx.query):
                    with pytest.raises(mk.MatKVError) as e:
                        fn(t_bad)
                    assert e.value.status == mk.EIO
                table = ctx.new_table()
                with pytest.raises(mk.MatKVError) as e:     # a table over a slot whose load failed
                    ctx.assemble([[(s0, 3000), (s1, 40)]], [2], table)
                assert e.value.status == mk.EIO
                with pytest.raises(mk.MatKVError) as e:     # wrong byte count: refused before anything is queued
                    ctx.load_file(fd, off1, n1 - 4096, 40, s1)
                assert e.value.status == mk.EINVAL
                # a good load into the same slot puts it right; pages loaded from the file are ordinary pages
                t1 = ctx.load_file(fd, off1, n1, 40, s1)
                ctx.wait(t0); ctx.wait(t1)                  # wait() blocks the host until the pieces are enqueued
                ctx.assemble([[(s0, 3000), (s1, 40)]], [2], table)
                ctx.sync(t1)
                assert torch.equal(s1.cpu(), b1)
            finally:
                os.close(fd)
        assert ran >= 1
    finally:
        ctx.close()


def test_load_file_returns_before_the_read_is_done(tmp_path):
    """Ten 8 MiB-piece blobs queued back to back: the calls return without reading (far less time
    than the reads take), the first ticket completes before the last, and everything is
    byte-exact at the end."""
    import os, time
    from paper_2512_22195_amd import binding as mk
    case = Case("load-file-async", n_layers=8, Hq=8, Hkv=8, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 2048}, retrieved=[[0]], q_lens=[2], steps=0)
    ctx = chain.make_context(case)
    path = str(tmp_path / "many.bin")
    try:
        n = mk.blob_bytes(ctx.cfg, 2048)                    # 67 MB
        g = torch.Generator().manual_seed(11)
        blobs = [torch.randint(0, 256, (n,), dtype=torch.uint8, generator=g) for _ in range(10)]
        with open(path, "wb") as f:
            for b in blobs:
                f.write(b.numpy().tobytes())
            f.flush(); os.fsync(f.fileno())
        fd = os.open(path, os.O_RDONLY)
        try:
            slots = [ctx.new_slot(2048) for _ in blobs]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            tickets = [ctx.load_file(fd, i * n, n, 2048, s) for i, s in enumerate(slots)]
            t_calls = time.perf_counter() - t0
            ctx.sync(tickets[0])
            last_done_early = ctx.query(tickets[-1])
            ctx.sync(tickets[-1])
            t_all = time.perf_counter() - t0
            assert t_calls < 0.5 * t_all, f"calls took {t_calls:.3f} s of {t_all:.3f} s"
            assert not last_done_early or t_all < 0.05      # 600 MB do not arrive with the first 67
            for s, b in zip(slots, blobs):
                assert torch.equal(s.cpu(), b)
        finally:
            os.close(fd)
    finally:
        ctx.close()


def test_assemble_rejects_bad_arguments():
    from paper_2512_22195_amd import binding as mk
    case = Case("asm", n_layers=1, Hq=4, Hkv=2, D=64, hidden=64, dtype="f32",
                chunk_lens={0: 32}, retrieved=[[0]], q_lens=[4], steps=2)
    ctx = chain.make_context(case)
    try:
        slot = ctx.new_slot(32)
        table = ctx.new_table()
        for pages, q_len in [([[(slot, 0)]], [4]), ([[(slot, 32)]], [0]), ([[(slot, 32)]], [999]),
                             ([[(slot, 32)], [(slot, 32)]], [4, 4])]:
            with pytest.raises(mk.MatKVError) as e:
                ctx.assemble(pages, q_len, table)
            assert e.value.status == mk.EINVAL
        q = torch.zeros((4, 4, 64), device="cuda")
        tail = ctx.new_tail()
        with pytest.raises(mk.MatKVError) as e:      # table never assembled
            ctx.decode_attn(0, q, table, tail[0, 0], tail[0, 1], q)
        assert e.value.status == mk.EINVAL
        ctx.assemble([[(slot, 32)]], [4], table)
        with pytest.raises(mk.MatKVError) as e:      # layer out of range
            ctx.decode_attn(1, q, table, tail[0, 0], tail[0, 1], q)
        assert e.value.status == mk.EINVAL
        ctx.advance(table, 2)
        with pytest.raises(mk.MatKVError) as e:      # tail capacity (8) exceeded
            ctx.advance(table, 8)
        assert e.value.status == mk.EINVAL
    finally:
        ctx.close()


# ------------------------------------------------------------------ load / compute overlap ---
def test_pipelined_instances_two_slot_sets():
    """Stream of instances (BASELINE config 5 in small): instance i+1's blobs are loaded on the
    side stream into the other slot set while instance i runs prefill and decode.  Slots start
    poisoned with NaN and every instance has different data, so attention that ran before its
    load finished, or a load that overwrote a slot still being read, cannot match the oracle."""
    from workload import normal
    n_inst = 5
    case = Case("pipe", n_layers=2, Hq=8, Hkv=2, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 300, 1: 180}, retrieved=[[0, 1]], q_lens=[6], steps=3, scale=1.0, decode_units=4)
    ctx = chain.make_context(case)
    try:
        inputs = []
        for i in range(n_inst):
            c = Case(f"pipe-{i}", **{k: getattr(case, k) for k in
                                     ("n_layers", "Hq", "Hkv", "D", "hidden", "dtype", "chunk_lens", "retrieved",
                                      "q_lens", "steps", "scale", "decode_units")})
            inputs.append((c, chain.make_attention_inputs(c)))
        host = [[inp["blobs"][cid].contiguous().view(torch.uint8).reshape(-1).pin_memory() for cid in (0, 1)]
                for _, inp in inputs]
        sets = [[ctx.new_slot(case.chunk_lens[cid]) for cid in (0, 1)] for _ in range(2)]
        for s in sets:
            for t in s:
                t.view(torch.bfloat16).fill_(float("nan"))
        torch.cuda.synchronize()
        outs = []
        with torch.cuda.stream(ctx.compute_stream):
            table = ctx.new_table()
            tails = [inp["tail"].cuda() for _, inp in inputs]
            qp = [inp["q_pre"].cuda() for _, inp in inputs]
            qd = [inp["q_dec"].cuda() for _, inp in inputs]
            ctx.compute_stream.synchronize()

            def load(i):
                return [ctx.load(host[i][k], case.chunk_lens[k], sets[i % 2][k]) for k in (0, 1)]

            tk = load(0)
            for i in range(n_inst):
                tk_next = load(i + 1) if i + 1 < n_inst else None
                for t in tk:
                    ctx.wait(t)
                ctx.assemble([[(sets[i % 2][k], case.chunk_lens[k]) for k in (0, 1)]], case.q_lens, table)
                o_pre = torch.full_like(qp[i], float("nan"))
                o_dec = torch.full_like(qd[i], float("nan"))
                for l in range(case.n_layers):
                    ctx.prefill_attn(l, qp[i][l], table, tails[i][l, 0], tails[i][l, 1], o_pre[l])
                for t in range(case.steps):
                    ctx.advance(table, 1)
                    for l in range(case.n_layers):
                        ctx.decode_attn(l, qd[i][t, l], table, tails[i][l, 0], tails[i][l, 1], o_dec[t, l])
                outs.append((o_pre, o_dec))
                tk = tk_next
            ctx.compute_stream.synchronize()
        for (c, inp), (o_pre, o_dec) in zip(inputs, outs):
            pre, dec = chain.run_oracle_attention(c, inp)
            chain.compare_attention(c, o_pre.cpu(), o_dec.cpu(), pre, dec)
    finally:
        ctx.close()


def test_assemble_refuses_pages_still_loading():
    """A page whose load has neither finished nor been waited for is refused (ENOTREADY), not
    read; after matkv_wait the same call goes through."""
    from paper_2512_22195_amd import binding as mk
    case = Case("notready", n_layers=32, Hq=32, Hkv=8, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 1000}, retrieved=[[0]], q_lens=[4], steps=0)
    ctx = chain.make_context(case)
    try:
        n = mk.blob_bytes(ctx.cfg, 1000)                       # 131 MB per blob
        host = torch.zeros(n, dtype=torch.uint8).pin_memory()
        slots = [ctx.new_slot(1000) for _ in range(12)]        # 1.5 GB queued on the load stream
        table = ctx.new_table()
        torch.cuda.synchronize()
        tickets = [ctx.load(host, 1000, s) for s in slots]
        with pytest.raises(mk.MatKVError) as e:
            ctx.assemble([[(slots[-1], 1000)]], [4], table)
        assert e.value.status == mk.ENOTREADY
        # the last ticket cannot be complete before the first: copies on one stream finish in order
        first_done, last_done = ctx.query(tickets[0]), ctx.query(tickets[-1])    # never blocks
        assert first_done or not last_done
        ctx.wait(tickets[-1])
        ctx.assemble([[(slots[-1], 1000)]], [4], table)
        ctx.sync(tickets[-1])
        assert ctx.query(tickets[-1])
    finally:
        ctx.close()


def test_attention_refuses_a_table_whose_slot_is_being_reloaded():
    """A load into a slot that a live table points into: attention over that table is refused
    (ENOTREADY) while the copy is neither finished nor waited for - never a silent race - and
    after matkv_wait it reads the new bytes."""
    from paper_2512_22195_amd import binding as mk
    case = Case("reload", n_layers=32, Hq=32, Hkv=8, D=128, hidden=64, dtype="bf16",
                chunk_lens={0: 1000}, retrieved=[[0]], q_lens=[4], steps=1, scale=1.0)
    inp = chain.make_attention_inputs(case)
    inp2 = chain.make_attention_inputs(Case("reload-2", n_layers=32, Hq=32, Hkv=8, D=128, hidden=64, dtype="bf16",
                                            chunk_lens={0: 1000}, retrieved=[[0]], q_lens=[4], steps=1, scale=1.0))
    ctx = chain.make_context(case)
    try:
        host_a = inp["blobs"][0].contiguous().view(torch.uint8).reshape(-1).pin_memory()
        host_b = inp2["blobs"][0].contiguous().view(torch.uint8).reshape(-1).pin_memory()
        slot = ctx.new_slot(1000)
        spare = [ctx.new_slot(1000) for _ in range(10)]       # 1.3 GB queued ahead of the reload
        cs = ctx.compute_stream
        with torch.cuda.stream(cs):
            tail = inp["tail"].to("cuda:0")
            q = inp["q_dec"][0].to("cuda:0")
            o = torch.full_like(q, float("nan"))
            table = ctx.new_table()
            ctx.wait(ctx.load(host_a, 1000, slot))
            ctx.assemble([[(slot, 1000)]], case.q_lens, table)
            ctx.advance(table, 1)
            ctx.decode_attn(0, q[0], table, tail[0, 0], tail[0, 1], o[0])
            q_pre = inp["q_pre"][0].to("cuda:0")
            o_pre = torch.empty_like(q_pre)
            cs.synchronize()
            for s in spare:
                ctx.load(host_a, 1000, s)
            tk = ctx.load(host_b, 1000, slot)                 # the table still points into `slot`
            # nothing between the load and these calls allocates or synchronises: 1.4 GB of copies are queued
            for fn in (lambda: ctx.decode_attn(0, q[0], table, tail[0, 0], tail[0, 1], o[0]),
                       lambda: ctx.prefill_attn(0, q_pre, table, tail[0, 0], tail[0, 1], o_pre)):
                with pytest.raises(mk.MatKVError) as e:
                    fn()
                assert e.value.status == mk.ENOTREADY
            ctx.wait(tk)
            for l in range(case.n_layers):
                ctx.decode_attn(l, q[l], table, tail[l, 0], tail[l, 1], o[l])
            cs.synchronize()
        # the outputs are those of the second blob
        case2 = Case("reload-2", n_layers=32, Hq=32, Hkv=8, D=128, hidden=64, dtype="bf16",
                     chunk_lens={0: 1000}, retrieved=[[0]], q_lens=[4], steps=1, scale=1.0)
        mixed = dict(blobs=inp2["blobs"], tail=inp["tail"], q_pre=inp["q_pre"], q_dec=inp["q_dec"])
        _, dec = chain.run_oracle_attention(case2, mixed, layers=[0, 17, 31])
        chain.compare_attention(case2, None, o.cpu()[None], {}, dec)
    finally:
        ctx.close()


# ------------------------------------------------- a chunk's own prefill attention (store side)
@pytest.mark.parametrize("name,Hq,Hkv,D,dtype,lens,max_tail", [
    ("chunk-g4", 8, 2, 128, "bf16", [1, 37, 64, 200, 1024], None),   # one row; ragged; one block; several tiles
    ("chunk-g1", 2, 2, 128, "bf16", [130], None),
    ("chunk-g2", 4, 2, 128, "bf16", [100, 129], None),
    ("chunk-g8", 8, 1, 128, "bf16", [77, 300], None),
    ("chunk-f32", 4, 2, 64, "f32", [50, 9], 56),                      # row-per-workgroup kernel
    ("chunk-bf16-d64", 4, 1, 64, "bf16", [40], 40),
])
def test_chunk_prefill_attention(name, Hq, Hkv, D, dtype, lens, max_tail):
    """Materialization pass (Section III-B): K/V of a chunk's hidden states, then the chunk's
    causal attention over its own K/V, against the oracle's chain."""
    case = Case(name, n_layers=2, Hq=Hq, Hkv=Hkv, D=D, hidden=256, dtype=dtype,
                chunk_lens=dict(enumerate(lens)), retrieved=[[0]], q_lens=[1], steps=0,
                scale=1.0 / 4.0, q_scale=1.0, max_tail=max_tail)
    inp = chain.make_chain_inputs(case)
    q_chunk = chain.make_chunk_queries(case)
    blobs, outs = chain.run_gpu_chunk_prefill(case, inp, q_chunk)
    ref = chain.run_oracle_chunk_prefill(case, inp, q_chunk)
    worst = chain.compare_chunk_prefill(case, outs, ref)
    print(f"{name}: worst abs err {worst:.3e}")


def test_chunk_attention_table_follows_the_chunk_length_across_graph_replays():
    """The one-instance table behind matkv_chunk_attn is rewritten only when the chunk length
    changes; a recorded chunk attention carries its own write, and a replay must not leave a
    later eager call of another length with the replay's table."""
    case = Case("chunk-graph", n_layers=1, Hq=8, Hkv=2, D=128, hidden=256, dtype="bf16",
                chunk_lens={0: 150, 1: 70}, retrieved=[[0]], q_lens=[1], steps=0, scale=1.0 / 4.0, q_scale=1.0)
    inp = chain.make_chain_inputs(case)
    q_chunk = chain.make_chunk_queries(case)
    ref = chain.run_oracle_chunk_prefill(case, inp, q_chunk)
    ctx = chain.make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            w = inp["w"].cuda()
            blob, q, o = {}, {}, {}
            for cid, n in case.chunk_lens.items():
                blob[cid] = torch.zeros((1, 2, case.Hkv, n, case.D), dtype=case.tdtype, device="cuda")
                q[cid] = q_chunk[cid].cuda()
                ctx.materialize(inp["x_chunk"][cid].cuda()[0], w[0, 0], w[0, 1], n, 0, blob[cid][0, 0], blob[cid][0, 1], n)
                o[cid] = [torch.full_like(q[cid][0], float("nan"), dtype=case.odtype) for _ in range(3)]
            ctx.graph_begin()
            ctx.chunk_attn(0, q[0][0], blob[0], 150, o[0][0])               # recorded: length 150
            g = ctx.graph_end()
            ctx.chunk_attn(0, q[1][0], blob[1], 70, o[1][0])                # eager: length 70
            ctx.graph_launch(g)                                             # the table holds 150 again
            ctx.chunk_attn(0, q[1][0], blob[1], 70, o[1][1])                # must not run with it
            ctx.chunk_attn(0, q[1][0], blob[1], 70, o[1][2])                # same length again: table kept
            ctx.chunk_attn(0, q[0][0], blob[0], 150, o[0][1])
            ctx.compute_stream.synchronize()
            ctx.graph_destroy(g)
        outs0 = {0: torch.stack([o[0][0].cpu()]), 1: torch.stack([o[1][0].cpu()])}
        chain.compare_chunk_prefill(case, outs0, ref)
        for t in (o[1][1], o[1][2]):
            assert torch.equal(t.cpu(), o[1][0].cpu())
        assert torch.equal(o[0][1].cpu(), o[0][0].cpu())
    finally:
        ctx.close()


def test_chunk_attn_arguments_and_workspace_limit():
    from paper_2512_22195_amd import binding as mk
    case = Case("chunk-args", n_layers=1, Hq=4, Hkv=2, D=64, hidden=128, dtype="f32",
                chunk_lens={0: 64}, retrieved=[[0]], q_lens=[1], steps=0, max_tail=16)
    ctx = chain.make_context(case)
    try:
        blob = torch.zeros((1, 2, 2, 64, 64), dtype=torch.float32, device="cuda")
        q = torch.zeros((64, 4, 64), dtype=torch.float32, device="cuda")
        o = torch.full_like(q, 7.0)
        ctx.chunk_attn(0, q, blob, 0, o)                       # no rows: nothing is written
        ctx.compute_stream.synchronize()
        assert (o == 7.0).all()
        with pytest.raises(mk.MatKVError) as e:
            ctx.chunk_attn(1, q, blob, 8, o)
        assert e.value.status == mk.EINVAL
        with pytest.raises(mk.MatKVError) as e:
            ctx.chunk_attn(0, q.view(-1)[1:], blob, 8, o)
        assert e.value.status == mk.EINVAL
        with pytest.raises(mk.MatKVError) as e:                # 64 rows, workspace sized for 16
            ctx.chunk_attn(0, q, blob, 64, o)
        assert e.value.status == mk.ENOMEM
        ctx.chunk_attn(0, q, blob[:, :, :, :16].contiguous(), 16, o)     # zero scores: mean of zero V
        ctx.compute_stream.synchronize()
        assert (o[:16] == 0).all() and (o[16:] == 7.0).all()
    finally:
        ctx.close()


@pytest.mark.parametrize("L,Hq,Hkv,rows", [
    (1000, 32, 8, None),                                       # config 2's chunk, every row
    (4096, 32, 8, [0, 1, 31, 32, 63, 64, 127, 128, 2047, 2048, 4000, 4095]),
    (1000, 64, 8, [0, 15, 16, 17, 500, 999]),                  # config 4's heads (group 8)
])
def test_full_size_chunk_attention(L, Hq, Hkv, rows):
    """A chunk's own attention at the shapes bench.py times (Llama-3-8B / 70B heads, D 128):
    K/V drawn directly into a two-layer blob, layer 1 checked.  rows: the rows the oracle
    computes one by one (None = the whole chunk)."""
    from workload import normal, to_f64
    import oracle
    name = f"chunk-full-{L}-{Hq}"
    case = Case(name, n_layers=2, Hq=Hq, Hkv=Hkv, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: L}, retrieved=[[0]], q_lens=[1], steps=0)
    blob = normal((name, "blob"), (2, 2, Hkv, L, 128), 1.0, torch.bfloat16)
    q = normal((name, "q"), (L, Hq, 128), 1.0, torch.bfloat16)
    ctx = chain.make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            o = torch.full((L, Hq, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
            ctx.chunk_attn(1, q.cuda(), blob.cuda(), L, o)
            ctx.compute_stream.synchronize()
        got = o.cpu()
    finally:
        ctx.close()
    assert torch.isfinite(got.float()).all()
    K, V = to_f64(blob[1, 0]), to_f64(blob[1, 1])
    if rows is None:
        ref = {(0, 0): oracle.chunk_attn(to_f64(q), K, V)}
        outs = {0: got[None]}
    else:
        # row r alone: keys 0..r, the causal limit starting at row r
        ref = {(i, 0): oracle.attn(to_f64(q[r:r + 1]), K[:, :r + 1], V[:, :r + 1], 0, r) for i, r in enumerate(rows)}
        outs = {i: got[None, r:r + 1] for i, r in enumerate(rows)}
    chain.compare_chunk_prefill(case, outs, ref)


# ------------------------------------------------------------------ compressed chunk blobs --
@pytest.mark.parametrize("L", [77, 1000, 1024, 1100])
def test_compress_is_bit_exact(L):
    """matkv_compress against the oracle: every code byte and every scale.  Heads of very
    different magnitudes, one head of zeros, one tiny head on the scale floor, values on exact
    ties of the 8-bit grid, a largest value just above a power-of-two boundary.  Chunks of up to
    1024 tokens take the kernel that keeps a head in registers, longer ones the two-pass kernel."""
    from paper_2512_22195_amd import binding as mk
    from workload import normal, to_f64
    import oracle
    nl, Hkv, D = 2, 4, 128
    case = Case("compress", n_layers=nl, Hq=8, Hkv=Hkv, D=D, hidden=256, dtype="bf16",
                chunk_lens={0: L}, retrieved=[[0]], q_lens=[1], steps=0)
    blob = normal(("compress", "blob"), (nl, 2, Hkv, L, D), 1.0, torch.bfloat16)
    blob[0, 0, 0] *= 1e-3
    blob[0, 1, 1] *= 300.0
    blob[1, 0, 2] = 0
    blob[1, 1, 3] *= 1e-24
    blob[1, 1, 0] = (blob[1, 1, 0].float().clamp(-3.4, 3.4)).to(torch.bfloat16)
    blob[1, 1, 0, 0, 0] = 3.515625                                   # largest value: just above 3.5 = 448 / 128
    blob[1, 1, 0, 1, :8] = torch.tensor([0.0625 * 17 / 16, 0.0625 * 19 / 16, 0.0625 * 21 / 16, -0.0625 * 23 / 16,
                                          2.0 ** -16, 3 * 2.0 ** -16, -5 * 2.0 ** -16, 0.0]).to(torch.bfloat16)   # ties of the grid at scale 2^-6, normal and subnormal
    ctx = chain.make_context(case)
    try:
        got = chain.compress_on_gpu(ctx, case, blob.cuda(), L).cpu()
    finally:
        ctx.close()
    n_codes = nl * 2 * Hkv * L * D
    assert got.numel() == mk.compressed_blob_bytes(ctx.cfg, L) == (n_codes + 15) // 16 * 16 + nl * 2 * Hkv * 4
    codes = got[:n_codes].view(nl, 2, Hkv, L, D).numpy()
    scales = got[(n_codes + 15) // 16 * 16:].view(torch.float32).view(nl, 2, Hkv).numpy()
    for l in range(nl):
        rc, rs = oracle.compress(to_f64(blob[l, 0]), to_f64(blob[l, 1]))
        assert np.array_equal(scales[l].astype(np.float64), rs), f"layer {l} scales {scales[l]} vs {rs}"
        # the sign of a zero is not information: compare the decoded values for equality, codes elsewhere
        same = codes[l] == rc
        zero = (rc & 0x7F) == 0
        assert (same | (zero & ((codes[l] & 0x7F) == 0))).all(), f"layer {l}: {np.argwhere(~same)[:5]}"
    assert scales[1, 0, 2] == 1.0 and (codes[1, 0, 2] & 0x7F == 0).all()       # head of zeros
    assert scales[1, 1, 3] == 2.0 ** -60                                       # floor
    assert scales[1, 1, 0] == 2.0 ** -6


@pytest.mark.parametrize("name,Hq,Hkv,use_graph", [("g4", 8, 2, False), ("g1", 2, 2, False), ("g8", 8, 1, True), ("g2", 4, 2, False)])
def test_attention_over_compressed_pages(name, Hq, Hkv, use_graph):
    """Prefill and decode attention over pages loaded in compressed form against the oracle over
    code * scale: ragged chunks, shared pages, an instance without pages, heads whose scales
    differ by orders of magnitude."""
    case = Case(f"f8-attn-{name}", n_layers=2, Hq=Hq, Hkv=Hkv, D=128, hidden=256, dtype="bf16",
                chunk_lens={0: 200, 1: 137, 2: 64, 3: 1000}, retrieved=[[0, 1], [2, 0, 3], [], [3]],
                q_lens=[9, 40, 3, 1], steps=4, scale=1.0, q_scale=1.0, compressed=True)
    inp = chain.make_attention_inputs(case)
    inp["blobs"][1][:, 1] *= 1.0 / 64.0    # chunk 1: small V
    inp["blobs"][2][:, 0] *= 1.0 / 32.0    # chunk 2: small K
    inp["blobs"][3][:, 0, 0] *= 2.0        # chunk 3: KV head 0 has larger K than the others
    o_pre, o_dec = chain.run_gpu_attention(case, inp, use_graph=use_graph)
    pre, dec = chain.run_oracle_attention(case, inp)
    chain.compare_attention(case, o_pre, o_dec, pre, dec)


@pytest.mark.parametrize("batch,fused,files", [(1, True, False), (3, True, True), (6, False, False)])
def test_chain_with_compressed_blobs(batch, fused, files, tmp_path):
    """materialize -> compress -> (file ->) load -> assemble -> prefill -> decode steps (one launch
    per layer where the fused step covers the batch) against the oracle's chain with the same
    compression of the stored values."""
    retrieved = [[0, 1], [1], [0], [1, 0], [], [0]][:batch]
    case = Case(f"f8-chain-{batch}", n_layers=2, Hq=8, Hkv=2, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: 150, 1: 333}, retrieved=retrieved, q_lens=[5, 17, 1, 8, 3, 33][:batch],
                steps=3, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0, compressed=True)
    inp = chain.make_chain_inputs(case)
    gpu = chain.run_gpu_chain(case, inp, fused=fused, blob_dir=str(tmp_path) if files else None)
    ref = chain.run_oracle_chain(case, inp)
    chain.compare_attention(case, gpu["o_pre"], gpu["o_dec"], ref["pre"], ref["dec"])


def test_compressed_pages_argument_checks():
    from paper_2512_22195_amd import binding as mk
    case = Case("f8-args", n_layers=1, Hq=4, Hkv=2, D=128, hidden=128, dtype="bf16",
                chunk_lens={0: 32}, retrieved=[[0, 0]], q_lens=[4], steps=1)
    ctx = chain.make_context(case)
    try:
        slot, table = ctx.new_slot(32), ctx.new_table()
        with pytest.raises(mk.MatKVError) as e:                       # two formats in one table
            ctx.assemble([[(slot, 32, mk.PAGE_PLAIN), (slot, 32, mk.PAGE_E4M3)]], [4], table)
        assert e.value.status == mk.EUNSUPPORTED
        with pytest.raises(mk.MatKVError) as e:                       # unknown format
            ctx.assemble([[(slot, 32, 7)]], [4], table)
        assert e.value.status == mk.EINVAL
        blob = torch.zeros(mk.blob_bytes(ctx.cfg, 32), dtype=torch.uint8, device="cuda")
        with pytest.raises(mk.MatKVError) as e:                       # output inside the input
            ctx.compress(blob, 32, blob[16:])
        assert e.value.status == mk.EINVAL
        host = torch.zeros(mk.compressed_blob_bytes(ctx.cfg, 32) + 16, dtype=torch.uint8).pin_memory()
        with pytest.raises(mk.MatKVError) as e:                       # neither of the two blob sizes
            ctx.load(host, 32, slot)
        assert e.value.status == mk.EINVAL
        ctx.sync(ctx.load(host[:-16], 32, slot))
    finally:
        ctx.close()
    case64 = Case("f8-args-64", n_layers=1, Hq=4, Hkv=2, D=64, hidden=128, dtype="bf16",
                  chunk_lens={0: 32}, retrieved=[[0]], q_lens=[4], steps=1)
    ctx = chain.make_context(case64)
    try:
        with pytest.raises(mk.MatKVError) as e:                       # head_dim 64 has no matrix-core kernel
            ctx.assemble([[(ctx.new_slot(32), 32, mk.PAGE_E4M3)]], [4], ctx.new_table())
        assert e.value.status == mk.EUNSUPPORTED
    finally:
        ctx.close()


def test_config2_full_size_compressed_sampled():
    """The compressed leg of bench.py: Llama-3-8B layer shape, 10 x 1000 cached tokens held as
    compressed blobs, all 32 layers resident, decode steps through matkv_decode_step recorded
    once and replayed.  The oracle checks layers {0, 31}: four question rows and decode steps
    {0, 5} (all heads) over code * scale."""
    from workload import normal
    case = chain.case_from_config(2)
    case.steps = 6
    case.compressed = True
    inp = chain.make_attention_inputs(case)
    proj = dict(w=normal((case.name, "w"), (case.n_layers, 2, case.Hkv * case.D, case.hidden), case.scale, case.tdtype),
                x_dec=normal((case.name, "x_dec"), (case.steps, case.n_layers, case.batch, case.hidden), 1.0, case.tdtype))
    o_pre, o_dec = chain.run_gpu_attention(case, inp, proj=proj)
    pre, dec = chain.run_oracle_attention(case, inp, layers=[0, 31], steps=[0, 5], prefill_rows=[0, 17, 40, 63], proj=proj)
    chain.compare_attention(case, o_pre, o_dec, pre, dec)
    assert torch.isfinite(o_dec.float()).all() and torch.isfinite(o_pre.float()).all()


# ------------------------------------------------- decode over pages that instances share ---
@pytest.mark.parametrize("name,Hq,Hkv,batch,use_graph,compressed", [
    ("g4", 8, 2, 6, False, False),      # 4 users per tile: the hot page needs two groups
    ("g1", 2, 2, 21, False, False),     # 16 users per tile, 21 users of the hot page
    ("g8", 16, 2, 6, True, False),      # 2 users per tile
    ("g2", 4, 2, 9, False, False),
    ("g4-f8", 8, 2, 6, True, True),     # the same over compressed pages (the tails stay plain)
    ("g1-f8", 2, 2, 21, False, True),
    ("g8-f8", 16, 2, 6, False, True),
    ("g3-f8", 6, 2, 9, False, True),
])
def test_decode_over_shared_pages(name, Hq, Hkv, batch, use_graph, compressed):
    """Requests of one batch that retrieved the same chunks (the paper's access-skew argument,
    Section II-C): the decode attention runs over the shared partition - every distinct page is
    read once per group of users - and every instance still gets exact attention over its own
    cache: one hot chunk used by everybody, chunks used by two or three, private chunks, an
    instance without pages, ragged lengths, different question lengths."""
    lens = {0: 700, 1: 333, 2: 64, 3: 129, 4: 1000, 5: 17}
    pool = [[0, 1], [0], [2, 0, 3], [0, 4], [], [3, 0], [0, 5, 1], [4, 0], [0, 2]]
    retrieved = [pool[i % len(pool)] if i != 4 else [] for i in range(batch)]
    case = Case(f"shared-{name}", n_layers=2, Hq=Hq, Hkv=Hkv, D=128, hidden=256, dtype="bf16",
                chunk_lens=lens, retrieved=retrieved, q_lens=[1 + (5 * i) % 23 for i in range(batch)],
                steps=3, scale=1.0, q_scale=1.0, compressed=compressed)
    inp = chain.make_attention_inputs(case)
    info = {}
    o_pre, o_dec = chain.run_gpu_attention(case, inp, use_graph=use_graph, info=info)
    assert info["shared_units"] > batch, info                 # the shared partition was built and holds page units
    pre, dec = chain.run_oracle_attention(case, inp)
    chain.compare_attention(case, o_pre, o_dec, pre, dec)


def test_shared_partition_is_built_only_where_it_applies():
    from paper_2512_22195_amd import binding as mk
    def units(case, pages_fn):
        ctx = chain.make_context(case)
        try:
            slots = {cid: ctx.new_slot(n) for cid, n in case.chunk_lens.items()}
            table = ctx.new_table()
            ctx.assemble(pages_fn(slots), case.q_lens, table)
            return ctx.table_shared_units(table)
        finally:
            ctx.close()
    base = dict(n_layers=1, Hq=8, Hkv=2, D=128, hidden=256, dtype="bf16", chunk_lens={0: 300, 1: 40},
                retrieved=[[0, 1], [0], [0]], q_lens=[3, 4, 2], steps=1)
    shared = lambda s: [[(s[0], 300), (s[1], 40)], [(s[0], 300)], [(s[0], 300)]]
    assert units(Case("sh-yes", **base), shared) >= 3      # 340 distinct of 940 page tokens; a unit holds at most one of the three tails
    assert units(Case("sh-private", **base), lambda s: [[(s[0], 300)], [(s[1], 40)], []]) == 0  # nothing shared
    assert units(Case("sh-some", **base), lambda s: [[(s[0], 300), (s[1], 40)], [(s[0], 300)], []]) >= 1    # 340 of 640 page tokens distinct
    big = dict(base, chunk_lens={0: 300, 1: 6000})
    assert units(Case("sh-little", **big), lambda s: [[(s[0], 300), (s[1], 6000)], [(s[0], 300)], []]) == 0  # 6300 of 6600: less than a twentieth saved
    assert units(Case("sh-units", **{**base, "decode_units": 2}), shared) == 0                  # explicit partition
    assert units(Case("sh-f32", **{**base, "dtype": "f32", "D": 64}), shared) == 0              # other kernels


def test_graph_refuses_a_table_cut_differently():
    """A recorded decode step bakes in the launch shape of its table: replaying it after the
    table was re-assembled with the same shape works (and reads the new contents), after a
    re-assembly into another partition it is refused."""
    from paper_2512_22195_amd import binding as mk
    case = Case("graph-sig", n_layers=1, Hq=8, Hkv=2, D=128, hidden=256, dtype="bf16",
                chunk_lens={0: 300, 1: 520}, retrieved=[[0], [1]], q_lens=[3, 5], steps=4)
    ctx = chain.make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            s0, s1 = ctx.new_slot(300), ctx.new_slot(520)
            s0.zero_(); s1.zero_()
            table, tail = ctx.new_table(), ctx.new_tail()
            tail.zero_()
            q = torch.zeros((2, 8, 128), dtype=torch.bfloat16, device="cuda")
            o = torch.ones_like(q)
            ctx.assemble([[(s0, 300)], [(s1, 520)]], [3, 5], table)
            ctx.graph_begin()
            ctx.advance(table, 1)
            ctx.decode_attn(0, q, table, tail[0, 0], tail[0, 1], o)
            g = ctx.graph_end()
            ctx.graph_launch(g)
            ctx.assemble([[(s1, 520)], [(s0, 300)]], [2, 4], table)          # same partition, other contents
            ctx.graph_launch(g)
            ctx.compute_stream.synchronize()
            assert (o == 0).all()                                            # zero V: zero output
            ctx.assemble([[(s0, 300)]], [3], table)                          # one instance instead of two
            with pytest.raises(mk.MatKVError) as e:
                ctx.graph_launch(g)
            assert e.value.status == mk.EINVAL
            ctx.assemble([[(s0, 300)], [(s1, 520)]], [3, 5], table)
            ctx.graph_launch(g)
            ctx.compute_stream.synchronize()
            ctx.graph_destroy(g)
    finally:
        ctx.close()


# ------------------------------------------- three query heads per KV head (Llama-3.2-3B) ---
@pytest.mark.parametrize("compressed,fused,hidden", [(False, False, 3072), (True, False, 3072), (False, True, 4096),
                                                     (False, True, 3072), (True, True, 3072)])
def test_group_of_three_chain(compressed, fused, hidden):
    """The 3B model of the paper's model-size experiment has 24 query / 8 KV heads and hidden
    size 3072: full chain at that grouping (6 / 2 heads here), decode steps as two launches or as
    one, a batch in which two instances share a chunk, plain and compressed blobs."""
    case = Case(f"g3-chain-{int(compressed)}{int(fused)}-{hidden}", n_layers=2, Hq=6, Hkv=2, D=128,
                hidden=hidden, dtype="bf16", chunk_lens={0: 150, 1: 333, 2: 40},
                retrieved=[[0, 1], [1, 2], []], q_lens=[5, 47, 2], steps=3, rope_base=500000.0,
                scale=1.0 / 8.0, q_scale=1.0, compressed=compressed)
    _chain_parity(case, fused=fused)


def test_group_of_three_shared_pages_and_chunk_attention():
    case = Case("g3-shared", n_layers=1, Hq=6, Hkv=2, D=128, hidden=256, dtype="bf16",
                chunk_lens={0: 500, 1: 77}, retrieved=[[0, 1], [0], [0], [1, 0], [0], [0], [0]],
                q_lens=[3, 1, 9, 2, 5, 4, 1], steps=2, scale=1.0, q_scale=1.0)
    inp = chain.make_attention_inputs(case)
    info = {}
    o_pre, o_dec = chain.run_gpu_attention(case, inp, info=info)
    assert info["shared_units"] > 0                       # five users per tile: the hot page needs two groups
    pre, dec = chain.run_oracle_attention(case, inp)
    chain.compare_attention(case, o_pre, o_dec, pre, dec)
    ccase = Case("g3-chunk", n_layers=1, Hq=6, Hkv=2, D=128, hidden=256, dtype="bf16",
                 chunk_lens={0: 301}, retrieved=[[0]], q_lens=[1], steps=0, scale=1.0 / 4.0, q_scale=1.0)
    cinp = chain.make_chain_inputs(ccase)
    q_chunk = chain.make_chunk_queries(ccase)
    _, outs = chain.run_gpu_chunk_prefill(ccase, cinp, q_chunk)
    chain.compare_chunk_prefill(ccase, outs, chain.run_oracle_chunk_prefill(ccase, cinp, q_chunk))


def test_group_of_three_fp32():
    case = Case("g3-f32", n_layers=1, Hq=6, Hkv=2, D=64, hidden=128, dtype="f32",
                chunk_lens={0: 90, 1: 33}, retrieved=[[0, 1], [1]], q_lens=[7, 3], steps=2, scale=0.5)
    _attention_parity(case)


@pytest.mark.parametrize("use_graph", [False, True])
def test_decode_step_over_shared_pages(use_graph):
    """matkv_decode_step on a batch whose instances share their chunks: the table carries the
    shared partition, so the step runs as projection + shared decode attention (two launches),
    eagerly and recorded in a graph."""
    case = Case(f"shared-step-{int(use_graph)}", n_layers=2, Hq=8, Hkv=2, D=128, hidden=4096, dtype="bf16",
                chunk_lens={0: 400, 1: 90}, retrieved=[[0, 1], [0], [1, 0], [0]], q_lens=[4, 9, 1, 17],
                steps=3, rope_base=500000.0, scale=1.0 / 8.0, q_scale=1.0)
    _chain_parity(case, fused=True, use_graph=use_graph)


# ------------------------------------------------------------- seeded random small chains ---
@pytest.mark.parametrize("seed", list(range(14)))
def test_random_small_chain(seed):
    """A net under the hand-picked cases: the full chain on a seeded random draw of the shape
    parameters (grouping, head_dim, dtype, hidden size, batch, chunk and question lengths,
    decode steps, page reuse, compressed blobs, fused step, explicit partition)."""
    rng = np.random.default_rng(1000 + seed)
    dtype = "bf16" if rng.random() < 0.75 else "f32"
    D = 128 if (dtype == "bf16" and rng.random() < 0.8) else 64
    G = int(rng.choice([1, 2, 3, 4, 8]))
    Hkv = int(rng.choice([1, 2, 4]))
    hidden = int(rng.choice([64, 256, 512, 3072, 4096])) if dtype == "bf16" else int(rng.choice([64, 192]))
    batch = int(rng.integers(1, 7))
    n_chunks = int(rng.integers(1, 5))
    lens = {c: int(rng.integers(1, 260)) for c in range(n_chunks)}
    retrieved = [sorted(rng.choice(n_chunks, size=int(rng.integers(0, n_chunks + 1)), replace=False).tolist()) for _ in range(batch)]
    q_lens = [int(rng.integers(1, 41)) for _ in range(batch)]
    steps = int(rng.integers(0, 4))
    compressed = bool(dtype == "bf16" and D == 128 and rng.random() < 0.4)
    case = Case(f"rand-{seed}", n_layers=int(rng.integers(1, 3)), Hq=G * Hkv, Hkv=Hkv, D=D, hidden=hidden, dtype=dtype,
                chunk_lens=lens, retrieved=retrieved, q_lens=q_lens, steps=steps, rope_base=float(rng.choice([10000.0, 500000.0])),
                scale=1.0 / np.sqrt(hidden) * 2.0, q_scale=1.0, compressed=compressed,
                decode_units=int(rng.choice([0, 0, 0, 1, 3])), max_tail=None)
    print(case)
    _chain_parity(case, fused=bool(rng.random() < 0.5))


@pytest.mark.parametrize("seed", list(range(20)))
def test_random_larger_chain(seed):
    """The same net over the shapes that take the tiled projection (one and two workgroups per
    tile), the staged skinny and few-rows forms and the shared decode partition: longer chunks
    and questions, larger batches, hidden sizes that are multiples of 512 and of 1024."""
    rng = np.random.default_rng(7000 + seed)
    G = int(rng.choice([1, 4, 8]))
    Hkv = int(rng.choice([2, 8]))
    hidden = int(rng.choice([512, 1024, 2048, 4096]))
    batch = int(rng.integers(1, 21))
    n_chunks = int(rng.integers(1, 4))
    lens = {c: int(rng.integers(200, 1201)) for c in range(n_chunks)}
    retrieved = [sorted(rng.choice(n_chunks, size=int(rng.integers(0, n_chunks + 1)), replace=False).tolist()) for _ in range(batch)]
    q_lens = [int(rng.integers(1, 151)) for _ in range(batch)]
    case = Case(f"rand-large-{seed}", n_layers=1, Hq=G * Hkv, Hkv=Hkv, D=128, hidden=hidden, dtype="bf16",
                chunk_lens=lens, retrieved=retrieved, q_lens=q_lens, steps=int(rng.integers(1, 3)),
                rope_base=500000.0, scale=1.0 / np.sqrt(hidden) * 2.0, q_scale=1.0,
                compressed=bool(rng.random() < 0.3), max_tail=None)
    print(case)
    _chain_parity(case, fused=bool(rng.random() < 0.5))
