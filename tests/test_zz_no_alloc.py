"""matkv_decode_attn_static (decode attention with the library's static device scratch, for
callers that cannot allocate) against matkv_decode_attn, through the C-ABI."""
from __future__ import annotations

import pytest
import torch

from tests.chain import (Case, compare_attention, load_blobs, make_attention_inputs, make_context, pages_of,
                         run_oracle_attention)

pytestmark = pytest.mark.gpu

ABS_BF16 = 1e-2     # max-abs bar for bf16 inputs with fp32 accumulation


def _case(name, batch, n_chunks, chunk_tokens, q_lens, steps, shared=False):
    if shared:       # every instance retrieves the same chunks: the shared decode partition is built
        retrieved = [list(range(n_chunks)) for _ in range(batch)]
    else:
        retrieved = [[b * n_chunks + c for c in range(n_chunks)] for b in range(batch)]
    ids = sorted({c for r in retrieved for c in r})
    return Case(name=name, n_layers=2, Hq=32, Hkv=8, D=128, hidden=4096, dtype="bf16",
                chunk_lens={c: chunk_tokens + 8 * (c % 3) for c in ids}, retrieved=retrieved,
                q_lens=q_lens, steps=steps, rope_base=500000.0, scale=1.0)


def _decode_both(case, device="cuda:0"):
    """Every decode step of every layer through both entry points; returns the two output
    tensors [steps, layers, B, Hq, D] (CPU) and the oracle's decode outputs."""
    inp = make_attention_inputs(case)
    ctx = make_context(case, device)
    try:
        slots, keep = load_blobs(ctx, case, inp["blobs"])
        with torch.cuda.stream(ctx.compute_stream):
            tail = inp["tail"].to(device)
            q_dec = inp["q_dec"].to(device)
            table = ctx.new_table()
            ctx.assemble(pages_of(case, slots), case.q_lens, table)
            o_ws = torch.full_like(q_dec, float("nan"))
            o_st = torch.full_like(q_dec, float("nan"))
            for t in range(case.steps):
                ctx.advance(table, 1)
                for l in range(case.n_layers):
                    ctx.decode_attn(l, q_dec[t, l], table, tail[l, 0], tail[l, 1], o_ws[t, l])
                    ctx.decode_attn_static(l, q_dec[t, l], table, tail[l, 0], tail[l, 1], o_st[t, l])
            ctx.compute_stream.synchronize()
        del keep
        return o_ws.cpu(), o_st.cpu(), inp
    finally:
        ctx.close()


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    # first call: batch 3, the larger input; second call, same process and same device array:
    # batch 1 and a shorter cache, so stale partials and counters of the first would show
    big = _case("noalloc-big", 3, 3, 640, [24, 40, 17], 3)
    small = _case("noalloc-small", 1, 1, 200, [9], 2)
    for case in (big, small):
        print(f"static-scratch decode: case {case.name}", flush=True)
        o_ws, o_st, inp = _decode_both(case)
        assert torch.isfinite(o_st.float()).all()
        diff = (o_ws.float() - o_st.float()).abs().max().item()
        assert diff <= ABS_BF16, f"{case.name}: static-scratch decode differs from matkv_decode_attn by {diff}"
        # and against the oracle, like every other decode path
        _, ref_dec = run_oracle_attention(case, inp)
        compare_attention(case, None, o_st, {}, ref_dec)


def test_static_scratch_decode_over_a_shared_partition():
    case = _case("noalloc-shared", 6, 2, 520, [12, 30, 8, 21, 16, 11], 2, shared=True)
    o_ws, o_st, _ = _decode_both(case)
    diff = (o_ws.float() - o_st.float()).abs().max().item()
    assert diff <= ABS_BF16, f"shared partition: differs by {diff}"


def test_static_scratch_refuses_a_batch_beyond_its_size():
    from paper_2512_22195_amd import binding as mk
    # 64 decode units per instance x 48 instances x 32 heads x 132 floats = 52 MB of partials
    case = Case(name="noalloc-toobig", n_layers=1, Hq=32, Hkv=8, D=128, hidden=4096, dtype="bf16",
                chunk_lens={b: 8192 for b in range(48)}, retrieved=[[b] for b in range(48)],
                q_lens=[8] * 48, steps=1, rope_base=500000.0, decode_units=64)
    ctx = make_context(case)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            slot = torch.zeros(mk.blob_bytes(ctx.cfg, 8192), dtype=torch.uint8, device="cuda:0")
            tail = ctx.new_tail()
            table = ctx.new_table()
            ctx.assemble([[(slot, 8192)] for _ in range(48)], case.q_lens, table)
            q = torch.zeros((48, 32, 128), dtype=torch.bfloat16, device="cuda:0")
            o = torch.empty_like(q)
            with pytest.raises(mk.MatKVError) as ei:
                ctx.decode_attn_static(0, q, table, tail[0, 0], tail[0, 1], o)
            assert ei.value.status == mk.ENOMEM and "static scratch" in str(ei.value)
            ctx.decode_attn(0, q, table, tail[0, 0], tail[0, 1], o)      # the workspace form takes it
            ctx.compute_stream.synchronize()
    finally:
        ctx.close()
