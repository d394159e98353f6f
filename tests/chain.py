"""Shared machinery of the GPU parity tests and of the smoke check.

``Case`` describes one synthetic RAG batch; ``make_inputs`` draws its tensors from the seeded
generator; ``run_gpu_*`` push them through libmatkv (C-ABI via the ctypes binding) and
``run_oracle_*`` through the fp64 oracle.  The two sides meet only in the comparisons.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

import oracle
from oracle.matkv_oracle import store_round
from workload import CONFIGS, normal, to_f64


@dataclass
class Case:
    name: str
    n_layers: int
    Hq: int
    Hkv: int
    D: int
    hidden: int
    dtype: str                       # "f32" | "bf16"
    chunk_lens: dict                 # chunk id -> tokens
    retrieved: list                  # per instance: list of chunk ids
    q_lens: list
    steps: int
    rope_base: float = 10000.0
    scale: float = 1.0               # std of the generated values
    q_scale: float | None = None     # std of Q (defaults to scale)
    decode_units: int = 0
    decode_variant: int = 0
    max_tail: int | None = None
    needle: bool = False             # plant one key that dominates the softmax
    compressed: bool = False         # chunk blobs go through matkv_compress before they are loaded
    out_f32: bool = False            # bf16 configuration whose attention outputs leave as float (config.out_f32)

    @property
    def batch(self):
        return len(self.retrieved)

    @property
    def tdtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def odtype(self):
        """Element type of the attention outputs."""
        return torch.float32 if (self.out_f32 or self.dtype == "f32") else torch.bfloat16

    @property
    def tail_cap(self):
        need = max(self.q_lens) + self.steps
        cap = self.max_tail if self.max_tail is not None else need
        return (max(cap, need) + 7) // 8 * 8

    @property
    def max_pages(self):
        return max(1, max(len(r) for r in self.retrieved))


def case_from_config(config_id: int, n_layers: int | None = None) -> Case:
    s = CONFIGS[config_id]
    from workload import question_lengths, retrieved_chunks
    retrieved = retrieved_chunks(s)
    ids = sorted({c for r in retrieved for c in r})
    return Case(name=s.name, n_layers=n_layers or s.n_layers, Hq=s.n_q_heads, Hkv=s.n_kv_heads,
                D=s.head_dim, hidden=s.hidden, dtype=s.dtype,
                chunk_lens={c: s.chunk_tokens for c in ids}, retrieved=retrieved,
                q_lens=question_lengths(s), steps=s.decode_steps, rope_base=s.rope_base,
                scale=s.value_scale)


# ------------------------------------------------------------------------------ inputs -----
def make_attention_inputs(case: Case):
    """K/V blobs, tail K/V and queries drawn directly (attention-only parity)."""
    c = case
    qs = c.q_scale if c.q_scale is not None else c.scale
    blobs = {cid: normal((c.name, "blob", cid), (c.n_layers, 2, c.Hkv, n, c.D), c.scale, c.tdtype)
             for cid, n in c.chunk_lens.items()}
    tail = normal((c.name, "tail"), (c.n_layers, 2, c.batch, c.Hkv, c.tail_cap, c.D), c.scale, c.tdtype)
    total_q = sum(c.q_lens)
    q_pre = normal((c.name, "q_pre"), (c.n_layers, total_q, c.Hq, c.D), qs, c.tdtype)
    q_dec = normal((c.name, "q_dec"), (max(c.steps, 1), c.n_layers, c.batch, c.Hq, c.D), qs, c.tdtype)
    if c.needle:
        # one key of the first chunk of every instance lines up with every query: component 0
        # of all queries is 16, of that key 24 (score about +34 at D = 128), rest of the key 0
        for b, r in enumerate(c.retrieved):
            if not r:
                continue
            pos = (7 * (b + 1)) % c.chunk_lens[r[0]]
            blobs[r[0]][:, 0, :, pos, :] = 0
            blobs[r[0]][:, 0, :, pos, 0] = 24.0
        q_pre[..., 0] = 16.0
        q_dec[..., 0] = 16.0
    return dict(blobs=blobs, tail=tail, q_pre=q_pre, q_dec=q_dec)


def make_chain_inputs(case: Case):
    """Hidden states, projection weights and queries (full M -> L -> P -> D chain)."""
    c = case
    qs = c.q_scale if c.q_scale is not None else c.scale
    w = normal((c.name, "w"), (c.n_layers, 2, c.Hkv * c.D, c.hidden), c.scale, c.tdtype)
    x_chunk = {cid: normal((c.name, "x_chunk", cid), (c.n_layers, n, c.hidden), c.scale, c.tdtype)
               for cid, n in c.chunk_lens.items()}
    total_q = sum(c.q_lens)
    x_q = normal((c.name, "x_q"), (c.n_layers, total_q, c.hidden), c.scale, c.tdtype)
    x_dec = normal((c.name, "x_dec"), (max(c.steps, 1), c.n_layers, c.batch, c.hidden), c.scale, c.tdtype)
    q_pre = normal((c.name, "q_pre"), (c.n_layers, total_q, c.Hq, c.D), qs, c.tdtype)
    q_dec = normal((c.name, "q_dec"), (max(c.steps, 1), c.n_layers, c.batch, c.Hq, c.D), qs, c.tdtype)
    return dict(w=w, x_chunk=x_chunk, x_q=x_q, x_dec=x_dec, q_pre=q_pre, q_dec=q_dec)


def make_chunk_queries(case: Case):
    """Queries of the chunks' own tokens (already rotated), for the materialization pass."""
    c = case
    qs = c.q_scale if c.q_scale is not None else c.scale
    return {cid: normal((c.name, "q_chunk", cid), (c.n_layers, n, c.Hq, c.D), qs, c.tdtype)
            for cid, n in c.chunk_lens.items()}


# ------------------------------------------------------------------------------ GPU side ---
def make_context(case: Case, device="cuda:0"):
    from paper_2512_22195_amd import binding as mk
    cfg = mk.make_config(case.n_layers, case.Hq, case.Hkv, case.D, case.hidden, case.dtype,
                         case.rope_base, max_batch=case.batch, max_pages=case.max_pages,
                         max_tail_tokens=case.tail_cap, decode_units=case.decode_units,
                         decode_variant=case.decode_variant, out_f32=int(case.out_f32))
    return mk.Context(cfg, device=device)


def page_format(case: Case):
    from paper_2512_22195_amd import binding as mk
    return mk.PAGE_E4M3 if case.compressed else mk.PAGE_PLAIN


def pages_of(case: Case, slots: dict):
    return [[(slots[cid], case.chunk_lens[cid], page_format(case)) for cid in r] for r in case.retrieved]


def compress_on_gpu(ctx, case: Case, dev_blob, n_tokens):
    """matkv_compress of a device blob; returns the compressed blob as a device byte tensor."""
    from paper_2512_22195_amd import binding as mk
    out = torch.empty(mk.compressed_blob_bytes(ctx.cfg, n_tokens), dtype=torch.uint8, device=dev_blob.device)
    with torch.cuda.stream(ctx.compute_stream):
        ctx.compress(dev_blob, n_tokens, out)
        ctx.compute_stream.synchronize()
    return out


def load_blobs(ctx, case: Case, blobs: dict):
    """store_KV stand-in: blobs sit in pinned host memory; load_KV: matkv_load into slots.
    With case.compressed the blob is compressed on the GPU first and its compressed form is
    what sits in host memory and is loaded."""
    slots, keep = {}, []
    for cid, blob in blobs.items():
        if case.compressed:
            with torch.cuda.stream(ctx.compute_stream):
                dev = blob.contiguous().to(ctx.device)
            host = compress_on_gpu(ctx, case, dev, case.chunk_lens[cid]).cpu().pin_memory()
        else:
            host = blob.contiguous().view(torch.uint8).reshape(-1).pin_memory()
        slot = ctx.new_slot(case.chunk_lens[cid])
        t = ctx.load(host, case.chunk_lens[cid], slot)
        ctx.wait(t)
        slots[cid] = slot
        keep.append(host)
    return slots, keep


def run_gpu_attention(case: Case, inp, device="cuda:0", use_graph=False, ctx=None, proj=None, info=None):
    """Returns (prefill O [n_layers, total_q, Hq, D], decode O [steps, n_layers, B, Hq, D]) as CPU tensors.
    info: a dict that receives what the table reports about itself (shared_units)."""
    c = case
    own = ctx is None
    ctx = ctx or make_context(c, device)
    try:
        slots, keep = load_blobs(ctx, c, inp["blobs"])
        with torch.cuda.stream(ctx.compute_stream):
            tail = inp["tail"].to(device, non_blocking=False)
            q_pre = inp["q_pre"].to(device)
            q_dec = inp["q_dec"].to(device)
            table = ctx.new_table()
            pages = pages_of(c, slots)
            ctx.assemble(pages, c.q_lens, table)
            if info is not None:
                info["shared_units"] = ctx.table_shared_units(table)
            o_pre = torch.full_like(q_pre, float("nan"), dtype=c.odtype)
            o_dec = torch.full_like(q_dec, float("nan"), dtype=c.odtype)
            for l in range(c.n_layers):
                ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
            if proj is not None and c.steps > 0:
                # decode steps through matkv_decode_step, recorded once and replayed (the launch
                # configuration bench.py times): the new token's K/V come from proj["x_dec"][t]
                w, x_dec = proj["w"].to(device), proj["x_dec"].to(device)
                q_stage, o_stage, x_stage = torch.empty_like(q_dec[0]), torch.empty_like(o_dec[0]), torch.empty_like(x_dec[0])
                ctx.graph_begin()
                ctx.advance(table, 1)
                for l in range(c.n_layers):
                    ctx.decode_step(l, x_stage[l], w[l, 0], w[l, 1], q_stage[l], table, tail[l, 0], tail[l, 1], o_stage[l])
                g = ctx.graph_end()
                for t in range(c.steps):
                    q_stage.copy_(q_dec[t]); x_stage.copy_(x_dec[t])
                    ctx.graph_launch(g)
                    o_dec[t].copy_(o_stage)
                    if t % 2 == 1:
                        ctx.compute_stream.synchronize()
                ctx.graph_destroy(g)
            elif use_graph and c.steps > 0:
                # one recording of a decode step (all layers), replayed for every step; q and
                # out live in fixed staging buffers that are refreshed between replays
                q_stage = torch.empty_like(q_dec[0])
                o_stage = torch.empty_like(o_dec[0])
                ctx.graph_begin()
                ctx.advance(table, 1)
                for l in range(c.n_layers):
                    ctx.decode_attn(l, q_stage[l], table, tail[l, 0], tail[l, 1], o_stage[l])
                g = ctx.graph_end()
                for t in range(c.steps):
                    q_stage.copy_(q_dec[t])
                    ctx.graph_launch(g)
                    o_dec[t].copy_(o_stage)
                    if t % 2 == 1:
                        ctx.compute_stream.synchronize()   # eager work and syncs between replays
                ctx.graph_destroy(g)
            else:
                for t in range(c.steps):
                    ctx.advance(table, 1)
                    for l in range(c.n_layers):
                        ctx.decode_attn(l, q_dec[t, l], table, tail[l, 0], tail[l, 1], o_dec[t, l])
            ctx.compute_stream.synchronize()
            res = o_pre.cpu(), (o_dec.cpu() if c.steps > 0 else o_dec[:0].cpu())
        del keep
        return res
    finally:
        if own:
            ctx.close()


def run_gpu_chain(case: Case, inp, device="cuda:0", fused=False, use_graph=False, blob_dir=None):
    """Full chain.  Returns dict with materialized blobs/tail (CPU tensors) and outputs.
    fused: each decode step of a layer is one matkv_decode_step call instead of
    matkv_materialize_tail + matkv_decode_attn; use_graph (with fused): the step of all layers
    is recorded once and replayed, with a synchronisation and an eager copy between replays.
    blob_dir: materialized chunks go to one file there (matkv_store_file) and come back into the
    slots from it (matkv_load_file) instead of through pinned host tensors."""
    c = case
    ctx = make_context(c, device)
    try:
        with torch.cuda.stream(ctx.compute_stream):
            w = inp["w"].to(device)
            # M: every chunk alone, positions from 0, straight into a blob-shaped buffer
            dev_blobs = {}
            for cid, n in c.chunk_lens.items():
                x = inp["x_chunk"][cid].to(device)
                blob = torch.zeros((c.n_layers, 2, c.Hkv, n, c.D), dtype=c.tdtype, device=device)
                for l in range(c.n_layers):
                    ctx.materialize(x[l], w[l, 0], w[l, 1], n, 0, blob[l, 0], blob[l, 1], n)
                dev_blobs[cid] = blob
            ctx.compute_stream.synchronize()
            host_blobs = {cid: b.cpu() for cid, b in dev_blobs.items()}     # store_KV stand-in
        if blob_dir is not None:
            import os
            path = os.path.join(blob_dir, f"{c.name}.kv")
            fd = os.open(path, os.O_RDWR | os.O_CREAT | os.O_TRUNC, 0o600)
            try:
                offs, off = {}, 0
                stored = {cid: (compress_on_gpu(ctx, c, b, c.chunk_lens[cid]) if c.compressed else b)
                          for cid, b in dev_blobs.items()}
                for cid, b in stored.items():                                # store_KV
                    offs[cid] = off
                    ctx.store_file(fd, off, b)
                    off += (b.numel() * b.element_size() + 4095) // 4096 * 4096
                os.fsync(fd)
                slots = {}
                for cid, n in c.chunk_lens.items():                          # load_KV
                    slots[cid] = ctx.new_slot(n)
                    nb = stored[cid].numel() * stored[cid].element_size()
                    ctx.wait(ctx.load_file(fd, offs[cid], nb, n, slots[cid]))
                with open(path, "rb") as f:                                  # the file holds the blobs' bytes
                    for cid, b in stored.items():
                        f.seek(offs[cid])
                        raw = f.read(b.numel() * b.element_size())
                        assert raw == b.cpu().contiguous().view(torch.uint8).numpy().tobytes(), f"file bytes of chunk {cid}"
                del stored
            finally:
                os.close(fd)
            keep = None
        del dev_blobs
        if blob_dir is None:
            slots, keep = load_blobs(ctx, c, host_blobs)                     # L
        with torch.cuda.stream(ctx.compute_stream):
            tail = ctx.new_tail()
            table = ctx.new_table()
            pages = pages_of(c, slots)
            ctx.assemble(pages, c.q_lens, table)                             # A
            x_q, x_dec = inp["x_q"].to(device), inp["x_dec"].to(device)
            q_pre, q_dec = inp["q_pre"].to(device), inp["q_dec"].to(device)
            o_pre = torch.full_like(q_pre, float("nan"), dtype=c.odtype)
            o_dec = torch.full_like(q_dec, float("nan"), dtype=c.odtype)
            for l in range(c.n_layers):                                      # M (question) + P
                ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
                ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
            if fused and use_graph and c.steps > 0:
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
                    ctx.compute_stream.synchronize()
                ctx.graph_destroy(g)
            else:
                for t in range(c.steps):                                     # M (token) + D
                    ctx.advance(table, 1)
                    for l in range(c.n_layers):
                        if fused:
                            ctx.decode_step(l, x_dec[t, l], w[l, 0], w[l, 1], q_dec[t, l], table,
                                            tail[l, 0], tail[l, 1], o_dec[t, l])
                        else:
                            ctx.materialize_tail(x_dec[t, l], w[l, 0], w[l, 1], table, 1, tail[l, 0], tail[l, 1])
                            ctx.decode_attn(l, q_dec[t, l], table, tail[l, 0], tail[l, 1], o_dec[t, l])
            ctx.compute_stream.synchronize()
            return dict(blobs=host_blobs, tail=tail.cpu(), o_pre=o_pre.cpu(),
                        o_dec=o_dec.cpu() if c.steps > 0 else o_dec[:0].cpu())
    finally:
        ctx.close()


# --------------------------------------------------------------------------- oracle side ---
def run_gpu_chunk_prefill(case: Case, inp, q_chunk, device="cuda:0"):
    """Materialization pass of every chunk: per layer, K/V of the chunk's hidden states into its
    blob (matkv_materialize), then the chunk's own causal attention over that section
    (matkv_chunk_attn).  Returns (blobs, outputs) as CPU tensors keyed by chunk id."""
    c = case
    ctx = make_context(c, device)
    try:
        blobs, outs = {}, {}
        with torch.cuda.stream(ctx.compute_stream):
            w = inp["w"].to(device)
            for cid, n in c.chunk_lens.items():
                x, q = inp["x_chunk"][cid].to(device), q_chunk[cid].to(device)
                blob = torch.zeros((c.n_layers, 2, c.Hkv, n, c.D), dtype=c.tdtype, device=device)
                o = torch.full_like(q, float("nan"), dtype=c.odtype)
                for l in range(c.n_layers):
                    ctx.materialize(x[l], w[l, 0], w[l, 1], n, 0, blob[l, 0], blob[l, 1], n)
                    ctx.chunk_attn(l, q[l], blob, n, o[l])
                ctx.compute_stream.synchronize()
                blobs[cid], outs[cid] = blob.cpu(), o.cpu()
        return blobs, outs
    finally:
        ctx.close()


def run_oracle_chunk_prefill(case: Case, inp, q_chunk):
    """fp64: K/V of the chunk at positions 0.., rounded once to the storage type, then causal
    attention of the chunk over itself.  Returns {(cid, layer): O [n, Hq, D]}."""
    c = case
    ref = {}
    for cid, n in c.chunk_lens.items():
        for l in range(c.n_layers):
            K, V = oracle.materialize(to_f64(inp["x_chunk"][cid][l]), to_f64(inp["w"][l, 0]),
                                      to_f64(inp["w"][l, 1]), c.Hkv, c.D, 0.0, c.rope_base)
            ref[(cid, l)] = oracle.chunk_attn(to_f64(q_chunk[cid][l]), store_round(K, c.dtype),
                                              store_round(V, c.dtype))
    return ref


def compare_chunk_prefill(case: Case, outs, ref):
    atol, rtol = tolerances(case.dtype)
    worst = 0.0
    for (cid, l), r in ref.items():
        got = to_f64(outs[cid][l])
        assert np.isfinite(got).all(), f"chunk {cid} layer {l}: non-finite output"
        err = np.abs(got - r)
        # the relative gate is per row: the first rows average a handful of values and are an
        # order of magnitude larger than rows that average hundreds
        rms = np.sqrt((r ** 2).mean(axis=(1, 2), keepdims=True))
        assert (err <= atol + store_slack(case.dtype, r, case.out_f32)).all(), f"chunk {cid} layer {l}: max abs {err.max():.3e} > {atol}"
        bad = err > rtol * rms + store_slack(case.dtype, r, case.out_f32)
        assert not bad.any(), f"chunk {cid} layer {l}: max abs {err.max():.3e} at rows {np.unique(np.nonzero(bad)[0])[:8]}"
        worst = max(worst, err.max())
    return worst


def cu_q(case: Case):
    cu = [0]
    for n in case.q_lens:
        cu.append(cu[-1] + n)
    return cu


def as_loaded(case: Case, K, V):
    """What the attention reads of a chunk's stored K/V: the values themselves, or - through a
    compressed blob - their 8-bit codes times the head's scale."""
    if not case.compressed:
        return K, V
    return oracle.decompress(*oracle.compress(K, V))


def run_oracle_attention(case: Case, inp, layers=None, steps=None, instances=None, prefill_rows=None, proj=None):
    """fp64 oracle over the same generated K/V.  Returns dicts keyed by (layer) / (step, layer)
    of arrays shaped like the GPU outputs restricted to the sampled instances.
    proj: the tail rows of the decode steps are not the generated ones but the projection of
    proj["x_dec"][t] at position (chunk tokens + question length + t), rounded to the storage type."""
    c = case
    layers = range(c.n_layers) if layers is None else layers
    steps = range(c.steps) if steps is None else steps
    instances = range(c.batch) if instances is None else instances
    cu = cu_q(c)
    tail = inp["tail"]
    pre, dec = {}, {}
    for l in layers:
        for b in instances:
            chunks = [as_loaded(c, to_f64(inp["blobs"][cid][l, 0]), to_f64(inp["blobs"][cid][l, 1])) for cid in c.retrieved[b]]
            lq = c.q_lens[b]
            tk, tv = to_f64(tail[l, 0, b]), to_f64(tail[l, 1, b])
            if prefill_rows is None:
                pre[(l, b)] = oracle.prefill_attn(to_f64(inp["q_pre"][l, cu[b]:cu[b + 1]]), chunks,
                                                  tk[:, :lq], tv[:, :lq])
            else:
                # sampled question rows: row r is a one-row attention that sees tail tokens 0..r
                K, V, n_ctx = oracle.assemble(chunks, tk[:, :lq], tv[:, :lq])
                for r in sorted({min(max(r, 0), lq - 1) for r in prefill_rows}):
                    pre[(l, b, r)] = oracle.attn(to_f64(inp["q_pre"][l, cu[b] + r])[None], K, V, n_ctx, r)
            if proj is not None and len(list(steps)) > 0:
                tk, tv = tk.copy(), tv.copy()
                p0 = float(sum(c.chunk_lens[cid] for cid in c.retrieved[b]))
                wk, wv = to_f64(proj["w"][l, 0]), to_f64(proj["w"][l, 1])
                for t in range(max(steps) + 1):
                    Kt, Vt = oracle.materialize(to_f64(proj["x_dec"][t, l, b])[None], wk, wv, c.Hkv, c.D,
                                                p0 + lq + t, c.rope_base)
                    tk[:, lq + t] = store_round(Kt, c.dtype)[:, 0]
                    tv[:, lq + t] = store_round(Vt, c.dtype)[:, 0]
            for t in steps:
                n = lq + t + 1
                dec[(t, l, b)] = oracle.decode_attn(to_f64(inp["q_dec"][t, l, b]), chunks, tk[:, :n], tv[:, :n])
    return pre, dec


def run_oracle_chain(case: Case, inp):
    """fp64 chain: materialize every chunk alone at positions 0.., round once to the storage
    type, question tokens at pos_base = total chunk tokens of the instance, then attention."""
    c = case
    cu = cu_q(c)
    blobs = {}
    for cid, n in c.chunk_lens.items():
        per_layer = []
        for l in range(c.n_layers):
            K, V = oracle.materialize(to_f64(inp["x_chunk"][cid][l]), to_f64(inp["w"][l, 0]),
                                      to_f64(inp["w"][l, 1]), c.Hkv, c.D, 0.0, c.rope_base)
            per_layer.append((K, V))
        blobs[cid] = per_layer
    pre, dec, tails = {}, {}, {}
    for l in range(c.n_layers):
        wk, wv = to_f64(inp["w"][l, 0]), to_f64(inp["w"][l, 1])
        for b in range(c.batch):
            lq = c.q_lens[b]
            p0 = float(sum(c.chunk_lens[cid] for cid in c.retrieved[b]))
            xs = [to_f64(inp["x_q"][l, cu[b]:cu[b + 1]])] + [to_f64(inp["x_dec"][t, l, b])[None] for t in range(c.steps)]
            Kt, Vt = oracle.materialize(np.concatenate(xs), wk, wv, c.Hkv, c.D, p0, c.rope_base)
            tails[(l, b)] = (Kt, Vt)
            Ktr, Vtr = store_round(Kt, c.dtype), store_round(Vt, c.dtype)
            chunks = [as_loaded(c, store_round(blobs[cid][l][0], c.dtype), store_round(blobs[cid][l][1], c.dtype))
                      for cid in c.retrieved[b]]
            pre[(l, b)] = oracle.prefill_attn(to_f64(inp["q_pre"][l, cu[b]:cu[b + 1]]), chunks,
                                              Ktr[:, :lq], Vtr[:, :lq])
            for t in range(c.steps):
                n = lq + t + 1
                dec[(t, l, b)] = oracle.decode_attn(to_f64(inp["q_dec"][t, l, b]), chunks, Ktr[:, :n], Vtr[:, :n])
    return dict(blobs=blobs, tails=tails, pre=pre, dec=dec)


# ----------------------------------------------------------------------------- comparing ---
def tolerances(dtype: str):
    """(max-abs gate, relative-to-rms gate) for attention outputs: the stated bars (1e-5 fp32,
    1e-2 bf16 inputs with fp32 accumulation) plus a relative gate, because with near-uniform
    softmax the outputs are far smaller than the absolute bar.  For bf16 the relative gate is
    applied per element with half an ulp of the stored output (2^-8 |ref|) added: an output
    several times the rms is rounded by more than the rms gate alone allows.  The same half ulp
    is added to the absolute bar: an output beyond 2.56 is stored with an error of up to more
    than 1e-2 whatever was computed (4.1381 is stored as 4.125)."""
    return (1e-5, 1e-4) if dtype == "f32" else (1e-2, 2e-2)


def store_slack(dtype: str, ref, out_f32: bool = False):
    """Per-element allowance for the one rounding of the output to its storage type: half an
    ulp of bf16, nothing to speak of for float outputs (fp32 configurations, and bf16
    configurations with out_f32, where the stated bars are asserted as they stand)."""
    return 1e-7 if (dtype == "f32" or out_f32) else 2.0 ** -8 * np.abs(ref)


def compare_attention(case: Case, o_pre, o_dec, pre, dec):
    """Max abs error over everything the oracle computed; asserts both gates."""
    cu = cu_q(case)
    atol, rtol = tolerances(case.dtype)
    worst = 0.0
    for key, ref in pre.items():
        l, b = key[0], key[1]
        got = to_f64(o_pre[l, cu[b]:cu[b + 1]]) if len(key) == 2 else to_f64(o_pre[l, cu[b] + key[2]])[None]
        assert np.isfinite(got).all(), f"prefill layer {l} instance {b}: non-finite output"
        err = np.abs(got - ref).max()
        rms = np.sqrt((ref ** 2).mean())
        assert (np.abs(got - ref) <= atol + store_slack(case.dtype, ref, case.out_f32)).all(), f"prefill layer {l} inst {b}: max abs {err:.3e} > {atol}"
        assert (np.abs(got - ref) <= rtol * rms + store_slack(case.dtype, ref, case.out_f32)).all(), \
            f"prefill layer {l} inst {b}: max abs {err:.3e} vs rms {rms:.3e}"
        worst = max(worst, err)
    for (t, l, b), ref in dec.items():
        got = to_f64(o_dec[t, l, b])
        assert np.isfinite(got).all(), f"decode step {t} layer {l} instance {b}: non-finite output"
        err = np.abs(got - ref).max()
        rms = np.sqrt((ref ** 2).mean())
        assert (np.abs(got - ref) <= atol + store_slack(case.dtype, ref, case.out_f32)).all(), f"decode step {t} layer {l} inst {b}: max abs {err:.3e} > {atol}"
        assert (np.abs(got - ref) <= rtol * rms + store_slack(case.dtype, ref, case.out_f32)).all(), \
            f"decode step {t} layer {l} inst {b}: max abs {err:.3e} vs rms {rms:.3e}"
        worst = max(worst, err)
    return worst


def compare_materialized(case: Case, got_kv, ref_kv, what: str):
    """Stored K/V against the unrounded fp64 value: half an ulp of the storage type plus the
    fp32 accumulation error of an Hd-term dot product."""
    got, ref = to_f64(got_kv), ref_kv
    assert np.isfinite(got).all(), f"{what}: non-finite"
    err = np.abs(got - ref)
    if case.dtype == "f32":
        bound = 1e-5 + 4e-6 * np.abs(ref)
    else:
        bound = 2.0 ** -8 * np.abs(ref) + 2e-4 * max(1.0, np.abs(ref).max())
        assert err.max() <= 1e-2 * max(1.0, np.abs(ref).max()), f"{what}: max abs {err.max():.3e}"
    assert (err <= bound).all(), f"{what}: worst excess {(err - bound).max():.3e} at {np.unravel_index((err - bound).argmax(), err.shape)}"
    return err.max()


def run_chain_case(config_id: int = 1, verbose: bool = False, device="cuda:0") -> float:
    """The smoke check: configuration 1 end to end against the oracle."""
    case = case_from_config(config_id)
    inp = make_chain_inputs(case)
    gpu = run_gpu_chain(case, inp, device)
    ref = run_oracle_chain(case, inp)
    worst = 0.0
    for cid in case.chunk_lens:
        for l in range(case.n_layers):
            worst = max(worst, compare_materialized(case, gpu["blobs"][cid][l, 0], ref["blobs"][cid][l][0], f"chunk {cid} K"))
            worst = max(worst, compare_materialized(case, gpu["blobs"][cid][l, 1], ref["blobs"][cid][l][1], f"chunk {cid} V"))
    for (l, b), (Kt, Vt) in ref["tails"].items():
        n = Kt.shape[1]
        worst = max(worst, compare_materialized(case, gpu["tail"][l, 0, b, :, :n], Kt, f"tail K layer {l} inst {b}"))
        worst = max(worst, compare_materialized(case, gpu["tail"][l, 1, b, :, :n], Vt, f"tail V layer {l} inst {b}"))
    worst = max(worst, compare_attention(case, gpu["o_pre"], gpu["o_dec"], ref["pre"], ref["dec"]))
    if verbose:
        print(f"chain case {case.name}: worst abs error {worst:.3e}")
    return worst
