#!/usr/bin/env python3
"""Benchmark of the MatKV hot path on one MI355X.

A "step" is one pass of the whole path over one RAG instance batch with its chunk KVs already
resident in HBM: cache assembly, K/V materialization of the question tokens + prefill attention
for every layer, then every decode step (K/V materialization of the new token + decode
attention for every layer, replayed from one captured graph).  ``value`` is generated tokens
per second over that pass.  Beside it: the decode-attention kernel's achieved HBM bandwidth
(``roofline``), the pinned-host-to-HBM load rate of the instance's blobs (``kv_load``, never
part of ``value``), and the fp64 oracle timed on the host cores (``cpu_baseline``).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--units N] [--variant V] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=2, help="BASELINE.json config number (1-based)")
    ap.add_argument("--units", type=int, default=0, help="decode workgroups per (instance, KV head); 0 = library's choice")
    ap.add_argument("--variant", type=int, default=0, help="decode kernel shape (waves*100 + loads in flight); 0 = default")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-load", action="store_true", help="skip the kv_load leg")
    ap.add_argument("--no-batch16", action="store_true", help="skip the batch-16 decode-attention leg")
    ap.add_argument("--no-compressed", action="store_true", help="skip the leg with the chunks held as compressed blobs")
    ap.add_argument("--with-others", action="store_true",
                    help="with --roofline-only: also run the other kernels' leg (few eager launches each)")
    ap.add_argument("--unfused", action="store_true",
                    help="decode steps as matkv_materialize_tail + matkv_decode_attn instead of matkv_decode_step")
    ap.add_argument("--decode-only-reps", type=int, default=20)
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the decode-attention leg, launched eagerly (short run for rocprofv3 --pmc)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--stream", type=int, default=8,
                    help="instances of the pipelined leg (next instance loads while this one decodes); 0 = skip")
    return ap.parse_args()


def file_load_leg(ctx, host, dst, L, nbytes, with_fd=None):
    import tempfile
    import torch
    path = os.path.join(tempfile.gettempdir(), f"matkv_bench_{os.getpid()}.bin")
    try:
        with open(path, "wb") as f:
            for h in host:
                f.write(h.numpy().data)
            f.flush(); os.fsync(f.fileno())
            try:
                os.posix_fadvise(f.fileno(), 0, 0, os.POSIX_FADV_DONTNEED)
            except OSError:
                pass
        direct = True
        try:
            fd = os.open(path, os.O_RDONLY | os.O_DIRECT)
        except OSError:
            direct, fd = False, os.open(path, os.O_RDONLY)
        try:
            best = None
            for rep in range(2):
                t0 = time.perf_counter()
                tickets = [ctx.load_file(fd, i * nbytes, nbytes, L, d) for i, d in enumerate(dst)]
                ctx.sync(tickets[-1])
                dt = time.perf_counter() - t0
                best = dt if best is None else min(best, dt)
            ok = torch.equal(dst[-1].cpu(), host[-1])
            extra = with_fd(fd) if with_fd else None
        finally:
            os.close(fd)
        return {"GBps": round(len(host) * nbytes / best / 1e9, 2), "ms_per_instance": round(best * 1e3, 3),
                "o_direct": direct, "byte_exact": bool(ok), "dir": os.path.dirname(path), "pipelined_stream": extra}
    finally:
        if os.path.exists(path):
            os.remove(path)


def batch16_decode_leg(reps=10, nl=8, compressed=False):
    """Decode attention at BASELINE config 3's shape (batch 16, five 1000-token chunks each from a
    pool of 200, question lengths 32..128, tails at mid-run), nl layers resident: the launch size
    at which the kernel is bandwidth-bound rather than bound by its fixed cost per launch."""
    import torch
    from paper_2512_22195_amd import binding as mk
    from workload import CONFIGS, normal, question_lengths, retrieved_chunks
    shape = CONFIGS[3]
    dev = torch.device("cuda:0")
    B, Hq, Hkv, D, Hd, L = shape.batch, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.hidden, shape.chunk_tokens
    q_lens, retrieved = question_lengths(shape), retrieved_chunks(shape)
    chunk_ids = sorted({c for r in retrieved for c in r})
    max_tail = (max(q_lens) + shape.decode_steps + 7) // 8 * 8
    cfg = mk.make_config(nl, Hq, Hkv, D, Hd, shape.dtype, shape.rope_base, max_batch=B, max_pages=shape.n_chunks,
                         max_tail_tokens=max_tail)
    ctx = mk.Context(cfg, device=dev)
    cs = ctx.compute_stream
    try:
        with torch.cuda.stream(cs):
            slots = {}
            for cid in chunk_ids:
                slots[cid] = normal((shape.name, "blob", cid), (nl, 2, Hkv, L, D), shape.value_scale, shape.torch_dtype, dev)
                if compressed:
                    out = torch.empty(mk.compressed_blob_bytes(cfg, L), dtype=torch.uint8, device=dev)
                    ctx.compress(slots[cid], L, out)
                    cs.synchronize()
                    slots[cid] = out
            fmt = mk.PAGE_E4M3 if compressed else mk.PAGE_PLAIN
            q = normal((shape.name, "q_dec"), (nl, B, Hq, D), shape.value_scale, shape.torch_dtype, dev)
            o = torch.empty_like(q)
            tail = normal((shape.name, "tail"), (nl, 2, B, Hkv, max_tail, D), shape.value_scale, shape.torch_dtype, dev)
            table = ctx.new_table()
            ctx.assemble([[(slots[cid], L, fmt) for cid in r] for r in retrieved], q_lens, table)
            ctx.advance(table, shape.decode_steps // 2)
            ctx.graph_begin()
            for l in range(nl):
                ctx.decode_attn(l, q[l], table, tail[l, 0], tail[l, 1], o[l])
            g = ctx.graph_end()
            for _ in range(3):
                ctx.graph_launch(g)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(cs)
            for _ in range(reps):
                ctx.graph_launch(g)
            b.record(cs)
            cs.synchronize()
            ctx.graph_destroy(g)
        us = a.elapsed_time(b) * 1e3 / (reps * nl)
        page_token_bytes = 2 * Hkv * D if compressed else shape.kv_bytes_per_token_layer()
        nbytes = sum(L * len(r) * page_token_bytes + (ql + shape.decode_steps // 2) * shape.kv_bytes_per_token_layer()
                     for r, ql in zip(retrieved, q_lens)) + 2 * B * Hq * D * shape.elem_bytes
        return {"workload": f"BASELINE config 3 shape: batch {B}, {shape.n_chunks} x {L} tokens each, {nl} layers resident "
                            f"({len(chunk_ids)} distinct chunks)",
                "bytes_per_launch": nbytes, "us_per_launch": round(us, 3), "GBps": round(nbytes / us / 1e3, 1),
                "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)}
    finally:
        ctx.close()


def compressed_leg(config_id, reps=5):
    """The same workload with the chunks held as compressed blobs (E4M3 codes + per-head scales,
    matkv_compress): compression rate, load rate, the whole pass, and the decode step alone."""
    import torch
    from paper_2512_22195_amd import binding as mk
    from workload import CONFIGS, normal, question_lengths, retrieved_chunks
    shape = CONFIGS[config_id]
    dev = torch.device("cuda:0")
    tdt, vs = shape.torch_dtype, shape.value_scale
    B, nl, Hq, Hkv, D, Hd, L = shape.batch, shape.n_layers, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.hidden, shape.chunk_tokens
    q_lens, retrieved = question_lengths(shape), retrieved_chunks(shape)
    chunk_ids = sorted({c for r in retrieved for c in r})
    max_tail = (max(q_lens) + shape.decode_steps + 7) // 8 * 8
    cfg = mk.make_config(nl, Hq, Hkv, D, Hd, shape.dtype, shape.rope_base, max_batch=B, max_pages=shape.n_chunks,
                         max_tail_tokens=max_tail)
    ctx = mk.Context(cfg, device=dev)
    cs = ctx.compute_stream
    ev = lambda: torch.cuda.Event(enable_timing=True)
    try:
        cbytes, pbytes = mk.compressed_blob_bytes(cfg, L), mk.blob_bytes(cfg, L)
        with torch.cuda.stream(cs):
            slots, t_comp = {}, []
            for cid in chunk_ids:
                blob = normal((shape.name, "blob", cid), (nl, 2, Hkv, L, D), vs, tdt, dev)
                slots[cid] = torch.empty(cbytes, dtype=torch.uint8, device=dev)
                a, b = ev(), ev()
                a.record(cs)
                ctx.compress(blob, L, slots[cid])
                b.record(cs)
                t_comp.append((a, b))
                cs.synchronize()
                del blob
            us_comp = min(a.elapsed_time(b) for a, b in t_comp[1:] or t_comp) * 1e3
            # load: one compressed blob from pinned host memory into a spare slot, several times
            host = slots[chunk_ids[0]].cpu().pin_memory()
            spare = torch.empty(cbytes, dtype=torch.uint8, device=dev)
        t0 = time.perf_counter()
        n_load = 10
        for _ in range(n_load):
            tk = ctx.load(host, L, spare)
        ctx.sync(tk)
        load_s = (time.perf_counter() - t0) / n_load
        with torch.cuda.stream(cs):
            w = normal((shape.name, "w"), (nl, 2, Hkv * D, Hd), vs, tdt, dev)
            total_q = sum(q_lens)
            x_q = normal((shape.name, "x_q"), (nl, total_q, Hd), vs, tdt, dev)
            x_dec = normal((shape.name, "x_dec"), (nl, B, Hd), vs, tdt, dev)
            q_pre = normal((shape.name, "q_pre"), (nl, total_q, Hq, D), vs, tdt, dev)
            q_dec = normal((shape.name, "q_dec"), (nl, B, Hq, D), vs, tdt, dev)
            o_pre, o_dec = torch.empty_like(q_pre), torch.empty_like(q_dec)
            tail, table = ctx.new_tail(), ctx.new_table()
            pages = [[(slots[cid], L, mk.PAGE_E4M3) for cid in r] for r in retrieved]

            def prefill_phase():
                ctx.assemble(pages, q_lens, table)
                for l in range(nl):
                    ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
                    ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])

            prefill_phase()
            ctx.graph_begin()
            ctx.advance(table, 1)
            for l in range(nl):
                ctx.decode_step(l, x_dec[l], w[l, 0], w[l, 1], q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
            g_step = ctx.graph_end()
            ctx.graph_begin()
            for l in range(nl):
                ctx.decode_step(l, x_dec[l], w[l, 0], w[l, 1], q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
            g_fixed = ctx.graph_end()
            for _ in range(shape.decode_steps):
                ctx.graph_launch(g_step)
            cs.synchronize()
            # the whole pass
            a, b, c = ev(), ev(), ev()
            a.record(cs)
            prefill_phase()
            b.record(cs)
            for _ in range(shape.decode_steps):
                ctx.graph_launch(g_step)
            c.record(cs)
            # the decode step alone, tail at its mid-run length
            ctx.assemble(pages, q_lens, table)
            ctx.advance(table, shape.decode_steps // 2)
            for _ in range(2):
                ctx.graph_launch(g_fixed)
            d, e = ev(), ev()
            d.record(cs)
            for _ in range(reps):
                ctx.graph_launch(g_fixed)
            e.record(cs)
            # question prefill attention alone
            f0, f1 = ev(), ev()
            f0.record(cs)
            for l in range(nl):
                ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
            f1.record(cs)
            cs.synchronize()
            ctx.graph_destroy(g_step); ctx.graph_destroy(g_fixed)
        ms_pass = a.elapsed_time(c)
        us_step = d.elapsed_time(e) * 1e3 / (reps * nl)
        page_b = sum(L * len(r) for r in retrieved) * 2 * Hkv * D                       # one byte per element
        tail_b = sum(q + shape.decode_steps // 2 for q in q_lens) * shape.kv_bytes_per_token_layer()
        proj_b = 2 * Hkv * D * Hd * shape.elem_bytes + B * Hd * shape.elem_bytes
        nbytes = page_b + tail_b + proj_b + 2 * B * Hq * D * shape.elem_bytes
        return {"format": "E4M3 codes + one power-of-two scale per (layer, K/V, KV head)",
                "blob_bytes": cbytes, "plain_blob_bytes": pbytes,
                "compress": {"us_per_chunk": round(us_comp, 1), "GBps_read_plus_written": round((pbytes + cbytes) / us_comp / 1e3, 1)},
                "load": {"GBps": round(cbytes / load_s / 1e9, 2), "ms_per_chunk": round(load_s * 1e3, 3)},
                "tokens_per_s": round(B * shape.decode_steps / (ms_pass * 1e-3), 2),
                "phases_ms": {"assemble+materialize+prefill": round(a.elapsed_time(b), 3), "decode": round(b.elapsed_time(c), 3)},
                "decode_step": {"bytes_per_launch": nbytes, "us_per_launch": round(us_step, 3), "GBps": round(nbytes / us_step / 1e3, 1),
                                "frac_of_hbm_peak": round(nbytes / us_step / 1e3 / HBM_PEAK_GBPS, 4)},
                "prefill_attn_us_per_layer": round(f0.elapsed_time(f1) * 1e3 / nl, 2)}
    finally:
        ctx.close()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU; --gpus above 1 is not supported "
              "(no collective or sharded path exists in this library).", file=sys.stderr)
        return 2

    import torch
    from paper_2512_22195_amd import binding as mk
    from workload import CONFIGS, normal, question_lengths, retrieved_chunks

    shape = CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    tdt = shape.torch_dtype
    B, nl, Hq, Hkv, D, Hd = shape.batch, shape.n_layers, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.hidden
    L = shape.chunk_tokens
    q_lens = question_lengths(shape)
    retrieved = retrieved_chunks(shape)
    chunk_ids = sorted({c for r in retrieved for c in r})
    max_tail = (max(q_lens) + shape.decode_steps + 7) // 8 * 8
    steps_dec = shape.decode_steps

    cfg = mk.make_config(nl, Hq, Hkv, D, Hd, shape.dtype, shape.rope_base, max_batch=B,
                         max_pages=shape.n_chunks, max_tail_tokens=max_tail, decode_units=args.units,
                         decode_variant=args.variant)
    ctx = mk.Context(cfg, device=dev)
    cs = ctx.compute_stream
    vs = shape.value_scale

    # ---------------------------------------------------------------- synthetic inputs -----
    with torch.cuda.stream(cs):
        slots = {cid: normal((shape.name, "blob", cid), (nl, 2, Hkv, L, D), vs, tdt, dev) for cid in chunk_ids}
        w = normal((shape.name, "w"), (nl, 2, Hkv * D, Hd), vs, tdt, dev)
        total_q = sum(q_lens)
        x_q = normal((shape.name, "x_q"), (nl, total_q, Hd), vs, tdt, dev)
        x_dec = normal((shape.name, "x_dec"), (nl, B, Hd), vs, tdt, dev)      # reused every step
        q_pre = normal((shape.name, "q_pre"), (nl, total_q, Hq, D), vs, tdt, dev)
        q_dec = normal((shape.name, "q_dec"), (nl, B, Hq, D), vs, tdt, dev)
        o_pre = torch.empty_like(q_pre)
        o_dec = torch.empty_like(q_dec)
        tail = ctx.new_tail()
        table = ctx.new_table()
        pages = [[(slots[cid], L) for cid in r] for r in retrieved]
    cs.synchronize()

    def prefill_phase():
        ctx.assemble(pages, q_lens, table)
        for l in range(nl):
            ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
            ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])

    # does matkv_decode_step run as one kernel here?  (bf16, head_dim 128, hidden % 4096, default shape)
    fused_kernel = (not args.unfused and shape.dtype == "bf16" and D == 128 and (Hd % 4096 == 0 or Hd % 3072 == 0)
                    and args.variant == 0 and B <= 4 and Hq // Hkv <= 4)

    # one decode step of all layers, recorded once, replayed for every step
    with torch.cuda.stream(cs):
        ctx.assemble(pages, q_lens, table)
        ctx.graph_begin()
        ctx.advance(table, 1)
        for l in range(nl):
            if args.unfused:
                ctx.materialize_tail(x_dec[l], w[l, 0], w[l, 1], table, 1, tail[l, 0], tail[l, 1])
                ctx.decode_attn(l, q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
            else:
                ctx.decode_step(l, x_dec[l], w[l, 0], w[l, 1], q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
        g_step = ctx.graph_end()
        # the dominant kernel alone, every layer, tail length fixed: the fused step (projection
        # of the new token + decode attention), or the attention launch when run unfused
        ctx.graph_begin()
        for l in range(nl):
            if fused_kernel:
                ctx.decode_step(l, x_dec[l], w[l, 0], w[l, 1], q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
            else:
                ctx.decode_attn(l, q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
        g_attn = ctx.graph_end()
        ctx.graph_begin()
        for l in range(nl):
            ctx.decode_attn(l, q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
        g_attn_only = ctx.graph_end()

    def one_pass():
        prefill_phase()
        for _ in range(steps_dec):
            ctx.graph_launch(g_step)

    ev = lambda: torch.cuda.Event(enable_timing=True)
    if args.roofline_only:
        args.steps, args.warmup, args.no_cpu, args.no_load = 0, 0, True, True
        print("bench: roofline-only run", file=sys.stderr, flush=True)
    with torch.cuda.stream(cs):
        for _ in range(args.warmup):
            one_pass()
        cs.synchronize()
        torch.cuda.synchronize()
        e0, e1, e2 = [], [], []
        t_wall0 = time.perf_counter()
        for _ in range(args.steps):
            a, b, c = ev(), ev(), ev()
            a.record(cs)
            prefill_phase()
            b.record(cs)
            for _ in range(steps_dec):
                ctx.graph_launch(g_step)
            c.record(cs)
            e0.append(a); e1.append(b); e2.append(c)
        cs.synchronize()
        torch.cuda.synchronize()
        t_wall = time.perf_counter() - t_wall0
    n_t = max(args.steps, 1)
    ms_prefill = sum(a.elapsed_time(b) for a, b in zip(e0, e1)) / n_t
    ms_decode = sum(b.elapsed_time(c) for b, c in zip(e1, e2)) / n_t
    ms_step = max(t_wall * 1e3 / n_t, 1e-9)
    tokens_per_s = B * steps_dec / (ms_step * 1e-3)

    # ------------------------------------------------- roofline of the dominant kernel (D) ---
    # decode attention alone, all layers back to back (working set = every layer's KV, far
    # beyond the last-level cache), tail at its mid-run length
    mid_tail = [q + steps_dec // 2 for q in q_lens]
    with torch.cuda.stream(cs):
        ctx.assemble(pages, q_lens, table)
        ctx.advance(table, steps_dec // 2)
        def attn_all_layers():
            if args.roofline_only:          # eager launches: one dispatch per layer, no graph
                for l in range(nl):
                    if fused_kernel:
                        ctx.decode_step(l, x_dec[l], w[l, 0], w[l, 1], q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
                    else:
                        ctx.decode_attn(l, q_dec[l], table, tail[l, 0], tail[l, 1], o_dec[l])
            else:
                ctx.graph_launch(g_attn)
        for _ in range(1 if args.roofline_only else 3):
            attn_all_layers()
        a, b = ev(), ev()
        a.record(cs)
        for _ in range(args.decode_only_reps):
            attn_all_layers()
        b.record(cs)
        cs.synchronize()
        if args.roofline_only:
            print("bench: decode-attention leg done", file=sys.stderr, flush=True)
    us_per_launch = a.elapsed_time(b) * 1e3 / (args.decode_only_reps * nl)
    kv_tok_bytes = shape.kv_bytes_per_token_layer()
    n_ctx = [sum(L for _ in r) for r in retrieved]
    attn_bytes = sum((n + t) * kv_tok_bytes for n, t in zip(n_ctx, mid_tail)) + 2 * B * Hq * D * shape.elem_bytes
    proj_bytes = (2 * Hkv * D * Hd + B * Hd) * shape.elem_bytes       # W_k, W_v once, the hidden rows
    bytes_per_launch = attn_bytes + (proj_bytes if fused_kernel else 0)
    achieved = bytes_per_launch / (us_per_launch * 1e-6) / 1e9
    kname = "attn_rows_kernel" if 0 < args.variant < 9000 or shape.dtype != "bf16" or D != 128 else "attn_mfma_kernel"
    entry = "matkv_decode_step" if fused_kernel else "matkv_decode_attn"
    # the attention launch on its own, for comparison with the fused step
    attn_only = None
    if fused_kernel and not args.roofline_only:
        with torch.cuda.stream(cs):
            ctx.graph_launch(g_attn_only)
            c, d = ev(), ev()
            c.record(cs)
            for _ in range(args.decode_only_reps):
                ctx.graph_launch(g_attn_only)
            d.record(cs)
            cs.synchronize()
        us_attn = c.elapsed_time(d) * 1e3 / (args.decode_only_reps * nl)
        attn_only = {"us_per_launch": round(us_attn, 3), "bytes_per_launch": attn_bytes,
                     "GBps": round(attn_bytes / us_attn / 1e3, 1),
                     "frac_of_hbm_peak": round(attn_bytes / us_attn / 1e3 / HBM_PEAK_GBPS, 4)}
    # HBM bytes per launch from the committed rocprofv3 --pmc summary of this same workload
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"{'decode_step' if fused_kernel else 'decode_attn'}_config{args.config}_hbm_traffic.txt")
    if args.units == 0 and args.variant == 0 and os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
    # practical ceiling: a plain 16-byte-load read of the same number of bytes per launch, walking
    # through the same blobs (one launch per layer's worth of bytes), captured and replayed alike
    read_ceiling = None
    if not args.roofline_only:
        with torch.cuda.stream(cs):
            flat = [slots[cid].view(torch.uint8).reshape(-1) for cid in chunk_ids]
            per = min(bytes_per_launch, flat[0].numel()) // 16 * 16
            regions = max(flat[0].numel() // per, 1)            # whole launches' worth per blob
            ctx.graph_begin()
            for l in range(nl):
                f = flat[l % len(flat)]
                off = ((l // len(flat)) % regions) * per
                ctx.probe_read(f[off:off + per], per)
            g_read = ctx.graph_end()
            ctx.graph_launch(g_read)
            c, d = ev(), ev()
            c.record(cs)
            for _ in range(5):
                ctx.graph_launch(g_read)
            d.record(cs)
            cs.synchronize()
            ctx.graph_destroy(g_read)
        us_read = c.elapsed_time(d) * 1e3 / (5 * nl)
        read_ceiling = {"bytes_per_launch": per, "us_per_launch": round(us_read, 3), "GBps": round(per / us_read / 1e3, 1)}
    roofline = {"bound": "hbm", "kernel": f"{kname} ({entry})",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "bytes_per_launch": bytes_per_launch, "us_per_launch": round(us_per_launch, 3),
                "plain_read_probe": read_ceiling, "decode_attn_alone": attn_only}

    # ------------------------------- other kernels: rates against their own rooflines -----------
    other = None
    if not args.roofline_only or args.with_others:
        with torch.cuda.stream(cs):
            # chunk materialization (ingest time in the paper; here: one chunk, every layer)
            x_chunk = normal((shape.name, "x_chunk"), (L, Hd), vs, tdt, dev)
            blob = torch.empty((nl, 2, Hkv, L, D), dtype=tdt, device=dev)
            for l in range(min(nl, 4)):
                ctx.materialize(x_chunk, w[l, 0], w[l, 1], L, 0, blob[l, 0], blob[l, 1], L)
            a, b = ev(), ev()
            a.record(cs)
            for l in range(nl):
                ctx.materialize(x_chunk, w[l, 0], w[l, 1], L, 0, blob[l, 0], blob[l, 1], L)
            b.record(cs)
            # the chunk's own causal attention over the K/V just materialized (ingest time too)
            q_chunk = normal((shape.name, "q_chunk"), (L, Hq, D), vs, tdt, dev)
            o_chunk = torch.empty_like(q_chunk)
            h0, h1 = ev(), ev()
            try:
                for l in range(min(nl, 4)):
                    ctx.chunk_attn(l, q_chunk, blob, L, o_chunk)
                h0.record(cs)
                for l in range(nl):
                    ctx.chunk_attn(l, q_chunk, blob, L, o_chunk)
                h1.record(cs)
                chunk_attn_ok = True
            except mk.MatKVError:        # the row-per-workgroup kernel needs a workspace sized for the chunk's rows
                chunk_attn_ok = False
            # question prefill attention alone
            ctx.assemble(pages, q_lens, table)
            for l in range(min(nl, 4)):
                ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
            c, d = ev(), ev()
            c.record(cs)
            for l in range(nl):
                ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
            d.record(cs)
            # question projection alone (the rows of the whole batch's questions)
            for l in range(min(nl, 4)):
                ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
            g0, g1 = ev(), ev()
            g0.record(cs)
            for l in range(nl):
                ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
            g1.record(cs)
            # decode-token projection alone
            for l in range(min(nl, 4)):
                ctx.materialize_tail(x_dec[l], w[l, 0], w[l, 1], table, 1, tail[l, 0], tail[l, 1])
            e, f = ev(), ev()
            e.record(cs)
            for l in range(nl):
                ctx.materialize_tail(x_dec[l], w[l, 0], w[l, 1], table, 1, tail[l, 0], tail[l, 1])
            f.record(cs)
            cs.synchronize()
        us_mat = a.elapsed_time(b) * 1e3 / nl
        us_pre = c.elapsed_time(d) * 1e3 / nl
        us_gemv = e.elapsed_time(f) * 1e3 / nl
        us_matq = g0.elapsed_time(g1) * 1e3 / nl
        us_chunk = h0.elapsed_time(h1) * 1e3 / nl if chunk_attn_ok else float("nan")
        fl_chunk = 4.0 * D * Hq * L * (L + 1) / 2
        fl_matq = 2.0 * total_q * Hd * 2 * Hkv * D
        fl_mat = 2.0 * L * Hd * 2 * Hkv * D
        fl_pre = sum(4.0 * q * (n + (q + 1) / 2) * D * Hq for q, n in zip(q_lens, n_ctx))
        by_gemv = 2 * Hkv * D * Hd * shape.elem_bytes + B * Hd * shape.elem_bytes
        mfma_peak = 2500.0 if shape.dtype == "bf16" else 157.3
        other = {
            "materialize_chunk": {"tokens": L, "us_per_layer": round(us_mat, 2), "TFLOPs": round(fl_mat / us_mat / 1e6, 1),
                                  "frac_of_mfma_peak": round(fl_mat / us_mat / 1e6 / mfma_peak, 4)},
            "chunk_attn": ({"tokens": L, "us_per_layer": round(us_chunk, 2), "TFLOPs": round(fl_chunk / us_chunk / 1e6, 1),
                            "frac_of_mfma_peak": round(fl_chunk / us_chunk / 1e6 / mfma_peak, 4)} if chunk_attn_ok else None),
            "materialize_question": {"rows": total_q, "us_per_layer": round(us_matq, 2), "TFLOPs": round(fl_matq / us_matq / 1e6, 1),
                                     "frac_of_mfma_peak": round(fl_matq / us_matq / 1e6 / mfma_peak, 4)},
            "prefill_attn": {"us_per_layer": round(us_pre, 2), "TFLOPs": round(fl_pre / us_pre / 1e6, 1),
                             "frac_of_mfma_peak": round(fl_pre / us_pre / 1e6 / mfma_peak, 4)},
            "materialize_decode_token": {"us_per_layer": round(us_gemv, 2), "GBps": round(by_gemv / us_gemv / 1e3, 1),
                                         "frac_of_hbm_peak": round(by_gemv / us_gemv / 1e3 / HBM_PEAK_GBPS, 4)},
        }
        del x_chunk, blob, q_chunk, o_chunk

    if args.calib_copy:
        with torch.cuda.stream(cs):
            src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
            dstc = torch.empty_like(src)
            dstc.copy_(src)
            cs.synchronize()
            del src, dstc

    # ---------------------------------------------------------- KV load (never in value) -----
    kv_load = None
    if not args.no_load:
        inst_chunks = retrieved[0]
        nbytes = mk.blob_bytes(cfg, L)
        host = [torch.empty(nbytes, dtype=torch.uint8).pin_memory() for _ in inst_chunks]
        for h, cid in zip(host, inst_chunks):
            h.copy_(slots[cid].view(torch.uint8).reshape(-1))
        dst = [ctx.new_slot(L) for _ in inst_chunks]
        torch.cuda.synchronize()
        best = None
        for rep in range(3):
            t0 = time.perf_counter()
            tickets = [ctx.load(h, L, d) for h, d in zip(host, dst)]
            ctx.sync(tickets[-1])
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        ok = all(torch.equal(d.cpu(), h) for d, h in zip(dst[:1], host[:1]))
        kv_load = {"GBps": round(len(host) * nbytes / best / 1e9, 2), "ms_per_instance": round(best * 1e3, 3),
                   "bytes": len(host) * nbytes, "chunks": len(host), "byte_exact": bool(ok)}

        # ---- the same blobs from a file (paper Section IV: KVs stored as raw bytes on flash):
        # written once, dropped from the page cache where possible, read with O_DIRECT if the
        # filesystem allows it, through the library's pinned bounce buffers
        # ---- pipelined stream (BASELINE config 5 at this shape): the next instance's blobs are
        # loaded on the side stream into the other slot set while this instance runs its
        # prefill and decode steps.  Host blobs: a ring of two distinct instance sets.
        overlap = None
        if args.stream > 0 and B == 1:
            n_inst = args.stream
            host2 = [torch.empty(nbytes, dtype=torch.uint8).pin_memory() for _ in inst_chunks]
            for h2, h in zip(host2, reversed(host)):
                h2.copy_(h)
            host_sets = [host, host2]
            slot_sets = [dst, [ctx.new_slot(L) for _ in inst_chunks]]

            def enqueue_load(i):
                return [ctx.load(h, L, d) for h, d in zip(host_sets[i % 2], slot_sets[i % 2])]

            def enqueue_compute(i, tickets):
                for t in tickets:
                    ctx.wait(t)
                ctx.assemble([[(d, L) for d in slot_sets[i % 2]]], q_lens, table)
                for l in range(nl):
                    ctx.materialize_tail(x_q[l], w[l, 0], w[l, 1], table, -1, tail[l, 0], tail[l, 1])
                    ctx.prefill_attn(l, q_pre[l], table, tail[l, 0], tail[l, 1], o_pre[l])
                for _ in range(steps_dec):
                    ctx.graph_launch(g_step)

            def run_stream(load_fn, n):
                with torch.cuda.stream(cs):
                    torch.cuda.synchronize()
                    # serial: load, wait for it, compute, wait for it
                    t0 = time.perf_counter()
                    for i in range(n):
                        tk = load_fn(i)
                        ctx.sync(tk[-1])
                        enqueue_compute(i, tk)
                        cs.synchronize()
                    t_ser = (time.perf_counter() - t0) / n
                    # pipelined: the compute of i is enqueued, then the load of i+1 is issued
                    tk = load_fn(0)                   # steady state: the first load is already there
                    ctx.sync(tk[-1])
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for i in range(n):
                        enqueue_compute(i, tk)
                        tk = load_fn(i + 1) if i + 1 < n else None
                    cs.synchronize()
                    torch.cuda.synchronize()
                    return t_ser, (time.perf_counter() - t0) / n

            t_serial, t_pipe = run_stream(enqueue_load, n_inst)
            t_load = best
            t_comp = ms_step * 1e-3
            overlap = {"instances": n_inst, "instances_per_s": round(1.0 / t_pipe, 3),
                       "ms_per_instance_pipelined": round(t_pipe * 1e3, 3),
                       "ms_per_instance_serial": round(t_serial * 1e3, 3),
                       "ms_load": round(t_load * 1e3, 3), "ms_compute": round(t_comp * 1e3, 3),
                       "overlap_frac": round(max(0.0, min(1.0, (t_serial - t_pipe) / min(t_load, t_comp))), 3)}
            del host2

            # the same stream with every instance's blobs read from the file (matkv_load_file
            # blocks the host for the read while the previous instance's work runs on the GPU)
            def file_stream(fd):
                n = min(n_inst, 3)
                ts, tp = run_stream(lambda i: [ctx.load_file(fd, j * nbytes, nbytes, L, d)
                                                for j, d in enumerate(slot_sets[i % 2])], n)
                return {"instances": n, "instances_per_s": round(1.0 / tp, 3),
                        "ms_per_instance_pipelined": round(tp * 1e3, 3), "ms_per_instance_serial": round(ts * 1e3, 3)}
            kv_load["from_file"] = file_load_leg(ctx, host, dst, L, nbytes, with_fd=file_stream)
        else:
            kv_load["from_file"] = file_load_leg(ctx, host, dst, L, nbytes)
        kv_load["pipelined_stream"] = overlap
        del host, dst

    # ----------------------------------- decode attention at a bandwidth-bound launch size ---
    if not args.roofline_only and not args.no_batch16 and shape.dtype == "bf16":
        try:
            roofline["decode_attn_batch16"] = batch16_decode_leg()
        except torch.cuda.OutOfMemoryError:
            roofline["decode_attn_batch16"] = None

    # ------------------------------------------- the same workload over compressed blobs -----
    compressed = None
    if not args.roofline_only and not args.no_compressed and shape.dtype == "bf16" and D == 128 and args.variant == 0:
        print("bench: compressed-blob leg", file=sys.stderr, flush=True)
        compressed = compressed_leg(args.config)
        if not args.no_batch16:
            compressed["decode_attn_batch16"] = batch16_decode_leg(compressed=True)

    # ------------------------------------------------------------------------ cpu_baseline ---
    cpu = None
    if not args.no_cpu:
        import numpy as np
        import oracle
        from workload import to_f64
        # bounded sample of the same workload: instance 0, layers {0, nl/2, nl-1}: the K/V
        # projection of one new token and its decode attention at the mid-run tail length
        b0 = 0
        layers = sorted({0, nl // 2, nl - 1})
        cs.synchronize()
        chunks = {l: [(to_f64(slots[cid][l, 0]), to_f64(slots[cid][l, 1])) for cid in retrieved[b0]] for l in layers}
        n_t = mid_tail[b0]
        tails = {l: (to_f64(tail[l, 0, b0, :, :n_t]), to_f64(tail[l, 1, b0, :, :n_t])) for l in layers}
        wk = {l: (to_f64(w[l, 0]), to_f64(w[l, 1])) for l in layers}
        xs = {l: to_f64(x_dec[l, b0:b0 + 1]) for l in layers}
        qs = {l: to_f64(q_dec[l, b0]) for l in layers}
        reps, t_cpu = 0, 0.0
        t_begin = time.perf_counter()
        while t_cpu < 12.0 and reps < 400:
            for l in layers:
                t0 = time.perf_counter()
                oracle.materialize(xs[l], wk[l][0], wk[l][1], Hkv, D, float(n_ctx[b0] + n_t - 1), shape.rope_base)
                oracle.decode_attn(qs[l], chunks[l], tails[l][0], tails[l][1])
                t_cpu += time.perf_counter() - t0
            reps += 1
        per_layer_step = t_cpu / (reps * len(layers))
        cpu_tok_s = 1.0 / (per_layer_step * nl)          # one instance: B tokens need B times this
        cpu = {"value": round(cpu_tok_s / 1.0, 4), "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"instance 0, layers {layers}, decode token at tail length {n_t}: K/V projection + decode "
                         f"attention, {reps} repetitions, {t_cpu:.1f} s of oracle time; tokens/s extrapolated "
                         f"linearly to {nl} layers (prefill not included)",
               "seconds_per_layer_step": round(per_layer_step, 5)}

    out = {
        "metric": "tokens/s over loaded KV (decode-attn HBM GB/s and % of peak in roofline; KV load GB/s in kv_load)",
        "value": round(tokens_per_s, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"BASELINE config {args.config}: {shape.name}, {B} instance(s) x {shape.n_chunks} chunks x "
                               f"{L} tokens, {nl} layers, Hq {Hq} / Hkv {Hkv} / D {D}, question {q_lens if B > 1 else q_lens[0]} "
                               f"tokens, {steps_dec} decode steps",
                   "batch": B, "cached_tokens": n_ctx if B > 1 else n_ctx[0], "decode_units": args.units, "decode_variant": args.variant},
        "phases_ms": {"assemble+materialize+prefill": round(ms_prefill, 3), "decode": round(ms_decode, 3),
                      "decode_us_per_layer_step": round(ms_decode * 1e3 / (steps_dec * nl), 3)},
        "roofline": roofline, "other_kernels": other, "kv_load": kv_load, "compressed_kv": compressed,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    ctx.graph_destroy(g_step)
    ctx.graph_destroy(g_attn)
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
