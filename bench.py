#!/usr/bin/env python3
"""Benchmark of the MatKV hot path on one MI355X.

A "step" is one pass of the whole path over one RAG instance batch with its chunk KVs already
resident in HBM: cache assembly, K/V materialization of the question tokens + prefill attention
for every layer, then every decode step (K/V materialization of the new token + decode
attention for every layer, replayed from one captured graph).  ``value`` is generated tokens
per second over that pass on the headline workload (the largest single-GPU configuration:
70B layer shape, batch 4, 20 x 1000 cached tokens each, 80 layers, 256 decode steps).  Beside
it: the decode-attention kernel's achieved HBM bandwidth (``roofline``), the same whole pass and
roofline on the 8B-shape configurations (``configs``), the pinned-host-to-HBM load rate and the
pipelined stream of instances (``kv_load``, never part of ``value``), and the fp64 oracle timed
on the host cores (``cpu_baseline``).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--subs 2,3] [--stream 64]
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4, help="BASELINE.json config number (1-based) of the headline workload")
    ap.add_argument("--subs", type=str, default="2,3", help="other configs run as whole passes beside the headline ('' = none)")
    ap.add_argument("--units", type=int, default=0, help="decode workgroups per (instance, KV head); 0 = library's choice")
    ap.add_argument("--variant", type=int, default=0, help="decode kernel shape; 0 = default")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-load", action="store_true", help="skip the kv_load leg (loads, file tier, pipelined stream)")
    ap.add_argument("--no-compressed", action="store_true", help="skip the leg with the chunks held as compressed blobs")
    ap.add_argument("--no-others", action="store_true", help="skip the other kernels' leg")
    ap.add_argument("--with-others", action="store_true",
                    help="with --roofline-only: also run the other kernels' leg (few eager launches each)")
    ap.add_argument("--unfused", action="store_true",
                    help="decode steps as matkv_materialize_tail + matkv_decode_attn instead of matkv_decode_step")
    ap.add_argument("--decode-only-reps", type=int, default=10)
    ap.add_argument("--roofline-only", action="store_true",
                    help="only the decode-kernel leg of the headline config, launched eagerly (short run for rocprofv3)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device copy (reference for scaling rocprofv3 byte counters)")
    ap.add_argument("--stream", type=int, default=64,
                    help="instances of the pipelined leg (next instance loads while this one decodes); 0 = skip")
    return ap.parse_args()


def log(msg):
    print(f"bench: {msg}", file=sys.stderr, flush=True)


def ev():
    import torch
    return torch.cuda.Event(enable_timing=True)


_STREAMS = None


def streams():
    """One compute stream and one load stream for every context of this run.  The box gives a
    process four hardware queues and the runtime deals streams onto them in creation order: with
    a fresh pair of streams per context, a later context's two streams can land on one queue,
    and its loads then run behind its kernels instead of beside them."""
    global _STREAMS
    if _STREAMS is None:
        import torch
        _STREAMS = (torch.cuda.Stream(device="cuda:0"), torch.cuda.Stream(device="cuda:0"))
    return _STREAMS


class Workload:
    """One BASELINE configuration resident on the GPU: context, synthetic inputs, captured graphs."""

    def __init__(self, config_id, units=0, variant=0, unfused=False):
        import torch
        from paper_2512_22195_amd import binding as mk
        from workload import CONFIGS, normal, question_lengths, retrieved_chunks
        self.mk, self.torch = mk, torch
        self.config_id = config_id
        s = self.shape = CONFIGS[config_id]
        self.dev = dev = torch.device("cuda:0")
        self.B, self.nl, self.Hq, self.Hkv, self.D, self.Hd, self.L = (s.batch, s.n_layers, s.n_q_heads, s.n_kv_heads,
                                                                       s.head_dim, s.hidden, s.chunk_tokens)
        self.q_lens = question_lengths(s)
        self.retrieved = retrieved_chunks(s)
        self.chunk_ids = sorted({c for r in self.retrieved for c in r})
        self.max_tail = (max(self.q_lens) + s.decode_steps + 7) // 8 * 8
        self.steps_dec = s.decode_steps
        self.units, self.variant, self.unfused = units, variant, unfused
        self.cfg = mk.make_config(self.nl, self.Hq, self.Hkv, self.D, self.Hd, s.dtype, s.rope_base, max_batch=self.B,
                                  max_pages=s.n_chunks, max_tail_tokens=self.max_tail, decode_units=units,
                                  decode_variant=variant)
        self.ctx = ctx = mk.Context(self.cfg, *streams(), device=dev)
        self.cs = cs = ctx.compute_stream
        tdt, vs = s.torch_dtype, s.value_scale
        self.blob_bytes = mk.blob_bytes(self.cfg, self.L)
        with torch.cuda.stream(cs):
            # every distinct chunk's blob, back to back in one allocation (the read probe walks it)
            self.pool = torch.empty(len(self.chunk_ids) * self.blob_bytes, dtype=torch.uint8, device=dev)
            self.slots = {}
            for i, cid in enumerate(self.chunk_ids):
                view = self.pool[i * self.blob_bytes:(i + 1) * self.blob_bytes].view(tdt).view(self.nl, 2, self.Hkv, self.L, self.D)
                g = torch.Generator(device=dev)
                from workload import seed_for
                g.manual_seed(seed_for(s.name, "blob", cid))
                view.normal_(0.0, float(vs), generator=g)
                self.slots[cid] = view
            self.w = normal((s.name, "w"), (self.nl, 2, self.Hkv * self.D, self.Hd), vs, tdt, dev)
            self.total_q = sum(self.q_lens)
            self.x_q = normal((s.name, "x_q"), (self.nl, self.total_q, self.Hd), vs, tdt, dev)
            self.x_dec = normal((s.name, "x_dec"), (self.nl, self.B, self.Hd), vs, tdt, dev)      # reused every step
            self.q_pre = normal((s.name, "q_pre"), (self.nl, self.total_q, self.Hq, self.D), vs, tdt, dev)
            self.q_dec = normal((s.name, "q_dec"), (self.nl, self.B, self.Hq, self.D), vs, tdt, dev)
            self.o_pre = torch.empty_like(self.q_pre)
            self.o_dec = torch.empty_like(self.q_dec)
            self.tail = ctx.new_tail()
            self.table = ctx.new_table()
            self.pages = [[(self.slots[cid], self.L) for cid in r] for r in self.retrieved]
        cs.synchronize()
        # does matkv_decode_step run as one kernel here?  (bf16, head_dim 128, hidden a multiple of
        # 4096 or 3072, default kernel shape, up to four instances, up to four query heads per KV head)
        self.fused_kernel = (not unfused and s.dtype == "bf16" and self.D == 128 and (self.Hd % 4096 == 0 or self.Hd % 3072 == 0)
                             and variant == 0 and self.B <= 4 and self.Hq // self.Hkv <= 4)
        self.n_ctx = [sum(self.L for _ in r) for r in self.retrieved]
        self.mid_tail = [q + self.steps_dec // 2 for q in self.q_lens]
        self.graphs = []
        self._record_graphs()

    def describe(self):
        s = self.shape
        return (f"BASELINE config {self.config_id}: {s.name}, {self.B} instance(s) x {s.n_chunks} chunks x {self.L} tokens, "
                f"{self.nl} layers, Hq {self.Hq} / Hkv {self.Hkv} / D {self.D}, hidden {self.Hd}, question "
                f"{self.q_lens if self.B > 1 else self.q_lens[0]} tokens, {self.steps_dec} decode steps, "
                f"{len(self.chunk_ids)} distinct chunks resident ({len(self.chunk_ids) * self.blob_bytes / 1e9:.1f} GB)")

    # -- the path ---------------------------------------------------------------------------
    def decode_layer(self, l, fused):
        c, t = self.ctx, self.tail
        if fused:
            c.decode_step(l, self.x_dec[l], self.w[l, 0], self.w[l, 1], self.q_dec[l], self.table, t[l, 0], t[l, 1], self.o_dec[l])
        else:
            c.materialize_tail(self.x_dec[l], self.w[l, 0], self.w[l, 1], self.table, 1, t[l, 0], t[l, 1])
            c.decode_attn(l, self.q_dec[l], self.table, t[l, 0], t[l, 1], self.o_dec[l])

    def dominant_kernel_layer(self, l):
        """The dominant kernel alone: the fused step where it is one kernel, else the attention launch."""
        c, t = self.ctx, self.tail
        if self.fused_kernel:
            c.decode_step(l, self.x_dec[l], self.w[l, 0], self.w[l, 1], self.q_dec[l], self.table, t[l, 0], t[l, 1], self.o_dec[l])
        else:
            c.decode_attn(l, self.q_dec[l], self.table, t[l, 0], t[l, 1], self.o_dec[l])

    def _graph(self, body):
        self.ctx.graph_begin()
        body()
        g = self.ctx.graph_end()
        self.graphs.append(g)
        return g

    def _record_graphs(self):
        torch, ctx = self.torch, self.ctx
        with torch.cuda.stream(self.cs):
            ctx.assemble(self.pages, self.q_lens, self.table)

            def step():
                ctx.advance(self.table, 1)
                for l in range(self.nl):
                    self.decode_layer(l, fused=not self.unfused)
            self.g_step = self._graph(step)
            self.g_kernel = self._graph(lambda: [self.dominant_kernel_layer(l) for l in range(self.nl)])
            self.g_attn_only = None
            if self.fused_kernel:
                t = self.tail
                self.g_attn_only = self._graph(lambda: [ctx.decode_attn(l, self.q_dec[l], self.table, t[l, 0], t[l, 1], self.o_dec[l])
                                                        for l in range(self.nl)])

    def prefill_phase(self, pages=None):
        ctx, t = self.ctx, self.tail
        ctx.assemble(pages or self.pages, self.q_lens, self.table)
        for l in range(self.nl):
            ctx.materialize_tail(self.x_q[l], self.w[l, 0], self.w[l, 1], self.table, -1, t[l, 0], t[l, 1])
            ctx.prefill_attn(l, self.q_pre[l], self.table, t[l, 0], t[l, 1], self.o_pre[l])

    def one_pass(self, pages=None):
        self.prefill_phase(pages)
        for _ in range(self.steps_dec):
            self.ctx.graph_launch(self.g_step)

    # -- measurements -------------------------------------------------------------------------
    def time_passes(self, steps, warmup):
        torch, cs = self.torch, self.cs
        with torch.cuda.stream(cs):
            for _ in range(warmup):
                self.one_pass()
            cs.synchronize()
            torch.cuda.synchronize()
            e0, e1, e2 = [], [], []
            t_wall0 = time.perf_counter()
            for _ in range(steps):
                a, b, c = ev(), ev(), ev()
                a.record(cs)
                self.prefill_phase()
                b.record(cs)
                for _ in range(self.steps_dec):
                    self.ctx.graph_launch(self.g_step)
                c.record(cs)
                e0.append(a); e1.append(b); e2.append(c)
            cs.synchronize()
            torch.cuda.synchronize()
            t_wall = time.perf_counter() - t_wall0
        n_t = max(steps, 1)
        ms_prefill = sum(a.elapsed_time(b) for a, b in zip(e0, e1)) / n_t
        ms_decode = sum(b.elapsed_time(c) for b, c in zip(e1, e2)) / n_t
        ms_step = max(t_wall * 1e3 / n_t, 1e-9)
        return {"tokens_per_s": round(self.B * self.steps_dec / (ms_step * 1e-3), 2), "ms_per_step": round(ms_step, 3),
                "steps": steps, "warmup": warmup,
                "phases_ms": {"assemble+materialize+prefill": round(ms_prefill, 3), "decode": round(ms_decode, 3),
                              "decode_us_per_layer_step": round(ms_decode * 1e3 / (self.steps_dec * self.nl), 3)}}

    def attn_bytes(self):
        s = self.shape
        return (sum((n + t) * s.kv_bytes_per_token_layer() for n, t in zip(self.n_ctx, self.mid_tail))
                + 2 * self.B * self.Hq * self.D * s.elem_bytes)

    def proj_bytes(self):
        return (2 * self.Hkv * self.D * self.Hd + self.B * self.Hd) * self.shape.elem_bytes     # W_k, W_v once, the hidden rows

    def roofline(self, reps, eager=False, probe=True):
        """The dominant kernel alone, every layer back to back (working set = every layer's KV,
        far beyond the last-level cache), tails at their mid-run length; HIP events on the
        compute stream.  eager: one dispatch per layer instead of a graph (for rocprofv3)."""
        torch, ctx, cs, nl = self.torch, self.ctx, self.cs, self.nl
        s = self.shape
        with torch.cuda.stream(cs):
            ctx.assemble(self.pages, self.q_lens, self.table)
            ctx.advance(self.table, self.steps_dec // 2)

            def all_layers():
                if eager:
                    for l in range(nl):
                        self.dominant_kernel_layer(l)
                else:
                    ctx.graph_launch(self.g_kernel)
            for _ in range(1 if eager else 3):
                all_layers()
            a, b = ev(), ev()
            a.record(cs)
            for _ in range(reps):
                all_layers()
            b.record(cs)
            cs.synchronize()
        us = a.elapsed_time(b) * 1e3 / (reps * nl)
        attn_b = self.attn_bytes()
        bytes_per_launch = attn_b + (self.proj_bytes() if self.fused_kernel else 0)
        achieved = bytes_per_launch / us / 1e3
        kname = "attn_rows_kernel" if 0 < self.variant < 9000 or s.dtype != "bf16" or self.D != 128 else "attn_mfma_kernel"
        entry = "matkv_decode_step" if self.fused_kernel else "matkv_decode_attn"
        attn_only = None
        if self.g_attn_only is not None and not eager:
            with torch.cuda.stream(cs):
                ctx.graph_launch(self.g_attn_only)
                c, d = ev(), ev()
                c.record(cs)
                for _ in range(reps):
                    ctx.graph_launch(self.g_attn_only)
                d.record(cs)
                cs.synchronize()
            us_attn = c.elapsed_time(d) * 1e3 / (reps * nl)
            attn_only = {"us_per_launch": round(us_attn, 3), "bytes_per_launch": attn_b, "GBps": round(attn_b / us_attn / 1e3, 1),
                         "frac_of_hbm_peak": round(attn_b / us_attn / 1e3 / HBM_PEAK_GBPS, 4)}
        # HBM bytes per launch from the committed rocprofv3 --pmc summary of this same workload
        traffic = None
        tfile = os.path.join(ROOT, "profiles", f"{'decode_step' if self.fused_kernel else 'decode_attn'}_config{self.config_id}_hbm_traffic.txt")
        if self.units == 0 and self.variant == 0 and os.path.exists(tfile):
            for line in open(tfile):
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = int(line.split(":")[1])
        # practical ceiling: a plain 16-byte-load read of the same number of bytes per launch,
        # walking through the same blobs (a different region per layer), captured and replayed alike
        read_ceiling = None
        if probe and not eager:
            with torch.cuda.stream(cs):
                per = min(bytes_per_launch, self.pool.numel()) // 16 * 16
                regions = max(self.pool.numel() // per, 1)
                ctx.graph_begin()
                for l in range(nl):
                    off = (l % regions) * per
                    ctx.probe_read(self.pool[off:off + per], per)
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
            read_ceiling = {"bytes_per_launch": per, "us_per_launch": round(us_read, 3), "GBps": round(per / us_read / 1e3, 1),
                            "frac_of_hbm_peak": round(per / us_read / 1e3 / HBM_PEAK_GBPS, 4)}
        return {"bound": "hbm", "kernel": f"{kname} ({entry})", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
                "bytes_per_launch": bytes_per_launch, "us_per_launch": round(us, 3),
                "plain_read_probe": read_ceiling, "decode_attn_alone": attn_only}

    def other_kernels(self):
        """Chunk materialization, the chunk's own attention, question prefill attention, question
        and decode-token projection, each alone, one launch per layer."""
        torch, ctx, cs, nl, s = self.torch, self.ctx, self.cs, self.nl, self.shape
        from workload import normal
        tdt, vs, L = s.torch_dtype, s.value_scale, self.L
        t = self.tail

        def timed(fn, warm=4):
            for l in range(min(nl, warm)):
                fn(l)
            a, b = ev(), ev()
            a.record(cs)
            for l in range(nl):
                fn(l)
            b.record(cs)
            return a, b

        with torch.cuda.stream(cs):
            x_chunk = normal((s.name, "x_chunk"), (L, self.Hd), vs, tdt, self.dev)
            blob = torch.empty((nl, 2, self.Hkv, L, self.D), dtype=tdt, device=self.dev)
            m = timed(lambda l: ctx.materialize(x_chunk, self.w[l, 0], self.w[l, 1], L, 0, blob[l, 0], blob[l, 1], L))
            q_chunk = normal((s.name, "q_chunk"), (L, self.Hq, self.D), vs, tdt, self.dev)
            o_chunk = torch.empty_like(q_chunk)
            try:
                h = timed(lambda l: ctx.chunk_attn(l, q_chunk, blob, L, o_chunk))
            except self.mk.MatKVError:     # the row-per-workgroup kernel needs a workspace sized for the chunk's rows
                h = None
            # the whole materialization pass of one chunk (paper Section III-B steps 1-3): per layer the
            # K/V projection with rotary, then the chunk's own causal attention over what was just
            # written; every layer's hidden states and queries come from the caller (synthetic)
            cp = None
            if h:
                def chunk_layer(l):
                    ctx.materialize(x_chunk, self.w[l, 0], self.w[l, 1], L, 0, blob[l, 0], blob[l, 1], L)
                    ctx.chunk_attn(l, q_chunk, blob, L, o_chunk)
                cp = timed(chunk_layer)
            ctx.assemble(self.pages, self.q_lens, self.table)
            p = timed(lambda l: ctx.prefill_attn(l, self.q_pre[l], self.table, t[l, 0], t[l, 1], self.o_pre[l]))
            mq = timed(lambda l: ctx.materialize_tail(self.x_q[l], self.w[l, 0], self.w[l, 1], self.table, -1, t[l, 0], t[l, 1]))
            md = timed(lambda l: ctx.materialize_tail(self.x_dec[l], self.w[l, 0], self.w[l, 1], self.table, 1, t[l, 0], t[l, 1]))
            cs.synchronize()
        us = lambda pair: pair[0].elapsed_time(pair[1]) * 1e3 / nl
        peak = MFMA_PEAK_TFLOPS[s.dtype]
        fl_mat = 2.0 * L * self.Hd * 2 * self.Hkv * self.D
        fl_chunk = 4.0 * self.D * self.Hq * L * (L + 1) / 2
        fl_matq = 2.0 * self.total_q * self.Hd * 2 * self.Hkv * self.D
        fl_pre = sum(4.0 * q * (n + (q + 1) / 2) * self.D * self.Hq for q, n in zip(self.q_lens, self.n_ctx))
        by_w = 2 * self.Hkv * self.D * self.Hd * s.elem_bytes
        by_gemv = by_w + self.B * self.Hd * s.elem_bytes
        by_matq = by_w + self.total_q * self.Hd * s.elem_bytes + 2 * self.total_q * self.Hkv * self.D * s.elem_bytes
        by_pre = sum(n + q for q, n in zip(self.q_lens, self.n_ctx)) * s.kv_bytes_per_token_layer() + 2 * self.total_q * self.Hq * self.D * s.elem_bytes

        def mfma(flops, pair, extra=None):
            u = us(pair)
            d = {"us_per_layer": round(u, 2), "TFLOPs": round(flops / u / 1e6, 1), "frac_of_mfma_peak": round(flops / u / 1e6 / peak, 4)}
            if extra:
                d.update(extra(u))
            return d
        return {
            "materialize_chunk": dict(tokens=L, **mfma(fl_mat, m)),
            "chunk_attn": dict(tokens=L, **mfma(fl_chunk, h)) if h else None,
            "chunk_pass": {"what": "materialize + chunk_attn back to back, every layer, one chunk", "tokens": L, "layers": nl,
                           "us_per_layer": round(us(cp), 2), "ms_per_chunk": round(us(cp) * nl / 1e3, 3),
                           "chunk_tokens_per_s": round(L / (us(cp) * nl / 1e6), 1)} if cp else None,
            "materialize_question": dict(rows=self.total_q, **mfma(fl_matq, mq, lambda u: {
                "bytes": by_matq, "frac_of_hbm_peak": round(by_matq / u / 1e3 / HBM_PEAK_GBPS, 4)})),
            "prefill_attn": mfma(fl_pre, p, lambda u: {"kv_bytes": by_pre, "frac_of_hbm_peak": round(by_pre / u / 1e3 / HBM_PEAK_GBPS, 4)}),
            "materialize_decode_token": {"us_per_layer": round(us(md), 2), "GBps": round(by_gemv / us(md) / 1e3, 1),
                                         "frac_of_hbm_peak": round(by_gemv / us(md) / 1e3 / HBM_PEAK_GBPS, 4)},
        }

    def cpu_baseline(self):
        """The oracle as it stands on a bounded sample of this workload: instance 0, layers
        {0, nl/2, nl-1}: the K/V projection of one new token and its decode attention at the
        mid-run tail length, repeated for about 12 s."""
        import oracle
        from workload import to_f64
        nl, s, b0 = self.nl, self.shape, 0
        layers = sorted({0, nl // 2, nl - 1})
        self.cs.synchronize()
        chunks = {l: [(to_f64(self.slots[cid][l, 0]), to_f64(self.slots[cid][l, 1])) for cid in self.retrieved[b0]] for l in layers}
        n_t = self.mid_tail[b0]
        tails = {l: (to_f64(self.tail[l, 0, b0, :, :n_t]), to_f64(self.tail[l, 1, b0, :, :n_t])) for l in layers}
        wk = {l: (to_f64(self.w[l, 0]), to_f64(self.w[l, 1])) for l in layers}
        xs = {l: to_f64(self.x_dec[l, b0:b0 + 1]) for l in layers}
        qs = {l: to_f64(self.q_dec[l, b0]) for l in layers}
        reps, t_cpu = 0, 0.0
        while t_cpu < 12.0 and reps < 400:
            for l in layers:
                t0 = time.perf_counter()
                oracle.materialize(xs[l], wk[l][0], wk[l][1], self.Hkv, self.D, float(self.n_ctx[b0] + n_t - 1), s.rope_base)
                oracle.decode_attn(qs[l], chunks[l], tails[l][0], tails[l][1])
                t_cpu += time.perf_counter() - t0
            reps += 1
        per_layer_step = t_cpu / (reps * len(layers))
        tok_s = 1.0 / (per_layer_step * nl)       # the B instances of a step one after the other: B tokens in B times this
        return {"value": round(tok_s, 4), "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
                "sample": f"config {self.config_id}, instance 0, layers {layers}, decode token at tail length {n_t}: K/V projection "
                          f"+ decode attention, {reps} repetitions, {t_cpu:.1f} s of oracle time; tokens/s extrapolated "
                          f"linearly to {nl} layers (prefill not included)",
                "seconds_per_layer_step": round(per_layer_step, 5)}

    def close(self):
        for g in self.graphs:
            self.ctx.graph_destroy(g)
        self.graphs = []
        self.ctx.close()
        for name in ("pool", "slots", "w", "x_q", "x_dec", "q_pre", "q_dec", "o_pre", "o_dec", "tail", "table", "pages"):
            setattr(self, name, None)
        self.torch.cuda.empty_cache()


def run_config(config_id, args, steps, warmup, others=True, cpu=False):
    wl = Workload(config_id, args.units, args.variant, args.unfused)
    try:
        log(f"config {config_id}: whole passes")
        out = {"workload": wl.describe(), "batch": wl.B}
        out.update(wl.time_passes(steps, warmup))
        log(f"config {config_id}: decode kernel alone")
        out["roofline"] = wl.roofline(args.decode_only_reps)
        if others:
            log(f"config {config_id}: other kernels")
            out["other_kernels"] = wl.other_kernels()
        if cpu:
            log(f"config {config_id}: cpu_baseline (oracle)")
            out["cpu_baseline"] = wl.cpu_baseline()
        return out
    finally:
        wl.close()


# ------------------------------------------------------------------------------- loads -------
def pcie_link():
    """PCIe generation / width of the GPU as the system reports it (None where it does not)."""
    out = None
    for dev in sorted(glob.glob("/sys/class/drm/card*/device")):
        try:
            rd = lambda n: open(os.path.join(dev, n)).read().strip()
            if not rd("vendor").lower().endswith("1002"):
                continue
            speed, width = rd("current_link_speed"), rd("current_link_width")
            gts = float(speed.split()[0])
            # 128b/130b encoding from 8 GT/s on: GB/s per direction
            nominal = gts * int(width) / 8.0 * (128.0 / 130.0 if gts >= 8.0 else 0.8)
            out = {"current_link_speed": speed, "current_link_width": width, "max_link_speed": rd("max_link_speed"),
                   "max_link_width": rd("max_link_width"), "nominal_GBps_per_direction": round(nominal, 1)}
            break
        except (OSError, ValueError):
            continue
    return out


def h2d_ceiling(stream, nbytes=1 << 30):
    """Best of three plain pinned-host-to-device copies of 1 GiB on the load stream."""
    import torch
    src = torch.empty(nbytes, dtype=torch.uint8).pin_memory()
    src.fill_(3)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    best = None
    with torch.cuda.stream(stream):
        dst.copy_(src, non_blocking=True)
        stream.synchronize()
        for _ in range(3):
            a, b = ev(), ev()
            a.record(stream)
            dst.copy_(src, non_blocking=True)
            b.record(stream)
            stream.synchronize()
            ms = a.elapsed_time(b)
            best = ms if best is None else min(best, ms)
    del src, dst
    return {"bytes": nbytes, "ms": round(best, 3), "GBps": round(nbytes / best / 1e6, 2)}


def file_leg(ctx, host, dst, L, nbytes, with_fd=None):
    """The instance's blobs through a file on the box's disk: matkv_store_file writes them from
    device memory, matkv_load_file reads them back (O_DIRECT where the filesystem allows it); the
    plain-read rate of the same file (8 MiB preads into host memory) is the disk's ceiling."""
    import tempfile
    import torch
    path = os.path.join(tempfile.gettempdir(), f"matkv_bench_{os.getpid()}.bin")
    try:
        fdw = os.open(path, os.O_RDWR | os.O_CREAT | os.O_TRUNC, 0o600)
        try:
            t0 = time.perf_counter()
            for i, d in enumerate(dst):
                ctx.store_file(fdw, i * nbytes, d)
            t_store = time.perf_counter() - t0
            os.fsync(fdw)
            t_store_sync = time.perf_counter() - t0
            try:
                os.posix_fadvise(fdw, 0, 0, os.POSIX_FADV_DONTNEED)
            except OSError:
                pass
        finally:
            os.close(fdw)
        direct = True
        try:
            fd = os.open(path, os.O_RDONLY | os.O_DIRECT)
        except OSError:
            direct, fd = False, os.open(path, os.O_RDONLY)
        try:
            # plain read of the same file: the disk's rate without the library
            import mmap
            buf = mmap.mmap(-1, 8 << 20)
            t0 = time.perf_counter()
            off, total = 0, len(dst) * nbytes
            while off < total:
                n = os.preadv(fd, [buf], off)
                if n <= 0:
                    break
                off += n
            t_plain = time.perf_counter() - t0
            buf.close()
            best = None
            for rep in range(2):
                t0 = time.perf_counter()
                tickets = [ctx.load_file(fd, i * nbytes, nbytes, L, d) for i, d in enumerate(dst)]
                t_call = time.perf_counter() - t0
                for t in tickets:
                    ctx.sync(t)
                dt = time.perf_counter() - t0
                if best is None or dt < best[0]:
                    best = (dt, t_call)
            ok = torch.equal(dst[-1].cpu(), host[-1])
            extra = with_fd(fd) if with_fd else None
        finally:
            os.close(fd)
        total = len(host) * nbytes
        return {"GBps": round(total / best[0] / 1e9, 2), "ms_per_instance": round(best[0] * 1e3, 3),
                "ms_host_blocked_in_calls": round(best[1] * 1e3, 3),
                "plain_read_GBps": round(total / t_plain / 1e9, 2),
                "store_GBps": round(total / t_store / 1e9, 2), "store_with_fsync_GBps": round(total / t_store_sync / 1e9, 2),
                "o_direct": direct, "byte_exact": bool(ok), "dir": os.path.dirname(path), "pipelined_stream": extra}
    finally:
        if os.path.exists(path):
            os.remove(path)


def load_leg(args, steps, warmup):
    """Row L and row O at the 8B shape (BASELINE config 5): the instance's ten blobs from pinned
    host memory, the link's ceilings, the same through a file, and the pipelined stream."""
    import torch
    wl = Workload(5, args.units, args.variant, args.unfused)
    ctx, cs, ls, L = wl.ctx, wl.cs, wl.ctx.load_stream, wl.L
    try:
        inst_chunks = wl.retrieved[0]
        nbytes = wl.blob_bytes
        host = [torch.empty(nbytes, dtype=torch.uint8).pin_memory() for _ in inst_chunks]
        for h, cid in zip(host, inst_chunks):
            h.copy_(wl.slots[cid].view(torch.uint8).reshape(-1))
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
        kv_load = {"workload": "BASELINE config 5 shape: one instance = 10 blobs x 131.07 MB (1000 tokens, 32 layers, 8 KV heads, D 128, bf16)",
                   "GBps": round(len(host) * nbytes / best / 1e9, 2), "ms_per_instance": round(best * 1e3, 3),
                   "bytes": len(host) * nbytes, "chunks": len(host), "byte_exact": bool(ok),
                   "ceiling_pinned_h2d_1GiB": h2d_ceiling(ls), "pcie_link": pcie_link()}

        # ---- pipelined stream: the next instance's blobs are loaded on the side stream into the
        # other slot set while this instance runs its prefill and decode steps.  Host blobs: a
        # ring of two distinct instance sets (2.6 GB pinned), the instances alternate between them.
        overlap, file_stream = None, None
        if args.stream > 0:
            n_inst = args.stream
            host2 = [torch.empty(nbytes, dtype=torch.uint8).pin_memory() for _ in inst_chunks]
            for h2, h in zip(host2, reversed(host)):
                h2.copy_(h)
            host_sets = [host, host2]
            slot_sets = [dst, [ctx.new_slot(L) for _ in inst_chunks]]
            pages_of = lambda i: [[(d, L) for d in slot_sets[i % 2]]]
            SL = 4                                            # decode slices timed per instance

            def enqueue_load(i):
                return [ctx.load(h, L, d) for h, d in zip(host_sets[i % 2], slot_sets[i % 2])]

            def enqueue_compute(i, tickets, marks=None):
                for t in tickets or []:
                    ctx.wait(t)
                if marks is not None:
                    marks.append(ev()); marks[-1].record(cs)
                wl.prefill_phase(pages_of(i))
                per = wl.steps_dec // SL
                for k in range(wl.steps_dec):
                    if marks is not None and k % per == 0 and k // per < SL:
                        marks.append(ev()); marks[-1].record(cs)
                    ctx.graph_launch(wl.g_step)
                if marks is not None:
                    marks.append(ev()); marks[-1].record(cs)

            def sync_all(tickets):
                for t in tickets:
                    ctx.sync(t)

            def run_stream(load_fn, n, n_serial):
                with torch.cuda.stream(cs):
                    torch.cuda.synchronize()
                    # compute alone: every instance's blobs already in place
                    tk = load_fn(0); sync_all(tk)
                    tk = load_fn(1); sync_all(tk)
                    t0 = time.perf_counter()
                    for i in range(n_serial):
                        enqueue_compute(i, None)
                    cs.synchronize()
                    t_comp = (time.perf_counter() - t0) / n_serial
                    # loads alone
                    t0 = time.perf_counter()
                    hist = []
                    for i in range(n_serial):
                        if i >= 2:
                            sync_all(hist[i - 2])     # the slot set is loaded into again
                        hist.append(load_fn(i))
                    sync_all(hist[-1])
                    t_ld = (time.perf_counter() - t0) / n_serial
                    # serial: load, wait for it, compute, wait for it
                    t0 = time.perf_counter()
                    for i in range(n_serial):
                        tk = load_fn(i)
                        sync_all(tk)
                        enqueue_compute(i, tk)
                        cs.synchronize()
                    t_ser = (time.perf_counter() - t0) / n_serial
                    # pipelined: the compute of i is enqueued, then the load of i+1 is issued
                    tk = load_fn(0)                   # steady state: the first load is already there
                    sync_all(tk)
                    torch.cuda.synchronize()
                    base = ev(); base.record(cs)
                    marks, lmarks = [], []
                    t0 = time.perf_counter()
                    for i in range(n):
                        m = []
                        enqueue_compute(i, tk, m)
                        marks.append(m)
                        if i + 1 < n:
                            l0 = ev(); l0.record(ls)
                            tk = load_fn(i + 1)
                            l1 = ev(); l1.record(ls)
                            lmarks.append((l0, l1))
                    cs.synchronize()
                    torch.cuda.synchronize()
                    t_pipe = (time.perf_counter() - t0) / n
                return t_comp, t_ld, t_ser, t_pipe, base, marks, lmarks

            log(f"pipelined stream of {n_inst} instances")
            n_serial = min(n_inst, 16)
            t_comp, t_ld, t_ser, t_pipe, base, marks, lmarks = run_stream(enqueue_load, n_inst, n_serial)
            # per instance: compute interval, its SL decode slices, and the interval during which the
            # load stream was busy with the next instance's copies (ms after the stream began)
            rel = lambda e: base.elapsed_time(e)
            timeline, slice_ms_in, slice_ms_out = [], [], []
            for i, m in enumerate(marks):
                c0, c1 = rel(m[0]), rel(m[-1])
                cuts = [rel(e) for e in m[1:]]
                lo = (rel(lmarks[i][0]), rel(lmarks[i][1])) if i < len(lmarks) else None
                # a load cannot start before the compute that last read its slot set has finished
                # (instance i-1): its copies run from about max(stream free, that moment) to lo[1]
                for k in range(SL):
                    s0, s1 = cuts[k], cuts[k + 1]
                    busy = lo is not None and min(s1, lo[1]) - max(s0, max(lo[0], c0)) > 0.5 * (s1 - s0)
                    (slice_ms_in if busy else slice_ms_out).append(s1 - s0)
                if i in (1, 2, n_inst // 2, n_inst - 2):
                    timeline.append({"instance": i, "compute_ms": [round(c0, 2), round(c1, 2)],
                                     "prefill_end_ms": round(cuts[0], 2),
                                     "decode_slice_ends_ms": [round(x, 2) for x in cuts[1:]],
                                     "next_load_ms": [round(max(lo[0], c0), 2), round(lo[1], 2)] if lo else None})
            mean = lambda v: round(sum(v) / len(v), 3) if v else None
            overlap = {"instances": n_inst, "host_blob_ring": "2 distinct instance sets (2.62 GB pinned), alternating",
                       "instances_per_s": round(1.0 / t_pipe, 3),
                       "ms_per_instance_pipelined": round(t_pipe * 1e3, 3),
                       "ms_per_instance_serial": round(t_ser * 1e3, 3), "serial_instances": n_serial,
                       "ms_load_alone": round(t_ld * 1e3, 3), "ms_compute_alone": round(t_comp * 1e3, 3),
                       "overlap_frac": round(max(0.0, min(1.0, (t_ld + t_comp - t_pipe) / min(t_ld, t_comp))), 3),
                       "decode_slice_ms_while_loading": mean(slice_ms_in), "decode_slice_ms_no_load": mean(slice_ms_out),
                       "slices_while_loading": len(slice_ms_in), "slices_no_load": len(slice_ms_out),
                       "timeline_ms": timeline}
            del host2

            def file_stream(fd):
                n = min(n_inst, 4)
                tc, tl, ts, tp, *_ = run_stream(lambda i: [ctx.load_file(fd, j * nbytes, nbytes, L, d)
                                                           for j, d in enumerate(slot_sets[i % 2])], n, n)
                return {"instances": n, "instances_per_s": round(1.0 / tp, 3), "ms_per_instance_pipelined": round(tp * 1e3, 3),
                        "ms_per_instance_serial": round(ts * 1e3, 3), "ms_load_alone": round(tl * 1e3, 3),
                        "ms_compute_alone": round(tc * 1e3, 3)}
        log("file tier")
        kv_load["from_file"] = file_leg(ctx, host, dst, L, nbytes, with_fd=file_stream if args.stream > 0 else None)
        kv_load["pipelined_stream"] = overlap
        del host, dst
        return kv_load
    finally:
        wl.close()


def batch16_compressed_leg(reps=10, nl=8):
    """Decode attention over compressed pages at BASELINE config 3's shape (batch 16, five
    1000-token chunks each from a pool of 200, tails at mid-run), nl layers resident."""
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
    ctx = mk.Context(cfg, *streams(), device=dev)
    cs = ctx.compute_stream
    try:
        with torch.cuda.stream(cs):
            slots = {}
            for cid in chunk_ids:
                blob = normal((shape.name, "blob", cid), (nl, 2, Hkv, L, D), shape.value_scale, shape.torch_dtype, dev)
                out = torch.empty(mk.compressed_blob_bytes(cfg, L), dtype=torch.uint8, device=dev)
                ctx.compress(blob, L, out)
                cs.synchronize()
                slots[cid] = out
            q = normal((shape.name, "q_dec"), (nl, B, Hq, D), shape.value_scale, shape.torch_dtype, dev)
            o = torch.empty_like(q)
            tail = normal((shape.name, "tail"), (nl, 2, B, Hkv, max_tail, D), shape.value_scale, shape.torch_dtype, dev)
            table = ctx.new_table()
            ctx.assemble([[(slots[cid], L, mk.PAGE_E4M3) for cid in r] for r in retrieved], q_lens, table)
            ctx.advance(table, shape.decode_steps // 2)
            ctx.graph_begin()
            for l in range(nl):
                ctx.decode_attn(l, q[l], table, tail[l, 0], tail[l, 1], o[l])
            g = ctx.graph_end()
            for _ in range(3):
                ctx.graph_launch(g)
            a, b = ev(), ev()
            a.record(cs)
            for _ in range(reps):
                ctx.graph_launch(g)
            b.record(cs)
            cs.synchronize()
            ctx.graph_destroy(g)
        us = a.elapsed_time(b) * 1e3 / (reps * nl)
        nbytes = sum(L * len(r) * 2 * Hkv * D + (ql + shape.decode_steps // 2) * shape.kv_bytes_per_token_layer()
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
    ctx = mk.Context(cfg, *streams(), device=dev)
    cs = ctx.compute_stream
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
        return {"workload": f"BASELINE config {config_id} with every chunk held as a compressed blob",
                "format": "E4M3 codes + one power-of-two scale per (layer, K/V, KV head)",
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
    torch.cuda.set_device(torch.device("cuda:0"))
    rc = 0
    try:
        rc = run(args)
    finally:
        # nothing of this program is left for the process's exit handlers: every context is
        # closed, every graph destroyed, and the caching allocators (device and pinned host
        # memory) are emptied here, while the runtime is still up
        import gc
        gc.collect()
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        if hasattr(torch._C, "_host_emptyCache"):
            torch._C._host_emptyCache()
    return rc


def run(args):
    import torch
    from workload import CONFIGS

    if args.roofline_only:
        # short run for rocprofv3: eager launches (one dispatch per layer) of the headline config's
        # dominant kernel; with --with-others also one launch per layer of the other kernels
        log("roofline-only run")
        wl = Workload(args.config, args.units, args.variant, args.unfused)
        try:
            r = wl.roofline(args.decode_only_reps, eager=True)
            log("decode-kernel leg done")
            other = wl.other_kernels() if args.with_others else None
            if args.calib_copy:
                with torch.cuda.stream(wl.cs):
                    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
                    dstc = torch.empty_like(src)
                    dstc.copy_(src)
                    wl.cs.synchronize()
                    del src, dstc
            print(json.dumps({"workload": wl.describe(), "roofline": r, "other_kernels": other}))
        finally:
            wl.close()
        return 0

    head = run_config(args.config, args, args.steps, args.warmup, others=not args.no_others, cpu=not args.no_cpu)
    shape = CONFIGS[args.config]
    cpu = head.pop("cpu_baseline", None)

    subs = {}
    sub_steps, sub_warm = min(args.steps, 10), min(args.warmup, 2)
    for cid in [int(x) for x in args.subs.split(",") if x.strip()]:
        if cid == args.config or CONFIGS[cid].dtype != "bf16":
            continue
        subs[f"config{cid}"] = run_config(cid, args, sub_steps, sub_warm, others=not args.no_others)

    kv_load = None if args.no_load else load_leg(args, sub_steps, sub_warm)

    compressed = None
    if not args.no_compressed and args.variant == 0:
        log("compressed-blob leg")
        compressed = compressed_leg(2)
        compressed["decode_attn_batch16"] = batch16_compressed_leg()

    out = {
        "metric": "tokens/s over loaded KV (decode-attn HBM GB/s and % of peak in roofline; KV load GB/s in kv_load)",
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": head["workload"], "batch": shape.batch, "decode_units": args.units, "decode_variant": args.variant},
        "phases_ms": head["phases_ms"],
        "roofline": head["roofline"], "other_kernels": head.get("other_kernels"),
        "configs": subs, "kv_load": kv_load, "compressed_kv": compressed,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))
    sys.stdout.flush()
    return 0


if __name__ == "__main__":
    sys.exit(main())
