"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its pure size arithmetic is right.  No compute call is made here."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mk():
    from paper_2512_22195_amd import LIB_PATH, build
    if not os.path.exists(LIB_PATH):
        build()
    from paper_2512_22195_amd import binding
    return binding


def test_library_exports_every_declared_symbol(mk):
    header = open(os.path.join(ROOT, "include", "matkv.h")).read()
    declared = set(re.findall(r"\b(matkv_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found in include/matkv.h"
    assert declared == set(mk.EXPORTS), declared ^ set(mk.EXPORTS)
    for name in declared:
        assert hasattr(mk.lib(), name), f"libmatkv.so does not export {name}"


def test_blob_bytes_formula_and_paper_orders_of_magnitude(mk):
    """n_layers * 2 * Hkv * n_tokens * D * 2 bytes.  The paper (Section II-C) quotes about
    100 MB per 1000 tokens for a 3B LLaMA and BASELINE's stream config about 1.3 GB for ten
    1000-token chunks of the 8B shape."""
    c8 = mk.make_config(32, 32, 8, 128, 4096, "bf16", 500000.0, 1, 10, 192)
    assert mk.blob_bytes(c8, 1000) == 32 * 2 * 8 * 1000 * 128 * 2 == 131_072_000
    assert abs(10 * mk.blob_bytes(c8, 1000) / 1e9 - 1.3) < 0.02
    # 3B shape: 28 layers, 8 KV heads, D 128 (its 24 query heads, group 3, do not enter the size)
    c3 = mk.make_config(28, 8, 8, 128, 3072, "bf16", 500000.0, 1, 10, 192)
    mb = mk.blob_bytes(c3, 1000) / 1e6
    assert mb == pytest.approx(114.688) and 80 < mb < 130      # "approximately 100 MB"
    c70 = mk.make_config(80, 64, 8, 128, 8192, "bf16", 500000.0, 4, 20, 384)
    assert mk.blob_bytes(c70, 1000) == 327_680_000
    c1 = mk.make_config(1, 4, 2, 64, 256, "f32", 10000.0, 1, 2, 40)
    assert mk.blob_bytes(c1, 256) == 262_144
    assert mk.tail_bytes(c1) == 1 * 2 * 40 * 64 * 4
    assert mk.blob_bytes(c1, -1) == 0


def test_config_check_rejects_what_is_not_built(mk):
    ok = dict(n_layers=1, n_q_heads=4, n_kv_heads=2, head_dim=64, hidden=256, dtype="f32",
              rope_base=10000.0, max_batch=1, max_pages=2, max_tail_tokens=40)
    assert mk.config_check(mk.make_config(**ok)) == mk.OK
    bad = [dict(head_dim=96), dict(n_q_heads=6, n_kv_heads=4), dict(n_q_heads=32, n_kv_heads=2),
           dict(hidden=100), dict(max_tail_tokens=41), dict(n_layers=0), dict(rope_base=1.0),
           dict(decode_units=1000), dict(max_batch=0)]
    for delta in bad:
        cfg = mk.make_config(**{**ok, **delta})
        assert mk.config_check(cfg) in (mk.EINVAL, mk.EUNSUPPORTED), delta
        assert mk.workspace_bytes(cfg) == 0 and mk.table_bytes(cfg) == 0
    assert mk.config_check(mk.make_config(**{**ok, "head_dim": 96})) == mk.EUNSUPPORTED
    assert mk.lib().matkv_status_string(3) == b"MATKV_ENOTREADY"


def test_workspace_and_table_sizes_are_positive_and_aligned(mk):
    c = mk.make_config(32, 32, 8, 128, 4096, "bf16", 500000.0, 16, 5, 192)
    assert mk.workspace_bytes(c) % 256 == 0 and mk.workspace_bytes(c) > 0
    assert mk.table_bytes(c) % 256 == 0 and mk.table_bytes(c) > 0
    # bf16 / head_dim 128: room for the projection's split tiles (128 tiles x two fp32 partials of
    # 128 x 128) however small the attention's own needs are
    small = mk.make_config(1, 8, 2, 128, 512, "bf16", 500000.0, 1, 1, 8)
    assert mk.workspace_bytes(small) >= 128 * 2 * 128 * 128 * 4


def test_null_context_is_an_error_not_a_crash(mk):
    assert mk.lib().matkv_destroy(None) == mk.EINVAL
    assert mk.lib().matkv_advance(None, None, 1) == mk.EINVAL
    assert mk.lib().matkv_last_error(None) == b"context is null"


def test_decode_partition_covers_every_token_once_and_is_balanced(mk):
    """Host logic of cache assembly: the units of an instance partition its page tokens
    (nothing lost, nothing twice), in nearly equal shares, whatever the chunk lengths."""
    cfg = mk.make_config(32, 32, 8, 128, 4096, "bf16", 500000.0, 1, 10, 192)
    toks, items = mk.plan_decode_units(cfg, [1000] * 10, batch=1, q_len=64)
    assert sum(toks) == 10000 and len(toks) == 32                  # 8 KV heads x 32 units = 256 workgroups
    body = toks[:-1]                                               # the last unit also streams the tail
    assert max(body) - min(body) <= 8 and toks[-1] <= max(body)
    assert all(1 <= i <= 2 for i in items[:-1])                    # a unit spans at most two 1000-token pages
    # ragged chunk lengths, including a 1-token chunk; forced unit counts
    for units in (1, 3, 7, 64):
        cfg = mk.make_config(2, 8, 2, 128, 512, "bf16", 500000.0, 4, 6, 64, decode_units=units)
        lens = [300, 77, 1, 129, 1000, 5]
        toks, items = mk.plan_decode_units(cfg, lens, batch=3, q_len=9)
        assert sum(toks) == sum(lens) and 1 <= len(toks) <= units
        assert all(t >= 0 for t in toks) and all(i >= 0 for i in items)
    # batch 16: one unit per (instance, KV head) pair is already 128 workgroups -> 2 units each
    cfg = mk.make_config(32, 32, 8, 128, 4096, "bf16", 500000.0, 16, 5, 192)
    toks, _ = mk.plan_decode_units(cfg, [1000] * 5, batch=16, q_len=100)
    assert len(toks) == 2 and sum(toks) == 5000
    # no pages at all: a single unit that only owns the tail
    toks, items = mk.plan_decode_units(cfg, [], batch=1, q_len=10)
    assert toks == [0] and items == [0]
    with pytest.raises(mk.MatKVError):
        mk.plan_decode_units(cfg, [0, 5], batch=1, q_len=10)


def test_decode_partition_never_exceeds_the_compute_units(mk):
    """Workgroups of a decode launch = units x KV heads over the batch: at most 256, so that no
    compute unit holds two (batch 3 x 8 KV heads: 10 units each, not 11)."""
    for batch in (1, 2, 3, 5, 7, 16):
        cfg = mk.make_config(32, 32, 8, 128, 4096, "bf16", 500000.0, batch, 10, 192)
        toks, _ = mk.plan_decode_units(cfg, [1000] * 10, batch=batch, q_len=64)
        assert len(toks) * batch * 8 <= 256 and len(toks) == 256 // (batch * 8)
        assert sum(toks) == 10000


def test_shared_partition_covers_every_instance_once(mk):
    """Host logic of the shared decode partition: built when the batch's distinct pages are at least
    a twentieth fewer tokens than all uses; every (instance, page token) is streamed by exactly one
    unit that lists the instance; a unit has at most 16 / G users and at most one tail; every
    instance's tail sits in exactly one unit; every instance owns a run of distinct partial slots
    that its units' entries use up exactly; the launch has at most one workgroup per compute unit."""
    rng = np.random.default_rng(7)
    for G, Hkv in ((4, 8), (1, 2), (3, 8), (8, 8), (2, 4)):
        for trial in range(8):
            batch = int(rng.integers(2, 17))
            n_chunks = int(rng.integers(1, 7))
            lens = [int(rng.integers(1, 1500)) for _ in range(n_chunks)]
            pages = []
            for _ in range(batch):
                k = int(rng.integers(0, n_chunks + 1))
                ids = sorted(rng.choice(n_chunks, size=k, replace=False).tolist())
                if 0 not in ids and rng.random() < 0.8:
                    ids = [0] + ids                         # a hot chunk
                pages.append([(i, lens[i]) for i in ids])
            q_lens = [int(rng.integers(1, 100)) for _ in range(batch)]
            cfg = mk.make_config(2, G * Hkv, Hkv, 128, 4096, "bf16", 500000.0, batch, 6, 128)
            units, slots = mk.plan_shared_units(cfg, pages, q_lens)
            all_tokens = sum(n for p in pages for _, n in p)
            distinct = sum(lens[i] for i in {i for p in pages for i, _ in p})
            if 20 * distinct > 19 * all_tokens:
                assert units == [] and slots is None
                continue
            assert units and len(units) * Hkv <= 256
            streamed = [0] * batch
            used = [set() for _ in range(batch)]
            tails = [0] * batch
            for u in units:
                assert 1 <= len(u["users"]) <= 16 // G
                assert u["tokens"] > 0 or u["tail"] is not None
                if u["tail"] is not None:
                    assert u["tail"] in [inst for inst, _, _ in u["users"]]
                    tails[u["tail"]] += 1
                assert len({inst for inst, _, _ in u["users"]}) == len(u["users"])
                for inst, slot, seen in u["users"]:
                    assert 0 <= seen <= u["tokens"]
                    streamed[inst] += seen
                    first, count = slots[inst]
                    assert first <= slot < first + count and slot not in used[inst]
                    used[inst].add(slot)
            assert tails == [1] * batch
            assert streamed == [sum(n for _, n in p) for p in pages]
            assert [len(s) for s in used] == [c for _, c in slots]
            ends = sorted((f, f + c) for f, c in slots)
            assert all(a[1] == b[0] for a, b in zip(ends, ends[1:])) and ends[0][0] == 0     # the runs tile 0 .. total
            # every distinct page is streamed once per group of 16 / G users
            groups = sum(-(-sum(1 for p in pages if any(i == c for i, _ in p)) // (16 // G)) * lens[c]
                         for c in {i for p in pages for i, _ in p})
            assert sum(u["tokens"] for u in units) == groups
    # BASELINE config 3 (batch 16, five chunks each out of 200: 65 distinct of 80): 32 even units per KV head
    from workload import CONFIGS, question_lengths, retrieved_chunks
    s3 = CONFIGS[3]
    cfg = mk.make_config(32, 32, 8, 128, 4096, "bf16", 500000.0, 16, 5, 192)
    units, slots = mk.plan_shared_units(cfg, [[(c, 1000) for c in r] for r in retrieved_chunks(s3)], question_lengths(s3))
    assert len(units) == 32 and sum(u["tokens"] for u in units) == 65000
    sizes = [u["tokens"] for u in units]
    assert max(sizes) - min(sizes) <= 2 * 192               # a unit holds at most one tail (uncut, at most 192 rows) and ends before a second
    # not built: explicit unit count, fp32, a batch of one
    pages = [[(0, 500)], [(0, 500)], [(0, 500)]]
    assert mk.plan_shared_units(mk.make_config(2, 8, 2, 128, 512, "bf16", 500000.0, 3, 2, 64, decode_units=2), pages, [3, 3, 3])[0] == []
    assert mk.plan_shared_units(mk.make_config(2, 8, 2, 64, 512, "f32", 10000.0, 3, 2, 64), pages, [3, 3, 3])[0] == []
    assert mk.plan_shared_units(mk.make_config(2, 8, 2, 128, 512, "bf16", 500000.0, 3, 2, 64), pages[:1], [3])[0] == []
    units, _ = mk.plan_shared_units(mk.make_config(2, 8, 2, 128, 512, "bf16", 500000.0, 3, 2, 64), pages, [3, 3, 3])
    assert units and sum(u["tokens"] for u in units) == 500 and all(len(u["users"]) <= 4 for u in units)
    with pytest.raises(mk.MatKVError):
        mk.plan_shared_units(mk.make_config(2, 8, 2, 128, 512, "bf16", 500000.0, 3, 2, 64), [[(0, 0)], [(0, 5)]], [3, 3])
