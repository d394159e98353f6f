"""ctypes binding of libmatkv.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module turns torch
tensors into device pointers, owns nothing but the ctypes handles, and raises
``MatKVError`` on any non-OK status.  There is no CPU fallback: if the library has
not been built the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, Structure, byref, c_char_p, c_float, c_int32, c_int64, c_size_t,
                    c_uint64, c_void_p)

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmatkv.so")

OK, EINVAL, EUNSUPPORTED, ENOTREADY, EBUSY, EHIP, ENOMEM, EIO = range(8)
PAGE_PLAIN, PAGE_E4M3 = 0, 1
F32, BF16 = 0, 1

EXPORTS = [
    "matkv_blob_bytes", "matkv_compressed_blob_bytes", "matkv_compress", "matkv_tail_bytes", "matkv_workspace_bytes", "matkv_table_bytes",
    "matkv_config_check", "matkv_status_string", "matkv_create", "matkv_destroy",
    "matkv_last_error", "matkv_materialize", "matkv_materialize_tail", "matkv_chunk_attn", "matkv_load", "matkv_load_file", "matkv_store_file",
    "matkv_wait", "matkv_query", "matkv_sync", "matkv_assemble", "matkv_advance",
    "matkv_prefill_attn", "matkv_decode_attn", "matkv_decode_step", "matkv_graph_begin", "matkv_graph_end",
    "matkv_graph_launch", "matkv_graph_destroy", "matkv_plan_decode_units", "matkv_probe_read",
    "matkv_table_shared_units", "matkv_plan_shared_units", "matkv_decode_attn_static",
]


class Config(Structure):
    _fields_ = [("n_layers", c_int32), ("n_q_heads", c_int32), ("n_kv_heads", c_int32),
                ("head_dim", c_int32), ("hidden", c_int32), ("dtype", c_int32),
                ("rope_base", c_float), ("softmax_scale", c_float),
                ("max_batch", c_int32), ("max_pages", c_int32), ("max_tail_tokens", c_int32),
                ("decode_units", c_int32), ("decode_variant", c_int32), ("out_f32", c_int32)]


class Page(Structure):
    _fields_ = [("slot", c_void_p), ("n_tokens", c_int32), ("format", c_int32)]


class Ticket(Structure):
    _fields_ = [("id", c_uint64)]


class MatKVError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        name = _lib.matkv_status_string(status).decode() if _lib is not None else str(status)
        super().__init__(f"{where}: {name}" + (f" ({detail})" if detail else ""))


def _load_library():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
            "libmatkv has no CPU fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    cfgp = POINTER(Config)
    lib.matkv_blob_bytes.argtypes = [cfgp, c_int32]; lib.matkv_blob_bytes.restype = c_size_t
    lib.matkv_tail_bytes.argtypes = [cfgp]; lib.matkv_tail_bytes.restype = c_size_t
    lib.matkv_workspace_bytes.argtypes = [cfgp]; lib.matkv_workspace_bytes.restype = c_size_t
    lib.matkv_table_bytes.argtypes = [cfgp]; lib.matkv_table_bytes.restype = c_size_t
    lib.matkv_config_check.argtypes = [cfgp]; lib.matkv_config_check.restype = c_int32
    lib.matkv_status_string.argtypes = [c_int32]; lib.matkv_status_string.restype = c_char_p
    lib.matkv_create.argtypes = [cfgp, c_void_p, c_size_t, c_void_p, c_void_p, POINTER(c_void_p)]
    lib.matkv_create.restype = c_int32
    lib.matkv_destroy.argtypes = [c_void_p]; lib.matkv_destroy.restype = c_int32
    lib.matkv_last_error.argtypes = [c_void_p]; lib.matkv_last_error.restype = c_char_p
    lib.matkv_materialize.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int32, c_int64,
                                      c_void_p, c_void_p, c_int64]
    lib.matkv_materialize.restype = c_int32
    lib.matkv_materialize_tail.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int32,
                                           c_void_p, c_void_p]
    lib.matkv_materialize_tail.restype = c_int32
    lib.matkv_load.argtypes = [c_void_p, c_void_p, c_size_t, c_int32, c_void_p, c_size_t, POINTER(Ticket)]
    lib.matkv_load.restype = c_int32
    lib.matkv_load_file.argtypes = [c_void_p, c_int32, c_uint64, c_size_t, c_int32, c_void_p, c_size_t, POINTER(Ticket)]
    lib.matkv_load_file.restype = c_int32
    lib.matkv_store_file.argtypes = [c_void_p, c_int32, c_uint64, c_void_p, c_size_t]
    lib.matkv_store_file.restype = c_int32
    for fn in (lib.matkv_wait, lib.matkv_query, lib.matkv_sync):
        fn.argtypes = [c_void_p, Ticket]; fn.restype = c_int32
    lib.matkv_assemble.argtypes = [c_void_p, POINTER(Page), POINTER(c_int32), POINTER(c_int32),
                                   POINTER(c_int64), c_int32, c_void_p]
    lib.matkv_assemble.restype = c_int32
    lib.matkv_advance.argtypes = [c_void_p, c_void_p, c_int32]; lib.matkv_advance.restype = c_int32
    for fn in (lib.matkv_prefill_attn, lib.matkv_decode_attn, lib.matkv_decode_attn_static):
        fn.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
        fn.restype = c_int32
    lib.matkv_compressed_blob_bytes.argtypes = [POINTER(Config), c_int32]
    lib.matkv_compressed_blob_bytes.restype = c_size_t
    lib.matkv_compress.argtypes = [c_void_p, c_void_p, c_int32, c_void_p]
    lib.matkv_compress.restype = c_int32
    lib.matkv_table_shared_units.argtypes = [c_void_p, c_void_p]
    lib.matkv_table_shared_units.restype = c_int32
    lib.matkv_chunk_attn.argtypes = [c_void_p, c_int32, c_void_p, c_void_p, c_int32, c_void_p]
    lib.matkv_chunk_attn.restype = c_int32
    lib.matkv_decode_step.argtypes = [c_void_p, c_int32] + [c_void_p] * 8
    lib.matkv_decode_step.restype = c_int32
    lib.matkv_plan_decode_units.argtypes = [cfgp, POINTER(c_int32), c_int32, c_int32, c_int32,
                                            POINTER(c_int32), POINTER(c_int32), c_int32]
    lib.matkv_plan_decode_units.restype = c_int32
    lib.matkv_plan_shared_units.argtypes = [cfgp] + [POINTER(c_int32)] * 4 + [c_int32, POINTER(c_int32), c_int32, POINTER(c_int32)]
    lib.matkv_plan_shared_units.restype = c_int32
    lib.matkv_probe_read.argtypes = [c_void_p, c_void_p, c_size_t]; lib.matkv_probe_read.restype = c_int32
    lib.matkv_graph_begin.argtypes = [c_void_p]; lib.matkv_graph_begin.restype = c_int32
    lib.matkv_graph_end.argtypes = [c_void_p, POINTER(c_void_p)]; lib.matkv_graph_end.restype = c_int32
    lib.matkv_graph_launch.argtypes = [c_void_p, c_void_p]; lib.matkv_graph_launch.restype = c_int32
    lib.matkv_graph_destroy.argtypes = [c_void_p, c_void_p]; lib.matkv_graph_destroy.restype = c_int32
    return lib


_lib = None
_lib = _load_library()


def lib():
    """The loaded ctypes library (for tests of the raw boundary)."""
    return _lib


def make_config(n_layers, n_q_heads, n_kv_heads, head_dim, hidden, dtype, rope_base,
                max_batch, max_pages, max_tail_tokens, softmax_scale=0.0, decode_units=0,
                decode_variant=0, out_f32=0) -> Config:
    if isinstance(dtype, torch.dtype):
        dtype = F32 if dtype == torch.float32 else BF16
    elif isinstance(dtype, str):
        dtype = F32 if dtype == "f32" else BF16
    return Config(n_layers, n_q_heads, n_kv_heads, head_dim, hidden, dtype, rope_base,
                  softmax_scale, max_batch, max_pages, max_tail_tokens, decode_units, decode_variant, int(out_f32))


def blob_bytes(cfg: Config, n_tokens: int) -> int:
    return int(_lib.matkv_blob_bytes(byref(cfg), n_tokens))


def compressed_blob_bytes(cfg: Config, n_tokens: int) -> int:
    return int(_lib.matkv_compressed_blob_bytes(byref(cfg), n_tokens))


def tail_bytes(cfg: Config) -> int:
    return int(_lib.matkv_tail_bytes(byref(cfg)))


def workspace_bytes(cfg: Config) -> int:
    return int(_lib.matkv_workspace_bytes(byref(cfg)))


def table_bytes(cfg: Config) -> int:
    return int(_lib.matkv_table_bytes(byref(cfg)))


def config_check(cfg: Config) -> int:
    return int(_lib.matkv_config_check(byref(cfg)))


def plan_shared_units(cfg: Config, pages, q_lens):
    """Shared decode partition matkv_assemble would build.  pages: per instance a list of
    (page id, tokens).  Returns (units, slots) with units = list of dicts {page, tokens, tail
    (the instance whose tail the unit holds, or None), users: [(instance, slot, page tokens of
    the unit this user sees)]} and slots = [(first, count)] per instance; ([], None) if none is built."""
    batch, mp = len(pages), max(cfg.max_pages, 1)
    ids, toks = (c_int32 * (batch * mp))(), (c_int32 * (batch * mp))()
    for b, plist in enumerate(pages):
        for i, (pid, n) in enumerate(plist):
            ids[b * mp + i], toks[b * mp + i] = pid, n
    npg = (c_int32 * batch)(*[len(p) for p in pages])
    ql = (c_int32 * batch)(*q_lens)
    cap, w = 4096, 52
    out, slots = (c_int32 * (cap * w))(), (c_int32 * (2 * batch))()
    n = _lib.matkv_plan_shared_units(byref(cfg), ids, toks, npg, ql, batch, out, cap, slots)
    if n < 0:
        raise MatKVError(EINVAL, "matkv_plan_shared_units")
    units = [dict(page=out[u * w], tokens=out[u * w + 1], tail=(out[u * w + 2] if out[u * w + 2] >= 0 else None),
                  users=[(out[u * w + 4 + 3 * k], out[u * w + 5 + 3 * k], out[u * w + 6 + 3 * k]) for k in range(out[u * w + 3])])
             for u in range(n)]
    return units, ([(slots[2 * b], slots[2 * b + 1]) for b in range(batch)] if n else None)


def plan_decode_units(cfg: Config, page_tokens, batch: int, q_len: int):
    """(tokens, page pieces) of each decode unit matkv_assemble would build for one instance."""
    n = len(page_tokens)
    pt = (c_int32 * max(n, 1))(*page_tokens)
    cap = 512
    toks, its = (c_int32 * cap)(), (c_int32 * cap)()
    made = _lib.matkv_plan_decode_units(byref(cfg), pt, n, batch, q_len, toks, its, cap)
    if made < 0:
        raise MatKVError(EINVAL, "matkv_plan_decode_units")
    return list(toks[:made]), list(its[:made])


def _ptr(t) -> int:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


class Context:
    """One matkv_ctx on the current device.  Device buffers are torch tensors owned here only
    to keep them alive (the library itself allocates no device memory)."""

    def __init__(self, cfg: Config, compute_stream: torch.cuda.Stream | None = None,
                 load_stream: torch.cuda.Stream | None = None, device="cuda:0"):
        self.cfg = cfg
        self.device = torch.device(device)
        self.compute_stream = compute_stream or torch.cuda.Stream(device=self.device)
        self.load_stream = load_stream or torch.cuda.Stream(device=self.device)
        nbytes = workspace_bytes(cfg)
        if nbytes == 0:
            raise MatKVError(config_check(cfg), "matkv_config_check")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.elem = 4 if cfg.dtype == F32 else 2
        self.torch_dtype = torch.float32 if cfg.dtype == F32 else torch.bfloat16
        h = c_void_p()
        torch.cuda.synchronize(self.device)
        st = _lib.matkv_create(byref(cfg), self.workspace.data_ptr(), nbytes,
                               self.compute_stream.cuda_stream, self.load_stream.cuda_stream, byref(h))
        if st != OK:
            raise MatKVError(st, "matkv_create")
        self._h = h

    # -- plumbing ---------------------------------------------------------------------------
    def _check(self, st: int, where: str):
        if st != OK:
            raise MatKVError(st, where, _lib.matkv_last_error(self._h).decode())

    def close(self):
        if getattr(self, "_h", None):
            _lib.matkv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def new_table(self) -> torch.Tensor:
        return torch.empty(table_bytes(self.cfg), dtype=torch.uint8, device=self.device)

    def new_tail(self) -> torch.Tensor:
        """Tail buffer of all layers: [layer][K|V][max_batch][Hkv][max_tail][D]."""
        c = self.cfg
        return torch.zeros((c.n_layers, 2, c.max_batch, c.n_kv_heads, c.max_tail_tokens, c.head_dim),
                           dtype=self.torch_dtype, device=self.device)

    def new_slot(self, n_tokens: int) -> torch.Tensor:
        return torch.empty(blob_bytes(self.cfg, n_tokens), dtype=torch.uint8, device=self.device)

    # -- the boundary, same names as the C entry points ---------------------------------------
    def materialize(self, hidden, w_k, w_v, n_tokens, pos0, k_out, v_out, token_stride):
        self._check(_lib.matkv_materialize(self._h, _ptr(hidden), _ptr(w_k), _ptr(w_v), n_tokens, pos0,
                                           _ptr(k_out), _ptr(v_out), token_stride), "matkv_materialize")

    def compress(self, blob, n_tokens, out):
        self._check(_lib.matkv_compress(self._h, _ptr(blob), n_tokens, _ptr(out)), "matkv_compress")

    def materialize_tail(self, hidden, w_k, w_v, table, rows_per_instance, tail_k, tail_v):
        self._check(_lib.matkv_materialize_tail(self._h, _ptr(hidden), _ptr(w_k), _ptr(w_v), _ptr(table),
                                                rows_per_instance, _ptr(tail_k), _ptr(tail_v)),
                    "matkv_materialize_tail")

    def load(self, host_blob, n_tokens, device_slot, nbytes=None, slot_bytes=None) -> Ticket:
        t = Ticket()
        nb = host_blob.numel() * host_blob.element_size() if nbytes is None else nbytes
        sb = device_slot.numel() * device_slot.element_size() if slot_bytes is None else slot_bytes
        self._check(_lib.matkv_load(self._h, _ptr(host_blob), nb, n_tokens, _ptr(device_slot), sb, byref(t)),
                    "matkv_load")
        return t

    def load_file(self, fd: int, offset: int, nbytes: int, n_tokens: int, device_slot, slot_bytes=None) -> Ticket:
        t = Ticket()
        sb = device_slot.numel() * device_slot.element_size() if slot_bytes is None else slot_bytes
        self._check(_lib.matkv_load_file(self._h, fd, offset, nbytes, n_tokens, _ptr(device_slot), sb, byref(t)),
                    "matkv_load_file")
        return t

    def store_file(self, fd: int, offset: int, device_blob, nbytes=None):
        nb = device_blob.numel() * device_blob.element_size() if nbytes is None else nbytes
        self._check(_lib.matkv_store_file(self._h, fd, offset, _ptr(device_blob), nb), "matkv_store_file")

    def wait(self, ticket: Ticket):
        self._check(_lib.matkv_wait(self._h, ticket), "matkv_wait")

    def query(self, ticket: Ticket) -> bool:
        st = _lib.matkv_query(self._h, ticket)
        if st == ENOTREADY:
            return False
        self._check(st, "matkv_query")
        return True

    def sync(self, ticket: Ticket):
        self._check(_lib.matkv_sync(self._h, ticket), "matkv_sync")

    def assemble(self, pages, q_len, table, pos_base=None):
        """pages: per instance a list of (slot tensor or address, n_tokens[, format])."""
        c = self.cfg
        batch = len(pages)
        arr = (Page * (max(batch, 1) * max(c.max_pages, 1)))()
        npg = (c_int32 * batch)(*[len(p) for p in pages])
        for b, plist in enumerate(pages):
            for i, pg in enumerate(plist[:c.max_pages]):
                arr[b * c.max_pages + i] = Page(_ptr(pg[0]), pg[1], pg[2] if len(pg) > 2 else PAGE_PLAIN)
        ql = (c_int32 * batch)(*q_len)
        pb = (c_int64 * batch)(*pos_base) if pos_base is not None else None
        self._check(_lib.matkv_assemble(self._h, arr, npg, ql, pb, batch, _ptr(table)), "matkv_assemble")

    def table_shared_units(self, table) -> int:
        return int(_lib.matkv_table_shared_units(self._h, _ptr(table)))

    def advance(self, table, n=1):
        self._check(_lib.matkv_advance(self._h, _ptr(table), n), "matkv_advance")

    def chunk_attn(self, layer, q, blob, n_tokens, out):
        self._check(_lib.matkv_chunk_attn(self._h, layer, _ptr(q), _ptr(blob), n_tokens, _ptr(out)), "matkv_chunk_attn")

    def prefill_attn(self, layer, q, table, tail_k, tail_v, out):
        self._check(_lib.matkv_prefill_attn(self._h, layer, _ptr(q), _ptr(table), _ptr(tail_k), _ptr(tail_v),
                                            _ptr(out)), "matkv_prefill_attn")

    def decode_attn(self, layer, q, table, tail_k, tail_v, out):
        self._check(_lib.matkv_decode_attn(self._h, layer, _ptr(q), _ptr(table), _ptr(tail_k), _ptr(tail_v),
                                           _ptr(out)), "matkv_decode_attn")

    def decode_attn_static(self, layer, q, table, tail_k, tail_v, out):
        self._check(_lib.matkv_decode_attn_static(self._h, layer, _ptr(q), _ptr(table), _ptr(tail_k), _ptr(tail_v),
                                                  _ptr(out)), "matkv_decode_attn_static")

    def decode_step(self, layer, hidden, w_k, w_v, q, table, tail_k, tail_v, out):
        self._check(_lib.matkv_decode_step(self._h, layer, _ptr(hidden), _ptr(w_k), _ptr(w_v), _ptr(q), _ptr(table),
                                           _ptr(tail_k), _ptr(tail_v), _ptr(out)), "matkv_decode_step")

    def probe_read(self, src, nbytes):
        self._check(_lib.matkv_probe_read(self._h, _ptr(src), nbytes), "matkv_probe_read")

    def graph_begin(self):
        self._check(_lib.matkv_graph_begin(self._h), "matkv_graph_begin")

    def graph_end(self):
        g = c_void_p()
        self._check(_lib.matkv_graph_end(self._h, byref(g)), "matkv_graph_end")
        return g

    def graph_launch(self, g):
        self._check(_lib.matkv_graph_launch(self._h, g), "matkv_graph_launch")

    def graph_destroy(self, g):
        self._check(_lib.matkv_graph_destroy(self._h, g), "matkv_graph_destroy")
