"""Thin ctypes binding of the C-ABI HIP library declared in ``include/gss.h``.

Argument marshalling only: every step of the sampler runs in the library's HIP kernels.  PyTorch
is used for device memory (the library's allocator callbacks hand out ``torch.empty`` buffers) and
for the HIP stream.  There is no CPU fallback: if ``libgss.so`` is missing or cannot be loaded the
import of this module's functions raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Dict, List, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgss.so")

GSS_OK, GSS_ERR_INVALID_ARG, GSS_ERR_INVALID_GRAPH, GSS_ERR_INVALID_SEED = 0, 1, 2, 3
GSS_ERR_OOM, GSS_ERR_DEVICE, GSS_ERR_STEP_ORDER = 4, 5, 6
GSS_MODE_FCR, GSS_MODE_OTF, GSS_MODE_SHARED_OTF, GSS_MODE_FBL, GSS_MODE_SHARED_FCR, GSS_MODE_OTF_FETCH, GSS_MODE_OTF_LAYER = \
    0, 1, 2, 3, 4, 5, 6
GSS_MAX_K = 64
GSS_MAX_IN_FLIGHT = 32

EXPORTS = ["gss_create", "gss_create_tuned", "gss_step", "gss_destroy", "gss_cache_read", "gss_cache_checksum",
           "gss_last_error", "gss_version", "gss_profile_enable", "gss_profile_read", "gss_step_async", "gss_step_wait",
           "gss_cache_bytes", "gss_gather_rows", "gss_pipeline_depth", "gss_cache_checksum_static"]
KERNEL_NAMES = ["fill_full", "step_tick"]


class gss_relation(C.Structure):
    _fields_ = [("src_type", C.c_int32), ("dst_type", C.c_int32), ("nnz", C.c_int64),
                ("indptr", C.c_void_p), ("indptr_is_64", C.c_int32), ("indices", C.c_void_p)]


class gss_graph(C.Structure):
    _fields_ = [("num_node_types", C.c_int32), ("num_nodes", C.POINTER(C.c_int64)),
                ("num_relations", C.c_int32), ("relations", C.POINTER(gss_relation))]


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_void_p, C.c_size_t)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class gss_config(C.Structure):
    _fields_ = [("k", C.c_int32), ("mode", C.c_int), ("num_layers", C.c_int32),
                ("refresh_fraction", C.c_double), ("refresh_period", C.c_int32),
                ("rng_seed", C.c_uint64), ("hip_stream", C.c_void_p),
                ("alloc", ALLOC_FN), ("free", FREE_FN), ("alloc_ctx", C.c_void_p),
                ("degree_threshold", C.c_int32)]


class gss_tuning(C.Structure):
    _fields_ = [("dedupe_layout", C.c_int32), ("table_sets", C.c_int32), ("pipeline_depth", C.c_int32),
                ("steps_per_tick", C.c_int32), ("insert_phase", C.c_int32), ("scan_phase", C.c_int32),
                ("tick_build", C.c_int32), ("first_dedupe_version", C.c_uint32), ("visit_once", C.c_int32),
                ("chain_workgroups", C.c_int32), ("lds_dedupe", C.c_int32), ("group_width", C.c_int32),
                ("reserved", C.c_int32 * 4)]


class gss_block_nodes(C.Structure):
    _fields_ = [("num_dst", C.c_int32), ("num_src", C.c_int32), ("src_nodes", C.c_void_p)]


class gss_block_edges(C.Structure):
    _fields_ = [("num_edges", C.c_int32), ("src_local", C.c_void_p), ("dst_local", C.c_void_p)]


class gss_blocks(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("num_node_types", C.c_int32), ("num_relations", C.c_int32),
                ("nodes", C.POINTER(gss_block_nodes)), ("edges", C.POINTER(gss_block_edges)),
                ("total_edges", C.c_int64)]


_lib = None


def load_library():
    """Load ``libgss.so`` (built by ``paper_2406_17918_amd.build``); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2406_17918_amd.build` "
                           "(there is no fallback path)")
    # PyTorch supplies the device memory and the streams: its HIP runtime must be the process's one, so it is loaded
    # first (a runtime loaded before torch's own copy ends up beside it and sees no device)
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    L.gss_create.argtypes = [C.POINTER(gss_graph), C.POINTER(gss_config), C.POINTER(C.c_void_p)]
    L.gss_create.restype = C.c_int
    L.gss_create_tuned.argtypes = [C.POINTER(gss_graph), C.POINTER(gss_config), C.POINTER(gss_tuning), C.POINTER(C.c_void_p)]
    L.gss_create_tuned.restype = C.c_int
    L.gss_step.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                           C.c_int64, C.POINTER(gss_blocks)]
    L.gss_step.restype = C.c_int
    L.gss_step_async.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_int64]
    L.gss_step_async.restype = C.c_int
    L.gss_step_wait.argtypes = [C.c_void_p, C.POINTER(gss_blocks)]
    L.gss_step_wait.restype = C.c_int
    L.gss_destroy.argtypes = [C.c_void_p]
    L.gss_destroy.restype = C.c_int
    L.gss_cache_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    L.gss_cache_read.restype = C.c_int
    L.gss_cache_checksum.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_uint64)]
    L.gss_cache_checksum.restype = C.c_int
    L.gss_cache_checksum_static.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.gss_cache_checksum_static.restype = C.c_int
    L.gss_cache_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
    L.gss_cache_bytes.restype = C.c_int
    L.gss_pipeline_depth.argtypes = [C.c_void_p]
    L.gss_pipeline_depth.restype = C.c_int32
    L.gss_gather_rows.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    L.gss_gather_rows.restype = C.c_int
    L.gss_last_error.argtypes = [C.c_void_p]
    L.gss_last_error.restype = C.c_char_p
    L.gss_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    L.gss_profile_enable.restype = C.c_int
    L.gss_profile_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.gss_profile_read.restype = C.c_int
    L.gss_version.argtypes = []
    L.gss_version.restype = C.c_char_p
    _lib = L
    return L


class GssError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"gss status {status}: {msg}")
        self.status = status


@dataclass
class DeviceRelation:
    src_type: int
    dst_type: int
    indptr: "torch.Tensor"    # device int32/int64 [n_dst + 1]
    indices: "torch.Tensor"   # device int32 [nnz]


@dataclass
class Block:
    num_dst: List[int]
    num_src: List[int]
    src_nodes: List["torch.Tensor"]   # per node type, device int32 views (valid until the next step)
    num_edges: List[int]
    src_local: List["torch.Tensor"]   # per relation
    dst_local: List["torch.Tensor"]


class _TorchAllocator:
    """Hands the library device memory from PyTorch's caching allocator."""

    def __init__(self, device):
        import torch
        self.torch = torch
        self.device = device
        self.live: Dict[int, "torch.Tensor"] = {}
        self.alloc_cb = ALLOC_FN(self._alloc)
        self.free_cb = FREE_FN(self._free)

    def _alloc(self, ctx, nbytes):
        try:
            t = self.torch.empty(int(nbytes), dtype=self.torch.uint8, device=self.device)
        except Exception:
            return None
        self.live[t.data_ptr()] = t
        return t.data_ptr()

    def _free(self, ctx, ptr):
        self.live.pop(int(ptr), None)

    def view_i32(self, ptr, n):
        if not ptr or n == 0:
            return self.torch.empty(0, dtype=self.torch.int32, device=self.device)
        t = self.live[int(ptr)]
        if t.numel() < 4 * n:              # (the library reported more elements than the buffer it asked for holds)
            raise GssError(GSS_ERR_DEVICE, f"output of {n} int32 in an allocation of {t.numel()} bytes")
        return t[: 4 * n].view(self.torch.int32)


def upload_graph(graph, device="cuda:0") -> List[DeviceRelation]:
    """Copy a host graph (``synth.Graph``-like: .relations with numpy indptr/indices) to the device."""
    import torch
    out = []
    for r in graph.relations:
        out.append(DeviceRelation(r.src_type, r.dst_type, torch.from_numpy(r.indptr).to(device),
                                  torch.from_numpy(r.indices).to(device)))
    return out


def gather_rows(table, ids, out=None):
    """gss_gather_rows on torch tensors: out[i] = table[ids[i]] (table: [N, ...] contiguous, ids: int32, both on the GPU);
    enqueued on torch's current stream."""
    import torch
    assert table.is_cuda and ids.is_cuda and ids.dtype == torch.int32 and table.is_contiguous() and ids.is_contiguous()
    n = ids.numel()
    if out is None:
        out = torch.empty((n,) + tuple(table.shape[1:]), dtype=table.dtype, device=table.device)
    assert out.is_contiguous() and out.dtype == table.dtype and out.numel() * table.shape[0] == n * table.numel()
    row_bytes = table.element_size()
    for d in table.shape[1:]:
        row_bytes *= int(d)
    st = load_library().gss_gather_rows(table.data_ptr() if table.numel() else None, table.shape[0], row_bytes,
                                        ids.data_ptr() if n else None, n, out.data_ptr() if n else None,
                                        torch.cuda.current_stream(table.device).cuda_stream)
    if st != GSS_OK:
        raise GssError(st, "gss_gather_rows failed")
    return out


class Sampler:
    """gss_create / gss_step / gss_destroy on one handle."""

    def __init__(self, num_nodes: Sequence[int], relations: Sequence[DeviceRelation], k: int, mode: int,
                 num_layers: int, refresh_fraction: float = 0.0, refresh_period: int = 1, rng_seed: int = 0,
                 device="cuda:0", degree_threshold: int = -1, tuning: Dict[str, int] = None, allocator=None):
        """`tuning`: fields of gss_tuning by name (layout choices; results do not depend on them).  `allocator`: an
        object with alloc_cb / free_cb / view_i32 like _TorchAllocator (default: a new _TorchAllocator)."""
        import torch
        self.torch = torch
        self._lib = load_library()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.num_nodes = [int(n) for n in num_nodes]
        self.relations = list(relations)
        self.k, self.mode, self.num_layers = k, mode, num_layers
        self.num_tables = 0 if mode == GSS_MODE_FBL else (1 if mode in (GSS_MODE_SHARED_OTF, GSS_MODE_SHARED_FCR) else num_layers)
        self._allocator = allocator if allocator is not None else _TorchAllocator(self.device)
        nn = (C.c_int64 * len(self.num_nodes))(*self.num_nodes)
        rels = (gss_relation * len(self.relations))()
        for i, r in enumerate(self.relations):
            assert r.indptr.is_cuda and r.indices.is_cuda and r.indices.dtype == torch.int32
            assert r.indptr.dtype in (torch.int32, torch.int64)
            assert r.indptr.is_contiguous() and r.indices.is_contiguous()
            assert r.indptr.numel() == self.num_nodes[r.dst_type] + 1
            rels[i] = gss_relation(r.src_type, r.dst_type, r.indices.numel(), r.indptr.data_ptr(),
                                   1 if r.indptr.dtype == torch.int64 else 0, r.indices.data_ptr())
        g = gss_graph(len(self.num_nodes), nn, len(self.relations), rels)
        self._stream = torch.cuda.current_stream(self.device)
        cfg = gss_config(k, mode, num_layers, refresh_fraction, refresh_period, rng_seed,
                         self._stream.cuda_stream, self._allocator.alloc_cb, self._allocator.free_cb, None,
                         degree_threshold)
        h = C.c_void_p()
        tn = gss_tuning(**(tuning or {}))
        st = self._lib.gss_create_tuned(C.byref(g), C.byref(cfg), C.byref(tn), C.byref(h))
        if st != GSS_OK:
            raise GssError(st, "gss_create failed: " + self._lib.gss_last_error(None).decode())
        self._h = h
        self.pipeline_depth = int(self._lib.gss_pipeline_depth(h))   # steps that may be in flight
        self._blocks = gss_blocks()
        self._fo_cache = {}

    def close(self):
        if getattr(self, "_h", None):
            self._lib.gss_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def step_raw(self, seeds, fanouts: Sequence[int], step: int, seed_type: int = 0) -> gss_blocks:
        """One gss_step; returns the raw gss_blocks struct (counts on the host, device pointers)."""
        fo = (C.c_int32 * len(fanouts))(*fanouts)
        st = self._lib.gss_step(self._h, seeds.data_ptr() if seeds.numel() else None, seeds.numel(), seed_type,
                                fo, len(fanouts), step, C.byref(self._blocks))
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())
        return self._blocks

    def _fanout_array(self, fanouts):
        key = tuple(fanouts)
        fo = self._fo_cache.get(key)
        if fo is None:
            fo = self._fo_cache[key] = (C.c_int32 * len(key))(*key)
        return fo

    def step_async(self, seeds, fanouts: Sequence[int], step: int, seed_type: int = 0) -> None:
        """gss_step_async: enqueue one step (at most `pipeline_depth` may be in flight); `seeds` must outlive it."""
        fo = self._fanout_array(fanouts)
        n = seeds.numel()
        st = self._lib.gss_step_async(self._h, seeds.data_ptr() if n else None, n, seed_type, fo, len(fanouts), step)
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())

    def step_wait_raw(self) -> gss_blocks:
        """gss_step_wait: block until the oldest step in flight is done; raw gss_blocks struct."""
        st = self._lib.gss_step_wait(self._h, C.byref(self._blocks))
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())
        return self._blocks

    def step_wait(self) -> List[Block]:
        return self._wrap(self.step_wait_raw())

    def step(self, seeds, fanouts: Sequence[int], step: int, seed_type: int = 0) -> List[Block]:
        return self._wrap(self.step_raw(seeds, fanouts, step, seed_type))

    def _wrap(self, b) -> List[Block]:
        T, R = b.num_node_types, b.num_relations
        out = []
        for l in range(b.num_layers):
            nd, ns, sn, ne, sl, dl = [], [], [], [], [], []
            for t in range(T):
                n = b.nodes[l * T + t]
                nd.append(n.num_dst); ns.append(n.num_src)
                sn.append(self._allocator.view_i32(n.src_nodes, n.num_src))
            for r in range(R):
                e = b.edges[l * R + r]
                ne.append(e.num_edges)
                sl.append(self._allocator.view_i32(e.src_local, e.num_edges))
                dl.append(self._allocator.view_i32(e.dst_local, e.num_edges))
            out.append(Block(nd, ns, sn, ne, sl, dl))
        return out

    def profile_enable(self, on: bool = True):
        st = self._lib.gss_profile_enable(self._h, 1 if on else 0)
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())

    def profile_read(self):
        """{kernel name: (total ms, launches)} since profiling was enabled."""
        ms = (C.c_double * len(KERNEL_NAMES))()
        n = (C.c_int64 * len(KERNEL_NAMES))()
        st = self._lib.gss_profile_read(self._h, ms, n)
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())
        return {name: (ms[i], n[i]) for i, name in enumerate(KERNEL_NAMES)}

    def cache(self, layer: int = 0, relation: int = 0):
        n = self.num_nodes[self.relations[relation].dst_type]
        out = self.torch.empty((n, self.k), dtype=self.torch.int32, device=self.device)
        st = self._lib.gss_cache_read(self._h, layer, relation, out.data_ptr())
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())
        return out

    def cache_bytes(self) -> int:
        v = C.c_int64()
        st = self._lib.gss_cache_bytes(self._h, C.byref(v))
        if st != GSS_OK:
            raise GssError(st, "gss_cache_bytes failed")
        return v.value

    def checksum_static(self, out, layer: int = 0, relation: int = 0) -> None:
        """gss_cache_checksum_static: the checksum into `out` (a device int64 tensor of one element), enqueued on
        torch's current stream and not waited for."""
        assert out.is_cuda and out.numel() == 1 and out.element_size() == 8
        st = self._lib.gss_cache_checksum_static(self._h, layer, relation, out.data_ptr(),
                                                 self.torch.cuda.current_stream(self.device).cuda_stream)
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())

    def checksum(self, layer: int = 0, relation: int = 0) -> int:
        v = C.c_uint64()
        st = self._lib.gss_cache_checksum(self._h, layer, relation, C.byref(v))
        if st != GSS_OK:
            raise GssError(st, self._lib.gss_last_error(self._h).decode())
        return v.value
