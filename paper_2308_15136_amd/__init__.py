"""MI355X-native CAGRA (graph build + batched greedy graph search).

Thin binding over the C ABI of include/cagra_hip.h: the functions below only
marshal arguments (device pointers of torch tensors, sizes, the current HIP
stream) into libcagra_hip.so; every step of the method runs in that library's
gfx950 kernels.  There is no CPU fallback: if the library is missing the calls
raise.

Node ids travel as torch.int32 tensors holding the uint32 bit patterns of the
C ABI (ids are below 2^31, the invalid id 0xFFFFFFFF reads as -1).
"""
from __future__ import annotations

import ctypes as C
import os
import dataclasses
from dataclasses import dataclass
from typing import Optional, Tuple

_PKG = os.path.dirname(os.path.abspath(__file__))
# CAGRA_HIP_LIB names another build of the same library (e.g. one with the phase timers compiled in)
LIB_PATH = os.environ.get("CAGRA_HIP_LIB") or os.path.join(_PKG, "libcagra_hip.so")
PROBE_LIB_PATH = os.path.join(_PKG, "libcagra_probe.so")

L2 = 0
IP = 1
F32 = 0
F16 = 1
U8 = 2
REORDER_RANK = 0
REORDER_DISTANCE = 1
EXACT_AUTO = 0
EXACT_PLAIN = 1
EXACT_FILTERED = 2
INVALID_ID = -1  # 0xFFFFFFFF seen through int32

_lib = None


class CagraError(RuntimeError):
    pass


class _SearchOpts(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("max_iterations", C.c_int32), ("mode", C.c_int32),
                ("team_size", C.c_int32), ("hash_bits", C.c_int32), ("reset_interval", C.c_int32),
                ("wg_per_query", C.c_int32), ("table_entries", C.c_int32), ("dataset_type", C.c_int32),
                ("table_policy", C.c_int32), ("workgroups_per_cu", C.c_int32), ("waves_per_query", C.c_int32),
                ("workspace_clean", C.c_int32), ("reserved", C.c_int32), ("stats", C.c_void_p)]


class _BuildOpts(C.Structure):
    _fields_ = [("reorder", C.c_int32), ("initial_graph", C.c_int32), ("nnd_rounds", C.c_int32),
                ("nnd_sample", C.c_int32), ("seed", C.c_uint64), ("exact_algo", C.c_int32), ("reserved", C.c_int32)]


class _SearchPlan(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("mode", "team_size", "table_entries", "reset_interval",
                                         "max_iterations", "wg_per_query", "itopk_local", "lds_bytes",
                                         "workgroups", "table_policy", "waves_per_query", "reserved")] + \
               [("ws_tickets_offset", C.c_int64), ("ws_which_offset", C.c_int64), ("ws_tables_offset", C.c_int64)]


def load_library():
    """Load libcagra_hip.so (built by paper_2308_15136_amd.buildlib) and declare its ABI."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise CagraError(f"{LIB_PATH} is missing: run `python -m paper_2308_15136_amd.buildlib` "
                         "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    opts_p = C.POINTER(_SearchOpts)
    lib.cagra_strerror.restype = C.c_char_p
    lib.cagra_strerror.argtypes = [C.c_int]
    lib.cagra_seed_id.restype = C.c_uint32
    lib.cagra_seed_id.argtypes = [C.c_uint64] * 4
    lib.cagra_search_auto_mode.restype = C.c_int
    lib.cagra_search_auto_mode.argtypes = [i64, i32]
    lib.cagra_search.restype = C.c_int
    lib.cagra_search.argtypes = [vp, i64, i32, vp, i32, i64, C.c_int, vp, i64, i64, i32, i32, i32,
                                 opts_p, vp, vp, vp, sz, vp]
    lib.cagra_search_static.restype = C.c_int
    lib.cagra_search_static.argtypes = [vp, i64, i32, vp, i32, i64, C.c_int, vp, i64, i64, i32, i32, i32,
                                        opts_p, vp, vp, vp]
    lib.cagra_search_workspace_init.restype = C.c_int
    lib.cagra_search_workspace_init.argtypes = [i64, i32, i32, i64, i32, i32, i32, opts_p, vp, sz, vp]
    lib.cagra_search_describe.restype = C.c_int
    lib.cagra_search_describe.argtypes = [i32, i32, i64, i32, i32, i32, opts_p, C.POINTER(_SearchPlan)]
    lib.cagra_search_workspace_bytes.restype = sz
    lib.cagra_search_workspace_bytes.argtypes = [i64, i32, i64, i32, i32, i32, opts_p]
    lib.cagra_convert_dataset.restype = C.c_int
    lib.cagra_convert_dataset.argtypes = [vp, i64, i32, i64, C.c_int, vp, i64, vp]
    lib.cagra_exact_search.restype = C.c_int
    lib.cagra_exact_search.argtypes = [vp, i64, i32, i64, C.c_int, vp, i64, i64, i32, i32, i64,
                                       vp, vp, vp, sz, vp]
    lib.cagra_exact_search_workspace_bytes.restype = sz
    lib.cagra_exact_search_workspace_bytes.argtypes = [i64, i64, i32]
    lib.cagra_exact_search_ex.restype = C.c_int
    lib.cagra_exact_search_ex.argtypes = [vp, i64, i32, i64, C.c_int, vp, i64, i64, i32, i32, i64, C.c_int,
                                          vp, vp, vp, vp, sz, vp]
    lib.cagra_exact_search_ex_workspace_bytes.restype = sz
    lib.cagra_exact_search_ex_workspace_bytes.argtypes = [i64, i32, i64, i32, C.c_int]
    lib.cagra_build.restype = C.c_int
    lib.cagra_build.argtypes = [vp, i64, i32, i64, C.c_int, i32, i32, vp, vp, sz, vp]
    lib.cagra_build_workspace_bytes.restype = sz
    lib.cagra_build_workspace_bytes.argtypes = [i64, i32, i32, i32]
    lib.cagra_optimize.restype = C.c_int
    lib.cagra_optimize.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.cagra_optimize_workspace_bytes.restype = sz
    lib.cagra_optimize_workspace_bytes.argtypes = [i64, i32, i32]
    lib.cagra_optimize_ex.restype = C.c_int
    lib.cagra_optimize_ex.argtypes = [vp, vp, i64, i32, i32, C.c_int, vp, vp, vp, vp, vp, sz, vp]
    bopts_p = C.POINTER(_BuildOpts)
    lib.cagra_build_ex.restype = C.c_int
    lib.cagra_build_ex.argtypes = [vp, i64, i32, i64, C.c_int, i32, i32, bopts_p, vp, vp, sz, vp]
    lib.cagra_build_ex_workspace_bytes.restype = sz
    lib.cagra_build_ex_workspace_bytes.argtypes = [i64, i32, i32, i32, bopts_p]
    lib.cagra_nn_descent.restype = C.c_int
    lib.cagra_nn_descent.argtypes = [vp, i64, i32, i64, C.c_int, i32, i32, i32, C.c_uint64, vp, vp, vp, sz, vp]
    lib.cagra_nn_descent_workspace_bytes.restype = sz
    lib.cagra_nn_descent_workspace_bytes.argtypes = [i64, i32, i32]
    lib.cagra_two_hop_counts.restype = C.c_int
    lib.cagra_two_hop_counts.argtypes = [vp, i64, i32, vp, vp]
    lib.cagra_count_components.restype = C.c_int
    lib.cagra_count_components.argtypes = [vp, i64, i32, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    _lib = lib
    return lib


_probe_lib = None


def load_probe_library():
    """Load libcagra_probe.so, the bandwidth probe built beside the product library (include/cagra_probe.h)."""
    global _probe_lib
    if _probe_lib is None:
        if not os.path.exists(PROBE_LIB_PATH):
            raise CagraError(f"{PROBE_LIB_PATH} is missing: run `python -m paper_2308_15136_amd.buildlib`")
        lib = C.CDLL(PROBE_LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        lib.cagra_probe_bandwidth.restype = C.c_int
        lib.cagra_probe_bandwidth.argtypes = [vp, i64, i64, i64, i32, i64, i32, i32, i32, C.c_uint64, vp, vp]
        _probe_lib = lib
    return _probe_lib


def strerror(code: int) -> str:
    return load_library().cagra_strerror(code).decode()


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise CagraError(f"{what}: {strerror(rc)} (code {rc})")


def _torch():
    import torch
    return torch


def _dev_f32(t, name):
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.dim() == 2
            and t.stride(1) == 1):
        raise TypeError(f"{name} must be a 2-D float32 device tensor with unit inner stride")
    return t


def _dev_dataset(t):
    """A dataset for the search: float32, float16 or uint8 rows; returns (tensor, cagra_dtype)."""
    torch = _torch()
    kinds = {torch.float32: F32, torch.float16: F16, torch.uint8: U8}
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype in kinds and t.dim() == 2 and t.stride(1) == 1):
        raise TypeError("dataset must be a 2-D float32 / float16 / uint8 device tensor with unit inner stride")
    return t, kinds[t.dtype]


def convert_dataset(dataset, dtype: int, row_bytes_multiple: int = 0):
    """fp32 dataset -> fp16 or uint8 copy (rounded to nearest even; uint8 clamped to 0..255), or an fp32 copy.
    row_bytes_multiple: pad the row stride of the copy to a multiple of that many bytes (64: rows start on the
    memory system's sector boundaries; 0: to the next 16 bytes, the least the search accepts); the result is a
    view [N, dim] into the padded matrix, whose padding the library has set to zero -- the form in which every
    entry point takes rows whose dim is not a whole number of 16-byte pieces."""
    torch = _torch()
    dataset = _dev_f32(dataset, "dataset")
    tdt = {F32: torch.float32, F16: torch.float16, U8: torch.uint8}[dtype]
    n, dim = dataset.shape
    es = torch.empty(0, dtype=tdt).element_size()
    row_bytes_multiple = row_bytes_multiple or 16
    if row_bytes_multiple % 16:
        raise ValueError("row_bytes_multiple must be a multiple of 16")
    ld = -(-dim * es // row_bytes_multiple) * row_bytes_multiple // es
    out = torch.empty((n, ld), dtype=tdt, device=dataset.device)[:, :dim]
    _check(load_library().cagra_convert_dataset(dataset.data_ptr(), dataset.shape[0], dataset.shape[1],
                                                dataset.stride(0), dtype, out.data_ptr(), out.stride(0),
                                                _stream(dataset.device)), "cagra_convert_dataset")
    return out


def two_hop_counts(graph):
    """Sec. III-A: per node, the number of other nodes reachable in one or two steps (int32 device tensor)."""
    torch = _torch()
    graph = _dev_i32(graph, "graph")
    out = torch.empty((graph.shape[0],), dtype=torch.int32, device=graph.device)
    _check(load_library().cagra_two_hop_counts(graph.data_ptr(), graph.shape[0], graph.shape[1], out.data_ptr(),
                                               _stream(graph.device)), "cagra_two_hop_counts")
    return out


def count_components(graph) -> Tuple[int, int]:
    """(strong, weak) connected component counts of the graph; runs on the host on a copy of the graph."""
    torch = _torch()
    g = graph.detach().to("cpu").contiguous() if isinstance(graph, torch.Tensor) else torch.as_tensor(graph)
    if g.dtype != torch.int32 or g.dim() != 2:
        raise TypeError("graph must be a 2-D int32 tensor")
    strong, weak = C.c_int64(0), C.c_int64(0)
    _check(load_library().cagra_count_components(g.data_ptr(), g.shape[0], g.shape[1], C.byref(strong),
                                                 C.byref(weak)), "cagra_count_components")
    return int(strong.value), int(weak.value)


def probe_bandwidth(data, pattern: int, n_read: int = 0, team_size: int = 0, rows_in_flight: int = 0,
                    waves_per_cu: int = 0, seed: int = 0, sink=None) -> None:
    """Enqueue one bandwidth-reference read of the 2-D device tensor `data` (pattern 0: streaming
    read of all of it, 1: n_read random whole rows).  The caller times it."""
    torch = _torch()
    if not (isinstance(data, torch.Tensor) and data.is_cuda and data.dim() == 2 and data.stride(1) == 1):
        raise TypeError("data must be a 2-D device tensor with unit inner stride")
    es = data.element_size()
    if sink is None:
        sink = torch.zeros(1, dtype=torch.int32, device=data.device)
    _check(load_probe_library().cagra_probe_bandwidth(data.data_ptr(), data.shape[0], data.shape[1] * es,
                                                data.stride(0) * es, pattern, n_read, team_size, rows_in_flight,
                                                waves_per_cu, seed, sink.data_ptr(), _stream(data.device)),
           "cagra_probe_bandwidth")


def _dev_i32(t, name):
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous int32 device tensor")
    return t


def _workspace(nbytes: int, device):
    torch = _torch()
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _stream(device) -> int:
    return int(_torch().cuda.current_stream(device).cuda_stream)


def seed_id(seed: int, query: int, slot: int, n: int) -> int:
    return int(load_library().cagra_seed_id(seed, query, slot, n))


def auto_mode(batch: int, itopk: int) -> int:
    return int(load_library().cagra_search_auto_mode(batch, itopk))


@dataclass
class SearchOptions:
    seed: int = 0
    max_iterations: int = 0
    mode: int = 0
    team_size: int = 0
    hash_bits: int = 0
    reset_interval: int = 0
    wg_per_query: int = 0
    table_entries: int = 0
    dataset_type: int = 0      # F32 / F16 / U8; search() sets it from the dataset tensor's dtype
    table_policy: int = 0      # 0 automatic, 1 periodic reset (the paper's), 2 replacement in sets of four
    workgroups_per_cu: int = 0  # single mode: persistent workgroups per compute unit, 0 automatic
    waves_per_query: int = 0   # single mode: wavefronts per query (0 automatic, 1, 2, 4)
    workspace_clean: int = 0   # multi mode: 1 = the workspace passed in is clean for these arguments (see the header)


def _copts(o: "SearchOptions", stats_ptr=None) -> _SearchOpts:
    return _SearchOpts(o.seed, o.max_iterations, o.mode, o.team_size, o.hash_bits, o.reset_interval,
                       o.wg_per_query, o.table_entries, o.dataset_type, o.table_policy, o.workgroups_per_cu,
                       o.waves_per_query, o.workspace_clean, 0, stats_ptr)


def describe(degree: int, dim: int, batch: int, k: int, itopk: int, search_width: int = 1,
             options: Optional["SearchOptions"] = None) -> dict:
    """The resolved mode and automatic parameters a search with these arguments would use."""
    plan = _SearchPlan()
    copts = _copts(options or SearchOptions())
    _check(load_library().cagra_search_describe(degree, dim, batch, k, itopk, search_width,
                                                C.byref(copts), C.byref(plan)), "cagra_search_describe")
    return {n: int(getattr(plan, n)) for n, _ in _SearchPlan._fields_ if n != "reserved"}


def search_workspace_init(workspace, n: int, degree: int, dim: int, batch: int, k: int, itopk: int, search_width: int = 1,
                          options: Optional["SearchOptions"] = None) -> None:
    """Clean `workspace` (uint8 device tensor) for multi-mode searches with these arguments; such a search may then
    set SearchOptions.workspace_clean = 1."""
    copts = _copts(options or SearchOptions())
    _check(load_library().cagra_search_workspace_init(n, degree, dim, batch, k, itopk, search_width, C.byref(copts),
                                                      workspace.data_ptr(), workspace.numel(), _stream(workspace.device)),
           "cagra_search_workspace_init")


def search_workspace_bytes(n: int, degree: int, batch: int, k: int, itopk: int, search_width: int = 1,
                           options: Optional["SearchOptions"] = None) -> int:
    copts = _copts(options or SearchOptions())
    return int(load_library().cagra_search_workspace_bytes(n, degree, batch, k, itopk, search_width,
                                                           C.byref(copts)))


def _search_tensors(graph, dataset, queries, k: int, out, stats):
    """Checks what the library cannot see behind raw pointers: shapes that belong together, one device,
    output buffers of the right type and size."""
    torch = _torch()
    graph = _dev_i32(graph, "graph")
    dataset, dtype = _dev_dataset(dataset)
    queries = _dev_f32(queries, "queries")
    if graph.dim() != 2 or graph.shape[0] != dataset.shape[0]:
        raise ValueError(f"graph has {tuple(graph.shape)} entries, dataset {dataset.shape[0]} rows: one graph row per dataset row")
    if queries.shape[1] != dataset.shape[1]:
        raise ValueError(f"queries have {queries.shape[1]} dimensions, dataset rows {dataset.shape[1]}")
    dev = dataset.device
    if graph.device != dev or queries.device != dev:
        raise ValueError("graph, dataset and queries must be on the same device")
    B = queries.shape[0]
    if stats is not None and not (isinstance(stats, torch.Tensor) and stats.device == dev and stats.dtype == torch.int32
                                  and stats.is_contiguous() and stats.numel() >= 4 * B):
        raise TypeError("stats must be a contiguous int32 tensor of at least B * 4 elements on the dataset's device")
    if out is not None:
        ids, dists = out
        for t, dt, name in ((ids, torch.int32, "ids"), (dists, torch.float32, "dists")):
            if not (isinstance(t, torch.Tensor) and t.device == dev and t.dtype == dt and t.is_contiguous()
                    and tuple(t.shape) == (B, k)):
                raise TypeError(f"out {name} must be a contiguous {dt} tensor of shape ({B}, {k}) on the dataset's device")
    return graph, dataset, dtype, queries


def search(graph, dataset, queries, k: int, itopk: int, search_width: int = 1, metric: int = L2,
           options: Optional[SearchOptions] = None, return_stats: bool = False,
           out: Optional[Tuple] = None, workspace=None, stats=None):
    """Batched greedy graph search: (ids[B, k] int32, dists[B, k] float32[, stats[B, 4] int32]).
    `out`, `workspace` and `stats` (int32 [B, 4], implies return_stats) may be preallocated."""
    torch = _torch()
    lib = load_library()
    graph, dataset, dtype, queries = _search_tensors(graph, dataset, queries, k, out, stats)
    dev = dataset.device
    B = queries.shape[0]
    o = dataclasses.replace(options or SearchOptions(), dataset_type=dtype)
    if stats is not None:
        return_stats = True
    elif return_stats:
        stats = torch.zeros((B, 4), dtype=torch.int32, device=dev)
    copts = _copts(o, stats.data_ptr() if stats is not None else None)
    if out is None:
        ids = torch.empty((B, k), dtype=torch.int32, device=dev)
        dists = torch.empty((B, k), dtype=torch.float32, device=dev)
    else:
        ids, dists = out
    N, degree = graph.shape
    if workspace is None:
        workspace = _workspace(lib.cagra_search_workspace_bytes(N, degree, B, k, itopk, search_width,
                                                                C.byref(copts)), dev)
    elif not (isinstance(workspace, torch.Tensor) and workspace.device == dev and workspace.dtype == torch.uint8
              and workspace.is_contiguous()):
        raise TypeError("workspace must be a contiguous uint8 tensor on the dataset's device")
    rc = lib.cagra_search(graph.data_ptr(), N, degree, dataset.data_ptr(), dataset.shape[1],
                          dataset.stride(0), metric, queries.data_ptr(), B, queries.stride(0),
                          k, itopk, search_width, C.byref(copts), ids.data_ptr(), dists.data_ptr(),
                          workspace.data_ptr(), workspace.numel(), _stream(dev))
    _check(rc, "cagra_search")
    return (ids, dists, stats) if return_stats else (ids, dists)


def search_static(graph, dataset, queries, k: int, itopk: int, search_width: int = 1, metric: int = L2,
                  options: Optional[SearchOptions] = None, out: Optional[Tuple] = None, stats=None):
    """cagra_search_static: the same search with the library's own static scratch array instead of a
    workspace (nothing is allocated inside the call; give `out` to keep this wrapper from allocating)."""
    torch = _torch()
    lib = load_library()
    graph, dataset, dtype, queries = _search_tensors(graph, dataset, queries, k, out, stats)
    dev = dataset.device
    B = queries.shape[0]
    o = dataclasses.replace(options or SearchOptions(), dataset_type=dtype)
    copts = _copts(o, stats.data_ptr() if stats is not None else None)
    if out is None:
        out = (torch.empty((B, k), dtype=torch.int32, device=dev), torch.empty((B, k), dtype=torch.float32, device=dev))
    ids, dists = out
    N, degree = graph.shape
    rc = lib.cagra_search_static(graph.data_ptr(), N, degree, dataset.data_ptr(), dataset.shape[1],
                                 dataset.stride(0), metric, queries.data_ptr(), B, queries.stride(0),
                                 k, itopk, search_width, C.byref(copts), ids.data_ptr(), dists.data_ptr(), _stream(dev))
    _check(rc, "cagra_search_static")
    return (ids, dists, stats) if stats is not None else (ids, dists)


class PreparedSearch:
    """A search call with everything but the launch resolved once: tensors checked, options
    marshalled, outputs and workspace allocated.  Calling it enqueues one search on the current stream
    and returns (ids, dists): the same tensors every time.  Without an argument it searches the
    `queries` buffer it was made for (write new queries into that buffer between calls); with one it
    searches that tensor instead (same shape, float32, same device; the caller keeps it alive until the
    search has run).  For loops that issue many small calls."""

    def __init__(self, graph, dataset, queries, k: int, itopk: int, search_width: int = 1, metric: int = L2,
                 options: Optional[SearchOptions] = None):
        torch = _torch()
        self._lib = load_library()
        graph, dataset, dtype, queries = _search_tensors(graph, dataset, queries, k, None, None)
        dev = dataset.device
        B = queries.shape[0]
        o = dataclasses.replace(options or SearchOptions(), dataset_type=dtype, workspace_clean=0)
        self._copts = _copts(o)
        self.ids = torch.empty((B, k), dtype=torch.int32, device=dev)
        self.dists = torch.empty((B, k), dtype=torch.float32, device=dev)
        N, degree = graph.shape
        self._ws = _workspace(self._lib.cagra_search_workspace_bytes(N, degree, B, k, itopk, search_width,
                                                                     C.byref(self._copts)), dev)
        # the workspace belongs to this object alone: cleaned once here, handed back clean by every search, so every
        # call may vouch for it (multi mode: one kernel launch per call)
        _check(self._lib.cagra_search_workspace_init(N, degree, dataset.shape[1], B, k, itopk, search_width,
                                                     C.byref(self._copts), self._ws.data_ptr(), self._ws.numel(),
                                                     _stream(dev)), "cagra_search_workspace_init")
        self._copts.workspace_clean = 1
        self._keep = (graph, dataset, queries)          # the call holds raw pointers into these
        self._device = dev
        self._shape = tuple(queries.shape)
        self._args = (graph.data_ptr(), N, degree, dataset.data_ptr(), dataset.shape[1], dataset.stride(0), metric,
                      queries.data_ptr(), B, queries.stride(0), k, itopk, search_width, C.byref(self._copts),
                      self.ids.data_ptr(), self.dists.data_ptr(), self._ws.data_ptr(), self._ws.numel())

    def __call__(self, queries=None):
        args = self._args
        if queries is not None:
            queries = _dev_f32(queries, "queries")
            if tuple(queries.shape) != self._shape or queries.device != self._device:
                raise ValueError("queries must have the shape and device this call was prepared for")
            args = args[:7] + (queries.data_ptr(), args[8], queries.stride(0)) + args[10:]
        rc = self._lib.cagra_search(*args, _stream(self._device))
        if rc != 0:
            _check(rc, "cagra_search")
        return self.ids, self.dists


def exact_search(dataset, queries, k: int, metric: int = L2, exclude_self: bool = False,
                 self_offset: int = 0, return_dists: bool = True, algo: int = EXACT_AUTO, blocks_redone=None):
    """Exhaustive k nearest neighbours (Eq. 1): (ids[B, k] int32, dists[B, k] float32).  algo: EXACT_PLAIN,
    EXACT_FILTERED (matrix-core filter in front of the exact arithmetic, same result) or EXACT_AUTO.
    blocks_redone: optional int32 tensor of one element that receives how many blocks of query rows the
    filtered algorithm had to hand to the plain kernels."""
    torch = _torch()
    lib = load_library()
    dataset = _dev_f32(dataset, "dataset")
    queries = _dev_f32(queries, "queries")
    dev = dataset.device
    B, N = queries.shape[0], dataset.shape[0]
    ids = torch.empty((B, k), dtype=torch.int32, device=dev)
    dists = torch.empty((B, k), dtype=torch.float32, device=dev) if return_dists else None
    ws = _workspace(lib.cagra_exact_search_ex_workspace_bytes(N, dataset.shape[1], B, k, algo), dev)
    rc = lib.cagra_exact_search_ex(dataset.data_ptr(), N, dataset.shape[1], dataset.stride(0), metric,
                                   queries.data_ptr(), B, queries.stride(0), k, int(exclude_self),
                                   self_offset, algo, ids.data_ptr(),
                                   dists.data_ptr() if dists is not None else None,
                                   blocks_redone.data_ptr() if blocks_redone is not None else None,
                                   ws.data_ptr(), ws.numel(), _stream(dev))
    _check(rc, "cagra_exact_search_ex")
    return (ids, dists) if return_dists else ids


def build(dataset, degree: int, init_degree: int = 0, metric: int = L2, reorder: int = REORDER_RANK,
          nn_descent: bool = False, nnd_rounds: int = 0, nnd_sample: int = 0, seed: int = 0,
          exact_algo: int = EXACT_AUTO):
    """dataset[N, dim] -> CAGRA graph[N, degree] (int32 tensor).  nn_descent: initial graph by
    NN-descent instead of the exhaustive search; exact_algo: how the exhaustive search computes."""
    torch = _torch()
    lib = load_library()
    dataset = _dev_f32(dataset, "dataset")
    dev = dataset.device
    N, dim = dataset.shape
    graph = torch.empty((N, degree), dtype=torch.int32, device=dev)
    bo = _BuildOpts(reorder, 1 if nn_descent else 0, nnd_rounds, nnd_sample, seed, exact_algo, 0)
    ws = _workspace(lib.cagra_build_ex_workspace_bytes(N, dim, degree, init_degree, C.byref(bo)), dev)
    rc = lib.cagra_build_ex(dataset.data_ptr(), N, dim, dataset.stride(0), metric, degree, init_degree, C.byref(bo),
                            graph.data_ptr(), ws.data_ptr(), ws.numel(), _stream(dev))
    _check(rc, "cagra_build_ex")
    return graph


def nn_descent(dataset, k: int, rounds: int = -1, sample: int = 0, metric: int = L2, seed: int = 0):
    """Approximate k-NN graph by NN-descent in synchronous rounds: (ids[N, k] int32, dists[N, k]),
    rows sorted by (distance, id).  rounds < 0: automatic; rounds = 0: only the random initial lists."""
    torch = _torch()
    lib = load_library()
    dataset = _dev_f32(dataset, "dataset")
    dev = dataset.device
    N, dim = dataset.shape
    ids = torch.empty((N, k), dtype=torch.int32, device=dev)
    dists = torch.empty((N, k), dtype=torch.float32, device=dev)
    ws = _workspace(lib.cagra_nn_descent_workspace_bytes(N, k, sample), dev)
    rc = lib.cagra_nn_descent(dataset.data_ptr(), N, dim, dataset.stride(0), metric, k, rounds, sample, seed,
                              ids.data_ptr(), dists.data_ptr(), ws.data_ptr(), ws.numel(), _stream(dev))
    _check(rc, "cagra_nn_descent")
    return ids, dists


def optimize(knn, degree: int, return_stages: bool = False, knn_dists=None):
    """Sorted k-NN graph[N, init_degree] -> CAGRA graph[N, degree]; optionally also the
    pruned graph, the reversed graph and its list lengths.  With knn_dists[N, init_degree]
    the reordering is distance-based, else rank-based."""
    torch = _torch()
    lib = load_library()
    knn = _dev_i32(knn, "knn")
    if knn_dists is not None:
        knn_dists = _dev_f32(knn_dists, "knn_dists")
        if knn_dists.shape != knn.shape or not knn_dists.is_contiguous():
            raise TypeError("knn_dists must be contiguous and shaped like knn")
    dev = knn.device
    N, init_degree = knn.shape
    graph = torch.empty((N, degree), dtype=torch.int32, device=dev)
    pruned = rev = rlen = None
    if return_stages:
        pruned = torch.empty((N, degree), dtype=torch.int32, device=dev)
        rev = torch.empty((N, degree), dtype=torch.int32, device=dev)
        rlen = torch.empty((N,), dtype=torch.int32, device=dev)
    ws = _workspace(lib.cagra_optimize_workspace_bytes(N, init_degree, degree), dev)
    rc = lib.cagra_optimize_ex(knn.data_ptr(), knn_dists.data_ptr() if knn_dists is not None else None,
                               N, init_degree, degree,
                               REORDER_DISTANCE if knn_dists is not None else REORDER_RANK, graph.data_ptr(),
                               pruned.data_ptr() if pruned is not None else None,
                               rev.data_ptr() if rev is not None else None,
                               rlen.data_ptr() if rlen is not None else None,
                               ws.data_ptr(), ws.numel(), _stream(dev))
    _check(rc, "cagra_optimize_ex")
    return (graph, pruned, rev, rlen) if return_stages else graph
