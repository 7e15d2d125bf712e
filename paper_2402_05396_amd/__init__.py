"""MI355X-native temporal neighbor finder + feature gather (TASER, arXiv 2402.05396).

Thin ctypes binding over ``libtaser.so`` (C ABI declared in ``include/taser.h``).
The functions here carry the same names as the C entry points and only marshal
arguments: torch supplies device memory and the current stream, every step of
the path runs in the library's HIP kernels. There is no fallback: if the
library has not been built, or no GPU is present, calls raise.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtaser.so")

RECENT, UNIFORM, WEIGHTED, INVERSE_TIMESPAN = 0, 1, 2, 3
INPUT_ON_DEVICE = 1
MAX_K, MAX_M, MAX_HOPS = 64, 64, 3

EXPORTS = ("taser_tcsr_build", "taser_tcsr_size", "taser_tcsr_view", "taser_tcsr_free", "taser_sample_temporal", "taser_sample_temporal_rows",
           "taser_candidate_encodings", "taser_select_weighted", "taser_gather_features", "taser_cache_init", "taser_cache_lookup", "taser_cache_lookup_static", "taser_cache_prefetch", "taser_cache_gather", "taser_cache_tune", "taser_cache_count_accesses", "taser_cache_access_counts",
           "taser_cache_epoch_end", "taser_cache_residents",
           "taser_cache_free", "taser_selector_init", "taser_selector_draw", "taser_selector_update",
           "taser_selector_scores", "taser_selector_size", "taser_selector_free", "taser_profile_begin", "taser_profile_begin_only", "taser_profile_end", "taser_last_error")


class TaserError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"taser error {code}: {message}")
        self.code = code


class _KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char_p), ("launches", ctypes.c_int64), ("total_ms", ctypes.c_double)]


class _HopOut(ctypes.Structure):
    _fields_ = [("nbr", ctypes.c_void_p), ("eid", ctypes.c_void_p), ("ts", ctypes.c_void_p),
                ("count", ctypes.c_void_p)]


_lib = None


def lib():
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2402_05396_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, u32, u64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint64
        L.taser_tcsr_build.argtypes = [vp, vp, vp, vp, i64, i32, u32, vp, ctypes.POINTER(vp)]
        L.taser_tcsr_size.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.taser_tcsr_view.argtypes = [vp, vp, vp, vp, vp, vp]
        L.taser_tcsr_free.argtypes = [vp]
        L.taser_tcsr_free.restype = None
        L.taser_sample_temporal.argtypes = [vp, vp, vp, i64, i32, i32, i32, u64, i32, vp,
                                            ctypes.POINTER(_HopOut), vp]
        L.taser_sample_temporal_rows.argtypes = [vp, vp, vp, i64, i32, i32, i32, u64, i32, vp, vp, i64, i32, i64,
                                                 ctypes.POINTER(_HopOut), ctypes.POINTER(vp), vp]
        L.taser_candidate_encodings.argtypes = [vp, vp, i64, i32, vp, vp, vp]
        L.taser_select_weighted.argtypes = [vp, vp, i64, i32, i32, u64, u32, vp, vp, ctypes.POINTER(_HopOut),
                                            ctypes.POINTER(_HopOut), vp]
        L.taser_gather_features.argtypes = [vp, i64, i32, i64, vp, i64, vp, vp]
        L.taser_cache_init.argtypes = [vp, i64, i32, i64, i64, vp, u64, i64, vp, ctypes.POINTER(vp)]
        L.taser_cache_lookup.argtypes = [vp, vp, i64, vp, vp, vp]
        L.taser_cache_lookup_static.argtypes = [vp, vp, i64, vp, vp, vp]
        L.taser_cache_prefetch.argtypes = [vp, vp, i64, vp, vp]
        L.taser_cache_gather.argtypes = [vp, vp, i64, vp, vp]
        L.taser_cache_tune.argtypes = [vp, i32, i32, i32]
        L.taser_cache_count_accesses.argtypes = [vp, i32, vp]
        L.taser_cache_access_counts.argtypes = [vp, vp, vp]
        L.taser_cache_epoch_end.argtypes = [vp, i64, ctypes.POINTER(i64), ctypes.POINTER(i32), vp]
        L.taser_cache_residents.argtypes = [vp, vp]
        L.taser_cache_free.argtypes = [vp]
        L.taser_cache_free.restype = None
        L.taser_selector_init.argtypes = [vp, i64, u32, vp, ctypes.POINTER(vp)]
        L.taser_selector_draw.argtypes = [vp, i64, u64, u64, vp, vp]
        L.taser_selector_update.argtypes = [vp, vp, vp, i64, vp]
        L.taser_selector_scores.argtypes = [vp, vp, ctypes.POINTER(u64), vp]
        L.taser_selector_size.argtypes = [vp, ctypes.POINTER(i64)]
        L.taser_selector_free.argtypes = [vp]
        L.taser_selector_free.restype = None
        L.taser_profile_begin.argtypes = []
        L.taser_profile_begin_only.argtypes = [ctypes.c_char_p]
        L.taser_profile_end.argtypes = [ctypes.POINTER(_KernelTime), i32, ctypes.POINTER(i32)]
        L.taser_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def last_error():
    return lib().taser_last_error().decode()


def _check(rc):
    if rc != 0:
        raise TaserError(rc, last_error())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _want(t, dtype, name, cuda=True):
    if t.dtype != dtype or not t.is_contiguous() or t.is_cuda != cuda:
        raise TypeError(f"{name}: expected a contiguous {'device' if cuda else 'host'} tensor of {dtype}")
    return t


class TCSR:
    """Owner of a taser_tcsr handle."""

    def __init__(self, handle, num_entries, num_nodes):
        self.handle, self.num_entries, self.num_nodes = handle, num_entries, num_nodes

    def free(self):
        if self.handle:
            lib().taser_tcsr_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def tcsr_build(src, dst, ts, eid, num_nodes, stream=None):
    """taser_tcsr_build. src/dst/eid int32, ts int64; all on the GPU or all on the host."""
    on_dev = src.is_cuda
    _want(src, torch.int32, "src", on_dev)
    _want(dst, torch.int32, "dst", on_dev)
    _want(ts, torch.int64, "ts", on_dev)
    if eid is not None:
        _want(eid, torch.int32, "eid", on_dev)
    n = src.numel()
    if dst.numel() != n or ts.numel() != n or (eid is not None and eid.numel() != n):
        raise ValueError("src, dst, ts, eid must have the same length")
    h = ctypes.c_void_p()
    _check(lib().taser_tcsr_build(_ptr(src), _ptr(dst), _ptr(ts), _ptr(eid), n, num_nodes,
                                  INPUT_ON_DEVICE if on_dev else 0, _stream(stream), ctypes.byref(h)))
    return TCSR(h, n, num_nodes)


def tcsr_size(g):
    """taser_tcsr_size -> (num_entries, num_nodes)."""
    ne, nn = ctypes.c_int64(), ctypes.c_int32()
    _check(lib().taser_tcsr_size(g.handle, ctypes.byref(ne), ctypes.byref(nn)))
    return ne.value, nn.value


def tcsr_view(g, stream=None):
    """taser_tcsr_view -> (indptr, nbr, ts, eid) as plain device tensors."""
    n, dev = g.num_entries, "cuda"
    indptr = torch.empty(g.num_nodes + 1, dtype=torch.int64, device=dev)
    nbr = torch.empty(n, dtype=torch.int32, device=dev)
    ts = torch.empty(n, dtype=torch.int64, device=dev)
    eid = torch.empty(n, dtype=torch.int32, device=dev)
    _check(lib().taser_tcsr_view(g.handle, _ptr(indptr), _ptr(nbr), _ptr(ts), _ptr(eid), _stream(stream)))
    return indptr, nbr, ts, eid


def tcsr_free(g):
    g.free()


def sample_outputs(n, k, hops, device):
    """Freshly allocated output tensors of a `hops`-hop call on n roots."""
    out, r = [], n
    for _ in range(max(hops, 0)):
        out.append(dict(nbr=torch.empty((r, k), dtype=torch.int32, device=device),
                        eid=torch.empty((r, k), dtype=torch.int32, device=device),
                        ts=torch.empty((r, k), dtype=torch.int64, device=device),
                        count=torch.empty((r,), dtype=torch.int32, device=device)))
        r *= k
    return out


def _hop_array(roots, times, n, k, edge_weight, out):
    """Checks the sampler's tensors and packs the per-hop output pointers."""
    _want(roots, torch.int32, "roots")
    _want(times, torch.int64, "times")
    if edge_weight is not None:
        _want(edge_weight, torch.int32, "edge_weight (uint32 bits in an int32 tensor)")
    if times.numel() != n:
        raise ValueError("roots and times must have the same length")
    arr = (_HopOut * max(len(out), 1))()
    r = n
    for h, o in enumerate(out):
        for name, dt, cnt in (("nbr", torch.int32, r * k), ("eid", torch.int32, r * k), ("ts", torch.int64, r * k),
                              ("count", torch.int32, r)):
            _want(o[name], dt, f"out[{h}].{name}")
            if o[name].numel() < cnt:
                raise ValueError(f"out[{h}].{name} is too small")
            setattr(arr[h], name, o[name].data_ptr())
        r *= k
    return arr


def sample_temporal(g, roots, times, k, hops, policy, seed, m=0, edge_weight=None, out=None, stream=None):
    """taser_sample_temporal. Returns a list of `hops` dicts of device tensors
    nbr/eid/ts [R_h, k] and count [R_h] (allocated here unless `out` is given)."""
    n = roots.numel()
    if out is None:
        out = sample_outputs(n, k, hops, roots.device)
    arr = _hop_array(roots, times, n, k, edge_weight, out)
    _check(lib().taser_sample_temporal(g.handle, _ptr(roots), _ptr(times), n, k, hops, policy, seed, m,
                                       _ptr(edge_weight), arr, _stream(stream)))
    return out


def sample_temporal_rows(g, roots, times, k, hops, policy, seed, table, m=0, edge_weight=None, out=None, rows_out=None,
                         row_elems=None, stream=None):
    """taser_sample_temporal_rows: sample_temporal plus, per hop, the rows of `table`
    (2-D device tensor with contiguous rows, as for gather_features) of the sampled edge
    ids. Returns (out, rows_out); rows_out[h] is [R_h * k, d] of the table's dtype."""
    if table.dim() != 2 or table.stride(1) != 1 or not table.is_cuda:
        raise TypeError("table: expected a 2-D device tensor with contiguous rows")
    n = roots.numel()
    es = table.element_size()
    d = table.shape[1] if row_elems is None else row_elems
    if out is None:
        out = sample_outputs(n, k, hops, roots.device)
    if rows_out is None:
        rows_out = [torch.empty((o["eid"].numel(), d), dtype=table.dtype, device=table.device) for o in out]
    arr = _hop_array(roots, times, n, k, edge_weight, out)
    ptrs = (ctypes.c_void_p * max(len(rows_out), 1))()
    r = n
    for h, t in enumerate(rows_out):
        r *= k
        if t.dtype != table.dtype or not t.is_contiguous() or t.numel() < r * d:
            raise TypeError(f"rows_out[{h}]: expected a contiguous device tensor of the table's dtype with R_h*k*d elements")
        ptrs[h] = t.data_ptr()
    _check(lib().taser_sample_temporal_rows(g.handle, _ptr(roots), _ptr(times), n, k, hops, policy, seed, m,
                                            _ptr(edge_weight), _ptr(table), table.shape[0], d * es, table.stride(0) * es,
                                            arr, ptrs, _stream(stream)))
    return out, rows_out


def candidate_encodings(nbr, count, want_identity=True, stream=None):
    """taser_candidate_encodings. nbr int32[R, m], count int32[R] ->
    (freq int32[R, m], identity uint8[R, m, m] or None)."""
    _want(nbr, torch.int32, "nbr")
    _want(count, torch.int32, "count")
    if nbr.dim() != 2 or count.numel() != nbr.shape[0]:
        raise ValueError("nbr must be [R, m] and count [R]")
    R, m = nbr.shape
    freq = torch.empty((R, m), dtype=torch.int32, device=nbr.device)
    ident = torch.empty((R, m, m), dtype=torch.uint8, device=nbr.device) if want_identity else None
    _check(lib().taser_candidate_encodings(_ptr(nbr), _ptr(count), R, m, _ptr(freq), _ptr(ident), _stream(stream)))
    return freq, ident


def select_weighted(weight, count, k, seed, hop, candidates=None, stream=None):
    """taser_select_weighted. weight int32[R, m] (uint32 bits), count int32[R] ->
    (sel int32[R, k], out_count int32[R], kept). With `candidates` (a dict of
    nbr/eid/ts [R, m] as sample_temporal returns) kept is a dict of nbr/eid/ts
    [R, k] and count, else None."""
    _want(weight, torch.int32, "weight (uint32 bits in an int32 tensor)")
    _want(count, torch.int32, "count")
    if weight.dim() != 2 or count.numel() != weight.shape[0]:
        raise ValueError("weight must be [R, m] and count [R]")
    R, m = weight.shape
    d = weight.device
    sel = torch.empty((R, k), dtype=torch.int32, device=d)
    out_count = torch.empty((R,), dtype=torch.int32, device=d)
    cand_arg = kept_arg = kept = None
    if candidates is not None:
        for name, dt in (("nbr", torch.int32), ("eid", torch.int32), ("ts", torch.int64)):
            _want(candidates[name], dt, f"candidates.{name}")
            if candidates[name].numel() != R * m:
                raise ValueError(f"candidates.{name} must hold R*m elements")
        kept = dict(nbr=torch.empty((R, k), dtype=torch.int32, device=d),
                    eid=torch.empty((R, k), dtype=torch.int32, device=d),
                    ts=torch.empty((R, k), dtype=torch.int64, device=d), count=out_count)
        cand_arg, kept_arg = _HopOut(), _HopOut()
        for name in ("nbr", "eid", "ts"):
            setattr(cand_arg, name, candidates[name].data_ptr())
            setattr(kept_arg, name, kept[name].data_ptr())
        cand_arg, kept_arg = ctypes.byref(cand_arg), ctypes.byref(kept_arg)
    _check(lib().taser_select_weighted(_ptr(weight), _ptr(count), R, m, k, seed, hop, _ptr(sel), _ptr(out_count),
                                       cand_arg, kept_arg, _stream(stream)))
    return sel, out_count, kept


def gather_features(table, ids, out=None, row_elems=None, stream=None):
    """taser_gather_features. table: 2-D device tensor whose rows are contiguous
    (row pitch = table.stride(0)); the first `row_elems` columns are gathered."""
    if table.dim() != 2 or table.stride(1) != 1 or not table.is_cuda:
        raise TypeError("table: expected a 2-D device tensor with contiguous rows")
    _want(ids, torch.int32, "ids")
    es = table.element_size()
    d = table.shape[1] if row_elems is None else row_elems
    n = ids.numel()
    if out is None:
        out = torch.empty((n, d), dtype=table.dtype, device=table.device)
    elif out.dtype != table.dtype or not out.is_contiguous() or out.numel() < n * d:
        raise TypeError("out: expected a contiguous device tensor of the table's dtype with n*d elements")
    _check(lib().taser_gather_features(_ptr(table), table.shape[0], d * es, table.stride(0) * es, _ptr(ids), n,
                                       _ptr(out), _stream(stream)))
    return out


class Cache:
    """Owner of a taser_cache handle (keeps the pinned host table alive)."""

    def __init__(self, handle, host_table, capacity, row_elems):
        self.handle, self.host_table, self.capacity, self.row_elems = handle, host_table, capacity, row_elems

    def free(self):
        if self.handle:
            lib().taser_cache_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def cache_init(host_table, capacity_rows, resident_ids=None, seed=0, staging_rows=0, stream=None):
    """taser_cache_init. host_table: 2-D pinned host tensor with contiguous rows;
    resident_ids: host int32 tensor or None."""
    if host_table.dim() != 2 or host_table.stride(1) != 1 or host_table.is_cuda:
        raise TypeError("host_table: expected a 2-D host tensor with contiguous rows")
    if resident_ids is not None:
        _want(resident_ids, torch.int32, "resident_ids", cuda=False)
        if resident_ids.numel() != capacity_rows:
            raise ValueError("resident_ids must hold capacity_rows ids")
    es = host_table.element_size()
    h = ctypes.c_void_p()
    _check(lib().taser_cache_init(_ptr(host_table), host_table.shape[0], host_table.shape[1] * es,
                                  host_table.stride(0) * es, capacity_rows, _ptr(resident_ids), seed,
                                  staging_rows, _stream(stream), ctypes.byref(h)))
    return Cache(h, host_table, capacity_rows, host_table.shape[1])


def cache_lookup(c, ids, out=None, hit_miss=None, stream=None):
    """taser_cache_lookup. hit_miss: device int64[2] tensor that is incremented, or None."""
    _want(ids, torch.int32, "ids")
    n = ids.numel()
    if out is None:
        out = torch.empty((n, c.row_elems), dtype=c.host_table.dtype, device=ids.device)
    elif out.dtype != c.host_table.dtype or not out.is_contiguous() or out.numel() < n * c.row_elems:
        raise TypeError("out: expected a contiguous device tensor of the table's dtype with n*d elements")
    if hit_miss is not None:
        _want(hit_miss, torch.int64, "hit_miss")
    _check(lib().taser_cache_lookup(c.handle, _ptr(ids), n, _ptr(out), _ptr(hit_miss), _stream(stream)))
    return out


def cache_lookup_static(c, ids, out, hit_miss=None, stream=None):
    """taser_cache_lookup_static: the lookup that allocates nothing (`out` must be given)."""
    _want(ids, torch.int32, "ids")
    n = ids.numel()
    if out.dtype != c.host_table.dtype or not out.is_contiguous() or out.numel() < n * c.row_elems:
        raise TypeError("out: expected a contiguous device tensor of the table's dtype with n*d elements")
    if hit_miss is not None:
        _want(hit_miss, torch.int64, "hit_miss")
    _check(lib().taser_cache_lookup_static(c.handle, _ptr(ids), n, _ptr(out), _ptr(hit_miss), _stream(stream)))
    return out


def cache_prefetch(c, ids, hit_miss=None, stream=None):
    """taser_cache_prefetch: classify the requests and stage the missing rows."""
    _want(ids, torch.int32, "ids")
    if hit_miss is not None:
        _want(hit_miss, torch.int64, "hit_miss")
    _check(lib().taser_cache_prefetch(c.handle, _ptr(ids), ids.numel(), _ptr(hit_miss), _stream(stream)))


def cache_gather(c, ids, out=None, stream=None):
    """taser_cache_gather: the dense output for the ids of the latest cache_prefetch."""
    _want(ids, torch.int32, "ids")
    n = ids.numel()
    if out is None:
        out = torch.empty((n, c.row_elems), dtype=c.host_table.dtype, device=ids.device)
    elif out.dtype != c.host_table.dtype or not out.is_contiguous() or out.numel() < n * c.row_elems:
        raise TypeError("out: expected a contiguous device tensor of the table's dtype with n*d elements")
    _check(lib().taser_cache_gather(c.handle, _ptr(ids), n, _ptr(out), _stream(stream)))
    return out


def cache_tune(c, stage_blocks=0, refresh_before_gather=False, partitioned_gather=None):
    """taser_cache_tune (partitioned_gather None keeps the current setting)."""
    _check(lib().taser_cache_tune(c.handle, stage_blocks, 1 if refresh_before_gather else 0,
                                  -1 if partitioned_gather is None else int(partitioned_gather)))


def cache_count_accesses(c, enable=True, stream=None):
    """taser_cache_count_accesses."""
    _check(lib().taser_cache_count_accesses(c.handle, 1 if enable else 0, _stream(stream)))


def cache_access_counts(c, stream=None):
    """taser_cache_access_counts -> device int32 tensor holding the uint32 counters."""
    out = torch.empty(c.host_table.shape[0], dtype=torch.int32, device="cuda")
    _check(lib().taser_cache_access_counts(c.handle, _ptr(out), _stream(stream)))
    return out


def cache_epoch_end(c, min_overlap, stream=None):
    """taser_cache_epoch_end -> (replaced, overlap)."""
    overlap, replaced = ctypes.c_int64(), ctypes.c_int32()
    _check(lib().taser_cache_epoch_end(c.handle, min_overlap, ctypes.byref(overlap), ctypes.byref(replaced),
                                       _stream(stream)))
    return bool(replaced.value), int(overlap.value)


def cache_residents(c):
    out = torch.empty(c.capacity, dtype=torch.int32)
    _check(lib().taser_cache_residents(c.handle, _ptr(out)))
    return out


def cache_free(c):
    c.free()


class Selector:
    """Owner of a taser_selector handle."""

    def __init__(self, handle, n):
        self.handle, self.n = handle, n

    def free(self):
        if self.handle:
            lib().taser_selector_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def selector_init(scores=None, n=None, initial_score=1, stream=None):
    """taser_selector_init. scores: device int32 tensor holding uint32 bits, or None with n."""
    if scores is not None:
        _want(scores, torch.int32, "scores (uint32 bits in an int32 tensor)")
        n = scores.numel()
    h = ctypes.c_void_p()
    _check(lib().taser_selector_init(_ptr(scores), n, initial_score, _stream(stream), ctypes.byref(h)))
    return Selector(h, n)


def selector_draw(s, b, seed, iteration, out=None, stream=None):
    """taser_selector_draw -> device int32[b] edge indices."""
    if out is None:
        out = torch.empty(b, dtype=torch.int32, device="cuda")
    else:
        _want(out, torch.int32, "out")
        if out.numel() < b:
            raise ValueError("out is too small")
    _check(lib().taser_selector_draw(s.handle, b, seed, iteration, _ptr(out), _stream(stream)))
    return out


def selector_update(s, batch, new_scores, stream=None):
    """taser_selector_update."""
    _want(batch, torch.int32, "batch")
    _want(new_scores, torch.int32, "new_scores (uint32 bits in an int32 tensor)")
    if batch.numel() != new_scores.numel():
        raise ValueError("batch and new_scores must have the same length")
    _check(lib().taser_selector_update(s.handle, _ptr(batch), _ptr(new_scores), batch.numel(), _stream(stream)))


def selector_scores(s, want_total=True, stream=None):
    """taser_selector_scores -> (device int32[n] holding the uint32 scores, total or None)."""
    out = torch.empty(s.n, dtype=torch.int32, device="cuda")
    total = ctypes.c_uint64()
    _check(lib().taser_selector_scores(s.handle, _ptr(out), ctypes.byref(total) if want_total else None,
                                       _stream(stream)))
    return out, (int(total.value) if want_total else None)


def selector_size(s):
    n = ctypes.c_int64()
    _check(lib().taser_selector_size(s.handle, ctypes.byref(n)))
    return n.value


def selector_free(s):
    s.free()


def profile_begin():
    """taser_profile_begin: start timing every kernel the library launches."""
    _check(lib().taser_profile_begin())


def profile_begin_only(kernel_name):
    """taser_profile_begin_only: time only the kernel of this name."""
    _check(lib().taser_profile_begin_only(kernel_name.encode() if kernel_name else None))


def profile_end(max_entries=64):
    """taser_profile_end -> {kernel name: (launches, total device ms)}."""
    arr = (_KernelTime * max_entries)()
    n = ctypes.c_int32()
    _check(lib().taser_profile_end(arr, max_entries, ctypes.byref(n)))
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms)) for i in range(n.value)}
