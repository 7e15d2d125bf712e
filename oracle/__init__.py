"""CPU oracle — TEST INFRASTRUCTURE, NOT PRODUCT CODE.

ctypes front end of ``oracle/oracle.cpp``: a plain CPU implementation of the
temporal neighbor finder + feature gather of TASER (arXiv 2402.05396), written
from the paper and independent of the HIP library (no shared code). Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product package never does.

numpy arrays in, numpy arrays out. ``threads`` > 1 runs the same per-root loop
under a static OpenMP parallel-for (results do not depend on it).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")

RECENT, UNIFORM, WEIGHTED, INVERSE_TIMESPAN = 0, 1, 2, 3


def build(force=False):
    """Compile oracle.cpp with g++ (no HIP headers, no GPU)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_draw64.restype = ctypes.c_uint64
        _lib.oracle_draw64.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64,
                                       ctypes.c_uint32]
        _lib.oracle_mulhi64.restype = ctypes.c_uint64
        _lib.oracle_mulhi64.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _c(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def max_threads():
    return int(_load().oracle_max_threads())


def philox4x32_10(ctr, key):
    ctr = _c(ctr, np.uint32)
    key = _c(key, np.uint32)
    out = np.empty(4, np.uint32)
    _load().oracle_philox4x32_10(_p(ctr), _p(key), _p(out))
    return out


def draw64(seed, hop, root, slot):
    return int(_load().oracle_draw64(seed, hop, root, slot))


def mulhi64(u, n):
    return int(_load().oracle_mulhi64(u, n))


def tcsr_build(src, dst, ts, eid, num_nodes, threads=1):
    """Return (indptr int64[N+1], nbr int32[E'], ts int64[E'], eid int32[E'])."""
    src, dst, ts, eid = _c(src, np.int32), _c(dst, np.int32), _c(ts, np.int64), _c(eid, np.int32)
    n = src.shape[0]
    indptr = np.empty(num_nodes + 1, np.int64)
    o_nbr = np.empty(n, np.int32)
    o_ts = np.empty(n, np.int64)
    o_eid = np.empty(n, np.int32)
    rc = _load().oracle_tcsr_build(_p(src), _p(dst), _p(ts), _p(eid), ctypes.c_int64(n),
                                   ctypes.c_int32(num_nodes), _p(indptr), _p(o_nbr), _p(o_ts),
                                   _p(o_eid), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError("oracle_tcsr_build: node id out of range")
    return indptr, o_nbr, o_ts, o_eid


def sample_temporal(tcsr, roots, times, k, hops, policy, seed, m=0, edge_weight=None, threads=1):
    """Return a list of `hops` dicts with nbr/eid/ts [R*k^h, k] and count [R*k^h]."""
    indptr, nbr, ts, eid = tcsr
    roots, times = _c(roots, np.int32), _c(times, np.int64)
    edge_weight = _c(edge_weight, np.uint32)
    num_nodes = indptr.shape[0] - 1
    outs, n = [], roots.shape[0]
    for _ in range(hops):
        outs.append(dict(nbr=np.empty((n, k), np.int32), eid=np.empty((n, k), np.int32),
                         ts=np.empty((n, k), np.int64), count=np.empty(n, np.int32)))
        n *= k

    def ptrs(name):
        return (ctypes.c_void_p * hops)(*[o[name].ctypes.data for o in outs])

    rc = _load().oracle_sample_temporal(
        _p(indptr), _p(nbr), _p(ts), _p(eid), ctypes.c_int32(num_nodes), _p(roots), _p(times),
        ctypes.c_int64(roots.shape[0]), ctypes.c_int32(k), ctypes.c_int32(hops),
        ctypes.c_int32(policy), ctypes.c_uint64(seed), ctypes.c_int32(m), _p(edge_weight),
        ptrs("nbr"), ptrs("eid"), ptrs("ts"), ptrs("count"), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError("oracle_sample_temporal: bad argument")
    return outs


def sample_hop(tcsr, roots, times, k, policy, seed, hop, m=0, edge_weight=None, threads=1):
    """One hop with an explicit hop tag for the random draws."""
    indptr, nbr, ts, eid = tcsr
    roots, times = _c(roots, np.int32), _c(times, np.int64)
    edge_weight = _c(edge_weight, np.uint32)
    n = roots.shape[0]
    o = dict(nbr=np.empty((n, k), np.int32), eid=np.empty((n, k), np.int32),
             ts=np.empty((n, k), np.int64), count=np.empty(n, np.int32))
    rc = _load().oracle_sample_hop(
        _p(indptr), _p(nbr), _p(ts), _p(eid), ctypes.c_int32(indptr.shape[0] - 1), _p(roots),
        _p(times), ctypes.c_int64(n), ctypes.c_int32(k), ctypes.c_int32(policy),
        ctypes.c_uint64(seed), ctypes.c_uint32(hop), ctypes.c_int32(m), _p(edge_weight),
        _p(o["nbr"]), _p(o["eid"]), _p(o["ts"]), _p(o["count"]), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError("oracle_sample_hop: bad argument")
    return o


def gather(table, ids, row_bytes=None, threads=1):
    """table: 2-D C-contiguous-rows numpy array (any dtype, row pitch = strides[0]).
    Returns a dense [n, row_elems] array of the same dtype."""
    assert table.ndim == 2 and table.strides[1] == table.itemsize
    ids = _c(ids, np.int32).ravel()
    rb = table.shape[1] * table.itemsize if row_bytes is None else row_bytes
    out = np.empty((ids.shape[0], rb // table.itemsize), table.dtype)
    rc = _load().oracle_gather(ctypes.c_void_p(table.ctypes.data), ctypes.c_int64(table.shape[0]),
                               ctypes.c_int32(rb), ctypes.c_int64(table.strides[0]), _p(ids),
                               ctypes.c_int64(ids.shape[0]), _p(out), ctypes.c_int(threads))
    if rc != 0:
        raise ValueError("oracle_gather: id out of range")
    return out


def cache_random_residents(rows, capacity, seed):
    out = np.empty(capacity, np.int32)
    _load().oracle_cache_random_residents(ctypes.c_int64(rows), ctypes.c_int64(capacity),
                                          ctypes.c_uint64(seed), _p(out))
    return out


def cache_hits(resident, rows, ids):
    resident, ids = _c(resident, np.int32), _c(ids, np.int32).ravel()
    hm = np.zeros(2, np.uint64)
    _load().oracle_cache_hits(_p(resident), ctypes.c_int64(resident.shape[0]),
                              ctypes.c_int64(rows), _p(ids), ctypes.c_int64(ids.shape[0]), _p(hm))
    return int(hm[0]), int(hm[1])


def cache_count(ids, rows, Q):
    """Q[id] += 1 for every valid request (in place; Q is uint32[rows])."""
    ids = _c(ids, np.int32).ravel()
    assert Q.dtype == np.uint32 and Q.flags.c_contiguous and Q.shape[0] == rows
    _load().oracle_cache_count(_p(ids), ctypes.c_int64(ids.shape[0]), ctypes.c_int64(rows), _p(Q))


def cache_epoch_end(Q, resident, min_overlap):
    """Returns (replaced, overlap, new_resident); clears Q in place."""
    resident = _c(resident, np.int32)
    assert Q.dtype == np.uint32 and Q.flags.c_contiguous
    new = np.empty_like(resident)
    overlap = ctypes.c_int64()
    rep = _load().oracle_cache_epoch_end(_p(Q), ctypes.c_int64(Q.shape[0]), _p(resident),
                                         ctypes.c_int64(resident.shape[0]), ctypes.c_int64(min_overlap),
                                         _p(new), ctypes.byref(overlap))
    return bool(rep), int(overlap.value), new


def candidate_encodings(nbr, count, want_identity=True):
    """nbr int32[R, m], count int32[R] -> (freq int32[R, m], identity uint8[R, m, m] or None)."""
    nbr, count = _c(nbr, np.int32), _c(count, np.int32)
    R, m = nbr.shape
    freq = np.empty((R, m), np.int32)
    ident = np.empty((R, m, m), np.uint8) if want_identity else None
    _load().oracle_candidate_encodings(_p(nbr), _p(count), ctypes.c_int64(R), ctypes.c_int32(m), _p(freq), _p(ident))
    return freq, ident


def select_weighted(weight, count, k, seed, hop):
    """weight uint32[R, m], count int32[R] -> (sel int32[R, k], out_count int32[R])."""
    weight, count = _c(weight, np.uint32), _c(count, np.int32)
    R, m = weight.shape
    sel = np.empty((R, k), np.int32)
    out_count = np.empty(R, np.int32)
    _load().oracle_select_weighted(_p(weight), _p(count), ctypes.c_int64(R), ctypes.c_int32(m), ctypes.c_int32(k),
                                   ctypes.c_uint64(seed), ctypes.c_uint32(hop), _p(sel), _p(out_count))
    return sel, out_count


def batch_draw(score, b, seed, iteration):
    """score uint32[n] -> int32[b] edge indices drawn with probability score / sum(score)."""
    score = _c(score, np.uint32)
    out = np.empty(b, np.int32)
    _load().oracle_batch_draw(_p(score), ctypes.c_int64(score.shape[0]), ctypes.c_int64(b), ctypes.c_uint64(seed),
                              ctypes.c_uint64(iteration), _p(out))
    return out


def score_update(score, idx, value):
    """In place: score[idx[j]] = value[j] for j in order (score is uint32[n])."""
    assert score.dtype == np.uint32 and score.flags.c_contiguous
    idx, value = _c(idx, np.int32), _c(value, np.uint32)
    _load().oracle_score_update(_p(score), ctypes.c_int64(score.shape[0]), _p(idx), _p(value),
                                ctypes.c_int64(idx.shape[0]))
