"""ctypes binding of include/pag.h: argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpag_hip.so")

L2, IP, COS = 0, 1, 2
FLAG_NO_PRT = 1
FLAG_NO_PES = 2
FLAG_FP16_VECTORS = 4
FLAG_KEEP_ORDER = 8
FLAG_EXACT_TEST_COUNT = 16
FLAG_PERMUTATION_TRANSFORM = 32
FLAG_KEEP_QUERY_ORDER = 64
_METRICS = {"l2": L2, "ip": IP, "cos": COS, "cosine": COS, L2: L2, IP: IP, COS: COS}

EXPORTED_SYMBOLS = (
    "pag_build", "pag_search", "pag_search_static", "pag_insert", "pag_free", "pag_describe", "pag_export", "pag_import",
    "pag_get_counters", "pag_reset_counters", "pag_set_search_options", "pag_set_seen_capacity_log2",
    "pag_prepare_queries", "pag_exact_distances", "pag_screen", "pag_edge_info", "pag_insertion_candidates",
    "pag_measure_row_reads",
    "pag_searcher_create", "pag_searcher_search", "pag_searcher_get_counters", "pag_searcher_free",
    "pag_last_error",
)


class PagError(RuntimeError):
    pass


class _Params(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("metric", C.c_int32), ("max_degree", C.c_uint32),
                ("num_subspaces", C.c_uint32), ("ef_construction", C.c_uint32), ("search_b", C.c_uint32),
                ("insert_subbatch", C.c_uint32), ("flags", C.c_uint32), ("capacity", C.c_uint64),
                ("seed", C.c_uint64), ("stream", C.c_void_p)]


class _Arrays(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("metric", C.c_int32), ("n", C.c_uint64), ("d", C.c_uint32),
                ("num_subspaces", C.c_uint32), ("max_degree", C.c_uint32), ("n_entry", C.c_uint32),
                ("vectors", C.c_void_p), ("adj", C.c_void_p), ("a", C.c_void_p), ("c", C.c_void_p),
                ("e2", C.c_void_p), ("codes", C.c_void_p), ("rotation", C.c_void_p),
                ("codebooks", C.c_void_p), ("entry", C.c_void_p)]


class _Counters(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("adj_record_bytes", C.c_uint32)] + \
               [(k, C.c_uint64) for k in ("queries", "hops", "tests", "passes", "exact", "rounds",
                                          "rf_overflow", "rt_overflow", "seen_spills")] + \
               [("last_search_kernel_ms", C.c_double), ("last_prepare_ms", C.c_double),
                ("last_build_ms", C.c_double), ("phase_cycles", C.c_uint64 * 6), ("relinked_batches", C.c_uint64),
                ("last_build_phase_ms", C.c_double * 4)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libpag_hip.so.  There is no fallback: without the built library nothing runs."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise PagError("libpag_hip.so is not built: run `python -m paper_2603_06660_amd.build` "
                           "(or __graft_entry__.build())")
        lib = C.CDLL(_LIB_PATH)
        lib.pag_last_error.restype = C.c_char_p
        for name in EXPORTED_SYMBOLS:
            getattr(lib, name)
        _lib = lib
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().pag_last_error()
        raise PagError("%s failed (%d): %s" % (what, rc, msg.decode() if msg else ""))


def _dev_f32(t, what):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise PagError("%s must be a contiguous float32 CUDA tensor" % what)
    return C.c_void_p(t.data_ptr())


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


class PagIndex:
    """Owner of one pag_index handle."""

    def __init__(self, handle, device):
        self._h = handle
        self._device = device

    # ---- construction --------------------------------------------------
    @staticmethod
    def _params(metric, max_degree, num_subspaces, ef_construction, search_b, insert_subbatch, flags,
                capacity, seed, stream):
        import torch
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        return _Params(C.sizeof(_Params), _METRICS[metric], max_degree, num_subspaces, ef_construction,
                       search_b, insert_subbatch, flags, capacity, seed, C.c_void_p(stream))

    @classmethod
    def build(cls, base, metric="l2", max_degree=32, num_subspaces=16, ef_construction=100, search_b=0,
              insert_subbatch=0, flags=0, capacity=0, seed=1, stream=None):
        lib = load_library()
        p = cls._params(metric, max_degree, num_subspaces, ef_construction, search_b, insert_subbatch, flags,
                        capacity, seed, stream)
        n, d = base.shape
        h = C.c_void_p()
        _check(lib.pag_build(_dev_f32(base, "base"), C.c_uint64(n), C.c_uint32(d), C.byref(p), C.byref(h)),
               "pag_build")
        return cls(h, base.device)

    @classmethod
    def from_arrays(cls, vectors, adj, a, c, e2, codes, rotation, codebooks, entry, metric="l2",
                    ef_construction=100, search_b=0, flags=0, capacity=0, seed=1, stream=None, device="cuda:0",
                    insert_subbatch=0):
        """pag_import from host numpy arrays (shapes as in pag_arrays)."""
        import torch
        lib = load_library()
        vectors = np.ascontiguousarray(vectors, np.float32)
        adj = np.ascontiguousarray(adj, np.uint32)
        a, c, e2 = (np.ascontiguousarray(x, np.float32) for x in (a, c, e2))
        codes = np.ascontiguousarray(codes, np.uint8)
        rotation = np.ascontiguousarray(rotation, np.float32)
        codebooks = np.ascontiguousarray(codebooks, np.float32)
        entry = np.ascontiguousarray(entry, np.uint32)
        n, d = vectors.shape
        deg = adj.shape[1]
        P = codebooks.shape[0]
        arr = _Arrays(C.sizeof(_Arrays), _METRICS[metric], n, d, P, deg, entry.size, _np_ptr(vectors), _np_ptr(adj),
                      _np_ptr(a), _np_ptr(c), _np_ptr(e2), _np_ptr(codes), _np_ptr(rotation), _np_ptr(codebooks),
                      _np_ptr(entry))
        with torch.cuda.device(device):
            p = cls._params(metric, deg, P, ef_construction, search_b, insert_subbatch, flags, capacity, seed, stream)
            h = C.c_void_p()
            _check(lib.pag_import(C.byref(arr), C.byref(p), C.byref(h)), "pag_import")
        return cls(h, torch.device(device))

    def save(self, path):
        """Writes the arrays of pag_export into one uncompressed .npz file."""
        ex = self.export()
        with open(path, "wb") as f:
            np.savez(f, **ex)

    @classmethod
    def load(cls, path, **kw):
        """pag_import of a file written by save().  Keyword arguments as for from_arrays: what an index file does
        not hold (ef_construction, search_b, flags, capacity, seed, stream, device, insert_subbatch)."""
        names = {v: k for k, v in _METRICS.items()}
        with np.load(path, allow_pickle=False) as z:
            arrays = {k: z[k] for k in ("vectors", "adj", "a", "c", "e2", "codes", "rotation", "codebooks", "entry")}
            metric = names[int(z["metric"])]
        return cls.from_arrays(metric=metric, **arrays, **kw)

    def close(self):
        if self._h is not None and self._h.value:
            load_library().pag_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the three calls of the problem statement ----------------------
    def search(self, queries, K, efS, out=None):
        """-> (ids int64 [nq,K], dists float32 [nq,K]) on the device."""
        import torch
        nq = queries.shape[0]
        if out is None:
            ids = torch.empty((nq, K), dtype=torch.int64, device=queries.device)
            dists = torch.empty((nq, K), dtype=torch.float32, device=queries.device)
        else:
            ids, dists = out
        _check(load_library().pag_search(self._h, _dev_f32(queries, "queries"), C.c_uint64(nq), C.c_uint32(K),
                                         C.c_uint32(efS), C.c_void_p(ids.data_ptr()), C.c_void_p(dists.data_ptr())),
               "pag_search")
        return ids, dists

    def search_static(self, queries, K, efS, out):
        """pag_search_static: the search without any allocation; `out` = (ids, dists) preallocated on the device."""
        ids, dists = out
        nq = queries.shape[0]
        _check(load_library().pag_search_static(self._h, _dev_f32(queries, "queries"), C.c_uint64(nq), C.c_uint32(K),
                                                C.c_uint32(efS), C.c_void_p(ids.data_ptr()),
                                                C.c_void_p(dists.data_ptr())), "pag_search_static")
        return ids, dists

    def insert(self, X):
        _check(load_library().pag_insert(self._h, _dev_f32(X, "X"), C.c_uint64(X.shape[0])), "pag_insert")

    def searcher(self, stream=None):
        """A PagSearcher on this index: searches on its own stream that may overlap with insert()."""
        return PagSearcher(self, stream)

    # ---- support -------------------------------------------------------
    def describe(self):
        arr = _Arrays(C.sizeof(_Arrays))
        _check(load_library().pag_describe(self._h, C.byref(arr)), "pag_describe")
        return dict(n=arr.n, d=arr.d, P=arr.num_subspaces, deg=arr.max_degree, n_entry=arr.n_entry, metric=arr.metric)

    def export(self):
        """-> dict of host numpy arrays (pag_arrays)."""
        m = self.describe()
        n, d, P, deg = m["n"], m["d"], m["P"], m["deg"]
        out = dict(vectors=np.empty((n, d), np.float32), adj=np.empty((n, deg), np.uint32),
                   a=np.empty((n, deg), np.float32), c=np.empty((n, deg), np.float32),
                   e2=np.empty((n, deg), np.float32), codes=np.empty((n, deg, P), np.uint8),
                   rotation=np.empty((d, d), np.float32), codebooks=np.empty((P, 16, d // P), np.float32),
                   entry=np.empty(m["n_entry"], np.uint32))
        arr = _Arrays(C.sizeof(_Arrays), m["metric"], n, d, P, deg, m["n_entry"], *(
            _np_ptr(out[k]) for k in ("vectors", "adj", "a", "c", "e2", "codes", "rotation", "codebooks", "entry")))
        _check(load_library().pag_export(self._h, C.byref(arr)), "pag_export")
        out["metric"] = m["metric"]
        return out

    def counters(self):
        c = _Counters(C.sizeof(_Counters))
        _check(load_library().pag_get_counters(self._h, C.byref(c)), "pag_get_counters")
        out = {k: getattr(c, k) for k, _ in c._fields_ if k not in ("struct_size", "phase_cycles", "last_build_phase_ms")}
        out["phase_cycles"] = list(c.phase_cycles)
        out["last_build_phase_ms"] = list(c.last_build_phase_ms)
        return out

    def reset_counters(self):
        _check(load_library().pag_reset_counters(self._h), "pag_reset_counters")

    def set_search_options(self, search_b=0, flags=0):
        _check(load_library().pag_set_search_options(self._h, C.c_uint32(search_b), C.c_uint32(flags)),
               "pag_set_search_options")

    def set_seen_capacity_log2(self, log2_slots):
        _check(load_library().pag_set_seen_capacity_log2(self._h, C.c_uint32(log2_slots)),
               "pag_set_seen_capacity_log2")

    # ---- single steps ----------------------------------------------------
    def prepare_queries(self, queries):
        import torch
        m = self.describe()
        nq = queries.shape[0]
        qrot = torch.empty((nq, m["d"]), dtype=torch.float32, device=queries.device)
        tables = torch.empty((nq, m["P"], 16), dtype=torch.float32, device=queries.device)
        _check(load_library().pag_prepare_queries(self._h, _dev_f32(queries, "queries"), C.c_uint64(nq),
                                                  C.c_void_p(qrot.data_ptr()), C.c_void_p(tables.data_ptr())),
               "pag_prepare_queries")
        return qrot, tables

    def exact_distances(self, q_rot, ids):
        import torch
        nq, m = ids.shape
        assert ids.dtype == torch.int32 and ids.is_cuda and ids.is_contiguous()
        keys = torch.empty((nq, m), dtype=torch.float32, device=q_rot.device)
        _check(load_library().pag_exact_distances(self._h, _dev_f32(q_rot, "q_rot"), C.c_uint64(nq),
                                                  C.c_void_p(ids.data_ptr()), C.c_uint32(m),
                                                  C.c_void_p(keys.data_ptr())), "pag_exact_distances")
        return keys

    def screen(self, tables, u, Du):
        import torch
        m = self.describe()
        nq = tables.shape[0]
        assert u.dtype == torch.int32 and u.is_cuda and u.is_contiguous()
        est = torch.empty((nq, m["deg"]), dtype=torch.float32, device=tables.device)
        _check(load_library().pag_screen(self._h, _dev_f32(tables, "tables"), C.c_uint64(nq),
                                         C.c_void_p(u.data_ptr()), _dev_f32(Du, "Du"),
                                         C.c_void_p(est.data_ptr())), "pag_screen")
        return est

    def measure_row_reads(self, rows, scattered):
        """GB/s at which whole rows of the vector store can be fetched (roofline diagnostic);
        scattered: 0 in order, 1 scattered, 2 with the side traffic of whole hops (records, seen-set reads and writes)."""
        out = C.c_double(0.0)
        _check(load_library().pag_measure_row_reads(self._h, C.c_uint64(rows), C.c_int(int(scattered)),
                                                    C.byref(out)), "pag_measure_row_reads")
        return out.value

    def insertion_candidates(self, X, ef_construction):
        """pag_insertion_candidates for the raw vectors X (device): per vector R_L (ids, keys, count) and the PES
        buffer H(v) (ids, keys, count) as host arrays.  ef_construction must be the index's own efC."""
        m = X.shape[0]
        deg = self.describe()["deg"]
        ci, ck = np.empty((m, ef_construction), np.uint32), np.empty((m, ef_construction), np.float32)
        hi, hk = np.empty((m, deg), np.uint32), np.empty((m, deg), np.float32)
        cn, hn = np.empty(m, np.uint32), np.empty(m, np.uint32)
        _check(load_library().pag_insertion_candidates(self._h, _dev_f32(X, "X"), C.c_uint64(m), _np_ptr(ci), _np_ptr(ck),
                                                       _np_ptr(cn), _np_ptr(hi), _np_ptr(hk), _np_ptr(hn)),
               "pag_insertion_candidates")
        return ci, ck, cn, hi, hk, hn

    def edge_info(self, node_begin, node_end):
        m = self.describe()
        k = node_end - node_begin
        codes = np.empty((k, m["deg"], m["P"]), np.uint8)
        a = np.empty((k, m["deg"]), np.float32)
        c = np.empty_like(a)
        e2 = np.empty_like(a)
        _check(load_library().pag_edge_info(self._h, C.c_uint64(node_begin), C.c_uint64(node_end), _np_ptr(codes),
                                            _np_ptr(a), _np_ptr(c), _np_ptr(e2)), "pag_edge_info")
        return codes, a, c, e2


class PagSearcher:
    """pag_searcher: a view of an index with its own workspaces, counters and stream."""

    def __init__(self, index, stream=None):
        import torch
        self._index = index              # keeps the index alive: searchers are freed first
        self._stream = stream if stream is not None else torch.cuda.Stream()
        h = C.c_void_p()
        _check(load_library().pag_searcher_create(index._h, C.c_void_p(self._stream.cuda_stream), C.byref(h)),
               "pag_searcher_create")
        self._h = h

    def search(self, queries, K, efS, out=None):
        import torch
        nq = queries.shape[0]
        if out is None:
            with torch.cuda.stream(self._stream):
                ids = torch.empty((nq, K), dtype=torch.int64, device=queries.device)
                dists = torch.empty((nq, K), dtype=torch.float32, device=queries.device)
        else:
            ids, dists = out
        _check(load_library().pag_searcher_search(self._h, _dev_f32(queries, "queries"), C.c_uint64(nq), C.c_uint32(K),
                                                  C.c_uint32(efS), C.c_void_p(ids.data_ptr()),
                                                  C.c_void_p(dists.data_ptr())), "pag_searcher_search")
        return ids, dists

    def counters(self):
        c = _Counters(C.sizeof(_Counters))
        _check(load_library().pag_searcher_get_counters(self._h, C.byref(c)), "pag_searcher_get_counters")
        out = {k: getattr(c, k) for k, _ in c._fields_ if k not in ("struct_size", "phase_cycles", "last_build_phase_ms")}
        out["phase_cycles"] = list(c.phase_cycles)
        out["last_build_phase_ms"] = list(c.last_build_phase_ms)
        return out

    def close(self):
        if self._h is not None and self._h.value:
            load_library().pag_searcher_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
