"""Python face of the CPU oracle (ctypes over oracle/pag_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The GPU package never imports this module and
this module never imports the GPU package.

Besides marshalling, this file holds the two pieces of the method that are
random draws rather than arithmetic on data:
  * the fixed random orthogonal transform Q (Sec. 3.1; Alg. 1, "generate a fixed
    random orthogonal transform"), drawn from the Haar measure by Gaussian -> QR;
  * the block codebooks C_l (Sec. 3.1): independently rotated cross-polytopes in
    every subspace, 16 vectors each, scaled by 1/sqrt(P).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pag_oracle.c")
_LIB = os.path.join(_HERE, "libpag_oracle.so")

EMPTY = 0xFFFFFFFF
M_CODES = 16
L2, IP, COS = 0, 1, 2
LITERAL, NO_PRT = 1, 2


def build_lib(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, no intrinsics, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-ffp-contract=off", "-shared",
                               "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Index(C.Structure):
    _fields_ = [("n", C.c_uint64), ("d", C.c_uint32), ("P", C.c_uint32), ("deg", C.c_uint32),
                ("n_entry", C.c_uint32), ("vec", C.c_void_p), ("adj", C.c_void_p),
                ("a", C.c_void_p), ("c", C.c_void_p), ("e2", C.c_void_p), ("codes", C.c_void_p),
                ("rot", C.c_void_p), ("cb", C.c_void_p), ("entry", C.c_void_p)]


class Counters(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in
                ("queries", "hops", "tests", "passes", "exact", "rounds", "rf_over", "rt_over")]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_lib())
        _lib.orc_sqdist64.restype = C.c_double
        _lib.orc_key.restype = C.c_float
        _lib.orc_S32.restype = C.c_float
        _lib.orc_est32.restype = C.c_float
        _lib.orc_est32.argtypes = [C.c_float] * 4
        _lib.orc_robust_prune.restype = C.c_uint32
        _lib.orc_pes_edge.restype = C.c_int
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


# ----------------------------------------------------------------------
# random structures of the method
# ----------------------------------------------------------------------

def haar(dim: int, rng: np.random.Generator) -> np.ndarray:
    g = rng.standard_normal((dim, dim))
    q, r = np.linalg.qr(g)
    return q * np.sign(np.diag(r))[None, :]


def make_transform(d: int, seed: int) -> np.ndarray:
    """Fixed random orthogonal transform Q, float32 [d, d]; q' = Q q."""
    return haar(d, np.random.default_rng([seed, 1])).astype(np.float32)


def make_codebooks(d: int, P: int, seed: int) -> np.ndarray:
    """Codebooks, float32 [P, 16, d/P].  Per subspace: independently Haar-rotated
    cross-polytopes; from each polytope its axes are taken in order, first with
    sign +, then with sign -, until 16 vectors are collected (one polytope cut to
    8 axes when d/P >= 8, two full ones when d/P = 4, ...).  All vectors are
    scaled to norm 1/sqrt(P) so that a concatenation over subspaces is a unit vector."""
    assert d % P == 0
    ds = d // P
    rng = np.random.default_rng([seed, 2])
    cb = np.zeros((P, M_CODES, ds), dtype=np.float64)
    for l in range(P):
        j = 0
        while j < M_CODES:
            rot = haar(ds, rng)                 # columns = rotated axes
            k = min(ds, (M_CODES - j) // 2)
            cb[l, j:j + k] = rot[:, :k].T
            cb[l, j + k:j + 2 * k] = -rot[:, :k].T
            j += 2 * k
    return (cb / np.sqrt(P)).astype(np.float32)


# ----------------------------------------------------------------------
# reference functions (fp64)
# ----------------------------------------------------------------------

def sqdist64(x, y) -> float:
    x, y = _f32(x), _f32(y)
    return float(lib().orc_sqdist64(C.c_uint32(x.size), _p(x), _p(y)))


def key(x, y) -> float:
    x, y = _f32(x), _f32(y)
    return float(lib().orc_key(C.c_uint32(x.size), _p(x), _p(y)))


def rotate(rot, x) -> np.ndarray:
    rot, x = _f32(rot), _f32(x)
    out = np.empty_like(x)
    lib().orc_rotate(C.c_uint32(x.size), _p(rot), _p(x), _p(out))
    return out


def table(cb, q, want64=False):
    cb, q = _f32(cb), _f32(q)
    P, _, ds = cb.shape
    T = np.empty((P, M_CODES), dtype=np.float32)
    T64 = np.empty((P, M_CODES), dtype=np.float64)
    lib().orc_table(C.c_uint32(P * ds), C.c_uint32(P), _p(cb), _p(q), _p(T), _p(T64))
    return (T, T64) if want64 else T


def edge_info(cb, u, w):
    """-> (codes uint8 [P], dict(e2, maxsum, cosb, off, a, c)) for the edge (u, w)."""
    cb, u, w = _f32(cb), _f32(u), _f32(w)
    P, _, ds = cb.shape
    codes = np.empty(P, dtype=np.uint8)
    out = np.empty(6, dtype=np.float64)
    lib().orc_edge_info(C.c_uint32(P * ds), C.c_uint32(P), _p(cb), _p(u), _p(w), _p(codes), _p(out))
    return codes, dict(zip(("e2", "maxsum", "cosb", "off", "a", "c"), out.tolist()))


def stats(cb, u, w, v, dmax2: float):
    """Sec. 3 statistics of the triple (u, w, v) in fp64, from the printed definitions."""
    cb, u, w, v = _f32(cb), _f32(u), _f32(w), _f32(v)
    P, _, ds = cb.shape
    out = np.empty(9, dtype=np.float64)
    lib().orc_stats(C.c_uint32(P * ds), C.c_uint32(P), _p(cb), _p(u), _p(w), _p(v),
                    C.c_double(dmax2), _p(out))
    names = ("cos_alpha", "cos_beta", "cos_theta", "tau", "prt", "delta", "pes_term", "est", "S")
    return dict(zip(names, out.tolist()))


def S32(T, codes) -> float:
    T = _f32(T)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    return float(lib().orc_S32(C.c_uint32(codes.size), _p(T), _p(codes)))


def est32(Du, a, c, S) -> float:
    return float(lib().orc_est32(Du, a, c, S))


# ----------------------------------------------------------------------
# index
# ----------------------------------------------------------------------

class OracleIndex:
    """Flat-array PAG index searched / built by the C oracle.

    vec    float32 [n, d]      rotated (and, for COS, normalised) base vectors
    adj    uint32  [n, deg]    out-neighbours, EMPTY = free slot
    a, c, e2 float32 [n, deg]  per-edge scalars
    codes  uint8   [n, deg, P] per-edge, per-subspace reference index
    rot    float32 [d, d], cb float32 [P, 16, d/P], entry uint32 [E]
    """

    def __init__(self, vec, adj, a, c, e2, codes, rot, cb, entry, metric=L2):
        self.vec = _f32(vec)
        self.adj = np.ascontiguousarray(adj, dtype=np.uint32)
        self.a, self.c, self.e2 = _f32(a), _f32(c), _f32(e2)
        self.codes = np.ascontiguousarray(codes, dtype=np.uint8)
        self.rot, self.cb = _f32(rot), _f32(cb)
        self.entry = np.ascontiguousarray(entry, dtype=np.uint32)
        self.metric = int(metric)
        self.n, self.d = self.vec.shape
        self.deg = self.adj.shape[1]
        self.P = self.cb.shape[0]
        assert self.codes.shape == (self.n, self.deg, self.P)
        assert self.cb.shape == (self.P, M_CODES, self.d // self.P)

    def _struct(self, n=None):
        return _Index(self.n if n is None else n, self.d, self.P, self.deg, self.entry.size,
                      _p(self.vec), _p(self.adj), _p(self.a), _p(self.c), _p(self.e2),
                      _p(self.codes), _p(self.rot), _p(self.cb), _p(self.entry))

    # -- construction ---------------------------------------------------
    @staticmethod
    def _ingest(data, metric, rot, vec_f16):
        """Rows of `data` normalised (COS), rotated by Q and, with vec_f16, rounded to 16-bit floats."""
        data = _f32(data)
        n, d = data.shape
        vec = np.empty_like(data)
        tmp = np.empty(d, dtype=np.float32)
        L = lib()
        for i in range(n):
            x = data[i]
            if metric == COS:
                L.orc_normalise(C.c_uint32(d), _p(x), _p(tmp))
                x = tmp
            L.orc_rotate(C.c_uint32(d), _p(rot), _p(x), _p(vec[i]))
        if vec_f16:
            vec = vec.astype(np.float16).astype(np.float32)
        return vec

    def _link(self, n_start, efC, pes, pes_every, max_batch, relink=True):
        """Alg. 1 over the nodes [n_start, n): sequential (max_batch = 0) or batch-synchronous."""
        L = lib()
        ctr = Counters()
        st = self._struct()
        added = C.c_uint64(0)
        batches = C.c_uint64(0)
        relinked = C.c_uint64(0)
        if max_batch:
            rc = L.orc_build_batched(C.byref(st), C.c_uint32(efC), C.c_uint64(n_start), C.c_uint64(self.n),
                                     C.c_uint64(max_batch), C.c_int(1 if pes else 0), C.c_int(1 if relink else 0),
                                     C.byref(ctr), C.byref(added), C.byref(batches), C.byref(relinked))
        else:
            rc = L.orc_build(C.byref(st), C.c_uint32(efC), C.c_uint64(n_start), C.c_uint64(self.n), C.byref(ctr),
                             C.c_int(1 if pes else 0), C.c_uint64(pes_every), C.byref(added))
        assert rc == 0
        self.build_counters = ctr.as_dict()
        self.pes_edges_added = int(added.value)
        self.batches = int(batches.value)
        self.relinked_batches = int(relinked.value)

    @classmethod
    def build(cls, data, metric=L2, deg=32, P=16, efC=100, seed=1, rot=None, cb=None, pes=True, vec_f16=False,
              pes_every=0, max_batch=0):
        """Alg. 1 over `data` (raw float32 [n, d]) in row order; pes=False leaves out Steps 2 and 3.
        pes_every: the PES buffers are verified after every so many insertions (0: after the last one).
        max_batch: 0 = one node after another; otherwise the batch-synchronous construction with batches
        of at most that many nodes.
        vec_f16: the rotated vectors are rounded to 16-bit floats (the paper's payload, Sec. 4.2) and the
        index is built over those values."""
        data = _f32(data)
        n, d = data.shape
        rot = make_transform(d, seed) if rot is None else _f32(rot)
        cb = make_codebooks(d, P, seed) if cb is None else _f32(cb)
        vec = cls._ingest(data, metric, rot, vec_f16)
        self = cls(vec, np.full((n, deg), EMPTY, np.uint32), np.zeros((n, deg), np.float32),
                   np.zeros((n, deg), np.float32), np.zeros((n, deg), np.float32),
                   np.zeros((n, deg, P), np.uint8), rot, cb,
                   np.arange(min(n, 1024), dtype=np.uint32), metric)
        self._link(0, efC, pes, pes_every, max_batch)
        return self

    def insert(self, data, efC=100, pes=True, pes_every=0, max_batch=0, vec_f16=False, relink=True):
        """Online insertion (Sec. 4.1): the rows of `data` are appended and linked like the nodes of build();
        the entry list grows with them until it holds 1024 nodes."""
        new = self._ingest(data, self.metric, self.rot, vec_f16)
        m, n0 = new.shape[0], self.n
        self.vec = np.ascontiguousarray(np.concatenate([self.vec, new]))
        self.adj = np.ascontiguousarray(np.concatenate([self.adj, np.full((m, self.deg), EMPTY, np.uint32)]))
        for k in ("a", "c", "e2"):
            setattr(self, k, np.ascontiguousarray(np.concatenate([getattr(self, k), np.zeros((m, self.deg), np.float32)])))
        self.codes = np.ascontiguousarray(np.concatenate([self.codes, np.zeros((m, self.deg, self.P), np.uint8)]))
        self.n = n0 + m
        if self.entry.size < 1024:
            grow = np.arange(n0, min(self.n, n0 + 1024 - self.entry.size), dtype=np.uint32)
            self.entry = np.ascontiguousarray(np.concatenate([self.entry, grow]))
        self._link(n0, efC, pes, pes_every, max_batch, relink)

    def index_search(self, v_rot, efC, n_nodes=None):
        """The search of one insertion (Alg. 1) for the rotated point v over the nodes [0, n_nodes):
        -> (R_L ids, R_L keys, H(v) ids, H(v) keys, counters)."""
        v_rot = _f32(v_rot)
        room = efC + min(efC, 100)
        ci, ck = np.empty(room, np.uint32), np.empty(room, np.float32)
        hi, hk = np.empty(self.deg, np.uint32), np.empty(self.deg, np.float32)
        nc, nh = C.c_uint32(0), C.c_uint32(0)
        ctr = Counters()
        st = self._struct()
        rc = lib().orc_index_search(C.byref(st), C.c_uint64(self.n if n_nodes is None else n_nodes), _p(v_rot),
                                    C.c_uint32(efC), _p(ci), _p(ck), C.byref(nc), _p(hi), _p(hk), C.byref(nh),
                                    C.byref(ctr))
        assert rc == 0
        return ci[:nc.value].copy(), ck[:nc.value].copy(), hi[:nh.value].copy(), hk[:nh.value].copy(), ctr.as_dict()

    def reverse_edge(self, u, v, duv):
        """The reverse edge u -> v of an insertion (Sec. 2.1; Eq. 1), applied in place."""
        st = self._struct()
        lib().orc_reverse_edge(C.byref(st), C.c_uint32(u), C.c_uint32(v), C.c_float(duv))

    def pes_edge(self, u, v, duv):
        """Verification of the PES candidate u -> v (Alg. 1, last loop), applied in place; -> 1 if added."""
        st = self._struct()
        return int(lib().orc_pes_edge(C.byref(st), C.c_uint32(u), C.c_uint32(v), C.c_float(duv)))

    # -- search ---------------------------------------------------------
    def search(self, Q, K, efS, b=0, flags=0, threads=1, want_seen=False):
        """Alg. 2 over raw queries Q.  Returns (ids int64 [nq,K], dists float32 [nq,K], counters)
        and, with want_seen, the per-query lists of nodes whose exact distance was computed."""
        Q = _f32(Q)
        nq = Q.shape[0]
        ids = np.empty((nq, K), dtype=np.int64)
        dists = np.empty((nq, K), dtype=np.float32)
        st = self._struct()
        L = lib()

        def run(lo, hi):
            ctr = Counters()
            seen = None
            if want_seen:
                cap = (hi - lo) * 65536
                log = np.empty(cap, dtype=np.uint32)
                off = np.zeros(hi - lo + 1, dtype=np.uint64)
                args = (_p(log), C.c_uint64(cap), _p(off))
            else:
                args = (None, C.c_uint64(0), None)
            rc = L.orc_search_batch(C.byref(st), C.c_int(self.metric), _p(Q[lo:hi]),
                                    C.c_uint64(hi - lo), C.c_uint32(K), C.c_uint32(efS),
                                    C.c_uint32(b), C.c_int(flags), _p(ids[lo:hi]), _p(dists[lo:hi]),
                                    C.byref(ctr), *args)
            assert rc == 0
            if want_seen:
                seen = [log[int(off[i]):int(off[i + 1])].copy() for i in range(hi - lo)]
            return ctr.as_dict(), seen

        threads = max(1, min(int(threads), nq))
        bounds = np.linspace(0, nq, threads + 1).astype(int)
        if threads == 1:
            parts = [run(0, nq)]
        else:
            with ThreadPoolExecutor(threads) as ex:
                parts = list(ex.map(lambda t: run(int(bounds[t]), int(bounds[t + 1])), range(threads)))
        total = {}
        for ctr, _ in parts:
            for k, v in ctr.items():
                total[k] = total.get(k, 0) + v
        if want_seen:
            seen_all = [s for _, sl in parts for s in sl]
            return ids, dists, total, seen_all
        return ids, dists, total

    def prepare(self, Q):
        """(rotated queries float32 [nq,d], tables float32 [nq,P,16])"""
        Q = _f32(Q)
        nq = Q.shape[0]
        qr = np.empty((nq, self.d), dtype=np.float32)
        T = np.empty((nq, self.P, M_CODES), dtype=np.float32)
        st = self._struct()
        lib().orc_prepare_queries(C.byref(st), C.c_int(self.metric), _p(Q), C.c_uint64(nq), _p(qr), _p(T))
        return qr, T

    def recompute_edge_info(self, lo=0, hi=None):
        """Inference information of every stored edge of nodes [lo, hi), from the vectors."""
        hi = self.n if hi is None else hi
        m = hi - lo
        codes = np.empty((m, self.deg, self.P), dtype=np.uint8)
        a = np.empty((m, self.deg), dtype=np.float32)
        c = np.empty_like(a)
        e2 = np.empty_like(a)
        st = self._struct()
        lib().orc_edge_info_all(C.byref(st), C.c_uint64(lo), C.c_uint64(hi), _p(codes), _p(a), _p(c), _p(e2))
        return codes, a, c, e2

    def robust_prune(self, cand_ids, cand_keys, max_keep):
        cand_ids = np.ascontiguousarray(cand_ids, dtype=np.uint32)
        cand_keys = _f32(cand_keys)
        kept = np.empty(max_keep, dtype=np.uint32)
        kkey = np.empty(max_keep, dtype=np.float32)
        st = self._struct()
        nk = lib().orc_robust_prune(C.byref(st), C.c_uint32(cand_ids.size), _p(cand_ids), _p(cand_keys),
                                    C.c_uint32(max_keep), _p(kept), _p(kkey))
        return kept[:nk].copy(), kkey[:nk].copy()
