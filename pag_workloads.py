"""Seeded synthetic inputs for the PAG search workloads.

This module only draws input data (base vectors, queries) and computes
brute-force ground truth.  It contains none of the method's arithmetic: no
rotation Q of the index, no codebooks, no projection test, no graph.  Both the
CPU oracle's tests and the HIP path's tests/bench get their inputs from here so
that the two sides see byte-identical arrays.

The shapes stand in for the embedding corpora the paper measures on
(Table 2: d = 384..3072, n = 1M..56M, 1,000-10,000 queries, one
out-of-distribution query set); those corpora are not available offline, so
every workload below is a seeded generator with the same (n, d, K, metric)
structure.

All generators are chunked so that peak memory stays near the size of the
output array, and the random stream is consumed row by row, so the result does
not depend on the chunk size.
"""
from __future__ import annotations

import dataclasses
import numpy as np

BASE_SEED = 260306660
CHUNK_ROWS = 1 << 16

L2, IP, COS = 0, 1, 2


@dataclasses.dataclass(frozen=True)
class Workload:
    """One synthetic configuration (index parameters + search parameters)."""
    name: str
    cfg: int            # configuration number (1..5)
    n: int              # base vectors
    d: int              # dimension
    nq: int             # queries
    metric: int         # L2 / IP / COS
    deg: int            # maximum out-degree (the paper's 2M)
    P: int              # number of subspaces (the paper's L)
    K: int              # retrieval size
    efs_grid: tuple     # efS sweep
    ood_frac: float = 0.0


def workload(cfg: int, n: int | None = None, nq: int | None = None) -> Workload:
    """Return configuration `cfg`; `n` / `nq` shrink it for tests."""
    table = {
        1: Workload("gmm16-128-l2", 1, 10_000, 128, 1_000, L2, 32, 16, 10, (64,)),
        2: Workload("aniso-768-ip", 2, 1_000_000, 768, 10_000, IP, 32, 32, 10,
                    (32, 48, 64, 96, 128, 192, 256, 384, 512)),
        3: Workload("aniso-clustered-1024-ip", 3, 1_000_000, 1024, 10_000, IP, 48, 32, 100,
                    (128, 192, 256, 384, 512, 768, 1024)),
        4: Workload("gmm1024-1536-cos-ood", 4, 2_000_000, 1536, 10_000, COS, 48, 64, 10,
                    (32, 48, 64, 96, 128, 192, 256, 384, 512), ood_frac=0.10),
        5: Workload("aniso-3072-ip-online", 5, 500_000, 3072, 5_000, IP, 32, 64, 10,
                    (32, 48, 64, 96, 128, 192, 256)),
    }
    w = table[cfg]
    if n is not None:
        w = dataclasses.replace(w, n=int(n))
    if nq is not None:
        w = dataclasses.replace(w, nq=int(nq))
    return w


def _rng(cfg: int, stream: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, cfg, stream]))


def _haar(d: int, rng: np.random.Generator) -> np.ndarray:
    """A d x d orthogonal matrix from the Haar measure (Gaussian -> QR, signs fixed).
    Part of the *data* recipe (the fixed rotation that hides the anisotropic axes),
    unrelated to the index's own transform."""
    g = rng.standard_normal((d, d))
    q, r = np.linalg.qr(g)
    q *= np.sign(np.diag(r))[None, :]
    return q.astype(np.float32)


def _normalise_rows(x: np.ndarray) -> None:
    nrm = np.sqrt(np.einsum("ij,ij->i", x, x, dtype=np.float64))
    nrm[nrm == 0] = 1.0
    x /= nrm[:, None].astype(np.float32)


def _chunks(n: int):
    for s in range(0, n, CHUNK_ROWS):
        yield s, min(n, s + CHUNK_ROWS)


def _gmm_rows(n, d, centres, sigma, rng, out):
    ncomp = centres.shape[0]
    for s, e in _chunks(n):
        comp = rng.integers(0, ncomp, size=e - s)
        z = rng.standard_normal((e - s, d), dtype=np.float32)
        out[s:e] = centres[comp] + sigma * z


def _aniso_rows(n, d, scale, rot, rng, out, centres=None, spread=1.0):
    for s, e in _chunks(n):
        z = rng.standard_normal((e - s, d), dtype=np.float32) * scale[None, :]
        if centres is not None:
            comp = rng.integers(0, centres.shape[0], size=e - s)
            z = centres[comp] + np.float32(spread) * z
        out[s:e] = z @ rot
    # normalisation is done by the caller (rotation keeps norms)


def make(w: Workload, part: str, n: int | None = None, stream_offset: int = 0) -> np.ndarray:
    """Draw the `part` ("base", "query", or "insert<k>") of workload `w` as float32 [rows, d].

    Base and query rows come from the same law but from different random
    streams.  `n` overrides the row count.
    """
    d = w.d
    rows = n if n is not None else (w.n if part == "base" else w.nq)
    if part == "base":
        stream = 1
    elif part == "query":
        stream = 2
    elif part.startswith("insert"):
        stream = 100 + int(part[len("insert"):])
    else:
        raise ValueError(part)
    stream += stream_offset
    rng_fixed = _rng(w.cfg, 0)           # mixture centres / data rotation: shared by all parts
    rng = _rng(w.cfg, stream)
    out = np.empty((rows, d), dtype=np.float32)

    if w.cfg == 1:
        centres = (2.0 * rng_fixed.standard_normal((16, d))).astype(np.float32)
        _gmm_rows(rows, d, centres, np.float32(1.0), rng, out)
    elif w.cfg in (2, 5):
        scale = (np.arange(1, d + 1, dtype=np.float64) ** -0.4).astype(np.float32)  # var ~ i^-0.8
        rot = _haar(d, rng_fixed)
        _aniso_rows(rows, d, scale, rot, rng, out)
        _normalise_rows(out)
    elif w.cfg == 3:
        scale = (np.arange(1, d + 1, dtype=np.float64) ** -0.4).astype(np.float32)
        rot = _haar(d, rng_fixed)
        centres = (rng_fixed.standard_normal((256, d)) * scale[None, :]).astype(np.float32)
        _aniso_rows(rows, d, scale, rot, rng, out, centres=centres, spread=0.5)
        _normalise_rows(out)
    elif w.cfg == 4:
        centres = (2.0 * rng_fixed.standard_normal((1024, d))).astype(np.float32)
        _gmm_rows(rows, d, centres, np.float32(1.0), rng, out)
        if part == "query" and w.ood_frac > 0:
            n_ood = int(round(rows * w.ood_frac))
            rng_ood = _rng(w.cfg, 50 + stream)
            idx = rng_ood.choice(rows, size=n_ood, replace=False)
            out[np.sort(idx)] = rng_ood.standard_normal((n_ood, d), dtype=np.float32)
        _normalise_rows(out)
    else:
        raise ValueError(w.cfg)
    return out


def keys_from(metric: int, sq_l2: np.ndarray) -> np.ndarray:
    """Ascending result keys: squared L2 for L2, 1 - <q,x> = ||q-x||^2 / 2 for IP/COS on unit vectors."""
    return sq_l2 if metric == L2 else 0.5 * sq_l2


def brute_force(base: np.ndarray, queries: np.ndarray, K: int, metric: int = L2,
                block: int = 256):
    """Exact K nearest neighbours by exhaustive fp64 squared-L2 scan, ordered by (dist, id).

    For COS the inputs are normalised first; IP expects unit-norm inputs (then
    all three metrics rank by squared L2).  Returns (ids int64 [nq,K], keys float64 [nq,K]).
    """
    b = np.asarray(base, dtype=np.float64)
    q = np.asarray(queries, dtype=np.float64)
    if metric == COS:
        b = b / np.maximum(np.linalg.norm(b, axis=1, keepdims=True), 1e-300)
        q = q / np.maximum(np.linalg.norm(q, axis=1, keepdims=True), 1e-300)
    n = b.shape[0]
    K = min(K, n)
    bn = np.einsum("ij,ij->i", b, b)
    ids = np.empty((q.shape[0], K), dtype=np.int64)
    keys = np.empty((q.shape[0], K), dtype=np.float64)
    for s in range(0, q.shape[0], block):
        qq = q[s:s + block]
        d2 = bn[None, :] - 2.0 * (qq @ b.T) + np.einsum("ij,ij->i", qq, qq)[:, None]
        np.maximum(d2, 0.0, out=d2)
        kk = min(n - 1, K + 8)
        part = np.argpartition(d2, kk, axis=1)[:, :kk + 1] if kk < n - 1 else \
            np.tile(np.arange(n), (qq.shape[0], 1))
        for r in range(qq.shape[0]):
            cand = part[r]
            # re-evaluate the shortlisted distances directly (no cancellation), then total order
            diff = b[cand] - qq[r]
            dd = np.einsum("ij,ij->i", diff, diff)
            order = np.lexsort((cand, dd))[:K]
            ids[s + r] = cand[order]
            keys[s + r] = dd[order]
    return ids, keys_from(metric, keys)


def recall_at_k(found_ids: np.ndarray, true_ids: np.ndarray) -> float:
    """|returned ∩ true top-K| / K averaged over queries (problem statement, Sec. 1)."""
    nq, K = true_ids.shape
    hit = 0
    for r in range(nq):
        hit += len(set(found_ids[r, :K].tolist()) & set(true_ids[r].tolist()))
    return hit / float(nq * K)


def brute_force_torch(base_t, queries_t, K: int, metric: int = L2, block: int = 512, shortlist: int = 32):
    """Ground truth on whatever device the tensors live on (harness only; used at the 1M scale).

    fp32 matrix products pick a shortlist of K + `shortlist` candidates per query, which is then
    re-ranked by directly evaluated fp64 squared distances and ordered by (dist, id).
    Returns (ids int64 [nq,K], keys float64 [nq,K]) as numpy arrays.
    """
    import torch
    n = base_t.shape[0]
    K = min(K, n)
    kk = min(n, K + shortlist)
    b = base_t
    q = queries_t
    if metric == COS:
        b = b / b.norm(dim=1, keepdim=True).clamp_min(1e-30)
        q = q / q.norm(dim=1, keepdim=True).clamp_min(1e-30)
    bn = (b.double() ** 2).sum(1).float()
    ids_out, keys_out = [], []
    for s in range(0, q.shape[0], block):
        qq = q[s:s + block]
        d2 = bn[None, :] - 2.0 * (qq @ b.T)
        cand = torch.topk(d2, kk, dim=1, largest=False).indices           # [blk, kk]
        diff = b[cand].double() - qq.double()[:, None, :]
        dd = (diff * diff).sum(-1)
        # total order (dist, id): sort by id first (stable), then by distance (stable)
        o1 = torch.argsort(cand, dim=1, stable=True)
        cand, dd = torch.gather(cand, 1, o1), torch.gather(dd, 1, o1)
        o2 = torch.argsort(dd, dim=1, stable=True)[:, :K]
        ids_out.append(torch.gather(cand, 1, o2).cpu().numpy())
        keys_out.append(torch.gather(dd, 1, o2).cpu().numpy())
    ids = np.concatenate(ids_out).astype(np.int64)
    keys = np.concatenate(keys_out)
    return ids, keys_from(metric, keys)
