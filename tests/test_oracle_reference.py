"""Pins for the oracle's fp64 reference functions (Sec. 3.1, Eq. 2-5, Appendix B/C).

Each test fixes the oracle to something other than itself: a hand-derived worked
example, a closed form, an algebraic identity, a planted special case, a library
routine, or a statistical statement of the paper (Theorem 3.1; the finite-(m, L)
property quoted from KS2 in Sec. 3.2).
"""
import os
from math import sqrt

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    vals = {}
    with open(os.path.join(HERE, "golden", "worked_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            vals[k] = float(v)
    return vals


def _axis_codebook(P, ds):
    """{+e1, -e1, +e2, -e2, ...}/sqrt(P) per block; unused slots repeat slot 0."""
    cb = np.zeros((P, 16, ds), dtype=np.float32)
    for l in range(P):
        j = 0
        for k in range(min(ds, 8)):
            cb[l, j, k] = 1.0
            cb[l, j + 1, k] = -1.0
            j += 2
        for jj in range(j, 16):
            cb[l, jj] = cb[l, 0]
    return (cb / np.float32(sqrt(P))).astype(np.float32)


def test_worked_example(orc):
    g = _golden()
    cb = _axis_codebook(2, 2)
    u = np.zeros(4, np.float32)
    w = np.array([3, 1, 0, -2], np.float32)
    v = np.array([2, 2, 1, -1], np.float32)
    codes, info = orc.edge_info(cb, u, w)
    assert codes.tolist() == [int(g["code_block1"]), int(g["code_block2"])]
    # float32 codebook entries (1/sqrt2 rounded) limit agreement to ~1e-7
    tol = dict(rel=3e-7, abs=3e-7)
    assert info["e2"] == g["e2"]
    assert info["maxsum"] == pytest.approx(g["maxsum"], **tol)
    assert info["cosb"] == pytest.approx(g["cos_beta"], **tol)
    assert info["a"] == pytest.approx(g["a"], **tol)
    assert info["off"] == g["off"]
    assert info["c"] == pytest.approx(14.0, **tol)
    for dmax, kt, kp in ((8.0, "tau_dmax8", "prt_dmax8"), (7.0, "tau_dmax7", "prt_dmax7")):
        s = orc.stats(cb, u, w, v, dmax)
        assert s["S"] == pytest.approx(g["S"], **tol)
        assert s["cos_theta"] == pytest.approx(g["cos_theta"], **tol)
        assert s["cos_alpha"] == pytest.approx(g["cos_alpha"], rel=1e-12)
        assert s["cos_theta"] / s["cos_beta"] == pytest.approx(g["ratio"], **tol)
        assert s["tau"] == pytest.approx(g[kt], rel=1e-12)
        assert s["prt"] == pytest.approx(g[kp], abs=3e-7)
        assert (s["prt"] > 0) == (g[kp] > 0) == (g["est"] < dmax)
        assert s["est"] == pytest.approx(g["est"], **tol)
        assert s["delta"] == pytest.approx(g["delta"], rel=1e-12)
        assert s["pes_term"] == pytest.approx(g["pes_term"], abs=3e-7)
    assert orc.sqdist64(v, w) == g["exact"]
    assert orc.sqdist64(v, u) == g["Du"]
    # fp32 search form of the same estimate
    T = orc.table(cb, v)
    S32 = orc.S32(T, codes)
    est32 = orc.est32(10.0, np.float32(info["a"]), np.float32(info["c"]), S32)
    assert est32 == pytest.approx(7.2, rel=1e-6)


def _random_case(rng, orc, d, P):
    cb = orc.make_codebooks(d, P, int(rng.integers(1 << 30)))
    u, w, v = (rng.standard_normal(d).astype(np.float32) for _ in range(3))
    return cb, u, w, v


def test_prt_sign_equals_estimate_comparison(orc):
    """Multiplying Eq. 3 with Eq. 4's threshold through by 2||v-u|| ||w-u|| cos(beta) > 0:
    PRT > 0  <=>  D_u + c - 2 a S < ||z_max - v||^2."""
    rng = np.random.default_rng(5)
    checked = 0
    for _ in range(300):
        d, P = [(8, 2), (16, 4), (32, 4), (24, 3)][int(rng.integers(4))]
        cb, u, w, v = _random_case(rng, orc, d, P)
        dmax = float(rng.uniform(0.2, 2.5)) * orc.sqdist64(v, u)
        s = orc.stats(cb, u, w, v, dmax)
        if s["cos_beta"] < 1e-3 or abs(s["prt"]) < 1e-9:
            continue
        assert (s["prt"] > 0) == (s["est"] < dmax)
        # the estimate is the law of cosines with <v-u, w-u> replaced by a (S - off)
        checked += 1
    assert checked > 250


def test_tau_minus_delta_needs_no_vw_distance(orc):
    """Sec. 3.4: tau_i - delta_i = (||u-v||^2 - ||z_max-v||^2) / (2 ||v-u|| ||w_i-u||)."""
    rng = np.random.default_rng(6)
    for _ in range(50):
        cb, u, w, v = _random_case(rng, orc, 16, 4)
        dmax = float(rng.uniform(0.2, 2.5))
        s = orc.stats(cb, u, w, v, dmax)
        du, e = orc.sqdist64(v, u), sqrt(orc.sqdist64(w, u))
        assert s["tau"] - s["delta"] == pytest.approx((du - dmax) / (2 * sqrt(du) * e), rel=1e-6, abs=1e-9)


def test_planted_reference_vector_gives_exact_distance(orc):
    """P = 1 and a codebook that contains (w-u)/||w-u||: cos(beta) = 1, cos(theta) = cos(alpha),
    and the estimate equals the exact squared distance."""
    rng = np.random.default_rng(7)
    d = 16
    for _ in range(20):
        u, w, v = (rng.standard_normal(d) for _ in range(3))
        # choose w so that (w-u)/||w-u|| is exactly representable: direction with entries in {0, +-1/2}
        direction = np.zeros(d)
        direction[rng.choice(d, 4, replace=False)] = rng.choice([-0.5, 0.5], 4)
        u32 = u.astype(np.float32)
        w32 = (u32.astype(np.float64) + 2.0 * direction).astype(np.float32)
        cb = np.zeros((1, 16, d), np.float32)
        cb[0, 5] = direction.astype(np.float32)
        cb[0, 6] = -direction.astype(np.float32)
        s = orc.stats(cb, u32, w32, v.astype(np.float32), 1.0)
        codes, info = orc.edge_info(cb, u32, w32)
        assert codes.tolist() == [5]
        assert s["cos_beta"] == pytest.approx(1.0, abs=1e-6)
        assert s["cos_theta"] == pytest.approx(s["cos_alpha"], abs=1e-6)
        assert s["est"] == pytest.approx(orc.sqdist64(v.astype(np.float32), w32), rel=1e-5)


def test_argmax_on_axis_codebook(orc):
    """With axis-aligned cross-polytopes the selected reference of a block is the signed axis of
    the largest |component| of (w-u)_l, and cos(beta) = sum_l max_k |(w-u)_lk| / (sqrt(P) ||w-u||)."""
    rng = np.random.default_rng(8)
    P, ds = 4, 8
    cb = _axis_codebook(P, ds)
    for _ in range(50):
        u = rng.standard_normal(P * ds).astype(np.float32)
        w = rng.standard_normal(P * ds).astype(np.float32)
        diff = (w - u).astype(np.float64).reshape(P, ds)
        codes, info = orc.edge_info(cb, u, w)
        k = np.abs(diff).argmax(1)
        expect = 2 * k + (diff[np.arange(P), k] < 0)
        assert codes.tolist() == expect.tolist()
        cosb = np.abs(diff).max(1).sum() / sqrt(P) / np.linalg.norm(diff)
        assert info["cosb"] == pytest.approx(cosb, rel=1e-6)
        off = sum(np.float64(cb[l, codes[l]]) @ np.float64(u[l * ds:(l + 1) * ds]) for l in range(P))
        assert info["off"] == pytest.approx(off, rel=1e-9, abs=1e-12)


def test_degenerate_edges(orc):
    cb = orc.make_codebooks(16, 4, 3)
    u = np.arange(16, dtype=np.float32)
    _, info = orc.edge_info(cb, u, u)      # w == u: estimate collapses to D_u
    assert info["a"] == 0.0 and info["c"] == 0.0 and info["e2"] == 0.0
    assert orc.est32(3.5, 0.0, 0.0, 123.0) == 3.5


def test_distance_rotation_table_against_numpy(orc):
    rng = np.random.default_rng(9)
    d, P = 48, 6
    x = rng.standard_normal(d).astype(np.float32)
    y = rng.standard_normal(d).astype(np.float32)
    assert orc.sqdist64(x, y) == pytest.approx(float(((x.astype(np.float64) - y) ** 2).sum()), rel=1e-6)
    assert orc.key(x, y) == np.float32(orc.sqdist64(x, y))
    rot = orc.make_transform(d, 4)
    assert np.allclose(rot.astype(np.float64) @ rot.astype(np.float64).T, np.eye(d), atol=1e-5)
    xr = orc.rotate(rot, x)
    assert np.array_equal(xr, (rot.astype(np.float64) @ x.astype(np.float64)).astype(np.float32)) or \
        np.allclose(xr, rot.astype(np.float64) @ x, rtol=0, atol=1e-6)
    # rotation preserves distances
    assert orc.sqdist64(orc.rotate(rot, x), orc.rotate(rot, y)) == pytest.approx(orc.sqdist64(x, y), rel=1e-5)
    cb = orc.make_codebooks(d, P, 4)
    T = orc.table(cb, x)
    ref = np.einsum("ljk,lk->lj", cb.astype(np.float64), x.astype(np.float64).reshape(P, d // P))
    assert np.allclose(T, ref, rtol=0, atol=1e-6)


def test_codebook_structure(orc):
    """Sec. 3.1: 16 vectors per subspace from rotated cross-polytopes, norm 1/sqrt(L)."""
    for d, P in ((128, 16), (768, 32), (64, 16), (32, 16)):
        cb = orc.make_codebooks(d, P, 12).astype(np.float64)
        ds = d // P
        assert cb.shape == (P, 16, ds)
        assert np.allclose(np.linalg.norm(cb, axis=2), 1 / sqrt(P), atol=1e-6)
        for l in range(P):
            g = cb[l] @ cb[l].T * P
            # every vector has its antipode in the set; others are orthogonal or (across polytopes) generic
            assert np.allclose(np.sort(g, axis=1)[:, 0], -1.0, atol=1e-5)
            k = min(ds, 8)
            blk = g[:k, :k]
            assert np.allclose(blk, np.eye(k), atol=1e-5)
        if P > 1:
            assert not np.allclose(cb[0], cb[1])     # independent rotations across subspaces


def test_theorem_3_1_mean_and_variance(orc):
    """Theorem 3.1: conditioned on (alpha, beta), cos(theta) is centred at cos(alpha) cos(beta)
    with covariance O(1/L).  Monte-Carlo over random codebooks at fixed (u, w, v)."""
    rng = np.random.default_rng(10)
    d = 256
    u = np.zeros(d, np.float32)
    w = rng.standard_normal(d)
    v = 0.6 * w + 0.8 * rng.standard_normal(d)
    w32, v32 = w.astype(np.float32), v.astype(np.float32)
    resid_sd = {}
    for P in (8, 32):
        r = []
        for t in range(400):
            cb = orc.make_codebooks(d, P, 1000 * P + t)
            s = orc.stats(cb, u, w32, v32, 1.0)
            r.append(s["cos_theta"] - s["cos_alpha"] * s["cos_beta"])
        r = np.array(r)
        resid_sd[P] = r.std()
        assert abs(r.mean()) < 4 * r.std() / sqrt(len(r)) + 2e-3     # centred
    assert resid_sd[32] < resid_sd[8]                              # variance shrinks with L


def test_routing_test_success_probability(orc):
    """Sec. 3.2 (property quoted from KS2, Lemma 4.3): if cos(alpha) >= tau then the test passes with
    probability >= 0.5, even for finite (m, L).  Take tau = cos(alpha) (the hardest admissible case)."""
    rng = np.random.default_rng(11)
    d, P = 128, 16
    hits = trials = 0
    for t in range(600):
        u = rng.standard_normal(d).astype(np.float32)
        w = (u + rng.standard_normal(d)).astype(np.float32)
        v = (u + rng.standard_normal(d) + 0.5 * (w - u)).astype(np.float32)
        cb = orc.make_codebooks(d, P, 50_000 + t)
        s0 = orc.stats(cb, u, w, v, 1.0)
        # choose ||z_max - v||^2 so that tau equals cos(alpha) exactly (law of cosines): the true ||v-w||^2
        dmax = orc.sqdist64(v, w)
        s = orc.stats(cb, u, w, v, dmax)
        assert s["tau"] == pytest.approx(s0["cos_alpha"], abs=1e-6)
        trials += 1
        hits += s["prt"] >= 0
    assert hits / trials >= 0.5 - 3 * 0.5 / sqrt(trials)


def test_pes_sign_equals_estimate_comparison(orc):
    """Eq. 5 term for one neighbour, cos(theta)/cos(beta) - delta with delta = ||w-u|| / (2 ||v-u||):
    negative  <=>  the estimate of ||v-w||^2 exceeds ||v-u||^2 (w is not an estimated witness).
    Also delta itself: cos(alpha) > delta  <=>  ||w-v|| < ||v-u|| (law of cosines, Sec. 3.4)."""
    rng = np.random.default_rng(21)
    checked = 0
    for _ in range(300):
        d, P = [(8, 2), (16, 4), (32, 4), (24, 3)][int(rng.integers(4))]
        cb, u, w, v = _random_case(rng, orc, d, P)
        v = (u + float(rng.uniform(0.3, 2.0)) * (v - u)).astype(np.float32)
        s = orc.stats(cb, u, w, v, 1.0)
        du = orc.sqdist64(v, u)
        if s["cos_beta"] < 1e-3 or abs(s["pes_term"]) < 1e-9:
            continue
        assert (s["pes_term"] < 0) == (s["est"] > du)
        if abs(s["cos_alpha"] - s["delta"]) > 1e-6:
            assert (s["cos_alpha"] > s["delta"]) == (orc.sqdist64(v, w) < du)
        checked += 1
    assert checked > 250
