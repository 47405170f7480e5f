"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

Each test states which part of the oracle it pins and against what (a published vector, a
hand-computed row, a closed form, a library routine, an order property, brute force).
"""
import itertools
import math
import os

import numpy as np
import pytest
from scipy import special, stats

from oracle import simple_oracle as O
from paper_2512_00719_amd import synth


def _par(**kw):
    return synth.make_params(1, **kw)[0]


# ------------------------------------------------------------------ Philox ----------------------
def test_philox_against_library_engine(tmp_path):
    """Philox4x32-10 against an independent library routine: the counter-based engine in PyTorch's
    ATen headers (at::philox_engine), compiled here with g++ and run on the CPU.  A wrong round
    constant, multiplier, word order or round count in the oracle fails this."""
    import shutil
    import subprocess
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    gxx = shutil.which("g++")
    if gxx is None or not os.path.exists(os.path.join(inc, "ATen", "core", "PhiloxRNGEngine.h")):
        pytest.skip("g++ or the ATen Philox header is not available")
    exe = str(tmp_path / "philox_library_check")
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "philox_library_check.cpp")
    subprocess.run([gxx, "-O1", "-std=c++17", "-I", inc, src, "-o", exe], check=True)
    rng = np.random.default_rng(11)
    cases = [(0, 0, 0), (2 ** 64 - 1, 2 ** 64 - 1, 2 ** 64 - 1), (synth.SAMPLER_SEED, 5 << 32, 123)]
    cases += [tuple(int(x) for x in rng.integers(0, 2 ** 63, 3)) for _ in range(200)]
    args = [str(v) for c in cases for v in c]
    out = subprocess.run([exe, *args], check=True, capture_output=True, text=True).stdout.split("\n")
    for (seed, subseq, offset), line in zip(cases, out):
        ctr = np.array([offset & 0xFFFFFFFF, offset >> 32, subseq & 0xFFFFFFFF, subseq >> 32], np.uint32)
        key = np.array([seed & 0xFFFFFFFF, seed >> 32], np.uint32)
        got = [int(x) for x in O.philox4x32_10(ctr, key)]
        assert got == [int(x, 16) for x in line.split()], (seed, subseq, offset)
    # the round constants have closed forms: the golden ratio and sqrt(3) - 1 in 32-bit fixed point
    assert O._PHILOX_W0 == int(((5 ** 0.5 - 1) / 2) * 2 ** 32) and O._PHILOX_W1 == int((3 ** 0.5 - 1) * 2 ** 32)


def test_philox_vectorised_matches_scalar_and_is_uniform():
    rows = np.arange(1 << 18)
    u0, u1, u2 = O.row_uniforms(synth.SAMPLER_SEED, rows, 7)
    for i in (0, 1, 77777, (1 << 18) - 1):
        s = O.row_uniforms(synth.SAMPLER_SEED, np.array(i), 7)
        assert (float(s[0]), float(s[1]), float(s[2])) == (u0[i], u1[i], u2[i])
    for u in (u0, u1, u2):
        assert u.min() >= 0.0 and u.max() < 1.0
        assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))  # 24-bit uniforms
        counts = np.bincount((u * 256).astype(int), minlength=256)
        assert stats.chisquare(counts).pvalue > 1e-4
    # the three words are distinct streams, and (row, step) pairs do not collide
    assert abs(np.corrcoef(u0, u1)[0, 1]) < 0.01 and abs(np.corrcoef(u0, u2)[0, 1]) < 0.01
    rr, ss = np.meshgrid(np.arange(1000, dtype=np.uint32), np.arange(1000, dtype=np.uint32))
    ctr = np.stack([rr.ravel(), ss.ravel(), np.zeros(10 ** 6, np.uint32), np.zeros(10 ** 6, np.uint32)], -1)
    blocks = O.philox4x32_10(ctr, np.array([1, 2], np.uint32))
    assert np.unique(blocks, axis=0).shape[0] == 10 ** 6  # a bijection per key: no two blocks equal
    # a step above 2^32 reaches the third counter word
    assert O.row_uniforms(1, np.array(3), 5)[0] != O.row_uniforms(1, np.array(3), 5 + (1 << 32))[0]
    # the seed's high word is part of the key
    assert O.row_uniforms(1, np.array(3), 5)[0] != O.row_uniforms(1 + (1 << 32), np.array(3), 5)[0]
    # a global row index above 2^32 reaches the fourth counter word: word placement checked against
    # the block function itself
    big = (7 << 32) + 3
    assert O.row_uniforms(1, np.array(3), 5)[0] != O.row_uniforms(1, np.array(big, dtype=np.uint64), 5)[0]
    x = O.philox4x32_10(np.array([3, 5, 9, 7], np.uint32), np.array([1, 0], np.uint32))
    u = O.row_uniforms(1, np.array(big, dtype=np.uint64), 5 + (9 << 32))
    assert [float(v) for v in u] == [float(int(w) >> 8) * 2.0 ** -24 for w in x[:3]]


# ------------------------------------------------------------------ penalties -------------------
def _penalty_cases(golden_dir):
    cases, cur = [], None
    for line in open(os.path.join(golden_dir, "penalty_rows.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "case":
            cur = {"name": t[1]}
            cases.append(cur)
        elif t[0] == "par":
            cur["par"] = (int(t[1]), float(t[2]), float(t[3]), float(t[4]))
        elif t[0] == "hist":
            cur["hist"] = np.array([int(x) for x in t[1:]], np.int32)
        else:
            cur[t[0]] = np.array([float(x) for x in t[1:]], np.float32)
    return cases


def test_penalties_hand_computed_rows(golden_dir):
    """Section 2.2 histogram -> mask -> factor, plus frequency/presence, on hand-computed rows."""
    cases = _penalty_cases(golden_dir)
    assert len(cases) == 4
    for c in cases:
        n_prompt, rep, freq, pres = c["par"]
        c_o, mask = O.history_histograms(c["hist"], n_prompt, c["z"].size)
        got = O.apply_penalties(c["z"], c_o, mask, rep, freq, pres)
        assert got.dtype == np.float32
        np.testing.assert_array_equal(got, c["expect"], err_msg=c["name"])
        lit = O.apply_penalties(c["z"], c_o, mask, rep, freq, pres, literal_division=True)
        np.testing.assert_array_equal(lit, c["literal"], err_msg=c["name"])


def test_penalties_invariants():
    rng = np.random.default_rng(1)
    V = 500
    z = rng.standard_normal(V).astype(np.float32) * 3
    z[7] = -0.0
    hist = rng.integers(0, V, 200).astype(np.int32)
    c_o, mask = O.history_histograms(hist, 50, V)
    out = O.apply_penalties(z, c_o, mask, 1.3, 0.4, 0.2)
    untouched = ~mask
    assert untouched.sum() > 0
    # columns outside the history are bit-identical (invariant named in the problem statement)
    np.testing.assert_array_equal(out[untouched].view(np.uint32), z[untouched].view(np.uint32))
    # every penalised column moved down (rep > 1, freq, pres > 0)
    assert np.all(out[mask] <= z[mask])
    # multiplicity: a token generated n times loses n*freq
    zz = np.array([10.0, 10.0], np.float32)
    for n in (1, 2, 5, 40):
        c_o, m = O.history_histograms(np.zeros(n, np.int32), 0, 2)
        got = O.apply_penalties(zz, c_o, m, 1.0, 0.25, 0.0)
        assert got[0] == np.float32(10.0 - 0.25 * n) and got[1] == 10.0
    # all penalties off is the identity, bit for bit
    c_o, mask = O.history_histograms(hist, 0, V)
    np.testing.assert_array_equal(O.apply_penalties(z, c_o, mask, 1.0, 0.0, 0.0).view(np.uint32),
                                  z.view(np.uint32))
    # incremental histogram update of section 5.2 (Eq. cpu-incremental) equals rebuilding it
    c_prev, _ = O.history_histograms(hist[:-1], 0, V)
    c_step = np.bincount(hist[-1:], minlength=V)
    np.testing.assert_array_equal(c_prev + c_step, c_o)
    with pytest.raises(ValueError):
        O.history_histograms(np.array([V]), 0, V)


# ------------------------------------------------------------------ filters ---------------------
def test_top_k_brute_force_with_ties():
    """top-k keeps exactly k, a prefix of (value descending, id ascending): every y in {0,1,2}^5."""
    V = 5
    for y in itertools.product((0.0, 1.0, 2.0), repeat=V):
        z = np.array(y, np.float32)
        ranked = sorted(range(V), key=lambda i: (-y[i], i))
        for k in range(1, V + 1):
            d = O.row_distribution(z, _par(top_k=k))
            assert list(d.ids) == sorted(ranked[:k]), (y, k)
        assert O.row_distribution(z, _par(top_k=1)).ids[0] == int(np.argmax(z))


def test_top_k_order_property_and_noop():
    rng = np.random.default_rng(2)
    V = 300
    z = np.round(rng.standard_normal(V) * 4).astype(np.float32) / 4  # many ties
    for k in (1, 2, 17, 299):
        d = O.row_distribution(z, _par(top_k=k, temperature=0.7))
        inside = np.zeros(V, bool)
        inside[d.ids] = True
        assert inside.sum() == k
        # every survivor beats every non-survivor in (value desc, id asc)
        for v in np.flatnonzero(inside):
            for u in np.flatnonzero(~inside):
                assert (z[v] > z[u]) or (z[v] == z[u] and v < u)
    full = O.row_distribution(z, _par())
    for k in (0, -3, V, V + 10):
        d = O.row_distribution(z, _par(top_k=k))
        np.testing.assert_array_equal(d.ids, full.ids)
    assert full.n == V


def test_min_p_postcondition():
    rng = np.random.default_rng(3)
    V = 2000
    for trial in range(5):
        z = (rng.standard_normal(V) * 2).astype(np.float32)
        tau = np.float32(0.9)
        p = special.softmax((z / tau).astype(np.float64))
        for min_p in (0.01, 0.05, 0.3):
            d = O.row_distribution(z, _par(min_p=min_p, temperature=tau))
            inside = np.zeros(V, bool)
            inside[d.ids] = True
            ratio = p / p.max()
            assert np.all(ratio[inside] >= min_p * (1 - 1e-5))
            assert np.all(ratio[~inside] <= min_p * (1 + 1e-5))
            assert d.n == d.n_m


def test_top_p_postcondition_monotone_and_noop():
    rng = np.random.default_rng(4)
    V = 3000
    z = (rng.standard_normal(V) * 2.5).astype(np.float32)
    y = (z / np.float32(0.8)).astype(np.float32).astype(np.float64)
    w = {i: math.exp(y[i] - y.max()) for i in range(V)}
    ranked = sorted(range(V), key=lambda i: (-y[i], i))
    prev = set()
    for top_p in (0.1, 0.5, 0.8, 0.95, 0.999):
        for k in (0, 200):
            d = O.row_distribution(z, _par(top_p=top_p, top_k=k, temperature=0.8))
            nk = k if k else V
            S_k = math.fsum(w[i] for i in ranked[:nk])
            K = list(d.ids)
            assert sorted(ranked[:d.n]) == K  # a prefix of the order
            target = float(np.float32(top_p)) * S_k
            assert math.fsum(w[i] for i in ranked[:d.n]) >= target * (1 - 1e-12)
            assert math.fsum(w[i] for i in ranked[:d.n - 1]) < target * (1 + 1e-12)
        d = O.row_distribution(z, _par(top_p=top_p, temperature=0.8))
        assert prev <= set(d.ids)
        prev = set(d.ids)
    assert O.row_distribution(z, _par(top_p=1.0)).n == V
    assert O.row_distribution(z, _par(top_p=0.0)).n == 1
    # top-p inside top-k: mass is relative to the top-k prefix
    d = O.row_distribution(z, _par(top_p=0.5, top_k=10, temperature=0.8))
    S10 = math.fsum(w[i] for i in ranked[:10])
    assert math.fsum(w[i] for i in ranked[:d.n]) >= 0.5 * S10 > math.fsum(w[i] for i in ranked[:d.n - 1])


def test_truncated_softmax_equals_masked_softmax():
    """Section 5.2: softmax on K_b equals the masked softmax over V (library softmax, -inf mask)."""
    rng = np.random.default_rng(5)
    V = 1500
    z = (rng.standard_normal(V) * 3).astype(np.float32)
    for par in (_par(top_k=40, temperature=0.6), _par(top_p=0.9, temperature=1.1),
                _par(min_p=0.02), _par(top_k=100, top_p=0.7, min_p=0.01, temperature=0.75), _par()):
        d = O.row_distribution(z, par)
        y = (z / np.float32(par["temperature"])).astype(np.float32).astype(np.float64)
        masked = np.full(V, -np.inf)
        masked[d.ids] = y[d.ids]
        ref = special.softmax(masked)
        p = d.probs()
        np.testing.assert_allclose(p, ref, rtol=1e-12, atol=0)
        assert abs(p.sum() - 1) < 1e-12
        assert np.all(p[np.setdiff1d(np.arange(V), d.ids)] == 0)


def test_filter_composition_is_shortest_prefix():
    """K_b against a prefix formed independently: sort once (value descending, id ascending), then
    three explicit scans for the lengths the filters allow, in exact rational-free arithmetic
    (math.fsum), and the shortest wins.  Pins the composition rule and each n_* of the oracle."""
    rng = np.random.default_rng(6)
    V = 4000
    z = (rng.standard_normal(V) * 2).astype(np.float32)
    z[[5, 17, 900]] = z[3]  # ties, also where a cut may fall
    for k, p, m, tau in ((50, 0.9, 0.0, 0.8), (50, 0.3, 0.0, 0.8), (0, 0.9, 0.05, 0.8), (1000, 0.99, 0.2, 1.3),
                         (5, 1.0, 0.5, 0.7), (0, 0.97, 0.0, 1.1), (3, 0.999, 1e-4, 1.0)):
        par = _par(top_k=k, top_p=p, min_p=m, temperature=tau)
        d = O.row_distribution(z, par)
        y = [float(np.float32(v) / np.float32(tau)) for v in z]            # IEEE float32 quotient
        order = sorted(range(V), key=lambda i: (-y[i], i))
        w = [math.exp(y[i] - y[order[0]]) for i in order]
        n_k = k if 1 <= k < V else V
        n_m = V
        if m > 0:
            thr = float(np.float32(np.float32(y[order[0]]) + np.float32(math.log(float(np.float32(m))))))
            n_m = 0
            while n_m < V and y[order[n_m]] >= thr:
                n_m += 1
        n_p = n_k
        if p < 1:
            target = float(np.float32(p)) * math.fsum(w[:n_k])
            n_p = 1
            while math.fsum(w[:n_p]) < target:
                n_p += 1
        n = max(1, min(n_k, n_m, n_p))
        assert (d.n_k, d.n_m, d.n_p, d.n) == (n_k, n_m, n_p, n), (k, p, m, tau)
        assert sorted(order[:n]) == d.ids.tolist()


def test_degenerate_rows():
    z = np.array([1.0, np.nan, 0.0], np.float32)
    assert O.row_distribution(z, _par()).error
    assert O.row_distribution(np.array([1.0, np.inf], np.float32), _par()).error
    assert O.row_distribution(np.full(4, -np.inf, np.float32), _par()).error
    assert O.row_distribution(np.zeros(4, np.float32), _par(temperature=-1.0)).error
    d = O.row_distribution(np.array([0.0, -np.inf, 0.0, -1.0], np.float32), _par())
    assert d.n == 4 and d.probs()[1] == 0.0
    ids, _, _ = O.draw(d, np.linspace(0, 1, 1000, endpoint=False))
    assert 1 not in set(ids.tolist())
    # +0 and -0 tie; lowest id wins
    d = O.row_distribution(np.array([-0.0, 0.0, -1.0], np.float32), _par(top_k=1))
    assert list(d.ids) == [0]
    # greedy: argmax of the penalised logits, lowest id on ties, filters ignored
    g = O.row_distribution(np.array([1.0, 3.0, 3.0, 2.0], np.float32), _par(temperature=0.0, top_k=3),
                           np.array([1], np.int32))
    assert g.greedy and g.greedy_id == 1
    g = O.row_distribution(np.array([1.0, 3.0, 3.0, 2.0], np.float32),
                           _par(temperature=0.0, rep_penalty=2.0), np.array([1], np.int32))
    assert g.greedy_id == 2


# ------------------------------------------------------------------ draw ------------------------
def test_draw_exhaustive_enumeration_of_all_uniforms():
    """All 2^24 values of u_draw on tiny vocabularies: the count of each id equals p~ * 2^24 up to
    one per CDF step, and a filtered-out token is never drawn."""
    u = np.arange(1 << 24, dtype=np.float64) * 2.0 ** -24
    rng = np.random.default_rng(7)
    for V, par in ((5, _par()), (16, _par(top_k=6, temperature=0.7)), (12, _par(top_p=0.8)),
                   (16, _par(min_p=0.1, temperature=1.3))):
        z = (rng.standard_normal(V) * 1.5).astype(np.float32)
        d = O.row_distribution(z, par)
        ids, _, _ = O.draw(d, u)
        counts = np.bincount(ids, minlength=V)
        expect = d.probs() * (1 << 24)
        assert np.all(np.abs(counts - expect) <= d.n)
        assert np.all(counts[np.setdiff1d(np.arange(V), d.ids)] == 0)
        # walk order is ascending token id: ids are non-decreasing in u
        assert np.all(np.diff(ids) >= 0)


# ------------------------------------------------------------------ SHVS ------------------------
def _tiny_row(rng, V=8):
    return (rng.standard_normal(V) * 1.2).astype(np.float32)


def test_shvs_identities_on_masses():
    """Eq. (7)-(9): p~/q = alpha on H, and alpha*q + (1-alpha)*r reproduces p~ exactly."""
    rng = np.random.default_rng(8)
    V = 64
    z = _tiny_row(rng, V)
    d = O.row_distribution(z, _par(top_k=20, temperature=0.9))
    for hot_ids in (rng.permutation(V)[:16], np.arange(V), rng.permutation(V)[:1]):
        hm = O.hot_mask_from_ids(hot_ids, V)
        S_H, S_T, alpha = O.shvs_masses(d, hm)
        p = d.probs()
        hot = hm[d.ids]
        q = np.zeros(V)
        r = np.zeros(V)
        if S_H > 0:
            q[d.ids[hot]] = d.w[hot] / S_H
        if S_T > 0:
            r[d.ids[~hot]] = d.w[~hot] / S_T
        np.testing.assert_allclose(alpha * q + (1 - alpha) * r, p, rtol=0, atol=1e-15)
        if S_H > 0:
            sel = d.ids[hot]
            np.testing.assert_allclose(p[sel] / q[sel], alpha, rtol=1e-12)
        assert abs(alpha - p[hm].sum()) < 1e-12  # alpha_b is the covered mass (section 4.1)


@pytest.mark.parametrize("H", [1, 4, 7, 8])
def test_shvs_exact_on_uniform_grid(H):
    """Enumerate a G x G grid of (u_acc, u_draw) and (u_acc, u_tail): the resulting distribution is
    p~ up to the grid resolution for every hot-set size (exactness does not depend on H)."""
    rng = np.random.default_rng(9)
    V, G = 8, 2048
    z = _tiny_row(rng, V)
    d = O.row_distribution(z, _par(top_k=6))
    hm = O.hot_mask_from_ids(rng.permutation(V)[:H], V)
    g = np.arange(G) / G
    ua, ud = np.meshgrid(g, g, indexing="ij")
    ids, _, _ = O.draw(d, ud.ravel(), ua.ravel(), ud.ravel()[::-1].copy(), hm)
    # u_tail must be independent of u_acc: use a second enumeration for the tail variate
    ids_t, _, acc = O.draw(d, np.zeros(G * G), ua.ravel(), ud.ravel(), hm)
    ids = np.where(acc, ids, ids_t)
    freq = np.bincount(ids, minlength=V) / (G * G)
    np.testing.assert_allclose(freq, d.probs(), atol=3.0 / G)


def test_shvs_chi_square_and_planted_biased_fallback():
    """Real Philox uniforms over 2*10^5 steps: SHVS output fits p~ (chi-square), the acceptance
    rate fits alpha, and re-running the full sampler on rejection (a planted mistake) is caught."""
    rng = np.random.default_rng(10)
    V, N = 200, 200_000
    steps = np.arange(N)
    pvals = []
    for row in range(3):
        z = (rng.standard_normal(V) * 2.0).astype(np.float32)
        d = O.row_distribution(z, _par(top_p=0.97, temperature=1.1))
        hm = O.hot_mask_from_ids(np.argsort(-z)[:12], V)
        alpha = O.shvs_masses(d, hm)[2]
        assert 0.2 < alpha < 0.95
        u_draw, u_acc, u_tail = O.row_uniforms(synth.SAMPLER_SEED, np.full(N, row), steps)
        p = d.probs()
        for biased in (False, True):
            ids, _, acc = O.draw(d, u_draw, u_acc, u_tail, hm, biased_fallback=biased)
            counts = np.bincount(ids, minlength=V).astype(float)
            order = np.argsort(-p)
            e, c = p[order] * N, counts[order]
            cut = int(np.searchsorted(-e, -5.0))  # pool the tail so every expected count is >= 5
            e = np.append(e[:cut], e[cut:].sum())
            c = np.append(c[:cut], c[cut:].sum())
            if e[-1] < 5:
                e, c = np.append(e[:-2], e[-2:].sum()), np.append(c[:-2], c[-2:].sum())
            pv = stats.chisquare(c, e * c.sum() / e.sum()).pvalue
            if biased:
                assert pv < 1e-9
            else:
                pvals.append(pv)
                assert abs(acc.mean() - alpha) < 4 * math.sqrt(alpha * (1 - alpha) / N)
                assert np.all(counts[p == 0] == 0)
    assert min(pvals) > 1e-3 / len(pvals)


def test_shvs_special_cases():
    rng = np.random.default_rng(11)
    V = 500
    z = (rng.standard_normal(V) * 2).astype(np.float32)
    par = _par(top_k=30, top_p=0.95, temperature=0.8)
    d = O.row_distribution(z, par)
    N = 20000
    u_draw, u_acc, u_tail = O.row_uniforms(5, np.zeros(N, int), np.arange(N))
    full, _, _ = O.draw(d, u_draw)
    # hot set = whole vocabulary: always accepted, identical ids to the full path
    ids, _, acc = O.draw(d, u_draw, u_acc, u_tail, np.ones(V, bool))
    assert acc.all() and np.array_equal(ids, full)
    # K_b inside H: alpha = 1, always accepted
    hm = np.zeros(V, bool)
    hm[d.ids] = True
    hm[np.setdiff1d(np.arange(V), d.ids)[:50]] = True
    ids, _, acc = O.draw(d, u_draw, u_acc, u_tail, hm)
    assert acc.all() and np.array_equal(ids, full) and O.shvs_masses(d, hm)[2] == 1.0
    # H disjoint from K_b: never accepted, tail draw over all of K_b with u_tail
    hm = np.ones(V, bool)
    hm[d.ids] = False
    ids, _, acc = O.draw(d, u_draw, u_acc, u_tail, hm)
    assert (~acc).all() and np.array_equal(ids, O.draw(d, u_tail)[0])
    with pytest.raises(ValueError):
        O.hot_mask_from_ids([1, 1], V)
    with pytest.raises(ValueError):
        O.hot_mask_from_ids([V], V)


def test_shvs_alpha_closed_form_zipf():
    """Noise-free Zipf(1.2) profile, temperature 1, no filter: alpha(H) is a ratio of partial sums
    of r^-1.2 (direct summation)."""
    V = 201_088
    ranks = np.arange(1, V + 1, dtype=np.float64)
    z = (-1.2 * np.log(ranks)).astype(np.float32)
    d = O.row_distribution(z, _par())
    terms = [r ** -1.2 for r in range(1, V + 1)]
    total = math.fsum(terms)
    for H, printed in ((4096, 0.9006), (8192, 0.9244), (16384, 0.9451), (32768, 0.9631)):
        alpha = O.shvs_masses(d, O.hot_mask_from_ids(np.arange(H), V))[2]
        closed = math.fsum(terms[:H]) / total
        assert abs(alpha - closed) < 1e-6
        assert round(closed, 4) == printed


# ------------------------------------------------------------------ whole call ------------------
def test_rows_are_independent_and_keyed_by_global_row():
    """Section 5.1: any partition of the batch gives the same ids (row_offset keys the RNG)."""
    w = synth.make_config(1)
    z = w.logits_f32()
    whole = [r.id for r in O.sample(z, w.params, w.hist_ptr, w.hist_ids, None, w.seed, 3)]
    parts = []
    for b in range(w.B):
        hp = w.hist_ptr[b:b + 2] - w.hist_ptr[b]
        hi = w.hist_ids[w.hist_ptr[b]:w.hist_ptr[b + 1]]
        parts.append(O.sample(z[b:b + 1], w.params[b:b + 1], hp, hi, None, w.seed, 3, row_offset=b)[0].id)
    assert whole == parts
    other = [r.id for r in O.sample(z, w.params, w.hist_ptr, w.hist_ids, None, w.seed, 4)]
    assert all(0 <= t < w.V for t in whole + other)


def test_top_k_one_is_argmax_and_filtered_tokens_never_drawn():
    w = synth.make_config(3, B=8, V=4096, nnz=128)
    z = w.logits_f32()
    par = w.params.copy()
    par["top_k"] = 1
    par["temperature"] = np.maximum(par["temperature"], 0.5)
    res = O.sample(z, par, w.hist_ptr, w.hist_ids, None, w.seed, 0, keep_dist=True)
    for b, r in enumerate(res):
        c_o, mask = O.history_histograms(w.hist_ids[w.hist_ptr[b]:w.hist_ptr[b + 1]], 0, w.V)
        zp = O.apply_penalties(z[b], c_o, mask, par[b]["rep_penalty"], par[b]["freq_penalty"],
                               par[b]["pres_penalty"])
        assert r.id == int(np.argmax(zp))
    res = O.sample(z, w.params, w.hist_ptr, w.hist_ids, None, w.seed, 0, keep_dist=True)
    for step in range(50):
        for b, r in enumerate(O.sample(z, w.params, w.hist_ptr, w.hist_ids, None, w.seed, step)):
            d = res[b].dist
            assert r.id == d.greedy_id if d.greedy else r.id in set(d.ids.tolist())


def test_ambiguity_protocol_reports_neighbours():
    """A uniform placed on a CDF step is flagged and both neighbouring ids are acceptable."""
    z = np.log(np.array([0.25, 0.25, 0.5], np.float64)).astype(np.float32)
    d = O.row_distribution(z, _par())
    ids, margin, _ = O.draw(d, np.array([0.25 - 1e-9, 0.25 + 1e-9, 0.1]))
    assert list(ids) == [0, 1, 0] and margin[0] < 1e-6 and margin[1] < 1e-6 and margin[2] > 0.09


def test_neighbours_are_the_adjacent_ids_of_the_walk():
    """`_neighbours`: the ids next to a token in the CDF walk that produced it (all of K_b without a
    hot set; the hot or the tail members of K_b with one), hand-listed."""
    d = O.RowDist(V=32, ids=np.array([3, 7, 8, 20]), w=np.ones(4), n=4)
    assert O._neighbours(d, 7, None, None) == {3, 8}
    assert O._neighbours(d, 3, None, None) == {7}
    assert O._neighbours(d, 20, None, None) == {8}
    hot = np.zeros(32, bool)
    hot[[7, 20, 31]] = True
    assert O._neighbours(d, 7, hot, True) == {20}     # hot walk: 7, 20
    assert O._neighbours(d, 20, hot, True) == {7}
    assert O._neighbours(d, 8, hot, False) == {3}     # tail walk: 3, 8
    assert O._neighbours(d, 3, hot, False) == {8}


def _nucleus_row():
    """Five exactly representable logits at temperature 1: w = e^0 .. e^-4, hand-summed."""
    z = np.array([-1.0, 2.0, 0.0, -2.0, 1.0], np.float32)    # order by value: ids 1, 4, 2, 0, 3
    w = [math.exp(-i) for i in range(5)]
    S = math.fsum(w)
    return z, w, S


def _f32_below(x):
    t = np.float32(x)
    return t if float(t) < x else np.nextafter(t, np.float32(-np.inf))


def test_nucleus_ambiguity_alternatives_hand_built():
    """The branch that builds RowDist.alt / RowResult.alt_p.  top_p is placed one float32 step
    below and above the mass of the two-token prefix (the boundary is then within 1e-7 of the
    target: exactly one alternative, the prefix one longer / one shorter, with hand-computed p~),
    and 1e-3 below it (no alternative, not ambiguous)."""
    z, w, S = _nucleus_row()
    r2 = (w[0] + w[1]) / S
    p_lo = _f32_below(r2)
    p_hi = np.nextafter(p_lo, np.float32(np.inf))
    if float(p_hi) <= r2:
        p_hi = np.nextafter(p_hi, np.float32(np.inf))
    assert float(p_lo) < r2 < float(p_hi) and float(p_hi) - float(p_lo) < 2e-7
    d = O.row_distribution(z, _par(top_p=p_lo))
    assert d.n == 2 and d.ids.tolist() == [1, 4] and d.nucleus_margin < 1e-6
    assert [(a.n, a.ids.tolist()) for a in d.alt] == [(3, [1, 2, 4])]
    d = O.row_distribution(z, _par(top_p=p_hi))
    assert d.n == 3 and d.ids.tolist() == [1, 2, 4] and d.nucleus_margin < 1e-6
    assert [(a.n, a.ids.tolist()) for a in d.alt] == [(2, [1, 4])]
    d = O.row_distribution(z, _par(top_p=np.float32(r2 - 1e-3)))
    assert d.n == 2 and d.alt == [] and 0.9e-3 < d.nucleus_margin < 1.1e-3
    # a top-k cut at the same place removes the longer alternative (the nucleus never exceeds n_k)
    d = O.row_distribution(z, _par(top_p=np.float32(0.999999), top_k=2))
    assert d.n == 2 and d.alt == []


def test_sample_row_alternatives_and_alt_p(monkeypatch):
    """sample_row's ambiguity protocol end to end, with the uniforms planted: ids and p~ of the
    neighbouring prefix, the neighbours of a draw on a CDF step, and none of it away from boundaries."""
    z, w, S = _nucleus_row()
    r2 = (w[0] + w[1]) / S

    def plant(u_draw, u_acc=0.5, u_tail=0.5):
        monkeypatch.setattr(O, "row_uniforms", lambda seed, rows, step: (np.float64(u_draw), np.float64(u_acc), np.float64(u_tail)))

    # walk in ascending id over K = {1, 4}: id 1 holds [0, w0 / (w0 + w1)), id 4 the rest
    s2, s3 = w[0] + w[1], w[0] + w[1] + w[2]
    plant(0.9)
    r = O.sample_row(z, _par(top_p=_f32_below(r2)), None, None, 1, 0, 0)
    assert r.id == 4 and r.ambiguous and r.n == 2
    assert abs(r.p_chosen - w[1] / s2) < 1e-15 and len(r.alt_p) == 1 and abs(r.alt_p[0] - w[1] / s3) < 1e-15
    # under the alternative K = {1, 2, 4} (masses w0, w2, w1 in id order) u = 0.9 falls on id 4 too
    # (0.9 * s3 > w0 + w2); what is forgiven is that draw and its neighbour in the alternative's walk
    assert 0.9 * s3 > w[0] + w[2] and r.alt_ids == {2}
    plant(0.74)  # K = {1, 4}: 0.74 * s2 > w0 -> id 4; K = {1, 2, 4}: 0.74 * s3 in [w0, w0 + w2) -> id 2
    assert 0.74 * s2 > w[0] and w[0] <= 0.74 * s3 < w[0] + w[2]
    r = O.sample_row(z, _par(top_p=_f32_below(r2)), None, None, 1, 0, 0)
    assert r.id == 4 and r.ambiguous and 2 in r.alt_ids and len(r.alt_p) == 1
    # away from the nucleus boundary and from every CDF step: nothing is forgiven
    r = O.sample_row(z, _par(top_p=np.float32(r2 - 1e-3)), None, None, 1, 0, 0)
    assert r.id == 4 and not r.ambiguous and r.alt_ids == set() and r.alt_p == ()
    # a uniform 1e-9 (relative) past the CDF step between ids 1 and 4: flagged, the other side allowed
    plant(w[0] / s2 + 1e-9)
    r = O.sample_row(z, _par(top_p=np.float32(r2 - 1e-3)), None, None, 1, 0, 0)
    assert r.id == 4 and r.ambiguous and r.alt_ids == {1} and r.alt_p == ()
    # SHVS: an acceptance test within the window allows the other proposal's draw
    hot = np.zeros(5, bool)
    hot[1] = True
    alpha = w[0] / s2
    plant(0.3, u_acc=alpha + 1e-9, u_tail=0.4)
    r = O.sample_row(z, _par(top_p=np.float32(r2 - 1e-3)), None, hot, 1, 0, 0)
    assert r.accepted is False and r.id == 4 and r.ambiguous and r.alt_ids == {1}
    plant(0.3, u_acc=alpha - 1e-3, u_tail=0.4)
    r = O.sample_row(z, _par(top_p=np.float32(r2 - 1e-3)), None, hot, 1, 0, 0)
    assert r.accepted is True and r.id == 1 and not r.ambiguous and r.alt_ids == set()


def test_ambiguity_flags_on_headline_shaped_rows():
    """On rows shaped like the headline configuration (V = 128,256, mixed controls, history): a row
    is flagged for its nucleus exactly when a neighbouring prefix mass, re-summed here in extended
    precision, lies within 1e-6 of the target (a wide nucleus ends among columns of probability
    1e-7 and less, so a few percent of such rows are, by the window's definition); draws flagged
    for a CDF step are rarer than 1e-3; and what a flagged row forgives is a handful of ids, never
    a class of rows wholesale."""
    w = synth.make_config(3, B=192)
    n_nucleus = n_step = total = 0
    for step in range(3):
        res = O.sample(w.logits, w.params, w.hist_ptr, w.hist_ids, None, w.seed, step, keep_dist=True)
        for b, r in enumerate(res):
            d, par = r.dist, w.params[b]
            total += 1
            assert len(r.alt_ids) <= 6
            if d.greedy:
                assert not r.ambiguous and not r.alt_ids
                continue
            if step == 0 and par["top_p"] < 1:
                c_o, mask = O.history_histograms(w.hist_ids[w.hist_ptr[b]:w.hist_ptr[b + 1]], 0, w.V)
                zp = O.apply_penalties(w.logits[b], c_o, mask, par["rep_penalty"], par["freq_penalty"], par["pres_penalty"])
                y = np.sort((zp / np.float32(par["temperature"])).astype(np.float32))[::-1]
                mass = np.exp(y[:d.n_k].astype(np.longdouble) - np.longdouble(y[0]))
                cum = np.cumsum(mass)
                target = np.longdouble(np.float32(par["top_p"])) * cum[-1]
                n_p = int(np.argmax(cum >= target)) + 1
                want = set()
                if n_p < d.n_k and (cum[n_p - 1] - target) / cum[-1] < 1e-6:
                    want.add(n_p + 1)
                if n_p >= 2 and (target - cum[n_p - 2]) / cum[-1] < 1e-6:
                    want.add(n_p - 1)
                want = {max(1, min(d.n_k, d.n_m, q)) for q in want} - {d.n}
                assert d.n_p == n_p and {a.n for a in d.alt} == want, (b, n_p, want, [a.n for a in d.alt])
            if d.alt:
                n_nucleus += 1
                assert r.ambiguous
            elif r.ambiguous:
                n_step += 1
    assert total == 576 and n_step <= 1 and n_nucleus <= 0.08 * total, (n_step, n_nucleus, total)


def test_incremental_history_equals_the_rebuild_at_every_step():
    """Section 5.2: the histograms carried by C_o += Hist(Y_s) equal the ones rebuilt from the whole
    token list (prompt first) at every step, through restarts of single sequences and steps on which
    a sequence generates nothing; the token buffer holds the generated tokens row by row."""
    rng = np.random.default_rng(12)
    B, V, L = 5, 50, 40
    st = O.IncrementalHistory(B, V, L)
    prompts = [rng.integers(0, V, int(rng.integers(0, 12))) for _ in range(B)]
    gen = [[] for _ in range(B)]
    for b in range(B):
        st.restart(b, prompts[b])
    for step in range(30):
        if step in (7, 19):  # one sequence ends and its slot is given to a new one
            b = int(rng.integers(0, B))
            prompts[b] = rng.integers(0, V, int(rng.integers(0, 12)))
            gen[b] = []
            st.restart(b, prompts[b])
        ids = rng.integers(0, V, B)
        ids[rng.random(B) < 0.2] = -1
        st.append(ids)
        for b in range(B):
            if ids[b] >= 0:
                gen[b].append(int(ids[b]))
            full = np.concatenate([prompts[b], np.array(gen[b], dtype=np.int64)]).astype(np.int64)
            c_ref, m_ref = O.history_histograms(full, len(prompts[b]), V)
            c_inc, m_inc = st.histograms(b)
            assert np.array_equal(c_ref, c_inc) and np.array_equal(m_ref, m_inc)
            assert st.Y[:len(gen[b]), b].tolist() == gen[b] and np.all(st.Y[len(gen[b]):, b] == -1)
    # hand-computed: prompt (3, 3, 9), generated 9, 4, 9 -> C_o = {9: 2, 4: 1}, mask = {3, 4, 9}
    st = O.IncrementalHistory(1, 12, 8)
    st.restart(0, [3, 3, 9])
    for t in (9, 4, 9):
        st.append([t])
    c, m = st.histograms(0)
    assert {i: int(v) for i, v in enumerate(c) if v} == {9: 2, 4: 1} and np.flatnonzero(m).tolist() == [3, 4, 9]
    # the sampling call on the carried state equals the call on the rebuilt token list
    z = (rng.standard_normal((1, 12)) * 2).astype(np.float32)
    par = synth.make_params(1, rep_penalty=1.3, freq_penalty=0.4, pres_penalty=0.2, top_k=5, temperature=0.8, n_prompt=3)
    a = O.sample_with_state(z, par, st, None, 5, 2)[0]
    b = O.sample(z, par, np.array([0, 6]), np.array([3, 3, 9, 9, 4, 9], np.int32), None, 5, 2)[0]
    assert (a.id, a.n, a.p_chosen) == (b.id, b.n, b.p_chosen)


def test_constraints_hand_computed_and_their_effect_on_the_draw():
    """apply_constraints: a hand-computed row (allow-list masks the rest, biases add in float32 and
    accumulate, a bias on a masked column leaves it masked); an allowed-only support of every draw;
    a large bias makes top-k = 1 pick the biased token; an empty allow-list is an error row."""
    z = np.array([1.5, -2.0, 0.25, 3.0, -0.5], np.float32)
    out = O.apply_constraints(z, [2, 0, 2, 3], [0.5, -1.0, 0.25, 2.0], [0, 2, 4])
    assert out.tolist() == [0.5, -np.inf, 1.0, -np.inf, -0.5] and out.dtype == np.float32
    assert O.apply_constraints(z).tolist() == z.tolist()
    assert O.apply_constraints(z, [1], [np.float32(0.1)])[1] == np.float32(np.float32(-2.0) + np.float32(0.1))
    rng = np.random.default_rng(31)
    zz = (rng.standard_normal(200) * 2).astype(np.float32)
    allow = rng.choice(200, 17, replace=False)
    d = O.row_distribution(O.apply_constraints(zz, allow_ids=allow), _par(temperature=1.3))
    assert set(d.ids[d.w > 0].tolist()) == set(allow.tolist())   # masked columns keep weight zero
    ids, _, _ = O.draw(d, np.linspace(0, 1, 4001)[:-1])
    assert set(ids.tolist()) <= set(allow.tolist())
    j = int(np.argmin(zz))
    d = O.row_distribution(O.apply_constraints(zz, [j], [100.0]), _par(top_k=1))
    assert d.ids.tolist() == [j]
    assert O.row_distribution(O.apply_constraints(zz, allow_ids=[]), _par()).error
