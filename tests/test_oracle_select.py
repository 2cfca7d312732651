"""Pins of the oracle's token selection (Alg. 1) and layer ratio (Sec. 3.4)
against what the paper and the mathematics fix: closed forms on hand-made
patches, invariants, extremes and brute force.  CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest

import synth
from oracle import vlac_oracle as O


def frames_from_patches(a, b):
    """1x1-pixel 'patches': frame of shape [1, n, 3] per list of rgb triples."""
    fa = np.array(a, dtype=np.uint8).reshape(1, -1, 3)
    fb = np.array(b, dtype=np.uint8).reshape(1, -1, 3)
    return fb, fa  # (prev, cur)


# ---------------- Eq. (sim) on hand-made patches ----------------

def test_sim_hand_values():
    # cur=(3,4,0), prev=(4,3,0): cos = 24/25 exactly
    prev, cur = frames_from_patches([(3, 4, 0)], [(4, 3, 0)])
    (dot, na, nb), = O.patch_terms(prev, cur, 1)
    assert (dot, na, nb) == (24, 25, 25)
    assert O.is_static(dot, na, nb, 24, 25)            # Sim >= 0.96 holds with equality
    assert not O.is_static(dot, na, nb, 97, 100)
    # cur=(1,0,0), prev=(1,1,0): cos = 1/sqrt(2) = 0.70710678...
    prev, cur = frames_from_patches([(1, 0, 0)], [(1, 1, 0)])
    (dot, na, nb), = O.patch_terms(prev, cur, 1)
    assert O.is_static(dot, na, nb, 7071, 10000)
    assert not O.is_static(dot, na, nb, 7072, 10000)
    # the norm of EACH patch enters (a dropped norm would pass this at 0.9)
    prev, cur = frames_from_patches([(10, 0, 0)], [(10, 10, 10)])
    (dot, na, nb), = O.patch_terms(prev, cur, 1)
    assert (dot, na, nb) == (100, 100, 300)
    assert O.is_static(dot, na, nb, 577, 1000) and not O.is_static(dot, na, nb, 578, 1000)


def test_sim_closed_forms():
    rng = np.random.default_rng(1)
    a = rng.integers(1, 120, size=(14, 14, 3), dtype=np.uint8)
    num, den = O.sim_fraction(*O.patch_terms(a, a, 14)[0])
    assert num == den                                   # identical -> exactly 1
    num, den = O.sim_fraction(*O.patch_terms(a, (2 * a).astype(np.uint8), 14)[0])
    assert num == den                                   # brightness scale -> exactly 1
    b = np.zeros_like(a)
    b[:7], a2 = a[:7], a.copy()
    a2[:7] = 0                                          # disjoint supports -> 0
    assert O.patch_terms(b, a2, 14)[0][0] == 0
    assert not O.is_static(*O.patch_terms(b, a2, 14)[0], 1, 1000)


def test_sim_symmetry_cauchy_schwarz_and_float():
    rng = np.random.default_rng(2)
    for _ in range(200):
        a = rng.integers(0, 256, size=(4, 4, 3), dtype=np.uint8)
        b = np.clip(a.astype(int) + rng.integers(-40, 41, size=a.shape), 0, 255).astype(np.uint8)
        (d1, na, nb), = O.patch_terms(b, a, 4)
        (d2, nb2, na2), = O.patch_terms(a, b, 4)
        assert (d1, na, nb) == (d2, na2, nb2)
        assert d1 * d1 <= na * nb
        cos = float(a.astype(np.float64).ravel() @ b.astype(np.float64).ravel()) / math.sqrt(na * nb)
        for tn, td in ((249, 250), (17, 20), (1, 2)):
            if abs(cos - tn / td) > 1e-9:
                assert O.is_static(d1, na, nb, tn, td) == (cos >= tn / td)


def test_zero_norm_reading():
    assert O.is_static(0, 0, 0, 249, 250)               # both black: identical
    assert not O.is_static(0, 0, 77, 249, 250)          # one black: dissimilar
    assert not O.is_static(0, 55, 0, 1, 1000)
    assert O.is_static(0, 55, 0, 0, 1)                  # tau = 0 accepts everything


def test_patch_raster_order_and_extent():
    H, p = 56, 14
    prev = np.full((H, H, 3), 100, dtype=np.uint8)
    for (y, x) in ((0, 0), (15, 30), (55, 55), (13, 14), (14, 13)):
        cur = prev.copy()
        cur[y, x] = (255, 0, 0)
        terms = O.patch_terms(prev, cur, p)
        changed = [i for i, (d, na, nb) in enumerate(terms) if not (d == na == nb)]
        assert changed == [(y // p) * (H // p) + x // p]


# ---------------- threshold and Eq. (topk) ----------------

def test_threshold_extremes():
    prev, cur, _ = synth.frame_pair(56, 56, 14, 5, seed=3)
    assert O.select_static(prev, cur, 14, 0, 1, 16) == list(range(16))       # tau=0
    assert O.select_static(prev, cur, 14, 1, 1, 16) == []                    # tau=1, nothing proportional
    prev2, cur2, _ = synth.frame_pair(56, 56, 14, 5, seed=3, jitter=0)
    redrawn = synth.frame_pair(56, 56, 14, 5, seed=3, jitter=0)[2]
    assert O.select_static(prev2, cur2, 14, 1, 1, 16) == [i for i in range(16) if not redrawn[i]]


def test_tiny_config_construction():
    # re-drawn uniform patches have cosine ~0.75, +-2 jitter ~1: exactly the 48 others pass
    prev, cur, redrawn = synth.frame_pair(112, 112, 14, 16, seed=0)
    got = O.select_static(prev, cur, 14, 249, 250, 64)
    assert got == [i for i in range(64) if not redrawn[i]] and len(got) == 48
    assert len(O.select_static(prev, cur, 14, 249, 250, 32)) == 32


def brute_topk(terms, tn, td, k):
    cand = []
    for i, (d, na, nb) in enumerate(terms):
        if na == 0 and nb == 0:
            s2 = Fraction(1)
        elif na == 0 or nb == 0:
            s2 = Fraction(0)
        else:
            s2 = Fraction(d * d, na * nb)
        if s2 >= Fraction(tn * tn, td * td):
            cand.append((-s2, i))
    return sorted(i for _, i in sorted(cand)[:k])


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force(seed):
    rng = np.random.default_rng(seed)
    H, p = 24, 4
    prev = rng.integers(0, 256, size=(H, H, 3), dtype=np.uint8)
    cur = np.clip(prev.astype(int) + rng.integers(-1, 2, size=prev.shape) *
                  rng.integers(0, 30, size=(H, H, 1)), 0, 255).astype(np.uint8)
    cur[:4, :8] = prev[:4, :8]          # exact ties (Sim = 1) at patches 0 and 1
    cur[8:12, 4:8] = 0                  # a black patch in the current frame only
    terms = O.patch_terms(prev, cur, p)
    for tn, td in ((249, 250), (9, 10), (1, 2)):
        for k in (0, 1, 3, 7, 36):
            got = O.select_static(prev, cur, p, tn, td, k)
            assert got == brute_topk(terms, tn, td, k)
            passers = brute_topk(terms, tn, td, 10 ** 6)
            assert set(got) <= set(passers) and len(got) == min(k, len(passers))


def test_topk_identical_frames():
    rng = np.random.default_rng(5)
    f = rng.integers(0, 256, size=(56, 56, 3), dtype=np.uint8)
    assert O.select_static(f, f, 14, 249, 250, 16) == list(range(16))   # every patch static
    assert O.select_static(f, f, 14, 249, 250, 5) == [0, 1, 2, 3, 4]    # all tied: lower index first


# ---------------- Eq. (ptask), Eq. (pfinal) ----------------

def test_task_relevance_mean_and_layer_mask():
    rng = np.random.default_rng(7)
    a = rng.random((5, 12)).astype(np.float32)
    np.testing.assert_allclose(O.task_relevance(a), a.astype(np.float64).mean(0), rtol=1e-6)
    mask = [1, 0, 0, 1, 0]
    np.testing.assert_allclose(O.task_relevance(a, mask), (a[0].astype(np.float64) + a[3]) / 2, rtol=1e-6)


def test_filter_properties_and_brute_force():
    rng = np.random.default_rng(8)
    for trial in range(50):
        n = int(rng.integers(4, 40))
        s = rng.random(n).astype(np.float32)
        s[rng.integers(0, n, size=3)] = s[0]            # ties
        p_static = sorted(rng.choice(n, size=int(rng.integers(0, n + 1)), replace=False).tolist())
        tau = float(rng.choice([0.0, 0.2, 0.5, 0.7, 1.0, 1.5, -1.0]))
        rel = O.relevant_set(s, tau)
        n_rel = min(max(n - math.floor(float(np.float32(tau)) * n), 0), n)
        assert len(rel) == n_rel
        # brute force: stable argsort of -s gives (score desc, index asc)
        assert rel == set(np.argsort(-s.astype(np.float64), kind="stable")[:n_rel].tolist())
        p_final, order = O.filter_task_relevant(p_static, s, tau)
        assert set(p_final) <= set(p_static) and not (set(p_final) & rel)
        assert set(p_final) == set(p_static) - rel and p_final == sorted(p_final)
        assert sorted(order) == p_final
        keys = [(float(s[v]), v) for v in order]
        assert keys == sorted(keys)
    s = rng.random(10).astype(np.float32)
    assert O.filter_task_relevant(list(range(10)), s, 0.0)[0] == []             # all relevant
    assert O.filter_task_relevant(list(range(10)), s, 1.0)[0] == list(range(10))  # none relevant
    # monotone: larger tau_task -> fewer relevant -> more reuse (Appendix sweep)
    sizes = [len(O.filter_task_relevant(list(range(10)), s, t)[0]) for t in (0.2, 0.3, 0.5, 0.7)]
    assert sizes == sorted(sizes)


# ---------------- Sec. 3.4 ----------------

def test_entropy_closed_forms():
    n = 37
    assert O.layer_entropy(np.full((1, n), 0.3))[0] == pytest.approx(math.log(n), rel=1e-12)
    onehot = np.zeros((1, n))
    onehot[0, 5] = 0.01
    assert O.layer_entropy(onehot)[0] == 0.0
    # two-point distribution (1/4, 3/4), unnormalised input
    e = O.layer_entropy(np.array([[0.1, 0.3, 0.0]]))[0]
    assert e == pytest.approx(-(0.25 * math.log(0.25) + 0.75 * math.log(0.75)), rel=1e-12)


def dist_with_entropy(n, target):
    """a distribution on n points with the given entropy: mix uniform and one-hot by bisection."""
    lo, hi = 0.0, 1.0
    for _ in range(200):
        mid = (lo + hi) / 2
        p = np.full(n, (1 - mid) / n)
        p[0] += mid
        e = -(p * np.log(p)).sum()
        lo, hi = (mid, hi) if e > target else (lo, mid)
    return p


def test_ratio_closed_forms():
    n, layers = 64, 8
    # constant entropy -> every R = 0 -> alpha = 0
    a = np.tile(dist_with_entropy(n, 3.0), (layers, 1))
    assert np.all(O.layer_ratio(a, 5.0) == 0)
    # geometric entropy decay E^l = E^1 (1-r)^(l-1)  ->  R^l = r (l >= 2), alpha^l = min(g (l-1) r, 1)
    r, g = 0.1, 2.0
    a = np.stack([dist_with_entropy(n, 4.0 * (1 - r) ** l) for l in range(layers)])
    want = [min(g * l * r, 1.0) for l in range(layers)]
    np.testing.assert_allclose(O.layer_ratio(a, g), want, atol=1e-9)
    # independent of the scale of A^l_avg
    np.testing.assert_allclose(O.layer_ratio(a * 0.37, g), want, atol=1e-9)


def test_ratio_clamps_and_monotone():
    rng = np.random.default_rng(11)
    a = rng.random((12, 50)) ** 3
    for g in (0.5, 3.0, 40.0):
        al = O.layer_ratio(a, g)
        assert al[0] == 0 and np.all(al >= 0) and np.all(al <= 1) and np.all(np.diff(al) >= 0)
    # rising entropy only -> negative cumulative sum -> clamped at 0
    up = np.stack([dist_with_entropy(50, e) for e in (1.0, 2.0, 3.0)])
    assert np.all(O.layer_ratio(up, 4.0) == 0)
    # entropy ratio does not depend on the log base: redo R with log2 by hand
    ent2 = np.array([-(p / p.sum() * np.log2(p / p.sum())).sum() for p in a])
    cum = np.concatenate([[0], np.cumsum((ent2[:-1] - ent2[1:]) / ent2[:-1])])
    np.testing.assert_allclose(O.layer_ratio(a, 3.0),
                               np.maximum.accumulate(np.clip(3.0 * cum, 0, 1)), atol=1e-9)


def test_layer_counts():
    assert O.layer_reuse_counts([0.0, 0.5, 0.999, 1.0], 100) == [0, 50, 99, 100]
    assert O.layer_reuse_counts([0.3], 0) == [0]


def test_plan_step_no_stats():
    prev, cur, redrawn = synth.frame_pair(112, 112, 14, 16, seed=0)
    p_final, order, per_layer, alpha = O.plan_step(prev, cur, 14, 249, 250, 32, None, 0.5, 1.0)
    assert per_layer is None and alpha is None and order == p_final and len(p_final) == 32


# ---------------- two camera views as one stacked frame ----------------

def test_two_stacked_views_select_like_each_view_alone():
    """The patch test is local to a patch, so two views stacked into one 2H x W frame
    (patches in raster order = view 0's, then view 1's) select what each view selects on
    its own, indices of the second shifted by the first view's patch count; with a
    top-k smaller than that, the k most similar of BOTH views are kept."""
    H, p = 112, 14
    n = (H // p) ** 2
    fr = synth.two_view_stream(H, H, 5, seed=11)
    assert fr.shape == (5, 2 * H, H, 3)
    for t in range(1, 5):
        both = O.select_static(fr[t - 1], fr[t], p, 249, 250, 2 * n)
        top = O.select_static(fr[t - 1][:H], fr[t][:H], p, 249, 250, n)
        bot = O.select_static(fr[t - 1][H:], fr[t][H:], p, 249, 250, n)
        assert both == top + [n + i for i in bot]
        assert len(top) > n // 2 and len(bot) < n // 8          # fixed view static, wrist view not
        terms = O.patch_terms(fr[t - 1], fr[t], p)
        sims = [Fraction(int(d) ** 2, int(a) * int(b)) for d, a, b in terms]
        k = 20
        want = sorted(sorted(both, key=lambda i: (-sims[i], i))[:k])
        assert O.select_static(fr[t - 1], fr[t], p, 249, 250, k) == want
