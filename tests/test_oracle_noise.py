"""Pins of the oracle's static-token test at the noise-tolerant threshold (tau = 0.85,
the real-robot setting of Sec. 4.4 / the implementation details) on camera-noise streams
with moving distractors.  What is checked is fixed by geometry, not by the oracle:

  * a patch a and its noisy copy a + e enclose an angle with sin <= |e| / |a|, so with
    every |e_i| <= n and every a_i >= m the similarity is at least sqrt(1 - n^2 / m^2):
    0.866 for n = 8, m = 16, above 17/20.  Every patch that no box touches in either
    frame MUST therefore be static at tau = 17/20;
  * the test is monotone in tau: static at 249/250 implies static at 17/20;
  * Eq. (sim) >= tau as an exact rational comparison (python integers).
CPU only."""
from fractions import Fraction

import numpy as np

import synth
from oracle import vlac_oracle as O

H, PATCH, N = 224, 14, 256


def test_untouched_patches_are_static_under_noise_at_085():
    frames, touched = synth.noisy_scene_stream(H, H, 10, seed=3, patch=PATCH, noise=8, lo=16, hi=80)
    assert np.sqrt(1 - 8 ** 2 / 16 ** 2) > 17 / 20          # the bound the generator's ranges give
    n_tight = 0
    for t in range(1, 10):
        loose = O.select_static(frames[t - 1], frames[t], PATCH, 17, 20, N)
        tight = O.select_static(frames[t - 1], frames[t], PATCH, 249, 250, N)
        untouched = np.flatnonzero(~(touched[t - 1] | touched[t]))
        assert len(untouched) > 150
        assert set(untouched.tolist()) <= set(loose)
        assert set(tight) <= set(loose)
        assert loose == sorted(loose)
        n_tight += len(tight)
    # the simulator threshold is useless on this stream: noise alone takes the similarity
    # of a dim patch to about 1 - sigma^2 / (2 E[v^2]) = 1 - 24 / 5290 < 0.996
    assert n_tight < 9 * 0.5 * N


def test_threshold_085_is_the_exact_rational_comparison():
    frames, _ = synth.noisy_scene_stream(H, H, 4, seed=5, patch=PATCH, noise=20, lo=8, hi=64,
                                         n_distractors=6)
    hits = 0
    for t in range(1, 4):
        terms = O.patch_terms(frames[t - 1], frames[t], PATCH)
        got = set(O.select_static(frames[t - 1], frames[t], PATCH, 17, 20, N))
        for i, (dot, na, nb) in enumerate(terms):
            dot, na, nb = int(dot), int(na), int(nb)
            want = na > 0 and nb > 0 and Fraction(dot * dot, na * nb) >= Fraction(17 * 17, 20 * 20)
            assert (i in got) == want
            hits += want
    assert 0 < hits < 3 * N                                   # both outcomes occur


def test_top_k_under_noise_keeps_the_most_similar():
    frames, _ = synth.noisy_scene_stream(H, H, 3, seed=7, patch=PATCH, noise=8)
    terms = O.patch_terms(frames[1], frames[2], PATCH)
    sims = [Fraction(int(d) * int(d), int(a) * int(b)) for d, a, b in terms]
    passing = [i for i in range(N) if sims[i] >= Fraction(289, 400)]
    for k in (10, 100):
        got = O.select_static(frames[1], frames[2], PATCH, 17, 20, k)
        want = sorted(sorted(passing, key=lambda i: (-sims[i], i))[:k])
        assert got == want
