"""Pin of the oracle's whole control-step plan (Alg. 1 followed by the layer-adaptive
subsets of Sec. 3.4 / Alg. 2) on a hand-made case whose every intermediate result is
worked out below by hand, not by the oracle's own functions.

Case: an 8 x 8 frame of 2 x 2 patches (16 visual tokens, raster order), 3 layers.

Static set (Eq. sim, Eq. topk).  Frame t copies frame t-1, except that in patches
3, 7 and 10 frame t-1 keeps only channel 0 and frame t only channels 1 and 2: their dot
product is 0, Sim = 0 < 249/250, and every other patch is identical, Sim = 1.
    P_static = {0,1,2,4,5,6,8,9,11,12,13,14,15}            (top-k 16 keeps all 13)

Previous step's statistic A^l_avg over the 16 tokens:
    layer 1  uniform, 1/16 each                             E = ln 16
    layer 2  1/4 on tokens {0, 1, 8, 9}                     E = ln 4
    layer 3  1/2 on tokens {9, 11}                          E = ln 2
Score S = mean over the layers (Eq. ptask), times 3:
    token 9: 1/16 + 1/4 + 1/2;  token 11: 1/16 + 1/2;  tokens 0, 1, 8: 1/16 + 1/4;
    every other token: 1/16.
tau_task = 0.75: the 16 - floor(12) = 4 highest scores are task-relevant, ties to the
lower index: {9, 11, 0, 1} (8 loses the tie with 0 and 1).
    P_final = P_static minus those = {2,4,5,6,8,12,13,14,15}           (Eq. pfinal)
    reuse order (least relevant first, ties to the lower index):
        2,4,5,6,12,13,14,15 (score 1/16), then 8 (1/16 + 1/4)

Layer ratio (Eq. reuse_ratio): R^1 = 0, R^2 = (ln 16 - ln 4) / ln 16 = 1/2,
R^3 = (ln 4 - ln 2) / ln 4 = 1/2; gain 0.6: alpha = 0, 0.3, 0.6; reuse counts
floor(alpha * 9) = 0, 2, 5; so the per-layer sets are the first 0, 2 and 5 entries of the
reuse order: {}, {2, 4}, {2, 4, 5, 6, 12}  (and not {2, 4, 5, 6, 8}, the first 5 of
P_final in index order)."""
import numpy as np

from oracle import vlac_oracle as O


def hand_made_frames():
    prev = np.zeros((8, 8, 3), dtype=np.uint8)
    for y in range(8):
        for x in range(8):
            for c in range(3):
                prev[y, x, c] = 10 + 7 * y + 3 * x + c
    cur = prev.copy()
    for patch in (3, 7, 10):
        r, c = divmod(patch, 4)
        sl = (slice(2 * r, 2 * r + 2), slice(2 * c, 2 * c + 2))
        prev[sl][..., 1:] = 0
        cur[sl][..., 0] = 0
    return prev, cur


def hand_made_stats():
    a = np.zeros((3, 16), dtype=np.float32)
    a[0, :] = 1.0 / 16
    a[1, [0, 1, 8, 9]] = 0.25
    a[2, [9, 11]] = 0.5
    return a


def test_plan_step_with_statistics_hand_worked():
    prev, cur = hand_made_frames()
    p_final, order, per_layer, alpha = O.plan_step(prev, cur, 2, 249, 250, 16, hand_made_stats(), 0.75, 0.6)
    assert p_final == [2, 4, 5, 6, 8, 12, 13, 14, 15]
    assert order == [2, 4, 5, 6, 12, 13, 14, 15, 8]
    np.testing.assert_allclose(alpha, [0.0, 0.3, 0.6], atol=1e-12)
    assert per_layer == [[], [2, 4], [2, 4, 5, 6, 12]]
    # the sets are nested over depth and prefixes of the reuse order, never of P_final
    assert per_layer[2] != p_final[:5]


def test_plan_step_top_k_cuts_before_the_filter():
    """top-k 5 of 13 equally similar static patches keeps the 5 lowest indices
    {0,1,2,4,5}; the filter then removes 0 and 1 (task-relevant): P_final = {2,4,5},
    counts floor(0.3 * 3) = 0 and floor(0.6 * 3) = 1."""
    prev, cur = hand_made_frames()
    p_final, order, per_layer, alpha = O.plan_step(prev, cur, 2, 249, 250, 5, hand_made_stats(), 0.75, 0.6)
    assert p_final == [2, 4, 5] and order == [2, 4, 5]
    assert per_layer == [[], [], [2]]


def test_plan_step_layer_mask_changes_the_ranking_only():
    """Scores from layer 3 alone: tokens 9 and 11 lead, every other token ties at 0, so the
    4 relevant ones are {9, 11, 0, 1} again by the index rule, but token 8 now ties with the
    rest and takes its place by index in the reuse order; alpha uses all layers as before."""
    prev, cur = hand_made_frames()
    p_final, order, per_layer, alpha = O.plan_step(prev, cur, 2, 249, 250, 16, hand_made_stats(), 0.75, 0.6,
                                                   layer_mask=[0, 0, 1])
    assert p_final == [2, 4, 5, 6, 8, 12, 13, 14, 15]
    assert order == [2, 4, 5, 6, 8, 12, 13, 14, 15]
    np.testing.assert_allclose(alpha, [0.0, 0.3, 0.6], atol=1e-12)
    assert per_layer == [[], [2, 4], [2, 4, 5, 6, 8]]


def test_plan_step_without_statistics():
    prev, cur = hand_made_frames()
    p_final, order, per_layer, alpha = O.plan_step(prev, cur, 2, 249, 250, 16, None, 0.75, 0.6)
    assert p_final == [0, 1, 2, 4, 5, 6, 8, 9, 11, 12, 13, 14, 15] and order == p_final
    assert per_layer is None and alpha is None
