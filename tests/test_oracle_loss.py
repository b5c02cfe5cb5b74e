"""Pins of the loss oracle: the paper's normaliser algebra, closed forms, finite differences."""
import numpy as np
import pytest

from oracle import loss as L


def rand_case(T, V, cu, seed, p_mask=0.3):
    r = np.random.default_rng(seed)
    z = r.normal(0, 2.0, (T, V))
    y = r.integers(0, V, T)
    y[r.random(T) < p_mask] = -100
    return z, y, np.asarray(cu)


def test_uniform_logits_give_ln_v_and_softmax_minus_onehot():
    V = 50
    z = np.full((3, V), 0.7)
    y = np.array([4, -1, 49])
    loss, tl, dz = L.packed_ce(z, y, [0, 3], L.TOKEN_MEAN)
    assert tl[0] == pytest.approx(np.log(V), rel=1e-14) and tl[1] == 0.0
    assert loss == pytest.approx(np.log(V), rel=1e-14)
    want = np.full(V, 1.0 / V); want[4] -= 1.0
    np.testing.assert_allclose(dz[0], want / 2, rtol=1e-13)
    assert not dz[1].any()


def test_dominant_logit_closed_form():
    z = np.zeros((1, 8)); z[0, 3] = 40.0
    loss, tl, dz = L.packed_ce(z, [3], [0, 1], L.TOKEN_MEAN)
    assert tl[0] == pytest.approx(7 * np.exp(-40.0), rel=1e-6)
    loss2, tl2, _ = L.packed_ce(z, [0], [0, 1], L.TOKEN_MEAN)
    assert tl2[0] == pytest.approx(40.0 + 7 * np.exp(-40.0), rel=1e-12)


def test_papers_two_rank_example_stable_equals_global_token_mean():
    """Section 4.3: ranks {1,2} and {3,4}; with T_ave = (T1+T2+T3+T4)/4 the mean of the two rank losses
    is (loss1+loss2+loss3+loss4)/(T1+T2+T3+T4); token-mean and sample-mean give the printed forms."""
    V = 17
    lens = [5, 9, 3, 12]
    r = np.random.default_rng(3)
    zs = [r.normal(0, 1.5, (n, V)) for n in lens]
    ys = [r.integers(0, V, n) for n in lens]
    ys[1][:4] = -1; ys[3][5:7] = -1                       # prompt tokens without loss
    Ti = [int((y >= 0).sum()) for y in ys]
    li = [L.packed_ce(z, y, [0, len(y)], L.TOKEN_MEAN)[1].sum() for z, y in zip(zs, ys)]
    t_ave = sum(Ti) / 4
    def rank(a, b, mode):
        z = np.concatenate([zs[a], zs[b]]); y = np.concatenate([ys[a], ys[b]])
        return L.packed_ce(z, y, [0, lens[a], lens[a] + lens[b]], mode, t_ave)[0]
    stable = (rank(0, 1, L.STABLE) + rank(2, 3, L.STABLE)) / 2
    assert stable == pytest.approx(sum(li) / sum(Ti), rel=1e-13)
    token = (rank(0, 1, L.TOKEN_MEAN) + rank(2, 3, L.TOKEN_MEAN)) / 2
    assert token == pytest.approx(((li[0] + li[1]) / (Ti[0] + Ti[1]) + (li[2] + li[3]) / (Ti[2] + Ti[3])) / 2, rel=1e-13)
    sample = (rank(0, 1, L.SAMPLE_MEAN) + rank(2, 3, L.SAMPLE_MEAN)) / 2
    assert sample == pytest.approx(sum(l / t for l, t in zip(li, Ti)) / 4, rel=1e-13)


@pytest.mark.parametrize("mode", [L.TOKEN_MEAN, L.SAMPLE_MEAN, L.STABLE])
def test_gradient_by_central_differences(mode):
    T, V = 7, 6
    z, y, cu = rand_case(T, V, [0, 3, 7], 5)
    _, _, dz = L.packed_ce(z, y, cu, mode, 2.5)
    h = 1e-6
    for r in range(T):
        for v in range(V):
            zp = z.copy(); zp[r, v] += h
            zm = z.copy(); zm[r, v] -= h
            num = (L.packed_ce(zp, y, cu, mode, 2.5)[0] - L.packed_ce(zm, y, cu, mode, 2.5)[0]) / (2 * h)
            assert dz[r, v] == pytest.approx(num, abs=2e-9)


def test_rows_sum_to_zero_and_masked_rows_are_zero_and_samples_are_isolated():
    z, y, cu = rand_case(40, 33, [0, 10, 25, 40], 8)
    loss, tl, dz = L.packed_ce(z, y, cu, L.SAMPLE_MEAN)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-15)
    assert not dz[y < 0].any() and not tl[y < 0].any()
    z2 = z.copy(); z2[30:] += 5.0 * np.random.default_rng(1).normal(size=(10, 33))
    _, tl2, dz2 = L.packed_ce(z2, y, cu, L.SAMPLE_MEAN)
    assert np.array_equal(dz2[:25], dz[:25]) and np.array_equal(tl2[:25], tl[:25])   # sample-mean weights are per sample


def test_weights_and_a_sample_without_loss_tokens():
    y = np.array([1, -1, 2, -1, -1, 0, 0, 0])
    cu = [0, 3, 5, 8]                       # counts 2, 0, 3
    np.testing.assert_allclose(L.token_weights(y, cu, L.TOKEN_MEAN), np.where(y >= 0, 1 / 5, 0))
    w = L.token_weights(y, cu, L.SAMPLE_MEAN)
    np.testing.assert_allclose(w, [1 / 6, 0, 1 / 6, 0, 0, 1 / 9, 1 / 9, 1 / 9])
    np.testing.assert_allclose(L.token_weights(y, cu, L.STABLE, 4.0), np.where(y >= 0, 1 / 12, 0))
    with pytest.raises(ValueError):
        L.token_weights(y, cu, 7)


def test_label_at_or_above_the_vocabulary_size_is_a_token_without_loss():
    """One reading for both sides: a label outside [0, V) behaves exactly like a negative one (no loss,
    zero gradient row, not counted in T_i)."""
    rng = np.random.default_rng(9)
    V = 11
    z = rng.normal(0, 2, (8, V))
    y = np.array([1, V, 2, -1, V + 5, 0, 10, 3])
    y_neg = np.where(y >= V, -1, y)
    cu = [0, 3, 5, 8]
    for mode in (L.TOKEN_MEAN, L.SAMPLE_MEAN, L.STABLE):
        a = L.packed_ce(z, y, cu, mode, 2.5)
        b = L.packed_ce(z, y_neg, cu, mode, 2.5)
        assert a[0] == b[0] and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
        assert not a[2][1].any() and not a[2][4].any() and a[1][1] == 0.0
    np.testing.assert_allclose(L.token_weights(y, cu, L.TOKEN_MEAN, vocab=V), np.where(y_neg >= 0, 1 / 5, 0))
    np.testing.assert_allclose(L.token_weights(y, cu, L.SAMPLE_MEAN, vocab=V),
                               [1 / 6, 0, 1 / 6, 0, 0, 1 / 9, 1 / 9, 1 / 9])
