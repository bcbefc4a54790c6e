"""Ensemble OMP counter selection (Section 3.2.3, Eq. 1) pinned to what the mathematics fixes:
with tau = 1 it is plain orthogonal matching pursuit (compared with scikit-learn's), a planted
sparse model is recovered, picks are drawn in proportion to correlation strength, and the
re-fitted residual is orthogonal to every chosen column.  The paper gives no kappa, tau, ensemble
size or data for this step, so nothing here is pinned to the paper."""
import numpy as np
import pytest

from paper_2510_00932_amd import counter_selection as cs


def _problem(seed, n=60, c=25, true=(3, 11, 17), coef=(4.0, -2.5, 1.5), noise=0.01):
    rng = np.random.RandomState(seed)
    D = rng.normal(size=(n, c)) * rng.uniform(0.1, 1e6, size=c) + rng.uniform(-1e3, 1e3, size=c)
    Dn, _, _ = cs.standardise(D, np.zeros(n))
    t = sum(w * Dn[:, j] for j, w in zip(true, coef)) + noise * rng.normal(size=n) + 123.0
    return D, t


def test_standardise():
    D, t = _problem(0)
    D[:, 5] = 7.0                                       # a constant counter
    Dn, tn, keep = cs.standardise(D, t)
    assert 5 not in keep and len(keep) == D.shape[1] - 1
    assert np.allclose(Dn.sum(axis=0), 0, atol=1e-9) and np.allclose((Dn * Dn).sum(axis=0), 1)
    assert abs(tn.sum()) < 1e-9


def test_tau_one_is_plain_omp_and_matches_scikit_learn():
    from sklearn.linear_model import OrthogonalMatchingPursuit
    for seed in range(5):
        D, t = _problem(seed, noise=0.05)
        Dn, tn, keep = cs.standardise(D, t)
        support, weights = cs.pursuit(Dn, tn, 4, 1, np.zeros(4))
        ref = OrthogonalMatchingPursuit(n_nonzero_coefs=4, fit_intercept=False).fit(Dn, tn)
        assert sorted(support) == sorted(np.nonzero(ref.coef_)[0].tolist())
        assert np.allclose(weights, ref.coef_[support], rtol=1e-8, atol=1e-10)


def test_planted_model_is_recovered_and_ranked():
    D, t = _problem(7)
    draws = np.random.RandomState(1).random_sample((100, 3))
    res = cs.ensemble_omp(D, t, kappa=3, tau=2, draws=draws)
    names = ["c%d" % j for j in range(D.shape[1])]
    top = cs.top_k(res, names, 3)
    assert [n for n, _ in top] == ["c3", "c11", "c17"]          # ordered by |weight|: 4.0, 2.5, 1.5
    assert top[0][1] > top[1][1] > top[2][1]


def test_residual_is_orthogonal_to_the_support():
    D, t = _problem(3, noise=0.5)
    Dn, tn, _ = cs.standardise(D, t)
    support, weights = cs.pursuit(Dn, tn, 5, 3, np.array([0.9, 0.1, 0.5, 0.7, 0.3]))
    r = tn - Dn[:, support] @ weights
    assert len(set(support)) == 5
    assert np.allclose(Dn[:, support].T @ r, 0, atol=1e-9)


def test_picks_are_proportional_to_correlation_strength():
    # two orthogonal counters with correlation strengths 3 : 1 and an irrelevant third; tau = 2, one step
    n = 40
    rng = np.random.RandomState(0)
    q, _ = np.linalg.qr(rng.normal(size=(n, 4)))
    q = q - q.mean(axis=0)
    q, _ = np.linalg.qr(q)
    D = q[:, :3]
    t = 3.0 * D[:, 0] + 1.0 * D[:, 1]
    draws = (np.arange(4000) + 0.5)[:, None] / 4000.0
    res = cs.ensemble_omp(D, t, kappa=1, tau=2, draws=draws)
    first = np.array([m[0][0] for m in res["members"]])
    assert set(first.tolist()) == {0, 1}
    assert abs((first == 0).mean() - 0.75) < 0.01


def test_full_support_is_least_squares():
    D, t = _problem(9, n=30, c=6, true=(0, 1, 2))
    Dn, tn, _ = cs.standardise(D, t)
    support, weights = cs.pursuit(Dn, tn, 6, 1, np.zeros(6))
    ls, *_ = np.linalg.lstsq(Dn, tn, rcond=None)
    full = np.zeros(6)
    full[support] = weights
    assert np.allclose(full, ls, atol=1e-8)


def test_draws_make_runs_reproducible():
    D, t = _problem(4, noise=0.3)
    draws = np.random.RandomState(5).random_sample((20, 4))
    a = cs.ensemble_omp(D, t, 4, 3, draws)
    b = cs.ensemble_omp(D, t, 4, 3, draws.copy())
    assert np.array_equal(a["importance"], b["importance"])
