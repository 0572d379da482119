"""Pins for oracle/gae.py: closed forms of the recursion and its unrolled (matrix) form."""
import numpy as np

from oracle.gae import gae, token_rewards


def test_gae_closed_forms():
    r = np.random.default_rng(0)
    L = 9
    rew, val = r.normal(size=L), r.normal(size=L)
    # lambda = 1, gamma = 1: advantage = reward-to-go minus value
    adv, ret = gae(rew, val, 1.0, 1.0)
    np.testing.assert_allclose(adv, np.cumsum(rew[::-1])[::-1] - val, atol=1e-13)
    np.testing.assert_allclose(ret, np.cumsum(rew[::-1])[::-1], atol=1e-13)
    # lambda = 0: one-step TD error, with V = 0 after the last token
    adv0, _ = gae(rew, val, 0.9, 0.0)
    np.testing.assert_allclose(adv0, rew + 0.9 * np.append(val[1:], 0.0) - val, atol=1e-14)
    # hand value, L = 2: A_2 = r2 - v2 ; A_1 = r1 + g v2 - v1 + g l A_2
    a, _ = gae([1.0, 2.0], [0.5, 0.25], 0.5, 0.5)
    assert abs(a[1] - 1.75) < 1e-15 and abs(a[0] - (1.0 + 0.125 - 0.5 + 0.25 * 1.75)) < 1e-15


def test_gae_unrolled_matrix_form():
    """Unrolling the recursion: A = U delta with U[t, s] = (gamma lam)^(s-t) for s >= t."""
    r = np.random.default_rng(1)
    L, g, lam = 33, 0.97, 0.9
    rew, val = r.normal(size=L), r.normal(size=L)
    delta = rew + g * np.append(val[1:], 0.0) - val
    t, s = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
    U = np.where(s >= t, (g * lam) ** np.clip(s - t, 0, None), 0.0)
    np.testing.assert_allclose(gae(rew, val, g, lam)[0], U @ delta, atol=1e-12)


def test_token_rewards():
    tr = token_rewards([-1.0, -2.0, -0.5], [-1.5, -1.0, -0.5], reward=3.0, kl_coef=0.1)
    np.testing.assert_allclose(tr, [-0.05, 0.1, 3.0], atol=1e-15)
