"""Generalized Advantage Estimation by its backward recursion.  TEST INFRASTRUCTURE ONLY.

Section 6 ("System optimizations", inference stage) says the product unrolls GAE's
recursion along the output length into one matrix multiply.  The definition it unrolls is
the textbook one (Schulman et al., GAE), written out here per sample in float64:

    delta_t = r_t + gamma * V_{t+1} - V_t          (V_{L+1} = 0: the episode ends at y_L)
    A_t     = delta_t + gamma * lam * A_{t+1}      (A_{L+1} = 0)
    R_t     = A_t + V_t                            (the return the Critic regresses on)

with t = 1..L over the response tokens.  The per-token reward is the usual RLHF shaping:
a KL penalty  -kl_coef * (lp_actor_t - lp_ref_t)  at every token, plus the Reward model's
scalar score added at the last token.  The paper does not print these formulas; this is
the reading the product follows too.
"""
import numpy as np


def token_rewards(lp_actor, lp_ref, reward: float, kl_coef: float) -> np.ndarray:
    r = -kl_coef * (np.asarray(lp_actor, np.float64) - np.asarray(lp_ref, np.float64))
    r[-1] += float(reward)
    return r


def gae(rewards, values, gamma: float, lam: float):
    """Backward recursion.  rewards, values: [L].  Returns (advantages [L], returns [L])."""
    r = np.asarray(rewards, np.float64)
    v = np.asarray(values, np.float64)
    L = r.shape[0]
    adv = np.zeros(L, np.float64)
    nxt_adv, nxt_v = 0.0, 0.0
    for t in range(L - 1, -1, -1):
        delta = r[t] + gamma * nxt_v - v[t]
        nxt_adv = delta + gamma * lam * nxt_adv
        adv[t] = nxt_adv
        nxt_v = v[t]
    return adv, adv + v
