"""Pins of the float64 oracle to things other than itself: hand-worked values of Eq. (2)/(4)/(5),
closed forms, invariants, brute-force enumeration in pure Python, central finite differences of
an independently written objective, and library routines (scipy log_softmax, torch autograd
cross-entropy).  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import rapid_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers (independent of oracle)
def _py_logsoftmax_at(h, W, y):
    """log softmax(h W)[y] with explicit python loops."""
    d, V = len(W), len(W[0])
    z = [sum(h[k] * W[k][v] for k in range(d)) for v in range(V)]
    return z[y] - math.log(sum(math.exp(zz) for zz in z))


def _py_surrogate(H, W, tok, mask, logp_b, adv_fixed):
    """-(1/N) sum_n A_n * prod_t pi(y_t)/mu(y_t): the objective whose gradient Eq. (3) gives,
    with advantages held fixed, written with explicit loops."""
    N, T = len(tok), len(tok[0])
    tot = 0.0
    for n in range(N):
        ratio = 1.0
        for t in range(T):
            if mask[n][t]:
                ratio *= math.exp(_py_logsoftmax_at(H[n][t], W, tok[n][t])) / math.exp(logp_b[n][t])
        tot += adv_fixed[n] * ratio
    return -tot / N


def _tiny(seed=0, N=4, T=3, d=3, V=5, G=2):
    rng = np.random.default_rng(seed)
    H = rng.normal(size=(N, T, d))
    W = rng.normal(size=(d, V)) * 0.5
    W_old = W + rng.normal(size=(d, V)) * 0.1
    tok = rng.integers(0, V, size=(N, T))
    lengths = rng.integers(1, T + 1, size=N)
    mask = (np.arange(T)[None, :] < lengths[:, None]).astype(np.uint8)
    R = rng.random(N)
    gid = np.arange(N) // G
    logp_b, _ = orc.logprob(H, W_old, tok, mask)
    return H, W, W_old, tok, mask, R, gid, logp_b


# ---------------------------------------------------------------- group advantage (Eq. 2, 4, 5)
def _golden():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "eq5_hand_example.txt"))
            if l.strip() and not l.startswith("#")]
    return np.array(rows, dtype=np.float64)


def test_eq5_hand_example():
    g = _golden()
    rho, R = g[:, 0], g[:, 1]
    gid = np.zeros(4, np.int64)
    s = np.log(rho)
    assert np.allclose(orc.group_advantage(R, gid, 1, s=s, eta=2.0)["adv"], g[:, 2], atol=1e-15)
    assert np.allclose(orc.group_advantage(R, gid, 1, s=None)["adv"], g[:, 3], atol=1e-15)
    assert np.allclose(orc.group_advantage(R, gid, 1, s=s, eta=math.inf)["adv"], g[:, 4], atol=1e-15)
    assert np.allclose(orc.group_advantage(R, gid, 1, s=s, eta=2.0, baseline_mode=1)["adv"],
                       g[:, 5], atol=1e-15)
    assert np.allclose(orc.group_advantage(R, gid, 1, s=s, eta=2.0, baseline_mode=2)["adv"],
                       g[:, 6], atol=1e-15)        # leave-one-out over N_k - 1 = 3 (hand values 5/6, -5/6, -5/6, 1/3)
    w = orc.clipped_weight(s, 2.0)
    assert np.allclose(w, [2.0, 1.0, 1.0, 0.5], atol=1e-15)


def test_clip_is_min_not_max():
    # s = ln 4, eta = 2 -> w = 2; s = ln 0.5 -> w = 0.5 (no lower clip)
    w = orc.clipped_weight(np.log([4.0, 0.5, 2.0, 1.0]), 2.0)
    assert np.allclose(w, [2.0, 0.5, 2.0, 1.0])
    assert orc.clipped_weight(np.array([0.0]), 2.0)[0] == 1.0


def test_group_adv_sums():
    rng = np.random.default_rng(1)
    N, K = 37, 5
    R = rng.random(N)
    gid = rng.integers(0, K, size=N)          # ragged, non-contiguous groups
    out = orc.group_advantage(R, gid, K, s=None)
    for k in range(K):                          # Eq. (2): zero sum per group
        assert abs(out["adv"][gid == k].sum()) < 1e-12
        assert out["group_size"][k] == (gid == k).sum()
        if (gid == k).any():
            assert abs(out["group_mean"][k] - R[gid == k].mean()) < 1e-14
            assert abs(out["group_std"][k] - R[gid == k].std()) < 1e-14
    s = rng.normal(size=N)
    out = orc.group_advantage(R, gid, K, s=s, eta=2.0)
    w = np.minimum(np.exp(s), 2.0)
    for k in range(K):                          # closed form from Eq. (5): sum A = sum (1-w) R
        m = gid == k
        assert abs(out["adv"][m].sum() - ((1 - w[m]) * R[m]).sum()) < 1e-12
    big = orc.group_advantage(R, gid, K, s=s, eta=1e300)
    inf = orc.group_advantage(R, gid, K, s=s, eta=math.inf)
    assert np.array_equal(big["adv"], inf["adv"])   # eta -> inf: Eq. (5) == Eq. (4)
    # brute force per element
    for n in range(N):
        b = np.mean([min(math.exp(s[j]), 2.0) * R[j] for j in range(N) if gid[j] == gid[n]])
        assert abs(out["adv"][n] - (R[n] - b)) < 1e-13


def test_leave_one_out_over_the_others():
    """baseline_mode 2 (Sec. 3.4, leave-one-out paragraph, normalised by N_k - 1): the baseline of
    sample n is the clipped-weight mean reward of the OTHER members of its group.  Pinned by explicit
    loops, by its independence of sample n's own reward and ratio (what makes the estimator unbiased),
    by the relation to the sum printed with 1/N_k, and by the degenerate group sizes."""
    rng = np.random.default_rng(8)
    N, K = 41, 6
    R = rng.random(N)
    gid = rng.integers(0, K - 1, size=N)         # ragged, shuffled; group K-1 empty
    gid[7] = K - 1                                # ... except for one lonely member
    s = rng.normal(size=N)
    eta = 2.0
    out = orc.group_advantage(R, gid, K, s=s, eta=eta, baseline_mode=2)
    as_printed = orc.group_advantage(R, gid, K, s=s, eta=eta, baseline_mode=1)
    for n in range(N):
        others = [j for j in range(N) if gid[j] == gid[n] and j != n]
        b = sum(min(math.exp(s[j]), eta) * R[j] for j in others) / len(others) if others else 0.0
        assert abs(out["adv"][n] - (R[n] - b)) < 1e-13
        # the same leave-one-out sum, divided by N_k as printed: b' = b (N_k - 1) / N_k
        nk = len(others) + 1
        assert abs((R[n] - as_printed["adv"][n]) * nk - b * (nk - 1)) < 1e-12
    assert out["adv"][7] == R[7]                  # a group of one: nobody else, baseline 0
    # sample n's own reward and ratio do not enter its baseline (they do enter Eq. (5)'s)
    for n in (0, 3, 19):
        R2, s2 = R.copy(), s.copy()
        R2[n] += 0.7
        s2[n] -= 1.3
        moved = orc.group_advantage(R2, gid, K, s=s2, eta=eta, baseline_mode=2)
        assert abs((R2[n] - moved["adv"][n]) - (R[n] - out["adv"][n])) < 1e-14
        eq5, eq5_moved = (orc.group_advantage(r, gid, K, s=ss, eta=eta)["adv"] for r, ss in ((R, s), (R2, s2)))
        assert abs((R2[n] - eq5_moved[n]) - (R[n] - eq5[n])) > 1e-3
    # on-policy, equal rewards in a group: every other member has the same reward, so A = 0
    flat = orc.group_advantage(np.full(N, 0.25), gid, K, s=None, baseline_mode=2)["adv"]
    assert np.allclose(np.delete(flat, 7), 0.0, atol=1e-15) and flat[7] == 0.25
    # exhaustive expectation on a two-armed bandit sampled on-policy: with the baseline of the others,
    # E[A_n grad log pi(y_n)] equals the exact policy gradient (it does not with Eq. (2)'s own-sample mean)
    p, r = np.array([0.3, 0.7]), np.array([1.0, 0.2])
    exact = p * (r - (p * r).sum())               # dJ/dlogit_a for a softmax policy
    est2, est0 = np.zeros(2), np.zeros(2)
    G = 3
    for ys in itertools.product(range(2), repeat=G):
        pr = np.prod(p[list(ys)])
        for mode, acc in ((2, est2), (0, est0)):
            A = orc.group_advantage(r[list(ys)], np.zeros(G, int), 1, s=None, baseline_mode=mode)["adv"]
            for n, y in enumerate(ys):
                acc += pr * A[n] * ((np.arange(2) == y) - p) / G
    assert np.allclose(est2, exact, atol=1e-14)
    assert np.allclose(est0, exact * (G - 1) / G, atol=1e-14)       # Eq. (2): biased by the factor (G-1)/G


def test_zero_variance_groups():
    R = np.array([0, 0, 0, 0, 1, 1, 1, 1], float)
    gid = np.array([0, 0, 0, 0, 1, 1, 1, 1])
    s = np.array([0.3, -1.0, 2.0, 0.0, 0.3, -1.0, 2.0, 0.0])
    out = orc.group_advantage(R, gid, 2, s=s, eta=2.0)
    assert np.all(out["adv"][:4] == 0.0)             # all-0 group: A = 0 whatever the weights
    w = np.minimum(np.exp(s[4:]), 2.0)
    assert np.allclose(out["adv"][4:], 1.0 - w.mean())  # all-1 group: A = 1 - mean(w)
    on = orc.group_advantage(R, gid, 2, s=None)
    assert np.all(on["adv"] == 0.0) and np.all(on["group_std"] == 0.0)
    empty = orc.group_advantage(R, gid, 3, s=None)
    assert empty["group_size"][2] == 0 and empty["group_mean"][2] == 0 and empty["group_std"][2] == 0


def test_all_zero_reward_group_carries_no_gradient():
    """What lets an implementation leave such generations out of the backward: if every reward of a group is 0,
    Eq. (5)'s weighted baseline is a mean of zeros, so A_n = 0 for its members whatever their ratios are, in
    every baseline mode, with either outer weight and either ratio level; their rows of dHidden are exact zeros
    and dW is what the other groups alone give.  The same holds for the baselines' normalised advantage when
    there is no KL term; with one, every token carries gradient."""
    H, W, W_old, tok, mask, R, gid, logp_b = _tiny(seed=5, N=6, T=4, d=3, V=5, G=2)
    R = R.copy()
    R[gid == 1] = 0.0
    rest = gid != 1
    for kw in (dict(), dict(baseline_mode=1), dict(baseline_mode=2), dict(coef_mode=1, eta=1.1), dict(ratio_level=1),
               dict(normalized_grads=True)):
        out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 3, **kw)
        assert np.all(out["adv"][gid == 1] == 0.0) and np.all(out["dH"][gid == 1] == 0.0), kw
        assert np.abs(out["dH"][rest]).max() > 0
        # the same batch without that group's generations: their share of dW is nothing (1/N stays that of the
        # full batch: loss_scale carries it)
        sub = orc.iw_pg_loss_fwd_bwd(H[rest], W, tok[rest], mask[rest], logp_b[rest], R[rest], np.array([0, 0, 1, 1]), 2,
                                     loss_scale=rest.sum() / len(R), **kw)
        scale = np.exp(sub["grad_log_scale"] - out["grad_log_scale"]) if kw.get("normalized_grads") else 1.0
        assert np.allclose(out["dW"], sub["dW"] * scale, rtol=1e-12, atol=1e-15), kw
        assert np.isclose(out["loss"], sub["loss"] * scale, rtol=1e-12)
    logp_ref, _ = orc.logprob(H, W + 0.05, tok, mask)
    no_kl = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, logp_ref, R, gid, 3, eps_low=0.2, eps_high=0.28, kl_beta=0.0,
                                        norm_mode=1)
    assert np.all(no_kl["adv"][gid == 1] == 0.0) and np.all(no_kl["dH"][gid == 1] == 0.0)
    kl = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, logp_ref, R, gid, 3, eps_low=0.2, eps_high=0.2, kl_beta=0.04,
                                     norm_mode=0)
    assert np.all(kl["adv"][gid == 1] == 0.0) and np.abs(kl["dH"][gid == 1]).max() > 0


# ---------------------------------------------------------------- log-probabilities
def test_logprob_closed_forms():
    rng = np.random.default_rng(2)
    N, T, d, V = 3, 5, 7, 11
    H = rng.normal(size=(N, T, d))
    tok = rng.integers(0, V, size=(N, T))
    mask = np.ones((N, T), np.uint8)
    mask[1, 3:] = 0
    lp, lse = orc.logprob(H, np.zeros((d, V)), tok, mask)
    assert np.allclose(lp[mask != 0], -math.log(V), atol=1e-15)   # W = 0 -> uniform
    assert np.allclose(lse[mask != 0], math.log(V), atol=1e-15)
    assert np.all(lp[mask == 0] == 0)
    W = rng.normal(size=(d, V))
    lp1, _ = orc.logprob(H, W, tok, mask)
    lp2, _ = orc.logprob(H, W + rng.normal(size=(d, 1)), tok, mask)  # same vector added to every column
    assert np.allclose(lp1, lp2, atol=1e-12)
    ref = scipy.special.log_softmax(H @ W, axis=-1)                  # library third leg
    pick = np.take_along_axis(ref, tok[..., None], axis=-1)[..., 0]
    assert np.allclose(lp1[mask != 0], pick[mask != 0], atol=1e-13)
    # probabilities over every token id sum to one
    tot = np.zeros((N, T))
    for v in range(V):
        lpv, _ = orc.logprob(H, W, np.full((N, T), v), mask)
        tot += np.exp(lpv) * (mask != 0)
    assert np.allclose(tot[mask != 0], 1.0, atol=1e-13)
    # temperature: logits divided by tau
    lpt, _ = orc.logprob(H, W, tok, mask, temperature=0.7)
    reft = scipy.special.log_softmax(H @ W / 0.7, axis=-1)
    pickt = np.take_along_axis(reft, tok[..., None], axis=-1)[..., 0]
    assert np.allclose(lpt[mask != 0], pickt[mask != 0], atol=1e-13)


def test_logprob_brute_force_python():
    H, W, _, tok, mask, *_ = _tiny(3)
    lp, _ = orc.logprob(H, W, tok, mask)
    for n in range(H.shape[0]):
        for t in range(H.shape[1]):
            if mask[n, t]:
                ref = _py_logsoftmax_at(H[n, t].tolist(), W.tolist(), int(tok[n, t]))
                assert abs(lp[n, t] - ref) < 1e-13
            else:
                assert lp[n, t] == 0.0


def test_token_out_of_range_raises():
    H, W, _, tok, mask, *_ = _tiny(3)
    tok = tok.copy()
    tok[0, 0] = W.shape[1]
    with pytest.raises(ValueError):
        orc.logprob(H, W, tok, mask)


# ---------------------------------------------------------------- ratio direction and on-policy case
def test_expected_ratio_is_one_exhaustive():
    """E_{y~mu}[pi(y)/mu(y)] = 1 by enumerating every generation of a tiny vocabulary: pins the
    direction of the ratio (pi/mu, not mu/pi) and the accumulation over tokens."""
    rng = np.random.default_rng(4)
    T, d, V = 3, 4, 3
    H = rng.normal(size=(1, T, d))
    W = rng.normal(size=(d, V))
    W_old = W + 0.5 * rng.normal(size=(d, V))
    mask = np.ones((1, T), np.uint8)
    tot, tot_inv = 0.0, 0.0
    for y in itertools.product(range(V), repeat=T):
        tok = np.array([y])
        lp_mu, _ = orc.logprob(H, W_old, tok, mask)
        lp_pi, _ = orc.logprob(H, W, tok, mask)
        s = orc.seq_logratio(lp_pi, lp_mu, mask)[0]
        mu = math.exp(lp_mu.sum())
        tot += mu * math.exp(s)
        tot_inv += mu * math.exp(-s)
    assert abs(tot - 1.0) < 1e-12
    assert abs(tot_inv - 1.0) > 1e-2     # the wrong direction does not integrate to one


def test_on_policy_reduction():
    """Equal policies: every weight exactly 1, Eq. (5) == Eq. (2), loss exactly 0 for complete
    groups, gradient equals the on-policy group-advantage policy gradient (Eq. (1) with Eq. (2))."""
    H, W, _, tok, mask, R, gid, _ = _tiny(5, N=6, G=3)
    lp, _ = orc.logprob(H, W, tok, mask)
    out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, lp, R, gid, 2)
    assert np.all(out["seq_logratio"] == 0.0)
    assert np.all(out["weight"] == 1.0)
    assert np.array_equal(out["adv"], orc.group_advantage(R, gid, 2, s=None)["adv"])
    assert abs(out["loss"]) < 1e-15
    assert out["n_clipped"] == 0 and out["mean_log_w"] == 0.0
    # on-policy gradient: d/dtheta of -(1/N) sum_n A_n log pi(y_n), by central differences
    A = out["adv"]

    def obj(Hx, Wx):
        tot = 0.0
        for n in range(6):
            for t in range(H.shape[1]):
                if mask[n, t]:
                    tot += A[n] * _py_logsoftmax_at(Hx[n, t].tolist(), Wx.tolist(), int(tok[n, t]))
        return -tot / 6

    eps = 1e-6
    for (i, j) in [(0, 0), (2, 3), (1, 4)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[i, j] += eps
        Wm[i, j] -= eps
        fd = (obj(H, Wp) - obj(H, Wm)) / (2 * eps)
        assert abs(out["dW"][i, j] - fd) < 1e-8


# ---------------------------------------------------------------- gradients
@pytest.mark.parametrize("coef_mode", [0])
def test_finite_differences_of_surrogate(coef_mode):
    H, W, _, tok, mask, R, gid, logp_b = _tiny(6)
    out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, eta=2.0, coef_mode=coef_mode)
    A = out["adv"].tolist()
    f0 = _py_surrogate(H.tolist(), W.tolist(), tok.tolist(), mask.tolist(), logp_b.tolist(), A)
    assert abs(f0 - out["loss"]) < 1e-13
    eps = 1e-6
    for idx in itertools.product(range(W.shape[0]), range(W.shape[1])):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        fd = (_py_surrogate(H.tolist(), Wp.tolist(), tok.tolist(), mask.tolist(), logp_b.tolist(), A)
              - _py_surrogate(H.tolist(), Wm.tolist(), tok.tolist(), mask.tolist(), logp_b.tolist(), A)) / (2 * eps)
        assert abs(out["dW"][idx] - fd) < 1e-8, idx
    for idx in itertools.product(range(H.shape[0]), range(H.shape[1]), range(H.shape[2])):
        Hp, Hm = H.copy(), H.copy()
        Hp[idx] += eps
        Hm[idx] -= eps
        fd = (_py_surrogate(Hp.tolist(), W.tolist(), tok.tolist(), mask.tolist(), logp_b.tolist(), A)
              - _py_surrogate(Hm.tolist(), W.tolist(), tok.tolist(), mask.tolist(), logp_b.tolist(), A)) / (2 * eps)
        assert abs(out["dH"][idx] - fd) < 1e-8, idx
        if not mask[idx[0], idx[1]]:
            assert out["dH"][idx] == 0.0


def test_coef_mode1_is_linear_surrogate():
    """coef_mode 1: the clipped weight is a constant coefficient on log pi; its gradient is the
    gradient of sum_n g_n sum_t logp_{n,t}, checked by finite differences."""
    H, W, _, tok, mask, R, gid, logp_b = _tiny(7)
    logp_b = logp_b - 0.4 * mask      # push ratios up so that some clip
    out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, eta=2.0, coef_mode=1)
    assert out["n_clipped"] > 0
    w = np.minimum(np.exp(out["seq_logratio"]), 2.0)
    assert np.allclose(out["g"], -w * out["adv"] / 4, atol=1e-15)
    g = out["g"]

    def obj(Wx):
        tot = 0.0
        for n in range(4):
            for t in range(H.shape[1]):
                if mask[n, t]:
                    tot += g[n] * _py_logsoftmax_at(H[n, t].tolist(), Wx.tolist(), int(tok[n, t]))
        return tot

    eps = 1e-6
    for idx in [(0, 0), (1, 2), (2, 4)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        assert abs(out["dW"][idx] - (obj(Wp) - obj(Wm)) / (2 * eps)) < 1e-8


def test_cross_entropy_special_case_torch_autograd():
    """Constant coefficient g = -1/M: the backward is the gradient of the mean token cross-entropy
    of a linear layer, a library routine (torch autograd, float64)."""
    rng = np.random.default_rng(8)
    N, T, d, V = 3, 6, 5, 9
    H = rng.normal(size=(N, T, d))
    W = rng.normal(size=(d, V))
    tok = rng.integers(0, V, size=(N, T))
    mask = np.ones((N, T), np.uint8)
    mask[0, 4:] = 0
    mask[2, 1:] = 0
    M = int(mask.sum())
    dH, dW = orc.backward(H, W, tok, mask, np.full(N, -1.0 / M))
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    logits = (Ht @ Wt)[torch.tensor(mask != 0)]
    loss = torch.nn.functional.cross_entropy(logits, torch.tensor(tok[mask != 0]), reduction="mean")
    loss.backward()
    assert np.allclose(dH, Ht.grad.numpy(), atol=1e-14)
    assert np.allclose(dW, Wt.grad.numpy(), atol=1e-14)
    # softmax identity: every row of dW (over the vocabulary) sums to zero
    assert np.allclose(dW.sum(axis=1), 0.0, atol=1e-14)
    # temperature scales logits: compare with autograd again
    dHt, dWt = orc.backward(H, W, tok, mask, np.full(N, -1.0 / M), temperature=0.5)
    Ht2 = torch.tensor(H, requires_grad=True)
    Wt2 = torch.tensor(W, requires_grad=True)
    logits = ((Ht2 @ Wt2) / 0.5)[torch.tensor(mask != 0)]
    torch.nn.functional.cross_entropy(logits, torch.tensor(tok[mask != 0]), reduction="mean").backward()
    assert np.allclose(dHt, Ht2.grad.numpy(), atol=1e-13)
    assert np.allclose(dWt, Wt2.grad.numpy(), atol=1e-13)


def test_importance_weighted_gradient_is_unbiased_exhaustive():
    """Eq. (3) with a known advantage: sum_y mu(y) [pi(y)/mu(y)] grad log pi(y) R(y) equals the
    gradient of J = sum_y pi(y) R(y), by enumeration of every generation and finite differences of
    a python-loop J."""
    rng = np.random.default_rng(9)
    T, d, V = 2, 3, 3
    H = rng.normal(size=(1, T, d))
    W = rng.normal(size=(d, V))
    W_old = W + 0.3 * rng.normal(size=(d, V))
    mask = np.ones((1, T), np.uint8)
    seqs = list(itertools.product(range(V), repeat=T))
    Rtab = {y: rng.random() for y in seqs}

    def J(Wx):
        tot = 0.0
        for y in seqs:
            lp = sum(_py_logsoftmax_at(H[0, t].tolist(), Wx.tolist(), y[t]) for t in range(T))
            tot += math.exp(lp) * Rtab[y]
        return tot

    acc = np.zeros_like(W)
    for y in seqs:
        tok = np.array([y])
        lp_mu, _ = orc.logprob(H, W_old, tok, mask)
        lp_pi, _ = orc.logprob(H, W, tok, mask)
        rho = math.exp(orc.seq_logratio(lp_pi, lp_mu, mask)[0])
        # descent coefficient -rho R (N = 1), weighted by the sampling probability mu(y)
        _, dW = orc.backward(H, W, tok, mask, np.array([-rho * Rtab[y] * math.exp(lp_mu.sum())]))
        acc += dW
    eps = 1e-6
    for idx in itertools.product(range(d), range(V)):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        assert abs(-acc[idx] - (J(Wp) - J(Wm)) / (2 * eps)) < 1e-8


# ---------------------------------------------------------------- scaling, diagnostics, bookkeeping
def test_normalized_grads_and_underflow():
    H, W, _, tok, mask, R, gid, logp_b = _tiny(10)
    a = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2)
    b = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, normalized_grads=True)
    lam = b["grad_log_scale"]
    assert abs(np.abs(b["g"]).max() - 1.0) < 1e-12
    assert np.allclose(b["dW"] * math.exp(lam), a["dW"], rtol=1e-12, atol=0)
    assert abs(b["loss"] * math.exp(lam) - a["loss"]) < 1e-14
    # ratios that underflow float64: normalised outputs stay finite and O(1)
    c = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b + 900.0 * mask, R, gid, 2, normalized_grads=True)
    assert np.isfinite(c["dW"]).all() and abs(np.abs(c["g"]).max() - 1.0) < 1e-12
    assert c["grad_log_scale"] < -800
    # loss_scale is linear
    d2 = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, loss_scale=0.25)
    assert np.allclose(d2["dW"], 0.25 * a["dW"], rtol=1e-12) and abs(d2["loss"] - 0.25 * a["loss"]) < 1e-15


def test_diagnostics_and_empty_sequence():
    H, W, _, tok, mask, R, gid, logp_b = _tiny(11)
    mask = mask.copy()
    mask[1, :] = 0                        # a generation with no valid token
    logp_b = logp_b * mask
    out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b - 0.5 * mask, R, gid, 2, eta=2.0)
    s = out["seq_logratio"]
    assert s[1] == 0.0 and out["weight"][1] == 1.0
    assert np.all(out["dH"][1] == 0.0)
    assert out["n_tokens"] == int(mask.sum())
    assert out["n_clipped"] == int((np.exp(s) > 2.0).sum())
    lw = np.log(np.minimum(np.exp(s), 2.0))
    assert abs(out["mean_log_w"] - lw.mean()) < 1e-14
    assert abs(out["mean_abs_log_w"] - np.abs(lw).mean()) < 1e-14
    # loss recomputed from rho and A
    assert abs(out["loss"] + (np.exp(s) * out["adv"]).mean()) < 1e-14

# ---------------------------------------------------------------- token-level outer weight (ratio_level 1)
def _py_token_surrogate(H, W, tok, mask, logp_b, adv_fixed):
    """-(1/N) sum_n A_n sum_t pi(y_t)/mu(y_t), advantages held fixed, explicit loops."""
    N, T = len(tok), len(tok[0])
    tot = 0.0
    for n in range(N):
        for t in range(T):
            if mask[n][t]:
                tot += adv_fixed[n] * math.exp(_py_logsoftmax_at(H[n][t], W, tok[n][t]) - logp_b[n][t])
    return -tot / N


def test_token_level_reduces_to_generation_level_for_one_token_generations():
    """A generation of one token has one ratio: both levels are the same estimator, in every mode."""
    H, W, _, tok, mask, R, gid, logp_b = _tiny(11, N=6, T=1, G=3)
    logp_b = logp_b - 0.5 * mask
    for kw in (dict(), dict(coef_mode=1), dict(normalized_grads=True), dict(baseline_mode=2, loss_scale=0.3)):
        a = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, ratio_level=0, **kw)
        b = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, ratio_level=1, **kw)
        assert abs(a["loss"] - b["loss"]) < 1e-15 and abs(a["grad_log_scale"] - b["grad_log_scale"]) < 1e-15
        assert np.allclose(a["g"], b["g"][:, 0], atol=1e-16)
        assert np.allclose(a["dH"], b["dH"], atol=1e-16) and np.allclose(a["dW"], b["dW"], atol=1e-16)


def test_token_level_on_policy():
    """pi = mu: every token ratio is exactly 1, so each token carries its generation's coefficient
    -A_n/N (the on-policy gradient of Eq. (1) with Eq. (2)) and the loss counts it once per token."""
    H, W, _, tok, mask, R, gid, _ = _tiny(12, N=4, T=5)
    logp_cur, _ = orc.logprob(H, W, tok, mask)
    a = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_cur, R, gid, 2, ratio_level=0)
    b = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_cur, R, gid, 2, ratio_level=1)
    assert np.array_equal(b["g"], a["g"][:, None] * (mask != 0))
    assert abs(b["loss"] - float((a["g"] * mask.sum(1)).sum())) < 1e-15
    assert np.allclose(a["dH"], b["dH"], atol=1e-16) and np.allclose(a["dW"], b["dW"], atol=1e-16)


def test_token_level_finite_differences():
    """coef_mode 0: the gradients are those of -(1/N) sum_n A_n sum_t rho_{n,t} with A fixed, an
    objective written independently with python loops; every element of dW and dH."""
    H, W, _, tok, mask, R, gid, logp_b = _tiny(13)
    out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, ratio_level=1)
    A = out["adv"].tolist()
    args = (tok.tolist(), mask.tolist(), logp_b.tolist(), A)
    assert abs(_py_token_surrogate(H.tolist(), W.tolist(), *args) - out["loss"]) < 1e-13
    eps = 1e-6
    for idx in itertools.product(range(W.shape[0]), range(W.shape[1])):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        fd = (_py_token_surrogate(H.tolist(), Wp.tolist(), *args) - _py_token_surrogate(H.tolist(), Wm.tolist(), *args)) / (2 * eps)
        assert abs(out["dW"][idx] - fd) < 1e-8, idx
    for idx in itertools.product(range(H.shape[0]), range(H.shape[1]), range(H.shape[2])):
        Hp, Hm = H.copy(), H.copy()
        Hp[idx] += eps
        Hm[idx] -= eps
        fd = (_py_token_surrogate(Hp.tolist(), W.tolist(), *args) - _py_token_surrogate(Hm.tolist(), W.tolist(), *args)) / (2 * eps)
        assert abs(out["dH"][idx] - fd) < 1e-8, idx


def test_token_level_clip_and_normalisation():
    """coef_mode 1 clips each token's ratio at eta (hand values), and normalized_grads rescales by
    the largest |g_{n,t}| without changing anything else."""
    mask = np.array([[1, 1, 1], [1, 1, 0]], np.uint8)
    D = np.log(np.array([[4.0, 0.5, 1.0], [3.0, 0.25, 7.0]])) * mask
    adv = np.array([0.5, -1.0])
    g, loss, lam = orc.token_coefficients(D, mask, adv, eta=2.0, coef_mode=1)
    assert np.allclose(g, [[-0.5, -0.125, -0.25], [1.0, 0.125, 0.0]], atol=1e-15) and lam == 0.0
    assert abs(loss - 0.25) < 1e-15
    g0, loss0, _ = orc.token_coefficients(D, mask, adv, eta=2.0, coef_mode=0)
    assert np.allclose(g0, [[-1.0, -0.125, -0.25], [1.5, 0.125, 0.0]], atol=1e-15)
    gn, lossn, lamn = orc.token_coefficients(D, mask, adv, eta=2.0, coef_mode=0, normalized=True)
    assert abs(lamn - math.log(1.5)) < 1e-15 and np.allclose(gn * 1.5, g0, atol=1e-15)
    assert abs(lossn * 1.5 - loss0) < 1e-15 and abs(np.abs(gn).max() - 1.0) < 1e-15
    # a planted mistake (ratio of the whole generation in place of the token's) fails the hand values
    wrong = -(np.exp(D.sum(1))[:, None] * mask) * adv[:, None] / 2
    assert not np.allclose(wrong, g0)


# ---------------------------------------------------------------- RMSNorm on the way in
def test_round_to_bf16_matches_library():
    """One rounding, to nearest, ties to even.  On float32-representable inputs that is torch's
    float32 -> bfloat16 conversion (library leg); next to a bfloat16 midpoint, where a detour through
    float32 would round twice, the values are worked out by hand."""
    rng = np.random.default_rng(21)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-6, 6, size=4000),
                        [0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38, 1e-39, -3e-41]])   # ties: to even
    x = x.astype(np.float32).astype(np.float64)
    ref = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).double().numpy()
    assert np.array_equal(orc.round_to_bf16(x), ref)
    assert orc.round_to_bf16(np.array([1.00390625]))[0] == 1.0 and orc.round_to_bf16(np.array([1.01171875]))[0] == 1.015625
    # bfloat16 neighbours of 1 are 1 and 1 + 2^-7; their midpoint is 1 + 2^-8.  A value 2^-30 above the
    # midpoint rounds up, 2^-30 below rounds down; float32 (spacing 2^-23) would first move both ONTO
    # the midpoint and the tie would then go to the even neighbour 1.0 in both cases.
    up, down = 1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -8 - 2.0 ** -30
    assert orc.round_to_bf16(np.array([up, down, -up, -down])).tolist() == [1.0 + 2.0 ** -7, 1.0, -(1.0 + 2.0 ** -7), -1.0]
    # odd neighbour below: midpoint of 1 + 2^-7 (odd) and 1 + 2^-6 (even) is 1 + 3 * 2^-8
    assert orc.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8 - 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    assert orc.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6                      # exact tie: to even
    # carry into the exponent, overflow, shape kept
    assert orc.round_to_bf16(np.array([2.0 - 2.0 ** -9]))[0] == 2.0
    assert np.isinf(orc.round_to_bf16(np.array([3.4e38]))[0]) and orc.round_to_bf16(np.zeros((2, 3))).shape == (2, 3)


def test_rmsnorm_forward_backward_against_torch_autograd():
    rng = np.random.default_rng(22)
    x = rng.normal(size=(3, 4, 7)) * 2.0
    wgt = rng.normal(size=7)
    dh = rng.normal(size=(3, 4, 7))
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(wgt, requires_grad=True)
    ht = torch.nn.functional.rms_norm(xt, (7,), wt, eps=1e-5)
    (ht * torch.tensor(dh)).sum().backward()
    assert np.allclose(orc.rmsnorm(x, wgt, 1e-5), ht.detach().numpy(), atol=1e-13)
    dx, dwt = orc.rmsnorm_backward(x, wgt, 1e-5, dh)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-13) and np.allclose(dwt, wt.grad.numpy(), atol=1e-13)
    # closed form: unit weight, eps = 0 => every row has mean square 1, and scaling x changes nothing
    h = orc.rmsnorm(x, np.ones(7), 0.0)
    assert np.allclose((h * h).mean(-1), 1.0, atol=1e-14)
    assert np.allclose(orc.rmsnorm(3.7 * x, np.ones(7), 0.0), h, atol=1e-14)


def test_fused_path_with_rmsnorm_finite_differences():
    """hidden = x before the norm: loss is the loss of the path on rmsnorm(x); dH = dL/dx and
    d_rms_weight by finite differences of the independently written surrogate."""
    H, W, _, tok, mask, R, gid, logp_b = _tiny(23)
    wgt = 1.0 + 0.3 * np.random.default_rng(24).normal(size=H.shape[2])
    eps_n = 1e-3
    out = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, rms_weight=wgt, rms_eps=eps_n)
    plain = orc.iw_pg_loss_fwd_bwd(orc.rmsnorm(H, wgt, eps_n), W, tok, mask, logp_b, R, gid, 2)
    assert out["loss"] == plain["loss"] and np.array_equal(out["dW"], plain["dW"])
    A = out["adv"].tolist()

    def py_norm(Hx, wx):
        return [[[Hx[n][t][k] * wx[k] / math.sqrt(sum(v * v for v in Hx[n][t]) / len(wx) + eps_n) for k in range(len(wx))]
                 for t in range(len(Hx[0]))] for n in range(len(Hx))]

    def obj(Hx, wx):
        return _py_surrogate(py_norm(Hx.tolist(), wx.tolist()), W.tolist(), tok.tolist(), mask.tolist(), logp_b.tolist(), A)

    assert abs(obj(H, wgt) - out["loss"]) < 1e-13
    e = 1e-6
    for idx in itertools.product(range(H.shape[0]), range(H.shape[1]), range(H.shape[2])):
        Hp, Hm = H.copy(), H.copy()
        Hp[idx] += e
        Hm[idx] -= e
        assert abs(out["dH"][idx] - (obj(Hp, wgt) - obj(Hm, wgt)) / (2 * e)) < 1e-8, idx
    for k in range(len(wgt)):
        wp, wm = wgt.copy(), wgt.copy()
        wp[k] += e
        wm[k] -= e
        assert abs(out["d_rms_weight"][k] - (obj(H, wp) - obj(H, wm)) / (2 * e)) < 1e-8, k
    # rounding the normalised hidden state to bf16 moves the loss by bf16's relative precision, no more
    r = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, logp_b, R, gid, 2, rms_weight=wgt, rms_eps=eps_n, round_normed_hidden=True)
    assert 0 < abs(r["loss"] - out["loss"]) < 0.05 * abs(out["loss"])



def test_compaction():
    rng = np.random.default_rng(12)
    mask = (rng.random((5, 9)) < 0.6).astype(np.uint8)   # arbitrary pattern, not only right padding
    mask[3] = 0
    seq_len, cu, row_index = orc.compaction(mask)
    ref_rows = [n * 9 + t for n in range(5) for t in range(9) if mask[n, t]]
    assert row_index.tolist() == ref_rows
    assert seq_len.tolist() == [int(mask[n].sum()) for n in range(5)]
    assert cu.tolist() == [0] + list(itertools.accumulate(seq_len.tolist()))


# ---------------------------------------------------------------- baseline loss steps (GRPO, DAPO)
def _py_clipped_objective(H, W, tok, mask, logp_old, logp_ref, adv, eps_low, eps_high, beta, norm_mode):
    """The loss of the clipped token-level surrogate written out with explicit loops (independent of
    the oracle's code): - sum omega (min(r A, clip(r) A) - beta kl)."""
    N, T = len(tok), len(tok[0])
    M = sum(1 for n in range(N) for t in range(T) if mask[n][t])
    tot = 0.0
    for n in range(N):
        L = sum(1 for t in range(T) if mask[n][t])
        for t in range(T):
            if not mask[n][t]:
                continue
            lp = _py_logsoftmax_at(H[n][t], W, tok[n][t])
            r = math.exp(lp - logp_old[n][t])
            surr = min(r * adv[n], max(min(r, 1 + eps_high), 1 - eps_low) * adv[n])
            kl = 0.0
            if beta:
                dlt = logp_ref[n][t] - lp
                kl = math.exp(dlt) - dlt - 1.0
            tot += (surr - beta * kl) / (N * L if norm_mode == 0 else M)
    return -tot


def test_clipped_surrogate_hand_example():
    rows = np.array([l.split() for l in open(os.path.join(GOLDEN, "clipped_surrogate_hand_example.txt"))
                     if l.strip() and not l.startswith("#")], dtype=np.float64)
    r = rows[:, 2].reshape(2, 2)
    A = np.array([1.0, -1.0])
    cur = np.log(r)                  # logp_old = 0
    g, loss, diag = orc.clipped_token_coefficients(cur, np.zeros((2, 2)), None, np.ones((2, 2)), A, 0.2, 0.2, 0.0, 0)
    assert abs(loss - (-0.05)) < 1e-15
    assert np.allclose(g.reshape(-1), -0.25 * rows[:, 4], atol=1e-15) and np.allclose(g.reshape(-1), [0, -0.225, 0, 0.275], atol=1e-15)
    assert diag["clip_fraction"] == 0.5 == rows[:, 5].mean()
    # token-level normalisation (DAPO): the same here, every generation has two tokens
    g1, loss1, _ = orc.clipped_token_coefficients(cur, np.zeros((2, 2)), None, np.ones((2, 2)), A, 0.2, 0.2, 0.0, 1)
    assert np.array_equal(g, g1) and loss == loss1
    # clip-higher (DAPO's eps_high = 0.28): the 1.5 token is still clipped, now at 1.28
    _, loss2, _ = orc.clipped_token_coefficients(cur, np.zeros((2, 2)), None, np.ones((2, 2)), A, 0.2, 0.28, 0.0, 1)
    assert abs(loss2 - (-0.25 * (1.28 + 0.9 - 0.8 - 1.1))) < 1e-15
    # the KL estimator and its derivative at log(pi_ref / pi) = ln 2, ln 0.5, 0 (one generation of three tokens, A = 0)
    ref = np.array([[math.log(2.0), math.log(0.5), 0.0]])
    g, loss, diag = orc.clipped_token_coefficients(np.zeros((1, 3)), np.zeros((1, 3)), ref, np.ones((1, 3)), np.zeros(1),
                                                   0.2, 0.2, 0.04, 0)
    kl = np.array([0.3068528194400547, 0.1931471805599453, 0.0])
    assert abs(loss - 0.04 * kl.sum() / 3) < 1e-15 and abs(diag["mean_kl"] - kl.mean()) < 1e-15
    assert np.allclose(g[0], 0.04 / 3 * np.array([-1.0, 0.5, 0.0]), atol=1e-15)     # dL/dlogp = omega beta (1 - exp(ref - cur))


def test_normalized_group_advantage():
    R = np.array([1.0, 0.0, 1.0, 1.0, 0.3, 0.3, 0.3, 7.0])
    gid = np.array([0, 0, 0, 0, 1, 1, 1, 2])
    out = orc.normalized_group_advantage(R, gid, 4, adv_eps=0.0, std_ddof=0)
    # group 0: mean 0.75, population std sqrt(3/16) = 0.4330127: A = (0.25, -0.75, 0.25, 0.25) / 0.4330127
    assert np.allclose(out["adv"][:4], np.array([0.25, -0.75, 0.25, 0.25]) / math.sqrt(3.0 / 16.0), atol=1e-15)
    assert abs(out["adv"][:4].sum()) < 1e-15 and abs((out["adv"][:4] ** 2).mean() - 1.0) < 1e-14    # zero mean, unit variance
    eps = orc.normalized_group_advantage(R, gid, 4, adv_eps=1e-4)
    assert np.all(eps["adv"][4:] == 0.0)              # equal rewards, and a group of one: no signal
    assert eps["group_size"].tolist() == [4, 3, 1, 0] and eps["group_std"][1] == 0.0
    assert np.allclose(eps["adv"][:4], np.array([0.25, -0.75, 0.25, 0.25]) / (math.sqrt(3.0 / 16.0) + 1e-4), atol=1e-15)
    s1 = orc.normalized_group_advantage(R, gid, 4, adv_eps=0.0, std_ddof=1)
    assert np.allclose(s1["adv"][:4], np.array([0.25, -0.75, 0.25, 0.25]) / math.sqrt(0.25), atol=1e-15)   # sample std: sqrt(0.75/3)
    assert s1["adv"][7] == 0.0 and np.allclose(s1["group_std"][:3], np.array([0.5, 0.0, 0.0]))
    assert np.allclose(np.array([R[:4].std(), R[:4].std(ddof=1)]), [out["group_std"][0], s1["group_std"][0]])    # numpy leg


@pytest.mark.parametrize("variant", ["grpo", "dapo"])
def test_clipped_pg_finite_differences_and_autograd(variant):
    kw = dict(grpo=dict(eps_low=0.2, eps_high=0.2, kl_beta=0.04, norm_mode=0),
              dapo=dict(eps_low=0.2, eps_high=0.28, kl_beta=0.0, norm_mode=1))[variant]
    H, W, W_old, tok, mask, R, gid, logp_old = _tiny(31, N=4, T=3, d=3, V=5, G=2)
    rng = np.random.default_rng(5)
    logp_old = logp_old + mask * rng.normal(size=logp_old.shape) * 0.3      # ratios spread around 1: some clip
    logp_ref = logp_old + mask * rng.normal(size=logp_old.shape) * 0.2
    out = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, logp_old, logp_ref, R, gid, 2, **kw)
    assert 0.0 < out["clip_fraction"] < 1.0
    # no ratio sits on a clip boundary (the objective has a kink there)
    r = np.exp(out["logp_cur"] - logp_old)[mask != 0]
    assert np.abs(r - (1 - kw["eps_low"])).min() > 1e-3 and np.abs(r - (1 + kw["eps_high"])).min() > 1e-3
    f = lambda Hx, Wx: _py_clipped_objective(Hx.tolist(), Wx.tolist(), tok.tolist(), mask.tolist(), logp_old.tolist(),
                                             logp_ref.tolist(), out["adv"].tolist(), kw["eps_low"], kw["eps_high"],
                                             kw["kl_beta"], kw["norm_mode"])
    assert abs(f(H, W) - out["loss"]) < 1e-14
    h = 1e-6
    for idx in np.ndindex(W.shape):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += h; Wm[idx] -= h
        assert abs((f(H, Wp) - f(H, Wm)) / (2 * h) - out["dW"][idx]) < 1e-7, idx
    for idx in np.ndindex(H.shape):
        Hp, Hm = H.copy(), H.copy()
        Hp[idx] += h; Hm[idx] -= h
        fd = (f(Hp, W) - f(Hm, W)) / (2 * h)
        assert abs(fd - out["dH"][idx]) < 1e-7, idx
        if mask[idx[0], idx[1]] == 0:
            assert out["dH"][idx] == 0.0
    # library leg: torch autograd of the same objective in plain tensor ops gives the oracle's dL/dlogp
    lp = torch.tensor(out["logp_cur"], requires_grad=True)
    m = torch.tensor(mask.astype(np.float64))
    A = torch.tensor(out["adv"])[:, None]
    ratio = torch.exp(lp - torch.tensor(logp_old))
    surr = torch.minimum(ratio * A, torch.clamp(ratio, 1 - kw["eps_low"], 1 + kw["eps_high"]) * A)
    dref = torch.tensor(logp_ref) - lp
    per_tok = (surr - kw["kl_beta"] * (torch.exp(dref) - dref - 1)) * m
    loss = -(per_tok.sum(1) / m.sum(1)).mean() if kw["norm_mode"] == 0 else -per_tok.sum() / m.sum()
    loss.backward()
    assert abs(loss.item() - out["loss"]) < 1e-14 and np.allclose(lp.grad.numpy(), out["g"], atol=1e-15)


def test_clipped_pg_special_cases():
    H, W, W_old, tok, mask, R, gid, _ = _tiny(33, N=6, T=4, d=3, V=6, G=3)
    cur, _ = orc.logprob(H, W, tok, mask)
    # (a) equal policies, no KL: every ratio is 1, nothing clips, and the gradient is that of the plain
    # group-relative policy gradient with the normalised advantages, - omega A_n per valid token
    out = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, cur, None, R, gid, 2, kl_beta=0.0, norm_mode=0)
    L = mask.sum(1)
    want = -(out["adv"] / (6 * L))[:, None] * (mask != 0)
    assert np.allclose(out["g"], want, atol=1e-16) and out["clip_fraction"] == 0.0
    dH, dW = orc.backward(H, W, tok, mask, want)
    assert np.allclose(out["dW"], dW, atol=1e-16) and np.allclose(out["dH"], dH, atol=1e-16)
    # its loss is - mean_n A_n, which is 0 for complete groups (advantages sum to zero per group)
    assert abs(out["loss"]) < 1e-14
    # (b) reference = current policy: the KL term and its gradient vanish
    with_kl = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, cur, cur, R, gid, 2, kl_beta=0.04)
    assert with_kl["mean_kl"] == 0.0 and np.array_equal(with_kl["g"], out["g"])
    # (c) the KL estimator is non-negative and pulls the policy towards the reference
    ref = cur + 0.5 * (mask != 0)
    k = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, cur, ref, np.zeros(6), gid, 2, kl_beta=0.04)
    assert k["mean_kl"] > 0 and k["loss"] > 0 and np.all(k["g"][mask != 0] < 0)        # descent raises log pi where pi_ref > pi
    # (d) the two normalisations agree when all generations have the same length, and differ otherwise
    full = np.ones_like(mask)
    cur_f, _ = orc.logprob(H, W, tok, full)
    old_f = cur_f + 0.1
    a = orc.clipped_pg_loss_fwd_bwd(H, W, tok, full, old_f, None, R, gid, 2, norm_mode=0)
    b = orc.clipped_pg_loss_fwd_bwd(H, W, tok, full, old_f, None, R, gid, 2, norm_mode=1)
    assert abs(a["loss"] - b["loss"]) < 1e-15 and np.allclose(a["dW"], b["dW"], atol=1e-16)
    if len(set(L.tolist())) > 1:
        a = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, cur + 0.1 * (mask != 0), None, R, gid, 2, norm_mode=0)
        b = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, cur + 0.1 * (mask != 0), None, R, gid, 2, norm_mode=1)
        assert abs(a["loss"] - b["loss"]) > 1e-6
    # (e) a group with equal rewards contributes nothing to the surrogate (A = 0): only the KL term is left
    Rz = R.copy(); Rz[:3] = 0.5          # exactly representable: the group mean is exact
    z = orc.clipped_pg_loss_fwd_bwd(H, W, tok, mask, cur + 0.2 * (mask != 0), None, Rz, gid, 2)
    assert np.all(z["adv"][:3] == 0.0) and np.all(z["g"][:3] == 0.0) and np.any(z["g"][3:] != 0.0)


def test_adamw_step_against_torch():
    """Library leg: torch.optim.AdamW in float64 over five steps, with and without weight decay; and the
    first step's closed form: m_hat = g, v_hat = g^2, so w moves by lr * sign(g) (up to eps)."""
    rng = np.random.default_rng(41)
    for wd in (0.0, 0.1):
        w0 = rng.normal(size=37)
        p = torch.nn.Parameter(torch.tensor(w0))
        opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
        w, m, v = w0.copy(), np.zeros(37), np.zeros(37)
        for step in range(1, 6):
            g = rng.normal(size=37) * 10.0 ** rng.integers(-3, 2)
            p.grad = torch.tensor(g)
            opt.step()
            w, m, v = orc.adamw_step(w, g, m, v, step, 3e-3, 0.9, 0.95, 1e-8, wd)
            assert np.allclose(w, p.detach().numpy(), rtol=0, atol=1e-14), (wd, step)
    g = np.array([0.5, -2.0, 1e-3])
    w, _, _ = orc.adamw_step(np.zeros(3), g, np.zeros(3), np.zeros(3), 1, 0.01, eps=0.0)
    assert np.allclose(w, -0.01 * np.sign(g), atol=1e-15)
