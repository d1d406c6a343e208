"""Float64 CPU oracle for RAPID's importance-weighted group-advantage policy-gradient loss.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP library is
checked against.  Only the tests, the smoke check and the benchmark's CPU-baseline leg may call
it; the product path never does.  It shares no code with the HIP path and imports nothing from
the package.

Every function restates a passage of the RAPID paper (arXiv 2510.03515):

* Sec. 3.1 (Preliminaries): a generation y has tokens y_t; pi_theta(y|x) is the product of the
  per-token probabilities, so log pi_theta(y|x) = sum_t log softmax(h_t W)[y_t].
* Sec. 3.3, Eq. (2): group advantage A_n = R_n - mean of R over the group of n.
* Sec. 3.4, Eq. (3): importance-weighted policy gradient, weight pi_theta(y_n|x_n)/mu(y_n|x_n).
* Sec. 3.4, Eq. (4)/(5): importance-weighted group baseline, ratio clipped at eta.
* Sec. 4.3, paragraph "Importance-weight clipping": per-token ratios are accumulated over the
  generation first, the clip acts on the generation-level ratio.
* Appendix A, RL hyper-parameter table: eta = 2.0.
* Sec. 4.3, first paragraph: staleness = mean of the clipped weight in log scale.
* Sec. 4.1, "Baselines", and Appendix A (KL coefficient 0.04, GRPO only): the loss steps of GRPO and
  DAPO, restated at the end of this file from the papers the RAPID paper cites for them.

Readings of the paper taken here (each also listed in the design document):

* Eq. (5) prints max{ratio, eta}; "standard importance weight clipping" that tames *large*
  weights is min{ratio, eta}.  With min, equal policies give every weight exactly 1 and Eq. (5)
  falls back to Eq. (2); with max it could not.  The oracle uses min.
* The stray upper limit N on the group sums of Eq. (4)/(5) is ignored: sums run over the group.
* The advantage is a constant with respect to theta (Alg. 1 computes it first, then the
  gradient of Eq. (3), whose nabla acts on pi_theta only).
* The outer weight in Eq. (3) is the unclipped ratio (coef_mode 0).  coef_mode 1 replaces it
  by the clipped weight held constant; the paper does not print that variant: parity unpinned
  for the *choice* between the two, both are computed the same way below.
* Normalisation is 1/N with N the number of generations in the call; nothing is divided by a
  length or by a group standard deviation (the paper never does).
* The library returns the loss to descend, L = -J_surrogate, since the paper ascends J.

Shapes: hidden [N,T,d]; W [d,V] (logical); tokens [N,T] int; mask [N,T] 0/1; logp_behav [N,T];
rewards [N]; group_ids [N] ints in [0,K).
"""
from __future__ import annotations

import math

import numpy as np

_F = np.float64


def _as64(a):
    return np.asarray(a, dtype=_F)


def logprob(hidden, W, tokens, mask, temperature=1.0, row_chunk=2048):
    """Per-token log-probability of the sampled token under softmax(h W / temperature).

    Sec. 3.1: pi_theta(y_t | .) is the softmax of the LM head output.  Returns (logp, lse),
    both [N,T] float64, zero at masked positions.
    lse = max(z) + log(sum(exp(z - max(z)))), logp = z[y] - lse.
    """
    H = _as64(hidden)
    Wd = _as64(W)
    tok = np.asarray(tokens).astype(np.int64)
    msk = np.asarray(mask) != 0
    N, T, d = H.shape
    V = Wd.shape[1]
    logp = np.zeros((N, T), _F)
    lse = np.zeros((N, T), _F)
    rows = np.argwhere(msk)
    for s in range(0, rows.shape[0], row_chunk):
        rr = rows[s:s + row_chunk]
        z = (H[rr[:, 0], rr[:, 1], :] @ Wd) / temperature
        zmax = z.max(axis=1)
        l = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
        y = tok[rr[:, 0], rr[:, 1]]
        if (y < 0).any() or (y >= V).any():
            raise ValueError("token id outside [0, V) at an unmasked position")
        logp[rr[:, 0], rr[:, 1]] = z[np.arange(z.shape[0]), y] - l
        lse[rr[:, 0], rr[:, 1]] = l
    return logp, lse


def round_to_bf16(x):
    """x (float64) rounded ONCE to the nearest bfloat16, ties to even, returned as float64: the value a
    bf16 tensor holds.  bfloat16 = sign, 8 exponent bits (those of float32), 7 fraction bits.  A normal
    float64 keeps the top 7 of its 52 fraction bits: the other 45 are rounded away on the integer
    pattern (a carry into the exponent is the correct result); values above the largest bfloat16
    become infinity; below 2^-126 (bfloat16 subnormals) the spacing is the fixed 2^-133.  Going
    through float32 first would round twice and differ for values within 2^-25 (relative) above or
    below a bfloat16 midpoint."""
    x64 = np.ascontiguousarray(np.asarray(x, _F))
    bits = x64.view(np.uint64)
    keep = np.uint64(45)
    low = np.uint64((1 << 45) - 1)
    rounded = (bits + np.uint64((1 << 44) - 1) + ((bits >> keep) & np.uint64(1))) & ~low
    out = rounded.view(_F).copy()
    big = np.abs(out) > 3.3895313892515355e38            # largest bfloat16 = (2 - 2^-7) 2^127
    out[big] = np.sign(out[big]) * np.inf
    tiny = np.abs(x64) < 2.0 ** -126
    out[tiny] = np.rint(x64[tiny] * 2.0 ** 133) * 2.0 ** -133
    nan = np.isnan(x64)
    out[nan] = np.nan
    return out.reshape(np.shape(x))


def rmsnorm(x, weight, eps=1e-6):
    """Root-mean-square layer normalisation over the last axis (Zhang & Sennrich 2019), the final
    norm of the Qwen2.5 models the paper trains: h = x * weight / sqrt(mean(x^2) + eps).  Not part of
    the paper's method: the operand the fused call can normalise on the way in."""
    x = _as64(x)
    inv = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    return x * inv * _as64(weight)


def rmsnorm_backward(x, weight, eps, dh):
    """Gradients of sum(dh * rmsnorm(x, weight)) with respect to x and weight.
    With r = 1/sqrt(mean(x^2) + eps):  dweight_k = sum_rows dh_k x_k r;
    dx_k = r weight_k dh_k - x_k r^3 (sum_j dh_j weight_j x_j) / d."""
    x, w, dh = _as64(x), _as64(weight), _as64(dh)
    d = x.shape[-1]
    r = 1.0 / np.sqrt((x * x).mean(axis=-1, keepdims=True) + eps)
    dweight = (dh * x * r).reshape(-1, d).sum(axis=0)
    t = (dh * w * x).sum(axis=-1, keepdims=True)
    dx = r * w * dh - x * (r ** 3) * t / d
    return dx, dweight


def token_logratio(logp_cur, logp_behav, mask):
    """Delta_{n,t} = mask * (log pi_theta(y_t) - log mu(y_t)): the token-level log ratio (Fig. 3)."""
    msk = (np.asarray(mask) != 0).astype(_F)
    return msk * (_as64(logp_cur) - _as64(logp_behav))


def seq_logratio(logp_cur, logp_behav, mask):
    """s_n = sum_t Delta_{n,t} = log(pi_theta(y_n|x_n) / mu(y_n|x_n)).

    Sec. 3.4, Eq. (3): the ratio is between whole-generation probabilities; Sec. 4.3 says the
    per-token ratios are accumulated over the generation before clipping.
    """
    return token_logratio(logp_cur, logp_behav, mask).sum(axis=1)


def clipped_weight(s, eta=2.0):
    """w_n = min(exp(s_n), eta)  (Eq. (5) with the clip read as min; eta = 2.0 in Appendix A)."""
    s = _as64(s)
    log_eta = math.log(eta) if math.isfinite(eta) else math.inf
    return np.exp(np.minimum(s, log_eta))


def group_advantage(rewards, group_ids, K, s=None, eta=2.0, baseline_mode=0):
    """Group advantage.

    s is None          -> Eq. (2):  A_n = R_n - (1/N_k) sum_{n' in group k} R_n'
    s given, eta=inf   -> Eq. (4):  A_n = R_n - (1/N_k) sum_{n'} rho_n' R_n'
    s given, eta<inf   -> Eq. (5):  rho replaced by min(rho, eta)
    baseline_mode 1    -> the leave-one-out sum of Sec. 3.4 (over the group without n), divided
                          by N_k as printed; baseline_mode 2 divides by N_k - 1 instead.

    Returns dict(adv[N], weight[N], group_mean[K], group_std[K], group_size[K]); mean/std are the
    plain (population) statistics of R per group, diagnostics only.  An empty group has size 0,
    mean 0, std 0.
    """
    R = _as64(rewards)
    gid = np.asarray(group_ids).astype(np.int64)
    N = R.shape[0]
    if (gid < 0).any() or (gid >= K).any():
        raise ValueError("group id outside [0, K)")
    w = np.ones(N, _F) if s is None else clipped_weight(s, eta)
    size = np.zeros(K, np.int64)
    sum_wr = np.zeros(K, _F)
    sum_r = np.zeros(K, _F)
    for n in range(N):
        size[gid[n]] += 1
        sum_wr[gid[n]] += w[n] * R[n]
        sum_r[gid[n]] += R[n]
    mean = np.where(size > 0, sum_r / np.maximum(size, 1), 0.0)
    sq = np.zeros(K, _F)
    for n in range(N):
        sq[gid[n]] += (R[n] - mean[gid[n]]) ** 2
    std = np.where(size > 0, np.sqrt(sq / np.maximum(size, 1)), 0.0)
    adv = np.zeros(N, _F)
    for n in range(N):
        k = gid[n]
        if baseline_mode == 0:
            b = sum_wr[k] / size[k]
        elif baseline_mode == 1:
            b = (sum_wr[k] - w[n] * R[n]) / size[k]
        elif baseline_mode == 2:
            b = (sum_wr[k] - w[n] * R[n]) / (size[k] - 1) if size[k] > 1 else 0.0
        else:
            raise ValueError("baseline_mode")
        adv[n] = R[n] - b
    return dict(adv=adv, weight=w, group_mean=mean, group_std=std, group_size=size)


def coefficients(s, adv, eta=2.0, coef_mode=0, loss_scale=1.0, normalized=False):
    """g_n = dL/d logp_{n,t} for every valid token t of generation n, and the loss.

    L = -(loss_scale/N) sum_n c_n A_n with c_n = rho_n (Eq. (3)), or the clipped weight for
    coef_mode 1.  d rho_n / d logp_{n,t} = rho_n, so g_n = -(loss_scale/N) c_n A_n and L = sum g_n.
    With normalized=True everything is scaled by exp(-lam), lam = log max_n |g_n| evaluated in
    the log domain (0 if every g_n is 0), so that values survive ratios that underflow.
    Returns (g[N], loss, lam).
    """
    s = _as64(s)
    A = _as64(adv)
    N = s.shape[0]
    log_c = s if coef_mode == 0 else np.minimum(s, math.log(eta) if math.isfinite(eta) else math.inf)
    nz = A != 0
    log_abs_g = np.full(N, -np.inf)
    log_abs_g[nz] = log_c[nz] + np.log(np.abs(A[nz])) + math.log(loss_scale) - math.log(N)
    lam = 0.0
    if normalized and nz.any():
        lam = float(log_abs_g.max())
    g = np.zeros(N, _F)
    g[nz] = -np.sign(A[nz]) * np.exp(log_abs_g[nz] - lam)
    return g, float(g.sum()), lam


def token_coefficients(tok_logratio, mask, adv, eta=2.0, coef_mode=0, loss_scale=1.0, normalized=False):
    """Token-level variant of the outer weight (ratio_level 1).  NOT an estimator the paper defines:
    its ratio is between whole generations (Sec. 3.4, Eq. (3)) and token-level ratios appear only as
    a diagnostic (Sec. 4.3).  Here the weight rho_n of Eq. (3) is replaced, token by token, by that
    token's ratio rho_{n,t} = exp(Delta_{n,t}); the advantages stay those of Eq. (5):

        L = -(loss_scale/N) sum_n A_n sum_{t valid} c_{n,t},   c_{n,t} = rho_{n,t}  (coef_mode 0)
                                                            or min(rho_{n,t}, eta) held constant (1)
        g_{n,t} = dL/d logp_{n,t} = -(loss_scale/N) c_{n,t} A_n,   L = sum_{n,t valid} g_{n,t}.

    With normalized=True everything is scaled by exp(-lam), lam = log max_{n,t} |g_{n,t}|.
    Returns (g[N,T] (0 at masked positions), loss, lam).
    """
    D = _as64(tok_logratio)
    A = _as64(adv)
    msk = np.asarray(mask) != 0
    N, T = D.shape
    log_c = D if coef_mode == 0 else np.minimum(D, math.log(eta) if math.isfinite(eta) else math.inf)
    g = np.zeros((N, T), _F)
    log_abs_g = np.full((N, T), -np.inf)
    for n in range(N):
        if A[n] != 0:
            log_abs_g[n, msk[n]] = log_c[n, msk[n]] + math.log(abs(A[n])) + math.log(loss_scale) - math.log(N)
    lam = 0.0
    if normalized and np.isfinite(log_abs_g).any():
        lam = float(log_abs_g.max())
    for n in range(N):
        if A[n] != 0:
            g[n, msk[n]] = -np.sign(A[n]) * np.exp(log_abs_g[n, msk[n]] - lam)
    return g, float(g.sum()), lam


def backward(hidden, W, tokens, mask, g, temperature=1.0, row_chunk=2048):
    """Gradients of sum_{n,t valid} g_{n,t} * logp_{n,t} with respect to hidden and W; g is [N]
    (one coefficient per generation, g_{n,t} = g_n) or [N,T] (one per token).

    For a valid row: p = softmax(z), dz = g_{n,t} (e_y - p) / temperature, dH = W dz,
    dW += outer(h, dz).  Masked rows get dH = 0.  Returns (dH [N,T,d], dW [d,V]).
    """
    H = _as64(hidden)
    Wd = _as64(W)
    tok = np.asarray(tokens).astype(np.int64)
    msk = np.asarray(mask) != 0
    g = _as64(g)
    N, T, d = H.shape
    dH = np.zeros((N, T, d), _F)
    dW = np.zeros_like(Wd)
    rows = np.argwhere(msk)
    for s0 in range(0, rows.shape[0], row_chunk):
        rr = rows[s0:s0 + row_chunk]
        h = H[rr[:, 0], rr[:, 1], :]
        z = (h @ Wd) / temperature
        zmax = z.max(axis=1, keepdims=True)
        e = np.exp(z - zmax)
        p = e / e.sum(axis=1, keepdims=True)
        dz = -p
        dz[np.arange(dz.shape[0]), tok[rr[:, 0], rr[:, 1]]] += 1.0
        g_rows = g[rr[:, 0]] if g.ndim == 1 else g[rr[:, 0], rr[:, 1]]
        dz *= (g_rows / temperature)[:, None]
        dH[rr[:, 0], rr[:, 1], :] = dz @ Wd.T
        dW += h.T @ dz
    return dH, dW


def iw_pg_loss_fwd_bwd(hidden, W, tokens, mask, logp_behav, rewards, group_ids, K,
                       eta=2.0, coef_mode=0, baseline_mode=0, loss_scale=1.0, temperature=1.0,
                       normalized_grads=False, coef_override=None, row_chunk=2048, ratio_level=0,
                       rms_weight=None, rms_eps=1e-6, round_normed_hidden=False):
    """The whole update-step loss of Alg. 1 (procedure IW-GRPG, one mini-batch): advantages by
    Eq. (5), gradient by Eq. (3).  ratio_level 1 swaps the outer weight for the token-level one of
    token_coefficients (then `g` is [N,T]).  With rms_weight, `hidden` is the input x of a final
    RMSNorm: the path runs on h = rmsnorm(x) (rounded to bf16 if round_normed_hidden: the
    normalised state of a bf16 model is a bf16 tensor; the rounding passes gradients through
    unchanged), dH is the gradient with respect to x and d_rms_weight is returned too.
    Returns a dict with loss, dH, dW and every intermediate."""
    x_in = hidden
    if rms_weight is not None:
        hidden = rmsnorm(x_in, rms_weight, rms_eps)
        if round_normed_hidden:
            hidden = round_to_bf16(hidden)
    logp_cur, lse = logprob(hidden, W, tokens, mask, temperature, row_chunk)
    tok_lr = token_logratio(logp_cur, logp_behav, mask)
    s = tok_lr.sum(axis=1)
    ga = group_advantage(rewards, group_ids, K, s=s, eta=eta, baseline_mode=baseline_mode)
    N = s.shape[0]
    if coef_override is not None:
        g = _as64(coef_override)
        loss, lam = float(g.sum()), 0.0
    elif ratio_level == 0:
        g, loss, lam = coefficients(s, ga["adv"], eta, coef_mode, loss_scale, normalized_grads)
    elif ratio_level == 1:
        g, loss, lam = token_coefficients(tok_lr, mask, ga["adv"], eta, coef_mode, loss_scale, normalized_grads)
    else:
        raise ValueError("ratio_level")
    dH, dW = backward(hidden, W, tokens, mask, g, temperature, row_chunk)
    d_rms_weight = None
    if rms_weight is not None:
        dH, d_rms_weight = rmsnorm_backward(x_in, rms_weight, rms_eps, dH)
    log_eta = math.log(eta) if math.isfinite(eta) else math.inf
    log_w = np.minimum(s, log_eta)
    return dict(loss=loss, dH=dH, dW=dW, d_rms_weight=d_rms_weight, logp_cur=logp_cur, lse=lse, tok_logratio=tok_lr,
                seq_logratio=s, adv=ga["adv"], weight=ga["weight"], g=g, grad_log_scale=lam,
                group_mean=ga["group_mean"], group_std=ga["group_std"],
                group_size=ga["group_size"],
                n_tokens=int((np.asarray(mask) != 0).sum()),
                n_clipped=int((s > log_eta).sum()),
                mean_log_w=float(log_w.mean()) if N else 0.0,
                mean_abs_log_w=float(np.abs(log_w).mean()) if N else 0.0,
                max_abs_s=float(np.abs(s).max()) if N else 0.0)


def compaction(mask):
    """Integer bookkeeping of the padding mask: seq_len[N], cu_seqlen[N+1], row_index[M] (flat
    n*T+t of every valid position in row-major order)."""
    msk = np.asarray(mask) != 0
    seq_len = msk.sum(axis=1).astype(np.int64)
    cu = np.zeros(msk.shape[0] + 1, np.int64)
    cu[1:] = np.cumsum(seq_len)
    row_index = np.flatnonzero(msk.reshape(-1)).astype(np.int64)
    return seq_len, cu, row_index


# ----------------------------------------------------------------------------------------------------
# Loss steps of the paper's RL baselines (Sec. 4.1, "Baselines": GRPO, Shao et al. 2024; DAPO, Yu et
# al. 2025; Appendix A: KL coefficient 0.04 for GRPO only).  The paper does not print their objectives:
# they are restated here from the cited papers, for a like-for-like comparison of the loss step on the
# same kernels.  Parity unpinned by the paper; pinned by hand values, special cases and finite
# differences of an objective written with explicit loops (tests).

def normalized_group_advantage(rewards, group_ids, K, adv_eps=1e-4, std_ddof=0):
    """A_n = (R_n - mean_k) / (std_k + adv_eps) over the group k of n (GRPO's outcome-supervision
    advantage; DAPO uses the same).  std_ddof 0: population std (1/N_k), 1: sample std (1/(N_k - 1)),
    0 for a group of one.  A group whose rewards are all equal has std 0 and A = 0 / adv_eps = 0: it
    carries no policy-gradient signal (the reading taken for the zero-std case).
    Returns dict(adv, group_mean, group_std, group_size)."""
    R = _as64(rewards)
    gid = np.asarray(group_ids).astype(np.int64)
    N = R.shape[0]
    if (gid < 0).any() or (gid >= K).any():
        raise ValueError("group id outside [0, K)")
    size = np.zeros(K, np.int64)
    mean = np.zeros(K, _F)
    std = np.zeros(K, _F)
    for k in range(K):
        members = [n for n in range(N) if gid[n] == k]
        size[k] = len(members)
        if members:
            mean[k] = sum(R[n] for n in members) / len(members)
            ss = sum((R[n] - mean[k]) ** 2 for n in members)
            den = len(members) - std_ddof
            std[k] = math.sqrt(ss / den) if den > 0 else 0.0
    adv = np.zeros(N, _F)
    for n in range(N):
        num = R[n] - mean[gid[n]]
        adv[n] = num / (std[gid[n]] + adv_eps) if num != 0.0 else 0.0     # 0 / 0 (equal rewards, adv_eps = 0) is 0
    return dict(adv=adv, group_mean=mean, group_std=std, group_size=size)


def clipped_token_coefficients(logp_cur, logp_old, logp_ref, mask, adv, eps_low=0.2, eps_high=0.2, kl_beta=0.0,
                               norm_mode=0, loss_scale=1.0):
    """Token-level clipped surrogate with an optional KL penalty, and its derivative with respect to
    the current log-probs.

    r_{n,t} = exp(logp_cur - logp_old)                                  (token-level ratio)
    surr    = min(r A_n, clip(r, 1 - eps_low, 1 + eps_high) A_n)        (PPO-style clip; GRPO: 0.2 / 0.2,
                                                                         DAPO: 0.2 / 0.28, "clip-higher")
    kl      = exp(logp_ref - logp_cur) - (logp_ref - logp_cur) - 1      (the unbiased, non-negative estimator
                                                                         GRPO uses; kl_beta = 0.04 in Appendix A,
                                                                         0 for DAPO, which drops the term)
    L = - loss_scale * sum_{n,t valid} omega_{n,t} (surr - kl_beta * kl)
    omega = 1 / (N L_n)   norm_mode 0: mean over a generation's tokens, then over generations (GRPO)
          = 1 / M         norm_mode 1: mean over all M valid tokens of the call (DAPO's token-level loss)
    d surr / d logp_cur = r A_n where the unclipped term is the minimum (ties included), else 0: a token
    whose ratio has left the clip range in the direction its advantage pushes gets no gradient.
    d kl / d logp_cur = 1 - exp(logp_ref - logp_cur).
    Returns (g [N,T] = dL/dlogp_cur, loss, dict(clip_fraction, mean_kl))."""
    cur, old = _as64(logp_cur), _as64(logp_old)
    msk = np.asarray(mask) != 0
    A = _as64(adv)
    N, T = cur.shape
    M = int(msk.sum())
    g = np.zeros((N, T), _F)
    loss = 0.0
    n_clipped = 0
    kl_sum = 0.0
    for n in range(N):
        L = int(msk[n].sum())
        for t in range(T):
            if not msk[n, t]:
                continue
            omega = loss_scale / (N * L) if norm_mode == 0 else loss_scale / M
            r = math.exp(cur[n, t] - old[n, t])
            rc = min(max(r, 1.0 - eps_low), 1.0 + eps_high)
            unclipped, clipped = r * A[n], rc * A[n]
            surr = min(unclipped, clipped)
            dsurr = r * A[n] if unclipped <= clipped else 0.0
            if unclipped > clipped:
                n_clipped += 1
            kl = dkl = 0.0
            if kl_beta != 0.0:
                dref = float(logp_ref[n, t]) - cur[n, t]
                kl = math.exp(dref) - dref - 1.0
                dkl = 1.0 - math.exp(dref)
                kl_sum += kl
            loss -= omega * (surr - kl_beta * kl)
            g[n, t] = -omega * (dsurr - kl_beta * dkl)
    return g, loss, dict(clip_fraction=n_clipped / M if M else 0.0, mean_kl=kl_sum / M if M else 0.0)


def clipped_pg_loss_fwd_bwd(hidden, W, tokens, mask, logp_old, logp_ref, rewards, group_ids, K, eps_low=0.2,
                            eps_high=0.2, kl_beta=0.0, norm_mode=0, adv_eps=1e-4, std_ddof=0, loss_scale=1.0,
                            temperature=1.0, row_chunk=2048):
    """One loss step of GRPO (eps 0.2 / 0.2, kl_beta 0.04, norm_mode 0) or DAPO (eps 0.2 / 0.28, kl_beta 0,
    norm_mode 1) through the LM head: current log-probs, std-normalised group advantages, the clipped
    token-level surrogate above, and its gradients with respect to hidden and W."""
    logp_cur, lse = logprob(hidden, W, tokens, mask, temperature, row_chunk)
    ga = normalized_group_advantage(rewards, group_ids, K, adv_eps, std_ddof)
    g, loss, diag = clipped_token_coefficients(logp_cur, logp_old, logp_ref, mask, ga["adv"], eps_low, eps_high, kl_beta,
                                               norm_mode, loss_scale)
    dH, dW = backward(hidden, W, tokens, mask, g, temperature, row_chunk)
    return dict(loss=loss, dH=dH, dW=dW, logp_cur=logp_cur, adv=ga["adv"], g=g, group_mean=ga["group_mean"],
                group_std=ga["group_std"], group_size=ga["group_size"], clip_fraction=diag["clip_fraction"],
                mean_kl=diag["mean_kl"], n_tokens=int((np.asarray(mask) != 0).sum()))


def adamw_step(w, grad, exp_avg, exp_avg_sq, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One step of AdamW (Adam with decoupled weight decay, Loshchilov & Hutter 2019), the optimiser family
    of the paper's training runs (Appendix A lists the learning rate; Alg. 1's update line is this step).
    m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
    w <- w - lr ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay w ).
    Returns (w, m, v) as new float64 arrays; step counts from 1."""
    w, g, m, v = _as64(w), _as64(grad), _as64(exp_avg), _as64(exp_avg_sq)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    return w - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * w), m, v
