"""Inner loop of RAPID (Alg. 1, procedure IW-GRPG) on a synthetic bandit: one inference batch, H
off-policy updates of the LM head, each on its own mini-batch.

As in Alg. 1 the inference batch Z (hidden states, sampled tokens, rewards, behaviour log-probs
stored with the initial W = mu) is cut into H = N_inference / N_step mini-batches of whole groups,
which the inner loop walks through in order (Sec. 3.2; Alg. 1, the loop over mini-batches).  Step h
calls rapid_iw_pg_loss_fwd_bwd on mini-batch h with the current W against the stored log mu, then
takes one gradient step (rapid_sgd_step, or rapid_adamw_step: the optimiser family of the paper's runs).  Step 1 is on-policy (all ratios exactly 1); the
staleness of Sec. 4.3 (mean |log clipped weight|) and the clip proportion grow with h, the trend of
the paper's study of the number of inner steps.  Everything numeric runs in the library; this
module only sequences calls and slices tensors.

    python -m paper_2510_03515_amd.iw_grpg [--inner-steps 8] [--lr 0.02] [--optimizer sgd|adamw] [--logits-cache]
"""
from __future__ import annotations

import argparse

import torch

from . import binding as rb
from . import workloads as wl


def _is_reward(w, W, logp_b):
    """Self-normalised importance-sampling estimate, on the whole inference batch, of the expected
    reward of the policy with weights W (equals the batch's mean reward for W = mu)."""
    lp, _ = rb.rapid_logprob_fwd(w["hidden"], W, w["tokens"], w["mask"])
    s, _ = rb.rapid_seq_logratio(lp, logp_b, w["mask"])
    # With the whole batch as one group and no clip, the unclipped baseline of Eq. (4) is (1/N) sum rho R:
    # once with the rewards, once with rewards of 1 (then it is the mean ratio); their quotient is the estimate.
    one_group = torch.zeros_like(w["group_ids"])
    ones = torch.ones_like(w["rewards"])
    num = rb.rapid_group_advantage(w["rewards"], one_group, 1, seq_logratio=s, eta=float("inf"))["adv"]
    den = rb.rapid_group_advantage(ones, one_group, 1, seq_logratio=s, eta=float("inf"))["adv"]
    return (w["rewards"][0] - num[0]).item() / (1.0 - den[0]).item()


def iw_grpg(w, inner_steps=8, lr=0.02, eta=2.0, coef_mode=1, logits_cache=False, optimizer="sgd"):
    """Runs Alg. 1's IW-GRPG on the workload dict `w` (device tensors of workloads.make_workload with
    sigma = 0 and tokens_from = "cur": the batch is sampled from W itself, and group_ids = n // G).
    The number of prompts must be a multiple of `inner_steps`.  Returns (per-step log, summary dict,
    final weights in the workload dtype).

    coef_mode 1 (clipped outer weight) is the default here: with the unclipped ratio of coef_mode 0
    a few generations whose ratio has grown dominate the later steps.  logits_cache (bf16 only): the
    backward of every step contracts the probability ratios its forward kept instead of regenerating
    the logits.  optimizer: "sgd" (plain descent with step lr) or "adamw" (lr is then AdamW's; its per-element
    step is about lr whatever the gradient's size, so it wants a far smaller value than SGD's)."""
    spec = w["spec"]
    K, G, H = w["K"], spec.G, int(inner_steps)
    assert K % H == 0, "prompts must divide into equal mini-batches"
    Kh, Nh = K // H, (K // H) * G
    W = w["W"].clone()
    master = W.float().contiguous()
    exp_avg, exp_avg_sq = (torch.zeros_like(master), torch.zeros_like(master)) if optimizer == "adamw" else (None, None)
    logp_b, _ = rb.rapid_logprob_fwd(w["hidden"], W, w["tokens"], w["mask"])   # log mu, stored at "inference"
    reward_mu = _is_reward(w, W, logp_b)
    gid_local = w["group_ids"][:Nh].contiguous()                                # 0 .. Kh-1 in every mini-batch
    buf = rb.IwPgBuffers(w["hidden"][:Nh], W, Kh, logits_cache=logits_cache)
    log = []
    for h in range(H):
        sl = slice(h * Nh, (h + 1) * Nh)
        out = rb.rapid_iw_pg_loss_fwd_bwd(w["hidden"][sl], W, w["tokens"][sl], w["mask"][sl], logp_b[sl],
                                          w["rewards"][sl], gid_local, Kh, buffers=buf, eta=eta,
                                          coef_mode=coef_mode, logits_cache=logits_cache)
        dg = out.read_diag()
        log.append(dict(step=h + 1, loss=out.loss.item(), staleness=dg["mean_abs_log_w"],
                        clip_fraction=dg["n_clipped"] / dg["n_sequences"], max_abs_s=dg["max_abs_s"]))
        if optimizer == "adamw":
            rb.rapid_adamw_step(master, out.dW, exp_avg, exp_avg_sq, h + 1, lr, w_out=W)
        else:
            rb.rapid_sgd_step(master, out.dW, lr, w_out=W)
    torch.cuda.synchronize()
    summary = dict(reward_behaviour=reward_mu, reward_final_is_estimate=_is_reward(w, W, logp_b))
    return log, summary, W


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--inner-steps", type=int, default=8)
    ap.add_argument("--lr", type=float, default=None, help="default 0.02 for sgd, 2e-4 for adamw")
    ap.add_argument("--optimizer", default="sgd", choices=["sgd", "adamw"])
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--logits-cache", action="store_true", help="bf16 only: keep the forward's ratios for the backward")
    args = ap.parse_args()
    rb.load()
    spec = wl.small_spec("bandit", args.dtype, d=256, V=4096, prompts=64, G=8, len_lo=8, len_hi=48, sigma=0.0,
                         reward="bernoulli", tokens_from="cur")
    w = wl.make_workload(spec, seed=0, device="cuda")
    lr = args.lr if args.lr is not None else (0.02 if args.optimizer == "sgd" else 2e-4)
    log, summary, _ = iw_grpg(w, inner_steps=args.inner_steps, lr=lr, logits_cache=args.logits_cache,
                              optimizer=args.optimizer)
    print("step  loss        staleness  clip_frac  max|s|")
    for r in log:
        print(f"{r['step']:4d}  {r['loss']:+.4e}  {r['staleness']:.4f}     {r['clip_fraction']:.3f}      {r['max_abs_s']:.3f}")
    print(f"mean reward of the batch (behaviour policy) {summary['reward_behaviour']:.4f}; "
          f"importance-sampling estimate for the final policy {summary['reward_final_is_estimate']:.4f}")


if __name__ == "__main__":
    main()
