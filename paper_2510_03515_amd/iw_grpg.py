"""Inner loop of RAPID (Alg. 1, procedure IW-GRPG) on a synthetic bandit: H off-policy updates of
the LM head on ONE inference batch.

The batch (hidden states, sampled tokens, rewards, stored behaviour log-probs) is fixed, as it is
between two inference phases of the paper's loop; every step calls rapid_iw_pg_loss_fwd_bwd with
the current W against the behaviour log-probs taken with the initial W, then takes one gradient
step (rapid_sgd_step).  Step 1 is on-policy (all ratios exactly 1); the staleness of Sec. 4.3
(mean |log clipped weight|) and the clip proportion grow with the step index, the trend of the
paper's inner-step study.  Everything numeric runs in the library; this module only sequences calls.

    python -m paper_2510_03515_amd.iw_grpg [--steps 8] [--lr 0.01]
"""
from __future__ import annotations

import argparse

import torch

from . import binding as rb
from . import workloads as wl


def iw_grpg(w, steps=8, lr=0.01, eta=2.0, coef_mode=1):
    """Runs `steps` IW-GRPG updates on the workload dict `w` (device tensors, see workloads.py) with
    behaviour policy W (the batch is sampled from it: build the workload with sigma = 0 and
    tokens_from = "cur").  Returns (per-step log, final weights in the workload dtype).

    coef_mode 1 (clipped outer weight) is the default here: with the unclipped ratio of coef_mode 0
    a few generations whose ratio has grown dominate every later step."""
    W = w["W"].clone()
    master = W.float().contiguous()
    K = w["K"]
    logp_b, _ = rb.rapid_logprob_fwd(w["hidden"], W, w["tokens"], w["mask"])   # log mu, stored at "inference"
    buf = rb.IwPgBuffers(w["hidden"], W, K)
    log = []
    for h in range(steps):
        out = rb.rapid_iw_pg_loss_fwd_bwd(w["hidden"], W, w["tokens"], w["mask"], logp_b, w["rewards"],
                                          w["group_ids"], K, buffers=buf, eta=eta, coef_mode=coef_mode)
        dg = out.read_diag()
        s = out.seq_logratio.double()
        rho = torch.exp(s)
        log.append(dict(step=h + 1, loss=out.loss.item(), staleness=dg["mean_abs_log_w"],
                        clip_fraction=dg["n_clipped"] / dg["n_sequences"], max_abs_s=dg["max_abs_s"],
                        # self-normalised importance-sampling estimate of the current policy's reward
                        is_reward=(rho * w["rewards"].double()).sum().item() / rho.sum().item()))
        rb.rapid_sgd_step(master, out.dW, lr, w_out=W)
    torch.cuda.synchronize()
    return log, W


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--dtype", default="bf16", choices=["bf16", "f32"])
    args = ap.parse_args()
    rb.load()
    spec = wl.small_spec("bandit", args.dtype, d=256, V=4096, prompts=32, G=8, len_lo=8, len_hi=48, sigma=0.0,
                         reward="bernoulli", tokens_from="cur")
    w = wl.make_workload(spec, seed=0, device="cuda")
    log, _ = iw_grpg(w, steps=args.steps, lr=args.lr)
    print("step  loss        staleness  clip_frac  max|s|   IS-reward")
    for r in log:
        print(f"{r['step']:4d}  {r['loss']:+.4e}  {r['staleness']:.4f}     {r['clip_fraction']:.3f}      "
              f"{r['max_abs_s']:.3f}   {r['is_reward']:.4f}")


if __name__ == "__main__":
    main()
