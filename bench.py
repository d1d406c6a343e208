#!/usr/bin/env python3
"""Benchmark of the fused importance-weighted group-advantage policy-gradient step on one MI355X.

A step = one rapid_iw_pg_loss_fwd_bwd call (all stages of the hot path) on one synthetic
Qwen2.5-1.5B-shaped mini-batch (d=1536, V=151936, 32 prompts x 8 generations, response length
U[256,2048]) whose inputs, including the stored behaviour log-probs, are resident in HBM.  The call
is timed with opts.logits_cache = 1 (the forward keeps every token row's probability ratios in the
workspace, 93 GiB at this shape with opts.max_tokens = the batch's token count, and the backward
contracts them: 6 d V flop per token executed) and, as a second figure, with the default 0 (27 GiB,
the backward regenerates the logits: 8 d V).
Prints ONE JSON line: response tokens/s, the roofline of the dominant kernel (HIP-event timing of
every stage, taken inside the timed region) and the float64 oracle timed on this machine's cores on
a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_MFMA = 2.5e15   # MI355X dense bf16, FLOP/s
PEAK_HBM = 8.0e12         # B/s
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled (see the profile named in the output), of one full launch:
# 16384 token rows for the two logits kernels, 65536 for dH and dW; keyed by (backward mode, stage)
MEASURED_TRAFFIC_BYTES = {("cache", "fwd_lse"): 11.5e9 + 5.2e9, ("cache", "dh"): 48.3e9 + 0.2e9, ("cache", "dw"): 49.7e9 + 1.0e9,
                          ("recompute", "fwd_lse"): 11.8e9 + 0.2e9, ("recompute", "dz"): 11.5e9 + 5.1e9,
                          ("recompute", "dh"): 51.2e9 + 0.2e9, ("recompute", "dw"): 49.8e9 + 1.0e9}


def cpu_baseline(w, rb, group=2, logits_cache=False):
    """Oracle (float64 numpy, as it stands) on one whole group of the workload at the full d and V: the
    first group whose rewards are not forced (its 8 generations, every token), timed on this machine's
    cores.  The same slice also goes through the library as a call of its own (in the backward mode
    the bench times), and the oracle's outputs, which are there anyway, give a full-size check of
    every output element of that call."""
    import numpy as np
    import torch

    from oracle import rapid_oracle as orc
    spec = w["spec"]
    G = spec.G
    group = group if spec.prompts > group else 0
    n0, n1 = group * G, (group + 1) * G
    Tm = int(w["lengths"][n0:n1].max().item())
    f64 = lambda t: t.float().cpu().numpy().astype(np.float64)
    hid, tok_g, mask_g = w["hidden"][n0:n1, :Tm].contiguous(), w["tokens"][n0:n1, :Tm].contiguous(), w["mask"][n0:n1, :Tm].contiguous()
    lb_g, rew_g = w["logp_behav"][n0:n1, :Tm].contiguous(), w["rewards"][n0:n1].contiguous()
    gid_g = torch.zeros(G, dtype=torch.int32, device=hid.device)
    out = rb.rapid_iw_pg_loss_fwd_bwd(hid, w["W"], tok_g, mask_g, lb_g, rew_g, gid_g, 1, normalized_grads=True,
                                      logits_cache=logits_cache)
    torch.cuda.synchronize()
    H, W = f64(hid), f64(w["W"])
    tok, mask = tok_g.cpu().numpy(), mask_g.cpu().numpy()
    n_tok = int(mask.sum())
    t0 = time.perf_counter()
    ref = orc.iw_pg_loss_fwd_bwd(H, W, tok, mask, f64(lb_g), f64(rew_g), np.zeros(G, np.int64), 1, normalized_grads=True,
                                 row_chunk=512)
    dt = time.perf_counter() - t0
    rel = lambda a, b: float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
    parity = {"loss_rel": abs(out.loss.item() - ref["loss"]) / max(abs(ref["loss"]), 1e-30),
              "dH_rel": rel(f64(out.dhidden), ref["dH"]), "dW_rel": rel(f64(out.dW), ref["dW"]),
              "seq_logratio_abs": float(np.abs(f64(out.seq_logratio) - ref["seq_logratio"]).max()),
              "grad_log_scale_abs": abs(out.read_diag()["grad_log_scale"] - ref["grad_log_scale"]),
              "tolerances": {"loss_rel": 1e-3, "dH_rel": 2e-2 if spec.dtype == "bf16" else 1e-5,
                             "dW_rel": 2e-2 if spec.dtype == "bf16" else 1e-5, "seq_logratio_abs": 1e-3}}
    threads = torch.get_num_threads()
    try:
        import threadpoolctl
        infos = [i for i in threadpoolctl.threadpool_info() if i.get("user_api") == "blas"]
        if infos:
            threads = max(i["num_threads"] for i in infos)
    except Exception:
        pass
    return {"value": n_tok / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"group {group} of the workload, whole ({G} generations, {n_tok} tokens) at full d={spec.d}, "
                      f"V={spec.V}; {dt:.1f} s of float64 numpy",
            "host_cpus": os.cpu_count(), "parity_of_the_library_on_this_sample": parity}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="index into the workload list (2 = headline)")
    ap.add_argument("--calibrated", action="store_true",
                    help="the workload's calibrated companion: same shapes and seed, behaviour weights close enough "
                         "that the generation-level ratios are O(1) (every generation carries gradient, dz is dense)")
    ap.add_argument("--rmsnorm", action="store_true",
                    help="treat the workload's hidden states as the input of a final RMSNorm that the call applies "
                         "on the way in and differentiates on the way out (opts.rms_weight); not the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=["cache", "recompute"], default="cache",
                    help="backward of the timed call: 'cache' = opts.logits_cache 1 (probability ratios kept in the "
                         "workspace, 6 d V flop per token executed), 'recompute' = 0 (logits regenerated, 8 d V)")
    ap.add_argument("--one-mode", action="store_true", help="skip the extra measurement of the other mode")
    ap.add_argument("--workspace-gib", type=float, default=0.0,
                    help="recompute mode: workspace size (0 = the library's recommended size)")
    ap.add_argument("--chunk-rows", type=int, default=0,
                    help="recompute mode: size the workspace for backward chunks of this many rows")
    ap.add_argument("--waves", type=int, default=0, help="4 or 8 waves per contraction workgroup (0 = library default)")
    ap.add_argument("--gi", type=str, default="", help="tile-order blocking fwd,dh,dw (tuning experiment)")
    ap.add_argument("--tune", type=str, default="", help="library tuning keys, key=value[,key=value...] (experiments)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    import torch

    from paper_2510_03515_amd import binding as rb
    from paper_2510_03515_amd import workloads as wl

    rb.load()   # raises if the HIP library is not built: there is no other path
    torch.cuda.set_device(0)
    spec = wl.calibrated(wl.CONFIGS[args.config]) if args.calibrated else wl.CONFIGS[args.config]
    w = wl.make_workload(spec, seed=0, device="cuda")
    N, T, d, V, K = spec.N, spec.T, spec.d, spec.V, w["K"]
    M = int(w["mask"].sum().item())

    if args.waves:
        rb.rapid_set_tuning(2, args.waves)
    if args.gi:
        for key, val in zip((10, 11, 12), args.gi.split(",")):
            rb.rapid_set_tuning(key, int(val))
    if args.tune:
        for kv in args.tune.split(","):
            key, val = kv.split("=")
            rb.rapid_set_tuning(int(key), int(val))
    fwd_only = spec.fwd_only
    dt_code = rb.DTYPE_BF16 if spec.dtype == "bf16" else rb.DTYPE_F32   # config 0 is the fp32 accuracy path
    rms = {}
    if args.rmsnorm:
        gen = torch.Generator(device="cuda").manual_seed(1)
        rms = dict(rms_weight=(1.0 + 0.1 * torch.randn(d, device="cuda", generator=gen)).to(torch.bfloat16), rms_eps=1e-6)

    def timed(step):
        """W warm-up steps, then exactly K steps between two synchronisations, with the library's
        per-stage HIP events recorded on the stream the kernels run on."""
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        rb.rapid_set_tuning(1, 1)
        rb.rapid_profile_read()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        prof = rb.rapid_profile_read()
        rb.rapid_set_tuning(1, 0)
        stages = {k: {"ms_per_step": ms / args.steps, "launches_per_step": n / args.steps,
                      "avg_ms": (ms / n if n else 0.0)} for k, (ms, n) in prof.items() if n}
        return dt, stages

    def fused_mode(cache):
        """Times rapid_iw_pg_loss_fwd_bwd in one backward mode; None if the cache does not fit."""
        if cache and spec.dtype != "bf16":
            return None              # the cache is a bf16 mode
        if cache:
            # the cache is sized for the batch's token count, which a trainer knows from its sampler
            need = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, N, T, d, V, K, dt_code, max_tokens=M)
            torch.cuda.empty_cache()     # what the workload generator left in torch's allocator counts as free
            free, _ = torch.cuda.mem_get_info()
            if not need or need + (8 << 30) > free:
                return None
            ws_bytes = None
        else:
            ws_bytes = int(args.workspace_gib * 2**30) if args.workspace_gib > 0 else None
            if args.chunk_rows:
                mn = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, N, T, d, V, K, dt_code, minimum=True)
                vpad = (V + 255) // 256 * 256
                ldv = vpad + 64 if (vpad // 64) % 2 == 0 else vpad
                ws_bytes = mn + (args.chunk_rows - 256) * ldv * 2
        buf = rb.IwPgBuffers(w["hidden"], w["W"], K, workspace_bytes=ws_bytes, logits_cache=cache, max_tokens=M)
        dt, stages = timed(lambda: rb.rapid_iw_pg_loss_fwd_bwd(
            w["hidden"], w["W"], w["tokens"], w["mask"], w["logp_behav"], w["rewards"], w["group_ids"], K,
            buffers=buf, optional_outputs=False, logits_cache=cache, max_tokens=M, **rms))
        ws_gib = buf.workspace.numel() / 2**30
        del buf                      # the workspace goes back before the other mode takes its own
        torch.cuda.empty_cache()
        return dt, stages, ws_gib

    if fwd_only:
        ws_bytes = rb.rapid_workspace_bytes(rb.OP_LOGPROB_FWD, N, T, d, V, 1, dt_code)
        ws = rb.alloc_workspace(ws_bytes)
        dt, stages = timed(lambda: rb.rapid_logprob_fwd(w["hidden"], w["W"], w["tokens"], w["mask"], workspace=ws, **rms))
        ws_gib = ws_bytes / 2**30
        flops_per_token = 2.0 * d * V
        mode = "forward only"
    else:
        logp_b, _ = rb.rapid_logprob_fwd(w["hidden"], w["W_old"], w["tokens"], w["mask"], **rms)
        w["logp_behav"] = logp_b
        flops_per_token = 6.0 * d * V
        mode = args.mode
        res = fused_mode(mode == "cache")
        if res is None:              # the ratios of every row do not fit beside the workload
            mode = "recompute"
            res = fused_mode(False)
        dt, stages, ws_gib = res
    torch.cuda.synchronize()

    ms_per_step = dt / args.steps * 1e3
    tok_s = M * args.steps / dt

    # roofline of the dominant kernel: algorithmic flop of ONE launch / its average duration.
    # Every contraction kernel does 2*d*V flop per token it processes; a step's tokens are split
    # over the launches of a stage (row blocks), so one launch processes M / (launches that hold
    # tokens) tokens on average.
    gemm_stages = [s for s in ("fwd_lse", "dz", "dh", "dw") if s in stages and stages[s]["launches_per_step"] > 1]
    if gemm_stages:
        dom = max(gemm_stages, key=lambda s: stages[s]["ms_per_step"])
        launches = stages[dom]["launches_per_step"]
        # blocks past the last valid row exit at once: count only launches that had rows
        Mmax_pad = (N * T + 255) // 256 * 256
        chunk_rows = Mmax_pad / launches
        live = max(1, -(-M // int(chunk_rows)))
        tokens_per_launch = M / live
        avg_ms = stages[dom]["ms_per_step"] / live
        achieved = 2.0 * d * V * tokens_per_launch / (avg_ms * 1e-3) / 1e12
        # HBM-side bytes per full launch from rocprofv3 FETCH_SIZE + WRITE_SIZE passes (scaled by a copy
        # kernel of known size); measured on the headline workload only, see profiles/
        traffic = MEASURED_TRAFFIC_BYTES.get((mode, dom)) if spec.name == "cfg2_qwen1.5b" else None
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_MFMA / 1e12,
                    "unit": "TFLOP/s", "frac": achieved / (PEAK_BF16_MFMA / 1e12), "traffic": traffic,
                    "traffic_unit": "bytes per full launch (fabric reads + writes)",
                    "traffic_source": "profiles/bench_cfg2_qwen1.5b_kernel_trace_and_traffic.md",
                    "avg_launch_ms": avg_ms, "live_launches_per_step": live,
                    "tokens_per_launch": tokens_per_launch, "flop_per_token": 2.0 * d * V}
        # the same figure for every contraction stage of the step (each does 2 d V flop per token)
        roofline["all_contraction_stages"] = {
            st: {"achieved": 2.0 * d * V * M / (stages[st]["ms_per_step"] * 1e-3) / 1e12,
                 "frac": 2.0 * d * V * M / (stages[st]["ms_per_step"] * 1e-3) / PEAK_BF16_MFMA,
                 "ms_per_step": stages[st]["ms_per_step"]} for st in gemm_stages}
    else:
        # the fp32 accuracy path (config 0): plain strided contractions with fp64 accumulation on the
        # vector ALUs, four of them per call (logits twice, dHidden, dW); all its launches are one stage
        ms = stages["f32_path"]["ms_per_step"]
        achieved = 8.0 * d * V * M / (ms * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "f32_path", "achieved": achieved, "peak": 78.6, "unit": "TFLOP/s",
                    "frac": achieved / 78.6, "traffic": None, "avg_launch_ms": ms,
                    "note": "fp64 vector peak; the path is an accuracy path and a few launches of tiny size"}

    out = {
        "metric": "response tokens/s for fused IW group-adv PG fwd+bwd; % bf16 MFMA peak",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": spec.name, "d": d, "V": V, "prompts": spec.prompts, "G": spec.G, "N": N,
                   "T": T, "response_tokens": M, "workspace_gib": ws_gib,
                   "call": "rapid_logprob_fwd" if fwd_only else "rapid_iw_pg_loss_fwd_bwd",
                   "backward_mode": mode, "final_rmsnorm": bool(args.rmsnorm),
                   "executed_flop_per_token": (2.0 if fwd_only else 6.0 if mode == "cache" else 8.0) * d * V},
        "frac_bf16_mfma_peak_algorithmic": flops_per_token * tok_s / PEAK_BF16_MFMA,
        "roofline": roofline,
        "stages": stages,
    }
    # the MFMA pipe on its own (no memory traffic), outside the timed region: what the published
    # peak turns into at the clock the chip sustains with integer-valued and with random operands
    tf_int, _ = rb.rapid_mfma_probe(0, 100000)
    tf_rnd, _ = rb.rapid_mfma_probe(1, 100000)
    out["mfma_probe"] = {"unit": "TFLOP/s", "small_integer_operands": tf_int, "random_bf16_operands": tf_rnd,
                         "note": "8 independent 32x32x16 bf16 MFMA chains per wave, 2 waves per SIMD, registers only"}
    # the same call in its other backward mode, timed the same way; reported beside `value`, never as it
    if not fwd_only and not args.one_mode:
        other = "recompute" if mode == "cache" else "cache"
        res = fused_mode(other == "cache")
        out["other_backward_mode"] = None if res is None else {
            "backward_mode": other, "value": M * args.steps / res[0], "unit": "tokens/s",
            "ms_per_step": res[0] / args.steps * 1e3,
            "frac_bf16_mfma_peak_algorithmic": flops_per_token * M * args.steps / res[0] / PEAK_BF16_MFMA,
            "workspace_gib": res[2], "executed_flop_per_token": (6.0 if other == "cache" else 8.0) * d * V,
            "stages_ms_per_step": {k: v["ms_per_step"] for k, v in res[1].items()}}
    if not args.no_cpu_baseline and not fwd_only and not args.rmsnorm:
        out["cpu_baseline"] = cpu_baseline(w, rb, logits_cache=(mode == "cache"))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
