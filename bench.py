#!/usr/bin/env python3
"""Benchmark of the fused importance-weighted group-advantage policy-gradient step on one MI355X.

A step = one rapid_iw_pg_loss_fwd_bwd call (all stages of the hot path) on one synthetic
Qwen2.5-1.5B-shaped mini-batch (d=1536, V=151936, 32 prompts x 8 generations, response length
U[256,2048]) whose inputs, including the stored behaviour log-probs, are resident in HBM.

`value` is timed with opts.logits_cache = 1 and the library's recommended workspace for it (a cache
of 90112 token rows, 32 GiB in all at this shape): the batch is worked through in chunks of whole
groups, the forward of a chunk keeps its rows' scaled probabilities in the cache and the chunk's
dHidden and dW contract them, so 6 d V flop per token are executed and nothing of size tokens x V
outlives a chunk.  Generations of a group whose rewards are all 0 have advantage 0 by Eq. (5) and so
no gradient; the backward leaves them out of its contractions (exactly), and the flop counts
here leave them out as well (`response_tokens_with_gradient`).  Beside it, never as `value`: the same call with a cache that holds the whole batch
at once ("whole", 91 GiB), with the backward that regenerates the logits ("recompute", 8 d V flop
per token), and on the workload's calibrated companion (dense gradients: every generation carries
weight).

Prints ONE JSON line: response tokens/s, the roofline of the dominant kernel (HIP-event timing of
every stage, taken inside the timed region on the stream the kernels run on) and the float64 oracle
timed on this machine's cores on a bounded sample of the same workload.
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
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic_cfg2_qwen1.5b.json")
FWD_BLOCK_ROWS = 16384    # token rows per launch of the forward kernel
BWD_BLOCK_ROWS = 65536    # token rows per launch of the dHidden and dW kernels


def measured_traffic(version, mode, stage):
    """HBM-side bytes per launch of `stage` from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes, as the
    profiling run of this library version wrote them into profiles/ (None if that file is from another
    version of the kernels: a stale figure is worse than none)."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return None, None
    if t.get("rapid_version") != version:
        return None, None
    e = t.get("modes", {}).get(mode, {}).get(stage)
    return (e.get("bytes_per_launch"), t.get("source")) if e else (None, None)


def chunk_rows_of(lengths, G, cap, with_gradient):
    """Host replica of the library's chunking (whole groups in order, each chunk as full as the cache
    allows), for reporting only: the tokens of every chunk, and how many of them carry gradient."""
    chunks, cur, cur_live = [], 0, 0
    for k in range(0, len(lengths), G):
        rows = int(sum(lengths[k:k + G]))
        if cur and cur + rows > cap:
            chunks.append((cur, cur_live))
            cur = cur_live = 0
        cur += rows
        cur_live += int(sum(l for l, g in zip(lengths[k:k + G], with_gradient[k:k + G]) if g))
    chunks.append((cur, cur_live))
    return chunks


def generations_with_gradient(w):
    """Per generation: does its group have a reward that is not 0 (host arithmetic on the workload)."""
    import numpy as np
    rew, gid = w["rewards"].cpu().numpy(), w["group_ids"].cpu().numpy()
    live = np.zeros(int(w["K"]), dtype=bool)
    np.logical_or.at(live, gid, rew != 0)
    return live[gid]


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

    def worst(got, want, axis):     # largest error of an element in units of 3 * 2^-8 of its row's / column's largest magnitude
        return float((np.abs(got - want) / (3 * 2.0 ** -8 * np.abs(want).max(axis=axis, keepdims=True) + 1e-30)).max())
    dH, dW = f64(out.dhidden), f64(out.dW)
    parity = {"loss_rel": abs(out.loss.item() - ref["loss"]) / max(abs(ref["loss"]), 1e-30),
              "dH_rel": rel(dH, ref["dH"]), "dW_rel": rel(dW, ref["dW"]),
              "dH_worst_element_in_units_of_its_bound": worst(dH, ref["dH"], -1),
              "dW_worst_element_in_units_of_its_bound": worst(dW, ref["dW"], 0),
              "seq_logratio_abs": float(np.abs(f64(out.seq_logratio) - ref["seq_logratio"]).max()),
              "grad_log_scale_abs": abs(out.read_diag()["grad_log_scale"] - ref["grad_log_scale"]),
              "tolerances": {"loss_rel": 1e-3, "dH_rel": 2e-2 if spec.dtype == "bf16" else 1e-5,
                             "dW_rel": 2e-2 if spec.dtype == "bf16" else 1e-5, "seq_logratio_abs": 1e-3,
                             "worst_element": 1.0}}
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
                    help="time the workload's calibrated companion instead: same shapes and seed, behaviour weights close "
                         "enough that the generation-level ratios are O(1) (every generation carries gradient, dz is dense)")
    ap.add_argument("--rmsnorm", action="store_true",
                    help="treat the workload's hidden states as the input of a final RMSNorm that the call applies "
                         "on the way in and differentiates on the way out (opts.rms_weight); not the headline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=["chunks", "whole", "recompute"], default="chunks",
                    help="backward of the timed call: 'chunks' = opts.logits_cache 1 with the recommended workspace (a cache "
                         "of 90112 rows, chunks of whole groups, 6 d V flop per token executed); 'whole' = the same with a "
                         "cache for every token of the batch; 'recompute' = logits_cache 0 (logits regenerated, 8 d V)")
    ap.add_argument("--one-mode", action="store_true", help="skip the extra measurements (other modes, calibrated companion)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1")

    import torch

    from paper_2510_03515_amd import binding as rb
    from paper_2510_03515_amd import workloads as wl

    rb.load()   # raises if the HIP library is not built: there is no other path
    torch.cuda.set_device(0)
    base_spec = wl.CONFIGS[args.config]
    spec = wl.calibrated(base_spec) if args.calibrated else base_spec
    fwd_only = spec.fwd_only
    dt_code = rb.DTYPE_BF16 if spec.dtype == "bf16" else rb.DTYPE_F32   # config 0 is the fp32 accuracy path
    N, T, d, V = spec.N, spec.T, spec.d, spec.V

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
        stages = {k: {"ms_per_step": ms / args.steps, "launches_per_step": n / args.steps}
                  for k, (ms, n) in prof.items() if n}
        return dt, stages

    def prepare(sp):
        w = wl.make_workload(sp, seed=0, device="cuda")
        rms = {}
        if args.rmsnorm:
            gen = torch.Generator(device="cuda").manual_seed(1)
            rms = dict(rms_weight=(1.0 + 0.1 * torch.randn(d, device="cuda", generator=gen)).to(torch.bfloat16), rms_eps=1e-6)
        if not sp.fwd_only:
            w["logp_behav"], _ = rb.rapid_logprob_fwd(w["hidden"], w["W_old"], w["tokens"], w["mask"], **rms)
        return w, rms, int(w["mask"].sum().item())

    def fused_mode(w, rms, M, mode):
        """Times rapid_iw_pg_loss_fwd_bwd in one backward mode; None if its workspace does not fit."""
        K = w["K"]
        cache = mode in ("chunks", "whole")
        if cache and spec.dtype != "bf16":
            return None              # the cache is a bf16 mode
        op = rb.OP_IW_PG_FWD_BWD_CACHED if cache else rb.OP_IW_PG_FWD_BWD
        # "whole": sized for the batch's token count, which a trainer knows from its sampler
        need = rb.rapid_workspace_bytes(op, N, T, d, V, K, dt_code, max_tokens=M if mode == "whole" else 0)
        torch.cuda.empty_cache()     # what the workload generator left in torch's allocator counts as free
        free, _ = torch.cuda.mem_get_info()
        if not need or need + (8 << 30) > free:
            return None
        buf = rb.IwPgBuffers(w["hidden"], w["W"], K, workspace_bytes=need)
        dt, stages = timed(lambda: rb.rapid_iw_pg_loss_fwd_bwd(
            w["hidden"], w["W"], w["tokens"], w["mask"], w["logp_behav"], w["rewards"], w["group_ids"], K,
            buffers=buf, optional_outputs=False, logits_cache=cache, max_tokens=M, **rms))
        status = int(buf.dev_status.item())
        ws_gib = buf.workspace.numel() / 2**30
        del buf                      # the workspace goes back before the next mode takes its own
        torch.cuda.empty_cache()
        if status:
            raise SystemExit(f"bench.py: the library reported device status {status} in mode {mode}")
        return dt, stages, ws_gib

    w, rms, M = prepare(spec)
    if fwd_only:
        ws_bytes = rb.rapid_workspace_bytes(rb.OP_LOGPROB_FWD, N, T, d, V, 1, dt_code)
        ws = rb.alloc_workspace(ws_bytes)
        dt, stages = timed(lambda: rb.rapid_logprob_fwd(w["hidden"], w["W"], w["tokens"], w["mask"], workspace=ws, **rms))
        ws_gib = ws_bytes / 2**30
        mode = "forward only"
    else:
        mode = args.mode
        res = fused_mode(w, rms, M, mode)
        if res is None:              # no cache for this dtype, or no room
            mode = "recompute"
            res = fused_mode(w, rms, M, mode)
        dt, stages, ws_gib = res
    torch.cuda.synchronize()

    ms_per_step = dt / args.steps * 1e3
    tok_s = M * args.steps / dt
    # Work one call needs: 2 d V flop per response token for the logits, and 2 d V each for dHidden and dW
    # per token that carries gradient.  A generation whose whole group has reward 0 has advantage 0 (Eq. (5)) and
    # gradient 0 whatever its ratio is; the backward leaves such generations out of its contractions
    # (exactly: their rows are zeros), so they are not counted as work either.
    with_gradient = None if fwd_only else generations_with_gradient(w)
    M_grad = 0 if fwd_only else int(w["lengths"].cpu().numpy()[with_gradient].sum())
    flops_needed = 2.0 * d * V * M + 4.0 * d * V * M_grad
    # the scope table's count: 6 d V per response token (2 d V for the forward-only workload), whatever its reward
    flops_per_call = (2.0 if fwd_only else 6.0) * d * V * M
    executed = {"forward only": 2.0, "chunks": 6.0, "whole": 6.0, "recompute": 8.0}[mode] * d * V

    # the MFMA pipe on its own (no memory traffic), outside the timed region: what the published
    # peak turns into at the clock the chip sustains with integer-valued and with random operands
    tf_int, _ = rb.rapid_mfma_probe(0, 100000)
    tf_rnd, _ = rb.rapid_mfma_probe(1, 100000)

    # Roofline of the dominant kernel.  Every contraction stage does 2 d V algorithmic flop per token, so a
    # stage's rate is 2 d V M / (its time per step); a launch that holds tokens (the launches are made for the
    # padded upper bound, those past the last token return at once) processes M / (live launches) of them.
    lengths = w["lengths"].tolist()
    chunk_tokens = chunk_tokens_grad = cache_rows = None
    if mode == "chunks":
        # the window the library takes from the workspace it was given (host arithmetic, the call's own)
        cache_rows = rb.rapid_logits_cache_rows(N, T, d, V, w["K"], M, int(round(ws_gib * 2**30)))
        chunks = chunk_rows_of(lengths, spec.G, cache_rows, with_gradient.tolist())
        live = {"fwd_lse": sum(-(-r // FWD_BLOCK_ROWS) for r, _ in chunks)}
        live["dh"] = sum(-(-g // BWD_BLOCK_ROWS) for _, g in chunks)
        live["dw"] = sum(1 for _, g in chunks if g)          # one dW launch per chunk
        chunk_tokens = [r for r, _ in chunks]
        chunk_tokens_grad = [g for _, g in chunks]
    else:
        Mb = M_grad if spec.dtype == "bf16" else M     # the backward leaves the rows without gradient out
        live = {"fwd_lse": -(-M // FWD_BLOCK_ROWS), "dz": -(-Mb // FWD_BLOCK_ROWS), "dh": -(-Mb // BWD_BLOCK_ROWS),
                "dw": 1 if mode == "whole" else -(-Mb // BWD_BLOCK_ROWS)}
    gemm_stages = [s for s in ("fwd_lse", "dz", "dh", "dw") if s in stages and (s != "dz" or mode == "recompute")]
    if gemm_stages:
        per_stage = {}
        for st_name in gemm_stages:
            ms = stages[st_name]["ms_per_step"]
            rate = 2.0 * d * V * (M if st_name == "fwd_lse" else M_grad) / (ms * 1e-3) / 1e12
            per_stage[st_name] = {"achieved": rate, "frac": rate * 1e12 / PEAK_BF16_MFMA, "frac_of_probe": rate / tf_rnd,
                                  "ms_per_step": ms, "live_launches_per_step": live.get(st_name),
                                  "avg_live_launch_ms": ms / live[st_name] if live.get(st_name) else None}
        dom = max(gemm_stages, key=lambda s: stages[s]["ms_per_step"])
        traffic, source = (measured_traffic(rb.rapid_version(), mode, dom) if spec.name == "cfg2_qwen1.5b" else (None, None))
        roofline = {"bound": "mfma", "kernel": dom, "achieved": per_stage[dom]["achieved"], "peak": PEAK_BF16_MFMA / 1e12,
                    "unit": "TFLOP/s", "frac": per_stage[dom]["frac"], "frac_of_probe": per_stage[dom]["frac_of_probe"],
                    "traffic": traffic, "traffic_unit": "bytes per live launch (fabric reads + writes)", "traffic_source": source,
                    "avg_launch_ms": per_stage[dom]["avg_live_launch_ms"], "live_launches_per_step": live.get(dom),
                    "tokens_per_launch": M / live[dom] if live.get(dom) else None, "flop_per_token": 2.0 * d * V,
                    "all_contraction_stages": per_stage}
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
                   "T": T, "response_tokens": M, "response_tokens_with_gradient": None if fwd_only else M_grad,
                   "workspace_gib": ws_gib,
                   "call": "rapid_logprob_fwd" if fwd_only else "rapid_iw_pg_loss_fwd_bwd",
                   "backward_mode": mode, "final_rmsnorm": bool(args.rmsnorm), "executed_flop_per_token": executed,
                   "cache_rows": cache_rows, "tokens_per_chunk": chunk_tokens,
                   "tokens_with_gradient_per_chunk": chunk_tokens_grad},
        "frac_bf16_mfma_peak_algorithmic": flops_per_call / (dt / args.steps) / PEAK_BF16_MFMA,
        "frac_of_mfma_probe_algorithmic": flops_per_call / (dt / args.steps) / (tf_rnd * 1e12),
        "frac_bf16_mfma_peak_needed_work": flops_needed / (dt / args.steps) / PEAK_BF16_MFMA,
        "roofline": roofline,
        "stages": stages,
        "mfma_probe": {"unit": "TFLOP/s", "small_integer_operands": tf_int, "random_bf16_operands": tf_rnd,
                       "note": "8 independent 32x32x16 bf16 MFMA chains per wave, 2 waves per SIMD, registers only"},
    }
    if not fwd_only and not args.one_mode:
        def summary(res, m, M_):
            return None if res is None else {
                "backward_mode": m, "value": M_ * args.steps / res[0], "unit": "tokens/s", "ms_per_step": res[0] / args.steps * 1e3,
                "frac_bf16_mfma_peak_algorithmic": flops_per_call / (res[0] / args.steps) / PEAK_BF16_MFMA,
                "workspace_gib": res[2], "executed_flop_per_token": (8.0 if m == "recompute" else 6.0) * d * V,
                "stages_ms_per_step": {k: v["ms_per_step"] for k, v in res[1].items()}}
        # the same call in its other backward modes, timed the same way; reported beside `value`, never as it
        out["other_backward_modes"] = [summary(fused_mode(w, rms, M, m), m, M) for m in ("chunks", "whole", "recompute") if m != mode]
        # and the timed mode on the workload's calibrated companion: dense gradient operands (the regime of the
        # paper's staleness table), which cost this power-limited chip a few per cent of clock
        if not args.calibrated and spec.sigma > 0:
            del w
            torch.cuda.empty_cache()
            wc, rmsc, Mc = prepare(wl.calibrated(base_spec))
            out["calibrated_companion"] = summary(fused_mode(wc, rmsc, Mc, mode), mode, Mc)
            del wc
            torch.cuda.empty_cache()
            w, rms, M = prepare(spec)
    if not args.no_cpu_baseline and not fwd_only and not args.rmsnorm:
        out["cpu_baseline"] = cpu_baseline(w, rb, logits_cache=(mode != "recompute"))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
