"""Full-size parity of the Qwen2.5-shaped workloads (configs 1, 2, 3; config 2 is the launch
configuration bench.py times: d=1536, V=151936, 256 generations, ~300k response tokens,
recommended workspace), on sampled outputs the oracle can compute one by one and on properties that
hold at any size, in both backward modes; one whole group of each of them as a call of its own, every
output element against the oracle.  Also the forward-only behaviour pass of config 4: sampled rows of
the full batch, and its first 8 sequences position by position."""
import math

import numpy as np
import pytest
import torch

import parity_bounds as pb
from oracle import rapid_oracle as orc
from paper_2510_03515_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rb():
    from paper_2510_03515_amd import binding
    binding.load()
    return binding


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _row_oracle(w, W64, n, t):
    """Oracle log-prob / lse of one position: the slice [n:n+1, t:t+1] of the batch."""
    lp, lse = orc.logprob(_f64(w["hidden"][n:n + 1, t:t + 1]), W64, w["tokens"][n:n + 1, t:t + 1].cpu().numpy(),
                          np.ones((1, 1), np.uint8))
    return lp[0, 0], lse[0, 0]


def _fp64_forward_leg(w, row_chunk=4096):
    """Third leg for the sizes the CPU oracle cannot sweep: log-sum-exp and sampled-token log-prob of
    EVERY valid position from torch's own float64 matmul and logsumexp on the GPU (library routines;
    nothing of the HIP path).  It is itself checked against the oracle wherever the oracle is run
    below, to 1e-9.  Returns (idx [M] flat positions, lse [M], logp [M]) as float64 GPU tensors."""
    N, T, d = w["hidden"].shape
    idx = torch.nonzero(w["mask"].view(-1), as_tuple=False).view(-1)
    Hf = w["hidden"].view(N * T, d)
    W64 = w["W"].double()
    tok = w["tokens"].view(-1)[idx].long()
    lse = torch.empty(idx.numel(), dtype=torch.float64, device="cuda")
    zy = torch.empty_like(lse)
    for s0 in range(0, idx.numel(), row_chunk):
        z = Hf[idx[s0:s0 + row_chunk]].double() @ W64
        lse[s0:s0 + row_chunk] = torch.logsumexp(z, dim=1)
        zy[s0:s0 + row_chunk] = z.gather(1, tok[s0:s0 + row_chunk, None]).squeeze(1)
        del z
    return idx, lse, zy - lse


@pytest.mark.parametrize("cfg,cache,cal", [(2, False, False), (2, "chunks", False), (2, "whole", True), (2, False, True),
                                           (2, "chunks", True), (1, False, False), (1, "chunks", False), (3, False, False),
                                           (3, "chunks", True)])
def test_full_size_sampled_parity(rb, cfg, cache, cal):
    """cal: the calibrated companion of the workload (same shapes and seed, behaviour weights close
    enough that the generation-level ratios are O(1) and a few per cent clip: the paper's regime,
    where every generation carries gradient and dz is dense).  cache: False = the backward that regenerates
    the logits; "chunks" = logits_cache with the recommended workspace (a cache of 90112 rows, the batch
    in chunks of whole groups: the launch configuration bench.py times); "whole" = logits_cache with a
    cache that holds every token of the batch at once.

    No expected value below comes from the library: per-position and per-generation references are
    the CPU oracle's; what needs every row of the batch (advantages, coefficients, loss, dW columns)
    is built by the oracle's own functions from the float64 leg above, which the oracle pins on the
    sampled positions and on whole generations (the two shortest and the longest)."""
    spec = wl.calibrated(wl.CONFIGS[cfg]) if cal else wl.CONFIGS[cfg]
    print("generating", spec.name, f"logits_cache ({cache})" if cache else "", flush=True)
    w = wl.make_workload(spec, seed=0, device="cuda")
    N, T, K = spec.N, spec.T, w["K"]
    n_tok = int(w["mask"].sum().item())
    logp_b, _ = rb.rapid_logprob_fwd(w["hidden"], w["W_old"], w["tokens"], w["mask"])
    buf = rb.IwPgBuffers(w["hidden"], w["W"], K, logits_cache=bool(cache), max_tokens=n_tok if cache == "whole" else 0)
    print("fused call, workspace %.1f GiB" % (buf.workspace.numel() / 2**30), flush=True)
    out = rb.rapid_iw_pg_loss_fwd_bwd(w["hidden"], w["W"], w["tokens"], w["mask"], logp_b, w["rewards"],
                                      w["group_ids"], K, buffers=buf, normalized_grads=True, logits_cache=bool(cache),
                                      max_tokens=n_tok)
    lp_cur2, lse_gpu = rb.rapid_logprob_fwd(w["hidden"], w["W"], w["tokens"], w["mask"], want_lse=True)
    torch.cuda.synchronize()
    assert out.dev_status.item() == 0
    assert torch.equal(lp_cur2, out.logp_cur)          # same bits from both entry points
    mask = w["mask"].cpu().numpy()
    lengths = mask.sum(1)
    W64 = _f64(w["W"])
    rng = np.random.default_rng(0)

    # (a) bit-exact integer work
    seq_len, cu, row_index = rb.rapid_compaction(w["mask"])
    o_len, o_cu, o_rows = orc.compaction(mask)
    M = int(o_cu[-1])
    assert np.array_equal(seq_len.cpu().numpy(), o_len) and np.array_equal(cu.cpu().numpy(), o_cu)
    assert np.array_equal(row_index.cpu().numpy()[:M], o_rows)
    dg = out.read_diag()
    assert dg["n_tokens"] == M and dg["n_sequences"] == N

    print("float64 leg", flush=True)
    idx, lse_leg, logp_leg = _fp64_forward_leg(w)
    assert np.array_equal(idx.cpu().numpy(), o_rows)
    lse_leg_nt = np.zeros(N * T); lse_leg_nt[o_rows] = lse_leg.cpu().numpy(); lse_leg_nt = lse_leg_nt.reshape(N, T)
    lp_leg_nt = np.zeros(N * T); lp_leg_nt[o_rows] = logp_leg.cpu().numpy(); lp_leg_nt = lp_leg_nt.reshape(N, T)

    # (b) sampled log-probs against the oracle, position by position (incl. first/last rows and tiles);
    # then every position against the leg the oracle has just pinned
    print("sampled logp", flush=True)
    pos = [(0, 0), (N - 1, int(lengths[N - 1]) - 1)]
    for _ in range(30):
        n = int(rng.integers(0, N))
        pos.append((n, int(rng.integers(0, lengths[n]))))
    lp_gpu, lse_g = _f64(out.logp_cur), _f64(lse_gpu)
    for n, t in pos:
        lp, lse = _row_oracle(w, W64, n, t)
        assert abs(lp_gpu[n, t] - lp) <= 2e-5, (n, t)
        assert abs(lse_g[n, t] - lse) <= 2e-5, (n, t)
        assert abs(lp_leg_nt[n, t] - lp) <= 1e-9 and abs(lse_leg_nt[n, t] - lse) <= 1e-9, (n, t)
    assert np.all(lp_gpu[mask == 0] == 0.0)
    assert np.abs(lp_gpu - lp_leg_nt).max() <= 2e-5 and np.abs(lse_g - lse_leg_nt).max() <= 2e-5

    # (c) generation-level log ratios: the two shortest and the longest generation whole by the oracle
    # (the error of a sum over tokens grows with the length), all of them against the leg
    print("sequence ratios", flush=True)
    s_gpu = _f64(out.seq_logratio)
    lb64 = _f64(logp_b)
    s_leg = orc.seq_logratio(lp_leg_nt, lb64, mask)
    order = np.argsort(lengths)
    for n in list(order[:2]) + [order[-1]]:
        L = int(lengths[n])
        lp, _ = orc.logprob(_f64(w["hidden"][n:n + 1, :L]), W64, w["tokens"][n:n + 1, :L].cpu().numpy(),
                            np.ones((1, L), np.uint8))
        s = orc.seq_logratio(lp, lb64[n:n + 1, :L], np.ones((1, L), np.uint8))[0]
        assert abs(s_gpu[n] - s) <= 1e-3, (n, L, s_gpu[n], s)
        assert abs(s_leg[n] - s) <= 1e-7, (n, L, s_leg[n], s)
    assert np.abs(s_gpu - s_leg).max() <= 1e-3
    assert np.abs(_f64(out.tok_logratio) - orc.token_logratio(lp_leg_nt, lb64, mask)).max() <= 4e-5

    # (d) advantages, coefficients, loss by the oracle from the reference ratios
    R, gid = _f64(w["rewards"]), w["group_ids"].cpu().numpy()
    ga = orc.group_advantage(R, gid, K, s=s_leg, eta=2.0)
    assert np.abs(_f64(out.adv) - ga["adv"]).max() <= 1e-3
    if spec.force_edge_groups:
        assert np.all(_f64(out.adv)[gid == 0] == 0.0)                   # forced all-0 group
    g_ref, loss_ref, lam = orc.coefficients(s_leg, ga["adv"], 2.0, 0, 1.0, normalized=True)
    assert abs(dg["grad_log_scale"] - lam) <= 1e-3
    assert abs(out.loss.item() - loss_ref) <= 1e-3 * abs(loss_ref)
    near = int((np.abs(s_leg - math.log(2.0)) < 1e-3).sum())
    assert abs(dg["n_clipped"] - int((s_leg > math.log(2.0)).sum())) <= near
    if cal:       # the regime the companion is made for
        assert np.abs(s_leg).max() < 6.0 and 0.01 * N <= dg["n_clipped"] <= 0.25 * N
        assert abs(lam) < 12.0 and (np.abs(g_ref) > 1e-3).sum() > N // 4      # most generations carry gradient

    # (e) sampled dHidden rows, every element: g_n (W[:, y] - W p) with p from the oracle for that row
    print("sampled dH rows", flush=True)
    live = np.argsort(-np.abs(g_ref))[:4]        # generations that carry the gradient
    dH = out.dhidden
    for n in live:
        for t in {0, int(lengths[n]) - 1, int(rng.integers(0, lengths[n]))}:
            dh_ref, _ = orc.backward(_f64(w["hidden"][n:n + 1, t:t + 1]), W64,
                                     w["tokens"][n:n + 1, t:t + 1].cpu().numpy(), np.ones((1, 1), np.uint8),
                                     np.array([g_ref[n]]))
            got = _f64(dH[n, t])
            assert np.linalg.norm(got - dh_ref[0, 0]) <= 2e-2 * np.linalg.norm(dh_ref[0, 0]), (n, t)
            pb.assert_dhidden_close(got, dh_ref[0, 0])
    n_pad = int(np.argmin(lengths))
    assert torch.all(dH[n_pad, int(lengths[n_pad]):] == 0)              # masked rows are zero

    # (f) dW: every row sums to zero over the vocabulary (softmax identity, any size); sampled columns,
    # every element, against sum_m g_m (1[y_m = v] - exp(h_m . W_v - lse_m)) h_m with the reference lse:
    # the first, the last, random ones, and columns of tokens the largest-coefficient generations sampled
    # (those hold a one-hot term)
    print("dW properties", flush=True)
    dW = out.dW
    rowsum = dW.double().sum(1).cpu().numpy()
    scale = dW.double().abs().sum(1).cpu().numpy()
    assert np.abs(rowsum).max() <= 2e-3 * scale.max()
    Hv = w["hidden"].view(N * T, -1)[idx].double()                      # [M, d] on the GPU, fp64
    g_rows = torch.tensor(g_ref, device="cuda")[idx // T]
    tok_rows = w["tokens"].view(-1)[idx]
    hot = [int(w["tokens"][int(n), t].item()) for n in live[:2] for t in (0, int(lengths[n]) // 2)]
    for v in [0, 5, spec.V - 1] + hot + [int(x) for x in rng.integers(0, spec.V, 3)]:
        z = Hv @ w["W"][:, v].double()
        coef = g_rows * ((tok_rows == v).double() - torch.exp(z - lse_leg))
        col = (Hv * coef[:, None]).sum(0).cpu().numpy()
        got = _f64(dW[:, v])
        assert np.linalg.norm(got - col) <= 2e-2 * max(np.linalg.norm(col), 1e-30), v
        pb.assert_dw_close(got[:, None], col[:, None])


@pytest.mark.parametrize("variant,cache", [("grpo", True), ("dapo", False)])
def test_full_size_clip_pg_sampled(rb, variant, cache):
    """The loss step of a baseline (Sec. 4.1) at full size: config 1's shapes (d=896, V=151936, 128 generations,
    ~76k response tokens), GRPO with its KL term against a reference policy through the chunked cache, DAPO through
    the backward that regenerates the logits.  References as in test_full_size_sampled_parity: the float64 leg for
    the current log-probs (pinned by the oracle on sampled positions), then the oracle's own advantage and
    token-coefficient functions; sampled dHidden rows and dW columns, every element."""
    spec = wl.CONFIGS[1]
    print("generating", spec.name, variant, flush=True)
    w = wl.make_workload(spec, seed=0, device="cuda")
    N, T, K, V = spec.N, spec.T, w["K"], spec.V
    gen = torch.Generator(device="cuda").manual_seed(11)
    W_ref = (w["W"].float() + 0.004 * torch.randn(w["W"].shape, device="cuda", generator=gen)).to(torch.bfloat16)
    lp_old, _ = rb.rapid_logprob_fwd(w["hidden"], w["W_old"], w["tokens"], w["mask"])
    lp_ref, _ = rb.rapid_logprob_fwd(w["hidden"], W_ref, w["tokens"], w["mask"])
    del W_ref
    out = rb.rapid_clip_pg_loss_fwd_bwd(w["hidden"], w["W"], w["tokens"], w["mask"], lp_old, lp_ref, w["rewards"], w["group_ids"], K,
                                        variant=variant, logits_cache=cache)
    torch.cuda.synchronize()
    assert out.dev_status.item() == 0
    mask = w["mask"].cpu().numpy()
    lengths = mask.sum(1)
    W64 = _f64(w["W"])
    rng = np.random.default_rng(1)
    print("float64 leg", flush=True)
    idx, lse_leg, logp_leg = _fp64_forward_leg(w)
    lp_leg_nt = np.zeros(N * T); lp_leg_nt[idx.cpu().numpy()] = logp_leg.cpu().numpy(); lp_leg_nt = lp_leg_nt.reshape(N, T)
    lp_gpu = _f64(out.logp_cur)
    for _ in range(12):
        n = int(rng.integers(0, N)); t = int(rng.integers(0, lengths[n]))
        lp, _ = _row_oracle(w, W64, n, t)
        assert abs(lp_leg_nt[n, t] - lp) <= 1e-9 and abs(lp_gpu[n, t] - lp) <= 2e-5, (n, t)
    assert np.abs(lp_gpu - lp_leg_nt).max() <= 2e-5
    # advantages, per-token coefficients, loss and diagnostics by the oracle
    o = rb.clip_pg_default_opts(variant)
    R, gid = _f64(w["rewards"]), w["group_ids"].cpu().numpy()
    adv = orc.normalized_group_advantage(R, gid, K, adv_eps=o.adv_eps, std_ddof=o.std_ddof)["adv"]
    assert np.abs(_f64(out.adv) - adv).max() <= 1e-3 * max(np.abs(adv).max(), 1.0)
    ckw = dict(eps_low=o.eps_low, eps_high=o.eps_high, kl_beta=o.kl_beta, norm_mode=o.norm_mode)
    old64, ref64 = _f64(lp_old), _f64(lp_ref)
    print("token coefficients", flush=True)
    g_ref, loss_ref, info = orc.clipped_token_coefficients(lp_leg_nt, old64, ref64, mask, adv, **ckw)
    assert abs(out.loss.item() - loss_ref) <= 1e-3 * abs(loss_ref)
    dg = rb.read_clip_diag(out)
    assert dg["n_tokens"] == int(mask.sum()) and dg["n_sequences"] == N
    r = np.exp(lp_leg_nt - old64)[mask != 0]
    near = int(((np.abs(r - (1 - o.eps_low)) < 1e-5) | (np.abs(r - (1 + o.eps_high)) < 1e-5)).sum())
    assert abs(dg["n_clipped"] - round(info["clip_fraction"] * dg["n_tokens"])) <= near
    assert 0.0 < info["clip_fraction"] < 0.9
    assert abs(dg["mean_kl"] - info["mean_kl"]) <= 1e-5 + 1e-3 * info["mean_kl"]
    tok_slack, col_slack = pb.token_coefficient_slack(
        lambda lp: orc.clipped_token_coefficients(lp, old64, ref64, mask, adv, **ckw)[0], lp_leg_nt, mask, w["tokens"].cpu().numpy(), V)
    # sampled dHidden rows, every element
    print("sampled dH rows", flush=True)
    dH = out.dhidden
    cand = np.argwhere((mask != 0) & (g_ref != 0))
    for n, t in [tuple(cand[0]), tuple(cand[-1])] + [tuple(cand[i]) for i in rng.integers(0, len(cand), 6)]:
        dh_ref, _ = orc.backward(_f64(w["hidden"][n:n + 1, t:t + 1]), W64, w["tokens"][n:n + 1, t:t + 1].cpu().numpy(),
                                 np.ones((1, 1), np.uint8), np.array([[g_ref[n, t]]]))
        got = _f64(dH[n, t])
        assert np.linalg.norm(got - dh_ref[0, 0]) <= 2e-2 * np.linalg.norm(dh_ref[0, 0]), (n, t)
        pb.assert_dhidden_close(got, dh_ref[0, 0], rel=pb.REL["bf16"] + tok_slack[n, t])
    assert torch.all(dH[w["mask"] == 0] == 0)
    if variant == "dapo":      # without a KL term, tokens whose ratio left the clip range the way their advantage pushes get nothing
        dead = np.argwhere((mask != 0) & (g_ref == 0))
        for n, t in dead[:: max(1, len(dead) // 8)][:8]:
            assert not dH[int(n), int(t)].any()
    # sampled dW columns, every element
    print("sampled dW columns", flush=True)
    dW = out.dW
    Hv = w["hidden"].view(N * T, -1)[idx].double()
    g_rows = torch.tensor(g_ref.reshape(-1), device="cuda")[idx]
    tok_rows = w["tokens"].view(-1)[idx]
    hot = [int(w["tokens"][int(n), int(t)].item()) for n, t in cand[:: max(1, len(cand) // 3)][:3]]
    for v in [0, V - 1] + hot + [int(x) for x in rng.integers(0, V, 3)]:
        z = Hv @ w["W"][:, v].double()
        coef = g_rows * ((tok_rows == v).double() - torch.exp(z - lse_leg))
        col = (Hv * coef[:, None]).sum(0).cpu().numpy()
        got = _f64(dW[:, v])
        assert np.linalg.norm(got - col) <= 2e-2 * max(np.linalg.norm(col), 1e-30), v
        pb.assert_dw_close(got[:, None], col[:, None], rel=pb.REL["bf16"] + col_slack[v])


def test_config4_behaviour_pass_sampled(rb):
    spec = wl.CONFIGS[4]
    print("generating", spec.name, flush=True)
    w = wl.make_workload(spec, seed=0, device="cuda")
    lp, lse = rb.rapid_logprob_fwd(w["hidden"], w["W"], w["tokens"], w["mask"], want_lse=True)
    torch.cuda.synchronize()
    W64 = _f64(w["W"])
    rng = np.random.default_rng(1)
    lp_g, lse_g = _f64(lp), _f64(lse)
    for n, t in [(0, 0), (spec.N - 1, spec.T - 1)] + [(int(rng.integers(0, spec.N)), int(rng.integers(0, spec.T)))
                                                       for _ in range(20)]:
        r_lp, r_lse = _row_oracle(w, W64, n, t)
        assert abs(lp_g[n, t] - r_lp) <= 2e-5 and abs(lse_g[n, t] - r_lse) <= 2e-5, (n, t)
    assert np.isfinite(lp_g).all() and (lp_g < 0).all()
    # the first 8 sequences as a call of their own, every position against the oracle; a position's
    # result does not depend on what else is in the batch, so the full batch holds the same bits
    print("first 8 sequences, every position", flush=True)
    n8 = 8
    lp8, lse8 = rb.rapid_logprob_fwd(w["hidden"][:n8].contiguous(), w["W"], w["tokens"][:n8].contiguous(),
                                     w["mask"][:n8].contiguous(), want_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(lp8, lp[:n8]) and torch.equal(lse8, lse[:n8])
    for n in range(n8):
        r_lp, r_lse = orc.logprob(_f64(w["hidden"][n:n + 1]), W64, w["tokens"][n:n + 1].cpu().numpy(),
                                  w["mask"][n:n + 1].cpu().numpy(), row_chunk=512)
        assert np.abs(lp_g[n] - r_lp[0]).max() <= 2e-5 and np.abs(lse_g[n] - r_lse[0]).max() <= 2e-5, n
        print("  sequence", n, "ok", flush=True)


def test_one_chunk_twice_bitwise(rb):
    """Every reduction has a fixed order and the hand-scheduled main loops carry no race: two calls on
    a full 65536-row block of the headline shape give identical bits, in both backward modes."""
    spec = wl.CONFIGS[5]
    print("generating", spec.name, flush=True)
    w = wl.make_workload(spec, seed=0, device="cuda")
    logp_b, _ = rb.rapid_logprob_fwd(w["hidden"], w["W_old"], w["tokens"], w["mask"])
    for cache in (False, True):
        buf = rb.IwPgBuffers(w["hidden"], w["W"], w["K"], logits_cache=cache)
        outs = []
        for rep in range(2):
            out = rb.rapid_iw_pg_loss_fwd_bwd(w["hidden"], w["W"], w["tokens"], w["mask"], logp_b, w["rewards"],
                                              w["group_ids"], w["K"], buffers=buf, normalized_grads=True,
                                              logits_cache=cache)
            torch.cuda.synchronize()
            outs.append({k: getattr(out, k).clone() for k in ("loss", "dhidden", "dW", "logp_cur")})
            out.dW.zero_(); out.dhidden.zero_()
        for k in outs[0]:
            assert torch.equal(outs[0][k], outs[1][k]), (cache, k)
        assert torch.isfinite(outs[0]["dW"]).all() and outs[0]["dW"].abs().max() > 0
        del buf


def _slice_group(spec, w, cfg):
    """The group the slice tests run: the first whose rewards are not forced at config 2, the one with
    the fewest tokens elsewhere (config 3's groups hold 16 generations of up to 4096 tokens: the
    oracle's float64 sweep of the smallest still takes a minute or two)."""
    if cfg == 2:
        return 2
    per_group = w["lengths"].view(spec.prompts, spec.G).sum(1)
    return int(torch.argmin(per_group).item())


@pytest.mark.parametrize("cfg", [1, 2, 3])
def test_one_group_every_element(rb, cfg):
    """One whole group of the workload at the full d and V as a call of its own (config 1: 8 generations,
    ~4k tokens; config 2: 8 generations, ~8k tokens; config 3: 16 generations, ~30k tokens): every element
    of loss, log-probs, ratios, advantages, dHidden and dW against the oracle, in both backward modes;
    the gradients by norm and element by element.  The same generations' log-probs and ratios inside
    the full batch are the slice call's bits (a position does not depend on the rest of the batch)."""
    spec = wl.CONFIGS[cfg]
    print("generating", spec.name, flush=True)
    w = wl.make_workload(spec, seed=0, device="cuda")
    G, grp = spec.G, None
    grp = _slice_group(spec, w, cfg)
    n0, n1 = grp * G, (grp + 1) * G
    Tm = int(w["lengths"][n0:n1].max().item())
    hid, tok, mask = (w[k][n0:n1, :Tm].contiguous() for k in ("hidden", "tokens", "mask"))
    rew = w["rewards"][n0:n1].contiguous()
    gid = torch.zeros(G, dtype=torch.int32, device="cuda")
    logp_b, _ = rb.rapid_logprob_fwd(hid, w["W_old"], tok, mask)
    outs = [rb.rapid_iw_pg_loss_fwd_bwd(hid, w["W"], tok, mask, logp_b, rew, gid, 1, normalized_grads=True,
                                        logits_cache=cache) for cache in (False, True)]
    lp_full, _ = rb.rapid_logprob_fwd(w["hidden"], w["W"], w["tokens"], w["mask"])
    torch.cuda.synchronize()
    assert torch.equal(lp_full[n0:n1, :Tm], outs[0].logp_cur)
    n_tok = int(mask.sum().item())
    print(f"oracle: group {grp}, {G} generations, {n_tok} tokens", flush=True)
    H64, W64 = _f64(hid), _f64(w["W"])
    tok_c, mask_c, lb64, R64 = tok.cpu().numpy(), mask.cpu().numpy(), _f64(logp_b), _f64(rew)
    # the oracle's steps in their order, generation by generation where a step is per generation, so that
    # the minutes of float64 work print their progress
    lp_ref = np.zeros((G, Tm))
    for n in range(G):
        lp_ref[n:n + 1], _ = orc.logprob(H64[n:n + 1], W64, tok_c[n:n + 1], mask_c[n:n + 1], row_chunk=512)
        print("  forward", n, flush=True)
    s_ref = orc.seq_logratio(lp_ref, lb64, mask_c)
    ga = orc.group_advantage(R64, np.zeros(G, np.int64), 1, s=s_ref, eta=2.0)
    g_ref, loss_ref, lam = orc.coefficients(s_ref, ga["adv"], 2.0, 0, 1.0, normalized=True)
    dH_ref = np.zeros((G, Tm, spec.d))
    dW_ref = np.zeros((spec.d, spec.V))
    for n in range(G):
        dh, dw = orc.backward(H64[n:n + 1], W64, tok_c[n:n + 1], mask_c[n:n + 1], g_ref[n:n + 1], row_chunk=512)
        dH_ref[n] = dh[0]
        dW_ref += dw
        print("  backward", n, flush=True)
    rel = lambda a, b: np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)
    for out in outs:
        assert out.dev_status.item() == 0
        assert np.abs(_f64(out.logp_cur) - lp_ref).max() <= 2e-5
        assert np.abs(_f64(out.seq_logratio) - s_ref).max() <= 1e-3
        assert np.abs(_f64(out.adv) - ga["adv"]).max() <= 1e-3
        assert abs(out.loss.item() - loss_ref) <= 1e-3 * abs(loss_ref)
        assert abs(out.read_diag()["grad_log_scale"] - lam) <= 1e-3
        assert out.read_diag()["n_tokens"] == n_tok
        dH, dW = _f64(out.dhidden), _f64(out.dW)
        assert rel(dH, dH_ref) <= 2e-2 and rel(dW, dW_ref) <= 2e-2
        pb.assert_dhidden_close(dH, dH_ref)
        pb.assert_dw_close(dW, dW_ref)
        assert np.all(dH[mask_c == 0] == 0.0)
        print("  mode ok", flush=True)


def test_config2_one_group_with_final_rmsnorm(rb):
    """The same kind of slice (group 3 of the headline workload, full d and V) with the hidden states
    taken as the input of a final RMSNorm: every element of log-probs, loss, dW, dL/dx and dL/dweight
    against the oracle (whose normalised state is a bf16 tensor, as a bf16 model's is)."""
    spec = wl.CONFIGS[2]
    print("generating", spec.name, flush=True)
    w = wl.make_workload(spec, seed=0, device="cuda")
    G, grp = spec.G, 3
    n0, n1 = grp * G, (grp + 1) * G
    Tm = int(w["lengths"][n0:n1].max().item())
    gen = torch.Generator(device="cuda").manual_seed(2)
    scale = 0.5 + 2.0 * torch.rand((G, Tm, 1), device="cuda", generator=gen)
    hid = (w["hidden"][n0:n1, :Tm].float() * scale).to(torch.bfloat16).contiguous()
    tok, mask = (w[k][n0:n1, :Tm].contiguous() for k in ("tokens", "mask"))
    wgt = (1.0 + 0.1 * torch.randn(spec.d, device="cuda", generator=gen)).to(torch.bfloat16)
    rew = w["rewards"][n0:n1].contiguous()
    gid = torch.zeros(G, dtype=torch.int32, device="cuda")
    eps = float(np.float32(1e-6))          # the ABI takes a float: give the oracle the same number
    logp_b, _ = rb.rapid_logprob_fwd(hid, w["W_old"], tok, mask, rms_weight=wgt, rms_eps=eps)
    out = rb.rapid_iw_pg_loss_fwd_bwd(hid, w["W"], tok, mask, logp_b, rew, gid, 1, normalized_grads=True,
                                      logits_cache=True, rms_weight=wgt, rms_eps=eps)
    torch.cuda.synchronize()
    print("oracle", flush=True)
    ref = orc.iw_pg_loss_fwd_bwd(_f64(hid), _f64(w["W"]), tok.cpu().numpy(), mask.cpu().numpy(), _f64(logp_b), _f64(rew),
                                 np.zeros(G, np.int64), 1, normalized_grads=True, row_chunk=512, rms_weight=_f64(wgt),
                                 rms_eps=eps, round_normed_hidden=True)
    rel = lambda a, b: np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)
    assert out.dev_status.item() == 0
    # the kernel takes the bf16 rounding of the normalised state from the same float64 value as the
    # oracle, so the usual tolerances hold
    assert np.abs(_f64(out.logp_cur) - ref["logp_cur"]).max() <= 2e-5
    assert np.abs(_f64(out.seq_logratio) - ref["seq_logratio"]).max() <= 1e-3
    assert abs(out.read_diag()["grad_log_scale"] - ref["grad_log_scale"]) <= 1e-3
    assert abs(out.loss.item() - ref["loss"]) <= 1e-3 * abs(ref["loss"])
    assert rel(_f64(out.dhidden), ref["dH"]) <= 2e-2 and rel(_f64(out.dW), ref["dW"]) <= 2e-2
    pb.assert_dw_close(_f64(out.dW), ref["dW"])
    pb.assert_dhidden_close(_f64(out.dhidden), ref["dH"], rel=2.0 ** -6)   # dL/dh stored in bf16, then through the norm
    assert rel(_f64(out.drms_weight), ref["d_rms_weight"]) <= 2e-2
