"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-side validation and workspace arithmetic behave (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rb():
    from paper_2510_03515_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2510_03515_amd import build
        build.build(verbose=False)
    binding.load()
    return binding


def _declared():
    """Every function declared in include/*.h (rapid.h: the product ABI; rapid_tuning.h: benchmark hooks)."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            src = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(rapid_[a-z_0-9]+)\s*\(", src))
    return sorted(names)


def test_exports_every_declared_symbol(rb):
    lib = rb.load()
    names = _declared()
    assert "rapid_logprob_fwd" in names and "rapid_group_advantage" in names
    assert "rapid_iw_pg_loss_fwd_bwd" in names and len(names) >= 9
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(rb.EXPORTS) == names
    assert rb.rapid_version() >= 1


def test_struct_layouts_match_header(rb):
    assert C.sizeof(rb.IwPgDiag) == 32
    assert C.sizeof(rb.IwPgOpts) == 88 and rb.IwPgOpts.max_tokens.offset == 48 and rb.IwPgOpts.coef_override.offset == 56
    assert rb.IwPgOpts.rms_weight.offset == 64 and rb.IwPgOpts.drms_weight_out.offset == 72 and rb.IwPgOpts.rms_eps.offset == 80
    o = rb.default_opts()
    assert o.eta == 2.0 and o.loss_scale == 1.0 and o.temperature == 1.0
    assert o.coef_mode == 0 and o.baseline_mode == 0 and o.w_layout == rb.W_DV and o.dw_dtype == rb.DTYPE_F32
    assert o.logits_cache == 0 and o.ratio_level == 0 and o.max_tokens == 0 and not o.coef_override
    assert not o.rms_weight and not o.drms_weight_out and abs(o.rms_eps - 1e-6) < 1e-12


def test_clip_pg_structs_and_validation(rb):
    """The baselines' loss step: struct layouts as in the header, the two variants' defaults (GRPO: eps 0.2 / 0.2,
    KL 0.04 as in the paper's Appendix A, per-generation mean; DAPO: eps 0.2 / 0.28, no KL, token mean), and its own
    host checks."""
    lib = rb.load()
    assert C.sizeof(rb.ClipPgOpts) == 56 and rb.ClipPgOpts.max_tokens.offset == 48 and C.sizeof(rb.ClipPgDiag) == 24
    g, dd = rb.clip_pg_default_opts("grpo"), rb.clip_pg_default_opts("dapo")
    assert abs(g.eps_low - 0.2) < 1e-7 and abs(g.eps_high - 0.2) < 1e-7 and abs(g.kl_beta - 0.04) < 1e-8 and g.norm_mode == 0
    assert abs(dd.eps_low - 0.2) < 1e-7 and abs(dd.eps_high - 0.28) < 1e-7 and dd.kl_beta == 0.0 and dd.norm_mode == 1
    assert abs(g.adv_eps - 1e-4) < 1e-10 and g.std_ddof == 0 and g.loss_scale == 1.0 and g.temperature == 1.0
    one = C.c_void_p(256)
    args = lambda o, ref=one: [one, one, one, one, one, ref, one, one, 4, 4, 8, 8, 1, rb.DTYPE_BF16, C.byref(o), one, one, one,
                               None, None, None, None, one, 1 << 30, None]
    assert lib.rapid_clip_pg_loss_fwd_bwd(*args(g, None)) == -1 and b"logp_ref" in lib.rapid_last_error()   # KL without a reference
    g.eps_low = 1.5
    assert lib.rapid_clip_pg_loss_fwd_bwd(*args(g)) == -2
    g = rb.clip_pg_default_opts("grpo"); g.norm_mode = 3
    assert lib.rapid_clip_pg_loss_fwd_bwd(*args(g)) == -3
    g = rb.clip_pg_default_opts("grpo"); g.kl_beta = -1.0
    assert lib.rapid_clip_pg_loss_fwd_bwd(*args(g)) == -2
    assert lib.rapid_clip_pg_loss_fwd_bwd(*[one, one, one, one, one, None, None, one, 4, 4, 8, 8, 1, rb.DTYPE_BF16, C.byref(dd),
                                            one, one, one, None, None, None, None, one, 1 << 30, None]) == -1   # rewards


def test_workspace_sizes(rb):
    args = (256, 2048, 1536, 151936, 32, rb.DTYPE_BF16)
    rec = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, *args)
    mn = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, *args, minimum=True)
    assert 0 < mn < rec < 288 * 2**30
    assert rb.rapid_workspace_bytes(rb.OP_GROUP_ADVANTAGE, *args) == 0
    assert rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, 0, 1, 1, 1, 1, 0) == 0       # invalid shape
    assert rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, 4, 4, 8, 8, 1, 7) == 0       # invalid dtype
    assert rb.rapid_workspace_bytes(rb.OP_LOGPROB_FWD, *args) < rec
    # the cache: with a token bound, a cache of that many rows (rounded to 256) holds the whole batch: one chunk, and
    # the compact row arrays shrink with it; without, every padded position
    full = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *args, max_tokens=256 * 2048)
    half = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *args, max_tokens=300630)
    ldv, ldk, slots = 152064 + 64, 1536 + 64, 2 * 152064 // 256
    rows = 256 * 2048 - 300800
    # cache, packed hidden row, log-sum-exp partials, nine row arrays, the final norm's partial sums (d floats per 512 rows)
    per_row = ldv * 2 + ldk * 2 + 2 * slots * 4 + 9 * 4 + 1536 * 4 // 512
    assert abs((full - half) - rows * per_row) <= 8192              # alignment of the buffers
    assert rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *args, max_tokens=10**9) == full
    assert rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, *args, max_tokens=1000) == rec       # other ops ignore it
    # recommended: a cache of 90112 rows, the batch in chunks of whole groups; it fits 32 GiB at this shape
    chunked = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *args)
    smallest = rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *args, minimum=True)
    assert smallest < chunked < half and chunked < 32 * 2**30 and chunked > 90112 * ldv * 2
    # the window a call takes from a given workspace: the recommended size gives 90112 rows when no token bound is
    # promised, more when the bound shrinks the per-row arrays (fewer regions); the one-chunk size gives every row;
    # below the minimum nothing
    dims = args[:5]
    assert rb.rapid_logits_cache_rows(*dims, 0, chunked) == 90112
    assert 90112 <= rb.rapid_logits_cache_rows(*dims, 300630, chunked) < 300800
    assert rb.rapid_logits_cache_rows(*dims, 300630, half) == 300800
    assert rb.rapid_logits_cache_rows(*dims, 0, full) == 256 * 2048
    assert rb.rapid_logits_cache_rows(*dims, 0, smallest) == 256 and rb.rapid_logits_cache_rows(*dims, 0, smallest - 4096) == 0
    assert rb.rapid_logits_cache_rows(*dims, 0, chunked - 4096) == 90112 - 256
    # a batch with fewer positions than that has the one-chunk size as its recommended size
    small_args = (16, 128, 1536, 151936, 4, rb.DTYPE_BF16)
    assert rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *small_args) == \
        rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD_CACHED, *small_args, max_tokens=16 * 128)


def test_host_validation_returns_codes_without_a_gpu(rb):
    lib = rb.load()
    one = C.c_void_p(256)   # fake, aligned, never dereferenced: validation fails first
    # NULL hidden
    rc = lib.rapid_logprob_fwd(None, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None,
                               one, 1 << 30, None)
    assert rc == -1 and b"NULL" in lib.rapid_last_error()
    # bad dtype, bad shape, bf16 with d % 8 != 0, bad layout, bad temperature, misaligned workspace
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 8, 8, 9, rb.W_DV, 1.0, one, None, None, one, 1 << 30, None) == -3
    assert lib.rapid_logprob_fwd(one, one, one, one, 0, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, one, 1 << 30, None) == -2
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 12, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, one, 1 << 30, None) == -2
    # past the maximum sizes: N * T <= 2e9 positions, d <= 65536, V <= 4e6
    assert lib.rapid_logprob_fwd(one, one, one, one, 1 << 20, 1 << 12, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, one, 1 << 30, None) == -2
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 65536 + 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, one, 1 << 30, None) == -2
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 8, 4 * 10**6 + 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, one, 1 << 30, None) == -2
    assert rb.rapid_workspace_bytes(rb.OP_IW_PG_FWD_BWD, 1 << 20, 1 << 12, 8, 8, 1, rb.DTYPE_BF16) == 0
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, 5, 1.0, one, None, None, one, 1 << 30, None) == -3
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 0.0, one, None, None, one, 1 << 30, None) == -2
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, C.c_void_p(8), 1 << 30, None) == -4
    # workspace too small
    assert lib.rapid_logprob_fwd(one, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, one, 16, None) == -4
    assert b"minimum" in lib.rapid_last_error()
    # group advantage
    assert lib.rapid_group_advantage(None, one, None, 4, 1, 2.0, 0, one, None, None, None, None, None, None) == -1
    assert lib.rapid_group_advantage(one, one, None, 4, 0, 2.0, 0, one, None, None, None, None, None, None) == -2
    assert lib.rapid_group_advantage(one, one, None, 4, 1, 2.0, 9, one, None, None, None, None, None, None) == -3
    # fused call: missing outputs, unknown mode, accumulate into bf16
    o = rb.default_opts()
    args = lambda **k: [one, one, one, one, one, one, one, 4, 4, 8, 8, 1, rb.DTYPE_BF16, C.byref(o),
                        k.get("loss", one), one, one, None, None, None, None, None, None, one, 1 << 30, None]
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args(loss=None)) == -1
    o.coef_mode = 7
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -3
    o = rb.default_opts()
    o.accumulate_dw, o.dw_dtype = 1, rb.DTYPE_BF16
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -3
    o = rb.default_opts()
    o.logits_cache = 2
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -3
    o = rb.default_opts()
    o.ratio_level = 2
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -3
    o = rb.default_opts()
    o.max_tokens = -5
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -2
    o = rb.default_opts()
    o.rms_weight, o.rms_eps = 256, -1.0                     # negative eps
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -2
    # the final norm is a bf16 option
    assert lib.rapid_logprob_fwd_rmsnorm(one, one, one, one, 4, 4, 8, 8, rb.DTYPE_F32, rb.W_DV, 1.0, one, 1e-6, one, None,
                                         None, one, 1 << 30, None) == -3
    assert lib.rapid_logprob_fwd_rmsnorm(one, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, None, 1e-6, one, None,
                                         None, one, 1 << 30, None) == -1
    # the entry point on the static scratch: shapes past its 768 MiB are refused on the host, with both sizes named
    assert lib.rapid_logprob_fwd_static(one, one, one, one, 256, 2048, 1536, 151936, rb.DTYPE_BF16, rb.W_DV, 1.0, one,
                                        None, None, None) == -4
    assert b"static scratch holds 805306368" in lib.rapid_last_error()
    assert lib.rapid_logprob_fwd_static(one, one, one, one, 0, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, None) == -2
    assert lib.rapid_logprob_fwd_static(one, one, one, one, 4, 4, 8, 8, 5, rb.W_DV, 1.0, one, None, None, None) == -3
    assert lib.rapid_logprob_fwd_static(None, one, one, one, 4, 4, 8, 8, rb.DTYPE_BF16, rb.W_DV, 1.0, one, None, None, None) in (-1, -6)
    o = rb.default_opts()
    o.loss_scale = -1.0
    assert lib.rapid_iw_pg_loss_fwd_bwd(*args()) == -2
    assert lib.rapid_set_tuning(12345, 0) == -3
    assert lib.rapid_set_tuning(13, 0) == -3          # forward row block of 0 tiles
    assert lib.rapid_set_tuning(16, 100) == -3        # pacing interval must be a power of two (or 0)
    assert lib.rapid_set_tuning(16, 128) == 0 and lib.rapid_set_tuning(16, 0) == 0
    assert lib.rapid_mfma_probe(0, 0, None, None, None) == -2       # iters out of range, checked before the device
    assert lib.rapid_mfma_probe(1, 10**8, None, None, None) == -2


def test_workload_generator_recipe():
    import torch
    from paper_2510_03515_amd import workloads as wl
    w = wl.make_workload(wl.CONFIGS[0], seed=0)
    spec = w["spec"]
    assert w["hidden"].shape == (32, 32, 64) and w["W"].shape == (64, 1000)
    L = w["lengths"]
    assert int(L.min()) >= 8 and int(L.max()) <= 32
    assert torch.equal(w["mask"].sum(1).long(), L)
    rms = w["hidden"].float().pow(2).mean(-1).sqrt()
    assert torch.allclose(rms, torch.ones_like(rms), atol=1e-5)
    assert int(w["tokens"].min()) >= 0 and int(w["tokens"].max()) < spec.V
    assert torch.all(w["tokens"][w["mask"] == 0] == 0)
    assert set(w["rewards"].tolist()) <= {0.0, 1.0}
    assert w["group_ids"].tolist() == [n // 4 for n in range(32)]
    w2 = wl.make_workload(wl.CONFIGS[0], seed=0)
    assert torch.equal(w["tokens"], w2["tokens"]) and torch.equal(w["hidden"], w2["hidden"])
    c = wl.calibrated(wl.CONFIGS[2])
    assert abs(c.sigma - (0.5 / (2048 * 1536)) ** 0.5) < 1e-12


def test_header_is_plain_c_and_links(tmp_path):
    """include/rapid.h compiles as C99 with nothing but the standard headers, and a C program that
    references every declared entry point links against the built library (no compute is run)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    names = _declared()
    src = tmp_path / "link_check.c"
    src.write_text('#include "rapid.h"\n#include "rapid_tuning.h"\n#include <stdio.h>\ntypedef void (*fn_t)(void);\nint main(void) {\n  fn_t f[] = {'
                   + ", ".join(f"(fn_t){n}" for n in names)
                   + '};\n  printf("%d %d\\n", (int)(sizeof f / sizeof f[0]), rapid_version());\n  return f[0] == 0;\n}\n')
    lib_dir = os.path.join(ROOT, "paper_2510_03515_amd")
    exe = tmp_path / "link_check"
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src),
                        "-L", lib_dir, "-l:librapid_hip.so", f"-Wl,-rpath,{lib_dir}", "-o", str(exe)],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.split()[0] == str(len(names))
