"""The entry point that allocates nothing, rapid_logprob_fwd_static (scratch = a static device array
inside the library), through the C ABI: its outputs are the bits of rapid_logprob_fwd, and meet the
oracle at the usual tolerance, on two calls in a row of which the second is smaller (the array
keeps the first call's contents), in bf16 and fp32; and nothing is allocated while it runs."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import rapid_oracle as orc
from paper_2510_03515_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_entry_point_matches_the_workspace_one(dtype):
    from paper_2510_03515_amd import binding as rb
    lib = rb.load()
    big = wl.small_spec("static_big", dtype, d=200, V=1321, prompts=5, G=3, len_lo=1, len_hi=90)
    small = wl.small_spec("static_small", dtype, d=64, V=300, prompts=2, G=2, len_lo=2, len_hi=17)
    atol = 2e-5 if dtype == "bf16" else 2e-6
    dt = rb.DTYPE_BF16 if dtype == "bf16" else rb.DTYPE_F32
    cases = []
    for spec, seed, layout in ((big, 0, rb.W_DV), (small, 1, rb.W_VD)):
        w = wl.make_workload(spec, seed=seed, device="cpu")
        g = {k: (v.cuda() if torch.is_tensor(v) else v) for k, v in w.items()}
        Wg = g["W"] if layout == rb.W_DV else g["W"].t().contiguous()
        N, T, d = g["hidden"].shape
        ref_lp, ref_lse = rb.rapid_logprob_fwd(g["hidden"], Wg, g["tokens"], g["mask"], w_layout=layout, want_lse=True)
        o_lp, o_lse = orc.logprob(_f64(w["hidden"]), _f64(w["W"]), w["tokens"].numpy(), w["mask"].numpy())
        lp = torch.full((N, T), 7.0, dtype=torch.float32, device="cuda")
        lse = torch.full((N, T), 7.0, dtype=torch.float32, device="cuda")
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        cases.append((spec, g, Wg, layout, ref_lp, ref_lse, o_lp, o_lse, lp, lse, status))
    torch.cuda.synchronize()
    vp = lambda t: C.c_void_p(t.data_ptr())
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    def call(case):
        spec, g, Wg, layout, _, _, _, _, lp, lse, status = case
        N, T, d = g["hidden"].shape
        return lib.rapid_logprob_fwd_static(vp(g["hidden"]), vp(Wg), vp(g["tokens"]), vp(g["mask"]), N, T, d, spec.V, dt,
                                            layout, 1.0, vp(lp), vp(lse), vp(status), stream)

    # Two rounds of two calls in a row, the larger input first.  In the first round the runtime loads the
    # kernels' code and the first call looks the array's address up; in the second round the free device
    # memory is read right before and right after each call (nothing else runs in between): unchanged.
    for rnd in range(2):
        for case in cases:
            spec, g, Wg, layout, ref_lp, ref_lse, o_lp, o_lse, lp, lse, status = case
            print(f"round {rnd}: static call {spec.name} {tuple(g['hidden'].shape)} V={spec.V}", flush=True)
            lp.fill_(7.0); lse.fill_(7.0)
            torch.cuda.synchronize()
            free_before, _ = torch.cuda.mem_get_info()
            reserved_before = torch.cuda.memory_reserved()
            rc = call(case)
            torch.cuda.synchronize()
            free_after, _ = torch.cuda.mem_get_info()
            assert rc == 0, lib.rapid_last_error()
            if rnd == 1:
                assert torch.cuda.memory_reserved() == reserved_before and free_after == free_before
            assert status.item() == 0
            assert torch.equal(lp, ref_lp) and torch.equal(lse, ref_lse)
            assert np.abs(_f64(lp) - o_lp).max() <= atol and np.abs(_f64(lse) - o_lse).max() <= atol
            assert np.all(_f64(lp)[g["mask"].cpu().numpy() == 0] == 0.0)
    spec, g, Wg, layout, *_, lp, lse, status = cases[1]
    # a shape whose scratch does not fit is refused with both sizes in the message, nothing launched
    rc = lib.rapid_logprob_fwd_static(vp(g["hidden"]), vp(Wg), vp(g["tokens"]), vp(g["mask"]), 256, 2048, 1536, 151936,
                                      rb.DTYPE_BF16, rb.W_DV, 1.0, vp(lp), None, None, stream)
    assert rc == -4 and b"static scratch holds" in lib.rapid_last_error()
