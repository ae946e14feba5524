"""The entry point for callers that cannot allocate (essa_svdlora_forward_noalloc) against essa_svdlora_forward: same
bits, on two calls in a row that share the library's fixed scratch array, the second one smaller."""
import numpy as np
import pytest
import torch

import essa_workloads as wl
import oracle as orc
from helpers import bf16_dev, bf16_host, candidate_sigmas, gpu_proj, oracle_proj, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx(essa):
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    c = essa.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("quant", ["int8", "int4"])
def test_noalloc_forward_matches_the_allocating_entry_point(essa, ctx, quant):
    d_in, d_out, r, K = 1024, 328, 16, 5
    p = wl.make_projection("t", d_in, d_out, r, quant, layer=16, proj=1)
    W, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, K, 0.05)
    sAd, sBd = to_dev(sA), to_dev(sB)
    for R, x_id in ((200, 50), (37, 51)):                    # the second call is smaller and finds the first one's leftovers
        print("noalloc %s R=%d" % (quant, R), flush=True)
        xb, xv = wl.make_x_bf16(R, d_in, x_id=x_id)
        r2c = np.random.default_rng(R).integers(0, K, R).astype(np.int32)
        Xd, rd = bf16_dev(xb), to_dev(r2c)
        for dtype in (torch.bfloat16, torch.float32):
            Y0 = torch.empty(R, d_out, device="cuda", dtype=dtype)
            Y1 = torch.full((R, d_out), float("nan"), device="cuda", dtype=dtype)
            essa.essa_svdlora_forward(ctx, gp, Xd, rd, sAd, sBd, Y0)
            essa.essa_svdlora_forward_noalloc(ctx, gp, Xd, rd, sAd, sBd, Y1)
            assert torch.equal(Y0, Y1)
        ref = orc.round_to_bf16(orc.svdlora_forward(W, f, xv, r2c, sA, sB))
        Yb = torch.empty(R, d_out, device="cuda", dtype=torch.bfloat16)
        essa.essa_svdlora_forward_noalloc(ctx, gp, Xd, rd, sAd, sBd, Yb)
        e_max, e_rms = orc.rel_errors(bf16_host(Yb), ref)
        assert e_rms <= 1e-3 and e_max <= 2e-2, (e_max, e_rms)
    gp.close()


def test_noalloc_forward_refuses_what_does_not_fit(essa, ctx):
    p = wl.make_projection("t", 2048, 64, 8, "int8", layer=17)
    _, f = oracle_proj(p)
    gp = gpu_proj(essa, ctx, p)
    sA, sB = candidate_sigmas(f, 2, 0.05)
    R = 4096                                                 # two limbs of 4096 x 2048 bytes: 16 MiB > the 8 MiB array
    X = torch.zeros(R, 2048, device="cuda", dtype=torch.bfloat16)
    Y = torch.full((R, 64), 3.0, device="cuda")
    with pytest.raises(essa.EssaError) as ei:
        essa.essa_svdlora_forward_noalloc(ctx, gp, X, torch.zeros(R, dtype=torch.int32, device="cuda"), to_dev(sA), to_dev(sB), Y)
    assert ei.value.code == 2 and "scratch" in str(ei.value)
    assert torch.all(Y == 3.0)
    with pytest.raises(essa.EssaError):                      # the debug flag allocates: not here
        essa.essa_svdlora_forward_noalloc(ctx, gp, X[:8], torch.zeros(8, dtype=torch.int32, device="cuda"), to_dev(sA), to_dev(sB), Y[:8], essa.VALIDATE)
    gp.close()
