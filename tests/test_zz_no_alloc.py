"""The entry point for callers that cannot allocate device memory: pmc_layernorm_backward_static keeps
its scratch (partial sums of the gain/bias gradients) in a device array built into the library.
Checked through the C ABI against pmc_layernorm_backward (same kernels, caller-attached workspace) and
against the oracle, on two calls in a row, the second with a smaller input (the array still holds the
first call's partial sums); runs last so that a failure here hides no other test."""
import numpy as np
import pytest
import torch

import paper_2405_15362_amd as P
import synth
from oracle import layer as OL
from gpu_util import assert_close, dev, host, mat

pytestmark = pytest.mark.gpu


def _case(dtype, rows, h):
    key = ("ln_static", dtype, rows, h)
    x = mat(key + ("x",), (rows, h), dtype, 2.0)
    g = mat(key + ("g",), (h,), "f32", 0.1) + 1.0
    if dtype == "bf16":
        g = synth.round_to_bf16(g)
    dy = mat(key + ("dy",), (rows, h), dtype)
    resid = mat(key + ("res",), (rows, h), dtype)
    return x, g, dy, resid


def _run(ctx, fn, dtype, x, g, dy, resid, mean, rstd):
    rows, h = x.shape
    dx = torch.empty_like(dev(x, dtype))
    dgain = torch.full((h,), 0.25, device="cuda")
    dbias = torch.full((h,), -0.5, device="cuda")
    fn(ctx, dev(dy, dtype), dev(x, dtype), dev(g, dtype), mean, rstd, dev(resid, dtype), dx, dgain, dbias)
    torch.cuda.synchronize()
    return dx, dgain, dbias


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_layernorm_backward_static_matches_workspace_entry_point(dtype):
    # a context with NO workspace for the static entry point, one with a workspace for the existing one
    bare = P.pmc_create(None)
    full = P.pmc_create(None)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    P.pmc_workspace_attach(full, ws)
    try:
        # first call: many workgroups, wide rows; second call: fewer rows AND narrower rows, so most of
        # the array keeps the first call's partial sums
        for rows, h in ((1544, 2048 if dtype == "bf16" else 1024), (72, 256)):
            print("static layernorm backward case", dtype, rows, h, flush=True)
            x, g, dy, resid = _case(dtype, rows, h)
            x64 = x.astype(np.float64)
            y_ref, xhat, rstd_ref = OL.layer_norm(x64, g.astype(np.float64), np.zeros(h), 1e-5)
            mean = torch.from_numpy(x64.mean(-1).astype(np.float32)).cuda()
            rstd = torch.from_numpy(rstd_ref[:, 0].astype(np.float32)).cuda()
            got = _run(bare, P.pmc_layernorm_backward_static, dtype, x, g, dy, resid, mean, rstd)
            want = _run(full, P.pmc_layernorm_backward, dtype, x, g, dy, resid, mean, rstd)
            for a, b in zip(got, want):      # same kernels, same launch shape: the same bits
                assert torch.equal(a, b)
            dx_ref, dg_ref, db_ref = OL.layer_norm_input_grad(dy.astype(np.float64), xhat, rstd_ref, g.astype(np.float64))
            assert_close(host(got[0]), dx_ref + resid, dtype, "dx")
            assert_close(host(got[1]) - 0.25, dg_ref, "f32" if dtype == "f32" else "bf16", "dgain", atol_scale=4.0)
            assert_close(host(got[2]) + 0.5, db_ref, "f32", "dbias", atol_scale=4.0)
        # beyond the array: 512 workgroups x 2 x 12288 floats = 48 MiB > 32 MiB -> refused, nothing launched
        if dtype == "bf16":
            rows, h = 1024, 12288
            z = torch.zeros(rows, h, dtype=torch.bfloat16, device="cuda")
            v = torch.zeros(rows, device="cuda")
            gz = torch.zeros(h, dtype=torch.bfloat16, device="cuda")
            f = torch.zeros(h, device="cuda")
            with pytest.raises(P.PmcError) as e:
                P.pmc_layernorm_backward_static(bare, z, z, gz, v, v, None, z, f, f)
            assert e.value.code == P.PMC_ERR_NOMEM and "scratch" in str(e.value)
    finally:
        torch.cuda.synchronize()
        P.pmc_destroy(bare)
        P.pmc_destroy(full)
