"""GPU parity of the single kernels against the CPU oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2405_15362_amd as P
import synth
from oracle import layer as OL
from gpu_util import assert_close, dev, host, mat, rel_l2, tol

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = P.pmc_create(None)
    ws = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    P.pmc_workspace_attach(c, ws)
    yield c
    torch.cuda.synchronize()
    P.pmc_destroy(c)


def _gemm_case(ctx, dtype, ta, tb, M, N, K, epi):
    key = (dtype, ta, tb, M, N, K, epi)
    print("gemm case", key, flush=True)
    a = mat(key + ("a",), (K, M) if ta else (M, K), dtype)
    b = mat(key + ("b",), (N, K) if tb else (K, N), dtype, 0.05)
    bias = mat(key + ("bias",), (N,), dtype)
    resid = mat(key + ("r",), (M, N), dtype)
    aux_in = mat(key + ("u",), (M, N), dtype)
    A = a.T.astype(np.float64) if ta else a.astype(np.float64)
    B = b.T.astype(np.float64) if tb else b.astype(np.float64)
    ref = A @ B
    out_dtype = "f32" if epi == P.EPI_ACCUM_F32 else dtype
    c0 = mat(key + ("c0",), (M, N), "f32")
    c = dev(c0, out_dtype)
    aux = dev(aux_in, dtype) if epi in (P.EPI_BIAS_GELU, P.EPI_DGELU, P.EPI_BIAS_GELU_GRAD, P.EPI_MUL) else None
    want_aux = None
    if epi == P.EPI_BIAS:
        ref = ref + bias
    elif epi == P.EPI_BIAS_RESID:
        ref = ref + bias + resid
    elif epi == P.EPI_BIAS_GELU:
        ref = ref + bias
        want_aux = OL.gelu(ref)
    elif epi == P.EPI_DGELU:
        ref = ref * OL.gelu_grad(aux_in.astype(np.float64))
    elif epi == P.EPI_ACCUM_F32:
        ref = ref + c0
    elif epi == P.EPI_BIAS_GELU_GRAD:
        want_aux = OL.gelu(ref + bias)
        ref = OL.gelu_grad(ref + bias)
    elif epi == P.EPI_MUL:
        ref = ref * aux_in.astype(np.float64)
    P.pmc_gemm(ctx, dev(a, dtype), dev(b, dtype), c, ta, tb, epi,
               dev(bias, dtype) if epi in (P.EPI_BIAS, P.EPI_BIAS_RESID, P.EPI_BIAS_GELU, P.EPI_BIAS_GELU_GRAD) else None,
               dev(resid, dtype) if epi == P.EPI_BIAS_RESID else None, aux)
    torch.cuda.synchronize()
    assert_close(host(c), ref, dtype, str(key))
    if want_aux is not None:
        assert_close(host(aux), want_aux, dtype, str(key))


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_gemm_f32_layouts_and_epilogues(ctx, ta, tb):
    for epi in range(8):
        _gemm_case(ctx, "f32", ta, tb, 77, 130, 45, epi)
    _gemm_case(ctx, "f32", ta, tb, 128, 256, 1024, P.EPI_NONE)


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_gemm_bf16_small_tiles_ragged(ctx, ta, tb):
    # several 128x128 tiles with ragged tails in M, N and K
    for epi in range(8):
        _gemm_case(ctx, "bf16", ta, tb, 200, 328, 136, epi)
    _gemm_case(ctx, "bf16", ta, tb, 8, 8, 8, P.EPI_NONE)
    _gemm_case(ctx, "bf16", ta, tb, 512, 768, 1024, P.EPI_NONE)


@pytest.mark.parametrize("ta,tb,epis", [(False, False, (P.EPI_NONE, P.EPI_BIAS, P.EPI_BIAS_RESID, P.EPI_BIAS_GELU, P.EPI_BIAS_GELU_GRAD)),
                                        (False, True, (P.EPI_NONE, P.EPI_DGELU, P.EPI_MUL)),
                                        (True, False, (P.EPI_NONE, P.EPI_ACCUM_F32))])
def test_gemm_bf16_direct_to_lds_path(ctx, ta, tb, epis):
    """K in whole 64-wide tiles takes the direct-to-LDS kernel: each of its three tile shapes, with
    ragged edges in M and N (clamped loads), a single K tile and many K tiles."""
    try:
        for tile in (4, 3, 2, 1, 0):      # 256x320, 64x128, 128x128, 256x128, 256x256 tiles
            P.pmc_tuning_set("gemm_tile", tile)
            for epi in epis:
                _gemm_case(ctx, "bf16", ta, tb, 200, 328, 192, epi)
                _gemm_case(ctx, "bf16", ta, tb, 1000, 1544, 64, epi)
            _gemm_case(ctx, "bf16", ta, tb, 8, 8, 64, epis[0])
            _gemm_case(ctx, "bf16", ta, tb, 264, 136, 2048, epis[-1])
    finally:
        P.pmc_tuning_set("gemm_tile", -1)
    _gemm_case(ctx, "bf16", ta, tb, 3848, 4104, 320, epis[-1])   # heuristic choice, many tiles


@pytest.mark.parametrize("ta,tb,epis", [(False, False, (P.EPI_BIAS, P.EPI_BIAS_RESID, P.EPI_BIAS_GELU, P.EPI_BIAS_GELU_GRAD)),
                                        (False, True, (P.EPI_NONE, P.EPI_DGELU, P.EPI_MUL)),
                                        (True, False, (P.EPI_ACCUM_F32,))])
def test_gemm_bf16_split_k(ctx, ta, tb, epis):
    """Skinny products are cut along K into fp32 partials that a second kernel adds in a fixed
    order; the result must also be identical from run to run."""
    for epi in epis:
        _gemm_case(ctx, "bf16", ta, tb, 512, 1024, 1024, epi)      # 4 splits
        _gemm_case(ctx, "bf16", ta, tb, 136, 264, 4096, epi)       # 8 splits, ragged tiles
    a = dev(mat(("sk", "a"), (1024, 256) if ta else (256, 1024), "bf16"), "bf16")
    b = dev(mat(("sk", "b"), (512, 1024) if tb else (1024, 512), "bf16", 0.05), "bf16")
    outs = []
    for _ in range(3):
        c = torch.zeros(256, 512, device="cuda", dtype=torch.bfloat16)
        P.pmc_gemm(ctx, a, b, c, ta, tb)
        outs.append(c)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_gemm_bf16_weight_gradient_persistent(ctx, tune):
    """The persistent W-pass kernel (fp32 C += A^T B; one workgroup per compute unit walks its
    256x256 tiles, its first tile cut in two along K to put the workgroups out of phase): fewer tiles
    than workgroups, more tiles than workgroups with ragged edges, short and long K; and the same
    result from run to run."""
    tune(gemm_wgrad=1)
    for M, N, K in ((512, 256, 256), (264, 136, 1024), (4104, 4360, 256), (4096, 4608, 576), (3848, 4872, 1280)):
        _gemm_case(ctx, "bf16", True, False, M, N, K, P.EPI_ACCUM_F32)
    a = dev(mat(("wg", "a"), (1024, 4104), "bf16"), "bf16")
    b = dev(mat(("wg", "b"), (1024, 4360), "bf16", 0.05), "bf16")
    c0 = dev(mat(("wg", "c"), (4104, 4360), "f32"), "f32")
    outs = []
    for flag in (1, 1, 0):
        tune(gemm_wgrad=flag)
        c = c0.clone()
        P.pmc_gemm(ctx, a, b, c, True, False, P.EPI_ACCUM_F32)
        outs.append(c)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1])
    assert rel_l2(host(outs[0]), host(outs[2])) <= 1e-6     # the plain kernel adds K in one piece


def test_gemm_bf16_weight_gradient_two_workgroups_per_unit(ctx, tune):
    """The W-pass kernel with 256x128 tiles and a ring of 32-deep stages (two workgroups share a compute
    unit): fewer tiles than units, many more, ragged edges in both directions, K of one 64-wide tile (two
    ring tiles, fewer than the ring has stages), short and long K; the same bits from run to run; and the
    same sums as the plain kernel up to fp32 summation order."""
    tune(gemm_wgrad=2)
    for M, N, K in ((512, 256, 64), (264, 136, 128), (264, 136, 1024), (4104, 4360, 256), (4096, 4608, 576), (3848, 4872, 1280)):
        _gemm_case(ctx, "bf16", True, False, M, N, K, P.EPI_ACCUM_F32)
    a = dev(mat(("wg", "a"), (1024, 4104), "bf16"), "bf16")
    b = dev(mat(("wg", "b"), (1024, 4360), "bf16", 0.05), "bf16")
    c0 = dev(mat(("wg", "c"), (4104, 4360), "f32"), "f32")
    outs = []
    for flag in (2, 2, 0):
        tune(gemm_wgrad=flag)
        c = c0.clone()
        P.pmc_gemm(ctx, a, b, c, True, False, P.EPI_ACCUM_F32)
        outs.append(c)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1])
    assert rel_l2(host(outs[0]), host(outs[2])) <= 1e-6


@pytest.mark.parametrize("wgrad", [0, 1, 2])
def test_gemm_bf16_grouped_weight_gradient(ctx, tune, wgrad):
    """Queued weight gradients as one product: C += sum_i A_i^T B_i over pieces that live in separate
    buffers.  Every tile shape of the plain kernel and the persistent one; one piece, several pieces,
    the maximum; pieces of a single 64-wide K tile (a piece boundary at every tile) and of many;
    ragged M and N; and the same bits from run to run.  Against the fp64 sum of the pieces' products;
    the result must also agree with adding the pieces one product at a time."""
    tune(gemm_wgrad=wgrad)
    cases = [(512, 256, 64, 3), (264, 136, 192, 2), (1000, 1544, 128, 8), (2048, 2304, 256, 4), (4104, 4360, 64, 5),
             (128, 128, 1024, 1)]
    for tile in (None, 0, 1, 2):
        tune(gemm_tile=tile)
        for M, N, K, count in (cases if tile is None else cases[:3]):
            key = ("grouped", M, N, K, count)
            print("grouped wgrad case", key, "tile", tile, "persistent", wgrad, flush=True)
            a = [mat(key + ("a", i), (K, M), "bf16") for i in range(count)]
            b = [mat(key + ("b", i), (K, N), "bf16", 0.05) for i in range(count)]
            c0 = mat(key + ("c0",), (M, N), "f32")
            ref = c0.astype(np.float64)
            for x, y in zip(a, b):
                ref = ref + x.T.astype(np.float64) @ y.astype(np.float64)
            da, db = [dev(x, "bf16") for x in a], [dev(y, "bf16") for y in b]
            outs = []
            for _ in range(2):
                c = dev(c0, "f32")
                P.pmc_gemm_grouped_wgrad(ctx, da, db, c)
                outs.append(c)
            one_by_one = dev(c0, "f32")
            for x, y in zip(da, db):
                P.pmc_gemm(ctx, x, y, one_by_one, True, False, P.EPI_ACCUM_F32)
            torch.cuda.synchronize()
            assert torch.equal(outs[0], outs[1]), key
            assert rel_l2(host(outs[0]), ref) <= 1e-5, (key, rel_l2(host(outs[0]), ref))   # fp32 sums of exact bf16 products
            assert rel_l2(host(outs[0]), host(one_by_one)) <= 1e-5, key


@pytest.mark.timeout(600)
def test_gemm_bf16_largest_workload_shapes(ctx):
    """The twelve products of a layer at the largest workload (hidden 5120, FFN 20480, 4096 tokens), at
    full size and in the launch configuration the passes use (heuristic tile choice, persistent W
    kernel).  Operands are drawn on the GPU from a seeded generator (2e8 elements per product);
    EVERY output element is checked against the fp64 product with the epilogue's definition applied
    (whole tensor, every 32 x 128 block, every element)."""
    T, h, f = 4096, 5120, 20480
    gen = torch.Generator(device="cuda").manual_seed(4)
    bf = torch.bfloat16

    def rnd(shape, scale):
        return (torch.randn(shape, device="cuda", generator=gen) * scale).to(bf)

    def f64(t):
        return t.float().cpu().numpy().astype(np.float64)

    cases = [("F qkv", False, False, T, 3 * h, h, P.EPI_BIAS), ("F proj", False, False, T, h, h, P.EPI_BIAS_RESID),
             ("F fc1", False, False, T, f, h, P.EPI_BIAS_GELU_GRAD), ("F fc2", False, False, T, h, f, P.EPI_BIAS_RESID),
             ("B dfc2", False, True, T, f, h, P.EPI_MUL), ("B dfc1", False, True, T, h, f, P.EPI_NONE),
             ("B dproj", False, True, T, h, h, P.EPI_NONE), ("B dqkv", False, True, T, h, 3 * h, P.EPI_NONE),
             ("W fc2", True, False, f, h, T, P.EPI_ACCUM_F32), ("W fc1", True, False, h, f, T, P.EPI_ACCUM_F32),
             ("W proj", True, False, h, h, T, P.EPI_ACCUM_F32), ("W qkv", True, False, h, 3 * h, T, P.EPI_ACCUM_F32)]
    for name, ta, tb, M, N, K, epi in cases:
        print("largest-shape gemm", name, M, N, K, flush=True)
        a = rnd((K, M) if ta else (M, K), 1.0)
        b = rnd((N, K) if tb else (K, N), 0.02)
        bias, extra = rnd((N,), 0.02), rnd((M, N), 1.0)          # extra: residual or GeLU input
        c = (torch.randn((M, N), device="cuda", generator=gen) if epi == P.EPI_ACCUM_F32
             else torch.zeros((M, N), device="cuda", dtype=bf))
        c0 = c.clone() if epi == P.EPI_ACCUM_F32 else None
        aux = extra.clone() if epi == P.EPI_MUL else (torch.zeros_like(extra) if epi == P.EPI_BIAS_GELU_GRAD else None)
        P.pmc_gemm(ctx, a, b, c, ta, tb, epi, bias if epi in (P.EPI_BIAS, P.EPI_BIAS_RESID, P.EPI_BIAS_GELU_GRAD) else None,
                   extra if epi == P.EPI_BIAS_RESID else None, aux)
        torch.cuda.synchronize()
        A = f64(a).T if ta else f64(a)
        B = f64(b).T if tb else f64(b)
        ref = A @ B
        del A, B
        if epi in (P.EPI_BIAS, P.EPI_BIAS_RESID, P.EPI_BIAS_GELU_GRAD):
            ref += f64(bias)
        if epi == P.EPI_BIAS_RESID:
            ref += f64(extra)
        if epi == P.EPI_MUL:
            ref *= f64(extra)
        if epi == P.EPI_ACCUM_F32:
            ref += f64(c0)
        if epi == P.EPI_BIAS_GELU_GRAD:
            assert_close(f64(aux), OL.gelu(ref), "bf16", name + " gelu")
            ref = OL.gelu_grad(ref)
        # fp32 sums of exact bf16 products: the fp32 accumulate is held to the fp32 bounds
        assert_close(f64(c), ref, "f32" if epi == P.EPI_ACCUM_F32 else "bf16", name,
                     whole_tol=1e-5 if epi == P.EPI_ACCUM_F32 else None)
        del a, b, c, c0, aux, extra, ref


@pytest.mark.parametrize("ta,tb,epis", [(False, False, (P.EPI_NONE, P.EPI_BIAS, P.EPI_BIAS_RESID, P.EPI_BIAS_GELU, P.EPI_BIAS_GELU_GRAD)),
                                        (False, True, (P.EPI_NONE, P.EPI_DGELU, P.EPI_MUL)),
                                        (True, False, (P.EPI_NONE, P.EPI_ACCUM_F32))])
def test_gemm_bf16_random_shapes(ctx, ta, tb, epis):
    """Seeded random shapes in the library's own choice of kernel and tile: M and N any multiple of 8
    up to a few tiles (ragged edges in both), K in whole 64-wide tiles (direct-to-LDS kernel, split K
    where the library picks it) or any multiple of 8 (general kernel); the epilogue drawn from those
    the layout is used with."""
    rng = np.random.default_rng(20240515 + 2 * ta + tb)
    for i in range(14):
        M, N = (int(8 * rng.integers(1, 190)) for _ in range(2))
        K = int(64 * rng.integers(1, 40)) if i % 3 else int(8 * rng.integers(1, 90))
        _gemm_case(ctx, "bf16", ta, tb, M, N, K, epis[int(rng.integers(0, len(epis)))])


def test_gemm_grouped_weight_gradient_rejects_bad_arguments(ctx):
    a = [torch.zeros(64, 128, device="cuda", dtype=torch.bfloat16)]
    b = [torch.zeros(64, 128, device="cuda", dtype=torch.bfloat16)]
    c = torch.zeros(128, 128, device="cuda", dtype=torch.float32)
    with pytest.raises(P.PmcError):
        P.pmc_gemm_grouped_wgrad(ctx, a * 9, b * 9, c)                       # more pieces than PMC_MAX_QUEUED_W
    a32 = [torch.zeros(32, 128, device="cuda", dtype=torch.bfloat16)]
    with pytest.raises(P.PmcError):
        P.pmc_gemm_grouped_wgrad(ctx, a32, a32, c)                           # K not in whole 64-wide tiles


@pytest.mark.parametrize("ta,tb", [(False, False), (False, True), (True, False)])
def test_gemm_bf16_large_tiles(ctx, ta, tb):
    # enough 256x256 tiles to take the large-tile path, ragged edge tiles included
    for epi in ((P.EPI_BIAS_GELU, P.EPI_BIAS_RESID) if not ta and not tb else
                (P.EPI_DGELU, P.EPI_NONE) if not ta else (P.EPI_ACCUM_F32,)):
        _gemm_case(ctx, "bf16", ta, tb, 3848, 3592, 200, epi)


def test_gemm_rejects_bad_arguments(ctx):
    a = torch.zeros(16, 16, device="cuda", dtype=torch.bfloat16)
    c = torch.zeros(16, 12, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(P.PmcError) as e:
        P.pmc_gemm(ctx, a, a[:, :12].contiguous(), c)          # N = 12 is not a multiple of 8
    assert e.value.code == P.PMC_ERR_INVALID
    with pytest.raises(P.PmcError):
        P.pmc_gemm(ctx, a, a, torch.zeros(16, 16, device="cuda", dtype=torch.bfloat16), epilogue=P.EPI_BIAS)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,h", [(37, 16), (64, 256), (5, 320), (1100, 1032), (130, 2048), (2100, 4096), (33, 5120), (9, 8192),
                                    (7, 9000), (17, 10240), (6, 12288), (2, 12296), (4096, 5120)])
def test_layernorm_forward_backward(ctx, dtype, rows, h):
    if h > (6144 if dtype == "f32" else 12288):
        # a wave keeps its row in registers: 24 vectors of 16 bytes per lane at most
        td = torch.float32 if dtype == "f32" else torch.bfloat16
        with pytest.raises(P.PmcError):
            P.pmc_layernorm_forward(ctx, *[torch.zeros(rows, h, device="cuda", dtype=td)] + [torch.zeros(h, device="cuda", dtype=td)] * 2,
                                    1e-5, torch.zeros(rows, h, device="cuda", dtype=td), torch.zeros(rows, device="cuda"),
                                    torch.zeros(rows, device="cuda"))
        return
    key = ("ln", dtype, rows, h)
    print("layernorm case", key, flush=True)
    x = mat(key + ("x",), (rows, h), dtype, 2.0)
    g = mat(key + ("g",), (h,), "f32", 0.1) + 1.0
    if dtype == "bf16":
        g = synth.round_to_bf16(g)
    b = mat(key + ("b",), (h,), dtype, 0.1)
    dy = mat(key + ("dy",), (rows, h), dtype)
    resid = mat(key + ("res",), (rows, h), dtype)
    eps = 1e-5
    y_ref, xhat, rstd = OL.layer_norm(x.astype(np.float64), g.astype(np.float64), b.astype(np.float64), eps)
    dx_ref, dg_ref, db_ref = OL.layer_norm_input_grad(dy.astype(np.float64), xhat, rstd, g.astype(np.float64))
    dx_ref = dx_ref + resid
    xd, y = dev(x, dtype), dev(np.zeros_like(x), dtype)
    xc = dev(np.zeros_like(x), dtype)
    mean = torch.zeros(rows, device="cuda")
    rs = torch.zeros(rows, device="cuda")
    P.pmc_layernorm_forward(ctx, xd, dev(g, dtype), dev(b, dtype), eps, y, mean, rs, xc)
    torch.cuda.synchronize()
    assert_close(host(y), y_ref, dtype, "")
    assert np.abs(host(mean) - x.astype(np.float64).mean(-1)).max() <= 1e-5
    assert rel_l2(host(rs), rstd[:, 0]) <= 1e-5
    assert torch.equal(xc, xd)
    dgain = torch.full((h,), 0.25, device="cuda")
    dbias = torch.full((h,), -0.5, device="cuda")
    dx = xd.clone()                      # in place over x, as the B pass does
    P.pmc_layernorm_backward(ctx, dev(dy, dtype), dx, dev(g, dtype), mean, rs, dev(resid, dtype), dx, dgain, dbias)
    torch.cuda.synchronize()
    assert_close(host(dx), dx_ref, dtype, "")
    assert_close(host(dgain) - 0.25, dg_ref, dtype, "dgain", whole_tol=5e-3 if dtype == "bf16" else 1e-5)
    assert_close(host(dbias) + 0.5, db_ref, "f32", "dbias")


@pytest.mark.parametrize("dtype,dh", [("f32", 4), ("f32", 16), ("f32", 64), ("f32", 128), ("bf16", 64), ("bf16", 128),
                                      ("bf16", 8), ("bf16", 40), ("bf16", 96), ("bf16", 112)])
@pytest.mark.parametrize("causal", [True, False])
def test_attention_forward_backward(ctx, dtype, dh, causal):
    batch, seq, heads = 2, 88, 3
    if dh == 4:
        seq = 24                                     # vectors of 4 fp32: hidden must be a multiple of 4
    h = heads * dh
    key = ("attn", dtype, dh, causal)
    print("attention case", key, flush=True)
    qkv = mat(key + ("qkv",), (batch * seq, 3 * h), dtype)
    d_o = mat(key + ("do",), (batch * seq, h), dtype)
    q64 = qkv.astype(np.float64)
    o_ref, probs, lse_ref = OL.attention(q64, heads, causal, batch)
    dqkv_ref = OL.attention_input_grad(d_o.astype(np.float64), q64, probs, heads, batch)
    qd = dev(qkv, dtype)
    o = dev(np.zeros((batch * seq, h)), dtype)
    lse = torch.zeros(batch * heads * seq, device="cuda")
    P.pmc_attention_forward(ctx, qd, o, lse, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, dtype, "")
    assert np.abs(host(lse) - lse_ref.reshape(-1)).max() <= (2e-2 if dtype == "bf16" else 2e-5)
    # separate output buffer
    dq = dev(np.zeros_like(qkv), dtype)
    P.pmc_attention_backward(ctx, qd, o, lse, dev(d_o, dtype), dq, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    for name, cols in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
        assert_close(host(dq)[:, cols], dqkv_ref[:, cols], dtype, str(name), scale=np.sqrt(np.mean(dqkv_ref ** 2)))
    # in place over qkv, as the B pass does
    inplace = qd.clone()
    P.pmc_attention_backward(ctx, inplace, o, lse, dev(d_o, dtype), inplace, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    assert torch.equal(inplace, dq)


def test_attention_random_shapes(ctx):
    """Seeded random batch, sequence length, head count and head size (every multiple of 8 up to 128),
    causal or not, in the library's own choice of launch shape: ragged last blocks, sequences shorter
    than a block, padded head sizes."""
    rng = np.random.default_rng(1536205)
    for i in range(12):
        batch, heads = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        seq, dh, causal = int(rng.integers(1, 600)), int(8 * rng.integers(1, 17)), bool(rng.integers(0, 2))
        h = heads * dh
        key = ("attn-random", i)
        print("attention random case", batch, seq, heads, dh, causal, flush=True)
        qkv = mat(key + ("qkv",), (batch * seq, 3 * h), "bf16")
        d_o = mat(key + ("do",), (batch * seq, h), "bf16")
        q64 = qkv.astype(np.float64)
        o_ref, probs, lse_ref = OL.attention(q64, heads, causal, batch)
        dqkv_ref = OL.attention_input_grad(d_o.astype(np.float64), q64, probs, heads, batch)
        qd = dev(qkv, "bf16")
        o = dev(np.zeros((batch * seq, h)), "bf16")
        lse = torch.zeros(batch * heads * seq, device="cuda")
        P.pmc_attention_forward(ctx, qd, o, lse, batch, seq, heads, dh, causal)
        dq = dev(np.zeros_like(qkv), "bf16")
        P.pmc_attention_backward(ctx, qd, o, lse, dev(d_o, "bf16"), dq, batch, seq, heads, dh, causal)
        torch.cuda.synchronize()
        assert_close(host(o), o_ref, "bf16", f"random {i} o")
        assert np.abs(host(lse) - lse_ref.reshape(-1)).max() <= 2e-2, i
        scale = np.sqrt(np.mean(dqkv_ref ** 2))
        for name, cols in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
            assert_close(host(dq)[:, cols], dqkv_ref[:, cols], "bf16", f"random {i} {name}", scale=scale)


@pytest.mark.parametrize("family", [0, 1, 2])
@pytest.mark.parametrize("dh,causal", [(128, True), (64, True), (128, False), (112, True), (48, False)])
def test_attention_launch_shapes(ctx, tune, family, dh, causal):
    """Every family of workgroup shapes (key/query splits, merges through LDS) on a ragged
    sequence that spans several streamed blocks; the library reads the override at each call.
    Head sizes 112 and 48 run in the 128- and 64-wide tiles with the remaining columns held at zero
    (112 = hidden 7168 over 64 heads, one of the paper's model shapes)."""
    tune(attn_shape=family)
    batch, seq, heads = 2, 333, 2
    h = heads * dh
    key = ("attn-shape", dh, causal)
    print("attention shape case", key, family, flush=True)
    qkv = mat(key + ("qkv",), (batch * seq, 3 * h), "bf16")
    d_o = mat(key + ("do",), (batch * seq, h), "bf16")
    q64 = qkv.astype(np.float64)
    o_ref, probs, lse_ref = OL.attention(q64, heads, causal, batch)
    dqkv_ref = OL.attention_input_grad(d_o.astype(np.float64), q64, probs, heads, batch)
    qd = dev(qkv, "bf16")
    o = dev(np.zeros((batch * seq, h)), "bf16")
    lse = torch.zeros(batch * heads * seq, device="cuda")
    P.pmc_attention_forward(ctx, qd, o, lse, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, "bf16", "")
    assert np.abs(host(lse) - lse_ref.reshape(-1)).max() <= 2e-2
    dq = dev(np.zeros_like(qkv), "bf16")
    P.pmc_attention_backward(ctx, qd, o, lse, dev(d_o, "bf16"), dq, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    for name, cols in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
        assert_close(host(dq)[:, cols], dqkv_ref[:, cols], "bf16", str(name), scale=np.sqrt(np.mean(dqkv_ref ** 2)))


@pytest.mark.parametrize("family", [0, 1])
def test_attention_long_sequence(ctx, tune, family):
    """Sequence length 4096 at head size 128 (the longest workload shape), four heads so that the
    oracle's probabilities fit in host memory: 32 to 64 streamed blocks per query block, the
    heaviest-first block order, both families of launch shapes."""
    tune(attn_shape=family)
    batch, seq, heads, dh = 1, 4096, 4, 128
    h = heads * dh
    key = ("attn-long",)
    print("attention long case", family, flush=True)
    qkv = mat(key + ("qkv",), (seq, 3 * h), "bf16")
    d_o = mat(key + ("do",), (seq, h), "bf16")
    q64 = qkv.astype(np.float64)
    o_ref, probs, lse_ref = OL.attention(q64, heads, True, batch)
    dqkv_ref = OL.attention_input_grad(d_o.astype(np.float64), q64, probs, heads, batch)
    del probs
    qd = dev(qkv, "bf16")
    o = dev(np.zeros((seq, h)), "bf16")
    lse = torch.zeros(heads * seq, device="cuda")
    P.pmc_attention_forward(ctx, qd, o, lse, batch, seq, heads, dh, True)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, "bf16", "")
    assert np.abs(host(lse) - lse_ref.reshape(-1)).max() <= 2e-2
    dq = dev(np.zeros_like(qkv), "bf16")
    P.pmc_attention_backward(ctx, qd, o, lse, dev(d_o, "bf16"), dq, batch, seq, heads, dh, True)
    torch.cuda.synchronize()
    for name, cols in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
        assert_close(host(dq)[:, cols], dqkv_ref[:, cols], "bf16", str(name), scale=np.sqrt(np.mean(dqkv_ref ** 2)))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("seq,heads", [(4096, 40), (2048, 32), (1024, 16)])
def test_attention_workload_shapes(ctx, seq, heads):
    """Attention at the full size of the three bf16 workloads (head size 128, causal), launched as the
    passes launch it (the library's own choice of workgroup shapes for that many heads and blocks).
    The dense oracle for all heads at once would need heads x seq^2 probabilities, so heads are checked
    one at a time, each as a one-head problem cut out of the packed q|k|v rows: output, log-sum-exp and
    all three input gradients, every element.  At the longest shape (4096 tokens, 40 heads) EVERY head
    is checked; at the two shorter ones the first, the last and one in between."""
    dh = 128
    h = heads * dh
    gen = torch.Generator(device="cuda").manual_seed(seq + heads)
    bf = torch.bfloat16
    qkv = torch.randn((seq, 3 * h), device="cuda", generator=gen).to(bf)
    d_o = torch.randn((seq, h), device="cuda", generator=gen).to(bf)
    o = torch.zeros((seq, h), device="cuda", dtype=bf)
    lse = torch.zeros(heads * seq, device="cuda")
    dq = torch.zeros_like(qkv)
    print("attention workload shape", seq, heads, flush=True)
    P.pmc_attention_forward(ctx, qkv, o, lse, 1, seq, heads, dh, True)
    P.pmc_attention_backward(ctx, qkv, o, lse, d_o, dq, 1, seq, heads, dh, True)
    torch.cuda.synchronize()
    lse_h = host(lse).reshape(heads, seq)
    for hd in (range(heads) if seq == 4096 else (0, heads // 2 + 1, heads - 1)):
        cols = [slice(part * h + hd * dh, part * h + (hd + 1) * dh) for part in range(3)]
        one = np.concatenate([host(qkv[:, c]) for c in cols], axis=1)              # [seq, 3 dh]: a one-head qkv
        o_ref, probs, lse_ref = OL.attention(one, 1, True, 1)
        g_ref = OL.attention_input_grad(host(d_o[:, hd * dh:(hd + 1) * dh]), one, probs, 1, 1)
        del probs
        assert_close(host(o[:, hd * dh:(hd + 1) * dh]), o_ref, "bf16", str(hd))
        assert np.abs(lse_h[hd] - lse_ref.reshape(-1)).max() <= 2e-2, hd
        for part, name in enumerate(("dq", "dk", "dv")):
            assert_close(host(dq[:, cols[part]]), g_ref[:, part * dh:(part + 1) * dh], "bf16", str((hd, name)), scale=np.sqrt(np.mean(g_ref ** 2)))


@pytest.mark.parametrize("family", [0, 1, 2])
@pytest.mark.parametrize("dh", [64, 128])
def test_attention_short_sequences(ctx, tune, family, dh):
    """Sequences shorter than one streamed block (a single query, a few, one 32-row tile plus
    one): every tile row past the end is a clamped copy of the last row and must be masked out."""
    tune(attn_shape=family)
    batch, heads = 2, 2
    h = heads * dh
    for seq in (1, 7, 33):
        key = ("attn-short", dh, seq)
        print("attention short case", key, family, flush=True)
        qkv = mat(key + ("qkv",), (batch * seq, 3 * h), "bf16")
        d_o = mat(key + ("do",), (batch * seq, h), "bf16")
        q64 = qkv.astype(np.float64)
        o_ref, probs, lse_ref = OL.attention(q64, heads, True, batch)
        dqkv_ref = OL.attention_input_grad(d_o.astype(np.float64), q64, probs, heads, batch)
        qd = dev(qkv, "bf16")
        o = dev(np.zeros((batch * seq, h)), "bf16")
        lse = torch.zeros(batch * heads * seq, device="cuda")
        P.pmc_attention_forward(ctx, qd, o, lse, batch, seq, heads, dh, True)
        torch.cuda.synchronize()
        assert_close(host(o), o_ref, "bf16", str(seq))
        assert np.abs(host(lse) - lse_ref.reshape(-1)).max() <= 2e-2, seq
        dq = dev(np.zeros_like(qkv), "bf16")
        P.pmc_attention_backward(ctx, qd, o, lse, dev(d_o, "bf16"), dq, batch, seq, heads, dh, True)
        torch.cuda.synchronize()
        for name, cols in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
            assert_close(host(dq)[:, cols], dqkv_ref[:, cols], "bf16", str((seq, name)), scale=np.sqrt(np.mean(dqkv_ref ** 2)))


@pytest.mark.parametrize("family", [0, 1])
@pytest.mark.parametrize("causal", [True, False])
def test_attention_sharp_softmax(ctx, tune, family, causal):
    """Queries and keys three times larger (scores with a standard deviation of 9, 13 in log2
    units): row maxima keep rising from block to block by more and by less than the slack the
    forward kernel allows before it moves its softmax reference, so both branches of the online
    softmax and their mix inside one wave are exercised."""
    tune(attn_shape=family)
    batch, seq, heads, dh = 1, 700, 2, 128
    h = heads * dh
    key = ("attn-sharp", causal)
    print("attention sharp case", key, family, flush=True)
    qkv = mat(key + ("qkv",), (batch * seq, 3 * h), "bf16").copy()
    qkv[:, :2 * h] *= 3.0
    d_o = mat(key + ("do",), (batch * seq, h), "bf16")
    qkv = host(dev(qkv, "bf16"))                             # exactly what the device holds after rounding
    q64 = qkv.astype(np.float64)
    o_ref, probs, lse_ref = OL.attention(q64, heads, causal, batch)
    dqkv_ref = OL.attention_input_grad(d_o.astype(np.float64), q64, probs, heads, batch)
    qd = dev(qkv, "bf16")
    o = dev(np.zeros((batch * seq, h)), "bf16")
    lse = torch.zeros(batch * heads * seq, device="cuda")
    P.pmc_attention_forward(ctx, qd, o, lse, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, "bf16", "")
    assert np.abs(host(lse) - lse_ref.reshape(-1)).max() <= 2e-2
    dq = dev(np.zeros_like(qkv), "bf16")
    P.pmc_attention_backward(ctx, qd, o, lse, dev(d_o, "bf16"), dq, batch, seq, heads, dh, causal)
    torch.cuda.synchronize()
    for name, cols in (("dq", slice(0, h)), ("dk", slice(h, 2 * h)), ("dv", slice(2 * h, 3 * h))):
        assert_close(host(dq)[:, cols], dqkv_ref[:, cols], "bf16", str(name), scale=np.sqrt(np.mean(dqkv_ref ** 2)))


def test_attention_rejects_rows_beyond_the_load_window(ctx):
    """The matrix-core kernels address one sequence's q|k|v rows with 32-bit offsets in a 2 GB
    window: a sequence whose rows exceed it is refused before anything is launched."""
    seq, heads, dh = 32768, 128, 128                    # 32768 rows of 96 KiB = 3 GiB
    small = torch.zeros(1024, device="cuda", dtype=torch.bfloat16)
    lse = torch.zeros(16, device="cuda")
    with pytest.raises(P.PmcError) as e:
        P.pmc_attention_forward(ctx, small, small, lse, 1, seq, heads, dh, True)
    assert "2 GB" in str(e.value)
    with pytest.raises(P.PmcError):
        P.pmc_attention_backward(ctx, small, small, lse, small, small, 1, seq, heads, dh, True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_column_sum(ctx, dtype):
    for rows, n in ((1, 8), (50, 264), (1000, 2048), (300, 6144)):
        a = mat(("cs", dtype, rows, n), (rows, n), dtype)
        out = torch.full((n,), 2.0, device="cuda")
        P.pmc_column_sum(ctx, dev(a, dtype), out)
        torch.cuda.synchronize()
        assert np.abs(host(out) - 2.0 - a.astype(np.float64).sum(0)).max() <= 1e-4 * max(1.0, np.sqrt(rows))
