"""GPU parity: the HIP path, called through the C-ABI, against the fp64 oracle on the same seeded inputs.

Tolerances (relative L2 on whole vectors, |df|/|f| on the objective): 1e-4 for f, grad f and G v;
1e-3 for CG iterates after <= 10 iterations.  fp32 arithmetic with fp32 MFMA accumulation over at most
a few thousand terms keeps rounding near 1e-6, so these bars leave room only for rounding, not for a
dropped term.
"""
import numpy as np
import pytest
import torch

import dn_inputs
import paper_1802_00130_amd as dn
from oracle import dn_oracle as orc
from tests.gpu_common import Workload, assert_close_blocks, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-4
TOL_CG = 1e-3

SMALL = {
    "cfg1": lambda: dn_inputs.config(1),
    # odd widths: unaligned theta slices, scalar load paths, ragged tiles everywhere
    "odd_5-3-2": lambda: dn_inputs.custom((5, 3, 2), l=37, s=11, C=0.9, seed=11),
    "odd_7-5-6-3": lambda: dn_inputs.custom((7, 5, 6, 3), l=150, s=67, C=2.0, seed=12),
    # no hidden layer, one hidden layer, four hidden layers
    "L1_9-4": lambda: dn_inputs.custom((9, 4), l=80, s=33, C=1.5, seed=13),
    "L2_12-10-5": lambda: dn_inputs.custom((12, 10, 5), l=90, s=40, C=1.0, seed=14),
    "L5_10-9-8-7-6-3": lambda: dn_inputs.custom((10, 9, 8, 7, 6, 3), l=100, s=50, C=3.0, seed=15),
    # several 64-tiles with ragged tails in every dimension; n_L > 16 takes the two-pass kernels
    "ragged_70-133-45-19": lambda: dn_inputs.custom((70, 133, 45, 19), l=333, s=131, C=10.0, seed=16),
    # wide enough for 128-tiles and split sums, normal features
    "mid_200-300-260-10": lambda: dn_inputs.custom((200, 300, 260, 10), l=2100, s=700, C=50.0,
                                                   features="normal3", seed=17),
    # two-pass path (n_L > 16) with one hidden layer (no stored block at all) and with four
    "twopass_L2_9-14-20": lambda: dn_inputs.custom((9, 14, 20), l=70, s=37, C=1.2, seed=19),
    "twopass_L5_10-9-8-7-11-24": lambda: dn_inputs.custom((10, 9, 8, 7, 11, 24), l=90, s=41, C=2.5, seed=20),
    # single output (the paper's two-class setting uses n_L = 1)
    "nL1_16-12-1": lambda: dn_inputs.custom((16, 12, 1), l=64, s=30, C=1.0, seed=18),
}


@pytest.fixture(scope="module", params=sorted(SMALL))
def wl(request):
    print(f"[case] {request.param}", flush=True)
    w = Workload(SMALL[request.param](), bias_scale=0.3)
    yield w
    w.ctx.close()


def test_forward_objective(wl):
    cfg = wl.cfg
    ZL = torch.empty(wl.l, cfg.dims[-1], dtype=torch.float32, device="cuda:0")
    f = dn.dn_forward(wl.ctx, wl.dtheta, wl.dX, wl.dY, ZL)
    th = wl.theta.astype(np.float64)
    f_ref = orc.loss(th, cfg.dims, cfg.C, wl.X.astype(np.float64), wl.Y.astype(np.float64))
    assert abs(f - f_ref) <= TOL * abs(f_ref)
    Z_ref = orc.forward(th, cfg.dims, wl.X.astype(np.float64))[-1]
    assert rel_l2(ZL.cpu().numpy(), Z_ref) <= TOL


def test_gradient(wl):
    cfg = wl.cfg
    g = wl.empty()
    f = dn.dn_grad(wl.ctx, wl.dtheta, wl.dX, wl.dY, g)
    g_ref, f_ref = orc.grad(wl.theta.astype(np.float64), cfg.dims, cfg.C, wl.X.astype(np.float64),
                            wl.Y.astype(np.float64))
    assert abs(f - f_ref) <= TOL * abs(f_ref)
    assert rel_l2(g.cpu().numpy(), g_ref) <= TOL


def test_stored_jacobian_blocks(wl):
    cfg = wl.cfg
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    P_ref = orc.jacobian_blocks(wl.theta.astype(np.float64), cfg.dims, wl.XS64)
    for m in range(1, cfg.L):
        P = torch.empty(wl.s, cfg.dims[-1], cfg.dims[m], dtype=torch.float32, device="cuda:0")
        dn.dn_jacobian_read(wl.ctx, m, P)
        assert rel_l2(P.cpu().numpy(), P_ref[m - 1]) <= TOL, f"P^{m}"


@pytest.mark.parametrize("mode", [dn.DN_FULL, dn.DN_BLOCKDIAG])
def test_gn_matvec(wl, mode):
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    for k in range(2):
        v = dn_inputs.make_probe(wl.cfg, k)
        out = wl.empty()
        dn.dn_gn_matvec(wl.ctx, wl.dev(v), out, mode)
        ref = wl.oracle_matvec(v, blockdiag=(mode == dn.DN_BLOCKDIAG))
        assert rel_l2(out.cpu().numpy(), ref) <= TOL


def test_gn_matvec_is_deterministic_and_symmetric(wl):
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    v = wl.dev(dn_inputs.make_probe(wl.cfg, 0))
    w = wl.dev(dn_inputs.make_probe(wl.cfg, 1))
    a, b, c = wl.empty(), wl.empty(), wl.empty()
    dn.dn_gn_matvec(wl.ctx, v, a, dn.DN_FULL)
    dn.dn_gn_matvec(wl.ctx, v, b, dn.DN_FULL)
    dn.dn_gn_matvec(wl.ctx, w, c, dn.DN_FULL)
    assert torch.equal(a, b)
    wGv = float((w.double() @ a.double()).item())
    vGw = float((v.double() @ c.double()).item())
    assert abs(wGv - vGw) <= 1e-4 * max(abs(wGv), abs(vGw))
    assert float((v.double() @ a.double()).item()) >= float((v.double() @ v.double()).item()) / wl.cfg.C * (1 - 1e-5)


@pytest.mark.parametrize("mode", [dn.DN_FULL, dn.DN_BLOCKDIAG])
def test_cg_fixed_iterations(wl, mode):
    cfg = wl.cfg
    th = wl.theta.astype(np.float64)
    g_ref, _ = orc.grad(th, cfg.dims, cfg.C, wl.X.astype(np.float64), wl.Y.astype(np.float64))
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    iters = min(cfg.cg_iters, 10)
    d = wl.empty()
    it, res = dn.dn_cg(wl.ctx, wl.dev(g_ref), cfg.lam, 0.0, iters, mode, d)
    bd = mode == dn.DN_BLOCKDIAG
    d_ref, it_ref, res_ref = orc.cg(th, cfg.dims, cfg.C, wl.XS64, g_ref.astype(np.float32).astype(np.float64),
                                    cfg.lam, iters, sigma=0.0, blockdiag=bd)
    assert it == it_ref == iters
    assert rel_l2(d.cpu().numpy(), d_ref) <= TOL_CG
    assert len(res) == len(res_ref)
    gn = np.linalg.norm(g_ref)
    for a, b in zip(res, res_ref):
        assert abs(a - b) <= 1e-3 * gn


@pytest.mark.parametrize("mode", [dn.DN_FULL, dn.DN_BLOCKDIAG])
def test_cg_stopping_rule(wl, mode):
    cfg = wl.cfg
    th = wl.theta.astype(np.float64)
    g_ref, _ = orc.grad(th, cfg.dims, cfg.C, wl.X.astype(np.float64), wl.Y.astype(np.float64))
    g32 = g_ref.astype(np.float32)
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    sigma = 0.05
    d = wl.empty()
    it, res = dn.dn_cg(wl.ctx, wl.dev(g32), cfg.lam, sigma, 60, mode, d)
    bd = mode == dn.DN_BLOCKDIAG
    blocks = orc.block_slices(cfg.dims) if bd else [slice(0, wl.n)]
    # every system met its test within the limit, and the recomputed residual agrees with the reported one
    prod = orc.gn_matvec_blockdiag if bd else orc.gn_matvec
    dd = d.cpu().numpy().astype(np.float64)
    true_res = prod(th, cfg.dims, cfg.C, wl.XS64, dd) + cfg.lam * dd + g32.astype(np.float64)
    assert it < 60
    for k, b in enumerate(blocks):
        gnorm = np.linalg.norm(g32[b].astype(np.float64))
        assert res[k] <= sigma * gnorm * (1 + 1e-6)
        assert abs(np.linalg.norm(true_res[b]) - res[k]) <= 2e-3 * gnorm
    d_ref, it_ref, _ = orc.cg(th, cfg.dims, cfg.C, wl.XS64, g32.astype(np.float64), cfg.lam, 60, sigma=sigma,
                              blockdiag=bd)
    # the stop decision sits on a rounding-sensitive threshold: allow one iteration of slack
    assert abs(it - it_ref) <= 1
    if it == it_ref:
        assert rel_l2(dd, d_ref) <= 5e-3


def test_zero_gradient_and_error_paths(wl):
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    d = wl.empty()
    it, res = dn.dn_cg(wl.ctx, torch.zeros_like(d), 1.0, 0.0, 5, dn.DN_FULL, d)
    assert it == 0 and res == [0.0] and float(d.abs().max()) == 0.0
    with pytest.raises(dn.DnError):
        dn.dn_gn_matvec(wl.ctx, d, wl.empty(), 7)
    with pytest.raises(dn.DnError):
        dn.dn_cg(wl.ctx, d, 1.0, 0.0, 0, dn.DN_FULL, wl.empty())


@pytest.mark.parametrize("l_max", [64, 100, 333, 1000])
def test_chunked_objective_and_gradient(l_max):
    """Section 6.1 pipeline: the samples go through in chunks of l_max rows that reuse the activation buffers;
    f and the gradient must be the same sums (chunk sizes that divide l, that leave a ragged last chunk, that
    equal l, and that exceed l)."""
    cfg = dn_inputs.custom((70, 133, 45, 19), l=333, s=131, C=10.0, seed=16)
    X, Y = dn_inputs.make_X(cfg), dn_inputs.make_Y(cfg)
    theta = dn_inputs.make_theta(cfg, bias_scale=0.3)
    dev = "cuda:0"
    dX, dY, dth = (torch.from_numpy(a).to(dev) for a in (X, Y, theta))
    ctx = dn.Context(cfg.dims, cfg.C, l_max, cfg.s)
    g = torch.empty(ctx.n, dtype=torch.float32, device=dev)
    ZL = torch.empty(cfg.l, cfg.dims[-1], dtype=torch.float32, device=dev)
    th64, X64, Y64 = theta.astype(np.float64), X.astype(np.float64), Y.astype(np.float64)
    g_ref, f_ref = orc.grad(th64, cfg.dims, cfg.C, X64, Y64)
    f = dn.dn_forward(ctx, dth, dX, dY, ZL)
    assert abs(f - f_ref) <= TOL * abs(f_ref)
    assert rel_l2(ZL.cpu().numpy(), orc.forward(th64, cfg.dims, X64)[-1]) <= TOL
    f2 = dn.dn_grad(ctx, dth, dX, dY, g)
    assert abs(f2 - f_ref) <= TOL * abs(f_ref)
    assert rel_l2(g.cpu().numpy(), g_ref) <= TOL
    # a Newton step whose f and gradient are chunked gives the same step as the oracle
    S = torch.from_numpy(dn_inputs.make_subset(cfg)).to(dev)
    d_prev = torch.zeros_like(g)
    th_new = dth.clone()
    out = dn.dn_newton_step(ctx, th_new, dX, dY, S, d_prev, 1.0, 6, sigma=0.0)
    ref = orc.newton_step(th64, cfg.dims, cfg.C, X64, Y64, dn_inputs.make_subset(cfg), np.zeros(ctx.n), 1.0, 6, sigma=0.0)
    assert out["alpha"] == ref["alpha"] and abs(out["f_new"] - ref["f_new"]) <= TOL * abs(ref["f_new"])
    ctx.close()


@pytest.mark.parametrize("init", ["sparse", "dense"])
def test_paper_initialisations(init):
    """Gradient and both products at the paper's own initial points (Section 6.2 sparse, Section 8.2 dense)."""
    cfg = dn_inputs.custom((200, 300, 260, 10), l=600, s=200, C=600.0, seed=17)
    w = Workload(cfg)
    w.theta = dn_inputs.make_theta(cfg, init=init)
    w.dtheta = torch.from_numpy(w.theta).to("cuda:0")
    g = w.empty()
    f = dn.dn_grad(w.ctx, w.dtheta, w.dX, w.dY, g)
    g_ref, f_ref = orc.grad(w.theta.astype(np.float64), cfg.dims, cfg.C, w.X.astype(np.float64), w.Y.astype(np.float64))
    assert abs(f - f_ref) <= TOL * abs(f_ref) and rel_l2(g.cpu().numpy(), g_ref) <= TOL
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(cfg, 0)
    out = w.empty()
    for mode in (dn.DN_FULL, dn.DN_BLOCKDIAG):
        dn.dn_gn_matvec(w.ctx, w.dev(v), out, mode)
        assert rel_l2(out.cpu().numpy(), w.oracle_matvec(v, blockdiag=(mode == dn.DN_BLOCKDIAG))) <= TOL
    w.ctx.close()


def test_product_without_stored_blocks(wl):
    """dn_gn_matvec_rop (forward-mode pass + back-propagation, no stored blocks) gives the same G^S v as the oracle
    and as the product from the stored blocks: two independent device paths to one result."""
    dn.dn_jacobian_prep(wl.ctx, wl.dtheta, wl.dX, wl.dS)
    v = dn_inputs.make_probe(wl.cfg, 1)
    a, b = wl.empty(), wl.empty()
    dn.dn_gn_matvec_rop(wl.ctx, wl.dev(v), a)
    dn.dn_gn_matvec(wl.ctx, wl.dev(v), b, dn.DN_FULL)
    ref = wl.oracle_matvec(v)
    assert rel_l2(a.cpu().numpy(), ref) <= TOL
    assert rel_l2(a.cpu().numpy(), b.cpu().numpy()) <= TOL


def test_products_keep_the_prepared_theta_after_a_gradient_elsewhere():
    """Both products belong to the theta handed to dn_jacobian_prep.  A gradient evaluated afterwards at another
    theta (it shares workspace buffers with the products, the transposed weights among them) changes neither."""
    cfg = dn_inputs.custom((23, 70, 90, 40, 11), l=150, s=60, C=5.0, seed=31)
    w = Workload(cfg)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    other = torch.from_numpy(dn_inputs.make_theta(dn_inputs.custom(cfg.dims, l=cfg.l, s=cfg.s, C=cfg.C, seed=32))).to("cuda:0")
    assert not torch.equal(other, w.dtheta)
    dn.dn_grad(w.ctx, other, w.dX, w.dY, w.empty())
    v = dn_inputs.make_probe(cfg, 2)
    ref = w.oracle_matvec(v)
    a, b = w.empty(), w.empty()
    for _ in range(2):
        dn.dn_gn_matvec_rop(w.ctx, w.dev(v), a)
        dn.dn_gn_matvec(w.ctx, w.dev(v), b, dn.DN_FULL)
        assert rel_l2(a.cpu().numpy(), ref) <= TOL
        assert rel_l2(b.cpu().numpy(), ref) <= TOL
    w.ctx.close()


def test_subsample_edge_cases():
    """Repeated row ids count twice (the product is a plain sum over the list), a subsample of one row, the
    subsample equal to all rows, and s below s_max after a larger one (the workspace keeps no stale rows)."""
    cfg = dn_inputs.custom((7, 5, 6, 3), l=40, s=40, C=2.0, seed=12)
    X, Y = dn_inputs.make_X(cfg), dn_inputs.make_Y(cfg)
    theta = dn_inputs.make_theta(cfg, bias_scale=0.3)
    dev = "cuda:0"
    dX, dth = torch.from_numpy(X).to(dev), torch.from_numpy(theta).to(dev)
    ctx = dn.Context(cfg.dims, cfg.C, cfg.l, cfg.s)
    v = dn_inputs.make_probe(cfg, 0)
    dv = torch.from_numpy(v).to(dev)
    out = torch.empty(ctx.n, dtype=torch.float32, device=dev)
    th64, X64 = theta.astype(np.float64), X.astype(np.float64)
    for S in (np.arange(40), np.array([3, 3, 3, 17, 17, 0]), np.array([39]), np.array([5, 9, 5])):
        S = S.astype(np.int32)
        dn.dn_jacobian_prep(ctx, dth, dX, torch.from_numpy(S).to(dev))
        for mode, fn in ((dn.DN_FULL, orc.gn_matvec), (dn.DN_BLOCKDIAG, orc.gn_matvec_blockdiag)):
            dn.dn_gn_matvec(ctx, dv, out, mode)
            assert rel_l2(out.cpu().numpy(), fn(th64, cfg.dims, cfg.C, X64[S], v.astype(np.float64))) <= TOL
    ctx.close()


WIDE = {
    # n_L <= 12, hidden widths 4096 < total <= 8192: the fused kernel with two strips per wave
    "fused2_16-2500-2100-10": lambda: dn_inputs.custom((16, 2500, 2100, 10), l=40, s=12, C=4.0, seed=81),
    "fused2_12-4100-3": lambda: dn_inputs.custom((12, 4100, 3), l=30, s=9, C=2.0, seed=82),
    # n_L <= 16 but too wide for the fused kernel: teams of work-groups share a sample (two hidden layers or more) ...
    "band_small_nL_8-5000-4000-6": lambda: dn_inputs.custom((8, 5000, 4000, 6), l=30, s=8, C=3.0, seed=83),
    # ... and with one hidden layer nothing is streamed at all (block L-1 is applied as dense products)
    "twopass_small_nL_10-8500-5": lambda: dn_inputs.custom((10, 8500, 5), l=30, s=8, C=3.0, seed=84),
    # 12 < n_L <= 16 with more than 4096 hidden columns: no fused variant
    "band_nL14_9-3000-1500-14": lambda: dn_inputs.custom((9, 3000, 1500, 14), l=30, s=8, C=3.0, seed=85),
}


@pytest.mark.parametrize("name", sorted(WIDE))
def test_wide_hidden_layers_small_output(name):
    print(f"[case] {name}", flush=True)
    w = Workload(WIDE[name](), bias_scale=0.3)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(w.cfg, 0)
    out = w.empty()
    w.ctx.profile_enable(True)
    w.ctx.profile_reset()
    for mode in (dn.DN_FULL, dn.DN_BLOCKDIAG):
        dn.dn_gn_matvec(w.ctx, w.dev(v), out, mode)
        err = rel_l2(out.cpu().numpy(), w.oracle_matvec(v, blockdiag=(mode == dn.DN_BLOCKDIAG)))
        print(f"  mode {mode}: rel err {err:.2e}", flush=True)
        assert err <= TOL
    prof = w.ctx.profile_read()
    assert (prof["jv_jtv_fused"][1] == 2) == name.startswith("fused2")
    assert (prof["jv_rows"][1] == 2) == name.startswith("twopass")
    assert (prof["jv_jtv_band"][1] == 2) == name.startswith("band")
    w.ctx.close()


def test_large_tiles_with_ragged_edges():
    """Launches big enough for the 128 x 128 tiles of the GEMM engine (whole rounds of two work-groups per CU), with
    ragged edges in every dimension: 32700 rows (255.5 tiles), 1150 columns (8.98 tiles), sums over 270 and 530 terms
    (neither a multiple of the K-tile), the bias + sigmoid epilogue (forward), the sigma' epilogue (back-propagation)
    and the sigma' epilogue with one activation row per n_L output rows (the sweeps over the stored blocks,
    818 * 40 = 32720 rows)."""
    cfg = dn_inputs.custom((270, 1150, 530, 40), l=32700, s=818, C=100.0, seed=86)
    w = Workload(cfg, bias_scale=0.3)
    th, X64, Y64 = w.theta.astype(np.float64), w.X.astype(np.float64), w.Y.astype(np.float64)
    ZL = torch.empty(w.l, cfg.dims[-1], dtype=torch.float32, device="cuda:0")
    f = dn.dn_forward(w.ctx, w.dtheta, w.dX, w.dY, ZL)
    g = w.empty()
    f2 = dn.dn_grad(w.ctx, w.dtheta, w.dX, w.dY, g)
    g_ref, f_ref = orc.grad(th, cfg.dims, cfg.C, X64, Y64)
    assert abs(f - f_ref) <= TOL * abs(f_ref) and abs(f2 - f_ref) <= TOL * abs(f_ref)
    assert rel_l2(ZL.cpu().numpy(), orc.forward(th, cfg.dims, X64)[-1]) <= TOL
    whole, worst = assert_close_blocks(g.cpu().numpy(), g_ref, cfg.dims, TOL, "gradient")
    print(f"  gradient: rel err {whole:.2e}, worst block {worst}", flush=True)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    P_ref = orc.jacobian_blocks(th, cfg.dims, w.XS64)
    for m in range(1, cfg.L):
        P = torch.empty(w.s, cfg.dims[-1], cfg.dims[m], dtype=torch.float32, device="cuda:0")
        dn.dn_jacobian_read(w.ctx, m, P)
        err = rel_l2(P.cpu().numpy(), P_ref[m - 1])
        print(f"  P^{m}: rel err {err:.2e}", flush=True)
        assert err <= TOL, f"P^{m}"
    w.ctx.close()


def test_sums_over_samples_with_transposed_left_operand():
    """A product whose sums over samples are large enough for the 128 x 128 tiles (512 of them: 4040 x 1858 and
    10 x 4041, ragged in both dimensions): the left operands T^m are then transposed first and both operands read
    K-contiguously.  Sums over 70 samples (four K-tiles and a ragged fifth), then over 37 of the 70 the context was
    created for (the transposed buffers keep the row stride of the largest subsample)."""
    cfg = dn_inputs.custom((1857, 4040, 10), l=100, s=70, C=20.0, seed=87)
    w = Workload(cfg, bias_scale=0.3)
    th64 = w.theta.astype(np.float64)
    out = w.empty()
    for S in (w.S, w.S[5:42]):
        dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, torch.from_numpy(np.ascontiguousarray(S)).to("cuda:0"))
        XS = w.X[S].astype(np.float64)
        v = dn_inputs.make_probe(cfg, 1)
        for mode, fn in ((dn.DN_FULL, orc.gn_matvec), (dn.DN_BLOCKDIAG, orc.gn_matvec_blockdiag)):
            ref = fn(th64, cfg.dims, cfg.C, XS, v.astype(np.float64))
            out.fill_(float("nan"))
            dn.dn_gn_matvec(w.ctx, w.dev(v), out, mode)
            whole, worst = assert_close_blocks(out.cpu().numpy(), ref, cfg.dims, TOL, f"mode {mode}")
            print(f"  {len(S)} samples, mode {mode}: rel err {whole:.2e}, worst block {worst}", flush=True)
        out.fill_(float("nan"))
        dn.dn_gn_matvec_rop(w.ctx, w.dev(v), out)
        assert_close_blocks(out.cpu().numpy(), orc.gn_matvec(th64, cfg.dims, cfg.C, XS, v.astype(np.float64)), cfg.dims,
                            TOL, "product without stored blocks")
    w.ctx.close()


def test_two_contexts_on_two_streams():
    """Two contexts for different networks, each bound to a stream of its own (default priority), with their
    calls interleaved from the host: every result matches the oracle, so nothing is shared between contexts
    and all work of a context stays on its stream."""
    cfg_a = dn_inputs.custom((30, 20, 12, 4), l=300, s=90, C=6.0, seed=71)
    # n_L > 16, two hidden layers, the streamed one wider than one column slice: the single-pass kernel whose
    # work-groups (two per team here) wait for each other runs beside the other stream's kernels
    cfg_b = dn_inputs.custom((18, 1100, 40, 35), l=260, s=70, C=2.0, seed=72)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    work = []
    for cfg, st in zip((cfg_a, cfg_b), streams):
        X, Y = dn_inputs.make_X(cfg), dn_inputs.make_Y(cfg)
        theta, S, v = dn_inputs.make_theta(cfg, bias_scale=0.3), dn_inputs.make_subset(cfg), dn_inputs.make_probe(cfg, 0)
        t = lambda a: torch.from_numpy(a).to("cuda:0")
        ctx = dn.Context(cfg.dims, cfg.C, cfg.l, cfg.s, stream=st)
        work.append(dict(cfg=cfg, ctx=ctx, st=st, X=X, Y=Y, theta=theta, S=S, v=v, dX=t(X), dY=t(Y), dth=t(theta),
                         dS=t(S), dv=t(v)))
    torch.cuda.synchronize()
    for w in work:
        for k in ("g", "out_full", "out_bd", "d"):
            w[k] = torch.empty(w["ctx"].n, dtype=torch.float32, device="cuda:0")
    # interleave: the same step of both contexts back to back, no synchronisation in between
    for w in work:
        dn.dn_grad(w["ctx"], w["dth"], w["dX"], w["dY"], w["g"], want_f=False)
    for w in work:
        dn.dn_jacobian_prep(w["ctx"], w["dth"], w["dX"], w["dS"])
    for _ in range(3):
        for w in work:
            dn.dn_gn_matvec(w["ctx"], w["dv"], w["out_full"], dn.DN_FULL)
            dn.dn_gn_matvec(w["ctx"], w["dv"], w["out_bd"], dn.DN_BLOCKDIAG)
    for w in work:
        w["iters"], _ = dn.dn_cg(w["ctx"], w["g"], 1.0, 0.0, 5, dn.DN_FULL, w["d"])
    for st in streams:
        st.synchronize()
    for w in work:
        cfg = w["cfg"]
        th64, X64, Y64 = w["theta"].astype(np.float64), w["X"].astype(np.float64), w["Y"].astype(np.float64)
        XS = X64[w["S"]]
        g_ref, _ = orc.grad(th64, cfg.dims, cfg.C, X64, Y64)
        assert rel_l2(w["g"].cpu().numpy(), g_ref) <= TOL
        v64 = w["v"].astype(np.float64)
        assert rel_l2(w["out_full"].cpu().numpy(), orc.gn_matvec(th64, cfg.dims, cfg.C, XS, v64)) <= TOL
        assert rel_l2(w["out_bd"].cpu().numpy(), orc.gn_matvec_blockdiag(th64, cfg.dims, cfg.C, XS, v64)) <= TOL
        g32 = w["g"].cpu().numpy().astype(np.float64)
        d_ref, _, _ = orc.cg(th64, cfg.dims, cfg.C, XS, g32, 1.0, 5)
        assert w["iters"] == 5 and rel_l2(w["d"].cpu().numpy(), d_ref) <= 1e-3
        w["ctx"].close()
