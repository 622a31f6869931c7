"""GPU parity at the full sizes of the benchmark configurations, in the launch shapes bench.py times.

Configurations 2 and 3 are checked whole: f, gradient, both products, 10 CG iterations.  Configurations 4 and 5
(5 is the benchmarked one) check both products whole (every entry of G v against the oracle), 10 CG iterations of
the full system, and f and the gradient on the first 20000 rows (the oracle's gradient over all l rows of those
two takes many minutes on the host); DN_TEST_LIGHT=1 skips their CG and block-diagonal legs.
Products and gradients are compared block by block (every A^m and b^m on its own) as well as whole.
The rows beyond the headline path at the same sizes: the product over the partitions of the split structure
1-2-...-2-1 (single-pass and two-pass kernels) and 6 CG iterations over them at configurations 2-4, that product at
configuration 5, the joint early termination at configuration 3, and two outer Newton iterations (20 CG
iterations, combination with the previous direction, the second one reusing the forward pass) at 2 and 3.
"""
import os

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
HEAVY = os.environ.get("DN_TEST_LIGHT", "0") != "1"


def _check_products(w, modes=(dn.DN_FULL, dn.DN_BLOCKDIAG)):
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(w.cfg, 0)
    dv = w.dev(v)
    for mode in modes:
        out = w.empty()
        dn.dn_gn_matvec(w.ctx, dv, out, mode)
        ref = w.oracle_matvec(v, blockdiag=(mode == dn.DN_BLOCKDIAG))
        err, worst = assert_close_blocks(out.cpu().numpy(), ref, w.cfg.dims, TOL, f"{w.cfg.name} mode {mode}")
        print(f"[{w.cfg.name}] mode {mode}: rel err {err:.2e}, worst block {worst[0]} {worst[1]:.2e}", flush=True)
        again = w.empty()
        dn.dn_gn_matvec(w.ctx, dv, again, mode)
        assert torch.equal(out, again)
        if mode == dn.DN_FULL:
            # the same product without the stored blocks (forward-mode pass + back-propagation)
            dn.dn_gn_matvec_rop(w.ctx, dv, again)
            err, worst = assert_close_blocks(again.cpu().numpy(), ref, w.cfg.dims, TOL, f"{w.cfg.name} rop")
            print(f"[{w.cfg.name}] without stored blocks: rel err {err:.2e}, worst block {worst[0]} {worst[1]:.2e}",
                  flush=True)


def _check_grad(w):
    cfg = w.cfg
    g = w.empty()
    f = dn.dn_grad(w.ctx, w.dtheta, w.dX, w.dY, g)
    g_ref, f_ref = orc.grad(w.theta.astype(np.float64), cfg.dims, cfg.C, w.X.astype(np.float64),
                            w.Y.astype(np.float64))
    f2 = dn.dn_forward(w.ctx, w.dtheta, w.dX, w.dY)
    assert abs(f - f_ref) <= TOL * abs(f_ref) and abs(f2 - f_ref) <= TOL * abs(f_ref)
    err, worst = assert_close_blocks(g.cpu().numpy(), g_ref, cfg.dims, TOL, f"{cfg.name} gradient")
    print(f"[{cfg.name}] f {f:.8f} ref {f_ref:.8f}; grad rel err {err:.2e}, worst block {worst[0]} {worst[1]:.2e}",
          flush=True)
    return g_ref


def _check_cg(w, g_ref, modes, iters=10):
    cfg = w.cfg
    th = w.theta.astype(np.float64)
    g32 = g_ref.astype(np.float32)
    for mode in modes:
        d = w.empty()
        it, res = dn.dn_cg(w.ctx, w.dev(g32), cfg.lam, 0.0, iters, mode, d)
        d_ref, it_ref, res_ref = orc.cg(th, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), cfg.lam, iters,
                                        blockdiag=(mode == dn.DN_BLOCKDIAG))
        err = rel_l2(d.cpu().numpy(), d_ref)
        print(f"[{cfg.name}] cg mode {mode}: {it} iterations, rel err {err:.2e}", flush=True)
        assert it == it_ref == iters
        assert err <= TOL_CG


def _split_of(cfg):
    """Every hidden layer in two neuron groups, input and output layer whole (Section 3.1; the structure bench.py
    times under --extras)."""
    return tuple(1 if m in (0, cfg.L) else 2 for m in range(cfg.L + 1))


def _check_partitions(w, g_ref, cg_iters):
    """Product over the partitions with both kernel choices, then CG over the partitions."""
    cfg = w.cfg
    split = _split_of(cfg)
    th = w.theta.astype(np.float64)
    nparts = w.ctx.set_split(split)
    v = dn_inputs.make_probe(cfg, 1)
    ref = orc.gn_matvec_partitioned(th, cfg.dims, cfg.C, w.XS64, v.astype(np.float64), split)
    out = w.empty()
    for passes in (0, 2):
        w.ctx.set_stream_passes(passes)
        out.fill_(float("nan"))
        dn.dn_gn_matvec(w.ctx, w.dev(v), out, dn.DN_PARTITION)
        assert w.ctx.sync_status() == 0
        err, worst = assert_close_blocks(out.cpu().numpy(), ref, cfg.dims, TOL, f"{cfg.name} partitions, passes {passes}")
        print(f"[{cfg.name}] split {split} ({nparts} partitions), passes {passes}: rel err {err:.2e}, worst block "
              f"{worst[0]} {worst[1]:.2e}", flush=True)
    w.ctx.set_stream_passes(0)
    if cg_iters:
        g32 = g_ref.astype(np.float32)
        d = w.empty()
        it, res = dn.dn_cg(w.ctx, w.dev(g32), cfg.lam, 0.0, cg_iters, dn.DN_PARTITION, d)
        d_ref, it_ref, _ = orc.cg(th, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), cfg.lam, cg_iters, blockdiag=True,
                                  split=split)
        err = rel_l2(d.cpu().numpy(), d_ref)
        print(f"[{cfg.name}] cg over {nparts} partitions: {it} iterations, rel err {err:.2e}", flush=True)
        assert it == it_ref == cg_iters and len(res) == nparts
        assert err <= TOL_CG


def _check_newton(w, steps=2, cg_max=20):
    """Outer iterations from the initial point, each compared with the oracle restarted from the device's
    theta and previous direction; the second one takes its forward pass from the first one's line search."""
    cfg = w.cfg
    X64, Y64 = w.X.astype(np.float64), w.Y.astype(np.float64)
    theta = w.dtheta.clone()
    d_prev = torch.zeros_like(theta)
    lam = cfg.lam
    for k in range(steps):
        S = np.random.default_rng(cfg.seed * 1000 + k).permutation(cfg.l)[:cfg.s].astype(np.int32)
        th_in = theta.cpu().numpy().astype(np.float64)
        dp_in = d_prev.cpu().numpy().astype(np.float64)
        out = dn.dn_newton_step(w.ctx, theta, w.dX, w.dY, torch.from_numpy(S).to("cuda:0"), d_prev, lam, cg_max,
                                sigma=0.0, mode=dn.DN_FULL, reuse_forward=(k > 0))
        ref = orc.newton_step(th_in, cfg.dims, cfg.C, X64, Y64, S, dp_in, lam, cg_max, sigma=0.0)
        e_d = rel_l2(d_prev.cpu().numpy(), ref["d"])
        step = np.linalg.norm(ref["theta"] - th_in)
        e_th = np.linalg.norm(theta.cpu().numpy().astype(np.float64) - ref["theta"])
        print(f"[{cfg.name}] newton k={k}: f {out['f_old']:.6f} -> {out['f_new']:.6f} (oracle {ref['f_new']:.6f}), alpha "
              f"{out['alpha']}, beta ({out['beta1']:.4f}, {out['beta2']:.4f}) oracle ({ref['beta'][0]:.4f}, "
              f"{ref['beta'][1]:.4f}), rho {out['rho']:.4f} ({ref['rho']:.4f}), d err {e_d:.1e}, theta err "
              f"{e_th / step:.1e} of the step", flush=True)
        assert out["alpha"] == ref["alpha"] and out["alpha"] > 0
        assert out["f_evals"] == ref["f_evals"] and out["cg_iters"] == ref["cg_iters"] == cg_max
        assert abs(out["f_old"] - ref["f_old"]) <= TOL * abs(ref["f_old"])
        assert abs(out["f_new"] - ref["f_new"]) <= TOL * abs(ref["f_new"]) + 2e-3 * abs(ref["f_new"] - ref["f_old"])
        assert e_d <= TOL_CG
        assert e_th <= TOL_CG * step + 1e-6 * np.linalg.norm(ref["theta"])
        assert abs(out["gTd"] - ref["gTd"]) <= 1e-3 * abs(ref["gTd"])
        assert abs(out["dGd"] - ref["dGd"]) <= 2e-3 * abs(ref["dGd"])
        assert abs(out["rho"] - ref["rho"]) <= 1e-2
        assert out["lam"] == pytest.approx(ref["lam"], rel=1e-12)
        if k == 0:
            assert out["beta"] == (1.0, 0.0)
        lam = out["lam"]


def _check_cg_sync(w, g_ref):
    """Joint early termination of the per-layer systems (Section 4.4): same stopping iteration and iterates as the
    oracle, for a tolerance that the blocks meet at different iterations."""
    cfg = w.cfg
    th = w.theta.astype(np.float64)
    g32 = g_ref.astype(np.float32)
    d = w.empty()
    sigma = 0.05
    _, _, _, hist = orc.cg(th, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), cfg.lam, 30, sigma=sigma,
                           blockdiag=True, history=True)
    for cg_min, r in ((0, 100.0), (0, 50.0), (2, 30.0)):
        it, res = dn.dn_cg_sync(w.ctx, w.dev(g32), cfg.lam, sigma, 30, cg_min, r, d)
        d_ref, it_ref, _ = orc.cg(th, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), cfg.lam, 30, sigma=sigma,
                                  blockdiag=True, cg_min=cg_min, r_percent=r)
        err = rel_l2(d.cpu().numpy(), d_ref)
        print(f"[{cfg.name}] cg_sync cg_min {cg_min} r {r}: {it} iterations (oracle {it_ref}, all blocks done after "
              f"{len(hist)}), rel err {err:.2e}", flush=True)
        assert it == it_ref and err <= TOL_CG


@pytest.mark.parametrize("idx", [2, 3])
def test_full_configuration(idx):
    w = Workload(dn_inputs.config(idx))
    g_ref = _check_grad(w)
    _check_products(w)
    _check_cg(w, g_ref, (dn.DN_FULL, dn.DN_BLOCKDIAG))
    _check_partitions(w, g_ref, cg_iters=6)
    if idx == 3:
        _check_cg_sync(w, g_ref)
    _check_newton(w)
    w.ctx.close()


@pytest.mark.parametrize("idx", [4, 5])
def test_large_configuration(idx):
    cfg = dn_inputs.config(idx)
    # gradient parity on a prefix of the samples (the oracle's full-l gradient takes many minutes);
    # the subsample S is drawn from that prefix, with the configuration's full |S|
    w = Workload(cfg, rows=20000)
    assert w.s == cfg.s
    g_ref = _check_grad(w)
    _check_products(w, modes=(dn.DN_FULL, dn.DN_BLOCKDIAG) if (idx == 4 or HEAVY) else (dn.DN_FULL,))
    if HEAVY:
        _check_cg(w, g_ref, (dn.DN_FULL,))
        _check_partitions(w, g_ref, cg_iters=6 if idx == 4 else 0)
    w.ctx.close()
