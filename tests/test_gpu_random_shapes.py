"""GPU parity on seeded random network shapes: every product path against the oracle.

Forty small networks drawn from a fixed seed: 1-5 weight layers, widths 1-90 (a few up to 700), outputs 1-40,
subsamples 1-60, random split structures.  Each runs f, the gradient, the products in all three block modes,
the product without stored blocks, both stored-block kernels where two exist, and six CG iterations.
The shapes hit ragged tiles, unaligned theta slices, single-neuron layers, n_L on both sides of 16, and
group boundaries inside groups of four columns.
"""
import numpy as np
import pytest
import torch

import dn_inputs
import paper_1802_00130_amd as dn
from oracle import dn_oracle as orc
from tests.gpu_common import Workload, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _draw(k):
    rng = np.random.default_rng(9000 + k)
    L = int(rng.integers(1, 6))
    widths = [int(rng.integers(1, 91)) for _ in range(L + 1)]
    if rng.random() < 0.3 and L >= 2:
        widths[int(rng.integers(1, L))] = int(rng.integers(200, 701))
    widths[-1] = int(rng.integers(1, 41))
    l = int(rng.integers(3, 120))
    s = int(rng.integers(1, min(l, 60) + 1))
    C = float(rng.choice([0.5, 1.0, 7.0, 100.0]))
    split = tuple(int(rng.integers(1, min(4, w) + 1)) for w in widths)
    return dn_inputs.custom(tuple(widths), l=l, s=s, C=C, seed=500 + k), split


@pytest.mark.parametrize("k", range(40))
def test_random_shape(k):
    cfg, split = _draw(k)
    print(f"[case {k}] dims {cfg.dims} l {cfg.l} s {cfg.s} C {cfg.C} split {split}", flush=True)
    w = Workload(cfg, bias_scale=0.4)
    th64, X64, Y64 = w.theta.astype(np.float64), w.X.astype(np.float64), w.Y.astype(np.float64)
    g = w.empty()
    f = dn.dn_grad(w.ctx, w.dtheta, w.dX, w.dY, g)
    g_ref, f_ref = orc.grad(th64, cfg.dims, cfg.C, X64, Y64)
    assert abs(f - f_ref) <= TOL * abs(f_ref)
    assert rel_l2(g.cpu().numpy(), g_ref) <= TOL
    w.ctx.set_split(split)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(cfg, 0)
    v64 = v.astype(np.float64)
    out = w.empty()
    refs = {
        dn.DN_FULL: orc.gn_matvec(th64, cfg.dims, cfg.C, w.XS64, v64),
        dn.DN_BLOCKDIAG: orc.gn_matvec_blockdiag(th64, cfg.dims, cfg.C, w.XS64, v64),
        dn.DN_PARTITION: orc.gn_matvec_partitioned(th64, cfg.dims, cfg.C, w.XS64, v64, split),
    }
    for passes in (0, 2):
        w.ctx.set_stream_passes(passes)
        for mode, ref in refs.items():
            out.fill_(float("nan"))
            dn.dn_gn_matvec(w.ctx, w.dev(v), out, mode)
            assert w.ctx.sync_status() == 0
            err = rel_l2(out.cpu().numpy(), ref)
            assert err <= TOL, (passes, mode, err)
    w.ctx.set_stream_passes(0)
    dn.dn_gn_matvec_rop(w.ctx, w.dev(v), out)
    assert rel_l2(out.cpu().numpy(), refs[dn.DN_FULL]) <= TOL
    g32 = g_ref.astype(np.float32)
    d = w.empty()
    for mode in (dn.DN_FULL, dn.DN_BLOCKDIAG, dn.DN_PARTITION):
        it, res = dn.dn_cg(w.ctx, w.dev(g32), 1.0, 0.0, 6, mode, d)
        d_ref, it_ref, _ = orc.cg(th64, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), 1.0, 6,
                                  blockdiag=(mode != dn.DN_FULL), split=split if mode == dn.DN_PARTITION else None)
        assert it == it_ref
        err = rel_l2(d.cpu().numpy(), d_ref)
        assert err <= 1e-3, (mode, err)
    w.ctx.close()


@pytest.mark.parametrize("k", [81, 87])
def test_cg_without_hidden_layer_follows_the_fp32_recurrence(k):
    """Two shapes found by running this file's recipe on further seeds: networks without a hidden layer, whose
    small quadratic systems have all but converged after six CG iterations (residual 3-4e-4 of |g|).  The sixth
    fp32 iterate is 1-2e-3 away from the fp64 one, above the 1e-3 bar of the other cases, because a nearly
    converged Krylov iterate is only determined up to about its residual: rounding any one of r, p, G p or the
    step lengths to fp32 moves it that far.  What can be checked is that the device follows the recurrence: the
    oracle's CG with its vectors and step lengths rounded to fp32 (products and inner products still fp64) lands
    within 1e-4 of the device's result and equally far from the fp64 iterate."""
    from tests.gpu_common import cg_fp32_vectors
    cfg, _ = _draw(k)
    assert len(cfg.dims) == 2
    w = Workload(cfg, bias_scale=0.4)
    th64, X64, Y64 = w.theta.astype(np.float64), w.X.astype(np.float64), w.Y.astype(np.float64)
    g_ref, _ = orc.grad(th64, cfg.dims, cfg.C, X64, Y64)
    g32 = g_ref.astype(np.float32)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    d = w.empty()
    it, _ = dn.dn_cg(w.ctx, w.dev(g32), 1.0, 0.0, 6, dn.DN_FULL, d)
    assert it == 6
    d_ref, _, _ = orc.cg(th64, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), 1.0, 6)
    d_em = cg_fp32_vectors(orc, th64, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), 1.0, 6)
    e_ref, e_em, e_gap = rel_l2(d.cpu().numpy(), d_ref), rel_l2(d.cpu().numpy(), d_em), rel_l2(d_em, d_ref)
    print(f"[case {k}] device vs fp64 {e_ref:.2e}, device vs fp32-vector recurrence {e_em:.2e}, "
          f"fp32-vector recurrence vs fp64 {e_gap:.2e}", flush=True)
    assert 1e-3 < e_ref <= 5e-3 and e_em <= 1e-4 and abs(e_gap - e_ref) <= 1e-4
    w.ctx.close()
