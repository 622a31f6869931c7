"""GPU parity of the block-diagonal product and CG over the variable partitions of a split structure
(neuron groups per layer, Section 3.1; DN_PARTITION) against the oracle's literal definition.

Split structures cover: groups on the input side only, on the output side only, on both, on the output
layer, ragged group sizes, n_L above and below 16, one hidden layer and none, and the paper's own 1-2-2-1.
Tolerances as for the other products (1e-4 relative L2) and CG iterates (1e-3).
"""
import numpy as np
import pytest
import torch

import dn_inputs
import paper_1802_00130_amd as dn
from oracle import dn_oracle as orc
from tests.gpu_common import Workload, rel_l2

pytestmark = pytest.mark.gpu

CASES = {
    "1-2-2-1": (lambda: dn_inputs.custom((36, 50, 30, 6), l=120, s=50, C=5.0, seed=71), (1, 2, 2, 1)),
    "3-2-2-1": (lambda: dn_inputs.custom((31, 23, 18, 5), l=90, s=40, C=3.0, seed=72), (3, 2, 2, 1)),
    "2-1-3-2": (lambda: dn_inputs.custom((20, 17, 13, 7), l=80, s=33, C=2.0, seed=73), (2, 1, 3, 2)),
    "4-4-4": (lambda: dn_inputs.custom((70, 133, 19), l=150, s=61, C=10.0, seed=74), (4, 4, 4)),
    "no_hidden_2-3": (lambda: dn_inputs.custom((12, 9), l=60, s=25, C=1.5, seed=75), (2, 3)),
    "wide_out_1-2-1-3": (lambda: dn_inputs.custom((24, 40, 36, 50), l=100, s=30, C=4.0, seed=76), (1, 2, 1, 3)),
    "five_layers": (lambda: dn_inputs.custom((10, 9, 8, 7, 6, 3), l=100, s=50, C=3.0, seed=77), (2, 2, 1, 2, 2, 1)),
    "mid_1-2-2-1": (lambda: dn_inputs.custom((200, 300, 260, 10), l=900, s=300, C=50.0, seed=78), (1, 2, 2, 1)),
    # more than 16 strip slots: two strips per wave in the single-pass kernel
    "wide_2-3-4-1": (lambda: dn_inputs.custom((14, 2600, 1700, 7), l=40, s=10, C=4.0, seed=79), (2, 3, 4, 1)),
    # n_L > 16: the single-pass kernel of wide outputs, one to several slices per output group, group bounds that
    # are no multiples of four, several bands of rows per sample
    "wide_out_2-3-4-1": (lambda: dn_inputs.custom((14, 2600, 1701, 37), l=40, s=10, C=4.0, seed=80), (2, 3, 4, 1)),
    "wide_out_3-2-3-4": (lambda: dn_inputs.custom((20, 1030, 45, 130), l=300, s=260, C=4.0, seed=81), (3, 2, 3, 4)),
    # narrow outputs, hidden layers beyond the register-strip kernel: the same single-pass kernel
    "narrow_out_wide_hidden_2-2-3-1": (lambda: dn_inputs.custom((9, 2300, 2200, 16), l=50, s=21, C=4.0, seed=83), (2, 2, 3, 1)),
    "wide_out_deep": (lambda: dn_inputs.custom((33, 2100, 530, 1200, 100), l=60, s=24, C=9.0, seed=82), (1, 2, 2, 2, 1)),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_partitioned_product_and_cg(name):
    make, split = CASES[name]
    cfg = make()
    print(f"[case] {name}", flush=True)
    w = Workload(cfg, bias_scale=0.3)
    nparts = w.ctx.set_split(split)
    assert nparts == sum(split[m - 1] * split[m] for m in range(1, len(split)))
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    th64 = w.theta.astype(np.float64)
    out = w.empty()
    for k in range(2):
        v = dn_inputs.make_probe(cfg, k)
        ref = orc.gn_matvec_partitioned(th64, cfg.dims, cfg.C, w.XS64, v.astype(np.float64), split)
        for passes in (0, 2):        # single-pass kernel where there is one, and the general two-pass kernels
            w.ctx.set_stream_passes(passes)
            out.fill_(float("nan"))
            dn.dn_gn_matvec(w.ctx, w.dev(v), out, dn.DN_PARTITION)
            err = rel_l2(out.cpu().numpy(), ref)
            print(f"  product {k}, passes {passes}: rel err {err:.2e}", flush=True)
            assert err <= 1e-4
    w.ctx.set_stream_passes(0)
    # the other modes are untouched by a split structure
    dn.dn_gn_matvec(w.ctx, w.dev(v), out, dn.DN_BLOCKDIAG)
    assert rel_l2(out.cpu().numpy(), w.oracle_matvec(v, blockdiag=True)) <= 1e-4
    # CG over the partitions
    g_ref, _ = orc.grad(th64, cfg.dims, cfg.C, w.X.astype(np.float64), w.Y.astype(np.float64))
    g32 = g_ref.astype(np.float32)
    d = w.empty()
    it, res = dn.dn_cg(w.ctx, w.dev(g32), 1.0, 0.0, 6, dn.DN_PARTITION, d)
    d_ref, it_ref, res_ref = orc.cg(th64, cfg.dims, cfg.C, w.XS64, g32.astype(np.float64), 1.0, 6, blockdiag=True,
                                    split=split)
    assert it == it_ref == 6 and len(res) == nparts
    err = rel_l2(d.cpu().numpy(), d_ref)
    print(f"  cg: rel err {err:.2e}", flush=True)
    assert err <= 1e-3
    np.testing.assert_allclose(res, res_ref, rtol=2e-2, atol=1e-6 * float(np.linalg.norm(g32)))
    w.ctx.close()


def test_one_group_per_layer_is_the_per_layer_mode():
    cfg = dn_inputs.custom((36, 50, 30, 6), l=120, s=50, C=5.0, seed=71)
    w = Workload(cfg, bias_scale=0.3)
    assert w.ctx.set_split((1, 1, 1, 1)) == 3
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(cfg, 0)
    a, b = w.empty(), w.empty()
    dn.dn_gn_matvec(w.ctx, w.dev(v), a, dn.DN_PARTITION)
    dn.dn_gn_matvec(w.ctx, w.dev(v), b, dn.DN_BLOCKDIAG)
    assert rel_l2(a.cpu().numpy(), b.cpu().numpy()) <= 1e-5
    w.ctx.close()


def test_newton_step_and_joint_termination_over_partitions():
    cfg = dn_inputs.custom((36, 50, 30, 6), l=120, s=50, C=5.0, seed=71)
    split = (1, 2, 2, 1)
    w = Workload(cfg, bias_scale=0.2)
    w.ctx.set_split(split)
    th64, X64, Y64 = w.theta.astype(np.float64), w.X.astype(np.float64), w.Y.astype(np.float64)
    theta = w.dtheta.clone()
    d_prev = torch.zeros_like(theta)
    out = dn.dn_newton_step(w.ctx, theta, w.dX, w.dY, w.dS, d_prev, 1.0, 8, sigma=0.0, mode=dn.DN_PARTITION)
    XS = X64[w.S]
    g, f0 = orc.grad(th64, cfg.dims, cfg.C, X64, Y64)
    d_ref, _, _ = orc.cg(th64, cfg.dims, cfg.C, XS, g, 1.0, 8, blockdiag=True, split=split)
    assert rel_l2(d_prev.cpu().numpy(), d_ref) <= 1e-3                     # first iteration: beta = (1, 0)
    alpha, f_new, _ = orc.line_search(th64, cfg.dims, cfg.C, X64, Y64, f0, float(g @ d_ref), d_ref)
    assert out["alpha"] == alpha and abs(out["f_new"] - f_new) <= 1e-4 * abs(f_new) + 2e-3 * abs(f_new - f0)
    # joint early termination over the 8 partitions
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    g32 = g.astype(np.float32)
    d = w.empty()
    # with sigma = 6e-3 the partitions meet their tests after 2, 2, 5, 4, 5, 4, 2, 2 iterations, each at least a
    # factor 1.4 away from the threshold on both sides
    stops = []
    for cg_min, r in ((0, 100.0), (0, 75.0), (0, 50.0), (3, 50.0)):
        it, res = dn.dn_cg_sync(w.ctx, w.dev(g32), 0.1, 6e-3, 100, cg_min, r, d, mode=dn.DN_PARTITION)
        d_ref, it_ref, _ = orc.cg(th64, cfg.dims, cfg.C, XS, g32.astype(np.float64), 0.1, 100, sigma=6e-3, blockdiag=True,
                                  split=split, cg_min=cg_min, r_percent=r)
        print(f"  cg_min {cg_min} r {r}: {it} iterations (oracle {it_ref})", flush=True)
        assert it == it_ref and rel_l2(d.cpu().numpy(), d_ref) <= 1e-3
        stops.append(it)
    assert stops == [5, 4, 2, 3]
    w.ctx.close()


def test_partition_counts_of_the_papers_split_structures():
    """dn_set_split gives the partition counts the paper prints for its own networks (tests/golden).  Only the
    count is checked here; the index map behind it is exercised by the parity cases above."""
    from tests.golden_io import split_structures
    rows, _ = split_structures()
    assert len(rows) == 10
    for name, dims, split, count in rows:
        print(f"[split] {name} {dims} {split}", flush=True)
        ctx = dn.Context(dims, 1.0, 8, 4)
        assert ctx.set_split(split) == count
        assert ctx.num_systems(dn.DN_PARTITION) == count
        ctx.close()
