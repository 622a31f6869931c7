"""GPU parity of the single-pass product kernel in which teams of work-groups share a sample: every product
with at least two hidden layers that the register-strip kernel cannot take (n_L > 16, or hidden layers too wide
for one work-group's registers).

Each case runs the product with that kernel (automatic choice) and with the two-pass kernels forced, both
against the fp64 oracle (1e-4 relative L2), in full and per-layer mode.  Output widths are chosen to hit both
kernel variants and one to many bands of rows per sample (n_L 19 ... 1000); hidden widths include ragged slices
and layers wider than one slice; one case has more samples than teams, so that teams walk over several samples
and the exchange words are reused.
The time-out path is forced from the host with a spin limit of zero: every wait gives up at once, every
work-group still leaves normally, and the two-pass kernels behind the single-pass kernel complete the product.
"""
import numpy as np
import pytest
import torch

import dn_inputs
import paper_1802_00130_amd as dn
from tests.gpu_common import Workload, rel_l2

pytestmark = pytest.mark.gpu

TOL = 1e-4

CASES = {
    "nL19_ragged": lambda: dn_inputs.custom((70, 133, 45, 19), l=333, s=131, C=10.0, seed=16),
    "nL24_L5": lambda: dn_inputs.custom((10, 9, 8, 7, 11, 24), l=90, s=41, C=2.5, seed=20),
    "nL64_many_samples": lambda: dn_inputs.custom((16, 24, 20, 64), l=1200, s=1000, C=4.0, seed=61),
    "nL100": lambda: dn_inputs.custom((30, 300, 130, 40, 100), l=200, s=60, C=5.0, seed=62),
    "nL200": lambda: dn_inputs.custom((20, 70, 50, 200), l=120, s=40, C=5.0, seed=63),
    "nL400": lambda: dn_inputs.custom((20, 40, 36, 400), l=100, s=30, C=5.0, seed=64),
    "nL1000": lambda: dn_inputs.custom((16, 70, 33, 20, 1000), l=60, s=20, C=5.0, seed=65),
    "wide_layers": lambda: dn_inputs.custom((12, 2100, 1030, 25, 40), l=80, s=37, C=5.0, seed=66),
    "nL33_two_bands": lambda: dn_inputs.custom((9, 1025, 77, 14, 33), l=150, s=90, C=3.0, seed=67),
    # narrow outputs whose hidden layers exceed the register-strip kernel (more than 32 strips; n_L = 16 with more than 16)
    "nL10_wide_hidden": lambda: dn_inputs.custom((12, 4300, 4100, 30, 10), l=40, s=14, C=5.0, seed=68),
    "nL16_wide_hidden": lambda: dn_inputs.custom((8, 2200, 2100, 16), l=70, s=33, C=5.0, seed=69),
    "nL3_deep_wide": lambda: dn_inputs.custom((6, 3000, 3100, 2300, 3), l=30, s=12, C=2.0, seed=70),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_single_pass_and_two_pass_products_match_the_oracle(name):
    print(f"[case] {name}", flush=True)
    w = Workload(CASES[name](), bias_scale=0.3)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(w.cfg, 0)
    dv, out = w.dev(v), w.empty()
    for mode in (dn.DN_FULL, dn.DN_BLOCKDIAG):
        ref = w.oracle_matvec(v, blockdiag=(mode == dn.DN_BLOCKDIAG))
        results = {}
        for passes in (0, 2):
            w.ctx.set_stream_passes(passes)
            out.fill_(float("nan"))
            dn.dn_gn_matvec(w.ctx, dv, out, mode)
            assert w.ctx.sync_status() == 0
            results[passes] = out.cpu().numpy()
            err = rel_l2(results[passes], ref)
            print(f"  mode {mode} passes {passes}: rel err {err:.2e}", flush=True)
            assert err <= TOL
        # the same product twice gives the same bits (fixed summation orders, no floating-point atomics)
        w.ctx.set_stream_passes(0)
        dn.dn_gn_matvec(w.ctx, dv, out, mode)
        assert w.ctx.sync_status() == 0
        assert np.array_equal(out.cpu().numpy(), results[0])
    w.ctx.close()


@pytest.mark.parametrize("name", ["nL100", "nL16_wide_hidden"])
def test_single_pass_kernel_is_the_one_that_runs(name):
    w = Workload(CASES[name](), bias_scale=0.3)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    dv, out = w.dev(dn_inputs.make_probe(w.cfg, 0)), w.empty()
    w.ctx.profile_enable(True)
    w.ctx.profile_reset()
    dn.dn_gn_matvec(w.ctx, dv, out, dn.DN_FULL)
    prof = w.ctx.profile_read()
    assert prof["jv_jtv_band"][1] == 1 and prof["jv_rows"][1] == 0 and prof["jtv_cols"][1] == 0
    w.ctx.set_stream_passes(2)
    w.ctx.profile_reset()
    dn.dn_gn_matvec(w.ctx, dv, out, dn.DN_FULL)
    prof = w.ctx.profile_read()
    assert prof["jv_jtv_band"][1] == 0 and prof["jv_rows"][1] == 1 and prof["jtv_cols"][1] == 1
    w.ctx.profile_enable(False)
    w.ctx.close()


def test_wait_that_runs_out_falls_back_to_the_two_pass_kernels():
    """A spin limit of zero makes every wait between work-groups give up at once (every work-group still leaves
    normally).  The two-pass kernels enqueued behind the single-pass kernel then complete the same product: its
    result equals the forced two-pass result bit for bit, dn_sync_status reports the event once, later products
    stay correct, and dn_bind restores the single-pass kernel."""
    w = Workload(CASES["nL100"](), bias_scale=0.3)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    v = dn_inputs.make_probe(w.cfg, 0)
    dv, out = w.dev(v), w.empty()
    results = {}
    for mode in (dn.DN_FULL, dn.DN_BLOCKDIAG):
        dn.dn_gn_matvec(w.ctx, dv, out, mode)
        assert w.ctx.sync_status() == 0
        results["band", mode] = out.cpu().numpy()
        w.ctx.set_stream_passes(2)
        dn.dn_gn_matvec(w.ctx, dv, out, mode)
        assert w.ctx.sync_status() == 0
        results["two", mode] = out.cpu().numpy()
        w.ctx.set_stream_passes(0)
    w.ctx.set_spin_limit(0)
    out.fill_(float("nan"))
    dn.dn_gn_matvec(w.ctx, dv, out, dn.DN_FULL)
    first = out.cpu().numpy()
    assert np.array_equal(first, results["two", dn.DN_FULL])
    assert w.ctx.sync_status() == -6             # reported once
    assert w.ctx.sync_status() == 0
    w.ctx.set_spin_limit(1 << 20)
    w.ctx.profile_enable(True)
    w.ctx.profile_reset()
    for mode in (dn.DN_FULL, dn.DN_BLOCKDIAG):   # the context has switched to the two-pass kernels
        dn.dn_gn_matvec(w.ctx, dv, out, mode)
        assert w.ctx.sync_status() == 0
        assert np.array_equal(out.cpu().numpy(), results["two", mode])
    prof = w.ctx.profile_read()
    assert prof["jv_jtv_band"][1] == 0 and prof["jv_rows"][1] == 2
    w.ctx.profile_enable(False)
    d = w.empty()
    it, _ = dn.dn_cg(w.ctx, dv, 1.0, 0.0, 2, dn.DN_FULL, d)
    assert it == 2
    w.ctx.rebind()
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    dn.dn_gn_matvec(w.ctx, dv, out, dn.DN_FULL)
    assert w.ctx.sync_status() == 0
    assert np.array_equal(out.cpu().numpy(), results["band", dn.DN_FULL])
    w.ctx.close()


def test_wait_that_runs_out_inside_cg_still_gives_the_two_pass_iterates():
    w = Workload(CASES["nL64_many_samples"](), bias_scale=0.3)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    g = w.dev(dn_inputs.make_probe(w.cfg, 1))
    d, d2 = w.empty(), w.empty()
    w.ctx.set_stream_passes(2)
    dn.dn_cg(w.ctx, g, 1.0, 0.0, 4, dn.DN_FULL, d2)
    w.ctx.set_stream_passes(0)
    w.ctx.set_spin_limit(0)
    it, _ = dn.dn_cg(w.ctx, g, 1.0, 0.0, 4, dn.DN_FULL, d)
    assert it == 4 and torch.equal(d, d2)
    assert w.ctx.sync_status() == -6 and w.ctx.sync_status() == 0
    w.ctx.close()


def test_phase_clocks_leave_the_product_unchanged():
    """The diagnostic variant of the single-pass kernel (phase clocks on) gives the same bits and reports where a
    work-group's cycles went; nothing is reported while the clocks are off."""
    w = Workload(CASES["wide_layers"](), bias_scale=0.3)
    dn.dn_jacobian_prep(w.ctx, w.dtheta, w.dX, w.dS)
    dv, out, out2 = w.dev(dn_inputs.make_probe(w.cfg, 0)), w.empty(), w.empty()
    dn.dn_gn_matvec(w.ctx, dv, out, dn.DN_FULL)
    off = w.ctx.profile_band_read()
    assert off["bands_per_work_group"] == 0 and off["load_cycles"] == 0
    w.ctx.profile_band_phases(True)
    dn.dn_gn_matvec(w.ctx, dv, out2, dn.DN_FULL)
    on = w.ctx.profile_band_read()
    w.ctx.profile_band_phases(False)
    print(on, flush=True)
    assert torch.equal(out, out2)
    assert on["bands_per_work_group"] >= 1 and on["load_cycles"] > 0 and on["exchange_wait_cycles"] > 0
    assert on["transposed_product_cycles"] > 0
    w.ctx.close()


@pytest.mark.parametrize("name", ["nL33_two_bands", "nL64_many_samples"])
def test_products_replayed_from_a_captured_graph(name):
    """Products captured in a HIP graph and replayed with new contents in the input vector: every replay must give
    what the same call gives eagerly.  The exchange words of the single-pass kernel carry sequence numbers whose
    base lives in device memory for exactly this (numbers fixed at capture time would repeat on every replay; with
    at most two bands per team, as in the first case, a word left by the previous replay would then pass for the
    current one's).  Eager products and synchronisations sit between the replays."""
    w_cfg = CASES[name]()
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    X, theta, S = dn_inputs.make_X(w_cfg), dn_inputs.make_theta(w_cfg, bias_scale=0.3), dn_inputs.make_subset(w_cfg)
    dev = "cuda:0"
    dX, dth, dS = torch.from_numpy(X).to(dev), torch.from_numpy(theta).to(dev), torch.from_numpy(S).to(dev)
    ctx = dn.Context(w_cfg.dims, w_cfg.C, 16, w_cfg.s, stream=st)
    n = ctx.n
    vin = torch.zeros(n, dtype=torch.float32, device=dev)
    out_full, out_bd, eager = (torch.empty(n, dtype=torch.float32, device=dev) for _ in range(3))
    probes = [torch.from_numpy(dn_inputs.make_probe(w_cfg, k)).to(dev) for k in range(4)]
    with torch.cuda.stream(st):
        dn.dn_jacobian_prep(ctx, dth, dX, dS)
        vin.copy_(probes[0])
        dn.dn_gn_matvec(ctx, vin, eager, dn.DN_FULL)          # first use of the kernel outside the capture
    st.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        dn.dn_gn_matvec(ctx, vin, out_full, dn.DN_FULL)
        dn.dn_gn_matvec(ctx, vin, out_bd, dn.DN_BLOCKDIAG)
    for k in (1, 2, 3, 1):
        with torch.cuda.stream(st):
            vin.copy_(probes[k])
            out_full.fill_(float("nan"))
            out_bd.fill_(float("nan"))
            g.replay()
        st.synchronize()
        got_full, got_bd = out_full.clone(), out_bd.clone()
        for mode, got in ((dn.DN_FULL, got_full), (dn.DN_BLOCKDIAG, got_bd)):
            with torch.cuda.stream(st):
                dn.dn_gn_matvec(ctx, probes[k], eager, mode)
            assert ctx.sync_status() == 0
            assert torch.equal(got, eager), (name, k, mode)
    # against the oracle once, so that "equal" is also "right"
    ref = orc_matvec(w_cfg, theta, X[S], dn_inputs.make_probe(w_cfg, 1))
    assert rel_l2(got_full.cpu().numpy(), ref) <= TOL
    ctx.close()


def orc_matvec(cfg, theta, XS, v):
    from oracle import dn_oracle as orc
    return orc.gn_matvec(theta.astype(np.float64), cfg.dims, cfg.C, XS.astype(np.float64), v.astype(np.float64))
