"""Helpers for the GPU parity tests: put a seeded workload on the device and run the oracle beside it."""
import numpy as np
import torch

import dn_inputs
import paper_1802_00130_amd as dn
from oracle import dn_oracle as orc


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def block_errors(a, b, dims):
    """Relative L2 error of every weight block A^m and every bias block b^m of two theta-layout vectors, as a
    list of (name, error): a whole-vector norm alone would let a percent-level error in a small block pass."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    out = []
    for m, (w, bo) in enumerate(dn_inputs.layer_offsets(dims), start=1):
        nw = dims[m - 1] * dims[m]
        out.append((f"A{m}", rel_l2(a[w:w + nw], b[w:w + nw])))
        out.append((f"b{m}", rel_l2(a[bo:bo + dims[m]], b[bo:bo + dims[m]])))
    return out


def assert_close_blocks(a, b, dims, tol, what=""):
    """Whole-vector relative L2 error within tol, and every block's own relative error within tol."""
    whole = rel_l2(a, b)
    blocks = block_errors(a, b, dims)
    worst = max(blocks, key=lambda t: t[1])
    assert whole <= tol, (what, whole)
    assert worst[1] <= tol, (what, worst)
    return whole, worst


class Workload:
    def __init__(self, cfg, bias_scale=0.0, rows=None, l_max=None):
        self.cfg = cfg
        self.X = dn_inputs.make_X(cfg, rows)
        self.Y = dn_inputs.make_Y(cfg, rows)
        self.theta = dn_inputs.make_theta(cfg, bias_scale=bias_scale)
        self.S = dn_inputs.make_subset(cfg, rows)
        self.l = self.X.shape[0]
        self.s = self.S.shape[0]
        dev = torch.device("cuda:0")
        self.dX = torch.from_numpy(self.X).to(dev)
        self.dY = torch.from_numpy(self.Y).to(dev)
        self.dtheta = torch.from_numpy(self.theta).to(dev)
        self.dS = torch.from_numpy(self.S).to(dev)
        self.ctx = dn.Context(cfg.dims, cfg.C, l_max or self.l, self.s)
        self.n = self.ctx.n

    def dev(self, a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")

    def empty(self):
        return torch.empty(self.n, dtype=torch.float32, device="cuda:0")

    @property
    def XS64(self):
        return self.X[self.S].astype(np.float64)

    def oracle_matvec(self, v, blockdiag=False):
        f = orc.gn_matvec_blockdiag if blockdiag else orc.gn_matvec
        return f(self.theta.astype(np.float64), self.cfg.dims, self.cfg.C, self.XS64, v.astype(np.float64))


def cg_fp32_vectors(oracle, theta, dims, C, XS, g, lam, iters, blockdiag=False):
    """The oracle's CG (full system, or the per-layer systems) with every vector rounded to fp32 after each update
    and the step lengths rounded to fp32, products and inner products in fp64: what limits a CG whose vectors are
    stored in fp32, whatever computes the products.  Test-side arithmetic on top of the oracle's product."""
    f32 = lambda a: a.astype(np.float32).astype(np.float64)
    g = np.asarray(g, dtype=np.float64)
    blocks = oracle.block_slices(dims) if blockdiag else [slice(0, g.shape[0])]
    product = oracle.gn_matvec_blockdiag if blockdiag else oracle.gn_matvec
    d = np.zeros_like(g)
    r = f32(-g)
    p = r.copy()
    rho = [r[b] @ r[b] for b in blocks]
    for _ in range(iters):
        q = f32(product(theta, dims, C, XS, p))
        for k, b in enumerate(blocks):
            if rho[k] == 0.0:
                continue
            alpha = np.float64(np.float32(rho[k] / (p[b] @ (q[b] + lam * p[b]))))
            d[b] = f32(d[b] + alpha * p[b])
            r[b] = f32(r[b] - alpha * f32(q[b] + f32(lam * p[b])))
            rho_new = r[b] @ r[b]
            p[b] = f32(r[b] + np.float64(np.float32(rho_new / rho[k])) * p[b])
            rho[k] = rho_new
    return d
