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


def cg_fp32_vectors(oracle, theta, dims, C, XS, g, lam, iters):
    """The oracle's CG (full system) with every vector rounded to fp32 after each update and the step lengths
    rounded to fp32, products and inner products in fp64: what limits a CG whose vectors are stored in fp32,
    whatever computes the products.  Test-side arithmetic on top of the oracle's product."""
    f32 = lambda a: a.astype(np.float32).astype(np.float64)
    d = np.zeros_like(g)
    r = f32(-g)
    p = r.copy()
    rho = r @ r
    for _ in range(iters):
        q = f32(oracle.gn_matvec(theta, dims, C, XS, p))
        alpha = np.float64(np.float32(rho / (p @ (q + lam * p))))
        d = f32(d + alpha * p)
        r = f32(r - alpha * f32(q + f32(lam * p)))
        rho_new = r @ r
        p = f32(r + np.float64(np.float32(rho_new / rho)) * p)
        rho = rho_new
    return d
