"""Index-by-index reference for tiny networks, used only to pin the oracle.

Pure Python scalars and loops in the paper's index notation (Section 2.1):
w^m_{tj} connects node t of layer m-1 to node j of layer m and sits at
theta[off_m + j * n_{m-1} + t]; b^m_j follows the weights of layer m.
Nothing here is shared with oracle/ or with the HIP path.
"""
import math

import numpy as np


def offsets(dims):
    offs, o = [], 0
    for m in range(1, len(dims)):
        offs.append((o, o + dims[m - 1] * dims[m]))
        o += dims[m - 1] * dims[m] + dims[m]
    return offs, o


def net_output(theta, dims, x):
    """z^L for one sample, scalar loops."""
    L = len(dims) - 1
    offs, _ = offsets(dims)
    z = [float(t) for t in x]
    for m in range(1, L + 1):
        ow, ob = offs[m - 1]
        nxt = []
        for j in range(dims[m]):
            s = float(theta[ob + j])
            for t in range(dims[m - 1]):
                s += float(theta[ow + j * dims[m - 1] + t]) * z[t]
            nxt.append(s if m == L else 1.0 / (1.0 + math.exp(-s)))
        z = nxt
    return z


def objective(theta, dims, C, X, Y):
    """f(theta) of Section 2.1 with the squared loss (no factor 1/2 on the loss)."""
    reg = sum(float(t) * float(t) for t in theta) / (2.0 * C)
    tot = 0.0
    for x, y in zip(X, Y):
        z = net_output(theta, dims, x)
        tot += sum((zu - float(yu)) ** 2 for zu, yu in zip(z, y))
    return reg + tot / len(X)


def fd_gradient(theta, dims, C, X, Y, h=1e-6):
    theta = np.array(theta, dtype=np.float64)
    g = np.zeros_like(theta)
    for k in range(theta.size):
        tp = theta.copy(); tp[k] += h
        tm = theta.copy(); tm[k] -= h
        g[k] = (objective(tp, dims, C, X, Y) - objective(tm, dims, C, X, Y)) / (2 * h)
    return g


def fd_jacobian(theta, dims, x, h=1e-6):
    """J^i (n_L x n) of Section 2.1 by central differences of the network output."""
    theta = np.array(theta, dtype=np.float64)
    nL = dims[-1]
    J = np.zeros((nL, theta.size))
    for k in range(theta.size):
        tp = theta.copy(); tp[k] += h
        tm = theta.copy(); tm[k] -= h
        zp = net_output(tp, dims, x)
        zm = net_output(tm, dims, x)
        for u in range(nL):
            J[u, k] = (zp[u] - zm[u]) / (2 * h)
    return J


def dense_gauss_newton(theta, dims, C, XS, h=1e-6):
    """G^S = I/C + (1/|S|) sum_i J_i^T (2I) J_i assembled from finite-difference Jacobians."""
    n = len(theta)
    G = np.eye(n) / C
    for x in XS:
        J = fd_jacobian(theta, dims, x, h)
        G += 2.0 * (J.T @ J) / len(XS)
    return G


def zero_offdiag_layer_blocks(G, dims):
    """Keep only the per-layer diagonal blocks (weights and biases of one layer together)."""
    out = np.zeros_like(G)
    o = 0
    for m in range(1, len(dims)):
        sz = dims[m - 1] * dims[m] + dims[m]
        out[o:o + sz, o:o + sz] = G[o:o + sz, o:o + sz]
        o += sz
    return out
