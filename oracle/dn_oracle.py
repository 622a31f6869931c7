"""fp64 CPU oracle for the subsampled Gauss-Newton path.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64, written from the paper's definitions.  It shares no code
with the HIP library and must never be imported by the product package; only
tests, the smoke check and the CPU-baseline leg of the benchmark call it.

What is computed, and from where in the paper:

* forward pass, objective f                     Section 2.1 (forward recursion, objective,
                                                squared loss); sigmoid hidden / linear
                                                output: Section 3.3.2
* gradient by back-propagation                  Section 2.2 (the four back-propagation
                                                equations), Section 3.4 (seed 2(z^L - y))
* J_i v  (forward-mode directional derivative of z^{L,i}) and
  sum_i J_i^T w_i (reverse sweep)               definition of J^i in Section 2.1
* G^S v = v/C + (1/|S|) sum_{i in S} J_i^T B_i J_i v, B_i = 2 I
                                                Section 4.3 (subsampled Gauss-Newton
                                                matrix), Section 3.1 (B for squared loss)
* block-diagonal product, one block per layer   Section 4.1
* the same for a general split structure        Section 3.1 (variable partitions, where the biases go),
  (neuron groups per layer)                     Section 4.1
* conjugate gradient on (G^S + lambda I) d = -g Section 2.2 / 4.3 linear system, Section 4.1
                                                stopping rule
* the stored blocks P^m_i = d z^{L,i} / d s^{m,i} by the backward recursion
                                                Section 3.3 (recursion for dz^L/dz^{m-1},
                                                product form of the Jacobian element)
* one outer Newton iteration: combination with the previous direction, backtracking line
  search, Levenberg-Marquardt update of lambda  Section 4.3 (two-variable problem), Section 4.5

The G v products here never build P: they differentiate the network directly,
so they are independent of the factored method the HIP path implements.

Pins (tests/test_oracle_pins.py): finite differences of f and of the network
outputs, brute-force dense G from an explicitly assembled Jacobian, symmetry,
positive definiteness, the gradient-through-Jacobian identity of Section 3.4,
the no-hidden-layer case against a normal-equations ridge solve, CG against a
dense solve and its first-step closed form; the outer iteration against a grid search of
the two-variable problem, an exhaustive scan of the step sizes, the rule table, and the
ridge problem where one undamped full step is exact (alpha = 1, rho = 1).
No function here is unpinned.

theta layout (Section 2.1): for m = 1..L, the n_m x n_{m-1} matrix A^m = (W^m)^T
stored row-major, then b^m.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- layout

def num_params(dims):
    """n = sum_m (n_{m-1} n_m + n_m), Section 2.1."""
    return sum(dims[m - 1] * dims[m] + dims[m] for m in range(1, len(dims)))


def unpack(theta, dims):
    """Views (A^m, b^m), m = 1..L, of a theta-layout vector.  A^m = (W^m)^T is n_m x n_{m-1}."""
    theta = np.asarray(theta, dtype=np.float64)
    assert theta.shape == (num_params(dims),)
    out = []
    o = 0
    for m in range(1, len(dims)):
        nw = dims[m - 1] * dims[m]
        A = theta[o:o + nw].reshape(dims[m], dims[m - 1])
        o += nw
        b = theta[o:o + dims[m]]
        o += dims[m]
        out.append((A, b))
    return out


def block_slices(dims):
    """Slice of theta owned by layer m (weights and biases), m = 1..L."""
    out = []
    o = 0
    for m in range(1, len(dims)):
        sz = dims[m - 1] * dims[m] + dims[m]
        out.append(slice(o, o + sz))
        o += sz
    return out


# --------------------------------------------------------------------------- forward, f

def forward(theta, dims, X):
    """Z^0..Z^L, one row per sample.

    s^m = (W^m)^T z^{m-1} + b^m; z^m = 1/(1+exp(-s^m)) for m < L, z^L = s^L
    (Section 2.1 forward recursion, Section 3.3.2 activation).
    """
    L = len(dims) - 1
    Z = [np.asarray(X, dtype=np.float64)]
    for m, (A, b) in enumerate(unpack(theta, dims), start=1):
        S = Z[-1] @ A.T + b
        Z.append(S if m == L else 1.0 / (1.0 + np.exp(-S)))
    return Z


def loss(theta, dims, C, X, Y):
    """f = theta^T theta / (2C) + (1/l) sum_i ||z^{L,i} - y^i||^2  (Section 2.1; no 1/2 on the loss)."""
    theta = np.asarray(theta, dtype=np.float64)
    ZL = forward(theta, dims, X)[-1]
    D = ZL - np.asarray(Y, dtype=np.float64)
    return float(theta @ theta / (2.0 * C) + np.sum(D * D) / X.shape[0])


# --------------------------------------------------------------------------- gradient

def _reverse_sweep(theta, dims, Z, seed):
    """sum_i J_i^T seed_i in theta layout, by one backward sweep.

    delta^L = seed (sigma' = 1 at the output layer); for each layer the weight part is
    sum_i delta^{m,i} z^{m-1,i T}, the bias part sum_i delta^{m,i}; then
    delta^{m-1} = (W^m delta^m) * z^{m-1}(1 - z^{m-1})   (Section 2.2 back-propagation).
    """
    L = len(dims) - 1
    layers = unpack(theta, dims)
    out = np.zeros(num_params(dims))
    parts = unpack_mutable(out, dims)
    delta = np.asarray(seed, dtype=np.float64)
    for m in range(L, 0, -1):
        A, _ = layers[m - 1]
        gA, gb = parts[m - 1]
        gA[...] = delta.T @ Z[m - 1]
        gb[...] = delta.sum(axis=0)
        if m > 1:
            zp = Z[m - 1]
            delta = (delta @ A) * (zp * (1.0 - zp))
    return out


def unpack_mutable(vec, dims):
    """Writable (A^m, b^m) views of a float64 theta-layout vector."""
    assert vec.dtype == np.float64 and vec.shape == (num_params(dims),)
    out = []
    o = 0
    for m in range(1, len(dims)):
        nw = dims[m - 1] * dims[m]
        A = vec[o:o + nw].reshape(dims[m], dims[m - 1])
        o += nw
        b = vec[o:o + dims[m]]
        o += dims[m]
        out.append((A, b))
    return out


def grad(theta, dims, C, X, Y):
    """(grad f, f).  grad f = theta/C + (1/l) sum_i J_i^T 2(z^{L,i} - y^i)  (Sections 2.1, 2.2, 3.4)."""
    theta = np.asarray(theta, dtype=np.float64)
    l = X.shape[0]
    Z = forward(theta, dims, X)
    D = Z[-1] - np.asarray(Y, dtype=np.float64)
    g = theta / C + _reverse_sweep(theta, dims, Z, 2.0 * D) / l
    f = float(theta @ theta / (2.0 * C) + np.sum(D * D) / l)
    return g, f


# --------------------------------------------------------------------------- J v, J^T w

def jv(theta, dims, Z, v):
    """Rows J_i v: derivative of z^{L,i} along direction v in parameter space.

    Differentiating the forward recursion: sdot^m = Vw^m z^{m-1} + vb^m + A^m zdot^{m-1},
    zdot^0 = 0, zdot^m = sigma'(s^m) * sdot^m (m < L), J_i v = sdot^L.
    """
    L = len(dims) - 1
    layers = unpack(theta, dims)
    vparts = unpack(v, dims)
    zdot = np.zeros_like(Z[0])
    for m in range(1, L + 1):
        A, _ = layers[m - 1]
        VA, vb = vparts[m - 1]
        sdot = Z[m - 1] @ VA.T + vb + zdot @ A.T
        zdot = sdot if m == L else sdot * (Z[m] * (1.0 - Z[m]))
    return zdot


def gn_matvec(theta, dims, C, XS, v):
    """G^S v = v/C + (1/|S|) sum_{i in S} J_i^T (2 J_i v)   (Section 4.3, B = 2I from Section 3.1).

    XS holds the rows of the subsample S.  No damping term is included.
    """
    theta = np.asarray(theta, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    Z = forward(theta, dims, XS)
    R = jv(theta, dims, Z, v)
    return v / C + _reverse_sweep(theta, dims, Z, 2.0 * R) / XS.shape[0]


def gn_matvec_blockdiag(theta, dims, C, XS, v):
    """Block-diagonal product, one block per layer (W^m together with b^m), Section 4.1.

    Taken literally: for each block m, zero the other blocks of v, apply the full
    product, keep block m of the result.
    """
    v = np.asarray(v, dtype=np.float64)
    out = np.zeros_like(v)
    for sl in block_slices(dims):
        vm = np.zeros_like(v)
        vm[sl] = v[sl]
        out[sl] = gn_matvec(theta, dims, C, XS, vm)[sl]
    return out


# --------------------------------------------------------------------------- variable partitions

def group_bounds(n, groups):
    """Boundaries of `groups` contiguous, as-equal-as-possible neuron groups of a layer with n neurons."""
    return [(k * n) // groups for k in range(groups + 1)]


def partition_index_sets(dims, split):
    """Index sets (into a theta-layout vector) of the variable partitions of Section 3.1.

    split[m] = number of neuron groups of layer m (m = 0..L).  The weights between group a of layer m-1
    and group b of layer m form one partition; the biases of group b of layer m go with the partition of
    the FIRST group of layer m-1 (a = 0).  Order: layer by layer, a outer, b inner.
    """
    assert len(split) == len(dims)
    sets = []
    o = 0
    for m in range(1, len(dims)):
        nprev, ncur = dims[m - 1], dims[m]
        ga = group_bounds(nprev, split[m - 1])
        gb = group_bounds(ncur, split[m])
        boff = o + nprev * ncur
        for a in range(split[m - 1]):
            for b in range(split[m]):
                j = np.arange(gb[b], gb[b + 1])
                t = np.arange(ga[a], ga[a + 1])
                idx = (o + j[:, None] * nprev + t[None, :]).ravel()      # w^m_{tj} sits at j * n_{m-1} + t
                if a == 0:
                    idx = np.concatenate([idx, boff + j])
                sets.append(idx)
        o = boff + ncur
    return sets


def gn_matvec_partitioned(theta, dims, C, XS, v, split):
    """Block-diagonal product for a general split structure (Section 4.1 with the partitions of
    Section 3.1), taken literally: for each partition p, zero the rest of v, apply the whole product,
    keep the entries of p."""
    v = np.asarray(v, dtype=np.float64)
    out = np.zeros_like(v)
    for idx in partition_index_sets(dims, split):
        vp = np.zeros_like(v)
        vp[idx] = v[idx]
        out[idx] = gn_matvec(theta, dims, C, XS, vp)[idx]
    return out


# --------------------------------------------------------------------------- CG

def cg(theta, dims, C, XS, g, lam, max_iter, sigma=0.0, blockdiag=False, history=False, cg_min=0, r_percent=None,
       split=None):
    """Conjugate gradient on (G^S + lam I) d = -g  (Sections 2.2, 4.3).

    d_0 = 0, r_0 = -g, p_0 = r_0, no preconditioner.  After each step the recurrence
    residual is tested against sigma ||g|| (Section 4.1 stopping rule).  With
    blockdiag=True the L per-layer systems are solved independently, each block with
    its own step lengths and its own stopping test; a block that has met its test is
    left unchanged afterwards.

    split (with blockdiag=True): the independent systems are those of the partitions of that split structure
    (Section 3.1) instead of one per layer.

    r_percent (block-diagonal systems only, Section 4.4): the early termination that spares the blocks still
    running from holding up the others: all blocks stop after the first iteration k >= cg_min at which the
    number of blocks that have met their own test is at least r_percent/100 of the number of blocks.  The
    blocks advance in lock-step here, so "every partition has done cg_min iterations" is k >= cg_min.

    Returns (d, iterations, residual norms); residual norms has one entry (full) or one
    per layer (block-diagonal).  With history=True also the list of iterates d_1, d_2, ...
    """
    g = np.asarray(g, dtype=np.float64)
    n = g.shape[0]
    if blockdiag and split is not None:
        blocks = partition_index_sets(dims, split)

        def product(th, dm, Cc, Xs, p):
            return gn_matvec_partitioned(th, dm, Cc, Xs, p, split)
    else:
        blocks = block_slices(dims) if blockdiag else [slice(0, n)]
        product = gn_matvec_blockdiag if blockdiag else gn_matvec
    d = np.zeros(n)
    r = -g.copy()
    p = r.copy()
    rho = np.array([r[b] @ r[b] for b in blocks])
    gnorm = np.sqrt(np.array([g[b] @ g[b] for b in blocks]))
    active = np.ones(len(blocks), dtype=bool)
    # a block with zero right-hand side is already solved
    active &= rho > 0.0
    iters = 0
    hist = []
    while iters < max_iter and active.any():
        q = product(theta, dims, C, XS, p) + lam * p
        for k, b in enumerate(blocks):
            if not active[k]:
                continue
            alpha = rho[k] / (p[b] @ q[b])
            d[b] += alpha * p[b]
            r[b] -= alpha * q[b]
            rho_new = r[b] @ r[b]
            if np.sqrt(rho_new) <= sigma * gnorm[k]:
                active[k] = False
            else:
                p[b] = r[b] + (rho_new / rho[k]) * p[b]
            rho[k] = rho_new
        iters += 1
        if history:
            hist.append(d.copy())
        if r_percent is not None and iters >= cg_min and np.count_nonzero(~active) >= r_percent / 100.0 * len(blocks):
            break
    res = np.sqrt(rho)
    if history:
        return d, iters, res, hist
    return d, iters, res


# --------------------------------------------------------------------------- stored Jacobian blocks

def jacobian_blocks(theta, dims, XS):
    """P^m, m = 1..L, with P^m[i, u, j] = d z^{L,i}_u / d s^{m,i}_j   (Section 3.3).

    dz^L/dz^L is the identity; dz^L/ds^m = dz^L/dz^m * sigma'(s^m);
    dz^L/dz^{m-1}_t = sum_j dz^L/ds^m_j * w^m_{tj}.
    """
    L = len(dims) - 1
    layers = unpack(theta, dims)
    Z = forward(theta, dims, XS)
    s = XS.shape[0]
    nL = dims[L]
    P = [None] * (L + 1)
    dz = np.broadcast_to(np.eye(nL), (s, nL, nL)).copy()      # dz^L/dz^L
    for m in range(L, 0, -1):
        if m == L:
            P[m] = dz                                           # sigma' = 1 at the output layer
        else:
            P[m] = dz * (Z[m] * (1.0 - Z[m]))[:, None, :]
        if m > 1:
            A, _ = layers[m - 1]                                # A[j, t] = w^m_{tj}
            dz = P[m] @ A                                       # [s, nL, n_{m-1}]
    return P[1:]


# --------------------------------------------------------------------------- outer Newton iteration

def combine_directions(theta, dims, C, XS, g, d, d_bar, eps=1e-5):
    """Coefficients (beta1, beta2) of the direction beta1 d + beta2 d_bar  (Section 4.3).

    They minimise  1/2 u^T G^S u + g^T u  over u = beta1 d + beta2 d_bar, G^S being the WHOLE
    subsampled Gauss-Newton matrix (also when d came from the block-diagonal systems), i.e.
    they solve the 2x2 system  [[d'Gd, db'Gd], [db'Gd, db'Gdb]] beta = [-g'd, -g'db].
    If its determinant is <= eps the system is taken as ill-conditioned and (1, 0) is returned.
    Also returns the three entries (d'Gd, db'Gd, db'Gdb) of the matrix.
    """
    g = np.asarray(g, dtype=np.float64)
    d = np.asarray(d, dtype=np.float64)
    d_bar = np.asarray(d_bar, dtype=np.float64)
    Gd = gn_matvec(theta, dims, C, XS, d)
    Gdb = gn_matvec(theta, dims, C, XS, d_bar)
    a11, a12, a22 = float(d @ Gd), float(d_bar @ Gd), float(d_bar @ Gdb)
    b1, b2 = -float(g @ d), -float(g @ d_bar)
    det = a11 * a22 - a12 * a12
    if det <= eps:
        return 1.0, 0.0, (a11, a12, a22)
    beta1 = (b1 * a22 - b2 * a12) / det
    beta2 = (a11 * b2 - a12 * b1) / det
    return beta1, beta2, (a11, a12, a22)


def line_search(theta, dims, C, X, Y, f0, gTd, d, eta=1e-4, max_trials=30):
    """Backtracking line search of Section 4.5: the largest alpha in {1, 1/2, 1/4, ...} with
    f(theta + alpha d) <= f(theta) + eta alpha grad f(theta)^T d.

    Returns (alpha, f(theta + alpha d), number of f evaluations); alpha = 0 (and f0) if none of the
    first max_trials candidates is accepted.
    """
    theta = np.asarray(theta, dtype=np.float64)
    d = np.asarray(d, dtype=np.float64)
    alpha = 1.0
    for k in range(max_trials):
        f_new = loss(theta + alpha * d, dims, C, X, Y)
        if f_new <= f0 + eta * alpha * gTd:
            return alpha, f_new, k + 1
        alpha *= 0.5
    return 0.0, f0, max_trials


def lm_update(lam, rho, drop=2.0 / 3.0, boost=1.5):
    """Levenberg-Marquardt rule of Section 4.5: lambda * drop if rho > 0.75, unchanged if
    0.25 <= rho <= 0.75, lambda * boost otherwise."""
    if rho > 0.75:
        return lam * drop
    if rho >= 0.25:
        return lam
    return lam * boost


def newton_step(theta, dims, C, X, Y, S, d_prev, lam, cg_max, sigma=1e-3, eta=1e-4, eps=1e-5,
                drop=2.0 / 3.0, boost=1.5, blockdiag=False, combine=True, max_trials=30, cg_min=0, r_percent=None):
    """One iteration of the subsampled Newton method (Section 4.5, the algorithm summarising the
    procedure, for a single partition owning every variable):

    gradient on all samples and the Gauss-Newton matrix on the rows S; CG on
    (G^S + lam I) d = -g (whole matrix, or the per-layer diagonal blocks); optional combination with the
    previous direction d_prev through the whole G^S; backtracking line search on f; ratio rho of actual to
    predicted reduction with the undamped G^S; next lam.

    Returns a dict: theta (new iterate), d (direction taken, to be passed as d_prev next time), lam (next),
    f_old, f_new, alpha, beta (pair), rho, gTd, dGd, cg_iters, f_evals.
    """
    theta = np.asarray(theta, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    Y = np.asarray(Y, dtype=np.float64)
    XS = X[np.asarray(S)]
    g, f0 = grad(theta, dims, C, X, Y)
    d, iters, _ = cg(theta, dims, C, XS, g, lam, cg_max, sigma=sigma, blockdiag=blockdiag, cg_min=cg_min,
                     r_percent=r_percent if blockdiag else None)
    if combine:
        beta1, beta2, (a11, a12, a22) = combine_directions(theta, dims, C, XS, g, d, d_prev, eps)
        d = beta1 * d + beta2 * np.asarray(d_prev, dtype=np.float64)
        dGd = beta1 * beta1 * a11 + 2.0 * beta1 * beta2 * a12 + beta2 * beta2 * a22
    else:
        beta1, beta2 = 1.0, 0.0
        dGd = float(d @ gn_matvec(theta, dims, C, XS, d))
    gTd = float(g @ d)
    alpha, f_new, evals = line_search(theta, dims, C, X, Y, f0, gTd, d, eta, max_trials)
    if alpha > 0.0:
        rho = (f_new - f0) / (alpha * gTd + 0.5 * alpha * alpha * dGd)
        lam_next = lm_update(lam, rho, drop, boost)
    else:
        rho = 0.0
        lam_next = lam * boost
    return dict(theta=theta + alpha * d, d=d, lam=lam_next, f_old=f0, f_new=f_new, alpha=alpha,
                beta=(beta1, beta2), rho=rho, gTd=gTd, dGd=dGd, cg_iters=iters, f_evals=evals)
