/*
 * dn.h -- C-ABI of libdn: the subsampled Gauss-Newton path of the Newton method for
 * fully-connected networks ("Distributed Newton Methods for Deep Neural Networks"), on one
 * AMD MI355X (gfx950).
 *
 * Network n_0-n_1-...-n_L, sigmoid hidden layers, linear output layer, squared loss
 * (Section 2.1, Section 3.3.2).  Notation follows the paper: W^m is n_{m-1} x n_m,
 * s^{m,i} = (W^m)^T z^{m-1,i} + b^m, z^{m,i} = sigma(s^{m,i}), l samples, n parameters.
 *
 * Conventions for every call
 *   - All array arguments are DEVICE pointers to fp32 unless the name ends in _host.
 *     Matrices are dense row-major with the sample index leading: X is [l x n_0],
 *     Y is [l x n_L] (one-hot class targets, or any real targets).
 *   - Parameter-shaped vectors (theta, g, v, out, d) use the layout of Section 2.1:
 *     for m = 1..L the n_m x n_{m-1} matrix (W^m)^T row-major, then the n_m biases.
 *   - The caller owns every buffer.  The library borrows argument pointers for the duration
 *     of the call only, except the workspace given to dn_bind, which it keeps using until the
 *     context is destroyed or re-bound.  The library itself allocates no device memory.
 *   - Work is enqueued on the HIP stream given to dn_bind.  Calls that return a host scalar
 *     (f, iteration counts, residual norms) synchronise that stream before returning; the
 *     others return as soon as the work is enqueued.
 *   - Every call returns DN_OK (0) or a negative error code; nothing is thrown across the ABI.
 *     Arguments are validated on the host before anything is launched.
 */
#ifndef DN_H
#define DN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dn_ctx dn_ctx;

enum {
    DN_OK = 0,
    DN_EINVAL = -1,   /* null pointer, non-positive size, s > s_max, bad mode, layer or parameter */
    DN_ENOSPC = -2,   /* workspace given to dn_bind is smaller than dn_workspace_bytes() */
    DN_ESTATE = -3,   /* call needs a bound workspace / a prior dn_jacobian_prep and there is none */
    DN_EHIP = -4,     /* a HIP runtime call failed; dn_last_hip_error() gives the HIP code */
    DN_ENOMEM = -5,   /* host allocation failed */
    DN_ETOOBIG = -7,  /* dn_forward_static: the problem needs more than DN_STATIC_SCRATCH_BYTES of scratch */
    DN_ETIMEOUT = -6  /* a bounded wait between work-groups of a kernel ran out; the products fell back to the
                         two-pass kernels (see dn_set_spin_limit, dn_sync_status) */
};

/* mode of dn_gn_matvec and dn_cg */
enum {
    DN_FULL = 0,      /* whole subsampled Gauss-Newton matrix (Section 4.3) */
    DN_BLOCKDIAG = 1, /* its diagonal blocks, one block per layer = W^m with b^m (Section 4.1) */
    DN_PARTITION = 2  /* its diagonal blocks for the split structure given to dn_set_split (Section 3.1, 4.1) */
};

/* Human-readable text for an error code (static storage). */
const char* dn_strerror(int code);

/*
 * Create a context for the network dims[0..L] (L >= 1 weight layers, every entry >= 1) with
 * regularisation parameter C > 0 of the objective (Section 2.1).  l_max is the number of rows whose
 * activations the workspace holds at a time: dn_forward / dn_grad take any number of rows l and send
 * them through in ceil(l / l_max) chunks that reuse the same buffers (the mini-batch pipeline of
 * Section 6.1: memory / R for R chunks; the results are the same sums).  s_max bounds the subsample
 * size passed to dn_jacobian_prep.  Both size the workspace.  Host-only: touches no device.
 */
int dn_create(dn_ctx** out, int L, const int* dims, double C, int l_max, int s_max);
void dn_destroy(dn_ctx* ctx);

/* n = sum_m (n_{m-1} n_m + n_m)  (Section 2.1).  0 if ctx is null. */
size_t dn_num_params(const dn_ctx* ctx);

/* Bytes of device workspace the context needs (activations for l_max rows, the stored
 * Jacobian blocks and activations for s_max rows, product temporaries, CG vectors). */
size_t dn_workspace_bytes(const dn_ctx* ctx);

/*
 * Host-only: number of slices into which a product (dn_gn_matvec, dn_cg, dn_gn_matvec_rop) on s stored samples
 * cuts its sums over samples (Section 4.2's outer sums; each slice writes partial sums to the workspace, which
 * are folded in a fixed order).  Always >= 1 and always a plan that fits a workspace of dn_workspace_bytes()
 * for every 1 <= s <= s_max; DN_EINVAL for a null context or s outside that range.
 */
int dn_product_slices(const dn_ctx* ctx, int s);

/*
 * Host-only: which of nprob (1..8) dense products C_i[M_i x N_i] = A_i[M_i x K_i] B_i[N_i x K_i]^T, issued as ONE
 * launch of the tile engine with both operands K-contiguous (the forward pass of Section 2.1, the back-propagation of
 * Section 2.2, the sweeps of Section 3.3, the inner sums of Section 4.2), go through 128 x 128 tiles (large[i] = 1)
 * and which through 64 x 64 tiles (large[i] = 0).  Large tiles are taken when there are at least 512 of them, they
 * fill whole rounds of work-groups and lose little to padding; a launch may be split into a large-tile and a
 * small-tile part.  Returns the number of problems on large tiles, or DN_EINVAL (null pointers, nprob outside 1..8,
 * a non-positive size).  No device is touched; for tests of the launch planning.
 */
int dn_gemm_large_tiles(int nprob, const int* M, const int* N, const int* K, int* large);

/*
 * Lend the context a device workspace of at least dn_workspace_bytes() bytes, 256-byte
 * aligned, and the HIP stream (hipStream_t passed as void*, NULL = default stream) on which
 * all later work is enqueued.  Invalidates a previous dn_jacobian_prep.
 */
int dn_bind(dn_ctx* ctx, void* d_workspace, size_t bytes, void* hip_stream);

/*
 * Objective value (Section 2.1):
 *   f = theta^T theta / (2C) + (1/l) sum_i || z^{L,i} - y^i ||^2 .
 * All l rows of X and Y are used (in chunks of l_max rows).  *f_host receives f (fp64 accumulation of
 * fp32 terms).
 * If ZL is non-null it receives the network outputs, [l x n_L] dense.
 */
int dn_forward(dn_ctx* ctx, const float* theta, const float* X, const float* Y, int l,
               double* f_host, float* ZL);

/*
 * dn_forward for callers that cannot allocate device memory or keep a workspace: tight serving loops, harnesses
 * that forbid hipMalloc, processes that may not grow their memory once they run.  Same value f (and outputs ZL,
 * nullable) as dn_forward on a context with l_max >= l, but no context and no workspace: the activations and
 * partial sums live in a scratch array that is part of the library's device code (DN_STATIC_SCRATCH_BYTES per GPU,
 * held from the first call on that GPU until the process ends).  The call allocates nothing, on the host or on
 * the device.  (It returns f on the host and therefore synchronises the stream: it cannot itself be recorded
 * into a graph.)
 * dims[0..L], C as in dn_create; theta, X, Y, ZL are device pointers as in dn_forward; the work is enqueued on
 * hip_stream (hipStream_t as void*, NULL = default stream), which is synchronised before *f_host is written.
 * The scratch needed is 4 l sum_{m=1..L} roundup4(n_m) bytes plus 17 KB; a problem beyond the limit is rejected
 * with DN_ETOOBIG before anything is launched (split the rows and add the loss terms, or use dn_forward).
 * All calls on one GPU share that GPU's scratch: calls that overlap in time on the same GPU race; calls one
 * after the other need no clean-up in between (the call writes every word of the scratch before it reads it).
 */
#define DN_STATIC_SCRATCH_BYTES (32u << 20)
int dn_forward_static(int L, const int* dims, double C, const float* theta, const float* X, const float* Y, int l,
                      void* hip_stream, double* f_host, float* ZL);

/*
 * Gradient by back-propagation (Section 2.2, Section 3.4):
 *   g = theta/C + (1/l) sum_i (J^i)^T 2 (z^{L,i} - y^i),   g in theta layout.
 * f_host may be null; otherwise it receives f as dn_forward does (and the call synchronises).
 */
int dn_grad(dn_ctx* ctx, const float* theta, const float* X, const float* Y, int l,
            float* g, double* f_host);

/*
 * Prepare the subsampled Gauss-Newton matrix for the rows S of X (Section 3.3, Section 4.3):
 * forward pass on the s = |S| selected rows keeping z^{m,i}, then the n_L simultaneous
 * backward sweeps that produce and store
 *   P^m_i[u][j] = d z^{L,i}_u / d s^{m,i}_j ,  m = 1..L-1      (P^L_i is the identity)
 * in the workspace.  S is a DEVICE array of s row indices into X, each in [0, l); repeated
 * indices are allowed (they simply count twice).  1 <= s <= s_max.
 * theta and X need not stay alive afterwards: everything the products need is in the workspace.
 */
int dn_jacobian_prep(dn_ctx* ctx, const float* theta, const float* X, int l, const int* S, int s);

/*
 * Copy stored block P^m (1 <= m <= L-1) to P_out as a dense [s][n_L][n_m] array.  For tests and
 * inspection; needs a prior dn_jacobian_prep.
 */
int dn_jacobian_read(dn_ctx* ctx, int m, float* P_out);

/*
 * out = G^S v  (no damping term), computed from the stored blocks by the factored products of
 * Section 4.2:
 *   DN_FULL:       out = v/C + (1/|S|) sum_{i in S} (J^i)^T B^i J^i v,            B^i = 2I
 *   DN_BLOCKDIAG:  out_m = v_m/C + (1/|S|) sum_{i in S} (J^i_m)^T B^i J^i_m v_m   for each layer m
 * v and out must not overlap.  Needs a prior dn_jacobian_prep.
 * The call only enqueues kernels (no allocation, no copy or memset node, no synchronisation, while profiling is
 * off), so it may be captured in a HIP graph and replayed with new contents in v: whatever the kernels keep
 * between launches (the sequence numbers of the single-pass kernel in which work-groups share a sample) lives in the workspace.
 */
int dn_gn_matvec(dn_ctx* ctx, const float* v, float* out, int mode);

/*
 * out = G^S v (whole matrix, no damping) WITHOUT the stored blocks: J^i v by differentiating the forward pass
 * along v (the R-operator approach that Section 2.2 mentions and Section 3 sets aside as sequential over the
 * layers), then (J^i)^T by back-propagation, all as dense products on the subsample's activations kept by
 * dn_jacobian_prep.  Same result as dn_gn_matvec(DN_FULL) up to rounding; on one GPU it is an independent
 * cross-check and the comparator for what storing the blocks costs or saves.  Needs a prior dn_jacobian_prep.
 */
int dn_gn_matvec_rop(dn_ctx* ctx, const float* v, float* out);

/*
 * Conjugate gradient on (G^S + lambda I) d = -g  (Section 2.2, Section 4.3), d_0 = 0, no
 * preconditioner, at most max_iter >= 1 iterations.  After every iteration the recurrence residual
 * r is tested: stop when ||r|| <= sigma ||g||  (Section 4.1).  sigma = 0 runs exactly max_iter
 * iterations without any host synchronisation inside the loop.
 * DN_BLOCKDIAG solves the L per-layer systems independently (own step lengths, own test;
 * a block that met its test is frozen).
 * Outputs: d (device, theta layout); *iters_host = iterations run; resnorm_host[0] (DN_FULL) or
 * resnorm_host[0..L-1] (DN_BLOCKDIAG) = final ||r|| per system.  Dot products are accumulated
 * in fp64.  g and d must not overlap.  Needs a prior dn_jacobian_prep.
 */
int dn_cg(dn_ctx* ctx, const float* g, double lambda, double sigma, int max_iter, int mode,
          float* d, int* iters_host, double* resnorm_host);

/*
 * dn_cg on independent systems (mode DN_BLOCKDIAG or DN_PARTITION) with the early termination of Section 4.4: besides each
 * block's own test and max_iter, ALL blocks stop after the first iteration k >= cg_min at which the number
 * of blocks that have met their own test is >= r_percent/100 of the number of blocks (0 < r_percent <= 100;
 * cg_min >= 0).  On one GPU the blocks advance in lock-step, so "every partition has run cg_min iterations"
 * is k >= cg_min; the rule then only cuts iterations, it saves no waiting.  Outputs as dn_cg with one
 * resnorm_host entry per system.  The host looks at the blocks' state after every iteration (one synchronisation each).
 */
int dn_cg_sync(dn_ctx* ctx, const float* g, double lambda, double sigma, int max_iter, int mode, int cg_min,
               double r_percent, float* d, int* iters_host, double* resnorm_host);

/*
 * One iteration of the subsampled Newton method (Section 4.5, the algorithm that summarises the
 * procedure, for one partition that owns every variable):
 *   1. g = grad f(theta) and f(theta) on all l rows;
 *   2. dn_jacobian_prep on the rows S (the subsample S_k of this iteration, chosen by the caller);
 *   3. d = CG solution of (G^S + lambda I) d = -g, whole matrix or per-layer blocks (params->mode),
 *      stopped by params->sigma or after params->cg_max iterations;
 *   4. if params->combine: d <- beta1 d + beta2 d_prev, (beta1, beta2) minimising
 *      1/2 u^T G^S u + g^T u over u = beta1 d + beta2 d_prev with the WHOLE G^S (two extra products);
 *      (beta1, beta2) = (1, 0) when the determinant of the 2x2 system is <= params->eps (Section 4.3);
 *   5. backtracking line search: the largest alpha in {1, 1/2, 1/4, ...} (at most params->max_trials
 *      candidates) with f(theta + alpha d) <= f(theta) + eta alpha g^T d;
 *   6. rho = (f(theta + alpha d) - f(theta)) / (alpha g^T d + alpha^2/2 d^T G^S d);
 *      lambda <- lambda*drop if rho > 0.75, unchanged if 0.25 <= rho <= 0.75, else lambda*boost.
 * theta (device, n floats) is advanced in place to theta + alpha d; d_prev (device, n floats; zeros before
 * the first iteration) receives the direction taken; params->lambda receives the next lambda.
 * If no candidate step is accepted, theta is left unchanged, alpha = 0 is reported and lambda is boosted.
 * The 2x2 system, the step-size test and the lambda rule are evaluated on the host in fp64 from dot
 * products accumulated in fp64 on the device.  The call synchronises the stream several times.
 * X is [l x n_0], Y is [l x n_L], S holds s row indices (device), as in dn_grad / dn_jacobian_prep.
 */
typedef struct dn_newton_params {
    double lambda;      /* in: lambda_k; out: lambda_{k+1} */
    double sigma;       /* CG stopping tolerance (0: run cg_max iterations) */
    double eta;         /* sufficient-decrease constant, 0 < eta < 1 */
    double eps;         /* determinant threshold of the two-variable system */
    double drop, boost; /* factors of the lambda rule, 0 < drop <= 1 <= boost */
    int cg_max;         /* >= 1 */
    int mode;           /* DN_FULL, DN_BLOCKDIAG or DN_PARTITION: matrix of the CG systems */
    int combine;        /* nonzero: step 4 */
    int max_trials;     /* >= 1 */
    int cg_min;         /* with independent systems and r_percent > 0: early termination as in dn_cg_sync */
    double r_percent;   /* <= 0: every block runs to its own test */
    int reuse_forward;  /* nonzero: the caller states that theta, X and Y are exactly as the previous
                           dn_newton_step on this context left them (same pointers, contents untouched, no
                           other call on the context in between).  The activations of the accepted line-search
                           point are then still in the workspace and the gradient skips its forward pass.
                           Ignored (full evaluation) when the library cannot confirm the pointers and l, after a
                           step that accepted no point, or when l exceeds l_max. */
} dn_newton_params;

typedef struct dn_newton_stats {
    double f_old, f_new;   /* f(theta) before and after the step */
    double alpha;          /* accepted step size, 0 if none */
    double beta1, beta2;   /* combination coefficients ((1,0) if not combined) */
    double rho;            /* actual / predicted reduction */
    double gTd, dGd;       /* g^T d and d^T G^S d of the direction taken */
    int cg_iters;          /* CG iterations run */
    int f_evals;           /* objective evaluations of the line search */
} dn_newton_stats;

int dn_newton_step(dn_ctx* ctx, float* theta, const float* X, const float* Y, int l, const int* S, int s,
                   float* d_prev, dn_newton_params* params, dn_newton_stats* stats_host);

/*
 * Split structure for DN_PARTITION (Section 3.1): groups[m], m = 0..L, is the number of contiguous,
 * as-equal-as-possible neuron groups of layer m (1 <= groups[m] <= min(4, n_m)); group k of a layer with
 * n neurons is [floor(k n / groups), floor((k+1) n / groups)).  The weights from group a of layer m-1 to
 * group b of layer m form one partition; the biases of group b go with the partition of a = 0.  Partitions
 * are numbered layer by layer, a outer, b inner; dn_num_partitions gives their count (sum of
 * groups[m-1] * groups[m]).  Needs a bound workspace (an index map of n ints is uploaded); dn_bind
 * forgets it.  With mode DN_PARTITION dn_gn_matvec applies the diagonal blocks of G^S over these
 * partitions, dn_cg / dn_cg_sync solve the independent systems (resnorm_host then has
 * dn_num_partitions entries), dn_newton_step uses them in its CG.  All groups[m] = 1 is DN_BLOCKDIAG.
 * The stored blocks are read once per product as in the other modes.
 */
int dn_set_split(dn_ctx* ctx, const int* groups);
int dn_num_partitions(const dn_ctx* ctx);

/*
 * Products whose stored blocks do not fit one work-group's registers (n_L > 16, or hidden layers wider than 8192
 * in total; at least two hidden layers) read each stored block ONCE per product by letting a team of work-groups
 * share a sample (the kernel's work-groups exchange partial sums through device memory and wait for each other;
 * every wait is bounded).  dn_set_stream_passes(ctx, 2) selects the plain two-pass kernels instead (one read
 * for J v, one for J^T), 0 restores the automatic choice.
 * dn_set_spin_limit sets the number of polls after which such a wait gives up (default 1 << 20, a few
 * seconds; it can only run out when the kernel's work-groups cannot all be resident, e.g. beside another
 * process's kernels).  A wait that runs out makes the kernel's work-groups leave; the two-pass kernels, which
 * are enqueued behind every single-pass launch and otherwise return at once, then compute the same product, so
 * results are complete either way.  The next synchronising call notices the condition and the context uses
 * the two-pass kernels directly until dn_bind; dn_sync_status reports it ONCE as DN_ETIMEOUT (information,
 * not a failure).
 */
int dn_set_stream_passes(dn_ctx* ctx, int passes);
int dn_set_spin_limit(dn_ctx* ctx, unsigned polls);
/* Wait for all work enqueued so far; DN_OK, DN_ETIMEOUT (once, see above) or DN_EHIP. */
int dn_sync_status(dn_ctx* ctx);

/*
 * Kernel timing.  With profiling enabled every launch of the library's kernels is bracketed
 * by HIP events on the bound stream; dn_profile_read returns, for kernel class `which`
 * (0 <= which < dn_profile_num_classes()), the summed duration in milliseconds and the
 * number of launches since the last dn_profile_reset.  Reading synchronises the stream.
 */
int dn_profile_enable(dn_ctx* ctx, int on);
/* Restrict the bracketing to the kernel classes whose bit is set (bit k = class k); default all. */
int dn_profile_select(dn_ctx* ctx, unsigned long long class_mask);
int dn_profile_reset(dn_ctx* ctx);
int dn_profile_num_classes(void);
const char* dn_profile_class_name(int which);
int dn_profile_read(dn_ctx* ctx, int which, double* total_ms_host, long long* launches_host);

/*
 * Phase clocks of the single-pass kernel in which work-groups share a sample (see dn_set_stream_passes): with on != 0 every later
 * launch of that kernel also records, per work-group, the shader-clock cycles it spent (a) from a band's first
 * load to the barrier behind its partial sums, (b) from there to the barrier behind the exchange with the other
 * work-groups of its team (the wait for the slowest of them plus one round trip through memory) and (c) in the
 * transposed product.  dn_profile_band_read synchronises the stream and returns, for the LAST such launch, the
 * mean cycles per band of the three phases in cycles_host[0..2] and the mean number of bands per work-group in
 * *bands_host (all zero if no such launch was made).  Costs two clock reads per phase; off by default.
 */
int dn_profile_band_phases(dn_ctx* ctx, int on);
int dn_profile_band_read(dn_ctx* ctx, double* cycles_host, double* bands_host);

/* HIP error code of the most recent DN_EHIP on this context (0 if none). */
int dn_last_hip_error(const dn_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* DN_H */
