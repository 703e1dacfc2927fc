/*
 * Plain-C state oracle: Child-Sum Tree-LSTM forward, node by node, in fp64
 * (the parity reference).  Compiled a second time with -DORACLE_REAL=float the
 * same source gives the fp32 build that is only ever timed, never compared.
 *
 * TEST INFRASTRUCTURE ONLY - never linked into or called by the product.
 *
 * Same definition as treelstm_oracle.py (the paper cites the cell, section 3
 * describes it as 33 operators of which 4 depend on the number of children;
 * section 1 requires the batched run to equal the per-sample run):
 *
 *   hs  = sum_k h_k ;  i,o = sigmoid(W x + U hs + b) ;  u = tanh(W x + U hs + b)
 *   f_k = sigmoid(W_f x + U_f h_k + b_f) ;  c = i*u + sum_k f_k*c_k ;  h = o*tanh(c)
 *
 * Gate row order in W [4H,D], U [4H,H], b [4H]: i, o, u, f.
 * Trees are independent, so they are spread over OpenMP threads; inside a
 * tree nodes are visited in postorder, children in ascending id.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

static real sigmoid(real z) {
    if (z >= 0.0) return 1.0 / (1.0 + exp(-z));
    real e = exp(z);
    return e / (1.0 + e);
}

static real dot(const real *a, const real *v, int n) {
    real s = 0.0;
    for (int t = 0; t < n; ++t) s += a[t] * v[t];
    return s;
}

/* one node: children are k = cidx[0..nc) */
static void eval_node(int64_t j, const int32_t *cidx, int nc, int D, int H,
                      const real *x, const real *W, const real *U, const real *b,
                      real *h, real *c, real *hs, real *fx) {
    const real *xj = x + (size_t)j * D;
    for (int d = 0; d < H; ++d) hs[d] = 0.0;
    for (int q = 0; q < nc; ++q) {
        const real *hk = h + (size_t)cidx[q] * H;
        for (int d = 0; d < H; ++d) hs[d] += hk[d];
    }
    real *cj = c + (size_t)j * H, *hj = h + (size_t)j * H;
    for (int d = 0; d < H; ++d) {
        int ri = d, ro = H + d, ru = 2 * H + d, rf = 3 * H + d;
        real gi = sigmoid(dot(W + (size_t)ri * D, xj, D) + dot(U + (size_t)ri * H, hs, H) + b[ri]);
        real gu = tanh(dot(W + (size_t)ru * D, xj, D) + dot(U + (size_t)ru * H, hs, H) + b[ru]);
        cj[d] = gi * gu;
        fx[d] = dot(W + (size_t)rf * D, xj, D) + b[rf];
        (void)ro;
    }
    for (int q = 0; q < nc; ++q) {
        const real *hk = h + (size_t)cidx[q] * H;
        const real *ck = c + (size_t)cidx[q] * H;
        for (int d = 0; d < H; ++d) {
            real f = sigmoid(fx[d] + dot(U + (size_t)(3 * H + d) * H, hk, H));
            cj[d] += f * ck[d];
        }
    }
    for (int d = 0; d < H; ++d) {
        int ro = H + d;
        real go = sigmoid(dot(W + (size_t)ro * D, xj, D) + dot(U + (size_t)ro * H, hs, H) + b[ro]);
        hj[d] = go * tanh(cj[d]);
    }
}

/*
 * parent[n] (-1 = root), x[n*D], W[4H*D], U[4H*H], b[4H]  ->  h[n*H], c[n*H].
 * Returns 0, or -1 if the parent array is not a forest, -2 on allocation failure.
 * n_threads <= 0 means the OpenMP default.  *threads_used (optional) receives
 * the number of threads that ran.
 */
int oracle_treelstm_forward(int64_t n, const int32_t *parent, int D, int H,
                            const real *x, const real *W, const real *U, const real *b,
                            real *h, real *c, int n_threads, int *threads_used) {
    if (threads_used) *threads_used = 1;
    if (n == 0) return 0;
    int32_t *cptr = (int32_t *)calloc((size_t)n + 1, sizeof(int32_t));
    int32_t *cidx = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *fill = (int32_t *)calloc((size_t)n, sizeof(int32_t));
    int32_t *roots = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *order = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int32_t *stack = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    int64_t *tstart = (int64_t *)malloc(((size_t)n + 1) * sizeof(int64_t));
    if (!cptr || !cidx || !fill || !roots || !order || !stack || !tstart) return -2;
    int64_t nroots = 0;
    for (int64_t v = 0; v < n; ++v) {
        int32_t p = parent[v];
        if (p < -1 || p >= n || p == v) return -1;
        if (p < 0) roots[nroots++] = (int32_t)v; else cptr[p + 1]++;
    }
    for (int64_t v = 0; v < n; ++v) cptr[v + 1] += cptr[v];
    for (int64_t v = 0; v < n; ++v) {           /* ascending v => ascending lists */
        int32_t p = parent[v];
        if (p >= 0) cidx[cptr[p] + fill[p]++] = (int32_t)v;
    }
    /* postorder of every tree (children before parents), trees one after another */
    int64_t cnt = 0;
    memset(fill, 0, (size_t)n * sizeof(int32_t));    /* reuse: next child to visit */
    for (int64_t r = 0; r < nroots; ++r) {
        tstart[r] = cnt;
        int64_t sp = 0;
        stack[sp++] = roots[r];
        while (sp > 0) {
            int32_t v = stack[sp - 1];
            int32_t nc = cptr[v + 1] - cptr[v];
            if (fill[v] < nc) {
                if (sp >= n) return -1;
                stack[sp++] = cidx[cptr[v] + fill[v]++];
            } else {
                order[cnt++] = v;
                --sp;
            }
        }
    }
    tstart[nroots] = cnt;
    if (cnt != n) return -1;                     /* nodes on a cycle are never reached */

    int rc = 0;
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
#pragma omp parallel
    {
        real *hs = (real *)malloc((size_t)H * sizeof(real));
        real *fx = (real *)malloc((size_t)H * sizeof(real));
#ifdef _OPENMP
#pragma omp single
        { if (threads_used) *threads_used = omp_get_num_threads(); }
#endif
        if (!hs || !fx) {
#pragma omp atomic write
            rc = -2;
        } else {
#pragma omp for schedule(dynamic, 4)
            for (int64_t r = 0; r < nroots; ++r)
                for (int64_t q = tstart[r]; q < tstart[r + 1]; ++q) {
                    int32_t j = order[q];
                    eval_node(j, cidx + cptr[j], cptr[j + 1] - cptr[j], D, H, x, W, U, b, h, c, hs, fx);
                }
        }
        free(hs); free(fx);
    }
    free(cptr); free(cidx); free(fill); free(roots); free(order); free(stack); free(tstart);
    return rc;
}
