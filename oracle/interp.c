/*
 * CPU oracle: node-at-a-time interpreter for a dynamic computation graph.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP library is checked against; the product never calls it.  It shares no
 * code, header or table with the GPU path.
 *
 * What it follows: the paper evaluates a graph "in topological order" forward
 * and "in reverse topological order" backward (Section 3.3), and batching is
 * an exact reorganisation of that evaluation (Section 2, the manual and naive
 * versions compute the same value; Section 4.1 footnote, results are the same
 * regardless of batching strategy).  So the reference is the definition itself:
 * visit nodes 0..n-1 one at a time (ids are a topological order, Section 1
 * footnote on Wengert lists), then n-1..0 for reverse-mode differentiation.
 * No blocking, no batching, no reordering.
 *
 * Compiled twice: -DREAL=double (parity reference, finite differences) and
 * -DREAL=float (timed CPU baseline).
 *
 * Op codes (graph data format): 0 INPUT, 1 LOOKUP, 2 MATVEC, 3 ADD, 4 CMULT,
 * 5 TANH, 6 SIGMOID, 7 CONCAT, 8 SLICE, 9 PICK_NLS, 10 SQNORM.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#endif

enum { INPUT = 0, LOOKUP, MATVEC, ADD, CMULT, TANH_, SIGMOID, CONCAT, SLICE, PICK_NLS, SQNORM };

typedef struct {
    int64_t n;                /* number of nodes */
    const uint8_t *op;
    const uint32_t *out_dim;
    const uint32_t *in_off;   /* n+1 */
    const uint32_t *in_idx;
    const int32_t *param;
    const int32_t *bias;
    const int32_t *aux0;
    const int32_t *aux1;
    const float *payload;     /* INPUT vectors, fp32 as handed to both sides */
    int64_t n_params;
    const int64_t *p_rows;
    const int64_t *p_cols;
    const int64_t *p_off;     /* element offset of each parameter in pdata */
    const int64_t *v_off;     /* n+1: element offset of each node value (prefix sum of out_dim) */
} graph_t;

int oracle_real_bytes(void) { return (int)sizeof(REAL); }

/*
 * Forward (Section 3.3, "forward computation is done in topological order").
 * Per-node definitions are the ordinary ones for each operation the workloads
 * use: shared-weight matrix-vector product with optional bias (Appendix A,
 * "operations with shared elements"; affine transform A x + y), component-wise
 * sum / product / tanh / logistic (Appendix A, "component-wise operations"),
 * slice and concatenation (Section 3.2's slice signature example), embedding
 * lookup and softmax log-loss (Section 4.1, lookups and softmax are batched
 * across time steps), and the squared norm of Section 2's regression loss.
 */
int oracle_forward(const graph_t *g, const REAL *pdata, REAL *val)
{
    for (int64_t v = 0; v < g->n; ++v) {
        const uint32_t *in = g->in_idx + g->in_off[v];
        const int64_t arity = (int64_t)g->in_off[v + 1] - (int64_t)g->in_off[v];
        const int64_t d = g->out_dim[v];
        REAL *y = val + g->v_off[v];
        switch (g->op[v]) {
        case INPUT:
            for (int64_t i = 0; i < d; ++i) y[i] = (REAL)g->payload[g->aux0[v] + i];
            break;
        case LOOKUP: {
            const REAL *E = pdata + g->p_off[g->param[v]];
            const int64_t cols = g->p_cols[g->param[v]];
            for (int64_t i = 0; i < d; ++i) y[i] = E[(int64_t)g->aux0[v] * cols + i];
            break;
        }
        case MATVEC: {
            const REAL *W = pdata + g->p_off[g->param[v]];
            const int64_t m = g->p_rows[g->param[v]], k = g->p_cols[g->param[v]];
            const REAL *x = val + g->v_off[in[0]];
            if (m != d || arity != 1) return -1;
            for (int64_t i = 0; i < m; ++i) {
                REAL acc = 0;
                for (int64_t j = 0; j < k; ++j) acc += W[i * k + j] * x[j];
                if (g->bias[v] >= 0) acc += pdata[g->p_off[g->bias[v]] + i];
                y[i] = acc;
            }
            break;
        }
        case ADD:
            for (int64_t i = 0; i < d; ++i) {
                REAL acc = 0;
                for (int64_t j = 0; j < arity; ++j) acc += val[g->v_off[in[j]] + i];
                y[i] = acc;
            }
            break;
        case CMULT:
            if (arity != 2) return -1;
            for (int64_t i = 0; i < d; ++i)
                y[i] = val[g->v_off[in[0]] + i] * val[g->v_off[in[1]] + i];
            break;
        case TANH_:
            for (int64_t i = 0; i < d; ++i) y[i] = (REAL)tanh((double)val[g->v_off[in[0]] + i]);
            break;
        case SIGMOID:
            for (int64_t i = 0; i < d; ++i)
                y[i] = (REAL)(1.0 / (1.0 + exp(-(double)val[g->v_off[in[0]] + i])));
            break;
        case CONCAT: {
            int64_t o = 0;
            for (int64_t j = 0; j < arity; ++j) {
                const int64_t dj = g->out_dim[in[j]];
                for (int64_t i = 0; i < dj; ++i) y[o + i] = val[g->v_off[in[j]] + i];
                o += dj;
            }
            if (o != d) return -1;
            break;
        }
        case SLICE:
            for (int64_t i = 0; i < d; ++i) y[i] = val[g->v_off[in[0]] + g->aux0[v] + i];
            break;
        case PICK_NLS: {
            /* -log softmax(x)[label], written so that a confident row keeps its digits: with
             * m the index of the row maximum,
             *   logsumexp(x) - x_label = log(1 + sum_{i != m} exp(x_i - x_m)) + (x_m - x_label).
             * The textbook form x_m + log(sum_i exp(x_i - x_m)) - x_label is the same number but
             * rounds a loss below 1e-16 * |x_m| to zero, which is coarser than the 1e-4 relative
             * bar the batched path is held to. */
            const REAL *x = val + g->v_off[in[0]];
            const int64_t K = g->out_dim[in[0]];
            int64_t m = 0;
            double s = 0;
            for (int64_t i = 1; i < K; ++i) if ((double)x[i] > (double)x[m]) m = i;
            for (int64_t i = 0; i < K; ++i) if (i != m) s += exp((double)x[i] - (double)x[m]);
            y[0] = (REAL)(log1p(s) + ((double)x[m] - (double)x[g->aux0[v]]));
            break;
        }
        case SQNORM: {
            const REAL *x = val + g->v_off[in[0]];
            const int64_t K = g->out_dim[in[0]];
            REAL acc = 0;
            for (int64_t i = 0; i < K; ++i) acc += x[i] * x[i];
            y[0] = acc;
            break;
        }
        default:
            return -2;
        }
    }
    return 0;
}

/*
 * Backward (Section 3.3, "backward calculation is done in reverse topological
 * order"; Section 2, Backward(L) returns dL/dtheta).  All gradients start at
 * zero, the root (a scalar node) is seeded with 1, and each node, visited in
 * descending id, adds its adjoint contribution to its operands and parameters.
 */
int oracle_backward(const graph_t *g, const REAL *pdata, const REAL *val, int64_t root,
                    REAL *grad, REAL *pgrad)
{
    if (root < 0 || root >= g->n || g->out_dim[root] != 1) return -3;
    memset(grad, 0, sizeof(REAL) * (size_t)g->v_off[g->n]);
    {
        int64_t tot = 0;
        for (int64_t p = 0; p < g->n_params; ++p) tot += g->p_rows[p] * g->p_cols[p];
        memset(pgrad, 0, sizeof(REAL) * (size_t)tot);
    }
    grad[g->v_off[root]] = 1;
    for (int64_t v = g->n - 1; v >= 0; --v) {
        const uint32_t *in = g->in_idx + g->in_off[v];
        const int64_t arity = (int64_t)g->in_off[v + 1] - (int64_t)g->in_off[v];
        const int64_t d = g->out_dim[v];
        const REAL *gy = grad + g->v_off[v];
        const REAL *y = val + g->v_off[v];
        switch (g->op[v]) {
        case INPUT:
            break;
        case LOOKUP: {
            REAL *dE = pgrad + g->p_off[g->param[v]];
            const int64_t cols = g->p_cols[g->param[v]];
            for (int64_t i = 0; i < d; ++i) dE[(int64_t)g->aux0[v] * cols + i] += gy[i];
            break;
        }
        case MATVEC: {
            const REAL *W = pdata + g->p_off[g->param[v]];
            REAL *dW = pgrad + g->p_off[g->param[v]];
            const int64_t m = g->p_rows[g->param[v]], k = g->p_cols[g->param[v]];
            const REAL *x = val + g->v_off[in[0]];
            REAL *dx = grad + g->v_off[in[0]];
            for (int64_t i = 0; i < m; ++i) {
                for (int64_t j = 0; j < k; ++j) {
                    dx[j] += W[i * k + j] * gy[i];
                    dW[i * k + j] += gy[i] * x[j];
                }
                if (g->bias[v] >= 0) pgrad[g->p_off[g->bias[v]] + i] += gy[i];
            }
            break;
        }
        case ADD:
            for (int64_t j = 0; j < arity; ++j)
                for (int64_t i = 0; i < d; ++i) grad[g->v_off[in[j]] + i] += gy[i];
            break;
        case CMULT:
            for (int64_t i = 0; i < d; ++i) {
                const REAL a = val[g->v_off[in[0]] + i], b = val[g->v_off[in[1]] + i];
                grad[g->v_off[in[0]] + i] += gy[i] * b;
                grad[g->v_off[in[1]] + i] += gy[i] * a;
            }
            break;
        case TANH_:
            for (int64_t i = 0; i < d; ++i) grad[g->v_off[in[0]] + i] += gy[i] * (1 - y[i] * y[i]);
            break;
        case SIGMOID:
            for (int64_t i = 0; i < d; ++i) grad[g->v_off[in[0]] + i] += gy[i] * y[i] * (1 - y[i]);
            break;
        case CONCAT: {
            int64_t o = 0;
            for (int64_t j = 0; j < arity; ++j) {
                const int64_t dj = g->out_dim[in[j]];
                for (int64_t i = 0; i < dj; ++i) grad[g->v_off[in[j]] + i] += gy[o + i];
                o += dj;
            }
            break;
        }
        case SLICE:
            for (int64_t i = 0; i < d; ++i) grad[g->v_off[in[0]] + g->aux0[v] + i] += gy[i];
            break;
        case PICK_NLS: {
            /* d/dx_i [logsumexp(x) - x_label] = softmax(x)_i - [i == label].  For i == label the
             * difference p_label - 1 is taken as -(sum of the other probabilities), the same
             * number without the cancellation when p_label is close to 1. */
            const REAL *x = val + g->v_off[in[0]];
            REAL *dx = grad + g->v_off[in[0]];
            const int64_t K = g->out_dim[in[0]];
            const int64_t label = g->aux0[v];
            int64_t m = 0;
            double s = 0, others = 0;
            for (int64_t i = 1; i < K; ++i) if ((double)x[i] > (double)x[m]) m = i;
            for (int64_t i = 0; i < K; ++i) if (i != m) s += exp((double)x[i] - (double)x[m]);
            for (int64_t i = 0; i < K; ++i)
                if (i != label) others += exp((double)x[i] - (double)x[m]) / (1.0 + s);
            for (int64_t i = 0; i < K; ++i) {
                const double p = (i == label) ? -others : exp((double)x[i] - (double)x[m]) / (1.0 + s);
                dx[i] += (REAL)((double)gy[0] * p);
            }
            break;
        }
        case SQNORM: {
            const REAL *x = val + g->v_off[in[0]];
            REAL *dx = grad + g->v_off[in[0]];
            const int64_t K = g->out_dim[in[0]];
            for (int64_t i = 0; i < K; ++i) dx[i] += 2 * gy[0] * x[i];
            break;
        }
        default:
            return -2;
        }
    }
    return 0;
}
