/*
 * CPU oracle for fused_linear_epilogue -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain float64 definition of the operator chain that the
 * GPU library fuses: a dense matmul z = x * W^T followed, in list order, by
 * elementwise and row-reduction ops with PyTorch-eager op semantics.  It is
 * what the paper's evaluator calls the "gold standard" side of its
 * comparison (Appendix A, Correctness): the original, unfused composition.
 * The fusion itself (Section 5.3: fusing a subgraph into one kernel removes
 * intermediate memory writes and launch overhead) never changes the
 * mathematical result, so the oracle is simply the definition written out.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this.  It shares no code, header, table or constant with the HIP path.
 *
 * Every op is local to one output row, so the outer loop over rows is the
 * only parallel loop; within a row everything runs in definition order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum {
    ORC_BIAS = 0,      /* z[n] += b[n]                                        */
    ORC_SCALE = 1,     /* z[n] *= alpha                                       */
    ORC_RELU = 2,      /* z[n] = max(z[n], 0), NaN kept                       */
    ORC_GELU_ERF = 3,  /* z * Phi(z), Phi = standard normal CDF (exact erf)   */
    ORC_GELU_TANH = 4, /* tanh approximation with the 0.044715 cubic term     */
    ORC_RESIDUAL = 5,  /* z[n] += r[m, n]                                     */
    ORC_LAYERNORM = 6, /* over the row, biased variance, eps inside the sqrt  */
    ORC_SOFTMAX = 7,   /* over the row, max-shifted                           */
    ORC_LOGSUMEXP = 8, /* over the row, max-shifted; output becomes one value */
    ORC_STORE = 9      /* t[m, n] = z[n]: a copy of the row as it stands; z unchanged */
};

typedef struct {
    int32_t kind;
    double alpha;     /* SCALE: factor.  LAYERNORM: eps.                       */
    const double *p0; /* RESIDUAL: r[M, ld].  LAYERNORM: gamma[N] or NULL (=1).  STORE: t[M, ld] (written) */
    const double *p1; /* LAYERNORM: beta[N] or NULL (=0)                       */
    int64_t ld;       /* RESIDUAL: row stride of r in elements                 */
} orc_op;

/* z[n] = sum_k x[k] * W[n, k]: the definition of a linear layer without bias. */
static void row_linear(const double *xrow, const double *w, int64_t ldw, int64_t N, int64_t K,
                       double *z) {
    for (int64_t n = 0; n < N; ++n) {
        const double *wrow = w + n * ldw;
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) acc += xrow[k] * wrow[k];
        z[n] = acc;
    }
}

static double row_max(const double *z, int64_t N) {
    double t = z[0];
    int has_nan = isnan(t);
    for (int64_t n = 1; n < N; ++n) {
        if (isnan(z[n])) has_nan = 1;
        if (z[n] > t) t = z[n];
    }
    return has_nan ? NAN : t;
}

/* Apply one op to row m held in z[0..N).  Returns the new row length. */
static int64_t row_apply(const orc_op *op, int64_t m, int64_t N, const double *b, double *z) {
    switch (op->kind) {
    case ORC_BIAS:
        for (int64_t n = 0; n < N; ++n) z[n] += b[n];
        return N;
    case ORC_SCALE:
        for (int64_t n = 0; n < N; ++n) z[n] *= op->alpha;
        return N;
    case ORC_RELU:
        for (int64_t n = 0; n < N; ++n)
            if (!(z[n] > 0.0) && !isnan(z[n])) z[n] = 0.0;
        return N;
    case ORC_GELU_ERF:
        for (int64_t n = 0; n < N; ++n) z[n] = 0.5 * z[n] * (1.0 + erf(z[n] / sqrt(2.0)));
        return N;
    case ORC_GELU_TANH: {
        const double c = sqrt(2.0 / M_PI);
        for (int64_t n = 0; n < N; ++n) {
            double v = z[n];
            z[n] = 0.5 * v * (1.0 + tanh(c * (v + 0.044715 * v * v * v)));
        }
        return N;
    }
    case ORC_RESIDUAL: {
        const double *r = op->p0 + m * op->ld;
        for (int64_t n = 0; n < N; ++n) z[n] += r[n];
        return N;
    }
    case ORC_STORE:
        memcpy((double *)op->p0 + m * op->ld, z, sizeof(double) * (size_t)N);
        return N;
    case ORC_LAYERNORM: {
        double mu = 0.0, var = 0.0;
        for (int64_t n = 0; n < N; ++n) mu += z[n];
        mu /= (double)N;
        for (int64_t n = 0; n < N; ++n) var += (z[n] - mu) * (z[n] - mu);
        var /= (double)N;
        double rstd = 1.0 / sqrt(var + op->alpha);
        for (int64_t n = 0; n < N; ++n) {
            double g = op->p0 ? op->p0[n] : 1.0;
            double be = op->p1 ? op->p1[n] : 0.0;
            z[n] = (z[n] - mu) * rstd * g + be;
        }
        return N;
    }
    case ORC_SOFTMAX: {
        double t = row_max(z, N), s = 0.0;
        for (int64_t n = 0; n < N; ++n) {
            z[n] = exp(z[n] - t);
            s += z[n];
        }
        for (int64_t n = 0; n < N; ++n) z[n] /= s;
        return N;
    }
    case ORC_LOGSUMEXP: {
        double t = row_max(z, N), s = 0.0;
        if (isinf(t)) { /* all -inf gives -inf, any +inf gives +inf, as the limit does */
            z[0] = t;
            return 1;
        }
        for (int64_t n = 0; n < N; ++n) s += exp(z[n] - t);
        z[0] = t + log(s);
        return 1;
    }
    default:
        return -1;
    }
}

/*
 * out = chain(x W^T).  All arrays are host float64, row-major.
 *   x [M, ldx>=K], w [N, ldw>=K], b [N] or NULL (needed by ORC_BIAS only),
 *   out [M, ldo>=N], or [M] (ldo ignored) when the chain ends in ORC_LOGSUMEXP.
 * ORC_LOGSUMEXP may only be the last op.  threads <= 0 means the OpenMP default.
 * Returns 0, or a negative value for an invalid argument (nothing is written then).
 */
int fle_oracle_run(int64_t M, int64_t N, int64_t K, const double *x, int64_t ldx, const double *w,
                   int64_t ldw, const double *b, const orc_op *ops, int32_t n_ops, double *out,
                   int64_t ldo, int32_t threads) {
    if (M < 0 || N <= 0 || K < 0 || n_ops < 0) return -1;
    if (M == 0) return 0;
    if (!x || !w || !out || (n_ops > 0 && !ops)) return -2;
    int ends_in_lse = 0;
    for (int32_t i = 0; i < n_ops; ++i) {
        int32_t kd = ops[i].kind;
        if (kd < ORC_BIAS || kd > ORC_STORE) return -3;
        if (kd == ORC_STORE && (!ops[i].p0 || ops[i].ld < N)) return -2;
        if (kd == ORC_BIAS && !b) return -2;
        if (kd == ORC_RESIDUAL && !ops[i].p0) return -2;
        if (kd == ORC_LOGSUMEXP) {
            if (i != n_ops - 1) return -4;
            ends_in_lse = 1;
        }
    }
    int failed = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)N);
        if (!z) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t m = 0; m < M; ++m) {
            if (!z) continue;
            row_linear(x + m * ldx, w, ldw, N, K, z);
            int64_t len = N;
            for (int32_t i = 0; i < n_ops; ++i) len = row_apply(&ops[i], m, len, b, z);
            if (ends_in_lse)
                out[m] = z[0];
            else
                memcpy(out + m * ldo, z, sizeof(double) * (size_t)N);
        }
        free(z);
    }
    return failed ? -5 : 0;
}

/*
 * Scaled dot-product attention over token-major operands, the definition written out (the
 * attention block that the paper's task-wise analysis, and its appendix on Level 3-pike and
 * Level 5 outliers, names as the largest recurring win once it is fused with its input and
 * output projections and masks causally on the fly):
 *
 *     s[j]   = scale * sum_d q[b,t,h,d] * k[b,j,h,d]        for every key j the mask allows
 *     p      = softmax over the allowed j
 *     o[b,t,h,:] = sum_j p[j] * v[b,j,h,:]
 *
 * causal = 1 allows keys j <= t only; causal = G > 1 is the same mask over groups of G consecutive
 * tokens (query t sees every key of its own and of earlier groups: j < (t / G + 1) * G), the form a
 * causal mask takes when a sequence is made of frames or patches that are not ordered internally.
 * There are T queries and Tk keys per sequence; with a causal mask the queries are the last T of
 * the Tk positions (query t stands at position t + Tk - T, as when earlier keys are kept from
 * previous calls), which needs Tk >= T.  Element (b,t,h,d) of q lives at q[(b*T + t)*ldq + h*D + d]
 * and likewise o; element (b,j,h,d) of k at k[(b*Tk + j)*ldk + h*D + d], likewise v.
 * Only queries t >= t_first are evaluated (the other rows of o are left
 * untouched), so that a few rows of a long sequence can be checked without computing all of them.
 * Returns 0, or a negative code for bad arguments / -5 out of memory.
 */
int fle_oracle_attention(int64_t B, int64_t H, int64_t T, int64_t Tk, int64_t D, const double *q, int64_t ldq,
                         const double *k, int64_t ldk, const double *v, int64_t ldv, int32_t causal,
                         double scale, double *o, int64_t ldo, int64_t t_first, int32_t threads) {
    if (B < 0 || H < 1 || T < 1 || Tk < 1 || D < 1 || t_first < 0 || t_first > T || causal < 0) return -1;
    if (causal && Tk < T) return -1;
    if (!q || !k || !v || !o) return -2;
    if (ldq < H * D || ldk < H * D || ldv < H * D || ldo < H * D) return -3;
    int failed = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Tk);
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int64_t b = 0; b < B; ++b)
            for (int64_t t = t_first; t < T; ++t) {
                if (!s) continue;
                int64_t keys = Tk;
                const int64_t pos = t + Tk - T;
                if (causal && (pos / causal + 1) * (int64_t)causal < Tk) keys = (pos / causal + 1) * (int64_t)causal;
                for (int64_t h = 0; h < H; ++h) {
                    const double *qr = q + (b * T + t) * ldq + h * D;
                    for (int64_t j = 0; j < keys; ++j) {
                        const double *kr = k + (b * Tk + j) * ldk + h * D;
                        double acc = 0.0;
                        for (int64_t d = 0; d < D; ++d) acc += qr[d] * kr[d];
                        s[j] = scale * acc;
                    }
                    const double mx = row_max(s, keys);
                    double sum = 0.0;
                    for (int64_t j = 0; j < keys; ++j) {
                        s[j] = exp(s[j] - mx);
                        sum += s[j];
                    }
                    double *orow = o + (b * T + t) * ldo + h * D;
                    for (int64_t d = 0; d < D; ++d) orow[d] = 0.0;
                    for (int64_t j = 0; j < keys; ++j) {
                        const double p = s[j] / sum;
                        const double *vr = v + (b * Tk + j) * ldv + h * D;
                        for (int64_t d = 0; d < D; ++d) orow[d] += p * vr[d];
                    }
                }
            }
        free(s);
    }
    return failed ? -5 : 0;
}

/* Number of threads the parallel loop above will use (for the timing report). */
int fle_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
