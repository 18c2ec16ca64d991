/*
 * fp64 CPU oracle for GFormer attention forward.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU library computes.  It
 * shares no source, header, table or helper with the HIP path and must never be
 * linked or called by it; only the tests, the smoke check and the cpu_baseline
 * leg of the benchmark use it.
 *
 * What is computed (GFormer, arXiv 2412.19829):
 *   - Section III-A: heads are split in two groups.  Heads [0, H0) run windowed
 *     causal softmax attention, heads [H0, H) run causal linear attention.  The
 *     output of head h lands in head h's slot; nothing is summed across groups.
 *   - Section III-B: windowed head.  Token i attends to the w tokens ending at
 *     itself, j in [max(0, i-w+1), i]; softmax (Eq. 1, with the causal mask of
 *     section II-A) over exactly those scores; weighted sum of V rows.
 *   - Section III-C, Algorithm 1: linear head.  A (E x E) and Z (E) are running
 *     sums of phi(K_j) (x) V_j and phi(K_j) over j <= i (token i is added before
 *     row i is read out); H_i = phi(Q_i)^T A / (phi(Q_i) . Z).  The printed last
 *     line of the algorithm names an undefined S and K'; it is read as Q'^T A,
 *     which is what the prose around it and section II-B describe.
 *   - Section II-B: phi(x) = elu(x) + 1.
 *   - Bidirectional variant (section IV's encoder / image workloads): window centred on the
 *     token, linear head over all keys; routines *_bidir_* below.
 *   - Section III-A (design text): positive random features as an alternative phi, applied as a
 *     pre-map of Q and K (gformer_oracle_random_features_f64 below) in front of Algorithm 1
 *     run with the identity map.
 *
 *   - Backward pass (the gradients training needs; the paper trains its models, sections IV-B to
 *     IV-D, but prints no backward formulas): routines *_bwd_* below are the derivatives of the
 *     two definitions above, written out term by term (chain rule through Eq. 1's softmax, and
 *     through the ratio of section II-B with weights a_ij = phi(q_i).phi(k_j)).
 *
 * Two routines cover the linear head: the explicit O(N^2) masked sum (the plain
 * definition: weights a_ij = phi(q_i).phi(k_j), j <= i) and Algorithm 1's
 * recurrence.  They are written separately and are tested against each other.
 *
 * Layout: dense row-major [B, H, N, d] doubles.  All arithmetic in double.
 * Pins: see tests/test_oracle_pins.py (worked 4-token examples in exact
 * rationals, a library softmax-attention routine, closed forms, invariants).
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_PHI_ELU1 = 0, ORACLE_PHI_IDENTITY = 1 };
enum { ORACLE_LINEAR_QUADRATIC = 0, ORACLE_LINEAR_RECURRENT = 1 };

/* Section II-B: phi(x) = elu(x) + 1, i.e. x + 1 for x > 0 and exp(x) otherwise. */
static double feature_map(double x, int phi)
{
    if (phi == ORACLE_PHI_IDENTITY) return x;
    return x > 0.0 ? x + 1.0 : exp(x);
}

/* Section III-B + Eq. 1: one windowed causal softmax head, [N, d] row-major. */
int gformer_oracle_windowed_head_f64(const double *q, const double *k, const double *v,
                                     double *out, int N, int d, int window, double scale)
{
    if (!q || !k || !v || !out || N < 0 || d < 1 || window < 1) return 1;
    double *s = (double *)malloc(sizeof(double) * (size_t)(window > N ? (N > 0 ? N : 1) : window));
    if (!s) return 2;
    for (int i = 0; i < N; ++i) {
        int lo = i - window + 1;
        if (lo < 0) lo = 0;
        int cnt = i - lo + 1;
        double m = -INFINITY;
        for (int j = lo; j <= i; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += q[(size_t)i * d + c] * k[(size_t)j * d + c];
            acc *= scale;
            s[j - lo] = acc;
            if (acc > m) m = acc;
        }
        double l = 0.0;
        for (int t = 0; t < cnt; ++t) {
            s[t] = exp(s[t] - m);
            l += s[t];
        }
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = lo; j <= i; ++j) acc += s[j - lo] * v[(size_t)j * d + c];
            out[(size_t)i * d + c] = acc / l;
        }
    }
    free(s);
    return 0;
}

/* Linear head, plain definition: out_i = sum_{j<=i} a_ij v_j / (sum_{j<=i} a_ij + eps),
 * a_ij = phi(q_i) . phi(k_j).  O(N^2 d). */
int gformer_oracle_linear_head_quadratic_f64(const double *q, const double *k, const double *v,
                                             double *out, int N, int d, int phi, double eps)
{
    if (!q || !k || !v || !out || N < 0 || d < 1) return 1;
    size_t nd = (size_t)N * d;
    double *fq = (double *)malloc(sizeof(double) * (nd ? nd : 1));
    double *fk = (double *)malloc(sizeof(double) * (nd ? nd : 1));
    double *a = (double *)malloc(sizeof(double) * (size_t)(N ? N : 1));
    if (!fq || !fk || !a) { free(fq); free(fk); free(a); return 2; }
    for (size_t t = 0; t < nd; ++t) {
        fq[t] = feature_map(q[t], phi);
        fk[t] = feature_map(k[t], phi);
    }
    for (int i = 0; i < N; ++i) {
        double den = 0.0;
        for (int j = 0; j <= i; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += fq[(size_t)i * d + c] * fk[(size_t)j * d + c];
            a[j] = acc;
            den += acc;
        }
        den += eps;
        for (int e = 0; e < d; ++e) {
            double num = 0.0;
            for (int j = 0; j <= i; ++j) num += a[j] * v[(size_t)j * d + e];
            out[(size_t)i * d + e] = num / den;
        }
    }
    free(fq); free(fk); free(a);
    return 0;
}

/* Linear head, Algorithm 1: running A (d x d) and Z (d), token i added before read-out. */
int gformer_oracle_linear_head_recurrent_f64(const double *q, const double *k, const double *v,
                                             double *out, int N, int d, int phi, double eps)
{
    if (!q || !k || !v || !out || N < 0 || d < 1) return 1;
    double *A = (double *)calloc((size_t)d * d, sizeof(double));
    double *Z = (double *)calloc((size_t)d, sizeof(double));
    double *qp = (double *)malloc(sizeof(double) * (size_t)d);
    double *kp = (double *)malloc(sizeof(double) * (size_t)d);
    if (!A || !Z || !qp || !kp) { free(A); free(Z); free(qp); free(kp); return 2; }
    for (int i = 0; i < N; ++i) {
        for (int c = 0; c < d; ++c) {
            qp[c] = feature_map(q[(size_t)i * d + c], phi);
            kp[c] = feature_map(k[(size_t)i * d + c], phi);
        }
        for (int c = 0; c < d; ++c) {
            for (int e = 0; e < d; ++e) A[(size_t)c * d + e] += kp[c] * v[(size_t)i * d + e];
            Z[c] += kp[c];
        }
        double den = 0.0;
        for (int c = 0; c < d; ++c) den += qp[c] * Z[c];
        den += eps;
        for (int e = 0; e < d; ++e) {
            double num = 0.0;
            for (int c = 0; c < d; ++c) num += qp[c] * A[(size_t)c * d + e];
            out[(size_t)i * d + e] = num / den;
        }
    }
    free(A); free(Z); free(qp); free(kp);
    return 0;
}

/* Whole layer (section III-A head split) over dense [B, H, N, d].
 * linear_form selects which of the two linear routines runs on heads >= n_sparse_heads.
 * threads <= 0 lets OpenMP decide.  Returns 0, or the first non-zero head status. */
int gformer_oracle_fwd_f64(const double *q, const double *k, const double *v, double *out,
                           int B, int H, int N, int d, int window, int n_sparse_heads,
                           int phi, double softmax_scale, double eps, int linear_form,
                           int threads)
{
    if (!q || !k || !v || !out) return 1;
    if (B < 0 || H < 0 || N < 0 || d < 1 || window < 1) return 1;
    if (n_sparse_heads < 0 || n_sparse_heads > H) return 1;
    int status = 0;
    long total = (long)B * H;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < total; ++bh) {
        int h = (int)(bh % H);
        size_t off = (size_t)bh * N * d;
        int rc;
        if (h < n_sparse_heads)
            rc = gformer_oracle_windowed_head_f64(q + off, k + off, v + off, out + off, N, d,
                                                  window, softmax_scale);
        else if (linear_form == ORACLE_LINEAR_RECURRENT)
            rc = gformer_oracle_linear_head_recurrent_f64(q + off, k + off, v + off, out + off,
                                                          N, d, phi, eps);
        else
            rc = gformer_oracle_linear_head_quadratic_f64(q + off, k + off, v + off, out + off,
                                                          N, d, phi, eps);
        if (rc != 0) {
#pragma omp critical
            if (status == 0) status = rc;
        }
    }
    return status;
}

/*
 * Bidirectional variant (the encoder / image workloads of section IV, where a token sees both
 * sides).  Section III-B speaks of a fixed-size window "surrounding each token" without saying
 * how w splits; it is read as the w tokens centred on token i,
 *     j in [i - floor(w/2), i + (w - 1 - floor(w/2))],  cut at the ends of the sequence
 * (odd w: symmetric; even w: one more on the left; w = 1: the token itself).
 */
int gformer_oracle_windowed_head_bidir_f64(const double *q, const double *k, const double *v,
                                           double *out, int N, int d, int window, double scale)
{
    if (!q || !k || !v || !out || N < 0 || d < 1 || window < 1) return 1;
    double *s = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    if (!s) return 2;
    const long left = window / 2, right = (long)window - 1 - left;
    for (int i = 0; i < N; ++i) {
        long lo = (long)i - left, hi = (long)i + right;
        if (lo < 0) lo = 0;
        if (hi > N - 1) hi = N - 1;
        double m = -INFINITY;
        for (long j = lo; j <= hi; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += q[(size_t)i * d + c] * k[(size_t)j * d + c];
            acc *= scale;
            s[j - lo] = acc;
            if (acc > m) m = acc;
        }
        double l = 0.0;
        for (long j = lo; j <= hi; ++j) {
            s[j - lo] = exp(s[j - lo] - m);
            l += s[j - lo];
        }
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (long j = lo; j <= hi; ++j) acc += s[j - lo] * v[(size_t)j * d + c];
            out[(size_t)i * d + c] = acc / l;
        }
    }
    free(s);
    return 0;
}

/* Non-causal linear head, plain definition (section II-B without the causal restriction):
 * out_i = sum_j a_ij v_j / (sum_j a_ij + eps) over ALL j, a_ij = phi(q_i) . phi(k_j). */
int gformer_oracle_linear_head_bidir_f64(const double *q, const double *k, const double *v,
                                         double *out, int N, int d, int phi, double eps)
{
    if (!q || !k || !v || !out || N < 0 || d < 1) return 1;
    double *a = (double *)malloc(sizeof(double) * (size_t)(N ? N : 1));
    if (!a) return 2;
    for (int i = 0; i < N; ++i) {
        double den = 0.0;
        for (int j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c)
                acc += feature_map(q[(size_t)i * d + c], phi) * feature_map(k[(size_t)j * d + c], phi);
            a[j] = acc;
            den += acc;
        }
        den += eps;
        for (int e = 0; e < d; ++e) {
            double num = 0.0;
            for (int j = 0; j < N; ++j) num += a[j] * v[(size_t)j * d + e];
            out[(size_t)i * d + e] = num / den;
        }
    }
    free(a);
    return 0;
}

/* The same head in the order section II-B recommends: S = phi(K)^T V and z = phi(K)^T 1 first,
 * then out_i = phi(q_i)^T S / (phi(q_i) . z + eps).  Written separately; tested against the sum. */
int gformer_oracle_linear_head_bidir_state_f64(const double *q, const double *k, const double *v,
                                               double *out, int N, int d, int phi, double eps)
{
    if (!q || !k || !v || !out || N < 0 || d < 1) return 1;
    double *S = (double *)calloc((size_t)d * d, sizeof(double));
    double *z = (double *)calloc((size_t)d, sizeof(double));
    if (!S || !z) { free(S); free(z); return 2; }
    for (int j = 0; j < N; ++j)
        for (int c = 0; c < d; ++c) {
            const double f = feature_map(k[(size_t)j * d + c], phi);
            z[c] += f;
            for (int e = 0; e < d; ++e) S[(size_t)c * d + e] += f * v[(size_t)j * d + e];
        }
    for (int i = 0; i < N; ++i) {
        double den = eps;
        for (int c = 0; c < d; ++c) den += feature_map(q[(size_t)i * d + c], phi) * z[c];
        for (int e = 0; e < d; ++e) {
            double num = 0.0;
            for (int c = 0; c < d; ++c) num += feature_map(q[(size_t)i * d + c], phi) * S[(size_t)c * d + e];
            out[(size_t)i * d + e] = num / den;
        }
    }
    free(S); free(z);
    return 0;
}

/* Whole bidirectional layer: same head split as gformer_oracle_fwd_f64.
 * linear_form: 0 = explicit sum over all keys, 1 = state first. */
int gformer_oracle_fwd_bidir_f64(const double *q, const double *k, const double *v, double *out,
                                 int B, int H, int N, int d, int window, int n_sparse_heads,
                                 int phi, double softmax_scale, double eps, int linear_form,
                                 int threads)
{
    if (!q || !k || !v || !out) return 1;
    if (B < 0 || H < 0 || N < 0 || d < 1 || window < 1) return 1;
    if (n_sparse_heads < 0 || n_sparse_heads > H) return 1;
    int status = 0;
    long total = (long)B * H;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#else
    (void)threads;
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (long bh = 0; bh < total; ++bh) {
        int h = (int)(bh % H);
        size_t off = (size_t)bh * N * d;
        int rc;
        if (h < n_sparse_heads)
            rc = gformer_oracle_windowed_head_bidir_f64(q + off, k + off, v + off, out + off, N, d,
                                                        window, softmax_scale);
        else if (linear_form == 1)
            rc = gformer_oracle_linear_head_bidir_state_f64(q + off, k + off, v + off, out + off,
                                                            N, d, phi, eps);
        else
            rc = gformer_oracle_linear_head_bidir_f64(q + off, k + off, v + off, out + off, N, d,
                                                      phi, eps);
        if (rc != 0) {
#pragma omp critical
            if (status == 0) status = rc;
        }
    }
    return status;
}

/*
 * Decode step (the inference setting the paper targets, one token at a time): what the causal
 * layer computes for token t alone, from what it keeps between steps.
 *   windowed head: the keys and values of the last `window` tokens in a ring (slot t % window);
 *     row t of section III-B's head is the softmax over the min(t+1, window) rows in the ring.
 *   linear head: Algorithm 1's loop body, once: A += phi(k_t) (x) v_t, Z += phi(k_t), then
 *     H_t = phi(q_t)^T A / (phi(q_t).Z + eps).
 * q, k, v, out: [d].  kring, vring: [window, d], read and written.  A: [d, d], Z: [d], read and
 * written.  Decoding t = 0, 1, ... from empty rings / zero state reproduces the full forward.
 */
int gformer_oracle_decode_windowed_f64(const double *q, const double *k, const double *v,
                                       double *out, double *kring, double *vring, int d,
                                       int window, long t, double scale)
{
    if (!q || !k || !v || !out || !kring || !vring || d < 1 || window < 1 || t < 0) return 1;
    const long slot = t % window;
    memcpy(kring + (size_t)slot * d, k, sizeof(double) * (size_t)d);
    memcpy(vring + (size_t)slot * d, v, sizeof(double) * (size_t)d);
    const long cnt = t + 1 < window ? t + 1 : window;
    double *s = (double *)malloc(sizeof(double) * (size_t)cnt);
    if (!s) return 2;
    double m = -INFINITY;
    for (long r = 0; r < cnt; ++r) {   /* while t < window the ring is filled from slot 0 up */
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += q[c] * kring[(size_t)r * d + c];
        s[r] = acc * scale;
        if (s[r] > m) m = s[r];
    }
    double l = 0.0;
    for (long r = 0; r < cnt; ++r) { s[r] = exp(s[r] - m); l += s[r]; }
    for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (long r = 0; r < cnt; ++r) acc += s[r] * vring[(size_t)r * d + c];
        out[c] = acc / l;
    }
    free(s);
    return 0;
}

int gformer_oracle_decode_linear_f64(const double *q, const double *k, const double *v,
                                     double *out, double *A, double *Z, int d, int phi, double eps)
{
    if (!q || !k || !v || !out || !A || !Z || d < 1) return 1;
    for (int c = 0; c < d; ++c) {
        const double f = feature_map(k[c], phi);
        Z[c] += f;
        for (int e = 0; e < d; ++e) A[(size_t)c * d + e] += f * v[e];
    }
    double den = eps;
    for (int c = 0; c < d; ++c) den += feature_map(q[c], phi) * Z[c];
    for (int e = 0; e < d; ++e) {
        double num = 0.0;
        for (int c = 0; c < d; ++c) num += feature_map(q[c], phi) * A[(size_t)c * d + e];
        out[e] = num / den;
    }
    return 0;
}

/*
 * Positive random features (section III-A names them for the linear heads, Algorithm 1 calls
 * them "random feature maps"; neither prints a formula, so this is the construction of the work
 * they cite): for a projection matrix W of m rows w_i,
 *     phi(x)_i = exp(w_i . x - |x|^2 / 2) / sqrt(m),   i = 0..m-1,
 * every entry positive, and over Gaussian rows E[phi(q) . phi(k)] = exp(q . k).
 * x: [rows, d], w: [m, d], out: [rows, m], all row-major doubles.
 */
int gformer_oracle_random_features_f64(const double *x, const double *w, double *out, long rows,
                                       int d, int m)
{
    if (!x || !w || !out || rows < 0 || d < 1 || m < 1) return 1;
    const double inv_sqrt_m = 1.0 / sqrt((double)m);
    for (long r = 0; r < rows; ++r) {
        const double *xr = x + (size_t)r * d;
        double half_sq = 0.0;
        for (int c = 0; c < d; ++c) half_sq += xr[c] * xr[c];
        half_sq *= 0.5;
        for (int i = 0; i < m; ++i) {
            const double *wi = w + (size_t)i * d;
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += wi[c] * xr[c];
            out[(size_t)r * m + i] = exp(dot - half_sq) * inv_sqrt_m;
        }
    }
    return 0;
}

/* ---- backward pass ------------------------------------------------------------------------
 * Given dO (the gradient of a scalar loss with respect to the head's output), the gradients with
 * respect to Q, K and V.  dq, dk, dv are overwritten. */

/* Windowed head, causal window (section III-B, Eq. 1).  With s_ij = scale q_i.k_j and
 * p_ij = softmax_j(s_ij) over the window, o_i = sum_j p_ij v_j:
 *   dv_j += p_ij dO_i
 *   dp_ij = dO_i . v_j
 *   ds_ij = p_ij (dp_ij - sum_j' p_ij' dp_ij')          (softmax Jacobian)
 *   dq_i += scale ds_ij k_j ;  dk_j += scale ds_ij q_i */
int gformer_oracle_windowed_head_bwd_f64(const double *q, const double *k, const double *v,
                                         const double *dout, double *dq, double *dk, double *dv,
                                         int N, int d, int window, double scale)
{
    if (N < 0 || d < 1 || window < 1) return 1;
    memset(dq, 0, sizeof(double) * (size_t)N * d);
    memset(dk, 0, sizeof(double) * (size_t)N * d);
    memset(dv, 0, sizeof(double) * (size_t)N * d);
    double *p = (double *)malloc(sizeof(double) * (size_t)(window > 0 ? window : 1));
    double *dp = (double *)malloc(sizeof(double) * (size_t)(window > 0 ? window : 1));
    if (!p || !dp) { free(p); free(dp); return 2; }
    for (int i = 0; i < N; ++i) {
        const int lo = i - window + 1 > 0 ? i - window + 1 : 0;
        const int cnt = i - lo + 1;
        double m = -INFINITY;
        for (int t = 0; t < cnt; ++t) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += q[(size_t)i * d + c] * k[(size_t)(lo + t) * d + c];
            p[t] = s * scale;
            if (p[t] > m) m = p[t];
        }
        double l = 0.0;
        for (int t = 0; t < cnt; ++t) { p[t] = exp(p[t] - m); l += p[t]; }
        double mean_dp = 0.0;
        for (int t = 0; t < cnt; ++t) {
            p[t] /= l;
            double x = 0.0;
            for (int c = 0; c < d; ++c) x += dout[(size_t)i * d + c] * v[(size_t)(lo + t) * d + c];
            dp[t] = x;
            mean_dp += p[t] * x;
        }
        for (int t = 0; t < cnt; ++t) {
            const int j = lo + t;
            const double ds = p[t] * (dp[t] - mean_dp);
            for (int c = 0; c < d; ++c) {
                dv[(size_t)j * d + c] += p[t] * dout[(size_t)i * d + c];
                dq[(size_t)i * d + c] += scale * ds * k[(size_t)j * d + c];
                dk[(size_t)j * d + c] += scale * ds * q[(size_t)i * d + c];
            }
        }
    }
    free(p); free(dp);
    return 0;
}

static double feature_map_slope(double x, int phi)
{
    if (phi != 0) return 1.0;          /* identity */
    return x > 0.0 ? 1.0 : exp(x);     /* d/dx (elu(x) + 1) */
}

/* Linear head, causal (section II-B's ratio, Algorithm 1's sums).  With a_ij = phi(q_i).phi(k_j)
 * for j <= i, den_i = sum_j a_ij + eps and o_i = sum_j a_ij v_j / den_i:
 *   dv_j      += a_ij dO_i / den_i
 *   da_ij      = (dO_i . v_j - dO_i . o_i) / den_i
 *   dphi(q_i) += da_ij phi(k_j) ;  dphi(k_j) += da_ij phi(q_i)
 *   dq = dphi(q) * phi'(q) ;  dk = dphi(k) * phi'(k)   (elementwise) */
int gformer_oracle_linear_head_bwd_f64(const double *q, const double *k, const double *v,
                                       const double *dout, double *dq, double *dk, double *dv,
                                       int N, int d, int phi, double eps)
{
    if (N < 0 || d < 1) return 1;
    const size_t nd = (size_t)N * d;
    double *fq = (double *)malloc(sizeof(double) * (nd ? nd : 1));
    double *fk = (double *)malloc(sizeof(double) * (nd ? nd : 1));
    double *a = (double *)malloc(sizeof(double) * (size_t)(N ? N : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    if (!fq || !fk || !a || !o) { free(fq); free(fk); free(a); free(o); return 2; }
    for (size_t x = 0; x < nd; ++x) { fq[x] = feature_map(q[x], phi); fk[x] = feature_map(k[x], phi); }
    memset(dq, 0, sizeof(double) * nd);
    memset(dk, 0, sizeof(double) * nd);
    memset(dv, 0, sizeof(double) * nd);
    for (int i = 0; i < N; ++i) {
        double den = eps;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j <= i; ++j) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += fq[(size_t)i * d + c] * fk[(size_t)j * d + c];
            a[j] = s;
            den += s;
            for (int c = 0; c < d; ++c) o[c] += s * v[(size_t)j * d + c];
        }
        double do_o = 0.0;
        for (int c = 0; c < d; ++c) { o[c] /= den; do_o += dout[(size_t)i * d + c] * o[c]; }
        for (int j = 0; j <= i; ++j) {
            double do_v = 0.0;
            for (int c = 0; c < d; ++c) do_v += dout[(size_t)i * d + c] * v[(size_t)j * d + c];
            const double da = (do_v - do_o) / den;
            for (int c = 0; c < d; ++c) {
                dv[(size_t)j * d + c] += a[j] * dout[(size_t)i * d + c] / den;
                dq[(size_t)i * d + c] += da * fk[(size_t)j * d + c];   /* still d/dphi(q) */
                dk[(size_t)j * d + c] += da * fq[(size_t)i * d + c];   /* still d/dphi(k) */
            }
        }
    }
    for (size_t x = 0; x < nd; ++x) {
        dq[x] *= feature_map_slope(q[x], phi);
        dk[x] *= feature_map_slope(k[x], phi);
    }
    free(fq); free(fk); free(a); free(o);
    return 0;
}

/* The layer: heads [0, H0) windowed, [H0, H) linear, dense [B, H, N, d]. */
int gformer_oracle_bwd_f64(const double *q, const double *k, const double *v, const double *dout,
                           double *dq, double *dk, double *dv, int B, int H, int N, int d,
                           int window, int n_sparse_heads, int phi, double scale, double eps)
{
    if (B < 0 || H < 0 || n_sparse_heads < 0 || n_sparse_heads > H) return 1;
    int rc = 0;
    const long heads = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long x = 0; x < heads; ++x) {
        const int h = (int)(x % H);
        const size_t off = (size_t)x * N * d;
        int r;
        if (h < n_sparse_heads)
            r = gformer_oracle_windowed_head_bwd_f64(q + off, k + off, v + off, dout + off, dq + off,
                                                     dk + off, dv + off, N, d, window, scale);
        else
            r = gformer_oracle_linear_head_bwd_f64(q + off, k + off, v + off, dout + off, dq + off,
                                                   dk + off, dv + off, N, d, phi, eps);
        if (r) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

/* ---- backward pass of the bidirectional variant -------------------------------------------
 * The same derivatives with the other index sets: the windowed head's softmax runs over the w
 * tokens centred on token i (cut at the ends, as in gformer_oracle_windowed_head_bidir_f64), the
 * linear head's sums run over ALL j (section II-B without the causal restriction). */
int gformer_oracle_windowed_head_bidir_bwd_f64(const double *q, const double *k, const double *v,
                                               const double *dout, double *dq, double *dk, double *dv,
                                               int N, int d, int window, double scale)
{
    if (N < 0 || d < 1 || window < 1) return 1;
    memset(dq, 0, sizeof(double) * (size_t)N * d);
    memset(dk, 0, sizeof(double) * (size_t)N * d);
    memset(dv, 0, sizeof(double) * (size_t)N * d);
    double *p = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    double *dp = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    if (!p || !dp) { free(p); free(dp); return 2; }
    const long left = window / 2, right = (long)window - 1 - left;
    for (int i = 0; i < N; ++i) {
        long lo = (long)i - left, hi = (long)i + right;
        if (lo < 0) lo = 0;
        if (hi > N - 1) hi = N - 1;
        const long cnt = hi - lo + 1;
        double m = -INFINITY;
        for (long t = 0; t < cnt; ++t) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += q[(size_t)i * d + c] * k[(size_t)(lo + t) * d + c];
            p[t] = s * scale;
            if (p[t] > m) m = p[t];
        }
        double l = 0.0;
        for (long t = 0; t < cnt; ++t) { p[t] = exp(p[t] - m); l += p[t]; }
        double mean_dp = 0.0;
        for (long t = 0; t < cnt; ++t) {
            p[t] /= l;
            double x = 0.0;
            for (int c = 0; c < d; ++c) x += dout[(size_t)i * d + c] * v[(size_t)(lo + t) * d + c];
            dp[t] = x;
            mean_dp += p[t] * x;
        }
        for (long t = 0; t < cnt; ++t) {
            const long j = lo + t;
            const double ds = p[t] * (dp[t] - mean_dp);
            for (int c = 0; c < d; ++c) {
                dv[(size_t)j * d + c] += p[t] * dout[(size_t)i * d + c];
                dq[(size_t)i * d + c] += scale * ds * k[(size_t)j * d + c];
                dk[(size_t)j * d + c] += scale * ds * q[(size_t)i * d + c];
            }
        }
    }
    free(p); free(dp);
    return 0;
}

/* Non-causal linear head: a_ij = phi(q_i).phi(k_j) for every j, den_i = sum_j a_ij + eps,
 * o_i = sum_j a_ij v_j / den_i; the same three lines as the causal head, summed over all j. */
int gformer_oracle_linear_head_bidir_bwd_f64(const double *q, const double *k, const double *v,
                                             const double *dout, double *dq, double *dk, double *dv,
                                             int N, int d, int phi, double eps)
{
    if (N < 0 || d < 1) return 1;
    const size_t nd = (size_t)N * d;
    double *fq = (double *)malloc(sizeof(double) * (nd ? nd : 1));
    double *fk = (double *)malloc(sizeof(double) * (nd ? nd : 1));
    double *a = (double *)malloc(sizeof(double) * (size_t)(N ? N : 1));
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    if (!fq || !fk || !a || !o) { free(fq); free(fk); free(a); free(o); return 2; }
    for (size_t x = 0; x < nd; ++x) { fq[x] = feature_map(q[x], phi); fk[x] = feature_map(k[x], phi); }
    memset(dq, 0, sizeof(double) * nd);
    memset(dk, 0, sizeof(double) * nd);
    memset(dv, 0, sizeof(double) * nd);
    for (int i = 0; i < N; ++i) {
        double den = eps;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int j = 0; j < N; ++j) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += fq[(size_t)i * d + c] * fk[(size_t)j * d + c];
            a[j] = s;
            den += s;
            for (int c = 0; c < d; ++c) o[c] += s * v[(size_t)j * d + c];
        }
        double do_o = 0.0;
        for (int c = 0; c < d; ++c) { o[c] /= den; do_o += dout[(size_t)i * d + c] * o[c]; }
        for (int j = 0; j < N; ++j) {
            double do_v = 0.0;
            for (int c = 0; c < d; ++c) do_v += dout[(size_t)i * d + c] * v[(size_t)j * d + c];
            const double da = (do_v - do_o) / den;
            for (int c = 0; c < d; ++c) {
                dv[(size_t)j * d + c] += a[j] * dout[(size_t)i * d + c] / den;
                dq[(size_t)i * d + c] += da * fk[(size_t)j * d + c];   /* still d/dphi(q) */
                dk[(size_t)j * d + c] += da * fq[(size_t)i * d + c];   /* still d/dphi(k) */
            }
        }
    }
    for (size_t x = 0; x < nd; ++x) {
        dq[x] *= feature_map_slope(q[x], phi);
        dk[x] *= feature_map_slope(k[x], phi);
    }
    free(fq); free(fk); free(a); free(o);
    return 0;
}

/* The bidirectional layer: heads [0, H0) windowed, [H0, H) linear, dense [B, H, N, d]. */
int gformer_oracle_bwd_bidir_f64(const double *q, const double *k, const double *v, const double *dout,
                                 double *dq, double *dk, double *dv, int B, int H, int N, int d,
                                 int window, int n_sparse_heads, int phi, double scale, double eps)
{
    if (B < 0 || H < 0 || n_sparse_heads < 0 || n_sparse_heads > H) return 1;
    int rc = 0;
    const long heads = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long x = 0; x < heads; ++x) {
        const int h = (int)(x % H);
        const size_t off = (size_t)x * N * d;
        int r;
        if (h < n_sparse_heads)
            r = gformer_oracle_windowed_head_bidir_bwd_f64(q + off, k + off, v + off, dout + off, dq + off,
                                                           dk + off, dv + off, N, d, window, scale);
        else
            r = gformer_oracle_linear_head_bidir_bwd_f64(q + off, k + off, v + off, dout + off, dq + off,
                                                         dk + off, dv + off, N, d, phi, eps);
        if (r) {
#pragma omp critical
            rc = r;
        }
    }
    return rc;
}

int gformer_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
