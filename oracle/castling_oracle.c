/*
 * CPU oracle for the inference-time linear-angular attention layer of
 * Castling-ViT (arXiv 2211.10526).  TEST INFRASTRUCTURE ONLY: this file is the
 * slow, plain reference that the HIP library is checked against.  It shares no
 * code with the HIP path and must never be on the product path.
 *
 * Everything is fp64, row-major, and written in the order the paper states it.
 *
 * Tensor layout (same as the library): q, k, v, out are [B][heads][N][d],
 * token n = y*grid_w + x on a grid_h x grid_w grid; depthwise filters are
 * [heads][d][ks][ks]; bias is [heads][d] or NULL.
 *
 * What each function follows:
 *   oracle_l2_normalize     unit row vectors along the feature axis (Sec. 3.1
 *                           text before Eq. 3; Sec. 3.2.1 after Eq. 8 and Eq. 9)
 *   oracle_sim_angular      Eq. 4 (spectral angle) and Eq. 5 (angular kernel)
 *   oracle_series_coeff     coefficient of the k-th residual term of Eq. 8
 *   oracle_sim_series       partial sum of Eq. 8
 *   oracle_sim_linear       the linear-angular terms of Eq. 8
 *   oracle_dwconv           the DWConv term of Eq. 9 (M_DW * V), direct loops
 *   oracle_forward_explicit the definition: explicit N x N similarity (Eq. 8
 *                           linear terms) times V, row-normalised as in Eq. 3,
 *                           plus DWConv (Eq. 9)
 *   oracle_forward_explicit_rows  same definition, selected output rows only
 *   oracle_state            reassociated K^T V state (Sec. 3.1, kernel-based
 *                           linear attention; Eq. 3 sums)
 *   oracle_forward          fast path: Eq. 3 with phi(x) = [x/|x| / sqrt(pi);
 *                           1/sqrt(2)] so that phi(q).phi(k) = 1/2 + q.k/pi
 *   oracle_backward_explicit, oracle_backward, oracle_backward_explicit_rows
 *                           gradients of the layer (the paper prints none: the chain rule on
 *                           the definition above), by the N x N definition, through the
 *                           reassociated state, and by the definition on selected rows
 *   oracle_softmax_probs    the softmax attention map inside Eq. 10
 *   oracle_sparse_attn      Eq. 10 (masked softmax attention) applied to V
 *   oracle_angular_attn     attention with the exact angular kernel, Eq. 4-5
 *
 * Readings taken where the paper is silent (also listed in the design notes):
 *   - the 1/2 term multiplies the column sum of V (Eq. 8 gives Sim_ij = 1/2 +
 *     ..., so Sim*V has 1/2 * sum_j V_j in every row);
 *   - norm_mode 0 divides by the row sum of the similarity (Eq. 3's
 *     denominator); norm_mode 1 is the literal Eq. 9 with no denominator;
 *   - DWConv: zero "same" padding, stride 1, cross-correlation (no flip),
 *     added outside the division;
 *   - x / max(|x|, eps);
 *   - tokens that are not on the grid (`extra` class tokens in front of the H*W
 *     grid tokens of a unit): they are keys and queries of the attention sums
 *     like any other token, and the DWConv term, defined on the grid (Sec.
 *     3.2.1), is zero for them and does not read them.
 *
 * Pins (tests/test_oracle_pins.py): closed forms for tiny cases, arccos /
 * arcsin identities, textbook arcsin series coefficients, row-stochastic
 * invariants, invariances, torch's grouped conv2d for the DWConv, explicit vs
 * reassociated agreement.  The whole layer has no closed form: it is pinned by
 * the sum of those (explicit form on tiny inputs + per-branch pins).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_BRANCH_LINEAR 1u
#define ORACLE_BRANCH_DWCONV 2u

static const double ORACLE_PI = 3.14159265358979323846264338327950288;

/* x_hat = x / max(||x||_2, eps), row by row. */
void oracle_l2_normalize(const double* x, int64_t rows, int d, double eps, double* out)
{
    for (int64_t r = 0; r < rows; ++r) {
        double ss = 0.0;
        for (int c = 0; c < d; ++c) ss += x[r * d + c] * x[r * d + c];
        double nrm = sqrt(ss);
        if (nrm < eps) nrm = eps;
        for (int c = 0; c < d; ++c) out[r * d + c] = x[r * d + c] / nrm;
    }
}

/* Eq. 4 + Eq. 5: A[t][j] = 1 - arccos(<q_t,k_j>/(|q_t||k_j|)) / pi, one head. */
void oracle_sim_angular(const double* q, const double* k, int N, int d, double eps, double* A)
{
    double* qh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    oracle_l2_normalize(q, N, d, eps, qh);
    oracle_l2_normalize(k, N, d, eps, kh);
    for (int t = 0; t < N; ++t)
        for (int j = 0; j < N; ++j) {
            double x = 0.0;
            for (int c = 0; c < d; ++c) x += qh[t * d + c] * kh[j * d + c];
            if (x > 1.0) x = 1.0;
            if (x < -1.0) x = -1.0;
            A[(size_t)t * N + j] = 1.0 - acos(x) / ORACLE_PI;
        }
    free(qh);
    free(kh);
}

/* Eq. 8 residual coefficient: (2k)! / (2^{2k} (k!)^2 (2k+1)), k >= 1. */
double oracle_series_coeff(int k)
{
    /* (2k)!/(k!)^2 = C(2k,k), built as a running product to stay in range */
    double binom = 1.0;
    for (int i = 1; i <= k; ++i) binom *= (double)(k + i) / (double)i;
    return binom / (pow(4.0, (double)k) * (2.0 * k + 1.0));
}

/* Eq. 8 truncated after `order` residual terms (order = 0: linear terms only). */
double oracle_sim_series(double x, int order)
{
    double s = 0.5 + x / ORACLE_PI;
    for (int k = 1; k <= order; ++k)
        s += oracle_series_coeff(k) * pow(x, 2.0 * k + 1.0) / ORACLE_PI;
    return s;
}

/* Linear-angular terms of Eq. 8: A[t][j] = 1/2 + (q_hat_t . k_hat_j) / pi, one head. */
void oracle_sim_linear(const double* q, const double* k, int N, int d, double eps, double* A)
{
    double* qh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    oracle_l2_normalize(q, N, d, eps, qh);
    oracle_l2_normalize(k, N, d, eps, kh);
    for (int t = 0; t < N; ++t)
        for (int j = 0; j < N; ++j) {
            double x = 0.0;
            for (int c = 0; c < d; ++c) x += qh[t * d + c] * kh[j * d + c];
            A[(size_t)t * N + j] = 0.5 + x / ORACLE_PI;
        }
    free(qh);
    free(kh);
}

/* One output value of the DWConv term of Eq. 9 at (b, h, y, x, c).  A unit holds `extra`
 * tokens that are not on the grid (class tokens) before its H*W grid tokens. */
static double dwconv_at(const double* v, const double* w, const double* bias,
                        int heads, int H, int W, int d, int ks, int extra,
                        int b, int h, int y, int x, int c)
{
    const int r = ks / 2;
    double acc = bias ? bias[h * d + c] : 0.0;
    for (int dy = 0; dy < ks; ++dy)
        for (int dx = 0; dx < ks; ++dx) {
            int yy = y + dy - r, xx = x + dx - r;
            if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
            size_t tok = (size_t)yy * W + xx;
            double val = v[(((size_t)b * heads + h) * ((size_t)extra + (size_t)H * W) + extra + tok) * d + c];
            acc += w[(((size_t)h * d + c) * ks + dy) * ks + dx] * val;
        }
    return acc;
}

/* DWConv on the value tokens over the token grid, direct loops. */
void oracle_dwconv(const double* v, const double* w, const double* bias,
                   int B, int heads, int H, int W, int d, int ks, double* out)
{
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h)
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x)
                    for (int c = 0; c < d; ++c) {
                        size_t tok = (size_t)y * W + x;
                        out[(((size_t)b * heads + h) * ((size_t)H * W) + tok) * d + c] =
                            dwconv_at(v, w, bias, heads, H, W, d, ks, 0, b, h, y, x, c);
                    }
}

/* Linear branch of one output row by the definition: sum_j A_tj v_j [/ sum_j A_tj]. */
static void explicit_row(const double* qrow, const double* kh, const double* vu,
                         int N, int d, int norm_mode, double eps, double* lin)
{
    double ss = 0.0;
    for (int c = 0; c < d; ++c) ss += qrow[c] * qrow[c];
    double nrm = sqrt(ss);
    if (nrm < eps) nrm = eps;
    double rowsum = 0.0;
    for (int c = 0; c < d; ++c) lin[c] = 0.0;
    for (int j = 0; j < N; ++j) {
        double x = 0.0;
        for (int c = 0; c < d; ++c) x += (qrow[c] / nrm) * kh[(size_t)j * d + c];
        double a = 0.5 + x / ORACLE_PI;
        rowsum += a;
        for (int c = 0; c < d; ++c) lin[c] += a * vu[(size_t)j * d + c];
    }
    if (norm_mode == 0)
        for (int c = 0; c < d; ++c) lin[c] /= rowsum;
}

/* The definition of the layer, all rows.  O(N^2 d) per head: small inputs only. */
void oracle_forward_explicit(const double* q, const double* k, const double* v,
                             const double* w, const double* bias,
                             int B, int heads, int H, int W, int d, int ks,
                             int norm_mode, unsigned branches, double eps, int extra, double* out)
{
    const int N = extra + H * W;
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* lin = (double*)malloc(sizeof(double) * d);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h) {
            size_t base = ((size_t)b * heads + h) * (size_t)N * d;
            oracle_l2_normalize(k + base, N, d, eps, kh);
            for (int t = 0; t < N; ++t) {
                for (int c = 0; c < d; ++c) lin[c] = 0.0;
                if (branches & ORACLE_BRANCH_LINEAR)
                    explicit_row(q + base + (size_t)t * d, kh, v + base, N, d, norm_mode, eps, lin);
                for (int c = 0; c < d; ++c) {
                    double dw = 0.0;
                    if ((branches & ORACLE_BRANCH_DWCONV) && t >= extra)
                        dw = dwconv_at(v, w, bias, heads, H, W, d, ks, extra, b, h, (t - extra) / W,
                                       (t - extra) % W, c);
                    out[base + (size_t)t * d + c] = lin[c] + dw;
                }
            }
        }
    free(kh);
    free(lin);
}

/* The definition on selected rows: row i is token tokens[i] of unit units[i]
 * (unit = b*heads + h); out is [nrows][d].  O(N d) per row, any N. */
void oracle_forward_explicit_rows(const double* q, const double* k, const double* v,
                                  const double* w, const double* bias,
                                  int B, int heads, int H, int W, int d, int ks,
                                  int norm_mode, unsigned branches, double eps, int extra,
                                  const int64_t* units, const int64_t* tokens, int64_t nrows,
                                  double* out)
{
    const int N = extra + H * W;
    (void)B;
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* lin = (double*)malloc(sizeof(double) * d);
    int64_t cached_unit = -1;
    for (int64_t i = 0; i < nrows; ++i) {
        int64_t u = units[i];
        int t = (int)tokens[i];
        int b = (int)(u / heads), h = (int)(u % heads);
        size_t base = (size_t)u * (size_t)N * d;
        if (u != cached_unit) {
            oracle_l2_normalize(k + base, N, d, eps, kh);
            cached_unit = u;
        }
        for (int c = 0; c < d; ++c) lin[c] = 0.0;
        if (branches & ORACLE_BRANCH_LINEAR)
            explicit_row(q + base + (size_t)t * d, kh, v + base, N, d, norm_mode, eps, lin);
        for (int c = 0; c < d; ++c) {
            double dw = 0.0;
            if ((branches & ORACLE_BRANCH_DWCONV) && t >= extra)
                dw = dwconv_at(v, w, bias, heads, H, W, d, ks, extra, b, h, (t - extra) / W,
                               (t - extra) % W, c);
            out[(size_t)i * d + c] = lin[c] + dw;
        }
    }
    free(kh);
    free(lin);
}

/* Reassociated state per unit, (d+1) x (d+1) row-major = [K_hat | 1]^T [V | 1]:
 *   M[i][j] = sum_n k_hat[n][i] v[n][j]   (i, j < d)    K_hat^T V
 *   M[i][d] = sum_n k_hat[n][i]                          K_hat column sum
 *   M[d][j] = sum_n v[n][j]                              V column sum
 *   M[d][d] = N                                                          */
void oracle_state(const double* k, const double* v, int B, int heads, int N, int d,
                  double eps, double* state)
{
    const int d1 = d + 1;
    const int64_t units = (int64_t)B * heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
        const double* vu = v + (size_t)u * N * d;
        double* M = state + (size_t)u * d1 * d1;
        oracle_l2_normalize(k + (size_t)u * N * d, N, d, eps, kh);
        memset(M, 0, sizeof(double) * d1 * d1);
        for (int n = 0; n < N; ++n) {
            for (int i = 0; i < d; ++i) {
                double ki = kh[(size_t)n * d + i];
                for (int j = 0; j < d; ++j) M[i * d1 + j] += ki * vu[(size_t)n * d + j];
                M[i * d1 + d] += ki;
            }
            for (int j = 0; j < d; ++j) M[d * d1 + j] += vu[(size_t)n * d + j];
            M[d * d1 + d] += 1.0;
        }
        free(kh);
    }
}

/* Fast path: Eq. 3 with the reassociated state; equals oracle_forward_explicit
 * up to fp64 rounding order. */
void oracle_forward(const double* q, const double* k, const double* v,
                    const double* w, const double* bias,
                    int B, int heads, int H, int W, int d, int ks,
                    int norm_mode, unsigned branches, double eps, int extra, double* out)
{
    const int N = extra + H * W;
    const int d1 = d + 1;
    const int64_t units = (int64_t)B * heads;
    double* state = (double*)malloc(sizeof(double) * (size_t)units * d1 * d1);
    if (branches & ORACLE_BRANCH_LINEAR) oracle_state(k, v, B, heads, N, d, eps, state);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        const int b = (int)(u / heads), h = (int)(u % heads);
        const size_t base = (size_t)u * N * d;
        const double* M = state + (size_t)u * d1 * d1;
        double* qh = (double*)malloc(sizeof(double) * d);
        for (int t = 0; t < N; ++t) {
            double* o = out + base + (size_t)t * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            if (branches & ORACLE_BRANCH_LINEAR) {
                oracle_l2_normalize(q + base + (size_t)t * d, 1, d, eps, qh);
                /* den = phi(q) . sum_j phi(k_j) = N/2 + q_hat . ksum / pi */
                double den = 0.5 * M[d * d1 + d];
                for (int i = 0; i < d; ++i) den += qh[i] * M[i * d1 + d] / ORACLE_PI;
                for (int j = 0; j < d; ++j) {
                    /* num = phi(q) . sum_j phi(k_j)^T v_j = vsum/2 + q_hat . S / pi */
                    double num = 0.5 * M[d * d1 + j];
                    for (int i = 0; i < d; ++i) num += qh[i] * M[i * d1 + j] / ORACLE_PI;
                    o[j] = (norm_mode == 0) ? num / den : num;
                }
            }
            if ((branches & ORACLE_BRANCH_DWCONV) && t >= extra)
                for (int c = 0; c < d; ++c)
                    o[c] += dwconv_at(v, w, bias, heads, H, W, d, ks, extra, b, h, (t - extra) / W,
                                      (t - extra) % W, c);
        }
        free(qh);
    }
    free(state);
}

/* ------------------------------------------------------------------------
 * Downsampling attention layers (Sec. 3.1, attention designs; Table 1, last row): the queries
 * are pooled after their projection, K and V keep every token, and the pooled query is added
 * to the result (residual connection).  The pooling operator itself runs before the layer:
 * q holds Nq = ceil(H/s) * ceil(W/s) pooled queries per unit, query (y, x) of that grid
 * standing at position (s*y, s*x) of the H x W token grid.
 *
 * Readings where the paper is silent: the N x N matrix M_DW of Eq. 9 keeps the rows of the
 * positions the queries stand at, i.e. the DWConv is evaluated with stride s; the residual adds
 * the pooled query as given (not its unit row), after the normaliser.
 * ---------------------------------------------------------------------- */

/* The definition, all rows: q, out [B][heads][Nq][d]; k, v [B][heads][H*W][d]. */
void oracle_forward_pooled_explicit(const double* q, const double* k, const double* v,
                                    const double* w, const double* bias,
                                    int B, int heads, int H, int W, int d, int ks, int s,
                                    int residual, int norm_mode, unsigned branches, double eps,
                                    double* out)
{
    const int N = H * W;
    const int Hq = (H + s - 1) / s, Wq = (W + s - 1) / s, Nq = Hq * Wq;
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* lin = (double*)malloc(sizeof(double) * d);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h) {
            const size_t kv = ((size_t)b * heads + h) * (size_t)N * d;
            const size_t qo = ((size_t)b * heads + h) * (size_t)Nq * d;
            oracle_l2_normalize(k + kv, N, d, eps, kh);
            for (int t = 0; t < Nq; ++t) {
                const double* qrow = q + qo + (size_t)t * d;
                for (int c = 0; c < d; ++c) lin[c] = 0.0;
                if (branches & ORACLE_BRANCH_LINEAR)
                    explicit_row(qrow, kh, v + kv, N, d, norm_mode, eps, lin);
                for (int c = 0; c < d; ++c) {
                    double val = lin[c];
                    if (branches & ORACLE_BRANCH_DWCONV)
                        val += dwconv_at(v, w, bias, heads, H, W, d, ks, 0, b, h, s * (t / Wq),
                                         s * (t % Wq), c);
                    if (residual) val += qrow[c];
                    out[qo + (size_t)t * d + c] = val;
                }
            }
        }
    free(kh);
    free(lin);
}

/* The same with the reassociated state (any N). */
void oracle_forward_pooled(const double* q, const double* k, const double* v,
                           const double* w, const double* bias,
                           int B, int heads, int H, int W, int d, int ks, int s,
                           int residual, int norm_mode, unsigned branches, double eps, double* out)
{
    const int N = H * W;
    const int Hq = (H + s - 1) / s, Wq = (W + s - 1) / s, Nq = Hq * Wq;
    const int d1 = d + 1;
    const int64_t units = (int64_t)B * heads;
    double* state = (double*)malloc(sizeof(double) * (size_t)units * d1 * d1);
    if (branches & ORACLE_BRANCH_LINEAR) oracle_state(k, v, B, heads, N, d, eps, state);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        const int b = (int)(u / heads), h = (int)(u % heads);
        const double* M = state + (size_t)u * d1 * d1;
        double* qh = (double*)malloc(sizeof(double) * d);
        for (int t = 0; t < Nq; ++t) {
            const double* qrow = q + ((size_t)u * Nq + t) * d;
            double* o = out + ((size_t)u * Nq + t) * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            if (branches & ORACLE_BRANCH_LINEAR) {
                oracle_l2_normalize(qrow, 1, d, eps, qh);
                double den = 0.5 * M[d * d1 + d];
                for (int i = 0; i < d; ++i) den += qh[i] * M[i * d1 + d] / ORACLE_PI;
                for (int j = 0; j < d; ++j) {
                    double num = 0.5 * M[d * d1 + j];
                    for (int i = 0; i < d; ++i) num += qh[i] * M[i * d1 + j] / ORACLE_PI;
                    o[j] = (norm_mode == 0) ? num / den : num;
                }
            }
            for (int c = 0; c < d; ++c) {
                if (branches & ORACLE_BRANCH_DWCONV)
                    o[c] += dwconv_at(v, w, bias, heads, H, W, d, ks, 0, b, h, s * (t / Wq),
                                      s * (t % Wq), c);
                if (residual) o[c] += qrow[c];
            }
        }
        free(qh);
    }
    free(state);
}

/* ------------------------------------------------------------------------
 * Backward pass of the layer: the gradients of a scalar loss with respect to q, k, v, the
 * DWConv filters and their bias, given g = dLoss/dout.  The paper trains the layer (Sec. 4.1)
 * and prints no gradient formulas: these are the derivatives of the forward definition
 * above (Eq. 3, 8, 9 with the same readings), by the chain rule.
 *
 *   x_hat = x / max(|x|, eps)  =>  dx = (dx_hat - x_hat (x_hat . dx_hat)) / |x|   if |x| >= eps,
 *                                  dx = dx_hat / eps                             otherwise
 *   A_tj = 1/2 + q_hat_t . k_hat_j / pi,  r_t = sum_j A_tj,  lin_t = sum_j A_tj v_j [/ r_t]
 *   dLoss/dA_tj = (g_t . v_j - g_t . lin_t) / r_t   (normalised)    or   g_t . v_j   (not)
 *
 * dw [heads][d][ks][ks] and dbias [heads][d] (may be NULL) are sums over the batch.
 * residual != 0: the forward added q_t to out_t, so dq_t gains g_t.
 * ---------------------------------------------------------------------- */

/* J^T applied to a gradient with respect to the unit row of x. */
static void normalize_backward(const double* x, const double* dxh, int d, double eps, double* dx)
{
    double ss = 0.0;
    for (int c = 0; c < d; ++c) ss += x[c] * x[c];
    const double nrm = sqrt(ss);
    if (nrm < eps) {
        for (int c = 0; c < d; ++c) dx[c] = dxh[c] / eps;
        return;
    }
    double dot = 0.0;
    for (int c = 0; c < d; ++c) dot += (x[c] / nrm) * dxh[c];
    for (int c = 0; c < d; ++c) dx[c] = (dxh[c] - (x[c] / nrm) * dot) / nrm;
}

/* The DWConv term's share: dv, dw, dbias gain their sums over the grid tokens of every unit. */
static void dwconv_backward(const double* v, const double* w, const double* g,
                            int B, int heads, int H, int W, int d, int ks, int extra,
                            double* dv, double* dw, double* dbias)
{
    const int r = ks / 2;
    const size_t N = (size_t)extra + (size_t)H * W;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h) {
            const size_t base = ((size_t)b * heads + h) * N * d;
            for (int y = 0; y < H; ++y)
                for (int x = 0; x < W; ++x) {
                    const double* gt = g + base + ((size_t)extra + (size_t)y * W + x) * d;
                    for (int c = 0; c < d; ++c) {
                        if (dbias) dbias[h * d + c] += gt[c];
                        for (int dy = 0; dy < ks; ++dy)
                            for (int dx = 0; dx < ks; ++dx) {
                                const int yy = y + dy - r, xx = x + dx - r;
                                if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                                const size_t src = base + ((size_t)extra + (size_t)yy * W + xx) * d + c;
                                const size_t wi = (((size_t)h * d + c) * ks + dy) * ks + dx;
                                dv[src] += w[wi] * gt[c];
                                dw[wi] += gt[c] * v[src];
                            }
                    }
                }
        }
}

/* By the definition: explicit N x N similarity, O(N^2 d) per head. */
void oracle_backward_explicit(const double* q, const double* k, const double* v, const double* w,
                              const double* g, int B, int heads, int H, int W, int d, int ks,
                              int norm_mode, unsigned branches, double eps, int extra, int residual,
                              double* dq, double* dk, double* dv, double* dw, double* dbias)
{
    const int N = extra + H * W;
    const size_t total = (size_t)B * heads * N * d;
    memset(dq, 0, sizeof(double) * total);
    memset(dk, 0, sizeof(double) * total);
    memset(dv, 0, sizeof(double) * total);
    memset(dw, 0, sizeof(double) * (size_t)heads * d * ks * ks);
    if (dbias) memset(dbias, 0, sizeof(double) * (size_t)heads * d);
    double* qh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* dkh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* A = (double*)malloc(sizeof(double) * N);
    double* lin = (double*)malloc(sizeof(double) * d);
    double* dqh = (double*)malloc(sizeof(double) * d);
    for (int64_t u = 0; u < (int64_t)B * heads; ++u) {
        const size_t base = (size_t)u * N * d;
        if (!(branches & ORACLE_BRANCH_LINEAR)) break;
        oracle_l2_normalize(q + base, N, d, eps, qh);
        oracle_l2_normalize(k + base, N, d, eps, kh);
        memset(dkh, 0, sizeof(double) * (size_t)N * d);
        for (int t = 0; t < N; ++t) {
            const double* gt = g + base + (size_t)t * d;
            double r = 0.0;
            for (int c = 0; c < d; ++c) lin[c] = 0.0;
            for (int j = 0; j < N; ++j) {
                double x = 0.0;
                for (int c = 0; c < d; ++c) x += qh[(size_t)t * d + c] * kh[(size_t)j * d + c];
                A[j] = 0.5 + x / ORACLE_PI;
                r += A[j];
                for (int c = 0; c < d; ++c) lin[c] += A[j] * v[base + (size_t)j * d + c];
            }
            const double scale = (norm_mode == 0) ? 1.0 / r : 1.0;
            double g_lin = 0.0;  /* g_t . lin_t of the normalised form */
            for (int c = 0; c < d; ++c) g_lin += gt[c] * lin[c] * scale;
            for (int c = 0; c < d; ++c) dqh[c] = 0.0;
            for (int j = 0; j < N; ++j) {
                double g_v = 0.0;
                for (int c = 0; c < d; ++c) g_v += gt[c] * v[base + (size_t)j * d + c];
                const double dA = (norm_mode == 0) ? (g_v - g_lin) / r : g_v;
                for (int c = 0; c < d; ++c) {
                    dv[base + (size_t)j * d + c] += A[j] * scale * gt[c];
                    dqh[c] += dA * kh[(size_t)j * d + c] / ORACLE_PI;
                    dkh[(size_t)j * d + c] += dA * qh[(size_t)t * d + c] / ORACLE_PI;
                }
            }
            normalize_backward(q + base + (size_t)t * d, dqh, d, eps, dq + base + (size_t)t * d);
        }
        for (int j = 0; j < N; ++j)
            normalize_backward(k + base + (size_t)j * d, dkh + (size_t)j * d, d, eps,
                               dk + base + (size_t)j * d);
    }
    if (branches & ORACLE_BRANCH_DWCONV)
        dwconv_backward(v, w, g, B, heads, H, W, d, ks, extra, dv, dw, dbias);
    if (residual)
        for (size_t i = 0; i < total; ++i) dq[i] += g[i];
    free(qh); free(kh); free(dkh); free(A); free(lin); free(dqh);
}

/* The definition's gradients on selected rows, any N: row i of dq_rows, dk_rows, dv_rows is the
 * gradient with respect to token tokens[i] of unit units[i] (unit = b*heads + h; rows of one
 * unit must be adjacent in the lists).  Per unit every query row's r_t and g_t . lin_t come from
 * the explicit similarities (O(N^2 d)); then dq of a selected token is a sum over all keys, dk
 * and dv of a selected token sums over all queries.  Nothing of the reassociated form (no state,
 * no a_t / b_t split) is used.  The filter and bias gradients are not sampled: the DWConv
 * term's share in oracle_backward is already the definition at any N. */
void oracle_backward_explicit_rows(const double* q, const double* k, const double* v,
                                   const double* w, const double* g, int B, int heads, int H, int W,
                                   int d, int ks, int norm_mode, unsigned branches, double eps,
                                   int extra, int residual, const int64_t* units,
                                   const int64_t* tokens, int64_t nrows,
                                   double* dq_rows, double* dk_rows, double* dv_rows)
{
    const int N = extra + H * W;
    const int rad = ks / 2;
    (void)B;
    double* qh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* rsum = (double*)malloc(sizeof(double) * N);   /* r_t = sum_j A_tj */
    double* glin = (double*)malloc(sizeof(double) * N);   /* g_t . lin_t (normalised form) */
    int64_t cached_unit = -1;
    for (int64_t i = 0; i < nrows; ++i) {
        const int64_t u = units[i];
        const int s = (int)tokens[i];
        const int h = (int)(u % heads);
        const size_t base = (size_t)u * (size_t)N * d;
        double* dq = dq_rows + (size_t)i * d;
        double* dk = dk_rows + (size_t)i * d;
        double* dv = dv_rows + (size_t)i * d;
        for (int c = 0; c < d; ++c) dq[c] = dk[c] = dv[c] = 0.0;
        if (branches & ORACLE_BRANCH_LINEAR) {
            if (u != cached_unit) {
                oracle_l2_normalize(q + base, N, d, eps, qh);
                oracle_l2_normalize(k + base, N, d, eps, kh);
#pragma omp parallel for schedule(static)
                for (int t = 0; t < N; ++t) {
                    double lin[d];  /* per iteration, so per thread */
                    double r = 0.0;
                    for (int c = 0; c < d; ++c) lin[c] = 0.0;
                    for (int j = 0; j < N; ++j) {
                        double x = 0.0;
                        for (int c = 0; c < d; ++c) x += qh[(size_t)t * d + c] * kh[(size_t)j * d + c];
                        const double a = 0.5 + x / ORACLE_PI;
                        r += a;
                        for (int c = 0; c < d; ++c) lin[c] += a * v[base + (size_t)j * d + c];
                    }
                    double gl = 0.0;
                    for (int c = 0; c < d; ++c) gl += g[base + (size_t)t * d + c] * lin[c] / r;
                    rsum[t] = r;
                    glin[t] = gl;
                }
                cached_unit = u;
            }
            /* token s as a query: dLoss/dq_hat_s = sum_j dA_sj k_hat_j / pi */
            {
                double dqh[d];
                const double* gs = g + base + (size_t)s * d;
                for (int c = 0; c < d; ++c) dqh[c] = 0.0;
                for (int j = 0; j < N; ++j) {
                    double g_v = 0.0;
                    for (int c = 0; c < d; ++c) g_v += gs[c] * v[base + (size_t)j * d + c];
                    const double dA = (norm_mode == 0) ? (g_v - glin[s]) / rsum[s] : g_v;
                    for (int c = 0; c < d; ++c) dqh[c] += dA * kh[(size_t)j * d + c] / ORACLE_PI;
                }
                normalize_backward(q + base + (size_t)s * d, dqh, d, eps, dq);
            }
            /* token s as a key: dv_s = sum_t A_ts g_t [/ r_t], dLoss/dk_hat_s = sum_t dA_ts q_hat_t / pi */
            {
                double dkh[d];
                const double* vs = v + base + (size_t)s * d;
                for (int c = 0; c < d; ++c) dkh[c] = 0.0;
                for (int t = 0; t < N; ++t) {
                    const double* gt = g + base + (size_t)t * d;
                    double x = 0.0, g_v = 0.0;
                    for (int c = 0; c < d; ++c) {
                        x += qh[(size_t)t * d + c] * kh[(size_t)s * d + c];
                        g_v += gt[c] * vs[c];
                    }
                    const double a = 0.5 + x / ORACLE_PI;
                    const double scale = (norm_mode == 0) ? 1.0 / rsum[t] : 1.0;
                    const double dA = (norm_mode == 0) ? (g_v - glin[t]) / rsum[t] : g_v;
                    for (int c = 0; c < d; ++c) {
                        dv[c] += a * scale * gt[c];
                        dkh[c] += dA * qh[(size_t)t * d + c] / ORACLE_PI;
                    }
                }
                normalize_backward(k + base + (size_t)s * d, dkh, d, eps, dk);
            }
        }
        /* DWConv term: v_s enters the output rows whose window covers it */
        if ((branches & ORACLE_BRANCH_DWCONV) && s >= extra) {
            const int ys = (s - extra) / W, xs = (s - extra) % W;
            for (int dy = 0; dy < ks; ++dy)
                for (int dx = 0; dx < ks; ++dx) {
                    const int yo = ys - (dy - rad), xo = xs - (dx - rad);
                    if (yo < 0 || yo >= H || xo < 0 || xo >= W) continue;
                    const double* go = g + base + ((size_t)extra + (size_t)yo * W + xo) * d;
                    for (int c = 0; c < d; ++c)
                        dv[c] += w[(((size_t)h * d + c) * ks + dy) * ks + dx] * go[c];
                }
        }
        if (residual)
            for (int c = 0; c < d; ++c) dq[c] += g[base + (size_t)s * d + c];
    }
    free(qh); free(kh); free(rsum); free(glin);
}

/* The same through the reassociated state (any N): with a_t = dLoss/dnum_t and
 * b_t = dLoss/dden_t of Eq. 3's numerator and denominator,
 *   dq_hat_t = (S a_t + ksum b_t) / pi,   S' = sum_t q_hat_t^T a_t,   kb' = sum_t q_hat_t b_t,
 *   dv_j = k_hat_j S' / pi + (sum_t a_t) / 2,   dk_hat_j = (S' v_j + kb') / pi.            */
void oracle_backward(const double* q, const double* k, const double* v, const double* w,
                     const double* g, int B, int heads, int H, int W, int d, int ks,
                     int norm_mode, unsigned branches, double eps, int extra, int residual,
                     double* dq, double* dk, double* dv, double* dw, double* dbias)
{
    const int N = extra + H * W;
    const int d1 = d + 1;
    const int64_t units = (int64_t)B * heads;
    const size_t total = (size_t)units * N * d;
    memset(dq, 0, sizeof(double) * total);
    memset(dk, 0, sizeof(double) * total);
    memset(dv, 0, sizeof(double) * total);
    memset(dw, 0, sizeof(double) * (size_t)heads * d * ks * ks);
    if (dbias) memset(dbias, 0, sizeof(double) * (size_t)heads * d);
    if (branches & ORACLE_BRANCH_LINEAR) {
        double* state = (double*)malloc(sizeof(double) * (size_t)units * d1 * d1);
        oracle_state(k, v, B, heads, N, d, eps, state);
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t u = 0; u < units; ++u) {
            const size_t base = (size_t)u * N * d;
            const double* M = state + (size_t)u * d1 * d1;
            double* S2 = (double*)calloc((size_t)d * d + 2 * (size_t)d, sizeof(double));
            double* kb2 = S2 + (size_t)d * d;
            double* va2 = kb2 + d;
            double* tmp = (double*)malloc(sizeof(double) * 4 * (size_t)d);
            double *xh = tmp, *a = tmp + d, *dxh = tmp + 2 * d, *lin = tmp + 3 * d;
            for (int t = 0; t < N; ++t) {
                const double* gt = g + base + (size_t)t * d;
                oracle_l2_normalize(q + base + (size_t)t * d, 1, d, eps, xh);
                double den = 0.5 * M[d * d1 + d];
                for (int i = 0; i < d; ++i) den += xh[i] * M[i * d1 + d] / ORACLE_PI;
                double bt = 0.0;
                for (int j = 0; j < d; ++j) {
                    double num = 0.5 * M[d * d1 + j];
                    for (int i = 0; i < d; ++i) num += xh[i] * M[i * d1 + j] / ORACLE_PI;
                    lin[j] = (norm_mode == 0) ? num / den : num;
                    a[j] = (norm_mode == 0) ? gt[j] / den : gt[j];
                    if (norm_mode == 0) bt -= gt[j] * lin[j] / den;
                }
                for (int i = 0; i < d; ++i) {
                    double s = M[i * d1 + d] * bt;
                    for (int j = 0; j < d; ++j) s += M[i * d1 + j] * a[j];
                    dxh[i] = s / ORACLE_PI;
                    for (int j = 0; j < d; ++j) S2[(size_t)i * d + j] += xh[i] * a[j];
                    kb2[i] += xh[i] * bt;
                }
                for (int j = 0; j < d; ++j) va2[j] += a[j];
                normalize_backward(q + base + (size_t)t * d, dxh, d, eps, dq + base + (size_t)t * d);
            }
            for (int j = 0; j < N; ++j) {
                const double* vj = v + base + (size_t)j * d;
                oracle_l2_normalize(k + base + (size_t)j * d, 1, d, eps, xh);
                for (int c = 0; c < d; ++c) {
                    double s = 0.0;
                    for (int i = 0; i < d; ++i) s += xh[i] * S2[(size_t)i * d + c];
                    dv[base + (size_t)j * d + c] = s / ORACLE_PI + 0.5 * va2[c];
                }
                for (int i = 0; i < d; ++i) {
                    double s = kb2[i];
                    for (int c = 0; c < d; ++c) s += S2[(size_t)i * d + c] * vj[c];
                    dxh[i] = s / ORACLE_PI;
                }
                normalize_backward(k + base + (size_t)j * d, dxh, d, eps, dk + base + (size_t)j * d);
            }
            free(S2);
            free(tmp);
        }
        free(state);
    }
    if (branches & ORACLE_BRANCH_DWCONV)
        dwconv_backward(v, w, g, B, heads, H, W, d, ks, extra, dv, dw, dbias);
    if (residual)
        for (size_t i = 0; i < total; ++i) dq[i] += g[i];
}

/* Backward of the downsampling layer (pooled queries on every s-th row and column, residual
 * query): the derivatives of oracle_forward_pooled_explicit by the chain rule, explicit Nq x N
 * similarity.  q, g, dq: [B][heads][Nq][d]; k, v, dk, dv: [B][heads][H*W][d]. */
void oracle_backward_pooled_explicit(const double* q, const double* k, const double* v,
                                     const double* w, const double* g, int B, int heads, int H, int W,
                                     int d, int ks, int s, int residual, int norm_mode,
                                     unsigned branches, double eps, double* dq, double* dk, double* dv,
                                     double* dw, double* dbias)
{
    const int N = H * W, r = ks / 2;
    const int Hq = (H + s - 1) / s, Wq = (W + s - 1) / s, Nq = Hq * Wq;
    const size_t kv_total = (size_t)B * heads * N * d, q_total = (size_t)B * heads * Nq * d;
    memset(dq, 0, sizeof(double) * q_total);
    memset(dk, 0, sizeof(double) * kv_total);
    memset(dv, 0, sizeof(double) * kv_total);
    memset(dw, 0, sizeof(double) * (size_t)heads * d * ks * ks);
    if (dbias) memset(dbias, 0, sizeof(double) * (size_t)heads * d);
    double* qh = (double*)malloc(sizeof(double) * (size_t)Nq * d);
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* dkh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* A = (double*)malloc(sizeof(double) * N);
    double* lin = (double*)malloc(sizeof(double) * d);
    double* dqh = (double*)malloc(sizeof(double) * d);
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < heads; ++h) {
            const size_t kv = ((size_t)b * heads + h) * (size_t)N * d;
            const size_t qo = ((size_t)b * heads + h) * (size_t)Nq * d;
            if (branches & ORACLE_BRANCH_LINEAR) {
                oracle_l2_normalize(q + qo, Nq, d, eps, qh);
                oracle_l2_normalize(k + kv, N, d, eps, kh);
                memset(dkh, 0, sizeof(double) * (size_t)N * d);
                for (int t = 0; t < Nq; ++t) {
                    const double* gt = g + qo + (size_t)t * d;
                    double rs = 0.0;
                    for (int c = 0; c < d; ++c) lin[c] = 0.0;
                    for (int j = 0; j < N; ++j) {
                        double x = 0.0;
                        for (int c = 0; c < d; ++c) x += qh[(size_t)t * d + c] * kh[(size_t)j * d + c];
                        A[j] = 0.5 + x / ORACLE_PI;
                        rs += A[j];
                        for (int c = 0; c < d; ++c) lin[c] += A[j] * v[kv + (size_t)j * d + c];
                    }
                    const double scale = (norm_mode == 0) ? 1.0 / rs : 1.0;
                    double g_lin = 0.0;
                    for (int c = 0; c < d; ++c) g_lin += gt[c] * lin[c] * scale;
                    for (int c = 0; c < d; ++c) dqh[c] = 0.0;
                    for (int j = 0; j < N; ++j) {
                        double g_v = 0.0;
                        for (int c = 0; c < d; ++c) g_v += gt[c] * v[kv + (size_t)j * d + c];
                        const double dA = (norm_mode == 0) ? (g_v - g_lin) / rs : g_v;
                        for (int c = 0; c < d; ++c) {
                            dv[kv + (size_t)j * d + c] += A[j] * scale * gt[c];
                            dqh[c] += dA * kh[(size_t)j * d + c] / ORACLE_PI;
                            dkh[(size_t)j * d + c] += dA * qh[(size_t)t * d + c] / ORACLE_PI;
                        }
                    }
                    normalize_backward(q + qo + (size_t)t * d, dqh, d, eps, dq + qo + (size_t)t * d);
                }
                for (int j = 0; j < N; ++j)
                    normalize_backward(k + kv + (size_t)j * d, dkh + (size_t)j * d, d, eps,
                                       dk + kv + (size_t)j * d);
            }
            if (branches & ORACLE_BRANCH_DWCONV)
                for (int t = 0; t < Nq; ++t) {
                    const double* gt = g + qo + (size_t)t * d;
                    const int y = s * (t / Wq), x = s * (t % Wq);
                    for (int c = 0; c < d; ++c) {
                        if (dbias) dbias[h * d + c] += gt[c];
                        for (int dy = 0; dy < ks; ++dy)
                            for (int dx = 0; dx < ks; ++dx) {
                                const int yy = y + dy - r, xx = x + dx - r;
                                if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                                const size_t src = kv + ((size_t)yy * W + xx) * d + c;
                                const size_t wi = (((size_t)h * d + c) * ks + dy) * ks + dx;
                                dv[src] += w[wi] * gt[c];
                                dw[wi] += gt[c] * v[src];
                            }
                    }
                }
        }
    if (residual)
        for (size_t i = 0; i < q_total; ++i) dq[i] += g[i];
    free(qh); free(kh); free(dkh); free(A); free(lin); free(dqh);
}

/* ------------------------------------------------------------------------
 * Training-time companions of the layer (Sec. 3.2.2, Eq. 10) and the exact
 * angular kernel it approximates (Eq. 4-5), as O(N^2) attention.
 *
 * Readings where the paper is silent: Eq. 10 prints Softmax(Q K^T) with no
 * scale; `normalize` chooses unit rows (the Q, K the angular branch uses) or the
 * raw ones, `scale` multiplies the logits (1 = as printed, 1/sqrt(d) = Eq. 1's
 * convention).  Mask_thr(x) = x if x > thr else 0 (strict, as printed).
 * ---------------------------------------------------------------------- */

/* P[t][j] = Softmax_j(scale * <a_t, b_j>), one head; a, b = q, k or their unit rows. */
void oracle_softmax_probs(const double* q, const double* k, int N, int d, int normalize,
                          double scale, double eps, double* P)
{
    double* qh = (double*)malloc(sizeof(double) * (size_t)N * d);
    double* kh = (double*)malloc(sizeof(double) * (size_t)N * d);
    if (normalize) {
        oracle_l2_normalize(q, N, d, eps, qh);
        oracle_l2_normalize(k, N, d, eps, kh);
    } else {
        memcpy(qh, q, sizeof(double) * (size_t)N * d);
        memcpy(kh, k, sizeof(double) * (size_t)N * d);
    }
    for (int t = 0; t < N; ++t) {
        double* row = P + (size_t)t * N;
        double mx = -INFINITY;
        for (int j = 0; j < N; ++j) {
            double x = 0.0;
            for (int c = 0; c < d; ++c) x += qh[t * d + c] * kh[j * d + c];
            row[j] = scale * x;
            if (row[j] > mx) mx = row[j];
        }
        double sum = 0.0;
        for (int j = 0; j < N; ++j) {
            row[j] = exp(row[j] - mx);
            sum += row[j];
        }
        for (int j = 0; j < N; ++j) row[j] /= sum;
    }
    free(qh);
    free(kh);
}

/* Eq. 10 applied to V for every unit: out_t = sum_j Mask_thr(P_tj) v_j;
 * nnz[unit] = number of entries the mask keeps. */
void oracle_sparse_attn(const double* q, const double* k, const double* v, int B, int heads,
                        int N, int d, int normalize, double scale, double thr, double eps,
                        double* out, int64_t* nnz)
{
    const int units = B * heads;
#pragma omp parallel for schedule(dynamic)
    for (int u = 0; u < units; ++u) {
        const size_t off = (size_t)u * N * d;
        double* P = (double*)malloc(sizeof(double) * (size_t)N * N);
        oracle_softmax_probs(q + off, k + off, N, d, normalize, scale, eps, P);
        int64_t kept = 0;
        for (int t = 0; t < N; ++t) {
            double* o = out + off + (size_t)t * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int j = 0; j < N; ++j) {
                const double p = P[(size_t)t * N + j];
                if (p > thr) {
                    ++kept;
                    for (int c = 0; c < d; ++c) o[c] += p * v[off + (size_t)j * d + c];
                }
            }
        }
        nnz[u] = kept;
        free(P);
    }
}

/* Attention with the exact angular kernel (Eq. 5) in place of its linear terms:
 * out_t = sum_j A_tj v_j / sum_j A_tj (norm_mode 0, Eq. 3's form) or the bare sum. */
void oracle_angular_attn(const double* q, const double* k, const double* v, int B, int heads,
                         int N, int d, int norm_mode, double eps, double* out)
{
    const int units = B * heads;
#pragma omp parallel for schedule(dynamic)
    for (int u = 0; u < units; ++u) {
        const size_t off = (size_t)u * N * d;
        double* A = (double*)malloc(sizeof(double) * (size_t)N * N);
        oracle_sim_angular(q + off, k + off, N, d, eps, A);
        for (int t = 0; t < N; ++t) {
            double* o = out + off + (size_t)t * d;
            double den = 0.0;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int j = 0; j < N; ++j) {
                const double a = A[(size_t)t * N + j];
                den += a;
                for (int c = 0; c < d; ++c) o[c] += a * v[off + (size_t)j * d + c];
            }
            if (norm_mode == 0)
                for (int c = 0; c < d; ++c) o[c] /= den;
        }
        free(A);
    }
}

/* Number of threads the parallel-for above will use (1 without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
