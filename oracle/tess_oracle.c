/*
 * tess_oracle.c -- CPU fp64 oracle for the per-processor compute of a linear
 * layer partitioned over a Tesseract [q, q, d] processor grid.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP library, and the HIP library
 * never calls it.
 *
 * Everything is the plain definition written out in double precision:
 * Tesseract re-brackets a dense matrix product exactly (the paper's
 * experiment section checks the partitioned result against the unpartitioned
 * one and its conclusion states that no approximation is introduced), so the
 * oracle is the definition of the blocked sums, evaluated with the panels in
 * ascending step order t = 0..q-1 and, inside a panel, the contracted index
 * ascending.  No tiling, no fusion, no BLAS.
 *
 * Pinned (tests/test_oracle_pins.py) against: numpy's fp64 matmul on the
 * unpartitioned matrices (reassembly invariant of Alg. 3, gradient identities
 * of the SUMMA gradient equation, depth sum of Section 3.1), the adjoint
 * identity <dY, XW> = <dX, X> = <dW, W>, one-hot inputs that expose the block
 * map h = i + k*q, the hand-written partition table under tests/golden/,
 * exact small-integer products, textbook values of the normal CDF for GELU,
 * bit-level ties for the bf16 rounding helper, central differences of the
 * (pinned) GELU forms and the location of GELU's minimum for the derivatives,
 * and the total-sum and all-ones identities for the bias gradient.
 *
 * Build: gcc -O2 -fopenmp -fPIC -shared -o libtess_oracle.so tess_oracle.c -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_ACT_NONE 0
#define ORC_ACT_GELU_ERF 1
#define ORC_ACT_GELU_TANH 2

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- scalar helpers ------------------------------------------------------ */

/* GELU as x * Phi(x), Phi the standard normal CDF (the definition), and the
 * tanh form that some frameworks use instead.  The paper only says that the
 * MLP has an activation between its two linears (Section 2.4). */
double orc_gelu_erf(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

double orc_gelu_tanh(double x)
{
    const double pi = 3.14159265358979323846;
    const double c = sqrt(2.0 / pi);
    return 0.5 * x * (1.0 + tanh(c * (x + 0.044715 * x * x * x)));
}

/* Derivatives of the two GELU forms (product and chain rule on the definitions
 * above): d/dx [x Phi(x)] = Phi(x) + x phi(x) with phi the standard normal
 * density; for the tanh form, with u = c (x + 0.044715 x^3):
 * 0.5 (1 + tanh u) + 0.5 x (1 - tanh^2 u) c (1 + 3 * 0.044715 x^2).          */
double orc_gelu_erf_grad(double x)
{
    const double pi = 3.14159265358979323846;
    const double Phi = 0.5 * (1.0 + erf(x / sqrt(2.0)));
    const double phi = exp(-0.5 * x * x) / sqrt(2.0 * pi);
    return Phi + x * phi;
}

double orc_gelu_tanh_grad(double x)
{
    const double pi = 3.14159265358979323846;
    const double c = sqrt(2.0 / pi);
    const double u = c * (x + 0.044715 * x * x * x);
    const double th = tanh(u);
    return 0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * c * (1.0 + 3.0 * 0.044715 * x * x);
}

static double orc_act_grad(double x, int act)
{
    if (act == ORC_ACT_GELU_ERF) return orc_gelu_erf_grad(x);
    if (act == ORC_ACT_GELU_TANH) return orc_gelu_tanh_grad(x);
    return 1.0;
}

static double orc_act(double x, int act)
{
    if (act == ORC_ACT_GELU_ERF) return orc_gelu_erf(x);
    if (act == ORC_ACT_GELU_TANH) return orc_gelu_tanh(x);
    return x;
}

/* Round an fp32 value to the nearest bfloat16 (ties to even mantissa) and
 * return it widened back to fp32.  bfloat16 is the upper 16 bits of the
 * IEEE-754 binary32 pattern. NaN stays NaN (quiet). */
float orc_round_bf16_scalar(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {
        u = (u | 0x00400000u) & 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    memcpy(&x, &u, 4);
    return x;
}

void orc_round_bf16(const float* in, double* out, int64_t count)
{
    for (int64_t e = 0; e < count; ++e) out[e] = (double)orc_round_bf16_scalar(in[e]);
}

/* ---- unpartitioned definitions ------------------------------------------- */

/* C[M,N] = A[M,K] * B[K,N], all row-major and packed. */
void orc_matmul_nn(const double* A, const double* B, double* C, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        double* crow = C + r * N;
        for (int64_t s = 0; s < N; ++s) crow[s] = 0.0;
        for (int64_t u = 0; u < K; ++u) {
            const double av = A[r * K + u];
            const double* brow = B + u * N;
            for (int64_t s = 0; s < N; ++s) crow[s] += av * brow[s];
        }
    }
}

/* C[M,N] = A[M,K] * B[N,K]^T. */
void orc_matmul_nt(const double* A, const double* B, double* C, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        for (int64_t s = 0; s < N; ++s) {
            double acc = 0.0;
            for (int64_t u = 0; u < K; ++u) acc += A[r * K + u] * B[s * K + u];
            C[r * N + s] = acc;
        }
    }
}

/* C[M,N] = A[K,M]^T * B[K,N]. */
void orc_matmul_tn(const double* A, const double* B, double* C, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        double* crow = C + r * N;
        for (int64_t s = 0; s < N; ++s) crow[s] = 0.0;
        for (int64_t u = 0; u < K; ++u) {
            const double av = A[u * M + r];
            const double* brow = B + u * N;
            for (int64_t s = 0; s < N; ++s) crow[s] += av * brow[s];
        }
    }
}

/* ---- partition of Alg. 3 --------------------------------------------------
 * A[a,b] is cut into q*d block rows and q block columns, B[b,c] into q x q
 * blocks that every depth layer holds a copy of, C[a,c] like A.  Processor
 * (i,j,k) holds block row h = i + k*q of A and C (Alg. 3, set-up loop).     */

int64_t orc_block_row(int q, int i, int k) { return (int64_t)i + (int64_t)k * q; }

/* Returns 0 when the grid and sizes are admissible: 1 <= d <= q
 * (Section 3.1), coordinates inside the grid, and the sizes divisible so that
 * every block has the shape [a/(qd), b/q], [b/q, c/q], [a/(qd), c/q].       */
int orc_check_grid(int q, int d, int i, int j, int k, int64_t a, int64_t b, int64_t c)
{
    if (q < 1 || d < 1 || d > q) return 1;
    if (i < 0 || i >= q || j < 0 || j >= q || k < 0 || k >= d) return 1;
    if (a < 1 || b < 1 || c < 1) return 2;
    if (a % ((int64_t)q * d) != 0 || b % q != 0 || c % q != 0) return 2;
    return 0;
}

/* ---- per-processor formulas on panels ------------------------------------
 * A "panel" is one block that the paper delivers by a row or column
 * broadcast at step t.  Panels are row-major with a leading dimension in
 * elements.  `rows`/`n_rows` select a subset of OUTPUT rows (NULL = all);
 * out is packed [n_rows_or_all, width].                                     */

/* Forward, Alg. 3 inner loop plus the bias/activation that follow it:
 *   Z[r,s] = sum_{t<q} sum_{u<kb} A_t[r,u] * B_t[u,s]
 *   Y[r,s] = act(Z[r,s] + bias[s])
 * a_panels[t]: [m,kb] (the block A_{i,t,k}); b_panels[t]: [kb,n] (B_{t,j});
 * bias: [n] slice j of the bias or NULL.  z_out (optional) receives Z+bias. */
void orc_fwd_panels(int q, int64_t m, int64_t kb, int64_t n,
                    const double* const* a_panels, int64_t lda,
                    const double* const* b_panels, int64_t ldb,
                    const double* bias, int act,
                    const int64_t* rows, int64_t n_rows,
                    double* y_out, double* z_out)
{
    const int64_t R = rows ? n_rows : m;
#pragma omp parallel for schedule(static)
    for (int64_t rr = 0; rr < R; ++rr) {
        const int64_t r = rows ? rows[rr] : rr;
        double* acc = y_out + rr * n;
        for (int64_t s = 0; s < n; ++s) acc[s] = 0.0;
        for (int t = 0; t < q; ++t) {
            const double* At = a_panels[t];
            const double* Bt = b_panels[t];
            for (int64_t u = 0; u < kb; ++u) {
                const double av = At[r * lda + u];
                const double* brow = Bt + u * ldb;
                for (int64_t s = 0; s < n; ++s) acc[s] += av * brow[s];
            }
        }
        for (int64_t s = 0; s < n; ++s) {
            const double z = acc[s] + (bias ? bias[s] : 0.0);
            if (z_out) z_out[rr * n + s] = z;
            acc[s] = orc_act(z, act);
        }
    }
}

/* Input gradient (A' = C' B^T of the SUMMA gradient equation, evaluated on
 * the owner of the block):
 *   dX[r,u] = sum_{t<q} sum_{s<n} dY_t[r,s] * W_t[u,s]
 * dy_panels[t]: [m,n] (dY_{i,t,k}); w_panels[t]: [kb,n] (W_{j,t}).          */
void orc_bwd_dx_panels(int q, int64_t m, int64_t kb, int64_t n,
                       const double* const* dy_panels, int64_t lddy,
                       const double* const* w_panels, int64_t ldw,
                       const int64_t* rows, int64_t n_rows, double* dx_out)
{
    const int64_t R = rows ? n_rows : m;
#pragma omp parallel for schedule(static)
    for (int64_t rr = 0; rr < R; ++rr) {
        const int64_t r = rows ? rows[rr] : rr;
        for (int64_t u = 0; u < kb; ++u) {
            double acc = 0.0;
            for (int t = 0; t < q; ++t) {
                const double* dyrow = dy_panels[t] + r * lddy;
                const double* wrow = w_panels[t] + u * ldw;
                for (int64_t s = 0; s < n; ++s) acc += dyrow[s] * wrow[s];
            }
            dx_out[rr * kb + u] = acc;
        }
    }
}

/* Input gradient followed by the backward of the activation that produced the
 * layer's input (the MLP's middle activation, Section 2.4): with Z the
 * pre-activation that the previous linear layer saved, [m,kb],
 *   dZ[r,u] = dX[r,u] * act'(Z[r,u]),   dX as in orc_bwd_dx_panels.          */
void orc_bwd_dx_act_panels(int q, int64_t m, int64_t kb, int64_t n,
                           const double* const* dy_panels, int64_t lddy,
                           const double* const* w_panels, int64_t ldw,
                           const double* z, int64_t ldz, int act,
                           const int64_t* rows, int64_t n_rows, double* dz_out)
{
    orc_bwd_dx_panels(q, m, kb, n, dy_panels, lddy, w_panels, ldw, rows, n_rows, dz_out);
    const int64_t R = rows ? n_rows : m;
    for (int64_t rr = 0; rr < R; ++rr) {
        const int64_t r = rows ? rows[rr] : rr;
        for (int64_t u = 0; u < kb; ++u) dz_out[rr * kb + u] *= orc_act_grad(z[r * ldz + u], act);
    }
}

/* Bias gradient.  The forward adds bias_j to every row of every block of block
 * column j (Section 3.2, bias-add); its gradient is therefore the sum of dY
 * over all those rows, which the paper collects on grid row 0 by a reduction
 * along the column.  The q panels dY_{t,j,k} of one depth layer are exactly the
 * blocks of that column, so
 *   db[s] = sum_{t<q} sum_{r<m} dY_t[r,s]
 * is what row 0 holds for depth layer k; `accumulate` adds further layers.   */
void orc_bias_grad_panels(int q, int64_t m, int64_t n,
                          const double* const* dy_panels, int64_t lddy,
                          int accumulate, double* db_out)
{
    for (int64_t s = 0; s < n; ++s) {
        double acc = 0.0;
        for (int t = 0; t < q; ++t)
            for (int64_t r = 0; r < m; ++r) acc += dy_panels[t][r * lddy + s];
        db_out[s] = accumulate ? db_out[s] + acc : acc;
    }
}

/* Weight gradient of one depth layer (B' = A^T C'):
 *   dW[u,s] = sum_{t<q} sum_{r<m} X_t[r,u] * dY_t[r,s]
 * x_panels[t]: [m,kb] (X_{t,i,k}); dy_panels[t]: [m,n] (dY_{t,j,k}).  When
 * `accumulate` is non-zero the result is added to dw_out (the sum over the d
 * depth layers that Section 3.1 obtains with an all-reduce).                */
void orc_bwd_dw_panels(int q, int64_t m, int64_t kb, int64_t n,
                       const double* const* x_panels, int64_t ldx,
                       const double* const* dy_panels, int64_t lddy,
                       const int64_t* rows, int64_t n_rows,
                       int accumulate, double* dw_out)
{
    const int64_t R = rows ? n_rows : kb;
#pragma omp parallel for schedule(static)
    for (int64_t uu = 0; uu < R; ++uu) {
        const int64_t u = rows ? rows[uu] : uu;
        double* acc = (double*)malloc((size_t)n * sizeof(double));
        for (int64_t s = 0; s < n; ++s) acc[s] = 0.0;
        for (int t = 0; t < q; ++t) {
            const double* Xt = x_panels[t];
            const double* dYt = dy_panels[t];
            for (int64_t r = 0; r < m; ++r) {
                const double xv = Xt[r * ldx + u];
                const double* dyrow = dYt + r * lddy;
                for (int64_t s = 0; s < n; ++s) acc[s] += xv * dyrow[s];
            }
        }
        double* orow = dw_out + uu * n;
        for (int64_t s = 0; s < n; ++s) orow[s] = accumulate ? orow[s] + acc[s] : acc[s];
        free(acc);
    }
}

/* ---- layer normalisation, local parts (Section 3.2, "Other procedure") -----
 * The hidden dimension of a row is spread over the q processors of a grid row.
 * Each computes the sum and the sum of squares of its own [m, w] block per row;
 * the two numbers are then summed over the grid row (an all-reduce that is the
 * caller's business; `accumulate` adds a further block's sums) and every
 * processor normalises its block with
 *   E[X] = S1 / n,  Var[X] = S2 / n - E[X]^2,  xhat = (x - E[X]) / sqrt(Var[X] + eps),
 * n the full hidden size.                                                     */
void orc_row_sums(const double* x, int64_t m, int64_t w, int64_t ldx, int accumulate,
                  double* sums_out /* [m, 2] */)
{
    for (int64_t r = 0; r < m; ++r) {
        double s1 = 0.0, s2 = 0.0;
        for (int64_t u = 0; u < w; ++u) {
            const double v = x[r * ldx + u];
            s1 += v;
            s2 += v * v;
        }
        sums_out[2 * r] = accumulate ? sums_out[2 * r] + s1 : s1;
        sums_out[2 * r + 1] = accumulate ? sums_out[2 * r + 1] + s2 : s2;
    }
}

void orc_layernorm_from_sums(const double* x, int64_t m, int64_t w, int64_t ldx,
                             const double* sums /* [m, 2] */, int64_t n_total, double eps,
                             double* xhat_out /* [m, w] packed */)
{
    for (int64_t r = 0; r < m; ++r) {
        const double mean = sums[2 * r] / (double)n_total;
        /* a variance is non-negative; the difference of the two moments may round below zero */
        const double var = fmax(sums[2 * r + 1] / (double)n_total - mean * mean, 0.0);
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t u = 0; u < w; ++u) xhat_out[r * w + u] = (x[r * ldx + u] - mean) * rstd;
    }
}

/* Backward of the normalisation (the X' equation of the same passage): with
 * g = dJ/dxhat and n the full hidden size,
 *   X' = ( g - ( xhat * sum_j(xhat_j g_j) + sum_j g_j ) / n ) / sqrt(Var[X] + eps).
 * The two row sums are again local partial sums that are reduced along the grid
 * row; Var comes from the forward sums S1, S2.                                */
void orc_row_sums_bwd(const double* xhat, const double* g, int64_t m, int64_t w, int64_t ldx,
                      int64_t ldg, int accumulate, double* sums_out /* [m, 2] */)
{
    for (int64_t r = 0; r < m; ++r) {
        double a = 0.0, b = 0.0;
        for (int64_t u = 0; u < w; ++u) {
            a += xhat[r * ldx + u] * g[r * ldg + u];
            b += g[r * ldg + u];
        }
        sums_out[2 * r] = accumulate ? sums_out[2 * r] + a : a;
        sums_out[2 * r + 1] = accumulate ? sums_out[2 * r + 1] + b : b;
    }
}

void orc_layernorm_bwd_from_sums(const double* xhat, const double* g, int64_t m, int64_t w,
                                 int64_t ldx, int64_t ldg, const double* sums_bwd,
                                 const double* sums_fwd, int64_t n_total, double eps,
                                 double* dx_out /* [m, w] packed */)
{
    for (int64_t r = 0; r < m; ++r) {
        const double mean = sums_fwd[2 * r] / (double)n_total;
        const double var = fmax(sums_fwd[2 * r + 1] / (double)n_total - mean * mean, 0.0);
        const double rstd = 1.0 / sqrt(var + eps);
        for (int64_t u = 0; u < w; ++u) {
            const double xh = xhat[r * ldx + u];
            dx_out[r * w + u] = (g[r * ldg + u] - (xh * sums_bwd[2 * r] + sums_bwd[2 * r + 1]) / (double)n_total) * rstd;
        }
    }
}

/* ---- per-processor formulas on the unpartitioned matrices ----------------
 * These cut the blocks out of the global matrices exactly as Alg. 3 lays
 * them out and hand them to the panel formulas above.                       */

/* Y_{i,j,k} [a/(qd), c/q] from A[a,b], B[b,c], bias[c] (or NULL). */
int orc_tess_fwd(int q, int d, int i, int j, int k, int64_t a, int64_t b, int64_t c,
                 const double* A, const double* B, const double* bias, int act,
                 double* y_block, double* z_block)
{
    int rc = orc_check_grid(q, d, i, j, k, a, b, c);
    if (rc) return rc;
    const int64_t m = a / ((int64_t)q * d), kb = b / q, n = c / q;
    const int64_t h = orc_block_row(q, i, k);
    const double** ap = (const double**)malloc(sizeof(double*) * q);
    const double** bp = (const double**)malloc(sizeof(double*) * q);
    for (int t = 0; t < q; ++t) {
        ap[t] = A + (h * m) * b + (int64_t)t * kb;       /* A_{i,t,k}: block (h, t) */
        bp[t] = B + ((int64_t)t * kb) * c + (int64_t)j * n; /* B_{t,j}              */
    }
    orc_fwd_panels(q, m, kb, n, ap, b, bp, c, bias ? bias + (int64_t)j * n : NULL, act,
                   NULL, 0, y_block, z_block);
    free(ap);
    free(bp);
    return 0;
}

/* dX_{i,j,k} [a/(qd), b/q] from dY[a,c], W[b,c]. */
int orc_tess_bwd_dx(int q, int d, int i, int j, int k, int64_t a, int64_t b, int64_t c,
                    const double* dY, const double* W, double* dx_block)
{
    int rc = orc_check_grid(q, d, i, j, k, a, b, c);
    if (rc) return rc;
    const int64_t m = a / ((int64_t)q * d), kb = b / q, n = c / q;
    const int64_t h = orc_block_row(q, i, k);
    const double** dyp = (const double**)malloc(sizeof(double*) * q);
    const double** wp = (const double**)malloc(sizeof(double*) * q);
    for (int t = 0; t < q; ++t) {
        dyp[t] = dY + (h * m) * c + (int64_t)t * n;            /* dY_{i,t,k}        */
        wp[t] = W + ((int64_t)j * kb) * c + (int64_t)t * n;    /* W_{j,t}           */
    }
    orc_bwd_dx_panels(q, m, kb, n, dyp, c, wp, c, NULL, 0, dx_block);
    free(dyp);
    free(wp);
    return 0;
}

/* Depth-k partial dW^{(k)}_{i,j} [b/q, c/q] from X[a,b], dY[a,c]. */
int orc_tess_bwd_dw(int q, int d, int i, int j, int k, int64_t a, int64_t b, int64_t c,
                    const double* X, const double* dY, int accumulate, double* dw_block)
{
    int rc = orc_check_grid(q, d, i, j, k, a, b, c);
    if (rc) return rc;
    const int64_t m = a / ((int64_t)q * d), kb = b / q, n = c / q;
    const double** xp = (const double**)malloc(sizeof(double*) * q);
    const double** dyp = (const double**)malloc(sizeof(double*) * q);
    for (int t = 0; t < q; ++t) {
        const int64_t h = orc_block_row(q, t, k);
        xp[t] = X + (h * m) * b + (int64_t)i * kb;    /* X_{t,i,k}: block (t+kq, i)  */
        dyp[t] = dY + (h * m) * c + (int64_t)j * n;   /* dY_{t,j,k}                  */
    }
    orc_bwd_dw_panels(q, m, kb, n, xp, b, dyp, c, NULL, 0, accumulate, dw_block);
    free(xp);
    free(dyp);
    return 0;
}

/* ||G - O||_F / ||O||_F ; returns ||G||_F when O is all zero. */
double orc_rel_frobenius(const double* G, const double* O, int64_t count)
{
    double num = 0.0, den = 0.0;
    for (int64_t e = 0; e < count; ++e) {
        const double df = G[e] - O[e];
        num += df * df;
        den += O[e] * O[e];
    }
    if (den == 0.0) return sqrt(num);
    return sqrt(num / den);
}
