/* Plain-loop fp64 definitions of the layer operators.  TEST INFRASTRUCTURE ONLY (part of the CPU oracle).
 *
 * Every function is the sum of its definition written out as nested loops, in fp64, with no blocking, no library call
 * and no reordering beyond running independent output rows on different threads:
 *   fully-connected layer (Sec. 2.1 of arXiv 1805.04170):  x_{l+1} = f(x_l W_l),
 *       dC/dx_l = df(dC/dx_{l+1}) W_l^T,  dC/dW_l = x_l^T df(dC/dx_{l+1}),  W_l is n_in x n_out;
 *   convolution (Sec. 4.5 names it; the paper gives no formula): the textbook stride-1 cross-correlation with zero
 *       padding, Y[n,ko,y,x] = sum_{c,r,s} X[n,c,y+r-pad,x+s-pad] W[ko,c,r,s], and its two exact adjoints.
 * All arrays are dense, row-major, C order.  oracle/layers.py (the numpy form used for large checks) is pinned against
 * these on small shapes, and the benchmark's cpu_baseline times these.
 */
#include <stdint.h>
#include <string.h>

/* Z[i][j] = sum_k A[i][k] B[k][j]   (i-k-j order: the inner loop walks rows of B and Z) */
void plain_matmul(const double *A, const double *B, double *Z, int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *z = Z + i * N;
        for (int64_t j = 0; j < N; ++j) z[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[i * K + k];
            const double *b = B + k * N;
            for (int64_t j = 0; j < N; ++j) z[j] += a * b[j];
        }
    }
}

/* Z[i][j] = sum_k A[i][k] B[j][k]   (second operand transposed: dX = G W^T) */
void plain_matmul_nt(const double *A, const double *B, double *Z, int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) acc += A[i * K + k] * B[j * K + k];
            Z[i * N + j] = acc;
        }
}

/* Z[i][j] = sum_k A[k][i] B[k][j]   (first operand transposed: dW = X^T G); A is K x M */
void plain_matmul_tn(const double *A, const double *B, double *Z, int64_t M, int64_t K, int64_t N)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *z = Z + i * N;
        for (int64_t j = 0; j < N; ++j) z[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = A[k * M + i];
            const double *b = B + k * N;
            for (int64_t j = 0; j < N; ++j) z[j] += a * b[j];
        }
    }
}

/* Y = f(X W), f = ReLU if relu else identity.  X: b x n_in, W: n_in x n_out, Y: b x n_out */
void plain_fc_forward(const double *X, const double *W, double *Y, int64_t b, int64_t n_in, int64_t n_out, int relu)
{
    plain_matmul(X, W, Y, b, n_in, n_out);
    if (relu)
        for (int64_t i = 0; i < b * n_out; ++i) Y[i] = Y[i] > 0.0 ? Y[i] : 0.0;
}

/* G = dY where Y > 0 (ReLU) else 0, or dY;  dX = G W^T;  dW = X^T G.  G is scratch of b x n_out. */
void plain_fc_backward(const double *dY, const double *X, const double *W, const double *Y, double *G, double *dX,
                       double *dW, int64_t b, int64_t n_in, int64_t n_out, int relu)
{
    for (int64_t i = 0; i < b * n_out; ++i) G[i] = (!relu || Y[i] > 0.0) ? dY[i] : 0.0;
    plain_matmul_nt(G, W, dX, b, n_out, n_in);
    plain_matmul_tn(X, G, dW, n_in, b, n_out);
}

/* X: [N][C][H][W], Wt: [K][C][R][S], Y: [N][K][P][Q] with P = H + 2 pad - R + 1, Q = W + 2 pad - S + 1 */
void plain_conv_forward(const double *X, const double *Wt, double *Y, int64_t N, int64_t C, int64_t H, int64_t Wd,
                        int64_t K, int64_t R, int64_t S, int64_t pad)
{
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t ko = 0; ko < K; ++ko)
            for (int64_t y = 0; y < P; ++y)
                for (int64_t x = 0; x < Q; ++x) {
                    double acc = 0.0;
                    for (int64_t c = 0; c < C; ++c)
                        for (int64_t r = 0; r < R; ++r)
                            for (int64_t s = 0; s < S; ++s) {
                                const int64_t h = y + r - pad, w = x + s - pad;
                                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                                acc += X[((n * C + c) * H + h) * Wd + w] * Wt[((ko * C + c) * R + r) * S + s];
                            }
                    Y[((n * K + ko) * P + y) * Q + x] = acc;
                }
}

/* dX[n][c][h][w] = sum over every (ko, y, x, r, s) whose forward term reads X[n][c][h][w] of dY[n][ko][y][x] W[ko][c][r][s] */
void plain_conv_dgrad(const double *dY, const double *Wt, double *dX, int64_t N, int64_t C, int64_t H, int64_t Wd,
                      int64_t K, int64_t R, int64_t S, int64_t pad)
{
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t h = 0; h < H; ++h)
                for (int64_t w = 0; w < Wd; ++w) {
                    double acc = 0.0;
                    for (int64_t ko = 0; ko < K; ++ko)
                        for (int64_t r = 0; r < R; ++r)
                            for (int64_t s = 0; s < S; ++s) {
                                const int64_t y = h - r + pad, x = w - s + pad;
                                if (y < 0 || y >= P || x < 0 || x >= Q) continue;
                                acc += dY[((n * K + ko) * P + y) * Q + x] * Wt[((ko * C + c) * R + r) * S + s];
                            }
                    dX[((n * C + c) * H + h) * Wd + w] = acc;
                }
}

/* dW[ko][c][r][s] = sum_{n,y,x} X[n][c][y+r-pad][x+s-pad] dY[n][ko][y][x] */
void plain_conv_wgrad(const double *X, const double *dY, double *dW, int64_t N, int64_t C, int64_t H, int64_t Wd,
                      int64_t K, int64_t R, int64_t S, int64_t pad)
{
    const int64_t P = H + 2 * pad - R + 1, Q = Wd + 2 * pad - S + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t ko = 0; ko < K; ++ko)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t r = 0; r < R; ++r)
                for (int64_t s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int64_t n = 0; n < N; ++n)
                        for (int64_t y = 0; y < P; ++y)
                            for (int64_t x = 0; x < Q; ++x) {
                                const int64_t h = y + r - pad, w = x + s - pad;
                                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                                acc += X[((n * C + c) * H + h) * Wd + w] * dY[((n * K + ko) * P + y) * Q + x];
                            }
                    dW[((ko * C + c) * R + r) * S + s] = acc;
                }
}
