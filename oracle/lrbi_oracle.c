/*
 * CPU oracle for low-rank binary indexing (arXiv 1905.05686).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code with the HIP path, is never
 * called from it, and must stay free of blocking, packing or fusion so that it
 * can be checked against the paper by eye.
 *
 * Conventions (one byte per bit, row-major everywhere):
 *   W     m x n      weights (already rounded to the storage dtype, widened to double)
 *   Ip01  [T][r][k]  left binary factor of every tile,  T = ceil(m/r)*ceil(n/c)
 *   Iz01  [T][k][c]  right binary factor of every tile
 *   tile t = ti*ceil(n/c) + tj covers rows ti*r .. ti*r+r-1, columns tj*c .. tj*c+c-1,
 *   cut off at the matrix edge: a tile of the last tile row / column that sticks out keeps
 *   its full-size factors and uses only their first m - ti*r rows (of I_p) and first
 *   n - tj*c columns (of I_z).  The paper's tilings all divide (Sec. 3.1); this is the
 *   builder's reading for the ones that do not.
 *   tile_rank [T] (optional): tile t uses only the first tile_rank[t] <= k columns of its
 *   I_p and rows of its I_z ("each submatrix can choose a different rank", end of Sec. 3.1).
 *   M     m x n      decoded mask, 1 = weight kept, 0 = weight pruned (Sec. 2, Eq. 2)
 *   X     n x N,  Y  m x N
 *
 * Pins (tests/test_oracle_*.py): the printed 5x5 example (Eq. 5 -> Eq. 6),
 * brute force against the set definition on tiny tiles, the integer-product
 * formulation, closed forms of Table 1 / Table 3, the density law of Eq. 7.
 * The LSTM recurrence and the CSR size formula (oracle/lstm.py, csr_bits) are
 * the builder's own definitions: parity unpinned by the paper (the LSTM cell is pinned to a
 * handwritten case of exact-rational gate activations, tests/test_oracle_lstm.py; the CSR
 * formula has no pin beyond its own statement).
 * Edge tiles and per-tile ranks (tests/test_oracle_general.py): brute force from the set
 * definition, the crop of the zero-padded matrix's decode, tile-by-tile decodes at each
 * tile's own rank, and the closed form k (ceil(n/c) m + ceil(m/r) n) of the size.
 * Backward pass of the masking layer (tests/test_oracle_backward.py): the adjoint identity
 * <dY, (W o M) X> = <(W o M)^T dY, X> against the pinned forward product, exact differences of
 * the (linear) loss in single weights, and numpy's dense products on the masked matrix.
 * Candidate evaluation of Algorithm 1 (threshold, decode, S_a, Cost): pinned by the
 * printed example (Eq. 4 with T_p = 0.5, T_z = 0.6 gives Eq. 5 and Eq. 6; its two
 * mismatches are kept weights, so Cost = 0), by an independent array formulation, by
 * the limits T = -inf / +inf and by monotonicity in the thresholds
 * (tests/test_oracle_threshold.py).
 */
#include <stddef.h>
#include <stdint.h>

/* Eq. 3, applied independently to every tile (Sec. 3.1):
 * (I_a)_{i,j} = OR_{l=1..k_t} (I_p)_{i,l} AND (I_z)_{l,j}, k_t = tile_rank[t] (k when tile_rank is NULL). */
int lrbi_oracle_decode_ranked(int64_t m, int64_t n, int64_t r, int64_t c, int64_t k, const int32_t *tile_rank,
                              const uint8_t *Ip01, const uint8_t *Iz01, uint8_t *M)
{
    if (m <= 0 || n <= 0 || r <= 0 || c <= 0 || k <= 0) return -1;
    const int64_t tile_rows = (m + r - 1) / r, tile_cols = (n + c - 1) / c;
    for (int64_t ti = 0; ti < tile_rows; ++ti) {
        for (int64_t tj = 0; tj < tile_cols; ++tj) {
            const int64_t t = ti * tile_cols + tj;
            const uint8_t *Ip = Ip01 + t * r * k;   /* r x k */
            const uint8_t *Iz = Iz01 + t * k * c;   /* k x c */
            const int64_t kt = tile_rank ? tile_rank[t] : k;
            if (kt < 0 || kt > k) return -3;
            for (int64_t i = 0; i < r && ti * r + i < m; ++i) {
                for (int64_t j = 0; j < c && tj * c + j < n; ++j) {
                    uint8_t bit = 0;
                    for (int64_t l = 0; l < kt; ++l) {
                        const uint8_t a = Ip[i * k + l] != 0;
                        const uint8_t b = Iz[l * c + j] != 0;
                        bit = bit | (a & b);
                    }
                    M[(ti * r + i) * n + (tj * c + j)] = bit;
                }
            }
        }
    }
    return 0;
}

int lrbi_oracle_decode(int64_t m, int64_t n, int64_t r, int64_t c, int64_t k,
                       const uint8_t *Ip01, const uint8_t *Iz01, uint8_t *M)
{
    return lrbi_oracle_decode_ranked(m, n, r, c, k, NULL, Ip01, Iz01, M);
}

/* Masked layer product (Sec. 2: the mask is a "binary masking layer" on W):
 * Y[i,q] = sum over j with M[i,j] = 1 of W[i,j] * X[j,q], in double.
 * A pruned weight is skipped, so whatever value sits under a 0 bit (even NaN
 * or Inf) never reaches Y.  Rows are independent; `threads` > 1 only spreads
 * rows over OpenMP threads and does not change any sum's order (ascending j). */
int lrbi_oracle_masked_gemm(int64_t m, int64_t n, int64_t N,
                            const double *W, const uint8_t *M, const double *X,
                            double *Y, int threads)
{
    if (m <= 0 || n <= 0 || N <= 0) return -1;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double *y = Y + i * N;
        for (int64_t q = 0; q < N; ++q) y[q] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            if (M[i * n + j] == 0) continue;
            const double w = W[i * n + j];
            const double *x = X + j * N;
            for (int64_t q = 0; q < N; ++q) y[q] += w * x[q];
        }
    }
    return 0;
}

/* Backward pass of the masked layer (Sec. 2: the mask is a masking layer on W, so retraining sends
 * gradients through the kept weights only).  With Y = (W o M) X and dY the gradient of a loss with
 * respect to Y:
 *   dX[j,q] = sum over i with M[i,j] = 1 of W[i,j] * dY[i,q]      (the transposed masked product),
 *   dW[i,j] = M[i,j] * sum over q of dY[i,q] * X[j,q]             (pruned weights get exactly 0).
 * Both in double; sums in ascending i resp. q. */
int lrbi_oracle_masked_gemm_t(int64_t m, int64_t n, int64_t N, const double *W, const uint8_t *M,
                              const double *dY, double *dX)
{
    if (m <= 0 || n <= 0 || N <= 0) return -1;
    for (int64_t j = 0; j < n; ++j)
        for (int64_t q = 0; q < N; ++q) dX[j * N + q] = 0.0;
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t j = 0; j < n; ++j) {
            if (M[i * n + j] == 0) continue;
            const double w = W[i * n + j];
            for (int64_t q = 0; q < N; ++q) dX[j * N + q] += w * dY[i * N + q];
        }
    }
    return 0;
}

int lrbi_oracle_masked_grad(int64_t m, int64_t n, int64_t N, const double *dY, const double *X,
                            const uint8_t *M, double *dW)
{
    if (m <= 0 || n <= 0 || N <= 0) return -1;
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t j = 0; j < n; ++j) {
            double s = 0.0;
            if (M[i * n + j] != 0)
                for (int64_t q = 0; q < N; ++q) s += dY[i * N + q] * X[j * N + q];
            dW[i * n + j] = s;
        }
    }
    return 0;
}

/* Index size of the factor pair: k(m+n) bits for one matrix (Sec. 2.2, the
 * compression ratio mn/(k(m+n))); with tiling every tile stores its own
 * r_t x k_t and k_t x c_t factors (Sec. 3.1), r_t x c_t the part of the tile inside
 * the matrix and k_t its rank: the sum over tiles of k_t (r_t + c_t) bits. */
uint64_t lrbi_oracle_index_bits_ranked(int64_t m, int64_t n, int64_t r, int64_t c, int64_t k, const int32_t *tile_rank)
{
    if (m <= 0 || n <= 0 || r <= 0 || c <= 0 || k <= 0) return 0;
    const int64_t tile_rows = (m + r - 1) / r, tile_cols = (n + c - 1) / c;
    uint64_t bits = 0;
    for (int64_t ti = 0; ti < tile_rows; ++ti) {
        for (int64_t tj = 0; tj < tile_cols; ++tj) {
            const int64_t rt = (m - ti * r < r) ? m - ti * r : r;
            const int64_t ct = (n - tj * c < c) ? n - tj * c : c;
            const int64_t kt = tile_rank ? tile_rank[ti * tile_cols + tj] : k;
            bits += (uint64_t)kt * (uint64_t)(rt + ct);
        }
    }
    return bits;
}

uint64_t lrbi_oracle_index_bits(int64_t m, int64_t n, int64_t r, int64_t c, int64_t k)
{
    return lrbi_oracle_index_bits_ranked(m, n, r, c, k, NULL);
}

/* The "binary" format of Fig. 1 / Table 1: one bit per weight. */
uint64_t lrbi_oracle_dense_bits(int64_t m, int64_t n)
{
    if (m <= 0 || n <= 0) return 0;
    return (uint64_t)m * (uint64_t)n;
}

/* Number of kept weights in a decoded mask. */
uint64_t lrbi_oracle_popcount(int64_t m, int64_t n, const uint8_t *M)
{
    uint64_t cnt = 0;
    for (int64_t e = 0; e < m * n; ++e) cnt += (M[e] != 0);
    return cnt;
}

/* CSR index size under the builder's own accounting (the paper prints CSR
 * sizes in Tables 1 and 3 but not the formula; parity unpinned):
 * one column index per kept weight plus m+1 row pointers. */
uint64_t lrbi_oracle_csr_bits(uint64_t nnz, int64_t m, int idx_bits, int ptr_bits)
{
    return nnz * (uint64_t)idx_bits + (uint64_t)(m + 1) * (uint64_t)ptr_bits;
}

/* Algorithm 1, the step "convert (M_p, M_z) into (I_p, I_z)" (Sec. 2.1): a factor entry
 * becomes 1 when it reaches the threshold, (I_p)_{i,l} = 1 iff (M_p)_{i,l} >= T_p, and the
 * same for I_z with T_z.  Every tile has its own pair of thresholds (the algorithm runs per
 * matrix, and a tiled layer is factorised tile by tile, Sec. 3.1).
 *   Mp [T][r][k], Mz [T][k][c] single precision; Tp, Tz [T]. */
int lrbi_oracle_threshold(int64_t T, int64_t r, int64_t c, int64_t k, const float *Mp, const float *Mz,
                          const float *Tp, const float *Tz, uint8_t *Ip01, uint8_t *Iz01)
{
    if (T <= 0 || r <= 0 || c <= 0 || k <= 0) return -1;
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t i = 0; i < r; ++i)
            for (int64_t l = 0; l < k; ++l)
                Ip01[(t * r + i) * k + l] = (Mp[(t * r + i) * k + l] >= Tp[t]) ? 1 : 0;
        for (int64_t l = 0; l < k; ++l)
            for (int64_t j = 0; j < c; ++j)
                Iz01[(t * k + l) * c + j] = (Mz[(t * k + l) * c + j] >= Tz[t]) ? 1 : 0;
    }
    return 0;
}

/* Algorithm 1, what is measured for one candidate pair of thresholds (Sec. 2.1), per tile:
 *   kept[t] = number of ones of I_a in the tile (S_a = 1 - kept / (r c)),
 *   cost[t] = sum of M_{i,j} over the tile's entries with I_{i,j} = 1 and (I_a)_{i,j} = 0
 *   (the part of an edge tile inside the matrix),
 * where I is the magnitude-pruning mask I_{i,j} = 1 iff |W_{i,j}| >= w_threshold (Eq. 1 -> Eq. 2),
 * I_a (the argument M here) the decoded mask of the candidate factors, and M_{i,j} the magnitude as the
 * factorisation saw it: Sec. 3.2 pre-processes the magnitudes and keeps this definition of the cost, so
 * method 1: |W|, method 2: |W|^2, method 3: amplify |W| where |W| >= w_threshold and |W| elsewhere.
 * Sums in double, row-major order. */
int lrbi_oracle_candidate_cost(int64_t m, int64_t n, int64_t r, int64_t c, const double *W, double w_threshold,
                               int method, double amplify, const uint8_t *M, uint64_t *kept, double *cost)
{
    if (m <= 0 || n <= 0 || r <= 0 || c <= 0 || method < 1 || method > 3) return -1;
    const int64_t tile_cols = (n + c - 1) / c;
    for (int64_t ti = 0; ti < (m + r - 1) / r; ++ti) {
        for (int64_t tj = 0; tj < tile_cols; ++tj) {
            uint64_t ones = 0;
            double sum = 0.0;
            for (int64_t i = 0; i < r && ti * r + i < m; ++i) {
                for (int64_t j = 0; j < c && tj * c + j < n; ++j) {
                    const int64_t at = (ti * r + i) * n + (tj * c + j);
                    const double mag = W[at] < 0.0 ? -W[at] : W[at];
                    if (M[at]) ones += 1;
                    double manipulated = mag;
                    if (method == 2) manipulated = mag * mag;
                    if (method == 3 && mag >= w_threshold) manipulated = mag * amplify;
                    if (mag >= w_threshold && !M[at]) sum += manipulated;
                }
            }
            kept[ti * tile_cols + tj] = ones;
            cost[ti * tile_cols + tj] = sum;
        }
    }
    return 0;
}
