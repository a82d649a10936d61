/*
 * CPU oracle for CLEAR local attention (arXiv 2412.16112).  TEST INFRASTRUCTURE ONLY:
 * this file is the slow, plain definition the GPU library is checked against.  Only the
 * tests, the smoke check and the bench's cpu_baseline leg may call it.  It shares no code
 * with the HIP path and is never tuned.
 *
 * What it computes, per batch item and head independently, in fp64:
 *   - the attention mask of Eq. 3 (Sec. 3.2): M[i][j] = 1 iff query i is a text token, or key j
 *     is a text token, or the squared Euclidean distance between the two image tokens on the
 *     gridH x gridW raster is strictly below r^2.  Text tokens come first (Eq. 3 tests
 *     i <= n_text with 1-based indices, i.e. i < n_text 0-based); image token (y, x) is row
 *     n_text + y*gridW + x.  The window is cut off at the image border (no wrap, no shift):
 *     this is the only border rule that reproduces the FLOP counts printed in Tables 2, 3, 7.
 *   - softmax attention of Eq. 1 (Sec. 2) restricted to the pairs with M = 1:
 *     O[i] = sum_j softmax_j(q_i . k_j / sqrt(d)) v_j.
 * Every row loops over ALL N key columns and tests M: no tiling, no window enumeration, no
 * reordering beyond that definition.
 *
 * Pins (tests/test_oracle_pins.py): FLOP counts 4*sum(M)*c printed in Tables 2, 3 and 7,
 * a lattice-point closed form, a pure-Python triple loop, the full-attention special case
 * against a library softmax, probability rows summing to one, one-hot V read-out of the
 * probability matrix, key-shift invariance, the r = 1 / no-text identity, transpose symmetry.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/*
 * Which local mask the image-image pairs follow.  0: the disc of Eq. 3 (CLEAR; the default).  The other two
 * are the sparse-attention variants the paper compares with, kept under the same text rule:
 * 1: square window, |dx| < r and |dy| < r (neighbourhood attention, window cut off at the border);
 * 2: Swin windows: both tokens in the same r x r cell of the partition whose origin is moved up and left
 *    by `shift` tokens;
 * 3: strided attention (appendix on the compared attentions): key j is kept when its offset from the query,
 *    taken modulo r on each axis (non-negative remainder), equals (r_x, r_y) = (l % r, (l / r) % r), where the
 *    layer index l travels in `shift`.  Reading: the offset is key minus query, and l / r wraps modulo r for
 *    layers beyond r^2 (the paper writes r_y = l // r and says nothing about either point).
 * A process-wide setting (set it, call the oracle, set it back): every function below goes through oracle_mask.
 */
static int g_mask_kind = 0, g_mask_shift = 0;
void oracle_set_mask(int kind, int shift) { g_mask_kind = kind; g_mask_shift = shift; }

/* Eq. 3 (or the variant selected above), 0-based.  Returns 1 when query row i may attend to key column j. */
int oracle_mask(int64_t i, int64_t j, int n_text, int gridH, int gridW, int r)
{
    (void)gridH;
    if (i < n_text || j < n_text) return 1;
    int pi = (int)(i - n_text), pj = (int)(j - n_text); /* raster index of the two image tokens */
    int yi = pi / gridW, xi = pi % gridW;
    int yj = pj / gridW, xj = pj % gridW;
    int64_t dx = xi - xj, dy = yi - yj;
    if (g_mask_kind == 1) return (llabs(dx) < r && llabs(dy) < r) ? 1 : 0;
    if (g_mask_kind == 2)
        return ((yi + g_mask_shift) / r == (yj + g_mask_shift) / r && (xi + g_mask_shift) / r == (xj + g_mask_shift) / r) ? 1 : 0;
    if (g_mask_kind == 3) {
        int rx = g_mask_shift % r, ry = (g_mask_shift / r) % r;
        int mx = (int)(((xj - xi) % r + r) % r), my = (int)(((yj - yi) % r + r) % r);
        return (mx == rx && my == ry) ? 1 : 0;
    }
    return (dx * dx + dy * dy < (int64_t)r * r) ? 1 : 0;
}

/* Number of keys row i attends to: a loop over every column. */
int64_t oracle_row_count(int64_t i, int n_text, int gridH, int gridW, int r)
{
    int64_t N = (int64_t)n_text + (int64_t)gridH * gridW, c = 0;
    for (int64_t j = 0; j < N; ++j) c += oracle_mask(i, j, n_text, gridH, gridW, r);
    return c;
}

/* sum(M) over the whole N x N mask, by visiting every (i, j). */
uint64_t oracle_mask_count(int n_text, int gridH, int gridW, int r)
{
    int64_t N = (int64_t)n_text + (int64_t)gridH * gridW;
    uint64_t total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int64_t i = 0; i < N; ++i) total += (uint64_t)oracle_row_count(i, n_text, gridH, gridW, r);
    return total;
}

/* Dense 0/1 mask, row-major N x N bytes (small N only). */
void oracle_mask_dense(int n_text, int gridH, int gridW, int r, uint8_t* M)
{
    int64_t N = (int64_t)n_text + (int64_t)gridH * gridW;
    for (int64_t i = 0; i < N; ++i)
        for (int64_t j = 0; j < N; ++j) M[i * N + j] = (uint8_t)oracle_mask(i, j, n_text, gridH, gridW, r);
}

/*
 * Attention for selected rows of ONE (batch, head) slice.
 *   Q, K, V : [N][d] fp64 row-major (bf16 / fp32 inputs widened exactly by the caller).
 *   rows    : n_rows query indices in [0, N).
 *   O       : [n_rows][d] fp64 out.   m_out, l_out (optional, may be NULL): per-row max logit and
 *             softmax denominator; cnt_out (optional): number of attended keys.
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int oracle_attention_rows(const double* Q, const double* K, const double* V, const int64_t* rows,
                          int64_t n_rows, int n_text, int gridH, int gridW, int d, int r, double* O,
                          double* m_out, double* l_out, int64_t* cnt_out)
{
    if (!Q || !K || !V || !rows || !O || d < 1 || r < 1 || gridH < 1 || gridW < 1 || n_text < 0) return -1;
    const int64_t N = (int64_t)n_text + (int64_t)gridH * gridW;
    const double scale = 1.0 / sqrt((double)d); /* Eq. 1: logits divided by sqrt(c) */
    int fail = 0;
#pragma omp parallel
    {
        double* s = (double*)malloc(sizeof(double) * (size_t)N);
        if (!s) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t t = 0; t < n_rows; ++t) {
            if (!s) continue;
            const int64_t i = rows[t];
            const double* q = Q + i * d;
            double m = -INFINITY;
            int64_t cnt = 0;
            for (int64_t j = 0; j < N; ++j) {
                if (!oracle_mask(i, j, n_text, gridH, gridW, r)) { s[j] = -INFINITY; continue; }
                const double* k = K + j * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += q[c] * k[c];
                s[j] = acc * scale;
                if (s[j] > m) m = s[j];
                ++cnt;
            }
            double l = 0.0;
            double* o = O + t * d;
            for (int c = 0; c < d; ++c) o[c] = 0.0;
            for (int64_t j = 0; j < N; ++j) {
                if (!oracle_mask(i, j, n_text, gridH, gridW, r)) continue;
                const double p = exp(s[j] - m);
                l += p;
                const double* v = V + j * d;
                for (int c = 0; c < d; ++c) o[c] += p * v[c];
            }
            for (int c = 0; c < d; ++c) o[c] /= l;
            if (m_out) m_out[t] = m;
            if (l_out) l_out[t] = l;
            if (cnt_out) cnt_out[t] = cnt;
        }
        free(s);
    }
    return fail ? -1 : 0;
}

/*
 * Backward pass of the same operator (needed to train the attention layers, Sec. 3.3; the gradients of
 * Eq. 1 under the mask of Eq. 3 are not printed in the paper: they follow from differentiating it).
 * With s_ij = q_i.k_j / sqrt(d), p_ij = softmax_j(s_ij) over the keys with M_ij = 1, O_i = sum_j p_ij v_j
 * and an upstream gradient dO:
 *     dV_j = sum_i p_ij dO_i
 *     dp_ij = dO_i . v_j,   delta_i = sum_j p_ij dp_ij  (= dO_i . O_i),   ds_ij = p_ij (dp_ij - delta_i)
 *     dQ_i = sum_j ds_ij k_j / sqrt(d),      dK_j = sum_i ds_ij q_i / sqrt(d)
 * Everything below is these sums written out in fp64, one (i, j) pair at a time, over ALL N columns
 * (or rows) with the mask tested per pair.
 *
 * Per-row statistics of the forward pass for the given rows: m (max logit), l (sum of exp(s - m)) and
 * delta (as defined above).  Returns 0 or -1.
 */
int oracle_row_stats(const double* Q, const double* K, const double* V, const double* dO, const int64_t* rows,
                     int64_t n_rows, int n_text, int gridH, int gridW, int d, int r, double* m_out,
                     double* l_out, double* delta_out)
{
    if (!Q || !K || !V || !dO || !rows || !m_out || !l_out || !delta_out || d < 1 || r < 1) return -1;
    const int64_t N = (int64_t)n_text + (int64_t)gridH * gridW;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t i = rows[t];
        const double* q = Q + i * d;
        const double* g = dO + i * d;
        double m = -INFINITY;
        for (int64_t j = 0; j < N; ++j) {
            if (!oracle_mask(i, j, n_text, gridH, gridW, r)) continue;
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += q[c] * K[j * d + c];
            if (acc * scale > m) m = acc * scale;
        }
        double l = 0.0, num = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            if (!oracle_mask(i, j, n_text, gridH, gridW, r)) continue;
            double acc = 0.0, dp = 0.0;
            for (int c = 0; c < d; ++c) { acc += q[c] * K[j * d + c]; dp += g[c] * V[j * d + c]; }
            const double e = exp(acc * scale - m);
            l += e;
            num += e * dp;
        }
        m_out[t] = m;
        l_out[t] = l;
        delta_out[t] = num / l;
    }
    return 0;
}

/* dQ for the given query rows: [n_rows][d]. */
int oracle_backward_dq_rows(const double* Q, const double* K, const double* V, const double* dO, const int64_t* rows,
                            int64_t n_rows, int n_text, int gridH, int gridW, int d, int r, double* dQ)
{
    if (!dQ) return -1;
    const int64_t N = (int64_t)n_text + (int64_t)gridH * gridW;
    const double scale = 1.0 / sqrt((double)d);
    double* m = (double*)malloc(sizeof(double) * (size_t)(3 * n_rows + 1));
    if (!m) return -1;
    double *l = m + n_rows, *delta = l + n_rows;
    if (oracle_row_stats(Q, K, V, dO, rows, n_rows, n_text, gridH, gridW, d, r, m, l, delta) != 0) { free(m); return -1; }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t i = rows[t];
        const double* q = Q + i * d;
        const double* g = dO + i * d;
        double* out = dQ + t * d;
        for (int c = 0; c < d; ++c) out[c] = 0.0;
        for (int64_t j = 0; j < N; ++j) {
            if (!oracle_mask(i, j, n_text, gridH, gridW, r)) continue;
            double acc = 0.0, dp = 0.0;
            for (int c = 0; c < d; ++c) { acc += q[c] * K[j * d + c]; dp += g[c] * V[j * d + c]; }
            const double p = exp(acc * scale - m[t]) / l[t];
            const double ds = p * (dp - delta[t]);
            for (int c = 0; c < d; ++c) out[c] += ds * K[j * d + c] * scale;
        }
    }
    free(m);
    return 0;
}

/*
 * dK and dV for the given key columns: [n_cols][d] each.  Every query row i is visited for every column
 * (mask tested per pair); the statistics of the rows that attend to at least one of the columns are
 * computed first.
 */
int oracle_backward_dkv_cols(const double* Q, const double* K, const double* V, const double* dO, const int64_t* cols,
                             int64_t n_cols, int n_text, int gridH, int gridW, int d, int r, double* dK, double* dV)
{
    if (!Q || !K || !V || !dO || !cols || !dK || !dV || d < 1 || r < 1) return -1;
    const int64_t N = (int64_t)n_text + (int64_t)gridH * gridW;
    const double scale = 1.0 / sqrt((double)d);
    /* rows that see any of the columns */
    int64_t* need = (int64_t*)malloc(sizeof(int64_t) * (size_t)(N + 1));
    int64_t* slot = (int64_t*)malloc(sizeof(int64_t) * (size_t)(N + 1));
    if (!need || !slot) { free(need); free(slot); return -1; }
    int64_t n_need = 0;
    for (int64_t i = 0; i < N; ++i) {
        int any = 0;
        for (int64_t t = 0; t < n_cols && !any; ++t) any = oracle_mask(i, cols[t], n_text, gridH, gridW, r);
        slot[i] = any ? n_need : -1;
        if (any) need[n_need++] = i;
    }
    double* m = (double*)malloc(sizeof(double) * (size_t)(3 * n_need + 1));
    if (!m) { free(need); free(slot); return -1; }
    double *l = m + n_need, *delta = l + n_need;
    int rc = oracle_row_stats(Q, K, V, dO, need, n_need, n_text, gridH, gridW, d, r, m, l, delta);
    if (rc == 0) {
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t t = 0; t < n_cols; ++t) {
            const int64_t j = cols[t];
            double* ok = dK + t * d;
            double* ov = dV + t * d;
            for (int c = 0; c < d; ++c) { ok[c] = 0.0; ov[c] = 0.0; }
            for (int64_t i = 0; i < N; ++i) {
                if (!oracle_mask(i, j, n_text, gridH, gridW, r)) continue;
                const int64_t u = slot[i];
                double acc = 0.0, dp = 0.0;
                for (int c = 0; c < d; ++c) { acc += Q[i * d + c] * K[j * d + c]; dp += dO[i * d + c] * V[j * d + c]; }
                const double p = exp(acc * scale - m[u]) / l[u];
                const double ds = p * (dp - delta[u]);
                for (int c = 0; c < d; ++c) {
                    ov[c] += p * dO[i * d + c];
                    ok[c] += ds * Q[i * d + c] * scale;
                }
            }
        }
    }
    free(m); free(need); free(slot);
    return rc;
}

/*
 * Reference tile schedule by brute force over the element mask (image tokens only; text keys
 * are attended by every query and are not part of the schedule).
 * Query tiles are qth x qtw patches, key tiles kth x ktw patches, both aligned to the grid
 * origin, numbered row-major; edge tiles hang over the border.
 *   cnt[qt * n_kt + kt] = number of (query, key) element pairs, both inside the grid, with M = 1.
 * A pair of tiles is LISTED iff cnt > 0 and FULL iff cnt == qth*qtw*kth*ktw (every slot pair is
 * inside the grid and unmasked).  The caller derives the CSR from cnt.
 */
void oracle_tile_pair_counts(int gridH, int gridW, int r, int qth, int qtw, int kth, int ktw, int32_t* cnt)
{
    const int nqx = (gridW + qtw - 1) / qtw, nqy = (gridH + qth - 1) / qth;
    const int nkx = (gridW + ktw - 1) / ktw, nky = (gridH + kth - 1) / kth;
    const int64_t n_kt = (int64_t)nkx * nky;
    memset(cnt, 0, sizeof(int32_t) * (size_t)((int64_t)nqx * nqy * n_kt));
    const int64_t n_img = (int64_t)gridH * gridW;
#pragma omp parallel for schedule(dynamic, 1)
    for (int qty = 0; qty < nqy; ++qty) { /* rows of query tiles write disjoint parts of cnt */
        for (int qy = qty * qth; qy < (qty + 1) * qth && qy < gridH; ++qy)
            for (int qx = 0; qx < gridW; ++qx) {
                int32_t* row = cnt + ((int64_t)qty * nqx + qx / qtw) * n_kt;
                const int64_t i = (int64_t)qy * gridW + qx;
                for (int64_t j = 0; j < n_img; ++j)
                    if (oracle_mask(i, j, 0, gridH, gridW, r)) {
                        const int ky = (int)(j / gridW), kx = (int)(j % gridW);
                        row[(int64_t)(ky / kth) * nkx + kx / ktw] += 1;
                    }
            }
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
