/*
 * CPU oracle for the DGQ quantized-inference path (arXiv 2501.04304).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded C that follows the
 * paper's definitions step by step; the tests compare the HIP library against
 * it.  It shares no code, header, table or constant with the HIP path, and the
 * product never calls it.  Compile with
 *     gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 * (no FMA contraction, so every float/double expression below is evaluated
 * exactly as written).
 *
 * What each function follows:
 *   linear quantizer / dequantizer ............ Section 3.1, first equation
 *   log2 quantizer / dequantizer .............. Section 3.1, second equation
 *   softmax attention score ................... Section 3.2, attention equation
 *   variability metric D_d and d* ............. Section 3.3, D_d and argmax equations
 *   K-means grouping by range ................. Section 3.3, paragraph after d*
 *   group scale s_k and zero-point z_k ........ Section 3.3, s_k / z_k equation
 *   cross-attention codes and split product ... Section 3.3, A^q / A-hat V-hat equations
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - rounding is round-half-to-even;
 *   - x/s is evaluated as (x - z) * (1.0f / s) in fp32 with a float offset
 *     z = min x subtracted before scaling (the s_k/z_k equation's z is a float);
 *   - the divisor of s_k is 2^b as printed, so x = max is clipped to 2^b - 1;
 *   - "K groups by range using K-means" is an exact 1-D 2-means on the widths
 *     (max - min) that separates an outlier cluster, followed by cutting each
 *     cluster, sorted by width, into blocks of G channels;
 *   - both outlier kinds are handled at once: P pixel classes x NG channel
 *     groups, one (s, z) per cell; the paper's single-dimension cases are the
 *     degenerate grids P = 1 and NG = 1;
 *   - the attention scale s is one value per prompt (batch element), taken
 *     over all heads and queries, keys 1..nk-1.
 *
 * Parity pins live in tests/test_oracle_*.py (closed forms, brute force on
 * tiny inputs, invariants, library routines).  Dataset metrics (FID/IS/CLIP)
 * are parity unpinned: the artefacts they need are not available.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Exact 1-D 2-means (used for pixel classes and for the channel outlier set) */
/* ------------------------------------------------------------------------- */

typedef struct {
    float v;
    int64_t i;
} dgqo_kv;

static int dgqo_kv_cmp(const void *a, const void *b)
{
    const dgqo_kv *x = (const dgqo_kv *)a, *y = (const dgqo_kv *)b;
    if (x->v < y->v) return -1;
    if (x->v > y->v) return 1;
    if (x->i < y->i) return -1;
    if (x->i > y->i) return 1;
    return 0;
}

/*
 * Sort v ascending (ties by index).  Among the splits "first k sorted values |
 * the rest" with v[k-1] < v[k], choose the one with the smallest within-cluster
 * sum of squares
 *     SSE(k) = (S2_L - S_L^2 / k) + (S2_R - S_R^2 / (n - k)),
 * prefix sums taken sequentially in sorted order in double, S_R = S_tot - S_L.
 * Ties go to the smallest k.  The threshold is the midpoint of the two cluster
 * means, rounded to fp32 and clamped into [v[k-1], nextbelow(v[k])] so that
 * "v > tau" reproduces the split on the data itself.
 *
 * order_out (nullable): the sorted index order.  Returns the size of the lower
 * cluster (n when all values are equal: no split, tau = +inf).
 */
int64_t dgqo_two_means(const float *v, int64_t n, float *tau_out, int64_t *order_out)
{
    dgqo_kv *a = (dgqo_kv *)malloc(sizeof(dgqo_kv) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) {
        a[i].v = v[i];
        a[i].i = i;
    }
    qsort(a, (size_t)n, sizeof(dgqo_kv), dgqo_kv_cmp);
    if (order_out)
        for (int64_t i = 0; i < n; ++i) order_out[i] = a[i].i;
    if (n < 2 || !(a[0].v < a[n - 1].v)) {
        *tau_out = INFINITY;
        free(a);
        return n;
    }
    double s_tot = 0.0, s2_tot = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double x = (double)a[i].v;
        s_tot = s_tot + x;
        s2_tot = s2_tot + x * x;
    }
    double s_l = 0.0, s2_l = 0.0, best = 0.0;
    int64_t best_k = -1;
    for (int64_t k = 1; k < n; ++k) {
        double x = (double)a[k - 1].v;
        s_l = s_l + x;
        s2_l = s2_l + x * x;
        if (!(a[k - 1].v < a[k].v)) continue;
        double s_r = s_tot - s_l;
        double s2_r = s2_tot - s2_l;
        double sse_l = s2_l - (s_l * s_l) / (double)k;
        double sse_r = s2_r - (s_r * s_r) / (double)(n - k);
        double sse = sse_l + sse_r;
        if (best_k < 0 || sse < best) {
            best = sse;
            best_k = k;
        }
    }
    /* recompute the left sum for the chosen split */
    double sl = 0.0;
    for (int64_t i = 0; i < best_k; ++i) sl = sl + (double)a[i].v;
    double mean_l = sl / (double)best_k;
    double mean_r = (s_tot - sl) / (double)(n - best_k);
    float tau = (float)(0.5 * (mean_l + mean_r));
    float lo = a[best_k - 1].v;
    float hi = nextafterf(a[best_k].v, -INFINITY);
    if (tau < lo) tau = lo;
    if (tau > hi) tau = hi;
    *tau_out = tau;
    free(a);
    return best_k;
}

/* ------------------------------------------------------------------------- */
/* Calibration: pixel classes, D_d, channel groups, cell parameters          */
/* ------------------------------------------------------------------------- */

static int32_t round_up(int32_t a, int32_t m) { return (a + m - 1) / m * m; }

/*
 * x: calibration activations [rows, C] (one row per pixel, batch flattened).
 * act_bits b, G regular group size, P in {1,2} pixel classes, granule: every
 * group is padded to a multiple of it (padded positions carry no channel).
 *
 * Outputs (caller allocates; ng_cap = capacity in groups, kp_cap in positions):
 *   scal[0]=NG, [1]=K' (padded length), [2]=number of outlier channels,
 *   [3]=number of regular groups, [4]=d* (0 channel, 1 pixel), [5]=class-1 rows
 *   perm[K']   original channel at padded position j, -1 for padding
 *   goff[NG+1] padded start of each group;  glen[NG] channels in the group
 *   tau_pix    row-width threshold (+inf if P == 1 or no split)
 *   s, z, inv_s  [2][ng_cap] cell tables (class-major, stride ng_cap)
 *   D[0]=D_channel, D[1]=D_pixel
 *   row_class[rows] (nullable) classes of the calibration rows
 * Returns 0, or -1 if a capacity is too small.
 */
int dgqo_calibrate(const float *x, int64_t rows, int32_t C, int32_t act_bits,
                   int32_t G, int32_t P, int32_t granule, int32_t ng_cap,
                   int32_t kp_cap, int32_t *scal, int32_t *perm, int32_t *goff,
                   int32_t *glen, float *tau_pix, float *s, float *z,
                   float *inv_s, double *D, uint8_t *row_class)
{
    float *rmx = (float *)malloc(sizeof(float) * (size_t)rows);
    float *rmn = (float *)malloc(sizeof(float) * (size_t)rows);
    float *rw = (float *)malloc(sizeof(float) * (size_t)rows);
    uint8_t *cls = (uint8_t *)malloc((size_t)rows);
    float *cmx_all = (float *)malloc(sizeof(float) * (size_t)C);
    float *cmn_all = (float *)malloc(sizeof(float) * (size_t)C);
    float *cmx0 = (float *)malloc(sizeof(float) * (size_t)C);
    float *cmn0 = (float *)malloc(sizeof(float) * (size_t)C);
    float *cw = (float *)malloc(sizeof(float) * (size_t)C);
    int64_t *order = (int64_t *)malloc(sizeof(int64_t) * (size_t)C);
    int rc = 0;

    /* per-pixel range over all channels */
    for (int64_t r = 0; r < rows; ++r) {
        float mx = -INFINITY, mn = INFINITY;
        for (int32_t c = 0; c < C; ++c) {
            float v = x[r * C + c];
            if (v > mx) mx = v;
            if (v < mn) mn = v;
        }
        rmx[r] = mx;
        rmn[r] = mn;
        rw[r] = mx - mn;
    }
    /* pixel classes: nearest of two centroids on the row widths == threshold */
    float tau = INFINITY;
    if (P == 2) dgqo_two_means(rw, rows, &tau, NULL);
    int64_t n1 = 0;
    for (int64_t r = 0; r < rows; ++r) {
        cls[r] = (uint8_t)(rw[r] > tau);
        n1 += cls[r];
    }
    *tau_pix = tau;
    if (row_class) memcpy(row_class, cls, (size_t)rows);

    /* per-channel range over all rows (for D_d) and over class-0 rows (groups) */
    for (int32_t c = 0; c < C; ++c) {
        cmx_all[c] = cmx0[c] = -INFINITY;
        cmn_all[c] = cmn0[c] = INFINITY;
    }
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t c = 0; c < C; ++c) {
            float v = x[r * C + c];
            if (v > cmx_all[c]) cmx_all[c] = v;
            if (v < cmn_all[c]) cmn_all[c] = v;
            if (!cls[r]) {
                if (v > cmx0[c]) cmx0[c] = v;
                if (v < cmn0[c]) cmn0[c] = v;
            }
        }

    /* D_d = (max_i a_i^max - min_i a_i^max) + (max_i a_i^min - min_i a_i^min) */
    {
        double mxmx = -INFINITY, mnmx = INFINITY, mxmn = -INFINITY, mnmn = INFINITY;
        for (int32_t c = 0; c < C; ++c) {
            if (cmx_all[c] > mxmx) mxmx = cmx_all[c];
            if (cmx_all[c] < mnmx) mnmx = cmx_all[c];
            if (cmn_all[c] > mxmn) mxmn = cmn_all[c];
            if (cmn_all[c] < mnmn) mnmn = cmn_all[c];
        }
        D[0] = (mxmx - mnmx) + (mxmn - mnmn);
        mxmx = -INFINITY; mnmx = INFINITY; mxmn = -INFINITY; mnmn = INFINITY;
        for (int64_t r = 0; r < rows; ++r) {
            if (rmx[r] > mxmx) mxmx = rmx[r];
            if (rmx[r] < mnmx) mnmx = rmx[r];
            if (rmn[r] > mxmn) mxmn = rmn[r];
            if (rmn[r] < mnmn) mnmn = rmn[r];
        }
        D[1] = (mxmx - mnmx) + (mxmn - mnmn);
    }
    int32_t dstar = (D[1] > D[0]) ? 1 : 0;

    /* channel groups: 2-means on class-0 widths, then blocks of G per cluster */
    for (int32_t c = 0; c < C; ++c) cw[c] = cmx0[c] - cmn0[c];
    float tau_c;
    int64_t n_reg = dgqo_two_means(cw, C, &tau_c, order);
    int32_t n_out = (int32_t)(C - n_reg);
    /* `order` is already sorted by (width, index); the lower cluster is its
       first n_reg entries, so (cluster, width, index) order == `order`. */
    int32_t ng = 0, pos = 0, n_reg_groups = 0;
    for (int pass = 0; pass < 2 && rc == 0; ++pass) {
        int64_t beg = pass == 0 ? 0 : n_reg;
        int64_t end = pass == 0 ? n_reg : C;
        for (int64_t b0 = beg; b0 < end; b0 += G) {
            int64_t len = end - b0 < G ? end - b0 : G;
            int32_t plen = round_up((int32_t)len, granule);
            if (ng >= ng_cap || pos + plen > kp_cap) { rc = -1; break; }
            goff[ng] = pos;
            glen[ng] = (int32_t)len;
            for (int32_t j = 0; j < plen; ++j)
                perm[pos + j] = j < len ? (int32_t)order[b0 + j] : -1;
            pos += plen;
            ++ng;
            if (pass == 0) ++n_reg_groups;
        }
    }
    if (rc == 0) {
        goff[ng] = pos;
        /* cell parameters: s = (max - min) / 2^b, z = min */
        float levels = (float)(1 << act_bits);
        for (int32_t p = 0; p < 2; ++p)
            for (int32_t g = 0; g < ng; ++g) {
                float mx = -INFINITY, mn = INFINITY;
                int64_t cnt = 0;
                for (int64_t r = 0; r < rows; ++r) {
                    if (cls[r] != p) continue;
                    ++cnt;
                    for (int32_t j = 0; j < glen[g]; ++j) {
                        float v = x[r * C + perm[goff[g] + j]];
                        if (v > mx) mx = v;
                        if (v < mn) mn = v;
                    }
                }
                float sc, zp;
                if (cnt == 0) { /* empty class: reuse class 0's cell */
                    sc = s[g];
                    zp = z[g];
                } else {
                    sc = (mx - mn) / levels;
                    zp = mn;
                    if (!(mx > mn)) sc = 1.0f;
                }
                s[p * ng_cap + g] = sc;
                z[p * ng_cap + g] = zp;
                inv_s[p * ng_cap + g] = 1.0f / sc;
            }
        scal[0] = ng;
        scal[1] = pos;
        scal[2] = n_out;
        scal[3] = n_reg_groups;
        scal[4] = dstar;
        scal[5] = (int32_t)n1;
    }
    free(rmx); free(rmn); free(rw); free(cls); free(cmx_all); free(cmn_all);
    free(cmx0); free(cmn0); free(cw); free(order);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Exact 1-D K-means and the single-dimension grouping of Section 3.3        */
/* ------------------------------------------------------------------------- */

/*
 * K-means of a 1-D sample, solved exactly.  In one dimension an optimal
 * clustering consists of intervals of the sorted sample, so the minimum of the
 * within-cluster sum of squares over all partitions into k intervals is found
 * by dynamic programming over the sorted values a[0..n):
 *     cost(i, j) = (S2[j] - S2[i]) - (S[j] - S[i])^2 / (j - i)     cluster a[i..j)
 *     best[1][j] = cost(0, j)
 *     best[k][j] = min_{i} best[k-1][i] + cost(i, j),  a[i-1] < a[i] (equal values
 *                  stay together), first minimum wins
 * with S, S2 the running sums of a and a^2 in double, taken in sorted order
 * (ties in the sort by index).  k = min(K, number of distinct values).
 *   bounds[0..k]  cluster c is sorted positions [bounds[c], bounds[c+1])
 *   taus[0..k-1)  threshold between clusters c and c+1: midpoint of their means,
 *                 rounded to fp32 and clamped into [a[b-1], nextbelow(a[b])], so
 *                 that "number of taus below v" reproduces the clusters
 *   order[n]      (nullable) sorted index order
 * Returns k.
 */
int32_t dgqo_k_means(const float *v, int64_t n, int32_t K, int64_t *bounds, float *taus,
                     int64_t *order_out)
{
    dgqo_kv *a = (dgqo_kv *)malloc(sizeof(dgqo_kv) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) {
        a[i].v = v[i];
        a[i].i = i;
    }
    qsort(a, (size_t)n, sizeof(dgqo_kv), dgqo_kv_cmp);
    if (order_out)
        for (int64_t i = 0; i < n; ++i) order_out[i] = a[i].i;
    int64_t distinct = n > 0 ? 1 : 0;
    for (int64_t i = 1; i < n; ++i) distinct += a[i - 1].v < a[i].v;
    int32_t k_use = (int32_t)(distinct < K ? distinct : K);
    if (k_use < 1) k_use = 1;
    double *S = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    double *S2 = (double *)malloc(sizeof(double) * (size_t)(n + 1));
    S[0] = 0.0;
    S2[0] = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double x = (double)a[i].v;
        S[i + 1] = S[i] + x;
        S2[i + 1] = S2[i] + x * x;
    }
    /* best[k][j], from[k][j] for k = 1..k_use, j = 0..n; unreachable = negative from */
    double *best = (double *)malloc(sizeof(double) * (size_t)(k_use + 1) * (size_t)(n + 1));
    int64_t *from = (int64_t *)malloc(sizeof(int64_t) * (size_t)(k_use + 1) * (size_t)(n + 1));
#define AT(k, j) ((size_t)(k) * (size_t)(n + 1) + (size_t)(j))
    for (int32_t k = 0; k <= k_use; ++k)
        for (int64_t j = 0; j <= n; ++j) from[AT(k, j)] = -1;
    for (int64_t j = 1; j <= n; ++j) {
        double d = S[j] - S[0];
        best[AT(1, j)] = (S2[j] - S2[0]) - (d * d) / (double)j;
        from[AT(1, j)] = 0;
    }
    for (int32_t k = 2; k <= k_use; ++k)
        for (int64_t j = k; j <= n; ++j) {
            int64_t arg = -1;
            double bv = 0.0;
            for (int64_t i = k - 1; i < j; ++i) {
                if (from[AT(k - 1, i)] < 0) continue;      /* i values cannot form k-1 clusters */
                if (!(a[i - 1].v < a[i].v)) continue;      /* no cut between equal values */
                double d = S[j] - S[i];
                double c = (S2[j] - S2[i]) - (d * d) / (double)(j - i);
                double t = best[AT(k - 1, i)] + c;
                if (arg < 0 || t < bv) {
                    bv = t;
                    arg = i;
                }
            }
            if (arg >= 0) {
                best[AT(k, j)] = bv;
                from[AT(k, j)] = arg;
            }
        }
    bounds[k_use] = n;
    for (int32_t k = k_use; k >= 1; --k) bounds[k - 1] = from[AT(k, bounds[k])];
#undef AT
    for (int32_t c = 0; c + 1 < k_use; ++c) {
        int64_t b0 = bounds[c], b1 = bounds[c + 1], b2 = bounds[c + 2];
        double mean_l = (S[b1] - S[b0]) / (double)(b1 - b0);
        double mean_r = (S[b2] - S[b1]) / (double)(b2 - b1);
        float tau = (float)(0.5 * (mean_l + mean_r));
        float lo = a[b1 - 1].v;
        float hi = nextafterf(a[b1].v, -INFINITY);
        if (tau < lo) tau = lo;
        if (tau > hi) tau = hi;
        taus[c] = tau;
    }
    free(a); free(S); free(S2); free(best); free(from);
    return k_use;
}

/*
 * Grouping along ONE dimension (Section 3.3): D_d for d in {channel, pixel},
 * d* = argmax (dim < 0) or the given dimension (0 channel, 1 pixel); the vectors
 * of d* (channels: all rows of a column; pixels: all channels of a row) are
 * clustered into K groups by their range max - min with dgqo_k_means; every
 * group k gets s_k = (max x - min x) / 2^b (1 if max == min) and z_k = min x over
 * the calibration activations that belong to it.
 *   channel: one pixel class; group g = cluster g in ascending range, channels in
 *            (range, index) order, padded to the granule
 *   pixel:   one channel group (all channels in natural order, padded); class p
 *            of a row = number of taus below its range
 * Outputs as dgqo_calibrate, except: scal[6] = number of pixel classes P,
 * taus[P-1], tables s, z, inv_s [P][ng_cap] (class-major, stride ng_cap),
 * scal[2] = scal[3] = 0.
 */
int dgqo_calibrate_kmeans(const float *x, int64_t rows, int32_t C, int32_t act_bits,
                          int32_t K, int32_t dim, int32_t granule, int32_t ng_cap,
                          int32_t kp_cap, int32_t *scal, int32_t *perm, int32_t *goff,
                          int32_t *glen, float *taus, float *s, float *z, float *inv_s,
                          double *D, uint8_t *row_class)
{
    float *rmx = (float *)malloc(sizeof(float) * (size_t)rows);
    float *rmn = (float *)malloc(sizeof(float) * (size_t)rows);
    float *cmx = (float *)malloc(sizeof(float) * (size_t)C);
    float *cmn = (float *)malloc(sizeof(float) * (size_t)C);
    for (int32_t c = 0; c < C; ++c) {
        cmx[c] = -INFINITY;
        cmn[c] = INFINITY;
    }
    for (int64_t r = 0; r < rows; ++r) {
        float mx = -INFINITY, mn = INFINITY;
        for (int32_t c = 0; c < C; ++c) {
            float v = x[r * C + c];
            if (v > mx) mx = v;
            if (v < mn) mn = v;
            if (v > cmx[c]) cmx[c] = v;
            if (v < cmn[c]) cmn[c] = v;
        }
        rmx[r] = mx;
        rmn[r] = mn;
    }
    for (int pass = 0; pass < 2; ++pass) {
        const float *vmx = pass == 0 ? cmx : rmx, *vmn = pass == 0 ? cmn : rmn;
        int64_t cnt = pass == 0 ? C : rows;
        double mxmx = -INFINITY, mnmx = INFINITY, mxmn = -INFINITY, mnmn = INFINITY;
        for (int64_t i = 0; i < cnt; ++i) {
            if (vmx[i] > mxmx) mxmx = vmx[i];
            if (vmx[i] < mnmx) mnmx = vmx[i];
            if (vmn[i] > mxmn) mxmn = vmn[i];
            if (vmn[i] < mnmn) mnmn = vmn[i];
        }
        D[pass] = (mxmx - mnmx) + (mxmn - mnmn);
    }
    int32_t dstar = (D[1] > D[0]) ? 1 : 0;
    int32_t use = dim < 0 ? dstar : dim;
    const float levels = (float)(1 << act_bits);
    int rc = 0;
    int64_t bounds[65];
    if (K > 64) K = 64;
    if (use == 0) {
        /* channels clustered by range over all rows */
        float *cw = (float *)malloc(sizeof(float) * (size_t)C);
        int64_t *order = (int64_t *)malloc(sizeof(int64_t) * (size_t)C);
        float dummy[64];
        for (int32_t c = 0; c < C; ++c) cw[c] = cmx[c] - cmn[c];
        int32_t ng = dgqo_k_means(cw, C, K, bounds, dummy, order);
        int32_t pos = 0;
        for (int32_t g = 0; g < ng && rc == 0; ++g) {
            int32_t len = (int32_t)(bounds[g + 1] - bounds[g]);
            int32_t plen = round_up(len, granule);
            if (g >= ng_cap || pos + plen > kp_cap) { rc = -1; break; }
            goff[g] = pos;
            glen[g] = len;
            float mx = -INFINITY, mn = INFINITY;
            for (int32_t j = 0; j < plen; ++j) {
                int32_t c = j < len ? (int32_t)order[bounds[g] + j] : -1;
                perm[pos + j] = c;
                if (c >= 0) {
                    if (cmx[c] > mx) mx = cmx[c];
                    if (cmn[c] < mn) mn = cmn[c];
                }
            }
            float sc = (mx - mn) / levels;
            if (!(mx > mn)) sc = 1.0f;
            s[g] = sc;
            z[g] = mn;
            inv_s[g] = 1.0f / sc;
            pos += plen;
        }
        if (rc == 0) {
            goff[ng] = pos;
            scal[0] = ng;
            scal[1] = pos;
            scal[6] = 1;
            if (row_class) memset(row_class, 0, (size_t)rows);
        }
        scal[5] = 0;
        free(cw); free(order);
    } else {
        /* pixels clustered by range over all channels */
        float *rw = (float *)malloc(sizeof(float) * (size_t)rows);
        for (int64_t r = 0; r < rows; ++r) rw[r] = rmx[r] - rmn[r];
        int32_t P = dgqo_k_means(rw, rows, K, bounds, taus, NULL);
        int32_t plen = round_up(C, granule);
        if (ng_cap < 1 || plen > kp_cap) rc = -1;
        if (rc == 0) {
            goff[0] = 0;
            goff[1] = plen;
            glen[0] = C;
            for (int32_t j = 0; j < plen; ++j) perm[j] = j < C ? j : -1;
            float mx[64], mn[64];
            for (int32_t p = 0; p < P; ++p) {
                mx[p] = -INFINITY;
                mn[p] = INFINITY;
            }
            int64_t n_upper = 0;
            for (int64_t r = 0; r < rows; ++r) {
                int p = 0;
                for (int32_t k = 0; k + 1 < P; ++k) p += rw[r] > taus[k];
                if (row_class) row_class[r] = (uint8_t)p;
                n_upper += p > 0;
                if (rmx[r] > mx[p]) mx[p] = rmx[r];
                if (rmn[r] < mn[p]) mn[p] = rmn[r];
            }
            for (int32_t p = 0; p < P; ++p) {
                float sc = (mx[p] - mn[p]) / levels;
                if (!(mx[p] > mn[p])) sc = 1.0f;
                s[p * ng_cap] = sc;
                z[p * ng_cap] = mn[p];
                inv_s[p * ng_cap] = 1.0f / sc;
            }
            scal[0] = 1;
            scal[1] = plen;
            scal[5] = (int32_t)n_upper;
            scal[6] = P;
        }
        free(rw);
    }
    scal[2] = 0;
    scal[3] = 0;
    scal[4] = dstar;
    scal[7] = use;
    free(rmx); free(rmn); free(cmx); free(cmn);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Activation codes (linear quantizer with the cell's scale and offset)      */
/* ------------------------------------------------------------------------- */

/*
 * For every row: class p = number of thresholds below max - min (one threshold
 * tau_pix for two classes), decided on the run-time row;
 * for every real position j of group g: t = x - z[p,g]; u = t * inv_s[p,g];
 * q = clamp(rne(u), 0, 2^b - 1).  q is the code the paper defines (unsigned).
 *   q_out   [rows, K'] codes at permuted positions (0 at padding)
 *   cls_out [rows]
 *   xdq_out [rows, C]  (nullable) s*q + z in double, original channel order
 *   clip_out[rows, C]  (nullable) 1 where u < -0.5 or u > 2^b - 0.5
 */
void dgqo_quantize_act_multi(const float *x, int64_t rows, int32_t C, int32_t act_bits,
                             int32_t ng, int32_t ng_cap, const int32_t *perm,
                             const int32_t *goff, const int32_t *glen,
                             const float *taus, int32_t n_tau,
                             const float *s, const float *z, const float *inv_s,
                             uint8_t *q_out, uint8_t *cls_out, double *xdq_out,
                             uint8_t *clip_out)
{
    const int32_t kp = goff[ng];
    const float qmax = (float)((1 << act_bits) - 1);
    for (int64_t r = 0; r < rows; ++r) {
        float mx = -INFINITY, mn = INFINITY;
        for (int32_t c = 0; c < C; ++c) {
            float v = x[r * C + c];
            if (v > mx) mx = v;
            if (v < mn) mn = v;
        }
        float w = mx - mn;
        /* nearest centroid of clusters that are intervals of the range = number of
           thresholds below the range (taus ascending) */
        int p = 0;
        for (int32_t k = 0; k < n_tau; ++k) p += w > taus[k];
        cls_out[r] = (uint8_t)p;
        for (int32_t j = 0; j < kp; ++j) q_out[r * kp + j] = 0;
        for (int32_t g = 0; g < ng; ++g) {
            float zz = z[p * ng_cap + g], is = inv_s[p * ng_cap + g];
            float sc = s[p * ng_cap + g];
            for (int32_t j = 0; j < glen[g]; ++j) {
                int32_t c = perm[goff[g] + j];
                float t = x[r * C + c] - zz;
                float u = t * is;
                float qf = nearbyintf(u); /* round-half-to-even */
                if (qf < 0.0f) qf = 0.0f;
                if (qf > qmax) qf = qmax;
                if (!(qf == qf)) qf = 0.0f; /* NaN -> 0 */
                q_out[r * kp + goff[g] + j] = (uint8_t)qf;
                if (xdq_out) xdq_out[r * C + c] = (double)sc * (double)qf + (double)zz;
                if (clip_out) clip_out[r * C + c] = (uint8_t)(u < -0.5f || u > qmax + 0.5f);
            }
        }
    }
}

/* Two pixel classes: one threshold. */
void dgqo_quantize_act(const float *x, int64_t rows, int32_t C, int32_t act_bits,
                       int32_t ng, int32_t ng_cap, const int32_t *perm,
                       const int32_t *goff, const int32_t *glen, float tau_pix,
                       const float *s, const float *z, const float *inv_s,
                       uint8_t *q_out, uint8_t *cls_out, double *xdq_out,
                       uint8_t *clip_out)
{
    dgqo_quantize_act_multi(x, rows, C, act_bits, ng, ng_cap, perm, goff, glen, &tau_pix, 1,
                            s, z, inv_s, q_out, cls_out, xdq_out, clip_out);
}

/* ------------------------------------------------------------------------- */
/* Weights: per-output-channel symmetric round-to-nearest                    */
/* ------------------------------------------------------------------------- */

/* sw[o] = max_c |W[o,c]| / qmax (1 for an all-zero row);
   wq = clamp(rne(W / sw), -qmax, qmax); qmax = 127 (8 bit) or 7 (4 bit). */
void dgqo_quantize_weight(const float *w, int32_t O, int32_t C, int32_t w_bits,
                          int8_t *wq, float *sw)
{
    const float qmax = w_bits == 8 ? 127.0f : 7.0f;
    for (int32_t o = 0; o < O; ++o) {
        float amax = 0.0f;
        for (int32_t c = 0; c < C; ++c) {
            float a = fabsf(w[(int64_t)o * C + c]);
            if (a > amax) amax = a;
        }
        float sc = amax > 0.0f ? amax / qmax : 1.0f;
        sw[o] = sc;
        for (int32_t c = 0; c < C; ++c) {
            float qf = nearbyintf(w[(int64_t)o * C + c] / sc);
            if (qf < -qmax) qf = -qmax;
            if (qf > qmax) qf = qmax;
            wq[(int64_t)o * C + c] = (int8_t)qf;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Grouped integer contraction + dequantization                              */
/* ------------------------------------------------------------------------- */

/*
 * code = q - off (off = 128 for 8-bit activations, 0 for 4-bit: the stored
 * signed code; x ~= s*code + z' with z' = z + off*s).
 *   acc[r,o,g] = sum_{j in g} code[r,j] * wq[o, perm[j]]            (int32)
 *   Y[r,o] = sw[o] * ( sum_g s[p,g]*acc[r,o,g] + sum_g z'[p,g]*wsum[g,o] ) + bias[o]
 * evaluated in double and rounded once to fp32; wsum[g,o] = sum_{j in g} wq.
 * q: [rows, K'] as written by dgqo_quantize_act; acc_out (nullable) [rows,O,NG].
 */
void dgqo_linear(const uint8_t *q, const uint8_t *cls, int64_t rows, int32_t C,
                 int32_t O, int32_t act_bits, int32_t ng, int32_t ng_cap,
                 const int32_t *perm, const int32_t *goff, const int32_t *glen,
                 const float *s, const float *z, const int8_t *wq,
                 const float *sw, const float *bias, float *y, int32_t *acc_out)
{
    const int32_t kp = goff[ng];
    const int32_t off = act_bits == 8 ? 128 : 0;
    int64_t *wsum = (int64_t *)malloc(sizeof(int64_t) * (size_t)ng * (size_t)O);
    for (int32_t g = 0; g < ng; ++g)
        for (int32_t o = 0; o < O; ++o) {
            int64_t t = 0;
            for (int32_t j = 0; j < glen[g]; ++j)
                t += wq[(int64_t)o * C + perm[goff[g] + j]];
            wsum[(int64_t)g * O + o] = t;
        }
    for (int64_t r = 0; r < rows; ++r) {
        int p = cls[r];
        for (int32_t o = 0; o < O; ++o) {
            double dot = 0.0, zt = 0.0;
            for (int32_t g = 0; g < ng; ++g) {
                int32_t acc = 0;
                for (int32_t j = 0; j < glen[g]; ++j) {
                    int32_t code = (int32_t)q[r * kp + goff[g] + j] - off;
                    acc += code * (int32_t)wq[(int64_t)o * C + perm[goff[g] + j]];
                }
                if (acc_out) acc_out[(r * O + o) * ng + g] = acc;
                double sg = (double)s[p * ng_cap + g];
                double zp = (double)z[p * ng_cap + g] + (double)off * sg;
                dot = dot + sg * (double)acc;
                zt = zt + zp * (double)wsum[(int64_t)g * O + o];
            }
            double v = (double)sw[o] * (dot + zt);
            if (bias) v = v + (double)bias[o];
            y[r * O + o] = (float)v;
        }
    }
    free(wsum);
}

/* ------------------------------------------------------------------------- */
/* Cross-attention with log2-quantized probabilities                         */
/* ------------------------------------------------------------------------- */

/*
 * A[b,h,i,j] = softmax_j( (Q[b,i,h,:] . K[b,j,h,:]) / sqrt(d) + kb[j] ) over all
 * nk keys, logits and softmax in double, A rounded to fp32.
 * Layouts: Q [B,N,H,d], K [B,nk,H,d], A [B,H,N,nk].
 */
void dgqo_attn_probs(const float *Q, const float *K, const float *kb, int32_t B,
                     int32_t N, int32_t H, int32_t d, int32_t nk, float *A)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    double *l = (double *)malloc(sizeof(double) * (size_t)nk);
    for (int32_t b = 0; b < B; ++b)
        for (int32_t h = 0; h < H; ++h)
            for (int32_t i = 0; i < N; ++i) {
                const float *q = Q + (((int64_t)b * N + i) * H + h) * d;
                double m = -INFINITY;
                for (int32_t j = 0; j < nk; ++j) {
                    const float *k = K + (((int64_t)b * nk + j) * H + h) * d;
                    double dot = 0.0;
                    for (int32_t t = 0; t < d; ++t) dot = dot + (double)q[t] * (double)k[t];
                    l[j] = dot * inv_sqrt_d + (kb ? (double)kb[j] : 0.0);
                    if (l[j] > m) m = l[j];
                }
                double sum = 0.0;
                for (int32_t j = 0; j < nk; ++j) {
                    l[j] = exp(l[j] - m);
                    sum = sum + l[j];
                }
                float *a = A + (((int64_t)b * H + h) * N + i) * nk;
                for (int32_t j = 0; j < nk; ++j) a[j] = (float)(l[j] / sum);
            }
    free(l);
}

/*
 * Given fp32 probabilities A [B,H,N,nk]:
 *   s[b]    = max over h, i, j >= 1 of A                       (fp32)
 *   q_ij    = clamp(rne(-log2(A_ij / s[b])), 0, 2^bits - 1),  j >= 1  (double)
 *             A_ij == 0 -> 2^bits - 1
 *   Ahat_ij = s[b] * 2^(-q_ij)  (j >= 1),  Ahat_i0 = A_i0
 *   Out[b,i,h,:] = A_i0 * V[b,0,h,:] + s[b] * sum_{j>=1} 2^(-q_ij) * V[b,j,h,:]
 * in double, rounded once to fp32.  No renormalisation.
 *   codes  [B,H,N,nk-1]
 *   margin [B,H,N,nk-1] (nullable): distance, in log2 units, from -log2(A/s)
 *          to the nearest rounding boundary k + 1/2, k = 0 .. 2^bits - 2
 *   ahat   [B,H,N,nk]   (nullable) in double
 */
/* first = 1: column 0 (the <start> token) bypasses the quantizer (cross-attention).
 * first = 0: every column goes through it (self-attention); codes and margin then have
 * nk columns instead of nk - 1. */
static void dgqo_xattn_logq_impl(const float *A, const float *V, int32_t B, int32_t N,
                                 int32_t H, int32_t d, int32_t nk, int32_t bits,
                                 int32_t first, const float *s_in, float *s_out,
                                 uint8_t *codes, float *margin, double *ahat, float *out)
{
    const int32_t nc = nk - first;
    const int32_t qmax = (1 << bits) - 1;
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    for (int32_t b = 0; b < B; ++b) {
        float s = 0.0f;
        for (int32_t h = 0; h < H; ++h)
            for (int32_t i = 0; i < N; ++i) {
                const float *a = A + (((int64_t)b * H + h) * N + i) * nk;
                for (int32_t j = first; j < nk; ++j)
                    if (a[j] > s) s = a[j];
            }
        s_out[b] = s;            /* this call's own maximum, whichever scale is used */
        if (s_in) s = s_in[b];   /* static scale: given, e.g. a running max of earlier calls */
        for (int32_t h = 0; h < H; ++h)
            for (int32_t i = 0; i < N; ++i) {
                const int64_t row = ((int64_t)b * H + h) * N + i;
                const float *a = A + row * nk;
                for (int32_t t = 0; t < d; ++t)
                    acc[t] = first ? (double)a[0] * (double)V[(((int64_t)b * nk + 0) * H + h) * d + t]
                                   : 0.0;
                if (ahat && first) ahat[row * nk] = (double)a[0];
                for (int32_t j = first; j < nk; ++j) {
                    int32_t q;
                    double mg;
                    if (a[j] > 0.0f && s > 0.0f) {
                        double t = -log2((double)a[j] / (double)s);
                        double qd = nearbyint(t);
                        if (qd < 0.0) qd = 0.0;
                        if (qd > (double)qmax) qd = (double)qmax;
                        q = (int32_t)qd;
                        /* boundaries sit at k + 1/2 for k = 0 .. qmax-1 */
                        if (t >= (double)qmax - 0.5) {
                            mg = t - ((double)qmax - 0.5);
                        } else {
                            double f = t - floor(t);
                            mg = fabs(f - 0.5);
                        }
                    } else {
                        q = qmax;
                        mg = 1.0e30;
                    }
                    codes[row * nc + (j - first)] = (uint8_t)q;
                    if (margin) margin[row * nc + (j - first)] = (float)mg;
                    double p2 = ldexp(1.0, -q); /* exact power of two */
                    double ah = (double)s * p2;
                    if (ahat) ahat[row * nk + j] = ah;
                    const float *v = V + (((int64_t)b * nk + j) * H + h) * d;
                    for (int32_t t = 0; t < d; ++t) acc[t] = acc[t] + ah * (double)v[t];
                }
                float *o = out + (((int64_t)b * N + i) * H + h) * d;
                for (int32_t t = 0; t < d; ++t) o[t] = (float)acc[t];
            }
    }
    free(acc);
}

void dgqo_xattn_logq(const float *A, const float *V, int32_t B, int32_t N,
                     int32_t H, int32_t d, int32_t nk, int32_t bits,
                     float *s_out, uint8_t *codes, float *margin, double *ahat,
                     float *out)
{
    dgqo_xattn_logq_impl(A, V, B, N, H, d, nk, bits, 1, NULL, s_out, codes, margin, ahat, out);
}

/*
 * The log quantizer without dynamic quantization (the ablation of Section 4.3): the scale
 * s[b] is GIVEN (calibrated, or a running maximum of earlier denoising steps) instead of
 * being this call's maximum.  Probabilities above s saturate at code 0, i.e. at s.
 * s_out still receives this call's own maximum (what a running estimate is updated with).
 */
void dgqo_xattn_logq_static(const float *A, const float *V, int32_t B, int32_t N,
                            int32_t H, int32_t d, int32_t nk, int32_t bits,
                            const float *s_in, float *s_out, uint8_t *codes, float *margin,
                            double *ahat, float *out)
{
    dgqo_xattn_logq_impl(A, V, B, N, H, d, nk, bits, 1, s_in, s_out, codes, margin, ahat, out);
}

/*
 * Self-attention (Section 3.3: the logarithmic quantizer is applied to self- and
 * cross-attention alike; separating the <start> column and the dynamic scale are stated
 * for cross-attention only): every probability goes through the log quantizer of
 * Section 3.1 with a GIVEN scale s[b], A^q = clamp(rne(-log2(A / s)), 0, 2^b - 1),
 * A^ = s 2^-A^q, out = A^ V.  A: [B,H,N,nk] (N queries, nk keys; nk = N in a layer, any
 * subset of the queries for sampled checks); codes, margin: [B,H,N,nk].  s_out receives
 * max A.
 */
void dgqo_selfattn_logq(const float *A, const float *V, int32_t B, int32_t N, int32_t H,
                        int32_t d, int32_t nk, int32_t bits, const float *s_in, float *s_out,
                        uint8_t *codes, float *margin, double *ahat, float *out)
{
    dgqo_xattn_logq_impl(A, V, B, N, H, d, nk, bits, 0, s_in, s_out, codes, margin, ahat, out);
}

/* ------------------------------------------------------------------------- */
/* Gated feed-forward activation (for the fused epilogue of the contraction)  */
/* ------------------------------------------------------------------------- */

/*
 * The transformer feed-forward of the models the paper quantizes (Section 4.1:
 * Stable Diffusion v1.4, SDXL-Turbo) gates its first projection: with
 * y = [a | b] (first and second half of the O output channels),
 *     out = a * GELU(b),   GELU(t) = t * Phi(t),
 * Phi the standard normal distribution function.  This is the models'
 * definition, not a formula of the paper; it is here because the contraction
 * kernel can apply it before the result ever reaches memory.  Evaluated in
 * double on the fp32 result of dgqo_linear, rounded once.
 */
void dgqo_geglu(const float *y, int64_t rows, int32_t O, float *out)
{
    const int32_t oh = O / 2;
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t c = 0; c < oh; ++c) {
            const double a = (double)y[r * O + c];
            const double b = (double)y[r * O + oh + c];
            const double phi = 0.5 * (1.0 + erf(b / sqrt(2.0)));
            out[r * oh + c] = (float)(a * (b * phi));
        }
}


/* ------------------------------------------------------------------------- */
/* Quantized value tensor of the attention product (Section 3.3, A^ V^)      */
/* ------------------------------------------------------------------------- */

/*
 * V^ of the product A^ V^: the value tensor goes through the linear quantizer of
 * Section 3.1 with the range of its own (prompt, head) slice,
 *   s = (max - min) / 2^b (1 if max == min),  z = min   over V[b, :, h, :]
 *   q = clamp(rne((v - z) * (1/s)), 0, 2^b - 1)         (fp32, separate operations)
 *   v^ = s * q + z, rounded once to fp32
 * V, vhat: [B, nk, H, d]; codes (nullable): [B, nk, H, d]; params (nullable):
 * [B, H, 2] = (s, z).
 */
void dgqo_quantize_value(const float *V, int32_t B, int32_t nk, int32_t H, int32_t d,
                         int32_t bits, float *vhat, uint8_t *codes, float *params)
{
    const float qmax = (float)((1 << bits) - 1);
    const float levels = (float)(1 << bits);
    for (int32_t b = 0; b < B; ++b)
        for (int32_t h = 0; h < H; ++h) {
            float mx = -INFINITY, mn = INFINITY;
            for (int32_t j = 0; j < nk; ++j)
                for (int32_t t = 0; t < d; ++t) {
                    float v = V[(((int64_t)b * nk + j) * H + h) * d + t];
                    if (v > mx) mx = v;
                    if (v < mn) mn = v;
                }
            float s = (mx - mn) / levels;
            if (!(mx > mn)) s = 1.0f;
            float inv = 1.0f / s;
            if (params) {
                params[((int64_t)b * H + h) * 2 + 0] = s;
                params[((int64_t)b * H + h) * 2 + 1] = mn;
            }
            for (int32_t j = 0; j < nk; ++j)
                for (int32_t t = 0; t < d; ++t) {
                    int64_t at = (((int64_t)b * nk + j) * H + h) * d + t;
                    float u = (V[at] - mn) * inv;
                    float qf = nearbyintf(u);
                    if (qf < 0.0f) qf = 0.0f;
                    if (qf > qmax) qf = qmax;
                    if (!(qf == qf)) qf = 0.0f;
                    if (codes) codes[at] = (uint8_t)qf;
                    vhat[at] = (float)((double)s * (double)qf + (double)mn);
                }
        }
}
