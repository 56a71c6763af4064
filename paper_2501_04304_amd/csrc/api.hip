// Host side of the C ABI: argument checks, the calibration driver (range
// reductions on the GPU, exact 1-D clustering and table construction on the
// host), handle lifetime, and dispatch to the kernels.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <new>
#include <numeric>

#include <atomic>
#include <utility>

#include "dgq_internal.h"

namespace dgq {

static thread_local std::string g_last_error;

void set_error(const std::string &msg) { g_last_error = msg; }

hipError_t raise_lds_limit(LdsLimit &state, const void *kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (state.bytes[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
    // two threads may both get here: the attribute call is idempotent
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) state.bytes[dev].store(bytes, std::memory_order_release);
    return e;
}

#ifdef DGQ_TUNING
static std::atomic<int> g_tuning[kTuneKeys];
int tuning_value(int key) { return key >= 0 && key < kTuneKeys ? g_tuning[key].load() : 0; }
extern "C" int dgq_tuning_set(int key, int value) {
    if (key < 0 || key >= kTuneKeys) return DGQ_EINVAL;
    g_tuning[key].store(value);
    return DGQ_OK;
}
#endif

int hip_fail(hipError_t e, const char *what) {
    set_error(std::string(what) + ": " + hipGetErrorString(e));
    return DGQ_EHIP;
}

namespace {

int fail(int code, const std::string &msg) {
    set_error(msg);
    return code;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct DevBuf {  // scoped device allocation for the blocking (offline) calls
    void *p = nullptr;
    ~DevBuf() {
        if (p) (void)hipFree(p);
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 16); }
    template <class T>
    T *as() const { return static_cast<T *>(p); }
};

// Exact K-means of a 1-D sample (the grouping "by range using K-means" of Section 3.3).
// An optimal 1-D clustering cuts the sorted sample into intervals, so the optimum over all
// partitions into k intervals is a shortest path through k layers,
//     layer_k(j) = min over cuts i < j of layer_{k-1}(i) + within(i, j),
//     within(i, j) = sum of squared deviations of sorted values i .. j-1 from their mean,
// where only positions between two DISTINCT values are cuts.  within() satisfies the
// quadrangle inequality, hence the leftmost best cut of layer_k(j) does not move left as j
// grows, and a layer is filled by divide and conquer: solve the middle j of a range over its
// window of candidate cuts, then the left half with the window's lower part and the right half
// with its upper part -- O(n log n) evaluations per layer instead of the O(n^2) of the
// definition, which is what lets the pixel dimension take every calibration row (64 prompts of
// 4096 pixels: 262144).  A range whose middle has no admissible cut keeps the whole window for
// both halves.  within() comes from running sums of the sorted values and their squares in
// double; ties go to the leftmost cut; k = min(K, number of distinct values).  The threshold
// between two neighbouring clusters is the midpoint of their means, rounded to fp32 and clamped
// between the two values it separates, so "number of thresholds below v" names v's cluster.
struct Clusters {
    std::vector<int64_t> bounds;  // cluster c = sorted positions [bounds[c], bounds[c+1])
    std::vector<float> taus;      // bounds.size() - 2 thresholds, ascending
    std::vector<int64_t> order;   // indices sorted by (value, index)
};

Clusters cluster_by_range(const std::vector<float> &v, int32_t K) {
    Clusters cl;
    const int64_t n = (int64_t)v.size();
    cl.order.resize(n);
    std::iota(cl.order.begin(), cl.order.end(), (int64_t)0);
    std::sort(cl.order.begin(), cl.order.end(), [&](int64_t x, int64_t y) {
        return v[x] < v[y] || (v[x] == v[y] && x < y);
    });
    std::vector<float> sorted(n);
    std::vector<double> sum1(n + 1, 0.0), sum2(n + 1, 0.0);
    std::vector<uint8_t> is_cut(n + 1, 0);  // position i separates two distinct values
    int64_t distinct = n > 0 ? 1 : 0;
    for (int64_t i = 0; i < n; ++i) {
        sorted[i] = v[cl.order[i]];
        const double x = sorted[i];
        sum1[i + 1] = sum1[i] + x;
        sum2[i + 1] = sum2[i] + x * x;
        if (i > 0 && sorted[i - 1] < sorted[i]) {
            is_cut[i] = 1;
            ++distinct;
        }
    }
    const int32_t k_use = (int32_t)std::max<int64_t>(1, std::min<int64_t>(K, distinct));
    auto within = [&](int64_t i, int64_t j) {
        const double d = sum1[j] - sum1[i];
        return (sum2[j] - sum2[i]) - (d * d) / (double)(j - i);
    };
    // value[k][j]: least total cost of the first j values in k clusters; from[k][j]: the cut
    // that reaches it, -1 where no admissible partition exists
    std::vector<std::vector<double>> value(k_use + 1, std::vector<double>(n + 1, 0.0));
    std::vector<std::vector<int64_t>> from(k_use + 1, std::vector<int64_t>(n + 1, -1));
    for (int64_t j = 1; j <= n; ++j) {
        value[1][j] = within(0, j);
        from[1][j] = 0;
    }
    struct Range {
        int64_t j_lo, j_hi, i_lo, i_hi;  // rows j_lo..j_hi, candidate cuts i_lo..i_hi (inclusive)
    };
    std::vector<Range> todo;
    for (int32_t k = 2; k <= k_use; ++k) {
        const std::vector<double> &below = value[k - 1];
        const std::vector<int64_t> &below_from = from[k - 1];
        todo.clear();
        todo.push_back({(int64_t)k, n, (int64_t)k - 1, n - 1});
        while (!todo.empty()) {
            const Range r = todo.back();
            todo.pop_back();
            if (r.j_lo > r.j_hi) continue;
            const int64_t j = r.j_lo + (r.j_hi - r.j_lo) / 2;
            int64_t pick = -1;
            double least = 0.0;
            const int64_t last = std::min(r.i_hi, j - 1);
            for (int64_t i = r.i_lo; i <= last; ++i) {
                if (!is_cut[i] || below_from[i] < 0) continue;
                const double t = below[i] + within(i, j);
                if (pick < 0 || t < least) {
                    least = t;
                    pick = i;
                }
            }
            if (pick >= 0) {
                value[k][j] = least;
                from[k][j] = pick;
                todo.push_back({r.j_lo, j - 1, r.i_lo, pick});
                todo.push_back({j + 1, r.j_hi, pick, r.i_hi});
            } else {
                todo.push_back({r.j_lo, j - 1, r.i_lo, r.i_hi});
                todo.push_back({j + 1, r.j_hi, r.i_lo, r.i_hi});
            }
        }
    }
    cl.bounds.assign(k_use + 1, 0);
    cl.bounds[k_use] = n;
    for (int32_t k = k_use; k >= 1; --k) cl.bounds[k - 1] = from[k][cl.bounds[k]];
    for (int32_t c = 0; c + 1 < k_use; ++c) {
        const int64_t b0 = cl.bounds[c], b1 = cl.bounds[c + 1], b2 = cl.bounds[c + 2];
        const double mean_lo = (sum1[b1] - sum1[b0]) / (double)(b1 - b0);
        const double mean_hi = (sum1[b2] - sum1[b1]) / (double)(b2 - b1);
        float tau = (float)(0.5 * (mean_lo + mean_hi));
        tau = std::max(tau, sorted[b1 - 1]);
        tau = std::min(tau, std::nextafterf(sorted[b1], -INFINITY));
        cl.taus.push_back(tau);
    }
    return cl;
}

// The two-cluster case (outlier rows against regular rows, outlier channels against regular
// channels): the same exact clustering with K = 2.
struct Split {
    int64_t n_lower = 0;         // size of the lower cluster (n if no split exists)
    float tau = INFINITY;        // value > tau  <=>  upper cluster
    std::vector<int64_t> order;  // indices sorted by (value, index)
};

Split split_two_clusters(const std::vector<float> &v) {
    Clusters cl = cluster_by_range(v, 2);
    Split sp;
    sp.n_lower = cl.bounds.size() == 3 ? cl.bounds[1] : (int64_t)v.size();
    if (!cl.taus.empty()) sp.tau = cl.taus[0];
    sp.order = std::move(cl.order);
    return sp;
}

// D_d of Section 3.3 from the per-vector maxima and minima along one dimension.
double variability(const std::vector<float> &vmax, const std::vector<float> &vmin) {
    const auto mx = std::minmax_element(vmax.begin(), vmax.end());
    const auto mn = std::minmax_element(vmin.begin(), vmin.end());
    return ((double)*mx.second - (double)*mx.first) + ((double)*mn.second - (double)*mn.first);
}

template <class T>
int upload(T **dst, const std::vector<T> &src) {
    DGQ_HIP(hipMalloc(reinterpret_cast<void **>(dst), std::max<size_t>(src.size() * sizeof(T), 16)));
    if (!src.empty())
        DGQ_HIP(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
    return DGQ_OK;
}

// Device copies of a finished host description: per-chunk (z, 1/s) rows for the
// quantizer, scale and offset rows and group boundaries for the contraction, thresholds.
int upload_tables(Groups *g) {
    const int32_t NG = (int32_t)g->glen.size();
    const int32_t T = g->n_tab;
    g->n_chunks = (int32_t)g->perm.size() / kGranule;
    (void)hipGetDevice(&g->device);
    std::vector<float> chunk_z((size_t)T * g->n_chunks), chunk_inv((size_t)T * g->n_chunks);
    std::vector<float> zoff((size_t)T * NG);
    std::vector<int32_t> gchunk(NG + 1);
    for (int32_t k = 0; k <= NG; ++k) gchunk[k] = g->goff[k] / kGranule;
    for (int p = 0; p < T; ++p)
        for (int32_t k = 0; k < NG; ++k) {
            for (int32_t ch = gchunk[k]; ch < gchunk[k + 1]; ++ch) {
                chunk_z[(size_t)p * g->n_chunks + ch] = g->z[p * NG + k];
                chunk_inv[(size_t)p * g->n_chunks + ch] = g->inv_s[p * NG + k];
            }
            zoff[(size_t)p * NG + k] =
                (float)((double)g->z[p * NG + k] + (double)g->info.code_offset * (double)g->s[p * NG + k]);
        }
    int rc = upload(&g->d_perm, g->perm);
    if (rc == DGQ_OK) rc = upload(&g->d_chunk_z, chunk_z);
    if (rc == DGQ_OK) rc = upload(&g->d_chunk_inv, chunk_inv);
    if (rc == DGQ_OK) rc = upload(&g->d_s, g->s);
    if (rc == DGQ_OK) rc = upload(&g->d_z, g->z);
    if (rc == DGQ_OK) rc = upload(&g->d_zoff, zoff);
    if (rc == DGQ_OK) rc = upload(&g->d_taus, g->taus);
    if (rc == DGQ_OK) rc = upload(&g->d_gchunk, gchunk);
    return rc;
}

void release(Groups *g) {
    if (!g) return;
    if (g->refs.fetch_sub(1, std::memory_order_acq_rel) != 1) return;  // a weight handle still uses it
    (void)hipFree(g->d_perm);
    (void)hipFree(g->d_chunk_z);
    (void)hipFree(g->d_chunk_inv);
    (void)hipFree(g->d_s);
    (void)hipFree(g->d_z);
    (void)hipFree(g->d_zoff);
    (void)hipFree(g->d_taus);
    (void)hipFree(g->d_gchunk);
    (void)hipFree(g->d_fill);
    (void)hipFree(g->d_fill_blocks);
    delete g;
}

void release(Weight *w) {
    if (!w) return;
    release(const_cast<Groups *>(w->groups));
    (void)hipFree(w->d_wq);
    (void)hipFree(w->d_wq4);
    (void)hipFree(w->d_sw);
    (void)hipFree(w->d_zb);
    (void)hipFree(w->d_rq_zi);
    (void)hipFree(w->d_rq_keep);
    delete w;
}

}  // namespace
}  // namespace dgq

using namespace dgq;

extern "C" {

int dgq_version(void) { return 100; }

const char *dgq_last_error(void) { return g_last_error.c_str(); }

int dgq_calibrate_groups(const float *x_cal, int64_t rows, int32_t channels, int32_t act_bits,
                         int32_t group_size, int32_t n_pixel_classes, void *stream,
                         dgq_groups_t **out) {
    if (!x_cal || !out) return fail(DGQ_EINVAL, "dgq_calibrate_groups: null pointer");
    *out = nullptr;
    if (rows < 1 || channels < 1) return fail(DGQ_EINVAL, "dgq_calibrate_groups: empty tensor");
    if (act_bits != 4 && act_bits != 8)
        return fail(DGQ_EINVAL, "dgq_calibrate_groups: act_bits must be 4 or 8");
    if (group_size < kGranule || group_size % kGranule)
        return fail(DGQ_EINVAL, "dgq_calibrate_groups: group_size must be a positive multiple of 64");
    if (n_pixel_classes != 1 && n_pixel_classes != 2)
        return fail(DGQ_EINVAL, "dgq_calibrate_groups: n_pixel_classes must be 1 or 2");
    if (!aligned16(x_cal)) return fail(DGQ_EALIGN, "dgq_calibrate_groups: x_cal not 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t C = channels;

    // 1. per-pixel range -> pixel classes
    DevBuf d_rmx, d_rmn;
    DGQ_HIP(d_rmx.alloc(sizeof(float) * rows));
    DGQ_HIP(d_rmn.alloc(sizeof(float) * rows));
    DGQ_HIP(launch_row_minmax(x_cal, rows, C, d_rmx.as<float>(), d_rmn.as<float>(), st));
    std::vector<float> rmx(rows), rmn(rows), width(rows);
    DGQ_HIP(hipMemcpyAsync(rmx.data(), d_rmx.p, sizeof(float) * rows, hipMemcpyDeviceToHost, st));
    DGQ_HIP(hipMemcpyAsync(rmn.data(), d_rmn.p, sizeof(float) * rows, hipMemcpyDeviceToHost, st));
    DGQ_HIP(hipStreamSynchronize(st));
    for (int64_t r = 0; r < rows; ++r) width[r] = rmx[r] - rmn[r];
    float tau = INFINITY;
    if (n_pixel_classes == 2) tau = split_two_clusters(width).tau;
    int64_t n_cls[2] = {0, 0};
    for (int64_t r = 0; r < rows; ++r) ++n_cls[width[r] > tau ? 1 : 0];

    // 2. per-channel range, separately for the two pixel classes
    const int32_t slabs = (int32_t)std::min<int64_t>(rows, 256);
    DevBuf d_part;
    DGQ_HIP(d_part.alloc(sizeof(float) * (size_t)slabs * 4 * C));
    DGQ_HIP(launch_col_minmax_by_class(x_cal, rows, C, d_rmx.as<float>(), d_rmn.as<float>(), tau,
                                       slabs, d_part.as<float>(), st));
    std::vector<float> part((size_t)slabs * 4 * C);
    DGQ_HIP(hipMemcpyAsync(part.data(), d_part.p, sizeof(float) * part.size(),
                           hipMemcpyDeviceToHost, st));
    DGQ_HIP(hipStreamSynchronize(st));
    std::vector<float> cmx[2], cmn[2];
    for (int p = 0; p < 2; ++p) {
        cmx[p].assign(C, -INFINITY);
        cmn[p].assign(C, INFINITY);
    }
    for (int32_t sl = 0; sl < slabs; ++sl) {
        const float *pp = part.data() + (size_t)sl * 4 * C;
        for (int p = 0; p < 2; ++p)
            for (int32_t c = 0; c < C; ++c) {
                cmx[p][c] = std::max(cmx[p][c], pp[(2 * p) * C + c]);
                cmn[p][c] = std::min(cmn[p][c], pp[(2 * p + 1) * C + c]);
            }
    }

    // 3. D_d over the whole tensor and the dimension it would select
    std::vector<float> all_mx(C), all_mn(C);
    for (int32_t c = 0; c < C; ++c) {
        all_mx[c] = std::max(cmx[0][c], cmx[1][c]);
        all_mn[c] = std::min(cmn[0][c], cmn[1][c]);
    }
    const double d_channel = variability(all_mx, all_mn);
    const double d_pixel = variability(rmx, rmn);

    // 4. channel groups: outlier cluster by range over class-0 pixels, then blocks of G
    std::vector<float> cw(C);
    for (int32_t c = 0; c < C; ++c) cw[c] = cmx[0][c] - cmn[0][c];
    const Split cs = split_two_clusters(cw);
    Groups *g = new (std::nothrow) Groups();
    if (!g) return fail(DGQ_EINVAL, "dgq_calibrate_groups: out of host memory");
    int32_t n_regular_groups = 0;
    g->goff.push_back(0);
    auto cut_cluster = [&](int64_t begin, int64_t end) {
        int32_t made = 0;
        for (int64_t at = begin; at < end; at += group_size) {
            const int32_t len = (int32_t)std::min<int64_t>(group_size, end - at);
            const int32_t padded = (len + kGranule - 1) / kGranule * kGranule;
            for (int32_t j = 0; j < padded; ++j)
                g->perm.push_back(j < len ? (int32_t)cs.order[at + j] : -1);
            g->glen.push_back(len);
            g->goff.push_back((int32_t)g->perm.size());
            ++made;
        }
        return made;
    };
    n_regular_groups = cut_cluster(0, cs.n_lower);
    cut_cluster(cs.n_lower, C);
    const int32_t NG = (int32_t)g->glen.size();
    const int32_t Kp = (int32_t)g->perm.size();

    // 5. cell parameters: s = (max - min) / 2^b, z = min
    const float levels = (float)(1 << act_bits);
    g->s.assign(2 * NG, 1.0f);
    g->z.assign(2 * NG, 0.0f);
    g->inv_s.assign(2 * NG, 1.0f);
    for (int p = 0; p < 2; ++p)
        for (int32_t k = 0; k < NG; ++k) {
            float sc, zp;
            if (n_cls[p] == 0) {
                sc = g->s[k];
                zp = g->z[k];
            } else {
                float mx = -INFINITY, mn = INFINITY;
                for (int32_t j = 0; j < g->glen[k]; ++j) {
                    const int32_t c = g->perm[g->goff[k] + j];
                    mx = std::max(mx, cmx[p][c]);
                    mn = std::min(mn, cmn[p][c]);
                }
                sc = mx > mn ? (mx - mn) / levels : 1.0f;
                zp = mn;
            }
            g->s[p * NG + k] = sc;
            g->z[p * NG + k] = zp;
            g->inv_s[p * NG + k] = 1.0f / sc;
        }

    dgq_groups_info_t &in = g->info;
    in.channels = C;
    in.act_bits = act_bits;
    in.group_size = group_size;
    in.n_pixel_classes = n_pixel_classes;
    in.n_groups = NG;
    in.k_padded = Kp;
    in.n_outlier_channels = (int32_t)(C - cs.n_lower);
    in.n_regular_groups = n_regular_groups;
    in.dstar = d_pixel > d_channel ? 1 : 0;
    in.code_offset = act_bits == 8 ? 128 : 0;
    in.n_class1_rows = (int32_t)n_cls[1];
    in.tau_pix = tau;
    in.d_channel = d_channel;
    in.d_pixel = d_pixel;
    in.grouping = DGQ_GROUPING_GRID;

    // 6. device tables
    g->n_tab = 2;
    g->taus.assign(1, tau);
    const int rc = upload_tables(g);
    if (rc != DGQ_OK) {
        release(g);
        return rc;
    }
    *out = reinterpret_cast<dgq_groups_t *>(g);
    return DGQ_OK;
}

int dgq_groups_info(const dgq_groups_t *h, dgq_groups_info_t *info) {
    if (!h || !info) return fail(DGQ_EINVAL, "dgq_groups_info: null pointer");
    *info = reinterpret_cast<const Groups *>(h)->info;
    return DGQ_OK;
}

int dgq_calibrate_kmeans(const float *x_cal, int64_t rows, int32_t channels, int32_t act_bits,
                         int32_t n_clusters, int32_t dimension, void *stream, dgq_groups_t **out) {
    if (!x_cal || !out) return fail(DGQ_EINVAL, "dgq_calibrate_kmeans: null pointer");
    *out = nullptr;
    if (rows < 1 || channels < 1) return fail(DGQ_EINVAL, "dgq_calibrate_kmeans: empty tensor");
    if (act_bits != 4 && act_bits != 8)
        return fail(DGQ_EINVAL, "dgq_calibrate_kmeans: act_bits must be 4 or 8");
    if (n_clusters < 1 || n_clusters > kMaxClasses)
        return fail(DGQ_EINVAL, "dgq_calibrate_kmeans: n_clusters must be 1..16");
    if (dimension < DGQ_DIM_AUTO || dimension > DGQ_DIM_PIXEL)
        return fail(DGQ_EINVAL, "dgq_calibrate_kmeans: dimension must be DGQ_DIM_AUTO, _CHANNEL or _PIXEL");
    if (!aligned16(x_cal)) return fail(DGQ_EALIGN, "dgq_calibrate_kmeans: x_cal not 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int32_t C = channels;

    // ranges of the vectors of both dimensions (Eq. 4): per pixel over its channels, per
    // channel over all pixels
    DevBuf d_rmx, d_rmn, d_part;
    DGQ_HIP(d_rmx.alloc(sizeof(float) * rows));
    DGQ_HIP(d_rmn.alloc(sizeof(float) * rows));
    DGQ_HIP(launch_row_minmax(x_cal, rows, C, d_rmx.as<float>(), d_rmn.as<float>(), st));
    const int32_t slabs = (int32_t)std::min<int64_t>(rows, 256);
    DGQ_HIP(d_part.alloc(sizeof(float) * (size_t)slabs * 4 * C));
    DGQ_HIP(launch_col_minmax_by_class(x_cal, rows, C, d_rmx.as<float>(), d_rmn.as<float>(),
                                       INFINITY, slabs, d_part.as<float>(), st));  // one class
    std::vector<float> rmx(rows), rmn(rows), part((size_t)slabs * 4 * C);
    DGQ_HIP(hipMemcpyAsync(rmx.data(), d_rmx.p, sizeof(float) * rows, hipMemcpyDeviceToHost, st));
    DGQ_HIP(hipMemcpyAsync(rmn.data(), d_rmn.p, sizeof(float) * rows, hipMemcpyDeviceToHost, st));
    DGQ_HIP(hipMemcpyAsync(part.data(), d_part.p, sizeof(float) * part.size(), hipMemcpyDeviceToHost, st));
    DGQ_HIP(hipStreamSynchronize(st));
    std::vector<float> cmx(C, -INFINITY), cmn(C, INFINITY);
    for (int32_t sl = 0; sl < slabs; ++sl) {
        const float *pp = part.data() + (size_t)sl * 4 * C;
        for (int32_t c = 0; c < C; ++c) {
            cmx[c] = std::max(cmx[c], pp[c]);
            cmn[c] = std::min(cmn[c], pp[C + c]);
        }
    }
    const double d_channel = variability(cmx, cmn);
    const double d_pixel = variability(rmx, rmn);
    const int32_t dstar = d_pixel > d_channel ? 1 : 0;  // Eq. 5
    const int32_t dim = dimension == DGQ_DIM_AUTO ? dstar : dimension;
    Groups *g = new (std::nothrow) Groups();
    if (!g) return fail(DGQ_EINVAL, "dgq_calibrate_kmeans: out of host memory");
    const float levels = (float)(1 << act_bits);
    auto cell = [&](float mx, float mn, int32_t at) {  // Eq. 6
        const float sc = mx > mn ? (mx - mn) / levels : 1.0f;
        g->s[at] = sc;
        g->z[at] = mn;
        g->inv_s[at] = 1.0f / sc;
    };
    int32_t P = 1, n_upper = 0;
    g->goff.push_back(0);
    if (dim == DGQ_DIM_CHANNEL) {
        std::vector<float> cw(C);
        for (int32_t c = 0; c < C; ++c) cw[c] = cmx[c] - cmn[c];
        const Clusters cl = cluster_by_range(cw, n_clusters);
        const int32_t NG = (int32_t)cl.bounds.size() - 1;
        g->n_tab = 2;  // a second, identical class row: the kernels always see two
        g->s.assign(2 * NG, 1.0f);
        g->z.assign(2 * NG, 0.0f);
        g->inv_s.assign(2 * NG, 1.0f);
        for (int32_t k = 0; k < NG; ++k) {
            const int32_t len = (int32_t)(cl.bounds[k + 1] - cl.bounds[k]);
            const int32_t padded = (len + kGranule - 1) / kGranule * kGranule;
            float mx = -INFINITY, mn = INFINITY;
            for (int32_t j = 0; j < padded; ++j) {
                const int32_t c = j < len ? (int32_t)cl.order[cl.bounds[k] + j] : -1;
                g->perm.push_back(c);
                if (c >= 0) {
                    mx = std::max(mx, cmx[c]);
                    mn = std::min(mn, cmn[c]);
                }
            }
            g->glen.push_back(len);
            g->goff.push_back((int32_t)g->perm.size());
            cell(mx, mn, k);
            cell(mx, mn, NG + k);
        }
        g->taus.assign(1, INFINITY);
    } else {
        std::vector<float> width(rows);
        for (int64_t r = 0; r < rows; ++r) width[r] = rmx[r] - rmn[r];
        const Clusters cl = cluster_by_range(width, n_clusters);
        P = (int32_t)cl.bounds.size() - 1;
        const int32_t padded = (C + kGranule - 1) / kGranule * kGranule;
        for (int32_t j = 0; j < padded; ++j) g->perm.push_back(j < C ? j : -1);
        g->glen.push_back(C);
        g->goff.push_back(padded);
        g->n_tab = std::max(P, 2);
        g->s.assign(g->n_tab, 1.0f);
        g->z.assign(g->n_tab, 0.0f);
        g->inv_s.assign(g->n_tab, 1.0f);
        g->taus = cl.taus;
        if (g->taus.empty()) g->taus.assign(1, INFINITY);
        for (int32_t p = 0; p < P; ++p) {
            float mx = -INFINITY, mn = INFINITY;
            for (int64_t i = cl.bounds[p]; i < cl.bounds[p + 1]; ++i) {
                mx = std::max(mx, rmx[cl.order[i]]);
                mn = std::min(mn, rmn[cl.order[i]]);
            }
            cell(mx, mn, p);
            if (P == 1) cell(mx, mn, 1);
        }
        n_upper = (int32_t)(rows - cl.bounds[1]);
    }

    dgq_groups_info_t &in = g->info;
    in.channels = C;
    in.act_bits = act_bits;
    in.group_size = 0;
    in.n_pixel_classes = P;
    in.n_groups = (int32_t)g->glen.size();
    in.k_padded = (int32_t)g->perm.size();
    in.n_outlier_channels = 0;
    in.n_regular_groups = 0;
    in.dstar = dstar;
    in.code_offset = act_bits == 8 ? 128 : 0;
    in.n_class1_rows = n_upper;
    in.tau_pix = g->taus[0];
    in.d_channel = d_channel;
    in.d_pixel = d_pixel;
    in.grouping = dim == DGQ_DIM_CHANNEL ? DGQ_GROUPING_CHANNEL : DGQ_GROUPING_PIXEL;
    const int rc = upload_tables(g);
    if (rc != DGQ_OK) {
        release(g);
        return rc;
    }
    *out = reinterpret_cast<dgq_groups_t *>(g);
    return DGQ_OK;
}

int dgq_groups_for_conv3x3(const dgq_groups_t *h, dgq_groups_t **out) {
    if (!h || !out) return fail(DGQ_EINVAL, "dgq_groups_for_conv3x3: null pointer");
    *out = nullptr;
    const Groups *g = reinterpret_cast<const Groups *>(h);
    if (g->info.n_pixel_classes != 1 || g->conv_taps)
        return fail(DGQ_EUNSUPPORTED,
                    "dgq_groups_for_conv3x3: needs a layer with one pixel class (the scale of a "
                    "tap's partial sum would otherwise follow the neighbouring pixel's class)");
    constexpr int32_t T = 9;
    const int32_t C = g->info.channels, Kp = g->info.k_padded, NG = g->info.n_groups;
    if ((int64_t)T * Kp > (1 << 24)) return fail(DGQ_EUNSUPPORTED, "dgq_groups_for_conv3x3: too many channels");
    Groups *g9 = new (std::nothrow) Groups();
    if (!g9) return fail(DGQ_EINVAL, "dgq_groups_for_conv3x3: out of host memory");
    g9->n_tab = 2;
    g9->taus.assign(1, INFINITY);
    g9->conv_taps = T;
    g9->base_kp = Kp;
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t j = 0; j < Kp; ++j) g9->perm.push_back(g->perm[j] < 0 ? -1 : t * C + g->perm[j]);
        for (int32_t k = 0; k < NG; ++k) {
            g9->goff.push_back(t * Kp + g->goff[k]);
            g9->glen.push_back(g->glen[k]);
        }
    }
    g9->goff.push_back(T * Kp);
    g9->s.resize((size_t)2 * T * NG);
    g9->z.resize((size_t)2 * T * NG);
    g9->inv_s.resize((size_t)2 * T * NG);
    for (int p = 0; p < 2; ++p)
        for (int32_t t = 0; t < T; ++t)
            for (int32_t k = 0; k < NG; ++k) {
                const size_t to = (size_t)p * T * NG + (size_t)t * NG + k, from = (size_t)p * NG + k;
                g9->s[to] = g->s[from];
                g9->z[to] = g->z[from];
                g9->inv_s[to] = g->inv_s[from];
            }
    g9->info = g->info;
    g9->info.channels = T * C;
    g9->info.n_groups = T * NG;
    g9->info.k_padded = T * Kp;
    g9->info.n_outlier_channels = T * g->info.n_outlier_channels;
    g9->info.n_regular_groups = T * g->info.n_regular_groups;
    // the code of the value 0 at every position of one tap: the quantizer's own operations
    // (fl(fl(0 - z) * (1/s)), round to nearest even, clamp), then the stored form
    const int bits = g->info.act_bits;
    const float qmax = (float)((1 << bits) - 1);
    std::vector<uint8_t> q0((size_t)Kp, 0), fill((size_t)(bits == 8 ? Kp : Kp / 2), 0);
    for (int32_t k = 0; k < NG; ++k) {
        const float t0 = 0.0f - g->z[k];
        float u = nearbyintf(t0 * g->inv_s[k]);
        u = u < 0.0f ? 0.0f : (u > qmax ? qmax : u);
        if (!(u == u)) u = 0.0f;
        for (int32_t j = g->goff[k]; j < g->goff[k + 1]; ++j)
            if (g->perm[j] >= 0) q0[j] = (uint8_t)u;
    }
    if (bits == 8) {
        for (int32_t j = 0; j < Kp; ++j) fill[j] = g->perm[j] >= 0 ? (uint8_t)(q0[j] ^ 0x80) : 0;
    } else {
        for (int32_t e = 0; e < Kp / 8; ++e)
            for (int b = 0; b < 4; ++b) fill[4 * e + b] = (uint8_t)(q0[8 * e + b] | (q0[8 * e + 4 + b] << 4));
    }
    // the fill row as code blocks: 16 rows of 64 B (32 rows of 32 B), 16-byte slots permuted by
    // row bits, and in 4-bit rows 16..31 the 8-byte halves of a slot swapped
    const int32_t nch = Kp / kGranule;
    std::vector<uint8_t> fill_blocks((size_t)nch * 1024, 0);
    for (int32_t c = 0; c < nch; ++c)
        for (int t = 0; t < (bits == 8 ? 16 : 32); ++t)
            for (int b = 0; b < (bits == 8 ? 64 : 32); ++b) {
                const int slot = b >> 4, in_slot = b & 15;
                const size_t to = bits == 8
                    ? (size_t)c * 1024 + t * 64 + ((slot ^ swz64(t)) << 4) + in_slot
                    : (size_t)c * 1024 + t * 32 + ((slot ^ swz32(t)) << 4) + (in_slot ^ (half32(t) << 3));
                fill_blocks[to] = fill[(size_t)c * (bits == 8 ? 64 : 32) + b];
            }
    int rc = upload(&g9->d_fill, fill);
    if (rc == DGQ_OK) rc = upload(&g9->d_fill_blocks, fill_blocks);
    if (rc == DGQ_OK) rc = upload_tables(g9);
    if (rc != DGQ_OK) {
        release(g9);
        return rc;
    }
    *out = reinterpret_cast<dgq_groups_t *>(g9);
    return DGQ_OK;
}

int dgq_conv3x3_codes(const dgq_groups_t *h9, const int8_t *codes, int32_t B, int32_t H, int32_t W,
                      int8_t *codes9, void *stream) {
    if (!h9 || !codes || !codes9) return fail(DGQ_EINVAL, "dgq_conv3x3_codes: null pointer");
    if (B < 1 || H < 1 || W < 1) return fail(DGQ_EINVAL, "dgq_conv3x3_codes: empty shape");
    const Groups *g9 = reinterpret_cast<const Groups *>(h9);
    if (g9->conv_taps != 9)
        return fail(DGQ_ESHAPE, "dgq_conv3x3_codes: the handle does not come from dgq_groups_for_conv3x3");
    if (!aligned16(codes) || !aligned16(codes9))
        return fail(DGQ_EALIGN, "dgq_conv3x3_codes: tensor not 16-byte aligned");
    if ((int64_t)B * H * W > ((int64_t)1 << 31))
        return fail(DGQ_EUNSUPPORTED, "dgq_conv3x3_codes: too many pixels");
    DGQ_HIP(launch_conv3x3_codes(*g9, codes, B, H, W, codes9, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

size_t dgq_conv3x3_codes3_bytes(const dgq_groups_t *h9, int32_t B, int32_t H, int32_t W) {
    if (!h9 || B < 1 || H < 1 || W < 1) return 0;
    const Groups *g9 = reinterpret_cast<const Groups *>(h9);
    if (g9->conv_taps != 9) return 0;
    const int64_t rpb = g9->info.act_bits == 8 ? 16 : 32;
    const int64_t rows = (int64_t)B * H * W;
    return (size_t)(3 * ((rows + rpb - 1) / rpb) * (int64_t)(g9->base_kp / kGranule) * 1024);
}

int dgq_quantize_act_conv3x3(const dgq_groups_t *h, const dgq_groups_t *h9, const float *x, int32_t B,
                             int32_t H, int32_t W, int8_t *codes3, uint8_t *row_class, void *stream) {
    if (!h || !h9 || !x || !codes3 || !row_class)
        return fail(DGQ_EINVAL, "dgq_quantize_act_conv3x3: null pointer");
    if (B < 1 || H < 1 || W < 1) return fail(DGQ_EINVAL, "dgq_quantize_act_conv3x3: empty shape");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const Groups *g9 = reinterpret_cast<const Groups *>(h9);
    if (g9->conv_taps != 9 || g9->base_kp != g->info.k_padded || g9->info.act_bits != g->info.act_bits ||
        g9->info.channels != 9 * g->info.channels || g->info.n_pixel_classes != 1)
        return fail(DGQ_ESHAPE, "dgq_quantize_act_conv3x3: g9 does not come from dgq_groups_for_conv3x3(g)");
    if (W % (g->info.act_bits == 8 ? 16 : 32))
        return fail(DGQ_EUNSUPPORTED,
                    "dgq_quantize_act_conv3x3: the image width must be a multiple of 16 (8-bit codes) or "
                    "32 (4-bit codes); use dgq_quantize_act + dgq_conv3x3_codes otherwise");
    if (g->info.channels % 4 || g->info.channels >= 65535)
        return fail(DGQ_EUNSUPPORTED, "dgq_quantize_act_conv3x3: channels must be a multiple of 4");
    if (!aligned16(x) || !aligned16(codes3))
        return fail(DGQ_EALIGN, "dgq_quantize_act_conv3x3: tensor not 16-byte aligned");
    if ((int64_t)B * H * W > ((int64_t)1 << 31))
        return fail(DGQ_EUNSUPPORTED, "dgq_quantize_act_conv3x3: too many pixels");
    if (quantize_act_lds_bytes(*g) > 160 * 1024)
        return fail(DGQ_EUNSUPPORTED, "dgq_quantize_act_conv3x3: too many channels for the LDS row buffers");
    const int64_t rows = (int64_t)B * H * W;
    const int64_t copy_bytes = (int64_t)(dgq_conv3x3_codes3_bytes(h9, B, H, W) / 3);
    DGQ_HIP(launch_quantize_act(*g, x, rows, codes3, row_class, static_cast<hipStream_t>(stream), W, copy_bytes,
                                reinterpret_cast<const uint32_t *>(g9->d_fill)));
    return DGQ_OK;
}

int dgq_linear_conv3x3(const dgq_groups_t *h9, const dgq_weight_t *hw, const int8_t *codes3,
                       const uint8_t *row_class, int32_t B, int32_t H, int32_t W, float *y, void *stream) {
    if (!h9 || !hw || !codes3 || !row_class || !y) return fail(DGQ_EINVAL, "dgq_linear_conv3x3: null pointer");
    if (B < 1 || H < 1 || W < 1) return fail(DGQ_EINVAL, "dgq_linear_conv3x3: empty shape");
    const Groups *g9 = reinterpret_cast<const Groups *>(h9);
    const Weight *w = reinterpret_cast<const Weight *>(hw);
    if (g9->conv_taps != 9) return fail(DGQ_ESHAPE, "dgq_linear_conv3x3: the handle does not come from dgq_groups_for_conv3x3");
    if (w->groups != g9) return fail(DGQ_ESHAPE, "dgq_linear_conv3x3: weight was packed for a different group handle");
    if (w->next_kp) return fail(DGQ_ESHAPE, "dgq_linear_conv3x3: weight was packed for dgq_linear_geglu_requant");
    if (w->d_wq4) return fail(DGQ_EUNSUPPORTED, "dgq_linear_conv3x3: nibble-packed weights are taken by dgq_linear only");
    if (W % (g9->info.act_bits == 8 ? 16 : 32))
        return fail(DGQ_EUNSUPPORTED, "dgq_linear_conv3x3: the image width must be a multiple of 16 (8-bit codes) or 32 (4-bit codes)");
    if (!aligned16(codes3) || !aligned16(y)) return fail(DGQ_EALIGN, "dgq_linear_conv3x3: tensor not 16-byte aligned");
    const int64_t rows = (int64_t)B * H * W;
    if (rows > ((int64_t)1 << 31) || (rows + 127) / 128 * (int64_t)(w->O_pad / kTileO) > (int64_t)1 << 30)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear_conv3x3: too many output tiles");
    DGQ_HIP(launch_linear_conv3x3(*g9, *w, codes3, row_class, B, H, W, y, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

int dgq_groups_thresholds(const dgq_groups_t *h, float *taus) {
    if (!h || !taus) return fail(DGQ_EINVAL, "dgq_groups_thresholds: null pointer");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const int32_t n = std::max(g->info.n_pixel_classes - 1, 0);
    for (int32_t k = 0; k < n; ++k) taus[k] = g->taus[k];
    return DGQ_OK;
}

int dgq_groups_tables(const dgq_groups_t *h, int32_t *perm, int32_t *goff, int32_t *glen, float *s,
                      float *z) {
    if (!h) return fail(DGQ_EINVAL, "dgq_groups_tables: null handle");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    if (perm) std::memcpy(perm, g->perm.data(), g->perm.size() * sizeof(int32_t));
    if (goff) std::memcpy(goff, g->goff.data(), g->goff.size() * sizeof(int32_t));
    if (glen) std::memcpy(glen, g->glen.data(), g->glen.size() * sizeof(int32_t));
    if (s) std::memcpy(s, g->s.data(), g->s.size() * sizeof(float));
    if (z) std::memcpy(z, g->z.data(), g->z.size() * sizeof(float));
    return DGQ_OK;
}

void dgq_groups_free(dgq_groups_t *h) {
    if (!h) return;
    release(reinterpret_cast<Groups *>(h));
}

namespace {

// Packs w for the layer described by g.  With `next` (a following layer with one pixel
// class and 8-bit codes whose input is this layer's gated output) the packed rows are in
// that layer's K' order -- value rows for positions 0 .. K'_next - 1, then the gate rows of
// the same positions, all-zero rows at padding positions -- and the handle carries the
// per-chunk (offset, 1 / step) and the padding mask of that layer's quantizer.
int pack_weight(const char *who, const Groups *g, const Groups *next, const float *w,
                const float *bias, int32_t out_channels, int32_t w_bits, hipStream_t st,
                dgq_weight_t **out) {
    Weight *wt = new (std::nothrow) Weight();
    if (!wt) return fail(DGQ_EINVAL, std::string(who) + ": out of host memory");
    wt->groups = g;
    g->refs.fetch_add(1, std::memory_order_relaxed);
    wt->O = next ? 2 * next->info.k_padded : out_channels;
    wt->O_pad = (wt->O + kTileO - 1) / kTileO * kTileO;
    wt->C = g->info.channels;
    wt->Kp = g->info.k_padded;
    wt->w_bits = w_bits;
    (void)hipGetDevice(&wt->device);
    DevBuf row_map;
    hipError_t e = hipSuccess;
    if (next) {
        const int32_t kn = next->info.k_padded, half = out_channels / 2;
        wt->next_channels = half;
        wt->next_kp = kn;
        wt->next_bits = next->info.act_bits;
        std::vector<int32_t> map((size_t)2 * kn);
        std::vector<uint8_t> keep((size_t)kn);
        std::vector<float2> zi((size_t)next->n_chunks);
        for (int32_t j = 0; j < kn; ++j) {
            const int32_t c = next->perm[j];
            map[j] = c;
            map[(size_t)kn + j] = c < 0 ? -1 : half + c;
            keep[j] = c < 0 ? 0 : 0xFF;
        }
        const int32_t NG = (int32_t)next->glen.size();
        for (int32_t k = 0; k < NG; ++k)
            for (int32_t ch = next->goff[k] / kGranule; ch < next->goff[k + 1] / kGranule; ++ch)
                zi[ch] = make_float2(next->z[k], next->inv_s[k]);  // class row 0
        e = row_map.alloc(map.size() * sizeof(int32_t));
        if (e == hipSuccess)
            e = hipMemcpy(row_map.p, map.data(), map.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&wt->d_rq_zi), zi.size() * sizeof(float2));
        if (e == hipSuccess)
            e = hipMemcpy(wt->d_rq_zi, zi.data(), zi.size() * sizeof(float2), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&wt->d_rq_keep), keep.size());
        if (e == hipSuccess) e = hipMemcpy(wt->d_rq_keep, keep.data(), keep.size(), hipMemcpyHostToDevice);
    }
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&wt->d_wq), (size_t)wt->O_pad * wt->Kp);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&wt->d_sw), sizeof(float) * wt->O_pad);
    if (e == hipSuccess)
        e = hipMalloc(reinterpret_cast<void **>(&wt->d_zb), sizeof(float) * 2 * wt->O_pad);
    if (e == hipSuccess)
        e = launch_pack_weight(w, bias, wt->O, wt->O_pad, wt->C, wt->Kp, g->info.n_groups, w_bits,
                               g->info.code_offset, g->d_perm, g->d_gchunk, g->d_s, g->d_z,
                               g->n_tab, next ? row_map.as<int32_t>() : nullptr, wt->d_wq,
                               wt->d_sw, wt->d_zb, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        release(wt);
        return hip_fail(e, who);
    }
    *out = reinterpret_cast<dgq_weight_t *>(wt);
    return DGQ_OK;
}

}  // namespace

int dgq_pack_weight(const dgq_groups_t *h, const float *w, const float *bias, int32_t out_channels,
                    int32_t w_bits, void *stream, dgq_weight_t **out) {
    if (!h || !w || !out) return fail(DGQ_EINVAL, "dgq_pack_weight: null pointer");
    *out = nullptr;
    if (out_channels < 1) return fail(DGQ_EINVAL, "dgq_pack_weight: out_channels < 1");
    if (w_bits != 4 && w_bits != 8) return fail(DGQ_EINVAL, "dgq_pack_weight: w_bits must be 4 or 8");
    if (!aligned16(w) || (bias && !aligned16(bias)))
        return fail(DGQ_EALIGN, "dgq_pack_weight: tensor not 16-byte aligned");
    return pack_weight("dgq_pack_weight", reinterpret_cast<const Groups *>(h), nullptr, w, bias,
                       out_channels, w_bits, static_cast<hipStream_t>(stream), out);
}

int dgq_pack_weight_gated_for(const dgq_groups_t *h, const dgq_groups_t *h_next, const float *w,
                              const float *bias, int32_t out_channels, int32_t w_bits,
                              void *stream, dgq_weight_t **out) {
    if (!h || !h_next || !w || !out) return fail(DGQ_EINVAL, "dgq_pack_weight_gated_for: null pointer");
    *out = nullptr;
    if (out_channels < 2 || out_channels % 2)
        return fail(DGQ_EINVAL, "dgq_pack_weight_gated_for: out_channels must be even (value and gate halves)");
    if (w_bits != 4 && w_bits != 8)
        return fail(DGQ_EINVAL, "dgq_pack_weight_gated_for: w_bits must be 4 or 8");
    if (!aligned16(w) || (bias && !aligned16(bias)))
        return fail(DGQ_EALIGN, "dgq_pack_weight_gated_for: tensor not 16-byte aligned");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const Groups *next = reinterpret_cast<const Groups *>(h_next);
    if (next->info.channels != out_channels / 2)
        return fail(DGQ_ESHAPE, "dgq_pack_weight_gated_for: the following layer must take out_channels / 2 channels");
    if (next->info.n_pixel_classes != 1)
        return fail(DGQ_EUNSUPPORTED,
                    "dgq_pack_weight_gated_for: the following layer needs one pixel class (its "
                    "quantizer must not depend on a row statistic)");
    if (g->n_tab > 2)
        return fail(DGQ_EUNSUPPORTED, "dgq_pack_weight_gated_for: this layer needs at most two pixel classes");
    return pack_weight("dgq_pack_weight_gated_for", g, next, w, bias, out_channels, w_bits,
                       static_cast<hipStream_t>(stream), out);
}

int dgq_weight_tables(const dgq_weight_t *h, int8_t *wq, float *sw) {
    if (!h) return fail(DGQ_EINVAL, "dgq_weight_tables: null handle");
    const Weight *w = reinterpret_cast<const Weight *>(h);
    if (w->next_kp)
        return fail(DGQ_EUNSUPPORTED, "dgq_weight_tables: rows of a weight packed for a following layer are not in the original order");
    if (sw) DGQ_HIP(hipMemcpy(sw, w->d_sw, sizeof(float) * w->O, hipMemcpyDeviceToHost));
    if (wq) {
        DevBuf tmp, wide;
        const size_t bytes = (size_t)w->O * w->C;
        DGQ_HIP(tmp.alloc(bytes));
        DGQ_HIP(hipMemset(tmp.p, 0, bytes));
        const int8_t *src = w->d_wq;
        if (w->d_wq4) {  // two weights per byte: widen into a temporary first
            const int64_t n8 = (int64_t)w->O_pad * w->Kp;
            DGQ_HIP(wide.alloc((size_t)n8));
            DGQ_HIP(launch_expand_nibbles(w->d_wq4, wide.as<int8_t>(), n8, nullptr));
            src = wide.as<int8_t>();
        }
        DGQ_HIP(launch_unpack_weight(src, w->O, w->C, w->Kp, w->groups->d_perm,
                                     tmp.as<int8_t>(), nullptr));
        DGQ_HIP(hipDeviceSynchronize());
        DGQ_HIP(hipMemcpy(wq, tmp.p, bytes, hipMemcpyDeviceToHost));
    }
    return DGQ_OK;
}

int dgq_weight_pack_nibbles(dgq_weight_t *h, void *stream) {
    if (!h) return fail(DGQ_EINVAL, "dgq_weight_pack_nibbles: null handle");
    Weight *w = reinterpret_cast<Weight *>(h);
    if (w->d_wq4) return fail(DGQ_ESHAPE, "dgq_weight_pack_nibbles: the handle is already nibble-packed");
    if (w->w_bits != 4)
        return fail(DGQ_EUNSUPPORTED, "dgq_weight_pack_nibbles: the weights were quantized to 8 bits");
    if (w->next_kp)
        return fail(DGQ_EUNSUPPORTED, "dgq_weight_pack_nibbles: handles of dgq_pack_weight_gated_for feed "
                                      "dgq_linear_geglu_requant, which takes one weight per byte");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n8 = (int64_t)w->O_pad * w->Kp;  // O_pad and K' are multiples of 64
    uint8_t *p4 = nullptr;
    DGQ_HIP(hipMalloc(reinterpret_cast<void **>(&p4), (size_t)(n8 / 2)));
    hipError_t e = launch_pack_nibbles(w->d_wq, p4, n8, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        (void)hipFree(p4);
        return hip_fail(e, "dgq_weight_pack_nibbles");
    }
    (void)hipFree(w->d_wq);
    w->d_wq = nullptr;
    w->d_wq4 = p4;
    return DGQ_OK;
}

size_t dgq_weight_device_bytes(const dgq_weight_t *h) {
    if (!h) return 0;
    const Weight *w = reinterpret_cast<const Weight *>(h);
    const size_t n8 = (size_t)w->O_pad * w->Kp;
    size_t b = (w->d_wq4 ? n8 / 2 : n8) + sizeof(float) * 3 * (size_t)w->O_pad;
    if (w->next_kp) b += sizeof(float2) * (size_t)(w->next_kp / kGranule) + (size_t)w->next_kp;
    return b;
}

void dgq_weight_free(dgq_weight_t *h) {
    if (!h) return;
    release(reinterpret_cast<Weight *>(h));
}

int dgq_quantize_act(const dgq_groups_t *h, const float *x, int64_t rows, int8_t *codes,
                     uint8_t *row_class, void *stream) {
    if (!h || !x || !codes || !row_class) return fail(DGQ_EINVAL, "dgq_quantize_act: null pointer");
    if (rows < 1) return fail(DGQ_EINVAL, "dgq_quantize_act: rows < 1");
    if (!aligned16(x) || !aligned16(codes))
        return fail(DGQ_EALIGN, "dgq_quantize_act: tensor not 16-byte aligned");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    if (quantize_act_lds_bytes(*g) > 160 * 1024)
        return fail(DGQ_EUNSUPPORTED, "dgq_quantize_act: too many channels for the LDS row buffers (about 7500)");
    DGQ_HIP(launch_quantize_act(*g, x, rows, codes, row_class, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

size_t dgq_codes_bytes(const dgq_groups_t *h, int64_t rows) {
    if (!h || rows < 1) return 0;
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const int64_t block_rows = g->info.act_bits == 8 ? 16 : 32;
    return (size_t)((rows + block_rows - 1) / block_rows) * (size_t)g->n_chunks * 1024;
}

size_t dgq_linear_workspace_bytes(const dgq_groups_t *, const dgq_weight_t *hw, int64_t) {
    if (!hw) return 0;
    const Weight *w = reinterpret_cast<const Weight *>(hw);
    return w->d_wq4 ? (size_t)w->O_pad * w->Kp : 0;  // the weights at one byte each
}

int dgq_linear(const dgq_groups_t *h, const dgq_weight_t *hw, const int8_t *codes,
               const uint8_t *row_class, int64_t rows, float *y, int32_t *acc_dump, void *workspace,
               size_t workspace_bytes, void *stream) {
    if (!h || !hw || !codes || !row_class || !y) return fail(DGQ_EINVAL, "dgq_linear: null pointer");
    if (rows < 1) return fail(DGQ_EINVAL, "dgq_linear: rows < 1");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const Weight *w = reinterpret_cast<const Weight *>(hw);
    if (w->groups != g)
        return fail(DGQ_ESHAPE, "dgq_linear: weight was packed for a different group handle");
    if (!aligned16(codes) || !aligned16(y) || (acc_dump && !aligned16(acc_dump)))
        return fail(DGQ_EALIGN, "dgq_linear: tensor not 16-byte aligned");
    if ((rows + 127) / 128 * (int64_t)(w->O_pad / kTileO) > (int64_t)1 << 30)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear: too many output tiles");
    if (g->n_tab > 2 && acc_dump)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear: acc_dump needs at most two pixel classes");
    if (w->next_kp)
        return fail(DGQ_ESHAPE, "dgq_linear: weight was packed for dgq_linear_geglu_requant");
    if (w->d_wq4) {
        // two weights per byte at rest: widened into the caller's workspace, then the
        // contraction as for any other handle
        const size_t need = (size_t)w->O_pad * w->Kp;
        if (!workspace || workspace_bytes < need)
            return fail(DGQ_EWORKSPACE, "dgq_linear: nibble-packed weights need a workspace of dgq_linear_workspace_bytes()");
        if (!aligned16(workspace)) return fail(DGQ_EALIGN, "dgq_linear: workspace not 16-byte aligned");
        DGQ_HIP(launch_expand_nibbles(w->d_wq4, static_cast<int8_t *>(workspace), (int64_t)need,
                                      static_cast<hipStream_t>(stream)));
        Weight wide = *w;
        wide.d_wq = static_cast<int8_t *>(workspace);
        DGQ_HIP(launch_linear(*g, wide, codes, row_class, rows, y, acc_dump, 0, nullptr,
                              static_cast<hipStream_t>(stream)));
        return DGQ_OK;
    }
    DGQ_HIP(launch_linear(*g, *w, codes, row_class, rows, y, acc_dump, 0, nullptr,
                          static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

int dgq_linear_geglu(const dgq_groups_t *h, const dgq_weight_t *hw, const int8_t *codes,
                     const uint8_t *row_class, int64_t rows, float *y, void *stream) {
    if (!h || !hw || !codes || !row_class || !y)
        return fail(DGQ_EINVAL, "dgq_linear_geglu: null pointer");
    if (rows < 1) return fail(DGQ_EINVAL, "dgq_linear_geglu: rows < 1");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const Weight *w = reinterpret_cast<const Weight *>(hw);
    if (w->groups != g)
        return fail(DGQ_ESHAPE, "dgq_linear_geglu: weight was packed for a different group handle");
    if (w->next_kp)
        return fail(DGQ_ESHAPE, "dgq_linear_geglu: weight was packed for dgq_linear_geglu_requant");
    if (w->d_wq4)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear_geglu: nibble-packed weights are taken by dgq_linear only");
    if (w->O % 256 != 0)
        return fail(DGQ_EUNSUPPORTED,
                    "dgq_linear_geglu: out_channels must be a multiple of 256 (value and gate "
                    "halves in whole 128-channel tiles)");
    if (g->n_tab > 2)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear_geglu: needs at most two pixel classes");
    if (!aligned16(codes) || !aligned16(y))
        return fail(DGQ_EALIGN, "dgq_linear_geglu: tensor not 16-byte aligned");
    if ((rows + 127) / 128 * (int64_t)(w->O_pad / kTileO) > (int64_t)1 << 30)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear_geglu: too many output tiles");
    DGQ_HIP(launch_linear(*g, *w, codes, row_class, rows, y, nullptr, 1, nullptr,
                          static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

int dgq_linear_geglu_requant(const dgq_groups_t *h, const dgq_weight_t *hw, const int8_t *codes,
                             const uint8_t *row_class, int64_t rows, int8_t *codes_next,
                             uint8_t *row_class_next, void *stream) {
    if (!h || !hw || !codes || !row_class || !codes_next || !row_class_next)
        return fail(DGQ_EINVAL, "dgq_linear_geglu_requant: null pointer");
    if (rows < 1) return fail(DGQ_EINVAL, "dgq_linear_geglu_requant: rows < 1");
    const Groups *g = reinterpret_cast<const Groups *>(h);
    const Weight *w = reinterpret_cast<const Weight *>(hw);
    if (w->groups != g)
        return fail(DGQ_ESHAPE, "dgq_linear_geglu_requant: weight was packed for a different group handle");
    if (!w->next_kp)
        return fail(DGQ_ESHAPE, "dgq_linear_geglu_requant: weight was not packed by dgq_pack_weight_gated_for");
    if (!aligned16(codes) || !aligned16(codes_next))
        return fail(DGQ_EALIGN, "dgq_linear_geglu_requant: tensor not 16-byte aligned");
    if ((rows + 127) / 128 * (int64_t)(w->O_pad / kTileO) > (int64_t)1 << 30)
        return fail(DGQ_EUNSUPPORTED, "dgq_linear_geglu_requant: too many output tiles");
    DGQ_HIP(launch_linear(*g, *w, codes, row_class, rows, reinterpret_cast<float *>(codes_next),
                          nullptr, 2, row_class_next, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

size_t dgq_xattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk) {
    return xattn_workspace_bytes(B, N, H, d, nk);
}

int dgq_xattn_logq(const float *q, const float *k, const float *v, const float *key_bias, int32_t B,
                   int32_t N, int32_t H, int32_t d, int32_t nk, int32_t attn_bits, float *out,
                   float *scale_out, uint8_t *codes_dump, void *workspace, size_t workspace_bytes,
                   void *stream) {
    if (!q || !k || !v || !out || !scale_out) return fail(DGQ_EINVAL, "dgq_xattn_logq: null pointer");
    if (B < 1 || N < 1 || H < 1) return fail(DGQ_EINVAL, "dgq_xattn_logq: empty tensor");
    if (attn_bits != 4 && attn_bits != 8)
        return fail(DGQ_EINVAL, "dgq_xattn_logq: attn_bits must be 4 or 8");
    if (nk < 2 || nk > 128 || d < 1 || d > 256)
        return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq: needs 2 <= nk <= 128 and 1 <= d <= 256");
    if (B > 65535 || H > 65535) return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq: B or H above 65535");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) ||
        (key_bias && !aligned16(key_bias)))
        return fail(DGQ_EALIGN, "dgq_xattn_logq: tensor not 16-byte aligned");
    const size_t need = xattn_workspace_min_bytes(B, N, H, d, nk);
    if (need && (!workspace || workspace_bytes < need || !aligned16(workspace)))
        return fail(DGQ_EWORKSPACE, "dgq_xattn_logq: workspace missing, too small or misaligned");
    DGQ_HIP(launch_xattn(q, k, v, key_bias, B, N, H, d, nk, attn_bits, out, scale_out, codes_dump,
                         workspace, workspace_bytes, nullptr, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

// ---- the attention for callers that cannot allocate ---------------------------------------
// dgq_xattn_logq keeps one float per (prompt, head, query) between its two kernels in a
// workspace the caller brings.  This variant keeps it in device memory that is part of the
// loaded library: a fixed array every GPU holds its own copy of.  The array's name is a
// host-side stand-in, not a device address; the address on the current device comes from
// hipGetSymbolAddress, once per device, and only that pointer is handed to kernels.
}  // extern "C"

// the row statistics of DGQ_XATTN_NOALLOC_MAX_ROWS rows and the per-piece maxima behind them
constexpr size_t kScratchFloats = DGQ_XATTN_NOALLOC_MAX_ROWS + (DGQ_XATTN_NOALLOC_MAX_ROWS >> 4) + 4096 + 64;
static __device__ __align__(256) float scratch[kScratchFloats];

namespace {
std::atomic<float *> g_scratch_ptr[kMaxDevices];

int scratch_on_current_device(float **out) {
    int dev = 0;
    DGQ_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_noalloc: device index above 63");
    float *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        DGQ_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym) return fail(DGQ_EHIP, "dgq_xattn_logq_noalloc: no device address for the scratch array");
        p = static_cast<float *>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release);  // the same value from every thread
    }
    *out = p;
    return DGQ_OK;
}
}  // namespace

extern "C" {

int dgq_xattn_logq_noalloc(const float *q, const float *k, const float *v, const float *key_bias,
                           int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk,
                           int32_t attn_bits, float *out, float *scale_out, uint8_t *codes_dump,
                           void *stream) {
    if (!q || !k || !v || !out || !scale_out)
        return fail(DGQ_EINVAL, "dgq_xattn_logq_noalloc: null pointer");
    if (B < 1 || N < 1 || H < 1) return fail(DGQ_EINVAL, "dgq_xattn_logq_noalloc: empty tensor");
    if (attn_bits != 4 && attn_bits != 8)
        return fail(DGQ_EINVAL, "dgq_xattn_logq_noalloc: attn_bits must be 4 or 8");
    if (nk < 2 || nk > 128 || d < 1 || d > 256)
        return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_noalloc: needs 2 <= nk <= 128 and 1 <= d <= 256");
    if (B > 65535 || H > 65535)
        return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_noalloc: B or H above 65535");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) ||
        (key_bias && !aligned16(key_bias)))
        return fail(DGQ_EALIGN, "dgq_xattn_logq_noalloc: tensor not 16-byte aligned");
    const size_t need = xattn_workspace_min_bytes(B, N, H, d, nk);
    if (need > sizeof(float) * DGQ_XATTN_NOALLOC_MAX_ROWS)
        return fail(DGQ_EWORKSPACE,
                    "dgq_xattn_logq_noalloc: B * H * N exceeds DGQ_XATTN_NOALLOC_MAX_ROWS; use "
                    "dgq_xattn_logq with a workspace");
    float *ws = nullptr;
    if (need) {
        const int rc = scratch_on_current_device(&ws);
        if (rc != DGQ_OK) return rc;
    }
    DGQ_HIP(launch_xattn(q, k, v, key_bias, B, N, H, d, nk, attn_bits, out, scale_out, codes_dump,
                         ws, sizeof(float) * kScratchFloats, nullptr, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

int dgq_xattn_logq_static(const float *q, const float *k, const float *v, const float *key_bias,
                          int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t attn_bits,
                          const float *scale_in, float *out, float *scale_out, uint8_t *codes_dump,
                          void *stream) {
    if (!q || !k || !v || !out || !scale_in)
        return fail(DGQ_EINVAL, "dgq_xattn_logq_static: null pointer");
    if (B < 1 || N < 1 || H < 1) return fail(DGQ_EINVAL, "dgq_xattn_logq_static: empty tensor");
    if (attn_bits != 4 && attn_bits != 8)
        return fail(DGQ_EINVAL, "dgq_xattn_logq_static: attn_bits must be 4 or 8");
    if (nk < 2 || nk > 128 || d < 1 || d > 256)
        return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_static: needs 2 <= nk <= 128 and 1 <= d <= 256");
    if (B > 65535 || H > 65535)
        return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_static: B or H above 65535");
    if (scale_in == scale_out)
        return fail(DGQ_EINVAL, "dgq_xattn_logq_static: scale_in and scale_out must differ");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) ||
        (key_bias && !aligned16(key_bias)))
        return fail(DGQ_EALIGN, "dgq_xattn_logq_static: tensor not 16-byte aligned");
    DGQ_HIP(launch_xattn(q, k, v, key_bias, B, N, H, d, nk, attn_bits, out, scale_out, codes_dump,
                         nullptr, 0, scale_in, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

int dgq_xattn_logq_intv(const float *q, const float *k, const uint8_t *v_codes, const float *v_params,
                        const float *key_bias, int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk,
                        int32_t attn_bits, float *out, float *scale_out, uint8_t *codes_dump,
                        int32_t *acc_dump, void *stream) {
    if (!q || !k || !v_codes || !v_params || !out || !scale_out)
        return fail(DGQ_EINVAL, "dgq_xattn_logq_intv: null pointer");
    if (B < 1 || N < 1 || H < 1) return fail(DGQ_EINVAL, "dgq_xattn_logq_intv: empty tensor");
    if (attn_bits != 4)
        return fail(DGQ_EUNSUPPORTED,
                    "dgq_xattn_logq_intv: the integer product needs 4-bit codes (q_v << (15 - code) "
                    "must fit the int32 accumulator)");
    if (nk < 2 || nk > 128 || d < 1 || d > 256)
        return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_intv: needs 2 <= nk <= 128 and 1 <= d <= 256");
    if (B > 65535 || H > 65535) return fail(DGQ_EUNSUPPORTED, "dgq_xattn_logq_intv: B or H above 65535");
    if (!aligned16(q) || !aligned16(k) || !aligned16(out) || (key_bias && !aligned16(key_bias)))
        return fail(DGQ_EALIGN, "dgq_xattn_logq_intv: tensor not 16-byte aligned");
    DGQ_HIP(launch_xattn_intv(q, k, v_codes, v_params, key_bias, B, N, H, d, nk, out, scale_out, codes_dump,
                              acc_dump, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

size_t dgq_selfattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d) {
    if (B < 1 || N < 1 || H < 1) return 0;
    return selfattn_workspace_bytes(B, N, H, d);
}

int dgq_selfattn_logq(const float *q, const float *k, const float *v, int32_t B, int32_t N, int32_t H,
                      int32_t d, int32_t attn_bits, const float *scale_in, float *out,
                      float *scale_out, uint8_t *codes_dump, void *workspace,
                      size_t workspace_bytes, void *stream) {
    if (!q || !k || !v || !scale_in || !out)
        return fail(DGQ_EINVAL, "dgq_selfattn_logq: null pointer");
    if (B < 1 || N < 1 || H < 1 || d < 1) return fail(DGQ_EINVAL, "dgq_selfattn_logq: empty shape");
    if (attn_bits != 4 && attn_bits != 8)
        return fail(DGQ_EINVAL, "dgq_selfattn_logq: attn_bits must be 4 or 8");
    if (d % 8 != 0 || d > 160)
        return fail(DGQ_EUNSUPPORTED, "dgq_selfattn_logq: head dimension must be a multiple of 8, at most 160");
    if ((int64_t)B * H > (1 << 20) || N > (1 << 20))
        return fail(DGQ_EUNSUPPORTED, "dgq_selfattn_logq: too many (prompt, head) pairs or tokens");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(workspace))
        return fail(DGQ_EALIGN, "dgq_selfattn_logq: tensor not 16-byte aligned");
    if (!workspace || workspace_bytes < selfattn_workspace_bytes(B, N, H, d))
        return fail(DGQ_ESHAPE, "dgq_selfattn_logq: workspace smaller than dgq_selfattn_workspace_bytes");
    DGQ_HIP(launch_selfattn(q, k, v, B, N, H, d, attn_bits, scale_in, out, scale_out, codes_dump,
                            workspace, static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

int dgq_quantize_value(const float *v, int32_t B, int32_t nk, int32_t H, int32_t d, int32_t v_bits,
                       float *v_hat, uint8_t *codes, float *params, void *stream) {
    if (!v || !v_hat) return fail(DGQ_EINVAL, "dgq_quantize_value: null pointer");
    if (B < 1 || nk < 1 || H < 1 || d < 1) return fail(DGQ_EINVAL, "dgq_quantize_value: empty tensor");
    if (v_bits != 4 && v_bits != 8) return fail(DGQ_EINVAL, "dgq_quantize_value: v_bits must be 4 or 8");
    if (B > 65535 || (int64_t)nk * d > (int64_t)1 << 30)
        return fail(DGQ_EUNSUPPORTED, "dgq_quantize_value: B above 65535 or a slice above 2^30 elements");
    if (!aligned16(v) || !aligned16(v_hat))
        return fail(DGQ_EALIGN, "dgq_quantize_value: tensor not 16-byte aligned");
    DGQ_HIP(launch_quantize_value(v, B, nk, H, d, v_bits, v_hat, codes, params,
                                  static_cast<hipStream_t>(stream)));
    return DGQ_OK;
}

}  // extern "C"
