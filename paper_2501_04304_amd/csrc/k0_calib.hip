// Calibration-side kernels (not on the timed path): range reductions that feed
// the host clustering (Section 3.3, D_d and the grouping by range), and the
// per-output-channel weight quantizer that lays rows out in the K' order.
#include "dgq_internal.h"

namespace dgq {

namespace {

constexpr int kWave = 64;

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float t = __shfl_xor(v, o, kWave);
        v = t > v ? t : v;
    }
    return v;
}
__device__ inline float wave_min(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float t = __shfl_xor(v, o, kWave);
        v = t < v ? t : v;
    }
    return v;
}

// One wavefront per row; rows are strided over the grid.
__global__ __launch_bounds__(256) void k_row_minmax(const float *__restrict__ x, int64_t rows,
                                                    int32_t C, float *__restrict__ rmx,
                                                    float *__restrict__ rmn) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int64_t r = (int64_t)blockIdx.x * 4 + wave; r < rows; r += (int64_t)gridDim.x * 4) {
        const float *xr = x + r * C;
        float mx = -INFINITY, mn = INFINITY;
        for (int32_t c = lane; c < C; c += kWave) {
            float v = xr[c];
            mx = v > mx ? v : mx;
            mn = v < mn ? v : mn;
        }
        mx = wave_max(mx);
        mn = wave_min(mn);
        if (lane == 0) {
            rmx[r] = mx;
            rmn[r] = mn;
        }
    }
}

// Thread = channel, blockIdx.y = slab of rows.  part[slab][4][C].
__global__ __launch_bounds__(256) void k_col_minmax_by_class(
    const float *__restrict__ x, int64_t rows, int32_t C, const float *__restrict__ rmx,
    const float *__restrict__ rmn, float tau, int32_t slabs, float *__restrict__ part) {
    const int32_t c = blockIdx.x * 256 + threadIdx.x;
    const int32_t slab = blockIdx.y;
    const int64_t per = (rows + slabs - 1) / slabs;
    const int64_t r0 = slab * per;
    const int64_t r1 = r0 + per < rows ? r0 + per : rows;
    float mx[2] = {-INFINITY, -INFINITY}, mn[2] = {INFINITY, INFINITY};
    if (c < C) {
        for (int64_t r = r0; r < r1; ++r) {
            const float w = rmx[r] - rmn[r];
            const float v = x[r * C + c];
            if (w > tau) {
                mx[1] = v > mx[1] ? v : mx[1];
                mn[1] = v < mn[1] ? v : mn[1];
            } else {
                mx[0] = v > mx[0] ? v : mx[0];
                mn[0] = v < mn[0] ? v : mn[0];
            }
        }
        float *p = part + (int64_t)slab * 4 * C;
        p[0 * C + c] = mx[0];
        p[1 * C + c] = mn[0];
        p[2 * C + c] = mx[1];
        p[3 * C + c] = mn[1];
    }
}

// One block per output channel.  Dynamic LDS: int gsum[NG], int chunk2grp[n_chunks].
__global__ __launch_bounds__(256) void k_pack_weight(
    const float *__restrict__ w, const float *__restrict__ bias, int32_t O, int32_t C,
    int32_t Kp, int32_t NG, int32_t w_bits, int32_t code_offset,
    const int32_t *__restrict__ perm, const int32_t *__restrict__ gchunk,
    const float *__restrict__ s, const float *__restrict__ z, int32_t n_classes,
    const int32_t *__restrict__ row_map, int8_t *__restrict__ wq, float *__restrict__ sw,
    float *__restrict__ zb, int32_t O_pad) {
    extern __shared__ int32_t smem[];
    int32_t *gsum = smem;
    int32_t *chunk2grp = smem + NG;
    __shared__ float red[4];
    const int32_t o = blockIdx.x;
    const int tid = threadIdx.x;
    const int32_t n_chunks = Kp / kGranule;
    // position j of row o in the block-tiled layout
    auto at = [&](int32_t j) -> int8_t & {
        return wq[tiled64_offset(o, j >> 6, n_chunks, (j >> 4) & 3) + (j & 15)];
    };
    // the row of w and bias behind packed row o: itself, or the one a row map names
    const int32_t src = o >= O ? -1 : (row_map ? row_map[o] : o);
    if (src < 0) {  // padding rows: all-zero weights
        for (int32_t j = tid; j < Kp; j += 256) at(j) = 0;
        if (tid == 0) {
            sw[o] = 0.0f;
            zb[o] = 0.0f;
            zb[O_pad + o] = 0.0f;
        }
        return;
    }
    for (int32_t g = tid; g < NG; g += 256) {
        gsum[g] = 0;
        for (int32_t ch = gchunk[g]; ch < gchunk[g + 1]; ++ch) chunk2grp[ch] = g;
    }
    const float *wr = w + (int64_t)src * C;
    float amax = 0.0f;
    for (int32_t c = tid; c < C; c += 256) {
        float a = fabsf(wr[c]);
        amax = a > amax ? a : amax;
    }
    amax = wave_max(amax);
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float qmax = w_bits == 8 ? 127.0f : 7.0f;
    const float sc = amax > 0.0f ? amax / qmax : 1.0f;
    for (int32_t j = tid; j < Kp; j += 256) {
        const int32_t c = perm[j];
        int32_t v = 0;
        if (c >= 0) {
            float qf = rintf(wr[c] / sc);
            qf = fminf(fmaxf(qf, -qmax), qmax);
            v = (int32_t)qf;
            atomicAdd(&gsum[chunk2grp[j / kGranule]], v);
        }
        at(j) = (int8_t)v;
    }
    __syncthreads();
    if (n_classes > 2) {
        // more than two pixel classes come with a single channel group: the class enters
        // the zero-point term as one factor, zb[p][o] = zoff[p] * (sw[o] * wsum[o]) + bias[o],
        // and the two class-independent rows are stored instead of one row per class
        if (tid == 0) {
            zb[o] = (float)((double)sc * (double)gsum[0]);
            zb[O_pad + o] = bias ? bias[src] : 0.0f;
            sw[o] = sc;
        }
    } else if (tid < 2) {
        const int p = tid;
        double t = 0.0;
        for (int32_t g = 0; g < NG; ++g) {
            const double sg = (double)s[p * NG + g];
            const double zo = (double)z[p * NG + g] + (double)code_offset * sg;
            t += zo * (double)gsum[g];
        }
        double v = (double)sc * t;
        if (bias) v += (double)bias[src];
        zb[p * O_pad + o] = (float)v;
        if (p == 0) sw[o] = sc;
    }
}

__global__ __launch_bounds__(256) void k_unpack_weight(const int8_t *__restrict__ wq, int32_t O,
                                                       int32_t C, int32_t Kp,
                                                       const int32_t *__restrict__ perm,
                                                       int8_t *__restrict__ out) {
    const int32_t o = blockIdx.x;
    for (int32_t j = threadIdx.x; j < Kp; j += 256) {
        const int32_t c = perm[j];
        if (c >= 0)
            out[(int64_t)o * C + c] = wq[tiled64_offset(o, j >> 6, Kp >> 6, (j >> 4) & 3) + (j & 15)];
    }
}

}  // namespace

hipError_t launch_row_minmax(const float *x, int64_t rows, int32_t C, float *rmx, float *rmn,
                             hipStream_t st) {
    int64_t blocks = (rows + 3) / 4;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(k_row_minmax, dim3((unsigned)blocks), dim3(256), 0, st, x, rows, C, rmx, rmn);
    return hipGetLastError();
}

hipError_t launch_col_minmax_by_class(const float *x, int64_t rows, int32_t C, const float *rmx,
                                      const float *rmn, float tau, int32_t slabs, float *part,
                                      hipStream_t st) {
    dim3 grid((C + 255) / 256, slabs);
    hipLaunchKernelGGL(k_col_minmax_by_class, grid, dim3(256), 0, st, x, rows, C, rmx, rmn, tau,
                       slabs, part);
    return hipGetLastError();
}

hipError_t launch_pack_weight(const float *w, const float *bias, int32_t O, int32_t O_pad,
                              int32_t C, int32_t Kp, int32_t NG, int32_t w_bits,
                              int32_t code_offset, const int32_t *perm, const int32_t *gchunk,
                              const float *s, const float *z, int32_t n_classes,
                              const int32_t *row_map, int8_t *wq, float *sw, float *zb,
                              hipStream_t st) {
    const size_t lds = sizeof(int32_t) * (size_t)(NG + Kp / kGranule);
    hipLaunchKernelGGL(k_pack_weight, dim3(O_pad), dim3(256), lds, st, w, bias, O, C, Kp, NG,
                       w_bits, code_offset, perm, gchunk, s, z, n_classes, row_map, wq, sw, zb, O_pad);
    return hipGetLastError();
}

// Two signed 4-bit weights per byte.  A thread converts 32 weights: 16 packed bytes <-> 32.
__global__ __launch_bounds__(256) void k_pack_nibbles(const int8_t *__restrict__ wq,
                                                      uint8_t *__restrict__ wq4, int64_t n16) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 a = reinterpret_cast<const uint4 *>(wq)[2 * i];
    const uint4 b = reinterpret_cast<const uint4 *>(wq)[2 * i + 1];
    // bytes (w0 w1 w2 w3) of a dword pair -> (w0 | w1 << 4, w2 | w3 << 4, ...)
    auto two = [](uint32_t lo, uint32_t hi) {
        auto half = [](uint32_t x) {  // four weights -> two packed bytes
            const uint32_t n = x & 0x0f0f0f0fu;
            return ((n | (n >> 4)) & 0xffu) | (((n >> 16) | (n >> 20)) & 0xffu) << 8;
        };
        return half(lo) | (half(hi) << 16);
    };
    uint4 r;
    r.x = two(a.x, a.y);
    r.y = two(a.z, a.w);
    r.z = two(b.x, b.y);
    r.w = two(b.z, b.w);
    reinterpret_cast<uint4 *>(wq4)[i] = r;
}

__global__ __launch_bounds__(256) void k_expand_nibbles(const uint8_t *__restrict__ wq4,
                                                        int8_t *__restrict__ wq, int64_t n16) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 p = reinterpret_cast<const uint4 *>(wq4)[i];
    // two packed bytes -> four sign-extended weights: spread the nibbles over the bytes,
    // then (n ^ 8) - 8 in every byte without a borrow between bytes: the +0x80 keeps each
    // byte's subtraction from borrowing and is taken out again by the final xor
    auto four = [](uint32_t h) {  // h: 16 bits = four nibbles
        const uint32_t n = (h & 0xfu) | ((h & 0xf0u) << 4) | ((h & 0xf00u) << 8) | ((h & 0xf000u) << 12);
        return (((n ^ 0x88888888u) - 0x08080808u) ^ 0x80808080u);
    };
    uint4 a, b;
    a.x = four(p.x & 0xffffu);
    a.y = four(p.x >> 16);
    a.z = four(p.y & 0xffffu);
    a.w = four(p.y >> 16);
    b.x = four(p.z & 0xffffu);
    b.y = four(p.z >> 16);
    b.z = four(p.w & 0xffffu);
    b.w = four(p.w >> 16);
    reinterpret_cast<uint4 *>(wq)[2 * i] = a;
    reinterpret_cast<uint4 *>(wq)[2 * i + 1] = b;
}

hipError_t launch_pack_nibbles(const int8_t *wq, uint8_t *wq4, int64_t n_bytes8, hipStream_t st) {
    const int64_t n16 = n_bytes8 / 32;
    hipLaunchKernelGGL(k_pack_nibbles, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, wq, wq4, n16);
    return hipGetLastError();
}

hipError_t launch_expand_nibbles(const uint8_t *wq4, int8_t *wq, int64_t n_bytes8, hipStream_t st) {
    const int64_t n16 = n_bytes8 / 32;
    hipLaunchKernelGGL(k_expand_nibbles, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, wq4, wq, n16);
    return hipGetLastError();
}

hipError_t launch_unpack_weight(const int8_t *wq, int32_t O, int32_t C, int32_t Kp,
                                const int32_t *perm, int8_t *wq_out, hipStream_t st) {
    hipLaunchKernelGGL(k_unpack_weight, dim3(O), dim3(256), 0, st, wq, O, C, Kp, perm, wq_out);
    return hipGetLastError();
}

}  // namespace dgq
