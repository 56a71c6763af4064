// K1: fused row statistics + pixel-class decision + group affine quantizer.
//
// Linear quantizer of Section 3.1 with the per-cell scale and offset of
// Section 3.3:  q = clamp(rne((x - z[p,g]) * inv_s[p,g]), 0, 2^b - 1).
//
// HBM-bound: every fp32 input is read once (4 B) and one code is written
// (1 B at 8 bit, 0.5 B at 4 bit), plus one class byte per row.  One wavefront
// owns a row: it streams the row with 16-byte loads into its LDS slice while
// reducing max/min with wave shuffles, decides the pixel class, then gathers
// the row from LDS in the permuted K' order and writes the codes as dwords into
// the block-tiled layout the GEMM loads (64 contiguous bytes per row and chunk).
#include "dgq_internal.h"

namespace dgq {

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;

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

// q as a float in [0, qmax]; separate subtract and multiply (no contraction).
__device__ inline float quant1(float x, float z, float inv_s, float qmax) {
    const float t = __fsub_rn(x, z);
    const float u = __fmul_rn(t, inv_s);
    return fminf(fmaxf(rintf(u), 0.0f), qmax);
}

template <int BITS, bool VEC4>
__global__ __launch_bounds__(256) void k_quantize_act(
    const float *__restrict__ x, int64_t rows, int32_t C, int32_t Kp, int32_t n_chunks,
    const int32_t *__restrict__ perm, const float *__restrict__ chunk_z,
    const float *__restrict__ chunk_inv, float tau, int8_t *__restrict__ codes,
    uint8_t *__restrict__ row_class) {
    extern __shared__ float lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float *xs = lds + (size_t)wave * C;  // this wave's copy of the row
    constexpr float qmax = (float)((1 << BITS) - 1);
    constexpr int kOff = BITS == 8 ? 128 : 0;

    for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + wave; r < rows;
         r += (int64_t)gridDim.x * kWavesPerBlock) {
        const float *xr = x + r * C;
        float mx = -INFINITY, mn = INFINITY;
        if (VEC4) {
            const float4 *x4 = reinterpret_cast<const float4 *>(xr);
            float4 *s4 = reinterpret_cast<float4 *>(xs);
            for (int32_t c = lane; c < (C >> 2); c += kWave) {
                const float4 v = x4[c];
                s4[c] = v;
                mx = fmaxf(fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)), mx);
                mn = fminf(fminf(fminf(v.x, v.y), fminf(v.z, v.w)), mn);
            }
        } else {
            for (int32_t c = lane; c < C; c += kWave) {
                const float v = xr[c];
                xs[c] = v;
                mx = fmaxf(v, mx);
                mn = fminf(v, mn);
            }
        }
        mx = wave_max(mx);
        mn = wave_min(mn);
        const int p = __fsub_rn(mx, mn) > tau ? 1 : 0;
        if (lane == 0) row_class[r] = (uint8_t)p;
        const float *zt = chunk_z + p * n_chunks;
        const float *it = chunk_inv + p * n_chunks;
        // The LDS slice is private to this wave and a wave's LDS operations
        // complete in issue order, so a compiler-level fence is all that is needed.
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();

        if (BITS == 8) {
            const int4 *perm4 = reinterpret_cast<const int4 *>(perm);
            for (int32_t j4 = lane; j4 < (Kp >> 2); j4 += kWave) {
                const int32_t ch = j4 >> 4;  // 16 dwords per 64-position chunk
                const float z = zt[ch], is = it[ch];
                const int4 c = perm4[j4];
                uint32_t word = 0;
                const int32_t cc[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    int32_t code = 0;
                    if (cc[k] >= 0) code = (int32_t)quant1(xs[cc[k]], z, is, qmax) - kOff;
                    word |= ((uint32_t)code & 0xffu) << (8 * k);
                }
                // dword (j4 & 15) of chunk ch: slot (j4 >> 2) & 3, dword j4 & 3 of the slot
                *reinterpret_cast<uint32_t *>(codes + tiled64_offset(r, ch, n_chunks, (j4 >> 2) & 3) +
                                              (j4 & 3) * 4) = word;
            }
        } else {
            const int4 *perm4 = reinterpret_cast<const int4 *>(perm);
            for (int32_t j8 = lane; j8 < (Kp >> 3); j8 += kWave) {
                const int32_t ch = j8 >> 3;  // 8 dwords per 64-position chunk
                const float z = zt[ch], is = it[ch];
                const int4 c0 = perm4[2 * j8], c1 = perm4[2 * j8 + 1];
                const int32_t cc[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
                uint32_t word = 0;
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    uint32_t qv = 0;
                    if (cc[k] >= 0) qv = (uint32_t)quant1(xs[cc[k]], z, is, qmax);
                    // byte i of the dword holds position i (low nibble) and i + 4 (high)
                    word |= qv << (k < 4 ? 8 * k : 8 * (k - 4) + 4);
                }
                *reinterpret_cast<uint32_t *>(codes + tiled32_offset(r, ch, n_chunks, (j8 >> 2) & 1) +
                                              (j8 & 3) * 4) = word;
            }
        }
        // the next row overwrites xs
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace

hipError_t launch_quantize_act(const Groups &g, const float *x, int64_t rows, int8_t *codes,
                               uint8_t *row_class, hipStream_t st) {
    const int32_t C = g.info.channels, Kp = g.info.k_padded;
    const size_t lds = sizeof(float) * (size_t)C * kWavesPerBlock;
    int64_t blocks = (rows + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t cap = 256 * 8;  // a few resident blocks per CU; rows are strided over them
    if (blocks > cap) blocks = cap;
    const bool vec4 = (C % 4) == 0;
    using Kern = void (*)(const float *, int64_t, int32_t, int32_t, int32_t, const int32_t *,
                          const float *, const float *, float, int8_t *, uint8_t *);
    Kern kern;
    if (g.info.act_bits == 8)
        kern = vec4 ? k_quantize_act<8, true> : k_quantize_act<8, false>;
    else
        kern = vec4 ? k_quantize_act<4, true> : k_quantize_act<4, false>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), lds, st, x, rows, C, Kp,
                       g.n_chunks, g.d_perm, g.d_chunk_z, g.d_chunk_inv, g.info.tau_pix, codes,
                       row_class);
    return hipGetLastError();
}

}  // namespace dgq
