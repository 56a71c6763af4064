// K3: text cross-attention with log2-quantized probabilities (Section 3.3,
// attention-aware quantization; log quantizer of Section 3.1).
//
//   L_ij = (Q_i . K_j) / sqrt(d) + key_bias_j,  A = softmax_j(L) over all keys (fp32)
//   s_b  = max over heads, queries and keys j >= 1 of A          (pass 1)
//   code = clamp(rne(-log2(A_ij / s_b)), 0, 2^bits - 1), j >= 1   (pass 2)
//   Out_i = A_i0 * V_0 + s_b * sum_{j>=1} 2^(-code_ij) * V_j
//
// The prompt scale is a maximum over every probability of the prompt, so no
// probability can be coded before all of them exist: two kernels.  Both
// recompute the logits from Q (a second read of Q costs less than storing the
// [N, nk] probabilities).  The code is evaluated in the log domain,
//   -log2(A/s) = log2(s) + log2(sum_j e^(L_ij - m_i)) - (L_ij - m_i) * log2(e),
// which needs no exponential per element and is exact to ~1e-6 in log2 units;
// a probability below 2^-150 rounds to zero in fp32 and takes the top code.
//
// One thread owns one (query, head) row: the nk logits live in registers, the
// keys (then the values, reusing the same LDS) of the (batch, head) pair are
// broadcast from LDS.
#include "dgq_internal.h"

namespace dgq {

namespace {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

__global__ void k_fill_zero(float *p, int32_t n) {
    const int32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0f;
}

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// Cooperative copy of one [nk, d] head slice (row stride H*d) into LDS
// [NKP][dpad], zero-filling the padding.
template <int NKP>
__device__ inline void stage_head(const float *__restrict__ src, int32_t nk, int32_t d,
                                  int32_t dpad, int64_t row_stride, float *dst) {
    for (int32_t idx = threadIdx.x; idx < NKP * dpad; idx += 256) {
        const int32_t j = idx / dpad, t = idx - j * dpad;
        dst[idx] = (j < nk && t < d) ? src[(int64_t)j * row_stride + t] : 0.0f;
    }
}

template <int NKP, int PASS>
__global__ __launch_bounds__(256) void k_xattn(
    const float *__restrict__ q, const float *__restrict__ k, const float *__restrict__ v,
    const float *__restrict__ key_bias, int32_t N, int32_t H, int32_t d, int32_t dpad, int32_t nk,
    int32_t bits, float inv_sqrt_d, float *__restrict__ out, float *__restrict__ scale,
    uint8_t *__restrict__ codes_dump) {
    extern __shared__ float kv[];  // [NKP][dpad]
    __shared__ float red[4];
    const int32_t b = blockIdx.z, h = blockIdx.y;
    const int32_t n_raw = blockIdx.x * 256 + threadIdx.x;
    const bool valid = n_raw < N;
    const int32_t n = valid ? n_raw : N - 1;
    const int64_t hs = (int64_t)H * d;  // stride between tokens

    stage_head<NKP>(k + ((int64_t)b * nk * H + h) * d, nk, d, dpad, hs, kv);
    __syncthreads();

    // ---- logits ------------------------------------------------------------------
    float L[NKP];
#pragma unroll
    for (int j = 0; j < NKP; ++j) L[j] = 0.0f;
    const float *qr = q + (((int64_t)b * N + n) * H + h) * d;
    const bool vec = (d & 3) == 0;
    for (int32_t t4 = 0; t4 < dpad; t4 += 4) {
        float4 qv;
        if (vec) {
            qv = *reinterpret_cast<const float4 *>(qr + t4);
        } else {
            qv.x = t4 + 0 < d ? qr[t4 + 0] : 0.0f;
            qv.y = t4 + 1 < d ? qr[t4 + 1] : 0.0f;
            qv.z = t4 + 2 < d ? qr[t4 + 2] : 0.0f;
            qv.w = t4 + 3 < d ? qr[t4 + 3] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < NKP; ++j) {
            const float4 kk = *reinterpret_cast<const float4 *>(kv + j * dpad + t4);
            L[j] = fmaf(qv.x, kk.x, L[j]);
            L[j] = fmaf(qv.y, kk.y, L[j]);
            L[j] = fmaf(qv.z, kk.z, L[j]);
            L[j] = fmaf(qv.w, kk.w, L[j]);
        }
    }
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < NKP; ++j) {
        if (j < nk) {
            L[j] = fmaf(L[j], inv_sqrt_d, key_bias ? key_bias[j] : 0.0f);
            m = fmaxf(m, L[j]);
        } else {
            L[j] = -INFINITY;
        }
    }
    // ---- softmax statistics in base 2 ----------------------------------------------
    float sum = 0.0f, l2max1 = -INFINITY;
#pragma unroll
    for (int j = 0; j < NKP; ++j) {
        L[j] = (L[j] - m) * kLog2e;  // log2 of the unnormalised probability (<= 0)
        sum += __builtin_amdgcn_exp2f(L[j]);
        if (j >= 1) l2max1 = fmaxf(l2max1, L[j]);
    }

    if (PASS == 1) {
        float amax = valid ? __builtin_amdgcn_exp2f(l2max1) / sum : 0.0f;
        amax = wave_max(amax);
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
        __syncthreads();
        if (threadIdx.x == 0) {
            amax = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
            // probabilities are non-negative: their bit patterns order like unsigned ints
            atomicMax(reinterpret_cast<unsigned int *>(scale + b), __float_as_uint(amax));
        }
        return;
    }

    // ---- pass 2: codes and de-quantized probabilities --------------------------------
    const float s = scale[b];
    const float l2s = __log2f(s);
    const float lse2 = __log2f(sum);
    const float qmax = (float)((1 << bits) - 1);
    const float a0 = __builtin_amdgcn_exp2f(L[0]) / sum;  // <start> column stays fp32
    uint8_t *cd = codes_dump
                      ? codes_dump + ((((int64_t)b * H + h) * N + n) * (int64_t)(nk - 1))
                      : nullptr;
#pragma unroll
    for (int j = 1; j < NKP; ++j) {
        if (j < nk) {
            const float l2a = L[j] - lse2;  // log2(A_ij)
            float c = fminf(fmaxf(rintf(l2s - l2a), 0.0f), qmax);
            if (l2a < -150.0f) c = qmax;  // A rounds to zero in fp32
            if (cd && valid) cd[j - 1] = (uint8_t)c;
            L[j] = ldexpf(s, -(int)c);
        } else {
            L[j] = 0.0f;
        }
    }
    L[0] = a0;

    // ---- product with V (V replaces K in LDS) ----------------------------------------
    __syncthreads();
    stage_head<NKP>(v + ((int64_t)b * nk * H + h) * d, nk, d, dpad, hs, kv);
    __syncthreads();
    float *orow = out + (((int64_t)b * N + n) * H + h) * d;
    for (int32_t t4 = 0; t4 < dpad; t4 += 4) {
        float4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int j = 0; j < NKP; ++j) {
            const float4 vv = *reinterpret_cast<const float4 *>(kv + j * dpad + t4);
            acc.x = fmaf(L[j], vv.x, acc.x);
            acc.y = fmaf(L[j], vv.y, acc.y);
            acc.z = fmaf(L[j], vv.z, acc.z);
            acc.w = fmaf(L[j], vv.w, acc.w);
        }
        if (valid) {
            if (vec) {
                *reinterpret_cast<float4 *>(orow + t4) = acc;
            } else {
                if (t4 + 0 < d) orow[t4 + 0] = acc.x;
                if (t4 + 1 < d) orow[t4 + 1] = acc.y;
                if (t4 + 2 < d) orow[t4 + 2] = acc.z;
                if (t4 + 3 < d) orow[t4 + 3] = acc.w;
            }
        }
    }
}

template <int NKP>
hipError_t launch_passes(const float *q, const float *k, const float *v, const float *key_bias,
                         int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
                         float *out, float *scale_out, uint8_t *codes_dump, hipStream_t st) {
    const int32_t dpad = (d + 3) / 4 * 4;
    const size_t lds = sizeof(float) * (size_t)NKP * dpad;
    const float inv_sqrt_d = (float)(1.0 / sqrt((double)d));
    const dim3 grid((N + 255) / 256, H, B);
    auto k1 = k_xattn<NKP, 1>;
    auto k2 = k_xattn<NKP, 2>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k1),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(k2),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    // scale_out accumulates a maximum: clear it with a fill kernel (capturable in a graph)
    hipLaunchKernelGGL(k_fill_zero, dim3((B + 63) / 64), dim3(64), 0, st, scale_out, B);
    hipLaunchKernelGGL(k1, grid, dim3(256), lds, st, q, k, v, key_bias, N, H, d, dpad, nk, bits,
                       inv_sqrt_d, out, scale_out, codes_dump);
    hipLaunchKernelGGL(k2, grid, dim3(256), lds, st, q, k, v, key_bias, N, H, d, dpad, nk, bits,
                       inv_sqrt_d, out, scale_out, codes_dump);
    return hipGetLastError();
}

}  // namespace

size_t xattn_workspace_bytes(int32_t, int32_t, int32_t, int32_t, int32_t) { return 0; }

hipError_t launch_xattn(const float *q, const float *k, const float *v, const float *key_bias,
                        int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
                        float *out, float *scale_out, uint8_t *codes_dump, void *, hipStream_t st) {
    if (nk <= 80)
        return launch_passes<80>(q, k, v, key_bias, B, N, H, d, nk, bits, out, scale_out,
                                 codes_dump, st);
    return launch_passes<128>(q, k, v, key_bias, B, N, H, d, nk, bits, out, scale_out, codes_dump,
                              st);
}

}  // namespace dgq
