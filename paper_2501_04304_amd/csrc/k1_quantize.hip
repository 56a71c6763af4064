// K1: fused row statistics + pixel-class decision + group affine quantizer.
//
// Linear quantizer of Section 3.1 with the per-cell scale and offset of
// Section 3.3:  q = clamp(rne((x - z[p,g]) * inv_s[p,g]), 0, 2^b - 1).
//
// HBM-bound: every fp32 input is read once (4 B) and one code is written
// (1 B at 8 bit, 0.5 B at 4 bit), plus one class byte per row.
//
// One wavefront owns a row.  The row arrives in registers with 16-byte loads
// (issued one row ahead, so the next row is in flight while the current one is
// processed), is reduced to max/min with wave shuffles, and is parked in the
// wave's LDS slice.  After the class decision every lane takes 4 (8-bit) or 8
// (4-bit) consecutive OUTPUT positions, gathers the inputs from LDS through the
// channel permutation, and writes one dword into the block-tiled code layout the
// GEMM loads (64 contiguous bytes per row and chunk; the four waves of a
// workgroup own four consecutive rows each of a 16-row block, so a 1 KiB block
// is completed by one workgroup).  Loaded once per workgroup into LDS: the
// permutation as byte offsets into the row slice (padding positions point at
// channel 0), one keep-mask per output dword that clears the padding positions
// of the packed word (so padding costs nothing per position), and the per-chunk
// (z, 1/s) pairs.  Per position that leaves: one address add, the gather, subtract,
// multiply, round, clamp and the byte pack.
#include "dgq_internal.h"

#include <cstdlib>
#include <type_traits>

namespace dgq {

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;

// Three-operand max / min as the instruction itself: written through the compiler's
// fmaxf they come wrapped in one canonicalising instruction per loaded value.
__device__ inline float max3(float a, float b, float c) {
    float d;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}
__device__ inline float min3(float a, float b, float c) {
    float d;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
    return d;
}

// Wave-wide maximum of mx and minimum of mn without LDS traffic, both returned as
// wave-uniform values.  Four cross-lane (DPP) steps leave every 16-lane row with its own
// extreme (lane ^ 1, lane ^ 2, mirrored halves, mirrored row), two row broadcasts carry
// it on to lane 63.  The two chains alternate and one s_nop separates the steps: a DPP
// operand may be read two wait states after the register was written at the earliest.
#define DGQ_DPP_STEP(ctrl)                                 \
    "v_max_f32_dpp %0, %0, %0 " ctrl " bank_mask:0xf\n\t" \
    "v_min_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t" \
    "s_nop 0\n\t"
__device__ inline void wave_max_min(float &mx, float &mn) {
    asm("s_nop 1\n\t"
        DGQ_DPP_STEP("quad_perm:[1,0,3,2] row_mask:0xf")
        DGQ_DPP_STEP("quad_perm:[2,3,0,1] row_mask:0xf")
        DGQ_DPP_STEP("row_half_mirror row_mask:0xf")
        DGQ_DPP_STEP("row_mirror row_mask:0xf")
        DGQ_DPP_STEP("row_bcast:15 row_mask:0xa")
        DGQ_DPP_STEP("row_bcast:31 row_mask:0xc")
        : "+v"(mx), "+v"(mn));
    mx = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mx), 63));
    mn = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mn), 63));
}
#undef DGQ_DPP_STEP

// q as a float in [0, qmax]; separate subtract and multiply (no contraction).
__device__ inline float quant1(float x, float z, float inv_s, float qmax) {
    const float t = __fsub_rn(x, z);
    const float u = __fmul_rn(t, inv_s);
    return fminf(fmaxf(rintf(u), 0.0f), qmax);
}

// The same value, unrounded, for v_cvt_pk_u8_f32 to finish: that instruction rounds to
// nearest even and saturates to [0, 255] (NaN -> 0) by itself (checked against
// rint + clamp on a million values, ties and the values next to them included), so at
// 8 bit nothing is left to do, and at 4 bit only the upper clamp, which commutes with
// the rounding because the bound is an integer.  v_med3_f32 returns the minimum of its
// operands when one is NaN, i.e. 0 here, as the three-step form does.
template <int BITS>
__device__ inline float quant_pre(float x, float z, float inv_s) {
    const float t = __fsub_rn(x, z);
    const float u = __fmul_rn(t, inv_s);
    return BITS == 8 ? u : __builtin_amdgcn_fmed3f(u, 0.0f, 15.0f);
}

// LDS: [off32: kPer u32 per output dword][keep: one u32 per output dword]
//      [cz: classes x chunks float2][rows: 4 * C floats].
// The tables are padded to whole steps of 64 output dwords (a step is what the 64 lanes
// do at once), so a lane of the last, partly filled step reads valid table entries
// (offset 0, keep-mask 0) and only its store is predicated.
struct QuantLds {
    int32_t n_dw, n_steps, n_dw_pad, nch_pad;
    size_t off_bytes, keep_bytes, cz_bytes;
    __host__ __device__ QuantLds(int32_t Kp, int bits, int classes) {
        const int per = bits == 8 ? 4 : 8;
        n_dw = Kp / per;
        n_steps = (n_dw + 63) >> 6;
        n_dw_pad = n_steps * 64;
        nch_pad = n_dw_pad / (64 / per);
        off_bytes = (size_t)n_dw_pad * per * 4;
        keep_bytes = (size_t)n_dw_pad * 4;
        cz_bytes = (size_t)classes * nch_pad * 8;
    }
    __host__ __device__ size_t table_bytes() const { return off_bytes + keep_bytes + cz_bytes; }
};

// NV: float4 registers per lane that hold one row (C <= NV * 256).
template <int BITS, int NV>
__global__ __launch_bounds__(256) void k_quantize_act(
    const float *__restrict__ x, int64_t rows, int32_t C, int32_t Kp, int32_t n_chunks,
    const int32_t *__restrict__ perm, const float *__restrict__ chunk_z,
    const float *__restrict__ chunk_inv, const float *__restrict__ taus, int32_t n_tau,
    int8_t *__restrict__ codes, uint8_t *__restrict__ row_class, int32_t rpw_log2,
    int32_t conv_w, int64_t copy_bytes, const uint32_t *__restrict__ fill32) {
    // conv_w > 0: the rows are the pixels of images conv_w wide and the codes are written three
    // times for the tap-gathering 3 x 3 convolution: copy 1 (codes + copy_bytes) is the map
    // itself, copy 0 holds in row r the codes of the pixel left of r, copy 2 of the pixel right
    // of r, and the code of the value 0 (fill32, one dword per output dword) where the image ends.
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_raw[];
    constexpr int kPer = BITS == 8 ? 4 : 8;          // positions per output dword
    constexpr int kDwPerChunk = 64 / kPer;           // 16 or 8
    constexpr int kChunkStep = kWave / kDwPerChunk;  // chunks per step: 4 or 8
    const QuantLds L(Kp, BITS, n_tau + 1);
    uint32_t *off32 = reinterpret_cast<uint32_t *>(lds_raw);
    uint32_t *keep = reinterpret_cast<uint32_t *>(lds_raw + L.off_bytes);
    float2 *cz = reinterpret_cast<float2 *>(lds_raw + L.off_bytes + L.keep_bytes);
    float *rowbuf = reinterpret_cast<float *>(lds_raw + L.table_bytes());
    const int tid = threadIdx.x;
    // the wave index as a scalar: rows, row pointers and classes are then wave-uniform
    // values in scalar registers and the loads and stores take scalar bases
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    float *xs = rowbuf + (size_t)wave * C;  // this wave's copy of the row
    const uint32_t c4n = (uint32_t)C >> 2;  // float4 per row
    const int32_t n_dw = L.n_dw;

    // rows: a workgroup takes units of 4 << rpw_log2 consecutive rows, wave w the rows
    // (w << rpw_log2) .. of the unit, one after the other.  rpw_log2 = 2: a unit is one
    // 16-row block of the tiled code layout; rpw_log2 = 0 (few rows): a quarter of one,
    // so that four times as many workgroups share the work.
    const int32_t us = 2 + rpw_log2;
    const int64_t n_units = (rows + (1 << us) - 1) >> us;
    auto row_of = [&](int64_t it) -> int64_t {  // it-th row of this wave's sequence
        const int64_t u = (int64_t)blockIdx.x + (it >> rpw_log2) * gridDim.x;
        return u < n_units ? (u << us) + (wave << rpw_log2) + (it & ((1 << rpw_log2) - 1)) : rows;
    };
    // A lane index past the end of the row is clamped to the last valid one, which
    // re-reads a value that is already part of the row, so max/min and the LDS copy are
    // unaffected.
    float4 v[NV];
    uint32_t cidx[NV];
#pragma unroll
    for (int k = 0; k < NV; ++k) {
        const uint32_t c = lane + k * kWave;
        cidx[k] = c < c4n ? c : c4n - 1;
    }
    auto fetch = [&](int64_t r) {  // r < rows, wave-uniform
        const float4 *x4 = reinterpret_cast<const float4 *>(x + r * C);
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            // the activations are read exactly once: non-temporal, keep the caches for the codes
            typedef float v4f __attribute__((ext_vector_type(4)));
            const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(x4 + cidx[k]));
            v[k] = make_float4(t.x, t.y, t.z, t.w);
        }
    };

    // the first row travels while the tables are built
    int64_t it = 0;
    int64_t r = row_of(0);
    if (r < rows) fetch(r);

    for (int32_t d = tid; d < L.n_dw_pad; d += 256) {
        uint32_t m = 0;
#pragma unroll
        for (int k = 0; k < kPer; ++k) {
            const int32_t j = d * kPer + k;
            const int32_t c = j < Kp ? perm[j] : -1;
            off32[j] = c >= 0 ? (uint32_t)c * 4u : 0u;
            // 8 bit: byte k of the word; 4 bit: byte k % 4, low nibble for k < 4, high otherwise
            const uint32_t field = BITS == 8 ? 0xffu << (8 * k) : 0xfu << (8 * (k & 3) + 4 * (k >> 2));
            if (c >= 0) m |= field;
        }
        keep[d] = m;
    }
    for (int32_t i = tid; i < (n_tau + 1) * L.nch_pad; i += 256) {
        const int32_t p = i / L.nch_pad, ch = i - p * L.nch_pad;
        cz[i] = ch < n_chunks ? make_float2(chunk_z[p * n_chunks + ch], chunk_inv[p * n_chunks + ch])
                              : make_float2(0.0f, 0.0f);
    }
    __syncthreads();

    // Output dword d of the row covers positions 4d..4d+3 (8 bit) or 8d..8d+7 (4 bit).
    // Lane l handles dwords l, l + 64, ... (one per step); in the tiled layout that is a
    // fixed place inside a 64-byte (32-byte) row segment and a chunk index that advances
    // by 4 (8 bit) or 8 (4 bit) per step, so every table and the output are read and
    // written at a per-lane base plus a multiple of the step.
    const char *off_lane = reinterpret_cast<const char *>(off32) + lane * (kPer * 4);
    const char *keep_lane = reinterpret_cast<const char *>(keep) + lane * 4;
    const uint32_t slot_lane = BITS == 8 ? (lane >> 2) & 3 : (lane >> 2) & 1;  // 16-byte slot
    const uint32_t out_lane = (uint32_t)(lane / kDwPerChunk) * 1024u + (lane & 3) * 4u;
    const char *xsb = reinterpret_cast<const char *>(xs);
    // lane k holds threshold k: the class of a row is the number of thresholds below its
    // range (the nearest cluster centre), counted with one compare and a mask population count
    const float tau_lane = lane < n_tau ? taus[lane] : INFINITY;

    while (true) {
        // the sequence ends at the first unit index past the end; rows inside the last
        // unit but past `rows` are skipped
        const int64_t u = (int64_t)blockIdx.x + (it >> rpw_log2) * gridDim.x;
        if (u >= n_units) break;
        const int64_t r_next = row_of(it + 1);
        if (r < rows) {
            float mx = -INFINITY, mn = INFINITY;
            float4 *s4 = reinterpret_cast<float4 *>(xs);
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                s4[cidx[k]] = v[k];
                mx = max3(max3(v[k].x, v[k].y, v[k].z), v[k].w, mx);
                mn = min3(min3(v[k].x, v[k].y, v[k].z), v[k].w, mn);
            }
            if (r_next < rows) fetch(r_next);  // in flight while this row is quantized
            wave_max_min(mx, mn);
            const int p = __builtin_popcountll(__ballot(__fsub_rn(mx, mn) > tau_lane));
            if (lane == 0) row_class[r] = (uint8_t)p;
            const char *cz_lane = reinterpret_cast<const char *>(cz + p * L.nch_pad + lane / kDwPerChunk);
            // The LDS slice is private to this wave and a wave's LDS operations complete
            // in issue order, so a compiler-level fence is all that is needed.
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();

            // a row's place in the tiled layout: scalar base, per-lane 32-bit offset
            auto row_base = [&](int64_t rr) -> int8_t * {
                const uint32_t t = (uint32_t)rr & (BITS == 8 ? 15u : 31u);
                return codes + (((rr >> (BITS == 8 ? 4 : 5)) * n_chunks) << 10) + t * (BITS == 8 ? 64u : 32u);
            };
            auto row_off = [&](int64_t rr) -> uint32_t {
                const uint32_t t = (uint32_t)rr & (BITS == 8 ? 15u : 31u);
                return (out_lane + ((slot_lane ^ (uint32_t)(BITS == 8 ? swz64((int)t) : swz32((int)t))) << 4)) ^
                       (BITS == 8 ? 0u : (uint32_t)half32((int)t) << 3);  // 4 bit: halves swapped in rows 16..31
            };
            int8_t *out_row = row_base(r) + (conv_w > 0 ? copy_bytes : 0);
            const uint32_t out_off = row_off(r);
            // the shifted copies (tap-gathering convolution): this row's codes are the left
            // neighbour of row r + 1 and the right neighbour of row r - 1 of the same image row
            const int32_t wcol = conv_w > 0 ? (int32_t)(r % conv_w) : 0;
            const bool to_left = conv_w > 0 && wcol + 1 < conv_w, to_right = conv_w > 0 && wcol > 0;
            const bool fill_left = conv_w > 0 && wcol == 0, fill_right = conv_w > 0 && wcol + 1 == conv_w;
            int8_t *rowL = to_left ? row_base(r + 1) : out_row;                       // copy 0, row r + 1
            int8_t *rowR = to_right ? row_base(r - 1) + 2 * copy_bytes : out_row;     // copy 2, row r - 1
            const uint32_t offL = to_left ? row_off(r + 1) : 0u, offR = to_right ? row_off(r - 1) : 0u;
            int8_t *rowF = fill_left ? row_base(r) : row_base(r) + 2 * copy_bytes;     // copy 0 or 2, row r

            // NT steps together, so that their LDS round trips overlap
            auto steps = [&](auto nt_tag, const int32_t j0) __attribute__((always_inline)) {
                constexpr int NT = decltype(nt_tag)::value;
                uint32_t off[NT][kPer];
                float2 zi[NT];
                uint32_t km[NT];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint32_t j = (uint32_t)(j0 + t);
                    zi[t] = *reinterpret_cast<const float2 *>(cz_lane + j * (kChunkStep * 8));
                    km[t] = *reinterpret_cast<const uint32_t *>(keep_lane + j * 256u);
                    const uint4 o0 = *reinterpret_cast<const uint4 *>(off_lane + j * (64u * kPer * 4));
                    off[t][0] = o0.x; off[t][1] = o0.y; off[t][2] = o0.z; off[t][3] = o0.w;
                    if constexpr (BITS == 4) {
                        const uint4 o1 = *reinterpret_cast<const uint4 *>(off_lane + j * (64u * kPer * 4) + 16);
                        off[t][4] = o1.x; off[t][5] = o1.y; off[t][6] = o1.z; off[t][7] = o1.w;
                    }
                }
                float xv[NT][kPer];
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int k = 0; k < kPer; ++k)
                        xv[t][k] = *reinterpret_cast<const float *>(xsb + off[t][k]);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    uint32_t lo = 0, hi = 0;
#pragma unroll
                    for (int k = 0; k < kPer; ++k) {
                        const float qf = quant_pre<BITS>(xv[t][k], zi[t].x, zi[t].y);
                        // rounds, saturates and places byte k of the word
                        if (k < 4)
                            lo = __builtin_amdgcn_cvt_pk_u8_f32(qf, k, lo);
                        else
                            hi = __builtin_amdgcn_cvt_pk_u8_f32(qf, k - 4, hi);
                    }
                    // 8 bit: stored code = q - 128 = q ^ 0x80 per byte.  4 bit: byte i holds
                    // position i (low nibble) and position i + 4 (high nibble).  Padding
                    // positions are cleared to the stored value 0.
                    const uint32_t word = (BITS == 8 ? (lo ^ 0x80808080u) : (lo | (hi << 4))) & km[t];
                    const uint32_t j = (uint32_t)(j0 + t);
                    if ((int32_t)(lane + 64u * j) < n_dw) {
                        *reinterpret_cast<uint32_t *>(out_row + (out_off + j * (kChunkStep * 1024u))) = word;
                        if (to_left) *reinterpret_cast<uint32_t *>(rowL + (offL + j * (kChunkStep * 1024u))) = word;
                        if (to_right) *reinterpret_cast<uint32_t *>(rowR + (offR + j * (kChunkStep * 1024u))) = word;
                        if (fill_left || fill_right) {
                            const uint32_t fw = fill32[lane + 64u * j];
                            *reinterpret_cast<uint32_t *>(rowF + (out_off + j * (kChunkStep * 1024u))) = fw;
                            // a one-pixel-wide image has both neighbours outside
                            if (fill_left && fill_right)
                                *reinterpret_cast<uint32_t *>(row_base(r) + 2 * copy_bytes +
                                                              (out_off + j * (kChunkStep * 1024u))) = fw;
                        }
                    }
                }
            };
            int32_t j0 = 0;
            for (; j0 + 4 <= L.n_steps; j0 += 4) steps(std::integral_constant<int, 4>{}, j0);
            switch (L.n_steps - j0) {
                case 3: steps(std::integral_constant<int, 3>{}, j0); break;
                case 2: steps(std::integral_constant<int, 2>{}, j0); break;
                case 1: steps(std::integral_constant<int, 1>{}, j0); break;
                default: break;
            }
            // the next row overwrites xs
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            __builtin_amdgcn_wave_barrier();
        } else if (r_next < rows) {
            fetch(r_next);
        }
        r = r_next;
        ++it;
    }
}

// Fallback for channel counts that are not a multiple of 4 (no 16-byte loads):
// scalar loads straight into LDS, tables read from global memory.
template <int BITS>
__global__ __launch_bounds__(256) void k_quantize_act_any(
    const float *__restrict__ x, int64_t rows, int32_t C, int32_t Kp, int32_t n_chunks,
    const int32_t *__restrict__ perm, const float *__restrict__ chunk_z,
    const float *__restrict__ chunk_inv, const float *__restrict__ taus, int32_t n_tau,
    int8_t *__restrict__ codes, uint8_t *__restrict__ row_class,
    int32_t /*rpw_log2: unused, one row per wave*/, int32_t /*conv_w: not built here*/,
    int64_t /*copy_bytes*/, const uint32_t * /*fill32*/) {
    extern __shared__ float lds[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float *xs = lds + (size_t)wave * C;
    constexpr float qmax = (float)((1 << BITS) - 1);
    constexpr int kOff = BITS == 8 ? 128 : 0;
    constexpr int kPer = BITS == 8 ? 4 : 8;  // positions per output dword
    const float tau_lane = lane < n_tau ? taus[lane] : INFINITY;

    for (int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + wave; r < rows;
         r += (int64_t)gridDim.x * kWavesPerBlock) {
        const float *xr = x + r * C;
        float mx = -INFINITY, mn = INFINITY;
        for (int32_t c = lane; c < C; c += kWave) {
            const float v = xr[c];
            xs[c] = v;
            mx = fmaxf(v, mx);
            mn = fminf(v, mn);
        }
        wave_max_min(mx, mn);
        const int p = __builtin_popcountll(__ballot(__fsub_rn(mx, mn) > tau_lane));
        if (lane == 0) row_class[r] = (uint8_t)p;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int32_t jd = lane; jd < Kp / kPer; jd += kWave) {
            const int32_t ch = (jd * kPer) >> 6;
            const float z = chunk_z[p * n_chunks + ch], is = chunk_inv[p * n_chunks + ch];
            uint32_t word = 0;
#pragma unroll
            for (int k = 0; k < kPer; ++k) {
                const int32_t c = perm[jd * kPer + k];
                uint32_t qv = 0;
                if (c >= 0) {
                    const int32_t q = (int32_t)quant1(xs[c], z, is, qmax) - kOff;
                    qv = BITS == 8 ? ((uint32_t)q & 0xffu) : (uint32_t)q;
                }
                word |= BITS == 8 ? qv << (8 * k) : qv << (k < 4 ? 8 * k : 8 * (k - 4) + 4);
            }
            const int64_t off = BITS == 8 ? tiled64_offset(r, ch, n_chunks, (jd >> 2) & 3)
                                          : tiled32_offset(r, ch, n_chunks, (jd >> 2) & 1);
            const int dw = BITS == 8 ? (jd & 3) : ((jd & 3) ^ (2 * half32((int)(r & 31))));
            *reinterpret_cast<uint32_t *>(codes + off + dw * 4) = word;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

using Kern = void (*)(const float *, int64_t, int32_t, int32_t, int32_t, const int32_t *,
                      const float *, const float *, const float *, int32_t, int8_t *, uint8_t *,
                      int32_t, int32_t, int64_t, const uint32_t *);

// A kernel instantiation and the state of its dynamic-LDS limit.
// Workgroups of a kernel that one CU holds at a given LDS size, as the runtime's occupancy
// calculation gives it (registers count too: the 640-channel kernel needs 71, seven
// workgroups per CU where LDS alone would admit eight).  Remembered per device together with
// the LDS size it was asked for.
struct Residency {
    std::atomic<uint64_t> v[kMaxDevices];  // (LDS bytes + 1) << 8 | workgroups per CU; 0 = not asked yet
};
struct Picked {
    Kern kern;
    LdsLimit *lim;
    Residency *res;
};
template <int BITS, int NV>
Picked vec_kernel() {
    static LdsLimit lim;
    static Residency res;
    return {k_quantize_act<BITS, NV>, &lim, &res};
}
hipError_t resident_workgroups(const Picked &k, size_t lds, int *per_cu) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    const uint64_t key = (uint64_t)lds + 1;
    const uint64_t cur = k.res->v[dev].load(std::memory_order_acquire);
    if ((cur >> 8) == key) {
        *per_cu = (int)(cur & 0xff);
        return hipSuccess;
    }
    int n = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(k.kern), 256, lds);
    if (e != hipSuccess) return e;
    n = n < 1 ? 1 : (n > 255 ? 255 : n);
    k.res->v[dev].store(key << 8 | (uint64_t)n, std::memory_order_release);
    *per_cu = n;
    return hipSuccess;
}
template <int BITS>
Picked any_kernel() {
    static LdsLimit lim;
    return {k_quantize_act_any<BITS>, &lim, nullptr};
}

// NV = float4 loads per lane per row; exact for the usual channel counts (320 .. 5120).
template <int BITS>
Picked pick_vec(int32_t C) {
    const int nv = (C + 255) / 256;
    if (nv <= 2) return vec_kernel<BITS, 2>();
    if (nv <= 3) return vec_kernel<BITS, 3>();
    if (nv <= 5) return vec_kernel<BITS, 5>();
    if (nv <= 8) return vec_kernel<BITS, 8>();
    if (nv <= 10) return vec_kernel<BITS, 10>();
    if (nv <= 20) return vec_kernel<BITS, 20>();
    return vec_kernel<BITS, 40>();
}

}  // namespace

size_t quantize_act_lds_bytes(const Groups &g) {
    const int32_t C = g.info.channels;
    const bool vec4 = (C % 4) == 0 && C < 65535;
    const size_t rows_bytes = sizeof(float) * (size_t)C * kWavesPerBlock;
    return vec4 ? QuantLds(g.info.k_padded, g.info.act_bits, g.n_tab).table_bytes() + rows_bytes
                : rows_bytes;
}

hipError_t launch_quantize_act(const Groups &g, const float *x, int64_t rows, int8_t *codes,
                               uint8_t *row_class, hipStream_t st, int32_t conv_w, int64_t copy_bytes,
                               const uint32_t *fill32) {
    const int32_t C = g.info.channels, Kp = g.info.k_padded;
    const bool vec4 = (C % 4) == 0 && C < 65535;
    if (conv_w > 0 && !vec4) return hipErrorInvalidValue;
    Picked kern;
    size_t lds;
    int64_t blocks;
    int32_t rpw_log2 = 2;
    if (vec4) {
        kern = g.info.act_bits == 8 ? pick_vec<8>(C) : pick_vec<4>(C);
        lds = QuantLds(Kp, g.info.act_bits, g.n_tab).table_bytes() +
              sizeof(float) * (size_t)C * kWavesPerBlock;
        blocks = (rows + 15) / 16;
        if (blocks < 256) {  // fewer 16-row blocks than CUs: quarter blocks, one row per wave
            rpw_log2 = 0;
            blocks = (rows + 3) / 4;
        }
        // As many workgroups as the chip holds at once, every one walking several units: one
        // more than that and the last ones start when the first are done, with their whole
        // share of the rows still to do on a mostly idle chip.
        if (lds > 64 * 1024) {
            hipError_t e = raise_lds_limit(*kern.lim, reinterpret_cast<const void *>(kern.kern), 160 * 1024);
            if (e != hipSuccess) return e;
        }
        int per_cu = 1;
        if (hipError_t e = resident_workgroups(kern, lds, &per_cu); e != hipSuccess) return e;
        per_cu = per_cu > 8 ? 8 : per_cu;
#ifdef DGQ_TUNING  // tuning builds only: cap on resident workgroups per CU
        if (const int cap_t = tuning_value(kTuneQuantWgPerCu); cap_t > 0 && per_cu > cap_t) per_cu = cap_t;
#endif
        const int64_t cap = 256 * (int64_t)per_cu;
        if (blocks > cap) blocks = cap;
    } else {
        kern = g.info.act_bits == 8 ? any_kernel<8>() : any_kernel<4>();
        lds = sizeof(float) * (size_t)C * kWavesPerBlock;
        blocks = (rows + kWavesPerBlock - 1) / kWavesPerBlock;
        if (blocks > 2048) blocks = 2048;
    }
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (lds > 64 * 1024) {
        hipError_t e = raise_lds_limit(*kern.lim, reinterpret_cast<const void *>(kern.kern), 160 * 1024);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern.kern, dim3((unsigned)blocks), dim3(256), lds, st, x, rows, C, Kp,
                       g.n_chunks, g.d_perm, g.d_chunk_z, g.d_chunk_inv, g.d_taus, g.n_tab - 1, codes,
                       row_class, rpw_log2, conv_w, copy_bytes, fill32);
    return hipGetLastError();
}

}  // namespace dgq
