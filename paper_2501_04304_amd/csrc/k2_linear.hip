// K2: grouped int8 x int8 -> int32 contraction on the gfx950 matrix cores with
// a per-(pixel class, channel group) dequantization epilogue.
//
//   acc[r,o,g] = sum_{j in g} code[r,j] * wq[o,j]                      (int32, exact)
//   y[r,o]     = sw[o] * sum_g s[class(r),g] * float(acc[r,o,g]) + zb[class(r)][o]
//
// i.e. the de-quantizer x_dq = s * x_q + z of Section 3.1 applied with the
// group-wise (s_k, z_k) of Section 3.3, moved behind the integer dot product.
//
// Work decomposition
//   workgroup = 256 threads = 4 wavefronts, output tile 128 rows x 128 channels
//   wavefront = 64 x 64 sub-tile = 2 x 2 blocks of v_mfma_i32_32x32x32_i8
//   K loop    = 64-position chunks (the K granule), double-buffered in LDS;
//               a group is a whole number of chunks, so each group ends on a
//               chunk boundary where its int32 block is folded into fp32.
// Activation rows are the MFMA's M index (spread over accumulator registers)
// and output channels its N index (lane % 32), so a store instruction writes
// 128 contiguous bytes per row, and sw / zb are per-lane constants.  Rows of the
// outlier pixel class are rare: a wavefront whose 64 rows are all class 0 takes
// the scale from a scalar register; otherwise it selects per register.
#include "dgq_internal.h"

namespace dgq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kTR = 128;           // rows per workgroup tile
constexpr int kTO = kTileO;        // output channels per workgroup tile
constexpr int kLdsStride = 80;     // 64 payload bytes + 16 pad: conflict-free 16-byte reads
constexpr int kTileBytes = 128 * kLdsStride;
constexpr int kSuperRows = 8;      // r-tiles per L2 super-tile

// Spread the unsigned nibbles of one dword (positions 0..7, position 2i in the
// low nibble of byte i) into two dwords of bytes in position order.
__device__ inline void unpack8(uint32_t w, uint32_t &p0123, uint32_t &p4567) {
    const uint32_t lo = w & 0x0f0f0f0fu;         // positions 0,2,4,6
    const uint32_t hi = (w >> 4) & 0x0f0f0f0fu;  // positions 1,3,5,7
    p0123 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
    p4567 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
}

template <int ABITS, bool DUMP>
__global__ __launch_bounds__(256, 2) void k_linear(
    const int8_t *__restrict__ codes, const uint8_t *__restrict__ row_class,
    const int8_t *__restrict__ wq, const float *__restrict__ sw, const float *__restrict__ zb,
    const float *__restrict__ s_tab, const int32_t *__restrict__ gchunk, int64_t rows, int32_t O,
    int32_t O_pad, int32_t Kp, int32_t NG, int32_t tiles_r, int32_t tiles_o, int32_t per_xcd,
    float *__restrict__ y, int32_t *__restrict__ acc_dump) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * 2 * kTileBytes];

    // ---- XCD-aware tile mapping: workgroup w runs on XCD w % 8; give every XCD a
    // contiguous range of tile indices and walk it in 8-row-tile super-columns so
    // that the tiles resident on one XCD share code rows and weight rows in its L2.
    const int32_t T = tiles_r * tiles_o;
    const int32_t t = (int32_t)(blockIdx.x & 7) * per_xcd + (int32_t)(blockIdx.x >> 3);
    if (t >= T) return;
    const int32_t in_super = kSuperRows * tiles_o;
    const int32_t first_r = (t / in_super) * kSuperRows;
    const int32_t gsz = tiles_r - first_r < kSuperRows ? tiles_r - first_r : kSuperRows;
    const int32_t tile_r = first_r + (t % in_super) % gsz;
    const int32_t tile_o = (t % in_super) / gsz;

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wr = wave >> 1, wo = wave & 1;
    const int m32 = lane & 31, kh = lane >> 5;
    const int64_t r0 = (int64_t)tile_r * kTR;
    const int32_t o0 = tile_o * kTO;
    const int32_t n_chunks = Kp >> 6;

    // ---- global -> register staging ------------------------------------------------
    // weights: 128 rows x 64 B per chunk = 512 x 16 B, two per thread
    // codes:   8 bit: same; 4 bit: 128 rows x 32 B = 256 x 16 B, one per thread
    const int8_t *wsrc[2];
    int wdst[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int slot = tid + 256 * i;
        const int row = slot >> 2, kq = slot & 3;
        wsrc[i] = wq + (int64_t)(o0 + row) * Kp + kq * 16;
        wdst[i] = kTileBytes + row * kLdsStride + kq * 16;
    }
    const int8_t *csrc[2];
    int cdst[2];
    if (ABITS == 8) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int slot = tid + 256 * i;
            const int row = slot >> 2, kq = slot & 3;
            int64_t r = r0 + row;
            r = r < rows ? r : rows - 1;  // clamp: rows past the end are never stored
            csrc[i] = codes + r * Kp + kq * 16;
            cdst[i] = row * kLdsStride + kq * 16;
        }
    } else {
        const int row = tid >> 1, half = tid & 1;
        int64_t r = r0 + row;
        r = r < rows ? r : rows - 1;
        csrc[0] = codes + r * (Kp >> 1) + half * 16;
        cdst[0] = row * kLdsStride + half * 32;
        csrc[1] = csrc[0];
        cdst[1] = cdst[0];
    }

    v4i stage_c[2], stage_w[2];
    auto load_chunk = [&](int32_t ch) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            stage_w[i] = *reinterpret_cast<const v4i *>(wsrc[i] + (int64_t)ch * 64);
        if (ABITS == 8) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                stage_c[i] = *reinterpret_cast<const v4i *>(csrc[i] + (int64_t)ch * 64);
        } else {
            stage_c[0] = *reinterpret_cast<const v4i *>(csrc[0] + (int64_t)ch * 32);
        }
    };
    auto store_chunk = [&](int buf) {
        uint8_t *base = lds + buf * 2 * kTileBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) *reinterpret_cast<v4i *>(base + wdst[i]) = stage_w[i];
        if (ABITS == 8) {
#pragma unroll
            for (int i = 0; i < 2; ++i) *reinterpret_cast<v4i *>(base + cdst[i]) = stage_c[i];
        } else {
            v4i a, b;
            uint32_t x0, x1;
            unpack8((uint32_t)stage_c[0].x, x0, x1); a.x = (int)x0; a.y = (int)x1;
            unpack8((uint32_t)stage_c[0].y, x0, x1); a.z = (int)x0; a.w = (int)x1;
            unpack8((uint32_t)stage_c[0].z, x0, x1); b.x = (int)x0; b.y = (int)x1;
            unpack8((uint32_t)stage_c[0].w, x0, x1); b.z = (int)x0; b.w = (int)x1;
            *reinterpret_cast<v4i *>(base + cdst[0]) = a;
            *reinterpret_cast<v4i *>(base + cdst[0] + 16) = b;
        }
    };

    // ---- pixel classes of this wavefront's 64 rows ---------------------------------
    uint32_t lane_cls = 0;  // bit (br*16 + i): class of the row held in register i of block br
    bool any_cls1;
    {
        int64_t r = r0 + wr * 64 + lane;
        const int c = (r < rows) ? (int)row_class[r] : 0;
        const uint64_t mask = __ballot(c != 0);
        any_cls1 = mask != 0;
        if (any_cls1) {
#pragma unroll
            for (int br = 0; br < 2; ++br)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int m = br * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                    lane_cls |= (uint32_t)((mask >> m) & 1) << (br * 16 + i);
                }
        }
    }

    float facc[2][2][16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) facc[a][b][i] = 0.0f;

    load_chunk(0);
    store_chunk(0);
    __syncthreads();

    const int a_off = (wr * 64 + m32) * kLdsStride + kh * 16;
    const int b_off = kTileBytes + (wo * 64 + m32) * kLdsStride + kh * 16;

    int32_t ch = 0;
    for (int32_t g = 0; g < NG; ++g) {
        v16i acc[2][2];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0;
        const int32_t ch_end = gchunk[g + 1];
        for (; ch < ch_end; ++ch) {
            const bool more = ch + 1 < n_chunks;
            if (more) load_chunk(ch + 1);
            const uint8_t *base = lds + (ch & 1) * 2 * kTileBytes;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                v4i af[2], bf[2];
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    af[a] = *reinterpret_cast<const v4i *>(base + a_off + a * 32 * kLdsStride + ks * 32);
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    bf[b] = *reinterpret_cast<const v4i *>(base + b_off + b * 32 * kLdsStride + ks * 32);
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
            }
            if (more) store_chunk((ch + 1) & 1);
            __syncthreads();
        }
        // ---- fold this group's int32 block into the fp32 sum with its scale ---------
        const float s0 = s_tab[g], s1 = s_tab[NG + g];
        if (!any_cls1) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        facc[a][b][i] = fmaf((float)acc[a][b][i], s0, facc[a][b][i]);
        } else {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float sg = ((lane_cls >> (a * 16 + i)) & 1) ? s1 : s0;
                        facc[a][b][i] = fmaf((float)acc[a][b][i], sg, facc[a][b][i]);
                    }
        }
        if (DUMP) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int32_t o = o0 + wo * 64 + b * 32 + m32;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int64_t r = r0 + wr * 64 + a * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                        if (r < rows && o < O) acc_dump[(r * O + o) * NG + g] = acc[a][b][i];
                    }
                }
        }
    }

    // ---- epilogue: y = sw[o] * sum + zb[class][o] ------------------------------------
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int32_t o = o0 + wo * 64 + b * 32 + m32;
        const float swo = sw[o];  // o < O_pad always
        const float zb0 = zb[o], zb1 = zb[O_pad + o];
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int64_t r = r0 + wr * 64 + a * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                const float zz = ((lane_cls >> (a * 16 + i)) & 1) ? zb1 : zb0;
                if (r < rows && o < O) y[r * O + o] = fmaf(swo, facc[a][b][i], zz);
            }
    }
}

}  // namespace

hipError_t launch_linear(const Groups &g, const Weight &w, const int8_t *codes,
                         const uint8_t *row_class, int64_t rows, float *y, int32_t *acc_dump,
                         hipStream_t st) {
    const int32_t tiles_r = (int32_t)((rows + kTR - 1) / kTR);
    const int32_t tiles_o = w.O_pad / kTO;
    const int64_t T = (int64_t)tiles_r * tiles_o;
    const int32_t per_xcd = (int32_t)((T + 7) / 8);
    const dim3 grid((unsigned)(per_xcd * 8));
    using Kern = void (*)(const int8_t *, const uint8_t *, const int8_t *, const float *,
                          const float *, const float *, const int32_t *, int64_t, int32_t, int32_t,
                          int32_t, int32_t, int32_t, int32_t, int32_t, float *, int32_t *);
    Kern kern;
    if (g.info.act_bits == 8)
        kern = acc_dump ? k_linear<8, true> : k_linear<8, false>;
    else
        kern = acc_dump ? k_linear<4, true> : k_linear<4, false>;
    hipLaunchKernelGGL(kern, grid, dim3(256), 0, st, codes, row_class, w.d_wq, w.d_sw, w.d_zb,
                       g.d_s, g.d_gchunk, rows, w.O, w.O_pad, w.Kp, g.info.n_groups, tiles_r,
                       tiles_o, per_xcd, y, acc_dump);
    return hipGetLastError();
}

}  // namespace dgq
