// Machine ceilings for the benchmark: the bare int8 matrix instruction and plain streaming
// kernels (see include/dgq_probe.h).  Not part of the method.
#include "dgq_internal.h"
#include "dgq_probe.h"

namespace dgq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void k_probe_mfma_i8(int32_t iters, int32_t *__restrict__ sink) {
    const v4i a = {0x01010101, 0x01010101, 0x01010101, 0x01010101};  // sixteen codes of value 1
    const v4i b = a;
    v16i c0 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
    for (int32_t i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
    }
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[5] + c2[10] + c3[15] - 3 * 32 * iters;
}

typedef uint32_t u4 __attribute__((ext_vector_type(4)));

template <int MODE>
__global__ __launch_bounds__(256) void k_probe_stream(const u4 *__restrict__ src, u4 *__restrict__ dst,
                                                      int64_t n16, uint32_t *__restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    u4 acc = {0, 0, 0, 0};
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        if (MODE == 0) {
            const u4 v = __builtin_nontemporal_load(src + i);
            acc ^= v;
        } else {
            __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
        }
    }
    if (MODE == 0) {
        const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
        if (x == 0x9e3779b9u) *sink = x;  // practically never: the loads must still happen
    }
}

// Block-contiguous writer: workgroup b fills bytes [b * CH, (b + 1) * CH) and exits (a
// grid-stride loop of the same stores reaches two thirds of this rate: consecutive
// workgroups then keep many DRAM pages open at once).
template <int CH>
__global__ __launch_bounds__(256) void k_probe_write_chunks(u4 *__restrict__ dst) {
    const u4 fill = {0x3f800000u, 0x3f800000u, 0x3f800000u, 0x3f800000u};
    u4 *p = dst + (int64_t)blockIdx.x * (CH / 16) + threadIdx.x;
#pragma unroll
    for (int i = 0; i < CH / 4096; ++i) p[i * 256] = fill;
}

// Tile writer shaped like the contraction's epilogue: a workgroup of 8 waves writes a tile of
// 128 rows x 512 B into a matrix of `row_bytes` per row; wave (wr, wo) writes 32 rows x 256 B,
// one dword per lane and instruction (two rows of 128 B).
__global__ __launch_bounds__(512) void k_probe_write_tiles(float *__restrict__ dst, int64_t row_bytes,
                                                           int32_t tiles_o) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, wr = wave >> 1, wo = wave & 1;
    const int m32 = lane & 31, kh = lane >> 5;
    const int64_t tile_r = blockIdx.x / tiles_o, tile_o = blockIdx.x % tiles_o;
    char *base = reinterpret_cast<char *>(dst) + (tile_r * 128 + wr * 32) * row_bytes + tile_o * 512 + wo * 256;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int row = 8 * (i >> 2) + 4 * kh + (i & 3);
        float *q = reinterpret_cast<float *>(base + row * row_bytes) + m32;
        __builtin_nontemporal_store(1.0f, q);
        __builtin_nontemporal_store(1.0f, q + 32);
    }
}

}  // namespace
}  // namespace dgq

using namespace dgq;

extern "C" {

int dgq_probe_mfma_i8(int32_t blocks, int32_t iters, int32_t *sink, void *stream) {
    if (!sink || blocks < 1 || iters < 1 || blocks > (1 << 20)) {
        set_error("dgq_probe_mfma_i8: bad argument");
        return DGQ_EINVAL;
    }
    hipLaunchKernelGGL(k_probe_mfma_i8, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       iters, sink);
    DGQ_HIP(hipGetLastError());
    return DGQ_OK;
}

int dgq_probe_stream(const void *src, void *dst, size_t bytes, int32_t mode, uint32_t *sink, void *stream) {
    const bool need_src = mode == 0 || mode == 2, need_dst = mode == 1 || mode == 2;
    if (mode < 0 || mode > 2 || bytes < 16384 || bytes % 16384 || bytes > ((size_t)1 << 40) ||
        (need_src && !src) || (need_dst && !dst) || (mode == 0 && !sink)) {
        set_error("dgq_probe_stream: bad argument");
        return DGQ_EINVAL;
    }
    if ((need_src && (reinterpret_cast<uintptr_t>(src) & 15)) || (need_dst && (reinterpret_cast<uintptr_t>(dst) & 15))) {
        set_error("dgq_probe_stream: buffer not 16-byte aligned");
        return DGQ_EALIGN;
    }
    const int64_t n16 = (int64_t)(bytes / 16);
    const unsigned grid = 256 * 16;  // sixteen workgroups per CU, each walks the buffer with the grid's stride
    hipStream_t st = static_cast<hipStream_t>(stream);
    const u4 *s = static_cast<const u4 *>(src);
    u4 *d = static_cast<u4 *>(dst);
    if (mode == 0)
        hipLaunchKernelGGL(k_probe_stream<0>, dim3(grid), dim3(256), 0, st, s, d, n16, sink);
    else if (mode == 1)
        hipLaunchKernelGGL(k_probe_write_chunks<16384>, dim3((unsigned)(bytes / 16384)), dim3(256), 0, st, d);
    else
        hipLaunchKernelGGL(k_probe_stream<2>, dim3(grid), dim3(256), 0, st, s, d, n16, sink);
    DGQ_HIP(hipGetLastError());
    return DGQ_OK;
}

int dgq_probe_write_tiles(float *dst, int64_t rows, int32_t out_channels, void *stream) {
    if (!dst || rows < 128 || rows % 128 || out_channels < 128 || out_channels % 128 ||
        (rows / 128) * (int64_t)(out_channels / 128) > ((int64_t)1 << 30)) {
        set_error("dgq_probe_write_tiles: rows and out_channels must be positive multiples of 128");
        return DGQ_EINVAL;
    }
    if (reinterpret_cast<uintptr_t>(dst) & 15) {
        set_error("dgq_probe_write_tiles: buffer not 16-byte aligned");
        return DGQ_EALIGN;
    }
    const int32_t tiles_o = out_channels / 128;
    hipLaunchKernelGGL(k_probe_write_tiles, dim3((unsigned)((rows / 128) * tiles_o)), dim3(512), 0,
                       static_cast<hipStream_t>(stream), dst, (int64_t)out_channels * 4, tiles_o);
    DGQ_HIP(hipGetLastError());
    return DGQ_OK;
}

}  // extern "C"
