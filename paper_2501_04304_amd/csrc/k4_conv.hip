// 3 x 3 convolution (stride 1, zero padding 1) through the grouped contraction: the paper
// quantizes every layer of the U-Net, convolutions included, with the activation quantizer
// of Section 3.3.  The activation map is quantized ONCE per pixel (k_quantize_act, codes
// [pixels, K']); this kernel unfolds the CODES, not the activations: the code row of output
// pixel (b, h, w) is the concatenation over the nine taps t = 3 (dy + 1) + (dx + 1) of the code
// row of pixel (b, h + dy, w + dx), and of the code of the value 0 where that pixel lies
// outside the image.  The result is the code buffer of a layer with 9 K' positions (group
// tables replicated per tap), which the contraction kernel takes as it is.  Needs one pixel
// class: with several, the scale of a tap's partial sum would follow the neighbour's class,
// not the output row's.
//
// Both buffers are block-tiled (1 KiB = one 64-position chunk of 16 rows of 64 B, or of 32
// rows of 32 B of packed 4-bit codes; 16-byte slots XOR-permuted by row bits).
#include "dgq_internal.h"

namespace dgq {

namespace {

// One workgroup per destination row block (16 or 32 pixels): lane (tid % 64) owns one
// 16-byte slot of every block of that row block, wave (tid / 64) takes every fourth chunk.
// Everything that needs a division (the pixel's place in its image) is done once per thread;
// the loops over taps and chunks only add strides, and a wave writes 1 KiB at a time.
template <int BITS>
__global__ __launch_bounds__(256) void k_conv3x3_codes(
    const int8_t *__restrict__ codes, const uint8_t *__restrict__ fill, int64_t rows, int32_t H,
    int32_t W, int32_t n_chunks, int8_t *__restrict__ out) {
    constexpr int SLOTS = BITS == 8 ? 4 : 2;        // 16-byte slots per row and chunk
    constexpr int ROWS = BITS == 8 ? 16 : 32;       // rows per block
    constexpr int ROW_BYTES = 16 * SLOTS;
    const int64_t rb = blockIdx.x;
    const int sl = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int tr = sl / SLOTS;                       // row in the block
    const int stored = sl % SLOTS;                   // stored slot = logical slot ^ swizzle(row)
    const int kq = stored ^ (BITS == 8 ? swz64(tr) : swz32(tr));
    const int64_t r = rb * ROWS + tr;
    if (r >= rows) return;                           // rows past the end are never read as results
    const int32_t w = (int32_t)(r % W);
    const int32_t h = (int32_t)((r / W) % H);
    int8_t *dst = out + ((rb * 9 * n_chunks) << 10) + sl * 16;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const int dy = t / 3 - 1, dx = t % 3 - 1;
        const bool inside = (uint32_t)(h + dy) < (uint32_t)H && (uint32_t)(w + dx) < (uint32_t)W;
        const int64_t rs = r + (int64_t)dy * W + dx;   // same image: no carry into the batch index
        const int8_t *src;
        int32_t stride;
        if (inside) {
            src = codes + (BITS == 8 ? tiled64_offset(rs, 0, n_chunks, kq) : tiled32_offset(rs, 0, n_chunks, kq));
            stride = 1024;
        } else {
            src = reinterpret_cast<const int8_t *>(fill) + kq * 16;
            stride = ROW_BYTES;
        }
        // 4-bit rows keep the 8-byte halves of a slot swapped in rows 16..31 of a block (the
        // fill row is stored unswapped): swap when source and destination differ in that
        const bool swap = BITS == 4 && ((inside ? (int)(rs >> 4) & 1 : 0) != ((tr >> 4) & 1));
        for (int32_t ch = q; ch < n_chunks; ch += 4) {
            uint4 v = *reinterpret_cast<const uint4 *>(src + (int64_t)ch * stride);
            if (swap) v = make_uint4(v.z, v.w, v.x, v.y);
            *reinterpret_cast<uint4 *>(dst + ((int64_t)(t * n_chunks + ch) << 10)) = v;
        }
    }
}

}  // namespace

hipError_t launch_conv3x3_codes(const Groups &g9, const int8_t *codes, int32_t B, int32_t H,
                                int32_t W, int8_t *codes9, hipStream_t st) {
    const int32_t n_chunks = g9.base_kp / kGranule;
    const int64_t rows = (int64_t)B * H * W;
    const int64_t rpb = g9.info.act_bits == 8 ? 16 : 32;
    const int64_t blocks = (rows + rpb - 1) / rpb;
    if (g9.info.act_bits == 8)
        hipLaunchKernelGGL(k_conv3x3_codes<8>, dim3((unsigned)blocks), dim3(256), 0, st, codes, g9.d_fill, rows,
                           H, W, n_chunks, codes9);
    else
        hipLaunchKernelGGL(k_conv3x3_codes<4>, dim3((unsigned)blocks), dim3(256), 0, st, codes, g9.d_fill, rows,
                           H, W, n_chunks, codes9);
    return hipGetLastError();
}

}  // namespace dgq
