// Internal declarations shared by the host API and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <string>
#include <vector>

#include "dgq.h"

namespace dgq {

constexpr int kGranule = DGQ_K_GRANULE;  // positions per K chunk
constexpr int kTileO = 256;              // weights are padded to a multiple of every GEMM tile width
constexpr int kMaxClasses = DGQ_MAX_PIXEL_CLASSES;

// ---- block-tiled operand layout shared by the quantizer, the weight packer and the
// GEMM.  A block is 1 KiB = one 64-position chunk of 16 rows (64 B per row: int8
// codes and weights) or of 32 rows (32 B per row: packed 4-bit codes); blocks are
// ordered [row block][chunk].  The 16-byte slots of a row are XOR-permuted so that the
// GEMM's 16-byte LDS fragment reads of 32 consecutive rows touch all banks; since a
// block is copied verbatim into LDS the permutation lives in the global layout.
__host__ __device__ inline int swz64(int row) {  // 4 slots
    return ((row >> 2) & 1) | ((((row >> 1) ^ (row >> 3)) & 1) << 1);
}
__host__ __device__ inline int swz32(int row) { return (row >> 3) & 1; }  // 2 slots
// Packed 4-bit rows are read 8 bytes per lane (one k-half of a 32-position step), 32 lanes at a
// time: with 32-byte rows the 32 rows of one k-half would touch only every other 8-byte bank
// pair, so rows 16..31 of a block keep the two 8-byte halves of every slot swapped.
__host__ __device__ inline int half32(int row) { return (row >> 4) & 1; }
// byte offset of 16-byte slot kq of (row, chunk) in a 64-B-per-row tensor
__host__ __device__ inline int64_t tiled64_offset(int64_t row, int32_t chunk, int32_t n_chunks, int kq) {
    const int t = (int)(row & 15);
    return (((row >> 4) * n_chunks + chunk) << 10) + t * 64 + ((kq ^ swz64(t)) << 4);
}
// byte offset of 16-byte slot h of (row, chunk) in a 32-B-per-row tensor
__host__ __device__ inline int64_t tiled32_offset(int64_t row, int32_t chunk, int32_t n_chunks, int h) {
    const int t = (int)(row & 31);
    return (((row >> 5) * n_chunks + chunk) << 10) + t * 32 + ((h ^ swz32(t)) << 4);
}

// One (layer, timestep) entry of the quantization tables.
struct Groups {
    dgq_groups_info_t info{};
    int32_t n_chunks = 0;  // K' / kGranule
    // host copies
    std::vector<int32_t> perm, goff, glen;
    int32_t n_tab = 2;               // class rows in the tables: 2, or P when P > 2
    std::vector<float> s, z, inv_s;  // [n_tab][NG]
    std::vector<float> taus;         // [n_tab - 1] ascending row-range thresholds; +inf = unused
    // device tables
    int32_t *d_perm = nullptr;     // [K'] original channel or -1
    float *d_chunk_z = nullptr;    // [n_tab][n_chunks]  offset of the chunk's group
    float *d_chunk_inv = nullptr;  // [n_tab][n_chunks]  1/s of the chunk's group
    float *d_s = nullptr;          // [n_tab][NG]
    float *d_z = nullptr;          // [n_tab][NG]
    float *d_zoff = nullptr;       // [n_tab][NG]  z + code_offset * s
    float *d_taus = nullptr;       // [n_tab - 1]
    int32_t *d_gchunk = nullptr;   // [NG+1] first chunk of each group
    // Tables of a 3 x 3 convolution (nine replicated taps of a base layer with base_kp
    // positions): d_fill is one tap's code row of the value 0 in position order, as stored
    // (8 bit: q - 128 per position; 4 bit: packed nibbles; padding positions 0).
    int32_t conv_taps = 0, base_kp = 0;
    uint8_t *d_fill = nullptr;
    // the same row as one 1 KiB code block per chunk (every row of the block the fill row, in
    // the block's slot order): what the tap-gathering contraction loads outside the image
    uint8_t *d_fill_blocks = nullptr;
    int device = 0;
    // One reference for the caller's handle and one per weight handle packed for it: the
    // tables live until the last of them is released.
    mutable std::atomic<int> refs{1};
};

struct Weight {
    const Groups *groups = nullptr;
    int32_t O = 0, O_pad = 0, C = 0, Kp = 0, w_bits = 8;
    int8_t *d_wq = nullptr;  // [O_pad x K'] permuted + padded rows, block-tiled (64 B per row)
    // the same buffer at two 4-bit weights per byte (byte i = weights 2i and 2i + 1 of d_wq,
    // low nibble first); d_wq is null while this is set
    uint8_t *d_wq4 = nullptr;
    float *d_sw = nullptr;   // [O_pad]
    // [2][O_pad].  Two class rows: zb[p][o].  More than two classes (one channel group):
    // row 0 = sw[o] * sum_j wq[o,j], row 1 = bias[o]; zb[p][o] = zoff[p] * row 0 + row 1.
    float *d_zb = nullptr;
    // Packed for a gated layer whose output feeds `next_channels` channels of a following
    // layer directly: output rows are in that layer's K' order (value rows, then gate
    // rows), and the two tables its quantizer needs travel with the weights.
    int32_t next_channels = 0, next_kp = 0, next_bits = 8;
    float2 *d_rq_zi = nullptr;     // [next_kp / 64] (offset, 1 / step) of each chunk
    uint8_t *d_rq_keep = nullptr;  // [next_kp] 0xFF, or 0 at padding positions
    int device = 0;
};

void set_error(const std::string &msg);
int hip_fail(hipError_t e, const char *what);

#define DGQ_HIP(call)                                          \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return ::dgq::hip_fail(e_, #call); \
    } while (0)

// Raise a kernel's dynamic-LDS limit to `bytes`, the first time only per kernel and device
// (the attribute call is a host round trip that hot calls should not repeat).  Every launch
// site keeps one LdsLimit per kernel instantiation; after the first call the check is one
// atomic load, with no lock and no table shared between kernels.
constexpr int kMaxDevices = 64;
struct LdsLimit {
    std::atomic<int> bytes[kMaxDevices];  // zero-initialised (static storage)
};
hipError_t raise_lds_limit(LdsLimit &state, const void *kernel, int bytes);
#define DGQ_ENSURE_LDS(kernel, nbytes)                                                        \
    ([&]() -> hipError_t {                                                                    \
        static ::dgq::LdsLimit lim_;                                                          \
        return ::dgq::raise_lds_limit(lim_, reinterpret_cast<const void *>(kernel), (nbytes)); \
    }())

#ifdef DGQ_TUNING
// Builds with -DDGQ_TUNING (never the shipped library) export dgq_tuning_set(key, value): launch
// parameters a sweep wants to force.  0 = the library's own choice.
enum TuneKey { kTuneLinearCfg = 0, kTuneSuperRows, kTuneQuantWgPerCu, kTuneXattnWgs, kTuneKeys };
int tuning_value(int key);
#endif

// ---- kernel launchers (each returns a hipError_t from the launch) ----------

// Per-row max and min of x [rows, C].
hipError_t launch_row_minmax(const float *x, int64_t rows, int32_t C, float *rmx,
                             float *rmn, hipStream_t st);

// Per-class channel max/min partials: part [slabs][4][C] = (max0, min0, max1, min1),
// class of row r = [rmx[r] - rmn[r] > tau].
hipError_t launch_col_minmax_by_class(const float *x, int64_t rows, int32_t C,
                                      const float *rmx, const float *rmn, float tau,
                                      int32_t slabs, float *part, hipStream_t st);

// Per-output-channel weight quantization into the K' layout plus the zero-point term.
// row_map (optional, [O]): packed row o comes from row row_map[o] of w and bias, or is
// all zero when that is negative.
hipError_t launch_pack_weight(const float *w, const float *bias, int32_t O, int32_t O_pad,
                              int32_t C, int32_t Kp, int32_t NG, int32_t w_bits,
                              int32_t code_offset, const int32_t *perm,
                              const int32_t *gchunk, const float *s, const float *z,
                              int32_t n_classes, const int32_t *row_map, int8_t *wq, float *sw,
                              float *zb, hipStream_t st);

// Two 4-bit weights per byte and back (n_bytes8: size of the one-byte-per-weight buffer, a
// multiple of 32).
hipError_t launch_pack_nibbles(const int8_t *wq, uint8_t *wq4, int64_t n_bytes8, hipStream_t st);
hipError_t launch_expand_nibbles(const uint8_t *wq4, int8_t *wq, int64_t n_bytes8, hipStream_t st);

// Inverse of the K' layout: wq_out [O][C] original order.
hipError_t launch_unpack_weight(const int8_t *wq, int32_t O, int32_t C, int32_t Kp,
                                const int32_t *perm, int8_t *wq_out, hipStream_t st);

// conv_w > 0: the rows are pixels of images conv_w wide and the codes are written as the three
// shifted copies of the tap-gathering 3 x 3 convolution (copy_bytes apart; fill32: the code of
// the value 0, one dword per output dword of a row).
hipError_t launch_quantize_act(const Groups &g, const float *x, int64_t rows, int8_t *codes,
                               uint8_t *row_class, hipStream_t st, int32_t conv_w = 0,
                               int64_t copy_bytes = 0, const uint32_t *fill32 = nullptr);
hipError_t launch_linear_conv3x3(const Groups &g9, const Weight &w, const int8_t *codes3,
                                 const uint8_t *row_class, int32_t B, int32_t H, int32_t W, float *y,
                                 hipStream_t st);
// LDS bytes a workgroup of the quantizer needs for this layer (tables + one row per wave).
size_t quantize_act_lds_bytes(const Groups &g);

// geglu 1: y is [rows, O / 2] and receives value * GELU(gate) (first / second half of the
// output channels); needs O % 128 == 0 and no accumulator dump.  geglu 2: the same value
// goes through the following layer's quantizer; y is that layer's code buffer, rq_cls its
// row classes, and w carries its tables.
hipError_t launch_linear(const Groups &g, const Weight &w, const int8_t *codes,
                         const uint8_t *row_class, int64_t rows, float *y, int32_t *acc_dump,
                         int geglu, uint8_t *rq_cls, hipStream_t st);

// Unfolds the codes of a [B, H, W] activation map into the code buffer of its 3 x 3
// convolution (nine taps, the code of zero outside the image).
hipError_t launch_conv3x3_codes(const Groups &g9, const int8_t *codes, int32_t B, int32_t H,
                                int32_t W, int8_t *codes9, hipStream_t st);

hipError_t launch_xattn(const float *q, const float *k, const float *v, const float *key_bias,
                        int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
                        float *out, float *scale_out, uint8_t *codes_dump, void *workspace,
                        size_t workspace_bytes, const float *scale_in, hipStream_t st);

// The attention on V^'s integer codes with 4-bit probability codes (shift-and-add product).
hipError_t launch_xattn_intv(const float *q, const float *k, const uint8_t *vq, const float *vparams,
                             const float *key_bias, int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk,
                             float *out, float *scale_out, uint8_t *codes_dump, int32_t *acc_dump,
                             hipStream_t st);

hipError_t launch_quantize_value(const float *v, int32_t B, int32_t nk, int32_t H, int32_t d,
                                 int32_t bits, float *vhat, uint8_t *codes, float *params,
                                 hipStream_t st);

// Self-attention with every probability log2-quantized against the given scale; needs
// d % 8 == 0, 8 <= d <= 160 and a workspace of selfattn_workspace_bytes.
hipError_t launch_selfattn(const float *q, const float *k, const float *v, int32_t B, int32_t N,
                           int32_t H, int32_t d, int32_t bits, const float *scale_in, float *out,
                           float *scale_out, uint8_t *codes_dump, void *workspace, hipStream_t st);
size_t selfattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d);

size_t xattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk);
// the least the attention can work with (the row statistics alone; its maximum then goes
// through atomics on scale[] and one more launch that clears it)
size_t xattn_workspace_min_bytes(int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk);

}  // namespace dgq
