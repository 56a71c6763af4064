/*
 * dgq.h -- C ABI of the MI355X (gfx950) DGQ quantized-inference library.
 *
 * DGQ = Distribution-aware Group Quantization for text-to-image diffusion
 * models (arXiv 2501.04304).  The library implements the inference hot path:
 *
 *   dgq_calibrate_groups   offline: pixel classes, channel groups and the
 *                          per-cell (s, z) table of one layer at one timestep
 *   dgq_pack_weight        offline: per-output-channel integer weights laid out
 *                          for the group structure
 *   dgq_quantize_act       fused row-statistics + pixel-class + group affine
 *                          quantizer, fp32 -> int8 / packed int4 codes
 *   dgq_linear             grouped int8 x int8 -> int32 contraction on the
 *                          matrix cores with a per-(pixel class, channel group)
 *                          dequantization epilogue
 *   dgq_xattn_logq         text cross-attention whose softmax probabilities,
 *                          except the <start> column, are log2-quantized with a
 *                          prompt-specific scale before the product with V
 * and, around it:
 *   dgq_calibrate_kmeans   the paper's single-dimension grouping (K clusters of
 *                          channels or of pixels), one handle per timestep
 *   dgq_linear_geglu, dgq_pack_weight_gated_for, dgq_linear_geglu_requant
 *                          the gated feed-forward activation in the contraction's
 *                          epilogue, optionally writing the next layer's codes
 *   dgq_groups_for_conv3x3, dgq_conv3x3_codes
 *                          3 x 3 convolutions through the same quantizer and
 *                          contraction
 *   dgq_quantize_value, dgq_xattn_logq_static, dgq_selfattn_logq, dgq_xattn_logq_intv
 *                          the quantized value tensor, the attention with a given
 *                          scale, self-attention over N keys, and the attention
 *                          product on V^'s integer codes by shifts and adds
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer unless the comment says "host".
 *     Tensors are row-major with the innermost dimension contiguous and a base
 *     address aligned to 16 bytes (else DGQ_EALIGN).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     The hot calls (quantize_act, linear and its variants, conv3x3_codes,
 *     quantize_value, the attentions) only enqueue work: they neither
 *     synchronise nor allocate.  The caller owns every tensor and
 *     keeps it alive until the stream has passed the call.
 *   - Return value: DGQ_OK or a negative dgq_status.  Nothing is enqueued when
 *     an argument error is returned.  dgq_last_error() gives a host string for
 *     the last failure on the calling thread.
 *   - Handles (dgq_groups_t, dgq_weight_t) own small device tables; they are
 *     immutable after creation, may be shared between streams, and are released
 *     with dgq_groups_free / dgq_weight_free.  A weight handle keeps the tables of the
 *     group handle it was packed for alive, so the two may be freed in either order.
 *     Freeing returns device memory to the runtime, which waits for the device to be idle
 *     first: drop handles outside the hot loop (the 25 per-timestep entries of one layer
 *     are a few KB; keep them all).
 *
 * Quantization grid.  Section 3.3 of the paper groups the vectors of ONE
 * dimension d* in {channel, pixel} by their range and gives each group its own
 * scale s_k = (max - min) / 2^b and offset z_k = min.  This library keeps both
 * outlier kinds at once: rows (pixels) fall into P <= 2 classes by their range,
 * channels into NG groups (regular groups of `group_size` channels in order of
 * range, then the outlier cluster), and every cell (pixel class, channel group)
 * has its own (s, z).  P = 1 is the paper's channel case, NG = 1 its pixel case.
 */
#ifndef DGQ_H
#define DGQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dgq_status {
    DGQ_OK = 0,
    DGQ_EINVAL = -1,        /* null pointer, bad enum value, rows < 1 ...          */
    DGQ_EALIGN = -2,        /* a tensor base is not 16-byte aligned                */
    DGQ_ESHAPE = -3,        /* sizes inconsistent with the handle / each other     */
    DGQ_EUNSUPPORTED = -4,  /* valid but outside what the kernels cover            */
    DGQ_EHIP = -5,          /* a HIP runtime call failed                           */
    DGQ_EWORKSPACE = -6     /* workspace missing or too small                      */
} dgq_status;

typedef struct dgq_groups dgq_groups_t; /* one (layer, timestep) entry of the S, Z tables */
typedef struct dgq_weight dgq_weight_t;

/* K granule: every channel group is padded to a multiple of this many
   positions; padded positions carry code 0 and weight 0. */
#define DGQ_K_GRANULE 64

/* Most pixel classes a group handle can hold (the paper uses K = 8 or 16 groups). */
#define DGQ_MAX_PIXEL_CLASSES 16

/* dgq_groups_info_t.grouping */
#define DGQ_GROUPING_GRID 0     /* dgq_calibrate_groups: pixel classes x channel groups  */
#define DGQ_GROUPING_CHANNEL 1  /* dgq_calibrate_kmeans along the channel dimension      */
#define DGQ_GROUPING_PIXEL 2    /* dgq_calibrate_kmeans along the pixel dimension        */

/* dgq_calibrate_kmeans `dimension` */
#define DGQ_DIM_AUTO (-1)    /* d* = argmax_d D_d (Eq. 5)                                */
#define DGQ_DIM_CHANNEL 0
#define DGQ_DIM_PIXEL 1

typedef struct dgq_groups_info {
    int32_t channels;            /* C                                               */
    int32_t act_bits;            /* 4 or 8                                          */
    int32_t group_size;          /* G                                               */
    int32_t n_pixel_classes;     /* P: as requested (grid), clusters found (pixel)  */
    int32_t n_groups;            /* NG                                              */
    int32_t k_padded;            /* K' = padded contraction length                  */
    int32_t n_outlier_channels;  /* size of the upper range cluster                 */
    int32_t n_regular_groups;    /* groups cut from the lower cluster               */
    int32_t dstar;               /* argmax_d D_d: 0 = channel, 1 = pixel            */
    int32_t code_offset;         /* stored code = q - code_offset (128 / 0)         */
    int32_t n_class1_rows;       /* calibration rows in the outlier pixel class     */
    float tau_pix;               /* row-range threshold (+inf: single class)        */
    double d_channel, d_pixel;   /* D_d of Section 3.3                              */
    int32_t grouping;            /* DGQ_GROUPING_*                                  */
    int32_t reserved;
} dgq_groups_info_t;

/*
 * Calibration of one layer (Section 3.3: D_d, d*, K-means grouping by range,
 * s_k and z_k).  x_cal: device fp32 [rows, channels], one row per pixel with the
 * batch flattened into rows.
 *   1. row range w_r = max_c - min_c; exact 1-D 2-means on {w_r} gives the
 *      threshold tau_pix; class(r) = [w_r > tau_pix]        (n_pixel_classes == 2)
 *   2. D_channel, D_pixel and d* over the whole tensor (reported)
 *   3. channel range over class-0 rows; exact 1-D 2-means separates the outlier
 *      cluster; each cluster, sorted by (range, index), is cut into blocks of
 *      group_size channels; every block is padded to DGQ_K_GRANULE positions
 *   4. per cell: s = (max - min) / 2^act_bits (1 if max == min), z = min; a cell
 *      with no calibration rows copies class 0
 * act_bits in {4, 8}; group_size a positive multiple of DGQ_K_GRANULE;
 * channels >= 1; rows >= 1.  Blocks until the tables are built (the reductions
 * run on `stream`, the clustering on the host).  *out receives a new handle.
 */
int dgq_calibrate_groups(const float *x_cal, int64_t rows, int32_t channels,
                         int32_t act_bits, int32_t group_size,
                         int32_t n_pixel_classes, void *stream,
                         dgq_groups_t **out);

/*
 * Calibration of one layer exactly as Section 3.3 states it: ONE dimension is grouped.
 *   1. D_channel and D_pixel (Eq. 4) from the per-channel and per-pixel maxima and minima
 *      of the whole tensor; d* = argmax (Eq. 5; channel on a tie), or `dimension` if it
 *      is not DGQ_DIM_AUTO
 *   2. the vectors of d* (channels: a column of x_cal; pixels: a row) are clustered by
 *      their range max - min into n_clusters groups by K-means, solved exactly (dynamic
 *      programme over the sorted ranges; fewer clusters if there are fewer distinct ranges)
 *   3. each group k: s_k = (max - min) / 2^act_bits (1 if max == min), z_k = min over the
 *      calibration activations that belong to it (Eq. 6)
 * Channel dimension: one pixel class, n_groups = clusters found, the channels of a
 * group in (range, index) order, every group padded to DGQ_K_GRANULE positions (groups
 * have whatever size the clustering gives them; group_size reads 0).
 * Pixel dimension: one channel group (natural channel order), n_pixel_classes = clusters
 * found (<= DGQ_MAX_PIXEL_CLASSES); at run time the class of a row is the number of
 * thresholds below its range (dgq_groups_thresholds), i.e. the nearest cluster centre.
 * One handle is one (layer, timestep) entry of the S, Z tables of Eq. 7: calibrate one
 * per denoising step and pass the step's handle to the hot calls.
 * 1 <= n_clusters <= DGQ_MAX_PIXEL_CLASSES.  The host clustering takes O(n_clusters * n log n)
 * operations for n vectors (divide and conquer over the monotone best cuts), so the pixel
 * dimension takes every calibration row (64 prompts of 4096 pixels are 262144).  Blocks.
 * The handle works with dgq_pack_weight, dgq_quantize_act and dgq_linear as any other;
 * dgq_linear_geglu and acc_dump need n_pixel_classes <= 2.
 */
int dgq_calibrate_kmeans(const float *x_cal, int64_t rows, int32_t channels,
                         int32_t act_bits, int32_t n_clusters, int32_t dimension,
                         void *stream, dgq_groups_t **out);

/*
 * 3 x 3 convolution (stride 1, zero padding 1) through the same quantizer and contraction:
 * the paper quantizes every layer of the U-Net with the activation quantizer of Section 3.3,
 * convolutions included.  With the activation map x [B*H*W, C] (one row per pixel, pixels
 * row-major) quantized once by dgq_quantize_act(g, x), the convolution is the linear layer
 *   y[r, o] = sum_t sum_c x^[r_t, c] w[o, t, c],  t = 3 (dy + 1) + (dx + 1),
 *   r_t = the pixel (h + dy, w + dx) of the same image, x^ = 0 outside it,
 * over 9 C "channels" (tap t's copy of channel c is channel t C + c).
 *
 * dgq_groups_for_conv3x3 (offline): the group tables of that layer -- g's permutation,
 * groups, scales and offsets replicated for the nine taps (channels = 9 C, k_padded = 9 K',
 * n_groups = 9 NG).  g must have one pixel class (DGQ_EUNSUPPORTED otherwise).  Pass the
 * new handle to dgq_pack_weight with w fp32 [O, 9 C] (tap-major rows [o][dy][dx][c]) and to
 * dgq_linear; free it with dgq_groups_free.
 *
 * dgq_conv3x3_codes (hot call; enqueues on `stream`, neither synchronises nor allocates):
 * unfolds the CODES of the map: codes9 (dgq_codes_bytes(g9, B*H*W) bytes) receives, for
 * every pixel and tap, the code row of the neighbouring pixel, and outside the image the
 * code of the value 0 (what quantizing the zero-padded, unfolded activations would give).
 *   codes: as written by dgq_quantize_act(g, x) for rows = B*H*W
 * The row classes written by dgq_quantize_act (all 0) serve the convolution's dgq_linear too.
 */
int dgq_groups_for_conv3x3(const dgq_groups_t *g, dgq_groups_t **out);
int dgq_conv3x3_codes(const dgq_groups_t *g9, const int8_t *codes, int32_t B, int32_t H,
                      int32_t W, int8_t *codes9, void *stream);

/*
 * The same convolution without the unfolded code buffer: the contraction's loads gather the
 * nine taps themselves.  A tap (dy, dx) of a block of 16 consecutive output pixels (32 with
 * 4-bit codes) is the code block dy image rows further -- one contiguous 1 KiB piece per chunk,
 * as for a linear layer -- of the map shifted by dx pixels, or a block of the code of 0 outside
 * the image; so the quantizer writes the map's codes three times (the map, and the map shifted
 * one pixel to either side inside its image rows, the code of 0 at the image's edge), and
 * nothing is unfolded.  Needs W % 16 == 0 (8-bit codes) or W % 32 == 0 (4-bit codes), channels a
 * multiple of 4, one pixel class (DGQ_EUNSUPPORTED otherwise: use the calls above).
 *
 * dgq_quantize_act_conv3x3 (hot call): x fp32 [B*H*W, C] -> codes3, dgq_conv3x3_codes3_bytes(g9,
 *   B, H, W) bytes (three copies of dgq_codes_bytes(g, B*H*W)), and row_class u8 [B*H*W] (zeros).
 *   g: the map's handle, g9 = dgq_groups_for_conv3x3(g).
 * dgq_linear_conv3x3 (hot call): y fp32 [B*H*W, O] = the convolution; w = dgq_pack_weight(g9,
 *   [O, 9 C] tap-major kernel).  Same arithmetic as dgq_linear on the unfolded codes: the two
 *   results are equal bit for bit.
 * Both enqueue on `stream` and neither synchronise nor allocate.
 */
size_t dgq_conv3x3_codes3_bytes(const dgq_groups_t *g9, int32_t B, int32_t H, int32_t W);
int dgq_quantize_act_conv3x3(const dgq_groups_t *g, const dgq_groups_t *g9, const float *x,
                             int32_t B, int32_t H, int32_t W, int8_t *codes3,
                             uint8_t *row_class, void *stream);
int dgq_linear_conv3x3(const dgq_groups_t *g9, const dgq_weight_t *w, const int8_t *codes3,
                       const uint8_t *row_class, int32_t B, int32_t H, int32_t W, float *y,
                       void *stream);

/* Host copy of the n_pixel_classes - 1 ascending row-range thresholds (taus: host). */
int dgq_groups_thresholds(const dgq_groups_t *g, float *taus);

/* Host copy of the scalar results.  info: host. */
int dgq_groups_info(const dgq_groups_t *g, dgq_groups_info_t *info);

/*
 * Host copy of the tables (any pointer may be NULL to skip it); all host:
 *   perm [K']   original channel at padded position j, -1 for padding
 *   goff [NG+1] first padded position of each group (multiples of the granule)
 *   glen [NG]   channels in each group
 *   s, z [max(P,2)*NG] cell tables, class-major: s[p*NG + g] (P = n_pixel_classes; with
 *               P = 1 the second row repeats the first)
 */
int dgq_groups_tables(const dgq_groups_t *g, int32_t *perm, int32_t *goff,
                      int32_t *glen, float *s, float *z);

void dgq_groups_free(dgq_groups_t *g);

/*
 * Weight preparation for dgq_linear.  The paper leaves weight quantization to
 * other methods (Section 4.1, "Weight quantization"); here it is
 * per-output-channel symmetric round-to-nearest-even:
 *   sw[o] = max_c |W[o,c]| / qmax (1 for an all-zero row), qmax = 127 (w_bits 8)
 *   or 7 (w_bits 4);  wq = clamp(rne(W / sw), -qmax, qmax).
 * The integer rows are permuted and padded to the K' order of `g`; the
 * zero-point term of the dequantization
 *   zb[p][o] = sw[o] * sum_g (z[p,g] + code_offset * s[p,g]) * (sum_{j in g} wq[o,j]) + bias[o]
 * is precomputed per pixel class.
 * w: device fp32 [out_channels, channels]; bias: device fp32 [out_channels] or
 * NULL.  Blocks until done.  The handle stays tied to the group structure of g.
 */
int dgq_pack_weight(const dgq_groups_t *g, const float *w, const float *bias,
                    int32_t out_channels, int32_t w_bits, void *stream,
                    dgq_weight_t **out);

/* Host copies for inspection: wq host int8 [out_channels, channels] in the
   ORIGINAL channel order, sw host fp32 [out_channels]; either may be NULL. */
int dgq_weight_tables(const dgq_weight_t *w, int8_t *wq, float *sw);

/*
 * 4-bit weights at half the bytes (Section 4.1 quantizes weights to 4 bits; Table 1's
 * model-size column counts them as 4 bits each).  dgq_pack_weight keeps every integer
 * weight in a byte, the operand format of the matrix cores.  This call converts a handle
 * packed with w_bits = 4 to two weights per byte in place: its device footprint
 * (dgq_weight_device_bytes) drops from O_pad * K' to O_pad * K' / 2 bytes plus the
 * 12 * O_pad bytes of sw and zb.  A converted handle is accepted by dgq_linear only, which
 * then needs a workspace of dgq_linear_workspace_bytes() bytes (O_pad * K', 16-byte
 * aligned, caller-owned device memory, reusable between layers on one stream): a small
 * kernel sign-extends the nibbles into it right before the contraction, which runs
 * unchanged -- results are bit-identical to the unconverted handle's.  (Expanding in the
 * contraction's own fragment path would cost it twelve more vector instructions per
 * matrix instruction; the expansion kernel costs a few microseconds per call.)
 * The other linear entry points return DGQ_EUNSUPPORTED for a converted handle.
 * Blocks until done; allocates.  The handle must not be in use by any stream while it is
 * converted (it is the one call that changes a handle after creation).  Errors: DGQ_EINVAL (null), DGQ_EUNSUPPORTED (w_bits != 4,
 * or a handle from dgq_pack_weight_gated_for), DGQ_ESHAPE (already converted).
 */
int dgq_weight_pack_nibbles(dgq_weight_t *w, void *stream);

/* Device bytes the handle owns (integer weights, sw, zb, and the tables of a gated handle). */
size_t dgq_weight_device_bytes(const dgq_weight_t *w);

void dgq_weight_free(dgq_weight_t *w);

/*
 * Activation quantizer (linear quantizer of Section 3.1 with the cell
 * parameters of Section 3.3).  For every row r of x [rows, C]:
 *   class p = [max_c x - min_c x > tau_pix], in general the number of thresholds
 *             below max_c x - min_c x                       (decided at run time)
 *   for every real padded position j in group g, c = perm[j]:
 *     q = clamp(rne((x[r,c] - z[p,g]) * (1/s[p,g])), 0, 2^b - 1)
 *     stored code = q - code_offset;  padding positions store 0.
 * Subtraction and multiplication are separate fp32 operations (no FMA).
 *   codes: dgq_codes_bytes(g, rows) bytes, written in the block-tiled layout
 *          dgq_linear reads with 1 KiB direct-to-LDS loads.  A block is 1 KiB and
 *          holds one 64-position chunk of R consecutive rows (R = 16 at 8 bit,
 *          R = 32 at 4 bit); blocks are ordered [row block][chunk].  Inside a block,
 *          row t occupies bytes [t*B, (t+1)*B), B = 64 (8 bit) or 32 (4 bit), and its
 *          16-byte slots are XOR-permuted: slot k is stored at slot
 *              k ^ ( bit2(t) | ((bit1(t) ^ bit3(t)) << 1) )          (8 bit, 4 slots)
 *              k ^ bit3(t)                                           (4 bit, 2 slots)
 *          and, at 4 bit, rows t >= 16 keep the two 8-byte halves of every slot swapped.
 *          8 bit: one int8 per position.  4 bit: positions are packed in groups of 8
 *          into 4 bytes, byte i holding position i in its low nibble and position
 *          i+4 in its high nibble, each nibble the unsigned q.
 *          Rows of the last row block past `rows` are not written.
 *   row_class: uint8 [rows].
 */
int dgq_quantize_act(const dgq_groups_t *g, const float *x, int64_t rows,
                     int8_t *codes, uint8_t *row_class, void *stream);

/* Size in bytes of the code buffer for `rows` rows (rows rounded up to a block). */
size_t dgq_codes_bytes(const dgq_groups_t *g, int64_t rows);

/*
 * Quantized linear layer: grouped integer contraction and dequantization.
 *   acc[r,o,g] = sum_{j in g} code[r,j] * wq[o,j]                         (int32, exact)
 *   y[r,o]     = sw[o] * sum_g s[class(r),g] * float(acc[r,o,g]) + zb[class(r)][o]
 * (x_dq = s*(x_q) + z of Section 3.1 applied group by group; fp32 epilogue).
 *   codes, row_class: as written by dgq_quantize_act with the same g
 *   y: fp32 [rows, out_channels]
 *   acc_dump: NULL, or int32 [rows, out_channels, NG] receiving every group
 *             accumulator (debug / parity; slows the kernel down)
 *   workspace: device memory of at least dgq_linear_workspace_bytes(g, w, rows) bytes,
 *             16-byte aligned: 0 bytes (pass NULL / 0) unless w was converted by
 *             dgq_weight_pack_nibbles, whose expanded weights it receives.  The call only
 *             enqueues work on `stream`; the workspace may be reused by the next call on
 *             the same stream.  Too small: DGQ_EWORKSPACE.
 */
int dgq_linear(const dgq_groups_t *g, const dgq_weight_t *w, const int8_t *codes,
               const uint8_t *row_class, int64_t rows, float *y,
               int32_t *acc_dump, void *workspace, size_t workspace_bytes,
               void *stream);

/*
 * The same layer with the gated activation of the transformer feed-forward fused into
 * the epilogue.  The networks the paper quantizes (Section 4.1: Stable Diffusion
 * v1.4, SDXL-Turbo) apply, to the result y = [a | b] of the first feed-forward
 * projection (a = channels [0, O/2), b = channels [O/2, O)),
 *   out[r,c] = a[r,c] * GELU(b[r,c]),   GELU(t) = t * Phi(t) = t * (1 + erf(t / sqrt 2)) / 2.
 * y[r,o] is formed exactly as in dgq_linear and never written.  Phi comes from the
 * rational approximation of erfc (Abramowitz and Stegun 7.1.26) in fp32: absolute
 * error of GELU(t) at most 4e-7 |t|.  w is an ordinary dgq_pack_weight handle of all
 * O rows.
 *   y: fp32 [rows, out_channels / 2]
 * out_channels must be a multiple of 256 (DGQ_EUNSUPPORTED otherwise).  No
 * accumulator dump, no workspace.  Enqueues on `stream`; does not synchronise or
 * allocate.
 */
int dgq_linear_geglu(const dgq_groups_t *g, const dgq_weight_t *w, const int8_t *codes,
                     const uint8_t *row_class, int64_t rows, float *y, void *stream);

/*
 * Two feed-forward layers chained without the fp32 activation between them: the gated
 * layer's epilogue puts out[r,c] = a[r,c] * GELU(b[r,c]) (as in dgq_linear_geglu) straight
 * through the FOLLOWING layer's activation quantizer (Section 3.1's linear quantizer with
 * that layer's group-wise static (s_k, z_k), Section 3.3) and writes that layer's codes.
 * The following layer must be grouped along the channel dimension only (one pixel class:
 * dgq_calibrate_kmeans with the channel dimension, or dgq_calibrate_groups with
 * n_pixel_classes = 1), so that a code depends on nothing but its own value and its
 * channel's group; its codes may be 8 or 4 bits wide.
 *
 * dgq_pack_weight_gated_for (offline, blocking): as dgq_pack_weight for layer g, whose
 * out_channels = 2 * (channels of g_next) rows of w are [value rows | gate rows]; the
 * packed rows are reordered into g_next's permuted, padded K' order so that the epilogue's
 * output columns are g_next's code positions, and the handle keeps a copy of g_next's
 * per-chunk (z, 1/s) and padding mask (g_next may be freed afterwards).  The handle is
 * accepted by dgq_linear_geglu_requant only.
 *
 * dgq_linear_geglu_requant (hot call; enqueues on `stream`, neither synchronises nor
 * allocates):
 *   codes, row_class: of layer g, as written by dgq_quantize_act
 *   codes_next: dgq_codes_bytes(g_next, rows) bytes; receives exactly what
 *               dgq_quantize_act(g_next, out) would write (8-bit: stored code = q - 128;
 *               4-bit: packed nibbles; padding positions 0; rows past `rows` in the last
 *               row block untouched), up to
 *               the rounding of out: a code whose pre-rounding value (out - z) / s lies
 *               within the fp32 error of out of a half-integer may differ by one
 *   row_class_next: u8 [rows], receives zeros (the single pixel class)
 */
int dgq_pack_weight_gated_for(const dgq_groups_t *g, const dgq_groups_t *g_next,
                              const float *w, const float *bias, int32_t out_channels,
                              int32_t w_bits, void *stream, dgq_weight_t **out);
int dgq_linear_geglu_requant(const dgq_groups_t *g, const dgq_weight_t *w,
                             const int8_t *codes, const uint8_t *row_class, int64_t rows,
                             int8_t *codes_next, uint8_t *row_class_next, void *stream);

size_t dgq_linear_workspace_bytes(const dgq_groups_t *g, const dgq_weight_t *w,
                                  int64_t rows);

/*
 * Cross-attention with log2-quantized probabilities (Section 3.3,
 * attention-aware quantization; log quantizer of Section 3.1).
 *   L[b,h,i,j] = (q[b,i,h,:] . k[b,j,h,:]) / sqrt(d) + key_bias[j]
 *   A = softmax_j(L) over all nk keys, fp32
 *   scale_out[b] = s_b = max over h, i and j >= 1 of A      (prompt-specific scale)
 *   code[b,h,i,j] = clamp(rne(-log2(A / s_b)), 0, 2^attn_bits - 1),  j >= 1;
 *                   a probability that rounds to zero in fp32 gets 2^attn_bits - 1
 *   out[b,i,h,:] = A[..,0] * v[b,0,h,:] + s_b * sum_{j>=1} 2^(-code) * v[b,j,h,:]
 * Column 0 (the <start> token) bypasses the quantizer; no renormalisation.
 *   q, out: fp32 [B, N, H, d];  k, v: fp32 [B, nk, H, d];  key_bias: fp32 [nk] or NULL
 *   scale_out: fp32 [B] (written);  codes_dump: NULL or uint8 [B, H, N, nk-1]
 *   workspace: device scratch of dgq_xattn_workspace_bytes(...) bytes, 16-byte aligned;
 *              contents are overwritten.  One float per (b, h, query), rounded up to 256
 *              bytes, is the least that is accepted (DGQ_EWORKSPACE below that); with the
 *              full size the maxima behind scale_out travel through the workspace as well
 *              and the call is one kernel launch shorter.  Same results either way.
 * Limits: 2 <= nk <= 128, 1 <= d <= 256, attn_bits in {4, 8}.
 * Two kernels run back to back on `stream` (all probabilities must be known
 * before any of them can be coded).  Shapes with d a multiple of 8 up to 96 and
 * nk <= 126, or up to 160 and nk <= 94, run on the matrix cores, with q and k each split into two fp16
 * pieces (|q| and |k| * log2(e) / sqrt(d) must stay below 65504 there) and one
 * float per (b, h, query) kept in the workspace between the two kernels; every
 * other shape uses fp32 vector arithmetic and no workspace.
 */
int dgq_xattn_logq(const float *q, const float *k, const float *v,
                   const float *key_bias, int32_t B, int32_t N, int32_t H,
                   int32_t d, int32_t nk, int32_t attn_bits, float *out,
                   float *scale_out, uint8_t *codes_dump, void *workspace,
                   size_t workspace_bytes, void *stream);

size_t dgq_xattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d,
                                 int32_t nk);

/*
 * dgq_xattn_logq for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same computation, same kernels and the same results bit for bit; the float per (b, h,
 * query) kept between the two kernels lives in a fixed array inside the library's device
 * image instead of a caller's workspace.  The call allocates nothing and frees nothing.
 *   Limit: B * H * N <= DGQ_XATTN_NOALLOC_MAX_ROWS (4 MiB of floats; DGQ_EWORKSPACE beyond,
 *          nothing is enqueued).  Every GPU the library runs on holds the array (those 4 MiB
 *          and 0.3 MiB for the maxima behind scale_out) from the first call on it until the
 *          process ends.
 *   Sharing: all calls on one GPU use the same array, whichever stream they run on, and the
 *          array keeps the last call's contents (nothing in it needs clearing: the first
 *          kernel writes every entry the second one reads).  Two calls that overlap in time
 *          on one GPU race; calls on one stream, or ordered by events, do not.
 * Arguments as in dgq_xattn_logq, without workspace and workspace_bytes.
 */
#define DGQ_XATTN_NOALLOC_MAX_ROWS (1u << 20)
int dgq_xattn_logq_noalloc(const float *q, const float *k, const float *v,
                           const float *key_bias, int32_t B, int32_t N, int32_t H,
                           int32_t d, int32_t nk, int32_t attn_bits, float *out,
                           float *scale_out, uint8_t *codes_dump, void *stream);

/* Host string describing the last error on this thread ("" if none). */
const char *dgq_last_error(void);

/* Library version as major*10000 + minor*100 + patch. */
int dgq_version(void);

/*
 * The same attention with a GIVEN prompt scale: the log quantizer without dynamic
 * quantization of the paper's ablation (Section 4.3), whose scale comes from calibration
 * or from a running maximum over earlier denoising steps.  scale_in: fp32 [B].  With the
 * scale known beforehand the two passes of dgq_xattn_logq collapse into one kernel and Q
 * is read once; probabilities above the scale saturate at code 0.  scale_out: NULL, or
 * fp32 [B] (not scale_in) receiving this call's own maximum, e.g. to update a running
 * estimate.  No workspace.  Everything else as in dgq_xattn_logq; with scale_in equal to
 * what dgq_xattn_logq reports, codes and product are the same bit for bit.
 */
int dgq_xattn_logq_static(const float *q, const float *k, const float *v,
                          const float *key_bias, int32_t B, int32_t N, int32_t H, int32_t d,
                          int32_t nk, int32_t attn_bits, const float *scale_in, float *out,
                          float *scale_out, uint8_t *codes_dump, void *stream);

/*
 * Self-attention with log2-quantized probabilities.  Section 3.3 applies the logarithmic
 * quantizer of Section 3.1 to self- and cross-attention alike; separating the <start>
 * column and the dynamic scale are stated for cross-attention only.  Here every
 * probability is quantized and the scale is given:
 *   L[b,h,i,j] = (q[b,i,h,:] . k[b,j,h,:]) / sqrt(d),  A = softmax_j(L) over all N keys
 *   A^q = clamp(rne(-log2(A / s[b])), 0, 2^attn_bits - 1)   (A = 0: the top code)
 *   out[b,i,h,:] = sum_j s[b] 2^-A^q[b,h,i,j] v[b,j,h,:]
 *   q, k, v, out: fp32 [B, N, H, d] (device); v may be the V^ of dgq_quantize_value
 *   scale_in:  fp32 [B], the given scale (1 for the plain log2 quantizer of a probability,
 *              or a calibrated maximum); a value <= 0 gives out = 0
 *   scale_out: NULL, or fp32 [B] receiving max A of this call
 *   codes_dump: NULL, or u8 [B, H, N, N] receiving every code (debug / parity)
 *   workspace: dgq_selfattn_workspace_bytes(B, N, H, d) bytes, 16-byte aligned; holds K
 *              and V^T in the matrix cores' operand pieces, rewritten by every call
 * d % 8 == 0 and d <= 160 (DGQ_EUNSUPPORTED otherwise; the workspace size reads 0).
 * attn_bits in {4, 8}.  Enqueues on `stream`; does not synchronise or allocate.
 */
size_t dgq_selfattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d);
int dgq_selfattn_logq(const float *q, const float *k, const float *v, int32_t B, int32_t N,
                      int32_t H, int32_t d, int32_t attn_bits, const float *scale_in,
                      float *out, float *scale_out, uint8_t *codes_dump, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * The quantized value tensor V^ of the attention product A^ V^ (Section 3.3).  Every
 * (prompt, head) slice V[b, :, h, :] goes through the linear quantizer of Section 3.1
 * with its own range:
 *   s = (max - min) / 2^v_bits (1 if max == min),  z = min
 *   q = clamp(rne((v - z) * (1/s)), 0, 2^v_bits - 1)      (separate fp32 operations)
 *   v_hat = s * q + z                                      (rounded once to fp32)
 * Pass v_hat as `v` to dgq_xattn_logq: the kernel then forms exactly A^ V^, the
 * power-of-two weights times the dequantized codes (on this hardware the matrix cores do
 * what shift-and-add does elsewhere).  The text context does not change over the
 * denoising steps, so this is one small launch per prompt, not per step.
 *   v, v_hat: fp32 [B, nk, H, d] (may be the same buffer);  v_bits: 4 or 8
 *   codes:  NULL, or uint8 [B, nk, H, d] receiving q
 *   params: NULL, or fp32 [B, H, 2] receiving (s, z)
 * Enqueues on `stream`; neither synchronises nor allocates.
 */
int dgq_quantize_value(const float *v, int32_t B, int32_t nk, int32_t H, int32_t d,
                       int32_t v_bits, float *v_hat, uint8_t *codes, float *params,
                       void *stream);

/*
 * The attention product on V^'s INTEGER codes, by shifts and adds (Section 3.1: the log
 * quantizer "allows bit-shifting operations"; Section 3.3: A^ V^ with the <start> column
 * multiplied in full precision).  With 4-bit probability codes every quantized weight is
 * s_b 2^-15 (1 << (15 - A^q)) and V^ = s_v q_v + z_v, so
 *   out[b,i,h,:] = A[..,0] * v_hat[b,0,h,:]
 *                + s_b 2^-15 * ( s_v * sum_{j>=1} (q_v[b,j,h,:] << (15 - A^q[b,h,i,j]))
 *                              + z_v * sum_{j>=1} (1 << (15 - A^q[b,h,i,j])) ),
 * both sums exact in int32; v_hat[0] = s_v q_v[0] + z_v rounded to fp32 as dgq_quantize_value
 * writes it.  Logits, soft-max, scale and codes as in dgq_xattn_logq (its fp32 vector
 * kernels; no workspace).
 *   v_codes:  uint8 [B, nk, H, d], the 8-bit codes of dgq_quantize_value
 *   v_params: fp32 [B, H, 2], its (s_v, z_v)
 *   attn_bits: 4 (with 8-bit codes 1 << (255 - A^q) has no integer accumulator:
 *              DGQ_EUNSUPPORTED)
 *   acc_dump: NULL, or int32 [B, N, H, d] receiving the first integer sum (debug / parity)
 * Enqueues on `stream`; neither synchronises nor allocates.
 */
int dgq_xattn_logq_intv(const float *q, const float *k, const uint8_t *v_codes,
                        const float *v_params, const float *key_bias, int32_t B, int32_t N,
                        int32_t H, int32_t d, int32_t nk, int32_t attn_bits, float *out,
                        float *scale_out, uint8_t *codes_dump, int32_t *acc_dump, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DGQ_H */
