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
//   workgroup = WR x WO wavefronts; wavefront = BR x BO blocks of
//               v_mfma_i32_32x32x32_i8 (default 4 x 2 waves of 1 x 2 blocks:
//               a 128 x 128 output tile, 32 x 64 per wave, so that 128
//               registers suffice and four waves share a SIMD: a wave's
//               fold follows its MFMAs, so the matrix pipe and the vector
//               ALU are kept busy together by waves in different phases)
//   K loop    = 64-position chunks (the K granule).  Chunks travel from global
//               memory straight into LDS (global_load_lds_dwordx4, no staging
//               registers) through a ring of stages, one barrier per chunk,
//               and the loop is software-pipelined over half chunks so LDS
//               reads overlap the matrix cores.  A group is a whole number of
//               chunks, so each group ends on a chunk boundary where its int32
//               block is folded into fp32 (convert + one FMA with a scalar scale
//               per output); the next group's first MFMA starts from C = 0.
//   classes   = a wavefront whose rows all share one pixel class p (almost all
//               wavefronts: outlier pixels are rare) takes s[p, g] from a scalar
//               register; a wavefront with mixed rows selects the scale per
//               accumulator register through lane masks prepared before the
//               loop.  The two cases are separate instantiations of the whole
//               loop + epilogue, so the common one carries no class logic.
// Codes and weights are stored block-tiled in global memory (1 KiB = one chunk
// of 16 rows, or of 32 rows of packed 4-bit codes), so that one direct-to-LDS
// instruction copies 1 KiB of contiguous memory: loads that gather 64-byte row
// pieces cost about twice as much in the address path.  LDS rows are 64 B
// (8-bit codes, weights) or 32 B (packed 4-bit codes); the 16-byte slots of a
// row are XOR-swizzled with row bits (already in global memory) so that the
// 16-byte fragment reads of 32 consecutive rows spread over all banks.
// Activation rows are the MFMA's M index (spread over accumulator registers)
// and output channels its N index (lane % 32), so a store instruction writes
// 128 contiguous bytes per row, and sw / zb are per-lane constants.
#include <cstdlib>
#include <type_traits>

#include "dgq_internal.h"

namespace dgq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kStageBudget = 160 * 1024;  // LDS bytes per CU

// One direct-to-LDS load: lane j copies 16 bytes from sbase + voff to LDS address l0 + 16 j.
// Written out so that the address is a scalar base plus one 32-bit lane offset (the
// compiler's form of the builtin keeps a 64-bit address per lane and spends two vector
// adds per load on it; a vector instruction costs this kernel about four clocks of SIMD
// time).  M0 carries the LDS address; nothing else in these kernels uses M0.  The load is
// invisible to the compiler's wait-count bookkeeping, which is what the kernel wants: it
// places every vmcnt wait itself.
#define DGQ_LDS_DMA16(sbase, voff, l0)                                                \
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"      \
                 :                                                                    \
                 : "v"(voff), "s"(sbase), "s"(l0)                                     \
                 : "memory", "m0")

#define DGQ_WAIT_VMCNT(N) \
    __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// Wait until at most min(later, L) chunks of LOADS loads each are still pending.
template <int L, int LOADS>
__device__ inline void wait_chunks_pending(int32_t later) {
    if constexpr (L <= 0) {
        DGQ_WAIT_VMCNT(0);
    } else {
        if (later >= L)
            DGQ_WAIT_VMCNT(L * LOADS);
        else
            wait_chunks_pending<L - 1, LOADS>(later);
    }
}

// GELU(t) = t * Phi(t).  Phi through the rational approximation 7.1.26 of Abramowitz and
// Stegun for erfc: with z = |t| / sqrt 2 and u = 1 / (1 + p z),
//     erfc(z) = (a1 u + a2 u^2 + a3 u^3 + a4 u^4 + a5 u^5) exp(-z^2),   |error| <= 1.5e-7,
// so Phi(t) = erfc(z) / 2 for t < 0 (no cancellation in the lower tail) and 1 - erfc(z) / 2
// otherwise: absolute error of Phi below 1e-7 plus fp32 rounding, at a third of the
// instructions of the library erf (which made the fused epilogue slower than the plain one).
__device__ inline float gelu(float t) {
    const float z = fabsf(t) * 0.70710678118654752f;
    const float u = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
    float pl = fmaf(1.061405429f, u, -1.453152027f);
    pl = fmaf(pl, u, 1.421413741f);
    pl = fmaf(pl, u, -0.284496736f);
    pl = fmaf(pl, u, 0.254829592f);
    pl = pl * u;
    // exp(-z^2) = 2^(-t^2 / 2 * log2 e)
    const float e = __builtin_amdgcn_exp2f(t * t * -0.72134752044448170f);
    const float half_erfc = 0.5f * pl * e;
    const float phi = t < 0.0f ? half_erfc : 1.0f - half_erfc;
    return t * phi;
}

// Tile shape: WR x WO wavefronts, each BR x BO blocks of 32 x 32 outputs.
template <int ABITS_, int WR_, int WO_, int BR_, int BO_, int STAGES_, int OCC_>
struct Cfg {
    static constexpr int ABITS = ABITS_, WR = WR_, WO = WO_, BR = BR_, BO = BO_, STAGES = STAGES_;
    static constexpr int OCC = OCC_;  // wavefronts per SIMD the register budget is sized for
    static constexpr int NW = WR * WO, THREADS = 64 * NW;
    static constexpr int TR = WR * BR * 32, TO = WO * BO * 32;
    static constexpr int AROW = ABITS == 8 ? 64 : 32;  // bytes per code row per chunk
    static constexpr int ABYTES = TR * AROW, BBYTES = TO * 64;
    static constexpr int STAGE_BYTES = ABYTES + BBYTES;
    static constexpr int AINSTR = ABYTES / 1024, BINSTR = BBYTES / 1024;  // 1 KB per DMA instruction
    // loads per wave per chunk; when the blocks do not divide evenly the last block is
    // copied by more than one wave (same bytes to the same place)
    static constexpr int LOADS = (AINSTR + BINSTR + NW - 1) / NW;
    static_assert(STAGES >= 3 && STAGES * STAGE_BYTES <= kStageBudget, "LDS ring does not fit");
    static_assert((STAGES - 2) * LOADS < 64, "vmcnt is a 6-bit counter");
};

// GEGLU: the tile's TO weight rows are TO/2 "value" rows o0/2 .. and the TO/2 "gate" rows
// O/2 + o0/2 .. of the same output channels; the epilogue writes value * GELU(gate) into
// y [rows, O/2] (the gated feed-forward of the transformer blocks), so the 2x wider
// pre-activation never reaches memory.  Needs BO == 2 and O % (2 TO) == 0.
//
// GEGLU == 2 (gated + requantized): the tile's output channels are, in order, the K'
// positions of the NEXT layer's channel groups (the weight rows were packed in that
// order), that layer has one pixel class, and the epilogue puts value * GELU(gate) straight
// through its quantizer: y is that layer's block-tiled code buffer (rq_bits wide), rq_zi the
// (offset, 1 / step) of each of its 64-position chunks, rq_keep one byte per position
// (0xFF, or 0 for padding, whose stored code is 0), rq_cls its row classes (all 0).  The
// fp32 activation between the two layers never reaches memory.
//
// MULTI: more than two pixel classes and ONE channel group (the pixel-dimension grouping
// of Section 3.3).  The class of the row behind every accumulator register travels as a
// 4-bit field; the single fold and the epilogue read that class's scale and offset from a
// small LDS table, and the zero-point term is zoff[class] * (sw[o] * wsum[o]) + bias[o],
// whose two class-independent rows arrive in place of zb[0] and zb[1].
//
// CONV: the layer is a 3 x 3 convolution (stride 1, zero padding 1) and the nine taps are
// GATHERED by the direct-to-LDS loads instead of being unfolded in memory.  `codes` holds
// three copies of the map's code tensor, copy c at codes + c * cv.copy_bytes: copy 1 is the map
// itself, copy 0 / copy 2 hold in row r the code row of the pixel to the left / right of r
// (the code of the value 0 where the image ends).  Tap t = 3 (dy + 1) + (dx + 1) of a 16-row
// (32-row) block of output pixels is then the block dy image rows further in copy dx + 1 --
// one contiguous 1 KiB piece per chunk, as for a linear layer -- or, outside the image, a block
// of the code of 0 (cv.fill: one 1 KiB block per chunk).  Needs the image width to be a
// multiple of the rows of a block.  The K' order is tap-major, K' = 9 K'_map.
struct ConvGather {
    int32_t w_blocks = 0;    // image width / rows per code block
    int32_t height = 0;      // image height
    int32_t chunks = 0;      // chunks per tap (K'_map / 64)
    int64_t copy_bytes = 0;  // bytes of one copy of the code tensor
    const int8_t *fill = nullptr;
};

template <class CF, bool DUMP, int GEGLU, bool MULTI, bool CONV = false>
__global__ __launch_bounds__(CF::THREADS, CF::OCC) void k_linear(
    const int8_t *__restrict__ codes, const uint8_t *__restrict__ row_class,
    const int8_t *__restrict__ wq, const float *__restrict__ sw, const float *__restrict__ zb,
    const float *__restrict__ s_tab, const float *__restrict__ zoff_tab, int32_t P,
    const int32_t *__restrict__ gchunk, int64_t rows, int32_t O,
    int32_t O_pad, int32_t Kp, int32_t NG, int32_t tiles_r, int32_t tiles_o, int32_t per_xcd,
    int32_t super_rows, float *__restrict__ y, int32_t *__restrict__ acc_dump,
    const float2 *__restrict__ rq_zi, const uint8_t *__restrict__ rq_keep,
    uint8_t *__restrict__ rq_cls, int32_t rq_bits, ConvGather cv) {
    constexpr int ABITS = CF::ABITS, BR = CF::BR, BO = CF::BO, STAGES = CF::STAGES;
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];

    // ---- tile and class of this workgroup.  Workgroup w runs on XCD w % 8: give every
    // XCD a contiguous range of tile indices and walk it in super-columns of `super_rows` row tiles so
    // that the tiles resident on one XCD share code rows and weight rows in its L2.
    const int32_t T = tiles_r * tiles_o;
    const int32_t t = (int32_t)(blockIdx.x & 7) * per_xcd + (int32_t)(blockIdx.x >> 3);
    if (t >= T) return;
    const int32_t in_super = super_rows * tiles_o;
    const int32_t first_r = (t / in_super) * super_rows;
    const int32_t gsz = tiles_r - first_r < super_rows ? tiles_r - first_r : super_rows;
    const int32_t tile_r = first_r + (t % in_super) % gsz;
    const int32_t tile_o = (t % in_super) / gsz;

    const int tid = threadIdx.x;
    // the wave index is uniform: say so, and everything derived from it (block
    // pointers, LDS stage addresses, the M0 values of the direct-to-LDS loads) is
    // computed on the scalar unit instead of per lane
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wr = wave / CF::WO, wo = wave % CF::WO;
    const int m32 = lane & 31, kh = lane >> 5;
    const int64_t r0 = (int64_t)tile_r * CF::TR;
    const int32_t o0 = tile_o * CF::TO;
    const int32_t n_chunks = Kp >> 6;

    // ---- direct-to-LDS load plan: the operands are stored block-tiled, one block =
    // 1 KiB = one chunk of 16 rows (32 rows of packed 4-bit codes), already in the
    // slot-swizzled order LDS wants.  One instruction copies one block (lane j moves
    // bytes [16j, 16j+16)); the blocks of a chunk are dealt round-robin to the waves.
    constexpr int kARows = ABITS == 8 ? 16 : 32;  // rows per code block
    const int64_t n_ablocks = (rows + kARows - 1) / kARows;
    const int8_t *src[CF::LOADS];  // uniform per wave
    int dst[CF::LOADS];
    int64_t a_blk[CF::LOADS];  // CONV: the load's row block (-1: a weight block) and its image row
    int32_t a_h[CF::LOADS];
    const uint32_t lane16 = lane * 16;
    auto lds_addr = [](const uint8_t *p) {  // 32-bit LDS address of a pointer into `lds`
        return (uint32_t)reinterpret_cast<uintptr_t>(
            (const __attribute__((address_space(3))) uint8_t *)p);
    };
#pragma unroll
    for (int j = 0; j < CF::LOADS; ++j) {
        int i = wave + CF::NW * j;
        i = i < CF::AINSTR + CF::BINSTR ? i : CF::AINSTR + CF::BINSTR - 1;
        if (i < CF::AINSTR) {
            int64_t blk = r0 / kARows + i;
            blk = blk < n_ablocks ? blk : n_ablocks - 1;  // clamp: rows past the end are never stored
            src[j] = codes + ((blk * n_chunks) << 10);
            dst[j] = i * 1024;
            a_blk[j] = blk;
            a_h[j] = CONV ? (int32_t)((blk / cv.w_blocks) % cv.height) : 0;
        } else {
            a_blk[j] = -1;
            a_h[j] = 0;
            const int ib = i - CF::AINSTR;
            int32_t rb = o0 / 16 + ib;  // 16-row block of the packed weights
            if (GEGLU) {
                constexpr int HB = CF::BINSTR / 2;  // value blocks first, then the gate blocks
                rb = ib < HB ? (o0 / 2) / 16 + ib : (O / 2 + o0 / 2) / 16 + (ib - HB);
            }
            src[j] = wq + (((int64_t)rb * n_chunks) << 10);
            dst[j] = CF::ABYTES + ib * 1024;
        }
    }
    // CONV: chunks are issued strictly in order, so the tap (dy + 1, dx + 1) and the chunk
    // inside the tap of the next chunk to issue are running counters, not divisions
    int32_t cv_c = 0, cv_dx = 0, cv_dy = 0;
    auto issue_chunk_at = [&](int32_t ch, int stage) __attribute__((always_inline)) {
        uint8_t *base = lds + stage * CF::STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < CF::LOADS; ++j) {
            const int8_t *p = src[j] + ((int64_t)ch << 10);
            if (CONV && a_blk[j] >= 0) {
                const int32_t hh = a_h[j] + cv_dy - 1;
                const int64_t blk = a_blk[j] + (int64_t)(cv_dy - 1) * cv.w_blocks;
                p = (uint32_t)hh < (uint32_t)cv.height
                        ? codes + cv_dx * cv.copy_bytes + ((blk * cv.chunks + cv_c) << 10)
                        : cv.fill + ((int64_t)cv_c << 10);
            }
            DGQ_LDS_DMA16(p, lane16, lds_addr(base + dst[j]));
        }
        if (CONV) {
            if (++cv_c == cv.chunks) {
                cv_c = 0;
                if (++cv_dx == 3) {
                    cv_dx = 0;
                    ++cv_dy;
                }
            }
        }
    };
    auto issue_chunk = [&](int32_t ch) { issue_chunk_at(ch, ch % STAGES); };

    // ---- prologue: fill the ring before anything else is loaded ----------------------------
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st)
        if (st < n_chunks) issue_chunk(st);

    // ---- small global loads, branch-free (clamped indices) so that none of them is
    // waited for before the lines that consume it, long after the ring is in flight
    bool row_in[BR];
    uint8_t row_c1[BR];
#pragma unroll
    for (int a = 0; a < BR; ++a) {
        const int64_t r = r0 + (wr * BR + a) * 32 + m32;
        row_in[a] = r < rows;
        row_c1[a] = row_class[row_in[a] ? r : rows - 1];
    }
    float col_sw[BO], col_zb0[BO], col_zb1[BO];  // per-lane output-channel constants
#pragma unroll
    for (int b = 0; b < BO; ++b) {
        int32_t o = o0 + (wo * BO + b) * 32 + m32;  // o < O_pad always
        if (GEGLU) o = (b ? O / 2 : 0) + o0 / 2 + wo * 32 + m32;
        col_sw[b] = sw[o];
        col_zb0[b] = zb[o];
        col_zb1[b] = zb[O_pad + o];
    }
    const int32_t tg = tid < NG ? tid : NG - 1;
    const int32_t t_end = gchunk[tg + 1];
    // MULTI: thread t < P carries class t's scale and offset
    const int32_t tp = tid < P ? tid : P - 1;
    const float t_s0 = MULTI ? s_tab[tp] : s_tab[tg], t_s1 = MULTI ? zoff_tab[tp] : s_tab[NG + tg];

    // ---- fragment read offsets (per lane, per k-step) ---------------------------------
    int a_off[2], b_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int rowa = wr * BR * 32 + m32, rowb = (GEGLU ? wo * 32 : wo * BO * 32) + m32;
        if (ABITS == 8)
            a_off[ks] = rowa * 64 + (((ks * 2 + kh) ^ swz64(rowa)) * 16);
        else
            a_off[ks] = rowa * 32 + ((ks ^ swz32(rowa)) * 16) + (kh ^ half32(rowa)) * 8;
        b_off[ks] = CF::ABYTES + rowb * 64 + (((ks * 2 + kh) ^ swz64(rowb)) * 16);
    }
    // 16 bytes of K per lane for each row-block / channel-block
    auto load_frags = [&](const uint8_t *base, int ks, v4i (&af)[BR], v4i (&bf)[BO]) {
#pragma unroll
        for (int a = 0; a < BR; ++a) {
            if (ABITS == 8) {
                af[a] = *reinterpret_cast<const v4i *>(base + a_off[ks] + a * 32 * 64);
            } else {
                // 16 unsigned nibbles; byte i of a dword holds positions i and i+4
                const v2i q = *reinterpret_cast<const v2i *>(base + a_off[ks] + a * 32 * 32);
                af[a].x = q.x & 0x0f0f0f0f;
                af[a].y = (int)(((uint32_t)q.x >> 4) & 0x0f0f0f0fu);
                af[a].z = q.y & 0x0f0f0f0f;
                af[a].w = (int)(((uint32_t)q.y >> 4) & 0x0f0f0f0fu);
            }
        }
#pragma unroll
        for (int b = 0; b < BO; ++b)
            bf[b] = *reinterpret_cast<const v4i *>(base + b_off[ks] + b * (GEGLU ? CF::TO / 2 : 32) * 64);
    };

    // Make the compiler wait for a fragment set HERE (before the next set's reads are
    // issued), so that each LDS wait only covers reads issued one MFMA batch earlier.
    auto touch_frags = [&](v4i (&af)[BR], v4i (&bf)[BO]) {
#pragma unroll
        for (int a = 0; a < BR; ++a) asm volatile("" : "+v"(af[a]));
#pragma unroll
        for (int b = 0; b < BO; ++b) asm volatile("" : "+v"(bf[b]));
    };

    v16i acc[BR][BO];
    float facc[BR][BO][16];
#pragma unroll
    for (int a = 0; a < BR; ++a)
#pragma unroll
        for (int b = 0; b < BO; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) facc[a][b][i] = 0.0f;
    // fresh: the group's first k-step starts from C = 0 (no register clearing)
    auto mfma_all = [&](const v4i (&af)[BR], const v4i (&bf)[BO], bool fresh) {
        if (fresh) {
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int a = 0; a < BR; ++a)
#pragma unroll
                for (int b = 0; b < BO; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[a], bf[b], zero, 0, 0, 0);
        } else {
#pragma unroll
            for (int a = 0; a < BR; ++a)
#pragma unroll
                for (int b = 0; b < BO; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[a], bf[b], acc[a][b], 0, 0, 0);
        }
    };

    // ---- group tables in LDS (behind the ring): last chunk of each group and the two
    // scale rows.  Reading them with LDS instructions keeps scalar memory loads out of
    // the main loop, so its LDS waits can be partial (LDS returns in order).
    int32_t *tab_end = reinterpret_cast<int32_t *>(lds + STAGES * CF::STAGE_BYTES);
    float *tab_s = reinterpret_cast<float *>(tab_end + NG);
    if (MULTI) {  // tab_s = [s[0..P) | zoff[0..P)], one group
        if (tid == 0) tab_end[0] = t_end;
        if (tid < P) {
            tab_s[tid] = t_s0;
            tab_s[P + tid] = t_s1;
        }
    } else if (tid < NG) {
        tab_end[tid] = t_end;
        tab_s[tid] = t_s0;
        tab_s[NG + tid] = t_s1;
    }
    for (int32_t i = tid + CF::THREADS; !MULTI && i < NG; i += CF::THREADS) {  // more groups than threads
        tab_end[i] = gchunk[i + 1];
        tab_s[i] = s_tab[i];
        tab_s[NG + i] = s_tab[NG + i];
    }

    // ---- pixel classes of the rows this lane holds: bit i of cls1[a] / past[a] says
    // whether the row in accumulator register i of row-block a is of class 1 / lies past
    // the end of the tensor.
    uint32_t cls1[BR], past[BR];
    bool any1 = false, all1 = true, any_past = false;
#pragma unroll
    for (int a = 0; a < BR; ++a) {
        const bool in = row_in[a];
        const bool c1 = in && row_c1[a] != 0;
        const uint64_t m1 = __ballot(c1 && kh == 0);   // bit m: row m of the block is class 1
        const uint64_t mp = __ballot(!in && kh == 0);  // bit m: row m is past the end
        any1 = any1 || m1 != 0;
        all1 = all1 && ((m1 | mp) & 0xffffffffull) == 0xffffffffull;
        any_past = any_past || mp != 0;
        cls1[a] = 0;
        past[a] = 0;
        if (m1 != 0 || mp != 0) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = 8 * (i >> 2) + 4 * kh + (i & 3);
                cls1[a] |= (uint32_t)((m1 >> m) & 1) << i;
                past[a] |= (uint32_t)((mp >> m) & 1) << i;
            }
        }
    }
    bool mixed = any1 && !all1;  // wave-uniform
    // MULTI: 4-bit class of the row behind accumulator register i in clsn[a][i / 8]; rows
    // past the end carry the last row's class (their results are never stored)
    uint32_t clsn[BR][2];
    int32_t c_first = 0;
    if constexpr (MULTI) {
        c_first = __builtin_amdgcn_readfirstlane((int32_t)row_c1[0]);
        bool same = true;
#pragma unroll
        for (int a = 0; a < BR; ++a) {
            same = same && __ballot((int32_t)row_c1[a] != c_first) == 0;
            clsn[a][0] = clsn[a][1] = 0;
            // rows 8 q + 4 kh + (0..3) sit in four neighbouring lanes: fetch their classes as
            // one packed value per lane (class of row m in bits 4 (m & 3) .. of lane m & ~3's
            // word), so that four cross-lane reads instead of sixteen build the fields
            uint32_t quad = (uint32_t)row_c1[a] & 15u;
            quad |= ((uint32_t)__shfl_down((int32_t)quad, 1, 64) & 15u) << 4;   // rows m, m+1
            quad |= ((uint32_t)__shfl_down((int32_t)quad, 2, 64) & 0xffu) << 8; // rows m .. m+3
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t four = (uint32_t)__shfl((int32_t)quad, 8 * q + 4 * kh, 64) & 0xffffu;
                clsn[a][q >> 1] |= four << (16 * (q & 1));
            }
            // opaque from here on: otherwise the sixteen unpacked values are kept (and
            // spilled) across the loop instead of these two registers
            asm volatile("" : "+v"(clsn[a][0]), "+v"(clsn[a][1]));
        }
        mixed = !same;
    }


    // ---- wait for chunk 0 and for everyone's table entries ---------------------------------
    asm volatile("" ::: "memory");
    if (NG > CF::THREADS)
        DGQ_WAIT_VMCNT(0);
    else
        wait_chunks_pending<STAGES - 2, CF::LOADS>(n_chunks - 1);
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): the table writes have landed
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    auto epilogue = [&](auto mixed_tag, const int32_t p) {
        constexpr bool MIXED = decltype(mixed_tag)::value;
        // ---- epilogue: y = sw[o] * sum + zb[class][o], in place -------------------------
        if constexpr (MULTI) {
            // zb[class][o] = zoff[class] * (sw[o] * wsum[o]) + bias[o]; one table read per
            // row register, used for both column blocks, four registers at a time
#pragma unroll
            for (int a = 0; a < BR; ++a)
#pragma unroll
                for (int i0 = 0; i0 < 16; i0 += 4) {
                    float zo[4];
#pragma unroll
                    for (int i = i0; i < i0 + 4; ++i) {
                        const int32_t c = MIXED ? (int32_t)((clsn[a][i >> 3] >> (4 * (i & 7))) & 15u) : p;
                        zo[i - i0] = tab_s[P + c];
                    }
#pragma unroll
                    for (int i = i0; i < i0 + 4; ++i)
#pragma unroll
                        for (int b = 0; b < BO; ++b)
                            facc[a][b][i] = fmaf(col_sw[b], facc[a][b][i], fmaf(zo[i - i0], col_zb0[b], col_zb1[b]));
                    asm volatile("" ::: "memory");  // keep the next four reads behind these
                }
        } else {
#pragma unroll
        for (int b = 0; b < BO; ++b) {
            const float swo = col_sw[b];
            const float zb0 = col_zb0[b], zb1 = col_zb1[b];
#pragma unroll
            for (int a = 0; a < BR; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float zz;
                    if (MIXED)
                        zz = ((cls1[a] >> i) & 1) ? zb1 : zb0;
                    else
                        zz = p ? zb1 : zb0;
                    facc[a][b][i] = fmaf(swo, facc[a][b][i], zz);
                }
        }
        }
        if constexpr (GEGLU != 0) {
            // block 0 holds the value, block 1 the gate of the same output channel:
            // out = value * gate * Phi(gate), written to y [rows, O / 2]
            const int32_t oh = O >> 1;
            const int32_t oc = (o0 >> 1) + wo * 32 + m32;  // < O / 2: the tiles divide it
#pragma unroll
            for (int a = 0; a < BR; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    facc[a][0][i] = facc[a][0][i] * gelu(facc[a][1][i]);
                }
            if constexpr (GEGLU == 2) {
                // Quantize for the next layer (Section 3.1's linear quantizer with the
                // chunk's static offset and step; same operations as the stand-alone
                // quantizer).  A lane holds one position (column) of 16 rows, the layout
                // wants four consecutive positions of one row in a dword: the four codes of
                // registers 4 g .. 4 g + 3 (rows 8 g + 4 kh + 0 .. 3) are packed into one
                // dword and the 4 x 4 bytes are transposed across the four lanes of a quad,
                // after which lane j of quad c holds row 8 g + 4 kh + j, positions 4 c .. 4 c + 3:
                // one dword store per four registers.  In its 16-row code block that row is
                // t = 8 (g % 2) + 4 kh + j with slot swizzle kh | 2 ((j / 2) ^ (g % 2)): one lane
                // offset per value of the compile-time bit.
                int8_t *cout = reinterpret_cast<int8_t *>(y);
                const int32_t posw = (o0 >> 1) + wo * 32;  // first position of this wave
                const int32_t nch2 = O >> 7, chunk = posw >> 6;
                const float2 zi = rq_zi[chunk];
                const uint32_t keep = rq_keep[posw + m32] ? 0xffffffffu : 0u;
                const uint32_t j = (uint32_t)m32 & 3u, c = (uint32_t)m32 >> 2;
                const uint32_t kq = (uint32_t)((posw & 63) >> 4) + (c >> 2);
                const uint32_t row_part = (4u * (uint32_t)kh + j) * 64u + 4u * (c & 3u);
                const uint32_t lane_off0 = row_part + ((kq ^ ((uint32_t)kh | ((j >> 1) << 1))) << 4);
                const uint32_t lane_off1 = row_part + ((kq ^ ((uint32_t)kh | (((j >> 1) ^ 1u) << 1))) << 4);
                const uint32_t sel = ((4u + j) << 8) | j;  // byte j of each of two sources
                // 4-bit codes for the next layer: blocks of 32 rows x 32 bytes, a dword holds
                // 8 positions (byte i: position i in the low, i + 4 in the high nibble).  After
                // the same transpose the even quad of a pair holds the low nibbles, the odd
                // quad (four lanes up) the high ones; the even quads store.  Row t = 8 g + 4 kh + j
                // of the block has slot swizzle g % 2.
                if (rq_bits == 4) {
                    const uint32_t eb = (uint32_t)((posw & 63) >> 3) + (c >> 1);  // 8-position block in the chunk
                    const uint32_t row4 = (4u * (uint32_t)kh + j) * 32u + 4u * (eb & 3u);
                    const uint32_t l4_0 = row4 + ((eb >> 2) << 4), l4_1 = row4 + (((eb >> 2) ^ 1u) << 4);
#pragma unroll
                    for (int a = 0; a < BR; ++a) {
                        const int64_t rb = (r0 + (wr * BR + a) * 32) >> 5;
                        int8_t *blk = cout + ((rb * nch2 + chunk) << 10);
#pragma unroll
                        for (int g4 = 0; g4 < 4; ++g4) {
                            uint32_t pk = 0;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const float t = __fsub_rn(facc[a][0][4 * g4 + k], zi.x);
                                const float u = __builtin_amdgcn_fmed3f(__fmul_rn(t, zi.y), 0.0f, 15.0f);
                                pk = __builtin_amdgcn_cvt_pk_u8_f32(u, k, pk);
                            }
                            pk &= keep;
                            const uint32_t q0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0x00, 0xf, 0xf, false);
                            const uint32_t q1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0x55, 0xf, 0xf, false);
                            const uint32_t q2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0xaa, 0xf, 0xf, false);
                            const uint32_t q3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0xff, 0xf, 0xf, false);
                            const uint32_t x01 = __builtin_amdgcn_perm(q1, q0, sel);
                            const uint32_t x23 = __builtin_amdgcn_perm(q3, q2, sel);
                            const uint32_t low = __builtin_amdgcn_perm(x23, x01, 0x05040100u);
                            const uint32_t high = (uint32_t)__shfl_down((int)low, 4, 64);
                            // rows 16..31 of the block (g4 >= 2): the 8-byte halves of a slot swapped
                            const uint32_t lo = (((g4 & 1) ? l4_1 : l4_0) ^ (g4 >= 2 ? 8u : 0u)) + 256u * g4;
                            if (!(c & 1u) && !((past[a] >> (4 * g4 + (int)j)) & 1))
                                *reinterpret_cast<uint32_t *>(blk + lo) = low | (high << 4);
                        }
                    }
                } else
#pragma unroll
                for (int a = 0; a < BR; ++a) {
                    const int64_t rb = (r0 + (wr * BR + a) * 32) >> 4;
#pragma unroll
                    for (int g4 = 0; g4 < 4; ++g4) {
                        uint32_t pk = 0;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float t = __fsub_rn(facc[a][0][4 * g4 + k], zi.x);
                            pk = __builtin_amdgcn_cvt_pk_u8_f32(__fmul_rn(t, zi.y), k, pk);
                        }
                        pk = (pk ^ 0x80808080u) & keep;  // stored code = q - 128; padding stores 0
                        const uint32_t q0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0x00, 0xf, 0xf, false);
                        const uint32_t q1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0x55, 0xf, 0xf, false);
                        const uint32_t q2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0xaa, 0xf, 0xf, false);
                        const uint32_t q3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)pk, 0xff, 0xf, 0xf, false);
                        const uint32_t x01 = __builtin_amdgcn_perm(q1, q0, sel);  // bytes: q0.j, q1.j
                        const uint32_t x23 = __builtin_amdgcn_perm(q3, q2, sel);  // bytes: q2.j, q3.j
                        const uint32_t word = __builtin_amdgcn_perm(x23, x01, 0x05040100u);
                        int8_t *blk = cout + (((rb + (g4 >> 1)) * nch2 + chunk) << 10) + (g4 & 1) * 512;
                        const uint32_t lo = (g4 & 1) ? lane_off1 : lane_off0;
                        if (!((past[a] >> (4 * g4 + (int)j)) & 1))
                            *reinterpret_cast<uint32_t *>(blk + lo) = word;
                    }
                }
                // the column-0 tiles also write the next layer's row classes
                if (o0 == 0 && wo == 0 && lane < 32 * BR) {
                    const int64_t r = r0 + wr * BR * 32 + lane;
                    if (r < rows) rq_cls[r] = 0;
                }
                return;
            }
            if (r0 + CF::TR <= rows) {
                const uint32_t lane_off = (uint32_t)(4 * kh * oh + m32) * 4u;
                const int64_t row_bytes = (int64_t)oh * 4;
                char *rp = reinterpret_cast<char *>(y + (r0 + wr * BR * 32) * oh + (o0 >> 1) + wo * 32);
#pragma unroll
                for (int a = 0; a < BR; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        asm volatile("global_store_dword %0, %1, %2 nt"
                                     :
                                     : "v"(lane_off), "v"(facc[a][0][i]), "s"(rp)
                                     : "memory");
                        rp += (i & 3) == 3 ? 5 * row_bytes : row_bytes;  // rows 0 1 2 3, 8 9 ...
                    }
            } else {
#pragma unroll
                for (int a = 0; a < BR; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int rl = (wr * BR + a) * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                        if (!((past[a] >> i) & 1)) y[(r0 + rl) * oh + oc] = facc[a][0][i];
                    }
            }
            return;
        }
        // Register i of a block holds row 8 (i / 4) + 4 kh + i % 4 at column m32: one
        // store instruction writes two 128-byte row pieces.  Interior tiles use a scalar
        // row pointer plus one per-lane 32-bit offset, so the 16 * BR * BO stores need no
        // vector address arithmetic; edge tiles predicate every element.
        const bool interior = r0 + CF::TR <= rows && o0 + CF::TO <= O;
        if (interior) {
            const uint32_t lane_off = (uint32_t)(4 * kh * O + m32) * 4u;
            // scalar row pointer + 32-bit lane offset + the column block as the instruction's
            // offset field, spelled out so that no vector instruction and one scalar add
            // per row is spent on addresses (rows go 0 1 2 3, 8 9 10 11, ...)
            const int64_t row_bytes = (int64_t)O * 4;
            char *rp = reinterpret_cast<char *>(y + (r0 + wr * BR * 32) * O + o0 + wo * BO * 32);
#pragma unroll
            for (int a = 0; a < BR; ++a)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    static_assert(BO <= 2, "column blocks are addressed by the offset field");
                    asm volatile("global_store_dword %0, %1, %2 nt"
                                 :
                                 : "v"(lane_off), "v"(facc[a][0][i]), "s"(rp)
                                 : "memory");
                    if (BO == 2)
                        asm volatile("global_store_dword %0, %1, %2 offset:128 nt"
                                     :
                                     : "v"(lane_off), "v"(facc[a][BO - 1][i]), "s"(rp)
                                     : "memory");
                    rp += (i & 3) == 3 ? 5 * row_bytes : row_bytes;  // after row 31: 8 * 3 + 3 + 5 = 32
                }
        } else {
#pragma unroll
            for (int b = 0; b < BO; ++b) {
                const int32_t o = o0 + (wo * BO + b) * 32 + m32;
#pragma unroll
                for (int a = 0; a < BR; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int rl = (wr * BR + a) * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                        if (o < O && !((past[a] >> i) & 1)) y[(r0 + rl) * O + o] = facc[a][b][i];
                    }
            }
        }
    };

    // The loop and the epilogue, instantiated for uniform-class and mixed-class waves.
    auto run = [&](auto mixed_tag) {
        constexpr bool MIXED = decltype(mixed_tag)::value;
        // the wave's class when it is uniform
        const int32_t p = MULTI ? (MIXED ? 0 : c_first) : ((!MIXED && any1) ? 1 : 0);
        v4i af0[BR], bf0[BO], af1[BR], bf1[BO];
        // The int32 blocks are not cleared (a group's first MFMA starts from C = 0): the empty
        // asm statement only tells the compiler that the registers hold a value.
#pragma unroll
        for (int a = 0; a < BR; ++a)
#pragma unroll
            for (int b = 0; b < BO; ++b) asm volatile("" : "=v"(acc[a][b]));
        load_frags(lds, 0, af0, bf0);
        const float *s_p = tab_s + p * NG;  // MULTI: NG == 1, so s_p[0] is class p's scale
        int32_t g = 0;
        int32_t g_end = __builtin_amdgcn_readfirstlane(tab_end[0]);
        bool fresh = true;

        // ---- main loop, software-pipelined over half chunks: while the matrix cores
        // work on one k-step the LDS reads of the next one are in flight.  The barrier
        // that publishes chunk ch+1 (and retires the stage chunk ch-1 used) sits between
        // the two k-steps of chunk ch.
        // One chunk.  STEADY: the ring is full and chunk ch + STAGES - 1 exists, so the wait
        // count is a constant, the next DMA unconditional, and `pos` (the ring stage of
        // chunk ch) a literal: the stage addresses then sit in the LDS instructions'
        // offset fields instead of costing vector adds (a vector instruction costs this
        // kernel about four clocks of SIMD time with nothing hidden behind it).
        // ---- fold the finished group's int32 block into the fp32 sum with its scale ---
        auto fold_group = [&]() __attribute__((always_inline)) {
            if (!MIXED) {
                const float sg = s_p[g];
#pragma unroll
                for (int a = 0; a < BR; ++a)
#pragma unroll
                    for (int b = 0; b < BO; ++b)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            facc[a][b][i] = fmaf((float)acc[a][b][i], sg, facc[a][b][i]);
            } else if (MULTI) {
#pragma unroll
                for (int a = 0; a < BR; ++a)
#pragma unroll
                    for (int i0 = 0; i0 < 16; i0 += 4) {
                        float sg[4];
#pragma unroll
                        for (int i = i0; i < i0 + 4; ++i)
                            sg[i - i0] = tab_s[(clsn[a][i >> 3] >> (4 * (i & 7))) & 15u];
#pragma unroll
                        for (int i = i0; i < i0 + 4; ++i)
#pragma unroll
                            for (int b = 0; b < BO; ++b)
                                facc[a][b][i] = fmaf((float)acc[a][b][i], sg[i - i0], facc[a][b][i]);
                        asm volatile("" ::: "memory");
                    }
            } else {
                const float s0 = tab_s[g], s1 = tab_s[NG + g];
#pragma unroll
                for (int a = 0; a < BR; ++a)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float sg = ((cls1[a] >> i) & 1) ? s1 : s0;
#pragma unroll
                        for (int b = 0; b < BO; ++b)
                            facc[a][b][i] = fmaf((float)acc[a][b][i], sg, facc[a][b][i]);
                    }
            }
        };
        auto chunk = [&](auto steady_tag, const int pos, const int32_t ch) __attribute__((always_inline)) {
            constexpr bool STEADY = decltype(steady_tag)::value;
            const int npos = pos + 1 == STAGES ? 0 : pos + 1;
            const uint8_t *base = lds + pos * CF::STAGE_BYTES;
            touch_frags(af0, bf0);
            load_frags(base, 1, af1, bf1);
            mfma_all(af0, bf0, fresh);
            fresh = false;
            touch_frags(af1, bf1);
            if (STEADY || ch + 1 < n_chunks) {
                asm volatile("" ::: "memory");
                if (DUMP)
                    DGQ_WAIT_VMCNT(0);
                else if (STEADY)
                    DGQ_WAIT_VMCNT((STAGES - 3) * CF::LOADS);
                else
                    wait_chunks_pending<STAGES - 3, CF::LOADS>(n_chunks - 2 - ch);
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (STEADY || ch + STAGES - 1 < n_chunks)
                    issue_chunk_at(ch + STAGES - 1, pos == 0 ? STAGES - 1 : pos - 1);
                load_frags(lds + npos * CF::STAGE_BYTES, 0, af0, bf0);
            }
            mfma_all(af1, bf1, false);

            // MULTI has one group: its only fold follows the loop, so the fp32 block does not
            // occupy registers inside it
            if (!MULTI && ch + 1 == g_end) {
                fold_group();
                if (DUMP) {
#pragma unroll
                    for (int a = 0; a < BR; ++a)
#pragma unroll
                        for (int b = 0; b < BO; ++b) {
                            const int32_t o = o0 + (wo * BO + b) * 32 + m32;
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                const int64_t r =
                                    r0 + (wr * BR + a) * 32 + 8 * (i >> 2) + 4 * kh + (i & 3);
                                if (r < rows && o < O) acc_dump[(r * O + o) * NG + g] = acc[a][b][i];
                            }
                        }
                }
                fresh = true;
                ++g;
                g_end = g < NG ? __builtin_amdgcn_readfirstlane(tab_end[g]) : 0x7fffffff;
            }
        };
        int32_t ch = 0;
        if (!DUMP && STAGES <= 4) {
            // STAGES chunks per trip, every one of them in the steady state
            while (ch + 2 * STAGES - 2 < n_chunks) {
#pragma unroll
                for (int u = 0; u < STAGES; ++u) chunk(std::true_type{}, u, ch + u);
                ch += STAGES;
            }
        }
        for (int pos = ch % STAGES; ch < n_chunks; ++ch) {
            chunk(std::false_type{}, pos, ch);
            pos = pos + 1 == STAGES ? 0 : pos + 1;
        }

        if constexpr (MULTI) fold_group();
        epilogue(mixed_tag, p);
    };

    if (mixed)
        run(std::true_type{});
    else
        run(std::false_type{});
}

template <class CF, bool DUMP, int GEGLU = 0, bool MULTI = false, bool CONV = false>
hipError_t launch_cfg(const Groups &g, const Weight &w, const int8_t *codes,
                      const uint8_t *row_class, int64_t rows, float *y, int32_t *acc_dump,
                      hipStream_t st, uint8_t *rq_cls = nullptr, const ConvGather *cvp = nullptr) {
    const int32_t tiles_r = (int32_t)((rows + CF::TR - 1) / CF::TR);
    const int32_t tiles_o = (w.O + CF::TO - 1) / CF::TO;  // O_pad is a multiple of every TO
    const int64_t T = (int64_t)tiles_r * tiles_o;
    const int32_t per_xcd = (int32_t)((T + 7) / 8);
    const dim3 grid((unsigned)(per_xcd * 8));
    size_t lds = (size_t)CF::STAGES * CF::STAGE_BYTES +
                 (MULTI ? 4 + 8 * (size_t)g.n_tab : 12 * (size_t)g.info.n_groups);
    static_assert(GEGLU == 0 || CF::BO == 2, "the gated epilogue pairs the two blocks of a wave");
    static_assert(!(GEGLU != 0 && MULTI), "the gated epilogue is built for at most two pixel classes");
    auto kern = k_linear<CF, DUMP, GEGLU, MULTI, CONV>;
    const ConvGather cv = cvp ? *cvp : ConvGather();
    {
        hipError_t e = DGQ_ENSURE_LDS(kern, kStageBudget);
        if (e != hipSuccess) return e;
    }
    if (lds > (size_t)kStageBudget) return hipErrorInvalidValue;  // too many groups for the table
    // Row tiles per super-column.  The workgroups resident on one XCD (32 CUs) share code
    // rows and weight rows in that XCD's 4 MB L2.  Narrow outputs: one band of row tiles
    // covers all column tiles.  Wide outputs (ff.in: the weights alone exceed L2): a band
    // 16 row tiles high, so the resident set is about 16 x 8 tiles and every weight tile
    // that streams through L2 is used by 16 row tiles instead of 2 (measured: the L2-miss
    // reads of the 16384 x 1280 -> 10240 layer were 1.8 GB against 36 MB of operands).
    constexpr int kWgPerCu = CF::OCC * 4 / CF::NW > 0 ? CF::OCC * 4 / CF::NW : 1;
    const int32_t resident = 32 * kWgPerCu;
    int32_t super_rows = (resident + tiles_o - 1) / tiles_o;
    super_rows = super_rows < 1 ? 1 : (super_rows > 8 ? 8 : super_rows);
    if (tiles_o >= 32) super_rows = 16;
#ifdef DGQ_TUNING
    if (const int v = tuning_value(kTuneSuperRows); v > 0) super_rows = v;
#endif
    hipLaunchKernelGGL(kern, grid, dim3(CF::THREADS), lds, st, codes, row_class, w.d_wq, w.d_sw,
                       w.d_zb, g.d_s, g.d_zoff, g.n_tab, g.d_gchunk, rows, w.O, w.O_pad, w.Kp,
                       g.info.n_groups,
                       tiles_r, tiles_o, per_xcd, super_rows, y, acc_dump, w.d_rq_zi, w.d_rq_keep, rq_cls,
                       w.next_bits, cv);
    return hipGetLastError();
}

}  // namespace


// The 3 x 3 convolution with its taps gathered by the loads (see ConvGather): `codes3` are the
// three shifted copies of the map's codes, g9 / w the replicated tables and the packed
// [O, 9 C] kernel.
hipError_t launch_linear_conv3x3(const Groups &g9, const Weight &w, const int8_t *codes3,
                                 const uint8_t *row_class, int32_t B, int32_t H, int32_t W, float *y,
                                 hipStream_t st) {
    const bool a8 = g9.info.act_bits == 8;
    const int32_t rpb = a8 ? 16 : 32;
    if (W % rpb != 0 || g9.conv_taps != 9 || !g9.d_fill_blocks) return hipErrorInvalidValue;
    const int64_t rows = (int64_t)B * H * W;
    ConvGather cv;
    cv.w_blocks = W / rpb;
    cv.height = H;
    cv.chunks = g9.base_kp / kGranule;
    cv.copy_bytes = ((rows + rpb - 1) / rpb) * (int64_t)cv.chunks * 1024;
    cv.fill = reinterpret_cast<const int8_t *>(g9.d_fill_blocks);
    const int64_t t128 = ((rows + 127) / 128) * ((w.O + 127) / 128);
    const int64_t t64x128 = ((rows + 63) / 64) * ((w.O + 127) / 128);
    const int cfg = t128 >= 512 ? 4 : (t64x128 >= 256 ? 2 : 6);
    if (cfg == 4)
        return a8 ? launch_cfg<Cfg<8, 4, 2, 1, 2, 4, 4>, false, 0, false, true>(g9, w, codes3, row_class, rows, y, nullptr, st, nullptr, &cv)
                  : launch_cfg<Cfg<4, 4, 2, 1, 2, 4, 4>, false, 0, false, true>(g9, w, codes3, row_class, rows, y, nullptr, st, nullptr, &cv);
    if (cfg == 2)
        return a8 ? launch_cfg<Cfg<8, 2, 2, 1, 2, 3, 4>, false, 0, false, true>(g9, w, codes3, row_class, rows, y, nullptr, st, nullptr, &cv)
                  : launch_cfg<Cfg<4, 2, 2, 1, 2, 3, 4>, false, 0, false, true>(g9, w, codes3, row_class, rows, y, nullptr, st, nullptr, &cv);
    return a8 ? launch_cfg<Cfg<8, 2, 2, 1, 1, 8, 4>, false, 0, false, true>(g9, w, codes3, row_class, rows, y, nullptr, st, nullptr, &cv)
              : launch_cfg<Cfg<4, 2, 2, 1, 1, 8, 4>, false, 0, false, true>(g9, w, codes3, row_class, rows, y, nullptr, st, nullptr, &cv);
}

hipError_t launch_linear(const Groups &g, const Weight &w, const int8_t *codes,
                         const uint8_t *row_class, int64_t rows, float *y, int32_t *acc_dump,
                         int geglu, uint8_t *rq_cls, hipStream_t st) {
    const bool a8 = g.info.act_bits == 8;
    const bool multi = g.n_tab > 2;  // more than two pixel classes (one channel group)
    if (multi && (geglu || acc_dump || g.info.n_groups != 1)) return hipErrorInvalidValue;
    if (geglu == 2 && (!w.d_rq_zi || !w.d_rq_keep || !rq_cls)) return hipErrorInvalidValue;
    // Four waves per SIMD in every shape: a wave's fold waits for its own MFMAs, so it is
    // the other waves that keep the matrix pipe busy meanwhile.  Large problems take
    // 128 x 128 tiles (fewer operand bytes per output), medium ones 64 x 128 tiles so that every CU still gets work, and
    // problems with fewer tiles than CUs (the projections of the 77-token prompt) 64 x 64
    // tiles of four 32 x 32 waves behind an 8-deep ring: there a workgroup is alone on its CU and only the
    // depth of the ring hides the latency of the chunks.
    const int64_t t128 = ((rows + 127) / 128) * ((w.O + 127) / 128);
    const int64_t t64x128 = ((rows + 63) / 64) * ((w.O + 127) / 128);
    int cfg = t128 >= 512 ? 4 : (t64x128 >= 256 ? 2 : 6);
    // Wide outputs (32 column tiles and more: the first feed-forward projections) run 2-4 % fewer
    // clocks on 64 x 128 tiles, four workgroups per CU, than on 128 x 128 (measured with the
    // launch's clock counter on 65536 x 640 -> 5120 and 16384 x 1280 -> 10240, both code widths);
    // every other large shape is 3-9 % slower there.
    if (cfg == 4 && !geglu && (w.O + 127) / 128 >= 32) cfg = 2;
#ifdef DGQ_TUNING  // tuning builds only: a forced tile shape
    if (const int v = tuning_value(kTuneLinearCfg); v > 0) cfg = v;
#endif
#define DGQ_CASE(ID, ...)                                                                          \
    case ID:                                                                                       \
        if (geglu == 2)                                                                            \
            return a8 ? launch_cfg<Cfg<8, __VA_ARGS__>, false, 2>(g, w, codes, row_class, rows, y, nullptr, st, rq_cls) \
                      : launch_cfg<Cfg<4, __VA_ARGS__>, false, 2>(g, w, codes, row_class, rows, y, nullptr, st, rq_cls); \
        if (geglu)                                                                                 \
            return a8 ? launch_cfg<Cfg<8, __VA_ARGS__>, false, 1>(g, w, codes, row_class, rows, y, nullptr, st) \
                      : launch_cfg<Cfg<4, __VA_ARGS__>, false, 1>(g, w, codes, row_class, rows, y, nullptr, st); \
        if (acc_dump) /* the same tile shape as the plain launch, every group accumulator stored */ \
            return a8 ? launch_cfg<Cfg<8, __VA_ARGS__>, true>(g, w, codes, row_class, rows, y, acc_dump, st) \
                      : launch_cfg<Cfg<4, __VA_ARGS__>, true>(g, w, codes, row_class, rows, y, acc_dump, st); \
        if (multi)                                                                                 \
            return a8 ? launch_cfg<Cfg<8, __VA_ARGS__>, false, false, true>(g, w, codes, row_class, rows, y, nullptr, st) \
                      : launch_cfg<Cfg<4, __VA_ARGS__>, false, false, true>(g, w, codes, row_class, rows, y, nullptr, st); \
        return a8 ? launch_cfg<Cfg<8, __VA_ARGS__>, false>(g, w, codes, row_class, rows, y, nullptr, st) \
                  : launch_cfg<Cfg<4, __VA_ARGS__>, false>(g, w, codes, row_class, rows, y, nullptr, st)
    switch (cfg) {
        DGQ_CASE(2, 2, 2, 1, 2, 3, 4);  // 64 x 128, 4 waves of 32 x 64, four workgroups per CU
        case 6:  // 64 x 64 behind an 8-stage ring: 4 waves of 32 x 32 (13-15 % faster on the
                 // 1232-row projections than 2 waves of 32 x 64); the gated epilogue needs
                 // two column blocks per wave and keeps the 2-wave shape
            if (geglu == 2)
                return a8 ? launch_cfg<Cfg<8, 2, 1, 1, 2, 8, 4>, false, 2>(g, w, codes, row_class, rows, y, nullptr, st, rq_cls)
                          : launch_cfg<Cfg<4, 2, 1, 1, 2, 8, 4>, false, 2>(g, w, codes, row_class, rows, y, nullptr, st, rq_cls);
            if (geglu)
                return a8 ? launch_cfg<Cfg<8, 2, 1, 1, 2, 8, 4>, false, 1>(g, w, codes, row_class, rows, y, nullptr, st)
                          : launch_cfg<Cfg<4, 2, 1, 1, 2, 8, 4>, false, 1>(g, w, codes, row_class, rows, y, nullptr, st);
            if (acc_dump)
                return a8 ? launch_cfg<Cfg<8, 2, 2, 1, 1, 8, 4>, true>(g, w, codes, row_class, rows, y, acc_dump, st)
                          : launch_cfg<Cfg<4, 2, 2, 1, 1, 8, 4>, true>(g, w, codes, row_class, rows, y, acc_dump, st);
            if (multi)
                return a8 ? launch_cfg<Cfg<8, 2, 2, 1, 1, 8, 4>, false, false, true>(g, w, codes, row_class, rows, y, nullptr, st)
                          : launch_cfg<Cfg<4, 2, 2, 1, 1, 8, 4>, false, false, true>(g, w, codes, row_class, rows, y, nullptr, st);
            return a8 ? launch_cfg<Cfg<8, 2, 2, 1, 1, 8, 4>, false>(g, w, codes, row_class, rows, y, nullptr, st)
                      : launch_cfg<Cfg<4, 2, 2, 1, 1, 8, 4>, false>(g, w, codes, row_class, rows, y, nullptr, st);
        default:
            DGQ_CASE(4, 4, 2, 1, 2, 4, 4);  // 128 x 128, 8 waves of 32 x 64, two workgroups per CU
    }
#undef DGQ_CASE
}

}  // namespace dgq
