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
//   -log2(A/s) = log2(s) + lse2_i - L_ij * log2(e),   lse2_i = log2(sum_j 2^(L_ij log2 e)),
// which needs no exponential per element and is exact to ~1e-6 in log2 units;
// a probability below 2^-150 rounds to zero in fp32 and takes the top code.
//
// Matrix-core path (head dim a multiple of 8 up to 96 with nk <= 126, up to 160 with nk <= 94)
// ----------------------------------------------------------------
// A workgroup owns one (prompt, head) pair and a range of queries; its eight
// wavefronts each take 32 queries at a time.  The logits are computed
// TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_f16: a lane then holds, for
// ONE query (lane % 32), half of that query's keys in its accumulator registers,
// so the soft-max maximum and sum are register reductions plus one exchange
// with lane ^ 32.  fp32 accuracy comes from splitting both operands into two
// fp16 pieces, x = hi + lo (round to nearest; lo may be subnormal, which these
// instructions honour), and adding three products hi*hi + hi*lo + lo*hi in the
// fp32 accumulator; the dropped lo*lo term is below 2^-24 relative.  Inputs
// must stay inside the fp16 range (|k| and |q| log2(e)/sqrt(d) below 65504).
// log2(e)/sqrt(d) is folded into Q before the
// split and key_bias*log2(e) is the accumulator's start value, with -inf for the
// padding keys so that they vanish from maximum and sum without a mask.
//
// Pass 1 writes lse2_i per (prompt, head, query) into the workspace and folds
// max_{j>=1} 2^(S_ij - lse2_i) into scale_out[b].  Pass 2 recomputes S^T the
// same way (bit-identical), turns each register into its code, and builds
// 2^-code directly as a bf16 bit pattern (an exact power of two).  The
// accumulator layout of S^T is, register for register, an operand layout of the
// next product (v_mfma_f32_32x32x16_bf16: a lane supplies eight keys of its
// query, as the A and the B operand alike) once the key order inside each 16-key
// step is permuted the same way on the V^T side, so the probabilities never
// leave the registers.  They go in as the A operand, Out = P V: a lane of the
// result then holds one output dimension of sixteen queries and a store writes
// 128 contiguous bytes per row (as the B operand, Out^T = V^T P^T, every store
// touched 32 rows 32 bytes at a time and the stores cost a third of the call).
// V is split into two bf16 pieces (2^-17 relative).  The <start> column is carried through the same product:
// a' = A_i0 / s_b, split into three bf16 pieces (24 bits), occupies key slot 0
// and the last two padding slots, whose V^T columns hold V_0.  The result is
// multiplied by s_b on the way out.
//
// Other shapes use the plain fp32 kernel at the bottom of the file: one thread
// per (query, head), logits in registers, K then V broadcast from LDS.
#include <cstdlib>
#include <type_traits>

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

// ======================================================================================
// Matrix-core path
// ======================================================================================

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// workgroup of the matrix-core kernels: eight wavefronts share one copy of K and V^T in LDS
constexpr int kXWaves = 8, kXThreads = 64 * kXWaves;

// NKB: 32-key blocks (keys padded to 32*NKB, the last two slots reserved).
// KS:  16-wide steps over the head dimension (d padded to 16*KS).
template <int NKB_, int KS_>
struct XCfg {
    static constexpr int NKB = NKB_, KS = KS_;
    static constexpr int NKP = 32 * NKB;        // padded keys
    static constexpr int DB = (KS + 1) / 2;     // 32-wide blocks of output dims
    static constexpr int DP = 32 * DB;
    static constexpr int KROW = 16 * KS + 8;    // halves per K row (+16 B against bank conflicts)
    static constexpr int VROW = NKP + 12;       // bf16 per V^T row: an odd multiple of 2 dwords, so the
                                                // 8-byte fragment reads of 32 rows hit 64 distinct banks
    static constexpr int NBIAS = 2 * NKB * 16;  // floats: start values per lane half
    // register budget: two workgroups per CU (128 registers) for head dims up to 64
    static constexpr int WAVES_PER_SIMD = KS <= 4 ? 4 : 2;
    static constexpr size_t lds_pass1 = (size_t)NKP * KROW * 2 * 2 + NBIAS * 4;
    static constexpr size_t lds_pass2 = lds_pass1 + (size_t)DP * VROW * 2 * 2;
};

__device__ inline uint32_t pack_h2(float a, float b) {
    v2h r = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(uint32_t, r);
}

// x = hi + lo, both fp16, round to nearest (lo may be subnormal: the matrix cores honour
// subnormal fp16 inputs).
struct HiLo {
    uint32_t hi, lo;
};
__device__ inline HiLo split_h2(float a, float b) {
    const v2h h = {(_Float16)a, (_Float16)b};
    HiLo r;
    r.hi = __builtin_bit_cast(uint32_t, h);
    // The residual must be taken from the very halves the matrix cores will see.  Without
    // this opaque copy the compiler converts twice, with the packed and with the scalar
    // instruction, and the two do not round alike next to a tie, which breaks hi + lo = x.
    asm("" : "+v"(r.hi));
    // a - float(hi.x), b - float(hi.y): the mixed-precision multiply-add reads the fp16 halves
    // directly (one instruction each instead of a conversion and a subtraction; the result is
    // the same exactly rounded difference)
    float la, lb;
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(la) : "v"(r.hi), "v"(a));
    asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(lb) : "v"(r.hi), "v"(b));
    r.lo = pack_h2(la, lb);
    return r;
}

__device__ inline uint32_t bf16_rne_bits(float x) {  // upper 16 bits hold the bf16
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u & 0xFFFF0000u;
}

// median of three = clamp(x, lo, hi) in one instruction (the compiler emits max + min)
__device__ inline int32_t clamp_i32(int32_t x, int32_t lo, int32_t hi) {
    int32_t r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "v"(lo), "v"(hi));
    return r;
}

// key held by accumulator register i of key block blk in lane half hh
__device__ __host__ constexpr int key_of(int blk, int i, int hh) {
    return 32 * blk + 8 * (i >> 2) + 4 * hh + (i & 3);
}

template <class CF, int PASS, bool DUMP>
__global__ __launch_bounds__(kXThreads, (PASS >= 2 && CF::WAVES_PER_SIMD > 2) ? 2 : CF::WAVES_PER_SIMD) void k_xattn_mfma(
    const float *__restrict__ q, const float *__restrict__ k, const float *__restrict__ v,
    const float *__restrict__ key_bias, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
    float qk_scale, int32_t trips_per_wg, int32_t n_pairs, float *__restrict__ out, float *__restrict__ scale,
    float *__restrict__ lse2, uint8_t *__restrict__ codes_dump,
    const float *__restrict__ scale_in, float *__restrict__ part_max, int32_t tpw1) {
    // part_max (passes 1 and 2; may be null): instead of folding its maximum into scale[b] with
    // an atomic, which needs scale[] cleared by a launch of its own before pass 1 (5 us of a
    // 110 us call), a pass-1 workgroup stores the maximum of every piece it walks, of pair p in
    // its range w, at part_max[p + w] (p + w grows along the sequence of pieces, so every piece
    // has a slot of its own, n_pairs + ranges slots in all, each written once per call); pass 2
    // takes the maximum over the slots of its prompt's pairs (tpw1 = pass 1's trips per range
    // tells which exist) and the workgroup that holds the prompt's first trip writes scale[b].
    // PASS 3: both passes in one, for a prompt scale that is GIVEN (scale_in): the soft-max
    // statistics of a query block are taken and used at once, Q is read a single time, and
    // `scale` (if not null) still collects this call's own maximum.
    constexpr int NKB = CF::NKB, KS = CF::KS, NKP = CF::NKP, DB = CF::DB, DP = CF::DP;
    constexpr int KROW = CF::KROW, VROW = CF::VROW;
    extern __shared__ __align__(16) unsigned char smem[];
    _Float16 *Kh = reinterpret_cast<_Float16 *>(smem);
    _Float16 *Kl = Kh + NKP * KROW;
    float *biasv = reinterpret_cast<float *>(Kl + NKP * KROW);
    uint16_t *Vh = reinterpret_cast<uint16_t *>(biasv + CF::NBIAS);
    uint16_t *Vl = Vh + DP * VROW;
    __shared__ float red[kXWaves];

    // the wave index is uniform: say so, and the query block, its row pointers and the
    // loop bounds derived from it live in scalar registers
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int n = lane & 31, hh = lane >> 5;
    const int64_t hs = (int64_t)H * d;  // stride between tokens

    // Work is counted in trips: one trip = the workgroup's eight waves taking 32 queries each of
    // one (prompt, head) pair.  The trips of all pairs, in order, are cut into equal ranges,
    // one per workgroup, so that every workgroup slot of the chip carries the same load (cut
    // per pair, the pieces of 4096 queries come out as 6 + 6 + 4 trips and the kernel waits for
    // the long ones with a third of its slots idle).  A range that crosses into the next pair
    // stages that pair's K and V^T again.
    const int32_t trips_per_pair = (N + 32 * kXWaves - 1) / (32 * kXWaves);
    const int32_t total_trips = n_pairs * trips_per_pair;
    // Pass 2 walks its range from the end: the queries pass 1 read last are the ones most likely
    // still held by the memory-side cache (256 MB; Q of 16 prompts is 168 MB, and the product
    // written next to it pushes the oldest lines out first).
    constexpr bool REV = PASS == 2;
    int32_t trip_lo = (int32_t)blockIdx.x * trips_per_wg;
    int32_t trip_hi = min(trip_lo + trips_per_wg, total_trips);
    for (bool first_pair = true; trip_lo < trip_hi; first_pair = false) {
    const int32_t pair = (REV ? trip_hi - 1 : trip_lo) / trips_per_pair;
    const int32_t seg = REV ? max(trip_lo, pair * trips_per_pair) : trip_lo;
    const int32_t trip0 = seg - pair * trips_per_pair;
    const int32_t n_trips = REV ? trip_hi - seg : min(trip_hi - trip_lo, trips_per_pair - trip0);
    if (REV) trip_hi = seg; else trip_lo += n_trips;
    const int32_t b = pair / H, head = pair - b * H;
    if (!first_pair) __syncthreads();  // every wave is done with the previous pair's K and V^T

    float s_b = 0.0f, s_eff = 1.0f, l2s = 0.0f;
    uint32_t pmask = 0xFFFFFFFFu;
    if (PASS == 2 && part_max != nullptr) {
        // every wave takes the maximum over the slots of prompt b by itself
        const int32_t per = (trips_per_pair + tpw1 - 1) / tpw1 + 1;  // pieces of a pair, at most
        float m = 0.0f;  // the slots hold probabilities (>= 0)
        for (int32_t idx = lane; idx < H * per; idx += kWave) {
            const int32_t p = b * H + idx / per, j = idx % per;
            const int32_t w = (p * trips_per_pair) / tpw1 + j;
            if (w <= ((p + 1) * trips_per_pair - 1) / tpw1) m = fmaxf(m, part_max[p + w]);
        }
        s_b = wave_max(m);
        if (tid == 0 && head == 0 && trip0 == 0) scale[b] = s_b;
    } else if (PASS >= 2) {
        s_b = PASS == 3 ? scale_in[b] : scale[b];
    }
    if (PASS >= 2) {
        // no probability above zero outside the <start> column: only that column contributes
        s_eff = s_b > 0.0f ? s_b : 1.0f;
        pmask = s_b > 0.0f ? 0xFFFFFFFFu : 0u;
        l2s = __log2f(s_eff);
    }

    const int32_t q_begin = trip0 * (32 * kXWaves);
    const int32_t q_end = min(q_begin + n_trips * (32 * kXWaves), N);
    const float *qbase = q + ((int64_t)b * N * H + head) * d;

    // raw fp32 query slices of this lane: dims 16 s + 8 hh .. + 7 of query qi
    struct QRaw {
        float4 x[KS][2];
        float lse;
    };
    // Only the last 16-dimension step can reach past the head dimension (d > 16 (KS - 1),
    // d % 8 == 0): its slice is clamped (K is zero in LDS there, any finite value will
    // do); the others sit at fixed distances from one per-lane pointer.
    const int32_t t_last = min(16 * (KS - 1) + 8 * hh, d - 8) - 8 * hh;
    // Addresses are a uniform block pointer (scalar registers) plus a 32-bit lane offset:
    // 64-bit pointers per lane cost two registers each, and this loop has none to spare.
    const float *lse_base = lse2 + ((int64_t)b * H + head) * N;
    auto load_q = [&](int32_t q0) {
        QRaw r;
        const int32_t q0c = min(q0, N - 1);                      // uniform
        const int32_t rl = min(n, N - 1 - q0c);                   // a row past the end re-reads the last one
        const char *blk = reinterpret_cast<const char *>(qbase + (int64_t)q0c * hs);
        const uint32_t lo = (uint32_t)(rl * (int32_t)hs + 8 * hh) * 4u;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint32_t os = s < KS - 1 ? lo + 64u * s : lo + 4u * (uint32_t)t_last;
            r.x[s][0] = *reinterpret_cast<const float4 *>(blk + os);
            r.x[s][1] = *reinterpret_cast<const float4 *>(blk + os + 16);
        }
        r.lse = 0.0f;
        if (PASS == 2)
            r.lse = *reinterpret_cast<const float *>(reinterpret_cast<const char *>(lse_base + q0c) + 4u * (uint32_t)rl);
        return r;
    };

    float run_l2 = -INFINITY;  // pass 1: running max of log2 A over this lane's queries
    // Registers 4 g .. 4 g + 3 of the last key block hold keys 32 (NKB - 1) + 8 g .. + 7 (both lane
    // halves): with 77 keys in three blocks the upper two groups are padding only (logit -inf,
    // weight 0), and the statistics and the code generation skip them.
    const int32_t live4 = min(4, (nk - 32 * (NKB - 1) + 7) >> 3);  // uniform
    auto live = [&](int blk, int i) { return blk < NKB - 1 || (i >> 2) < live4; };

    const int32_t q_first = q_begin + 32 * wave;
    const int32_t n_it = q_first < q_end ? (q_end - q_first + 32 * kXWaves - 1) / (32 * kXWaves) : 0;
    auto q_of = [&](int32_t it) { return q_first + (REV ? n_it - 1 - it : it) * (32 * kXWaves); };
    // the wave's first query block travels while K and V^T are staged
    QRaw cur = load_q(n_it > 0 ? q_of(0) : q_first);

    // ---- stage K (two fp16 pieces), the start values and, in pass 2, V^T ---------------
    {
        const float *kb = k + ((int64_t)b * nk * H + head) * d;
        for (int idx = tid; idx < NKP * KS * 4; idx += kXThreads) {
            const int j = idx / (KS * 4), t4 = (idx - j * (KS * 4)) * 4;
            float4 x = {0.0f, 0.0f, 0.0f, 0.0f};
            if (j < nk && t4 < d) x = *reinterpret_cast<const float4 *>(kb + (int64_t)j * hs + t4);
            // log2(e) / sqrt(d) is folded into K here, once per workgroup, not into every query
            const HiLo p0 = split_h2(x.x * qk_scale, x.y * qk_scale);
            const HiLo p1 = split_h2(x.z * qk_scale, x.w * qk_scale);
            const u32x2 hi = {p0.hi, p1.hi}, lo = {p0.lo, p1.lo};
            *reinterpret_cast<u32x2 *>(Kh + j * KROW + t4) = hi;
            *reinterpret_cast<u32x2 *>(Kl + j * KROW + t4) = lo;
        }
        for (int idx = tid; idx < CF::NBIAS; idx += kXThreads) {
            const int half = idx / (NKB * 16), r = idx - half * (NKB * 16);
            const int key = key_of(r >> 4, r & 15, half);
            biasv[idx] = key < nk ? (key_bias ? key_bias[key] * kLog2e : 0.0f) : -INFINITY;
        }
        if (PASS >= 2) {
            const float *vb = v + ((int64_t)b * nk * H + head) * d;
            for (int idx = tid; idx < NKP * (DP / 4); idx += kXThreads) {
                const int j = idx / (DP / 4), t4 = (idx - j * (DP / 4)) * 4;
                // the last two key slots repeat V_0 for the low pieces of the <start> weight
                const int js = j >= NKP - 2 ? 0 : j;
                float4 x = {0.0f, 0.0f, 0.0f, 0.0f};
                if (js < nk && t4 < d)
                    x = *reinterpret_cast<const float4 *>(vb + (int64_t)js * hs + t4);
                // V carries the prompt scale, so the product needs no multiply on the way out
                const float xe[4] = {x.x * s_eff, x.y * s_eff, x.z * s_eff, x.w * s_eff};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const uint32_t hb = bf16_rne_bits(xe[e]);
                    const uint32_t lb = bf16_rne_bits(xe[e] - __uint_as_float(hb));
                    Vh[(t4 + e) * VROW + j] = (uint16_t)(hb >> 16);
                    Vl[(t4 + e) * VROW + j] = (uint16_t)(lb >> 16);
                }
            }
        }
    }
    __syncthreads();

    for (int32_t it = 0; it < n_it; ++it) {
        const int32_t q0 = q_of(it);
        const int32_t qi = q0 + n;
        const bool valid = qi < N;
        // The K and V^T fragments of a lane do not depend on the query block; an opaque
        // zero keeps their LDS reads inside the loop (hoisted, they would not fit in
        // the register file next to the accumulators).
        int lds_ofs = 0;
        asm volatile("" : "+v"(lds_ofs));
        // ---- split the query into fp16 pieces ----------------------------------------------
        u32x4 qh[KS], ql[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const float4 a = cur.x[s][0], c = cur.x[s][1];
            const HiLo p0 = split_h2(a.x, a.y);
            const HiLo p1 = split_h2(a.z, a.w);
            const HiLo p2 = split_h2(c.x, c.y);
            const HiLo p3 = split_h2(c.z, c.w);
            qh[s] = u32x4{p0.hi, p1.hi, p2.hi, p3.hi};
            ql[s] = u32x4{p0.lo, p1.lo, p2.lo, p3.lo};
        }
        float lse_i = cur.lse;

        // ---- S^T = K Q^T in log2 units --------------------------------------------------------
        v16f sm[NKB];
#pragma unroll
        for (int blk = 0; blk < NKB; ++blk) {
            const float4 *bp = reinterpret_cast<const float4 *>(biasv + hh * (NKB * 16) + blk * 16);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const float4 t = bp[a];
                sm[blk][4 * a + 0] = t.x;
                sm[blk][4 * a + 1] = t.y;
                sm[blk][4 * a + 2] = t.z;
                sm[blk][4 * a + 3] = t.w;
            }
        }
        {
            // K fragments are read one (step, key block) ahead of the MFMAs that use them:
            // left alone the compiler reads each fragment right in front of its MFMAs, and
            // a wave then spends an LDS round trip per fragment doing nothing.
            auto k_frag = [&](int t, u32x4 &fh, u32x4 &fl) {
                const int off = (32 * (t % NKB) + n) * KROW + 16 * (t / NKB) + 8 * hh + lds_ofs;
                fh = *reinterpret_cast<const u32x4 *>(Kh + off);
                fl = *reinterpret_cast<const u32x4 *>(Kl + off);
            };
            u32x4 fh[2], fl[2];
            k_frag(0, fh[0], fl[0]);
#pragma unroll
            for (int t = 0; t < KS * NKB; ++t) {
                const int s = t / NKB, blk = t % NKB;
                if (t + 1 < KS * NKB) k_frag(t + 1, fh[(t + 1) & 1], fl[(t + 1) & 1]);
                asm volatile("" : "+v"(fh[t & 1]), "+v"(fl[t & 1]));  // wait for this pair only
                const v8h bqh = __builtin_bit_cast(v8h, qh[s]);
                const v8h bql = __builtin_bit_cast(v8h, ql[s]);
                const v8h akh = __builtin_bit_cast(v8h, fh[t & 1]);
                const v8h akl = __builtin_bit_cast(v8h, fl[t & 1]);
                sm[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(akh, bqh, sm[blk], 0, 0, 0);
                sm[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(akh, bql, sm[blk], 0, 0, 0);
                sm[blk] = __builtin_amdgcn_mfma_f32_32x32x16_f16(akl, bqh, sm[blk], 0, 0, 0);
            }
        }
        // Prefetch the wave's next block (past its last block re-read this one, a cache hit,
        // rather than rows that belong to another workgroup).  Issued here, not before the
        // product above: the split query is dead now and the raw one takes its registers;
        // issued earlier the two overlap, registers spill, and every reload of a spilled
        // value waits for ALL outstanding vector memory, i.e. for this very prefetch.
        // (Passes 2 and 3 are built for two waves per SIMD: at four, 128 registers do not
        // hold the 48 logits, the packed codes and the prefetched query together, and the
        // reloads' waits, which cover all outstanding vector memory, undo the prefetch:
        // 105 us against 77 us for pass 2 on 16 x 10 x 4096 x 64.)
        {
            int32_t qn = it + 1 < n_it ? q_of(it + 1) : q0;
            asm volatile("" : "+v"(qn) : "v"(sm[NKB - 1][15]));  // not before the last MFMA
            cur = load_q(qn);
        }

        if (PASS == 1 || PASS == 3) {
            if (PASS == 3) __builtin_amdgcn_sched_barrier(0);
            // ---- soft-max statistics of the lane's query ---------------------------------------
            float rest = -INFINITY;  // every key of this lane except register (0, 0)
#pragma unroll
            for (int blk = 0; blk < NKB; ++blk)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if ((blk || i) && live(blk, i)) rest = fmaxf(rest, sm[blk][i]);
            const float s00 = sm[0][0];  // key 0 in the lower lane half, key 4 in the upper
            float m = fmaxf(rest, s00);
            float m1 = fmaxf(rest, hh == 0 ? -INFINITY : s00);
            m = fmaxf(m, __shfl_xor(m, 32, kWave));
            m1 = fmaxf(m1, __shfl_xor(m1, 32, kWave));
            float sum = 0.0f;
#pragma unroll
            for (int blk = 0; blk < NKB; ++blk)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (live(blk, i)) sum += __builtin_amdgcn_exp2f(sm[blk][i] - m);
            sum += __shfl_xor(sum, 32, kWave);
            const float lse = m + __log2f(sum);
            if (valid) {
                run_l2 = fmaxf(run_l2, m1 - lse);
                if (PASS == 1 && hh == 0) lse2[((int64_t)b * H + head) * N + qi] = lse;
            }
            if (PASS == 1) continue;
            lse_i = lse;
            // keep the statistics and the code generation apart: interleaved, both hold
            // their temporaries next to the 48 logits and the register file overflows
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- pass 2: codes -> bf16 powers of two, packed as the next B operand --------------
        // code = clamp(rne(t)), t = c0 - S.  Adding 1.5 * 2^23 to -t leaves -rne(t) in the low
        // mantissa bits (round-to-nearest-even is symmetric), so rounding and clamping (an
        // integer median m = magic - code) are integer work, and the bf16 exponents 127 - code
        // of a pair of keys are two shift-and-adds of m onto one constant:
        // (m0 << 7) + (m1 << 23) - ((magic - 127) << 7) - ((magic - 127) << 23) mod 2^32.  A probability that rounds to zero in fp32
        // (t above l2s + 150) takes the top code; with 4-bit codes the clamp already does
        // that unless the prompt scale is below 2^-135, so the common 4-bit path skips it.
        const float c0 = l2s + lse_i;
        const float thr = l2s + 150.0f;
        constexpr int32_t kMagic = 0x4B400000;  // bit pattern of 12582912.0f
        constexpr uint32_t kPairBase = 0u - (((uint32_t)(kMagic - 127) << 7) + ((uint32_t)(kMagic - 127) << 23));
        const int32_t cq = (1 << bits) - 1;
        const int32_t ce = cq < 127 ? cq : 127;  // 2^-127 and below leave the product as zero
        uint8_t *cd = nullptr;
        if (DUMP) cd = codes_dump + ((((int64_t)b * H + head) * N + qi) * (int64_t)(nk - 1));
        uint32_t pk[NKB][8];
        auto make_codes = [&](auto rule_tag) {
            constexpr bool RULE = decltype(rule_tag)::value;
#pragma unroll
            for (int blk = 0; blk < NKB; ++blk)
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    if (!live(blk, i)) {  // padding keys only: V^T is zero there, any weight will do
                        pk[blk][i >> 1] = 0;
                        continue;
                    }
                    uint32_t m[2];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        float t = sm[blk][i + u] - c0;  // minus the code before rounding
                        if (RULE) t = t < -thr ? -300.0f : t;
                        const int32_t r = __float_as_int(t + 12582912.0f);
                        if (DUMP) {
                            const int key = key_of(blk, i + u, hh);
                            const int32_t c = kMagic - clamp_i32(r, kMagic - cq, kMagic);
                            if (valid && key >= 1 && key < nk) cd[key - 1] = (uint8_t)c;
                        }
                        m[u] = (uint32_t)clamp_i32(r, kMagic - ce, kMagic);
                    }
                    pk[blk][i >> 1] = ((m[0] << 7) + ((m[1] << 23) + kPairBase)) & pmask;
                }
        };
        if (thr < (float)cq)
            make_codes(std::true_type{});
        else
            make_codes(std::false_type{});
        {
            // <start> weight a' = A_i0 / s in three bf16 pieces (truncation keeps each exact)
            const float s_start = __shfl(sm[0][0], n, kWave);
            const float ap = __builtin_amdgcn_exp2f(s_start - c0);
            const uint32_t a1 = __float_as_uint(ap) & 0xFFFF0000u;
            const float r1 = ap - __uint_as_float(a1);
            const uint32_t a2 = __float_as_uint(r1) & 0xFFFF0000u;
            const float r2 = r1 - __uint_as_float(a2);
            const uint32_t a3 = __float_as_uint(r2) & 0xFFFF0000u;
            if (hh == 0) pk[0][0] = (pk[0][0] & 0xFFFF0000u) | (a1 >> 16);
            if (hh == 1) pk[NKB - 1][7] = (a2 >> 16) | a3;  // key slots NKP-2 and NKP-1
        }

        // ---- Out = P V, one block of 32 output dimensions after the other (both at once would
        // hold 32 more accumulator registers than the file has left).  The probabilities are
        // the A operand (a lane's registers are its query's row of P) and V^T's rows the B
        // operand, so that a lane of the result holds ONE output dimension of sixteen queries:
        // a store instruction then writes 128 contiguous bytes of each of two rows.  (With
        // the operands the other way round a lane held four dimensions of one query, every
        // store touched 32 rows 32 bytes at a time, and the stores cost a third of the call.)
        float *oblk = out + ((int64_t)b * N * H + head) * d + (int64_t)q0 * hs;  // uniform
        const uint32_t o_lane = (uint32_t)(4 * hh * hs + n) * 4u;  // row 4 hh, dimension n
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            v16f o;
#pragma unroll
            for (int i = 0; i < 16; ++i) o[i] = 0.0f;
            // V^T fragments, too, are read one 16-key step ahead
            auto v_frag = [&](int s16, u32x4 &ah, u32x4 &al) {
                // slots 0..3: keys 16 s16 + 4 hh + (0..3); slots 4..7: the same + 8
                const int off = (32 * db + n) * VROW + 16 * s16 + 4 * hh + lds_ofs;
                const u32x2 h0 = *reinterpret_cast<const u32x2 *>(Vh + off);
                const u32x2 h1 = *reinterpret_cast<const u32x2 *>(Vh + off + 8);
                const u32x2 l0 = *reinterpret_cast<const u32x2 *>(Vl + off);
                const u32x2 l1 = *reinterpret_cast<const u32x2 *>(Vl + off + 8);
                ah = u32x4{h0.x, h0.y, h1.x, h1.y};
                al = u32x4{l0.x, l0.y, l1.x, l1.y};
            };
            u32x4 vh[2], vl[2];
            v_frag(0, vh[0], vl[0]);
#pragma unroll
            for (int s16 = 0; s16 < 2 * NKB; ++s16) {
                if (s16 + 1 < 2 * NKB) v_frag(s16 + 1, vh[(s16 + 1) & 1], vl[(s16 + 1) & 1]);
                asm volatile("" : "+v"(vh[s16 & 1]), "+v"(vl[s16 & 1]));  // wait for this pair only
                u32x4 pb;
                pb.x = pk[s16 >> 1][4 * (s16 & 1) + 0];
                pb.y = pk[s16 >> 1][4 * (s16 & 1) + 1];
                pb.z = pk[s16 >> 1][4 * (s16 & 1) + 2];
                pb.w = pk[s16 >> 1][4 * (s16 & 1) + 3];
                const v8bf bp = __builtin_bit_cast(v8bf, pb);
                o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bp, __builtin_bit_cast(v8bf, vh[s16 & 1]), o, 0, 0, 0);
                o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bp, __builtin_bit_cast(v8bf, vl[s16 & 1]), o, 0, 0, 0);
            }
            // register i: query q0 + 8 (i / 4) + 4 hh + i % 4, dimension 32 db + n
            if (q0 + 32 <= N && 32 * db + 32 <= d) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    char *rowp = reinterpret_cast<char *>(oblk + (int64_t)(8 * (i >> 2) + (i & 3)) * hs + 32 * db);
                    // streaming stores: the product is not read again by this call, and written
                    // through the caches it pushes out the queries pass 2 has yet to read
                    // (measured: pass 2 of 16 prompts 77 -> 69 us; the same hint on the
                    // query LOADS costs 60 %)
                    __builtin_nontemporal_store(o[i], reinterpret_cast<float *>(rowp + o_lane));
                }
            } else {
                // the last query block of a (prompt, head) pair or a head dimension that ends inside
                // this block: every element predicated.  The opaque copy keeps the sixteen
                // addresses from being computed (and spilled) ahead of the loop.
                int32_t rows_left = N - q0;
                int64_t hs_here = hs;
                asm volatile("" : "+s"(rows_left), "+s"(hs_here));
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int32_t rl = 8 * (i >> 2) + 4 * hh + (i & 3);
                    if (rl < rows_left && 32 * db + n < d) oblk[(int64_t)rl * hs_here + 32 * db + n] = o[i];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    if (PASS == 1 || (PASS == 3 && scale != nullptr)) {
        float amax = wave_max(run_l2);
        if (lane == 0) red[wave] = amax;
        __syncthreads();
        if (tid == 0) {
            amax = red[0];
#pragma unroll
            for (int w = 1; w < kXWaves; ++w) amax = fmaxf(amax, red[w]);
            // probabilities are non-negative: their bit patterns order like unsigned ints
            if (PASS == 1 && part_max != nullptr)
                part_max[pair + (int32_t)blockIdx.x] = __builtin_amdgcn_exp2f(amax);
            else
                atomicMax(reinterpret_cast<unsigned int *>(scale + b),
                          __float_as_uint(__builtin_amdgcn_exp2f(amax)));
        }
    }
    }  // pairs of this workgroup's range
}

// Workgroup slots of the chip for the kernels that write the product (one workgroup per CU).
constexpr int kTargetWgs2 = 256;

// bytes of the per-row statistics at the start of the attention's workspace
inline size_t xattn_lse_bytes(int32_t B, int32_t N, int32_t H) {
    return ((size_t)B * H * N * sizeof(float) + 255) / 256 * 256;
}

template <class CF>
hipError_t launch_mfma(const float *q, const float *k, const float *v, const float *key_bias,
                       int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
                       float *out, float *scale_out, uint8_t *codes_dump, float *lse2,
                       size_t ws_bytes, const float *scale_in, hipStream_t st) {
    auto k1 = k_xattn_mfma<CF, 1, false>;
    auto k2 = codes_dump ? k_xattn_mfma<CF, 2, true> : k_xattn_mfma<CF, 2, false>;
    hipError_t e = DGQ_ENSURE_LDS((k_xattn_mfma<CF, 1, false>), (int)CF::lds_pass1);
    if (e != hipSuccess) return e;
    e = codes_dump ? DGQ_ENSURE_LDS((k_xattn_mfma<CF, 2, true>), (int)CF::lds_pass2)
                   : DGQ_ENSURE_LDS((k_xattn_mfma<CF, 2, false>), (int)CF::lds_pass2);
    if (e != hipSuccess) return e;
    // Trips (8 x 32 queries of one pair) per workgroup: all trips of the call, in order, in as
    // many equal ranges as the chip has workgroup slots for the kernel.
    constexpr int kPerTrip = 32 * kXWaves;
    const int32_t n_pairs = B * H;
    const int64_t total_trips = (int64_t)n_pairs * ((N + kPerTrip - 1) / kPerTrip);
    // (pass 1 could hold two workgroups per CU when the head dimension is at most 64; one per CU,
    // twice as long, measured faster: 114 against 127 us for the call on 16 x 10 x 4096 x 64)
    int target_wgs = 256, target_wgs2 = kTargetWgs2;
#ifdef DGQ_TUNING  // tuning builds only: the slot counts (pass 1: 1000 x value)
    if (const int v = tuning_value(kTuneXattnWgs); v > 0) {
        if (v % 1000) target_wgs2 = v % 1000 * 8;
        if (v / 1000) target_wgs = v / 1000 * 8;
    }
#endif
    const int32_t tpw = (int32_t)((total_trips + target_wgs - 1) / target_wgs);
    const int32_t tpw2 = (int32_t)((total_trips + target_wgs2 - 1) / target_wgs2);
    const dim3 grid((unsigned)((total_trips + tpw - 1) / tpw)), grid2((unsigned)((total_trips + tpw2 - 1) / tpw2));
    const float qk_scale = (float)(1.4426950408889634 / sqrt((double)d));
    if (scale_in) {  // given scale: one kernel, Q read once
        auto k3 = codes_dump ? k_xattn_mfma<CF, 3, true> : k_xattn_mfma<CF, 3, false>;
        e = codes_dump ? DGQ_ENSURE_LDS((k_xattn_mfma<CF, 3, true>), (int)CF::lds_pass2)
                       : DGQ_ENSURE_LDS((k_xattn_mfma<CF, 3, false>), (int)CF::lds_pass2);
        if (e != hipSuccess) return e;
        if (scale_out)
            hipLaunchKernelGGL(k_fill_zero, dim3((B + 63) / 64), dim3(64), 0, st, scale_out, B);
        hipLaunchKernelGGL(k3, grid2, dim3(kXThreads), CF::lds_pass2, st, q, k, v, key_bias, N, H, d,
                           nk, bits, qk_scale, tpw2, n_pairs, out, scale_out, nullptr, codes_dump, scale_in,
                           nullptr, 0);
        return hipGetLastError();
    }
    // the per-piece maxima behind the row statistics, if the workspace has room for them
    // (a workspace of xattn_workspace_bytes() has); otherwise atomics on a cleared scale[]
    const size_t lse_bytes = xattn_lse_bytes(B, N, H);
    float *part_max = nullptr;
    if (ws_bytes >= lse_bytes + sizeof(float) * ((size_t)n_pairs + grid.x))
        part_max = reinterpret_cast<float *>(reinterpret_cast<char *>(lse2) + lse_bytes);
    if (!part_max) hipLaunchKernelGGL(k_fill_zero, dim3((B + 63) / 64), dim3(64), 0, st, scale_out, B);
    hipLaunchKernelGGL(k1, grid, dim3(kXThreads), CF::lds_pass1, st, q, k, v, key_bias, N, H, d, nk,
                       bits, qk_scale, tpw, n_pairs, out, scale_out, lse2, codes_dump, nullptr, part_max, tpw);
    hipLaunchKernelGGL(k2, grid2, dim3(kXThreads), CF::lds_pass2, st, q, k, v, key_bias, N, H, d, nk,
                       bits, qk_scale, tpw2, n_pairs, out, scale_out, lse2, codes_dump, nullptr, part_max, tpw);
    return hipGetLastError();
}

// Head dims above 96 keep K and V^T of at most 94 keys in LDS (the 96-key tile: 134 KB).
bool mfma_shape(int32_t d, int32_t nk) {
    return (d % 8) == 0 && ((d <= 96 && nk + 2 <= 128) || (d <= 160 && nk + 2 <= 96));
}

// ======================================================================================
// Self-attention: every key quantized, given scale, keys streamed in tiles of 32
// ======================================================================================
// Section 3.3 applies the log quantizer to self-attention too; there is no <start> column
// and the scale s_b is given.  The number of keys equals the number of queries (4096 on
// the 64 x 64 latent), so K and V^T cannot live in LDS whole as in the kernels above.  A
// first kernel writes them once per (prompt, head), in tiles of 32 keys, as the very bytes
// LDS will hold:
//   [Kh | Kl]  32 keys x PITCH   fp16 hi / lo of K log2(e) / sqrt(d) (64, 128 or 192 dims,
//                                zero-padded)
//   [Vh | Vl]  DV dims x 64 B    bf16 hi / lo of s_b V^T, the 32 key slots of a tile in the
//                                order the accumulator registers of S^T hold them
// with the 16-byte slots of every row XOR-permuted by row bits, so that the 16-byte fragment
// reads of 32 consecutive rows spread over all banks.  The second kernel gives each of its
// eight wavefronts 32 queries (their fp16 pieces stay in registers) and sweeps the key tiles
// twice through a three-stage LDS ring filled by direct-to-LDS loads of 1 KiB (the tile
// image is copied verbatim): sweep A takes the running maximum and sum of 2^(S - max) for
// lse2, sweep B recomputes S^T bit-identically, forms the codes from log2 s + lse2 - S as
// above and accumulates Out^T = V^T P^T.  A code depends on the row's full sum, so one
// sweep cannot do both.  (Read straight from memory by every wavefront, the fragments cost
// 24 KB of cache traffic per wavefront and tile pair and the texture path, not the matrix
// cores, set the pace: 5.8 ms on 16 x 10 x 4096 x 64.)
template <int KS_>
struct SCfg {
    static constexpr int KS = KS_;
    static constexpr int DB = (KS + 1) / 2;   // 32-wide blocks of output dims
    static constexpr int DV = 32 * DB;
    static constexpr int PITCH = 128 * ((KS + 3) / 4);  // bytes per K row: whole groups of 8 slots
    static constexpr int K_BYTES = 2 * 32 * PITCH;      // hi + lo
    static constexpr int V_BYTES = 2 * DV * 64;    // hi + lo
    static constexpr int TILE_BYTES = K_BYTES + V_BYTES;
    static constexpr int K_CHUNKS = K_BYTES / 1024, TILE_CHUNKS = TILE_BYTES / 1024;
    static constexpr int STAGES = 3;
    // direct-to-LDS loads per wave and tile (8 waves): sweep A copies the K part, sweep B all
    static constexpr int LA = K_CHUNKS / 8, LB = (TILE_CHUNKS + 7) / 8;
    // wavefronts per SIMD the registers are budgeted for: the query pieces and the output
    // blocks of a wide head take most of the file
    static constexpr int OCC = KS <= 4 ? 2 : 1;
};
constexpr int kSWaves = 8;  // wavefronts per workgroup: 256 queries share every tile

// slot of key j (0..31) of a tile in the V^T rows: inside each 16-key step the lower lane
// half takes keys 0..3 and 8..11, the upper half keys 4..7 and 12..15
__device__ __host__ constexpr int v_slot(int j) {
    return 16 * (j >> 4) + 8 * ((j >> 2) & 1) + (j & 3) + 4 * ((j >> 3) & 1);
}
// byte offsets inside a tile image: 16-byte slot c of K row j / of V^T row t.  A wave reads
// 16 bytes per lane from 32 consecutive rows, and LDS serves 16 lanes (256 bytes, 64 banks)
// at a time: the sixteen 16-byte bank groups those lanes touch -- address bits 4..7 -- must
// all differ.  64-byte rows (V^T): bits 6..7 are row bits 0..1, the slot takes bit 2 and
// bit 1 ^ bit 3 (the permutation of the contraction kernel's rows, which measures no bank
// conflict).  128- and 384-byte rows: bit 7 is row bit 0, the slot takes row bits 1..3.
// 256-byte rows: no row bit reaches the bank bits, the slot takes all four.  (XOR-ing with
// row % 8 left half of the LDS cycles in conflict.)
__device__ __host__ inline int k_row_key(int pitch, int j) {
    return ((j >> 1) & 7) | (pitch == 256 ? (j & 1) << 3 : 0);
}
__device__ __host__ inline int k_row_slot(int pitch, int j, int c) {
    return j * pitch + ((c ^ k_row_key(pitch, j)) << 4);
}
__device__ __host__ inline int v_row_slot(int t, int c) { return t * 64 + ((c ^ swz64(t)) << 4); }

#define DGQ_X_LDS_DMA16(sbase, voff, l0)                                              \
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"      \
                 :                                                                    \
                 : "v"(voff), "s"(sbase), "s"(l0)                                     \
                 : "memory", "m0")
#define DGQ_X_WAIT_VMCNT(N) \
    __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

template <class CF>
__global__ __launch_bounds__(256) void k_selfattn_prep(
    const float *__restrict__ k, const float *__restrict__ v, int32_t nk, int32_t H, int32_t d,
    float qk_scale, const float *__restrict__ scale_in, int32_t n_tiles,
    uint8_t *__restrict__ ws) {
    constexpr int DV = CF::DV;
    const int32_t tile = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int64_t hs = (int64_t)H * d;
    const int64_t bh = (int64_t)b * H + head;
    const float s_b = scale_in[b];
    const float s_eff = s_b > 0.0f ? s_b : 1.0f;
    const float *kb = k + ((int64_t)b * nk * H + head) * d;
    const float *vb = v + ((int64_t)b * nk * H + head) * d;
    uint8_t *img = ws + (bh * n_tiles + tile) * CF::TILE_BYTES;
    uint8_t *khp = img, *klp = img + 32 * CF::PITCH;
    uint8_t *vhp = img + CF::K_BYTES, *vlp = vhp + DV * 64;
    constexpr int QUADS = CF::PITCH / 8;  // fours of dims per K row
    for (int idx = tid; idx < 32 * QUADS; idx += 256) {
        const int j = idx / QUADS, t4 = (idx - j * QUADS) * 4;
        const int32_t key = 32 * tile + j;
        float4 x = {0.0f, 0.0f, 0.0f, 0.0f};
        if (key < nk && t4 < d) x = *reinterpret_cast<const float4 *>(kb + (int64_t)key * hs + t4);
        const HiLo p0 = split_h2(x.x * qk_scale, x.y * qk_scale);
        const HiLo p1 = split_h2(x.z * qk_scale, x.w * qk_scale);
        const int off = k_row_slot(CF::PITCH, j, t4 >> 3) + (t4 & 7) * 2;
        *reinterpret_cast<u32x2 *>(khp + off) = u32x2{p0.hi, p1.hi};
        *reinterpret_cast<u32x2 *>(klp + off) = u32x2{p0.lo, p1.lo};
    }
    for (int idx = tid; idx < 32 * (DV / 4); idx += 256) {
        const int j = idx / (DV / 4), t4 = (idx - j * (DV / 4)) * 4;
        const int32_t key = 32 * tile + j;
        float4 x = {0.0f, 0.0f, 0.0f, 0.0f};
        if (key < nk && t4 < d) x = *reinterpret_cast<const float4 *>(vb + (int64_t)key * hs + t4);
        const float xe[4] = {x.x * s_eff, x.y * s_eff, x.z * s_eff, x.w * s_eff};
        const int slot = v_slot(j);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t hb = bf16_rne_bits(xe[e]);
            const uint32_t lb = bf16_rne_bits(xe[e] - __uint_as_float(hb));
            const int off = v_row_slot(t4 + e, slot >> 3) + (slot & 7) * 2;
            *reinterpret_cast<uint16_t *>(vhp + off) = (uint16_t)(hb >> 16);
            *reinterpret_cast<uint16_t *>(vlp + off) = (uint16_t)(lb >> 16);
        }
    }
}

template <class CF, bool DUMP>
__global__ __launch_bounds__(64 * kSWaves, CF::OCC) void k_selfattn(
    const float *__restrict__ q, int32_t BH, int32_t N, int32_t H, int32_t d, int32_t bits,
    int32_t n_tiles, int32_t q_tiles, const uint8_t *__restrict__ ws,
    const float *__restrict__ scale_in, float *__restrict__ out, float *__restrict__ scale_out,
    uint8_t *__restrict__ codes_dump) {
    constexpr int KS = CF::KS, DB = CF::DB, DV = CF::DV, STAGES = CF::STAGES;
    extern __shared__ __attribute__((aligned(1024))) uint8_t ring[];
    // Workgroup w runs on XCD w % 8: give every XCD whole (prompt, head) pairs, so that the
    // pair's tile images (2 MB at 4096 keys) are fetched into one L2 only.
    const int32_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int32_t bh = (slot / q_tiles) * 8 + xcd;
    if (bh >= BH) return;  // the whole workgroup
    const int32_t b = bh / H, head = bh - b * H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int32_t q0 = ((slot % q_tiles) * kSWaves + wave) * 32;
    const int n = lane & 31, hh = lane >> 5;
    const int32_t nk = N;
    const int32_t qi = q0 + n;
    const bool valid = qi < N;  // a wave past the end still walks the ring with the others
    const int64_t hs = (int64_t)H * d;

    const float s_b = scale_in[b];
    const float s_eff = s_b > 0.0f ? s_b : 1.0f;
    const uint32_t pmask = s_b > 0.0f ? 0xFFFFFFFFu : 0u;  // scale 0: every product is 0
    const float l2s = __log2f(s_eff);

    // ---- the lane's query slices as fp16 pieces: dims 16 s + 8 hh .. + 7 -------------------
    u32x4 qh[KS], ql[KS];
    {
        const float *p = q + ((int64_t)b * N * H + head) * d + (int64_t)(valid ? qi : N - 1) * hs + 8 * hh;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            float4 a = {0.0f, 0.0f, 0.0f, 0.0f}, c = a;
            if (16 * s + 8 * hh < d) {
                a = *reinterpret_cast<const float4 *>(p + 16 * s);
                c = *reinterpret_cast<const float4 *>(p + 16 * s + 4);
            }
            const HiLo p0 = split_h2(a.x, a.y), p1 = split_h2(a.z, a.w);
            const HiLo p2 = split_h2(c.x, c.y), p3 = split_h2(c.z, c.w);
            qh[s] = u32x4{p0.hi, p1.hi, p2.hi, p3.hi};
            ql[s] = u32x4{p0.lo, p1.lo, p2.lo, p3.lo};
        }
    }

    // ---- the ring: tile kt lives in stage kt % STAGES; wave w copies 1 KiB chunk w of the
    // image, w + 8, ... (sweep A: the K part only; past the last chunk a wave copies the last
    // one again: same bytes, same place)
    const uint8_t *img0 = ws + (int64_t)bh * n_tiles * CF::TILE_BYTES;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const uint32_t ring0 = (uint32_t)reinterpret_cast<uintptr_t>(
        (const __attribute__((address_space(3))) uint8_t *)ring);
    auto issue = [&](const bool with_v, int32_t kt) __attribute__((always_inline)) {
        const uint8_t *src = img0 + (int64_t)kt * CF::TILE_BYTES;
        const uint32_t dst = ring0 + (uint32_t)(kt % STAGES) * CF::TILE_BYTES;
#pragma unroll
        for (int j = 0; j < CF::LB; ++j) {
            if (!with_v && j >= CF::LA) break;
            int c = wave + kSWaves * j;
            c = c < CF::TILE_CHUNKS ? c : CF::TILE_CHUNKS - 1;
            DGQ_X_LDS_DMA16(src + c * 1024, lane16, dst + (uint32_t)c * 1024u);
        }
    };
    // One step of a sweep: tile kt has landed for every wave, and the stage the tile after
    // next goes to is no longer read by anyone.
    auto advance = [&](const bool with_v, int32_t kt) __attribute__((always_inline)) {
        asm volatile("" ::: "memory");
        // the code dump's stores share the counter and need not return in order with loads
        if (DUMP || kt + 1 >= n_tiles)
            DGQ_X_WAIT_VMCNT(0);
        else if (with_v)
            DGQ_X_WAIT_VMCNT(CF::LB);
        else
            DGQ_X_WAIT_VMCNT(CF::LA);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (kt + 2 < n_tiles) issue(with_v, kt + 2);
    };

    const int k_row = n * CF::PITCH, k_key = k_row_key(CF::PITCH, n) ^ hh;  // slot 2 s + hh of row n
    // S^T of the tile in `stage` for the wave's 32 queries, in log2 units; padding keys -inf
    auto s_tile = [&](int32_t kt, v16f &sm) {
        const uint8_t *st = ring + (kt % STAGES) * CF::TILE_BYTES;
        // all fragments of a narrow head are read up front; a wide head (whose query pieces
        // and output blocks fill the register file) reads them one step ahead of their MFMAs
        constexpr int NF = KS <= 4 ? KS : 2;
        u32x4 fh[NF], fl[NF];
        auto frag = [&](int s) __attribute__((always_inline)) {
            const int off = k_row + ((k_key ^ (2 * s)) << 4);
            fh[s % NF] = *reinterpret_cast<const u32x4 *>(st + off);
            fl[s % NF] = *reinterpret_cast<const u32x4 *>(st + 32 * CF::PITCH + off);
        };
#pragma unroll
        for (int s = 0; s < (KS <= 4 ? KS : 1); ++s) frag(s);
#pragma unroll
        for (int i = 0; i < 16; ++i) sm[i] = 0.0f;
        if (32 * kt + 32 > nk) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (32 * kt + key_of(0, i, hh) >= nk) sm[i] = -INFINITY;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (KS > 4 && s + 1 < KS) frag(s + 1);
            const v8h bqh = __builtin_bit_cast(v8h, qh[s]);
            const v8h bql = __builtin_bit_cast(v8h, ql[s]);
            const v8h akh = __builtin_bit_cast(v8h, fh[s % NF]);
            const v8h akl = __builtin_bit_cast(v8h, fl[s % NF]);
            sm = __builtin_amdgcn_mfma_f32_32x32x16_f16(akh, bqh, sm, 0, 0, 0);
            sm = __builtin_amdgcn_mfma_f32_32x32x16_f16(akh, bql, sm, 0, 0, 0);
            sm = __builtin_amdgcn_mfma_f32_32x32x16_f16(akl, bqh, sm, 0, 0, 0);
        }
    };

    // ---- sweep A: lse2 of the lane's query (each lane half sees half of the keys) -------
    float m = -INFINITY, l = 0.0f;
    issue(false, 0);
    if (n_tiles > 1) issue(false, 1);
    for (int32_t kt = 0; kt < n_tiles; ++kt) {
        advance(false, kt);
        v16f sm;
        s_tile(kt, sm);
        float tm = sm[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tm = fmaxf(tm, sm[i]);
        const float mn = fmaxf(m, tm);
        const float ms = mn == -INFINITY ? 0.0f : mn;
        float add = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) add += __builtin_amdgcn_exp2f(sm[i] - ms);
        l = l * __builtin_amdgcn_exp2f(m - ms) + add;
        m = mn;
    }
    float lse;
    {
        const float mo = __shfl_xor(m, 32, kWave), lo = __shfl_xor(l, 32, kWave);
        const float m2 = fmaxf(m, mo);  // finite: key 0 exists
        const float l2 = l * __builtin_amdgcn_exp2f(m - m2) + lo * __builtin_amdgcn_exp2f(mo - m2);
        lse = m2 + __log2f(l2);
        if (scale_out) {
            // the row's largest probability; probabilities order like their bit patterns
            float amax = valid ? m2 - lse : -INFINITY;
            amax = wave_max(amax);
            if (lane == 0 && q0 < N)
                atomicMax(reinterpret_cast<unsigned int *>(scale_out + b),
                          __float_as_uint(__builtin_amdgcn_exp2f(amax)));
        }
    }

    // ---- sweep B: codes and Out^T = V^T P^T -------------------------------------------------
    const float c0 = l2s + lse;
    const float thr = l2s + 150.0f;
    constexpr int32_t kMagic = 0x4B400000;  // bit pattern of 12582912.0f
    // exponents 127 - code of two keys from m = magic - code: (m0 << 7) + (m1 << 23) + this
    constexpr uint32_t kPairBase = 0u - (((uint32_t)(kMagic - 127) << 7) + ((uint32_t)(kMagic - 127) << 23));
    const int32_t cq = (1 << bits) - 1;
    const int32_t ce = cq < 127 ? cq : 127;  // 2^-127 and below leave the product as zero
    uint8_t *cd = nullptr;
    if (DUMP) cd = codes_dump + ((int64_t)bh * N + (valid ? qi : 0)) * (int64_t)nk;
    v16f o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = 0.0f;
    const int v_off = v_row_slot(n, hh);  // slot 2 u + hh: the step enters as an XOR of 2 u
    __builtin_amdgcn_s_barrier();  // every wave has left sweep A's last stage
    asm volatile("" ::: "memory");
    issue(true, 0);
    if (n_tiles > 1) issue(true, 1);
    for (int32_t kt = 0; kt < n_tiles; ++kt) {
        advance(true, kt);
        v16f sm;
        s_tile(kt, sm);
        const uint8_t *st = ring + (kt % STAGES) * CF::TILE_BYTES + CF::K_BYTES;
        // V^T fragments of this tile.  Narrow heads: all read before the code arithmetic that
        // hides them; wide heads: each right before its MFMAs (registers)
        constexpr bool V_AHEAD = DB <= 2;
        auto v_frag = [&](int db, int u, u32x4 &h, u32x4 &l) __attribute__((always_inline)) {
            const int off = db * 32 * 64 + (v_off ^ (u << 5));
            h = *reinterpret_cast<const u32x4 *>(st + off);
            l = *reinterpret_cast<const u32x4 *>(st + DV * 64 + off);
        };
        u32x4 fvh[V_AHEAD ? DB : 1][2], fvl[V_AHEAD ? DB : 1][2];
        if (V_AHEAD) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int u = 0; u < 2; ++u) v_frag(db, u, fvh[V_AHEAD ? db : 0][u], fvl[V_AHEAD ? db : 0][u]);
        }
        uint32_t pk[8];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            uint32_t m[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                float t = sm[i + u] - c0;  // minus the code before rounding
                // a probability that is zero in fp32 takes the top code; the product does not
                // need the rule (every code above 126 gives a zero weight anyway)
                if (DUMP) t = t < -thr ? -300.0f : t;
                const int32_t r = __float_as_int(t + 12582912.0f);
                if (DUMP) {
                    const int32_t key = 32 * kt + key_of(0, i + u, hh);
                    const int32_t c = kMagic - clamp_i32(r, kMagic - cq, kMagic);
                    if (valid && key < nk) cd[key] = (uint8_t)c;
                }
                m[u] = (uint32_t)clamp_i32(r, kMagic - ce, kMagic);
            }
            pk[i >> 1] = ((m[0] << 7) + ((m[1] << 23) + kPairBase)) & pmask;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const u32x4 pb = {pk[4 * u + 0], pk[4 * u + 1], pk[4 * u + 2], pk[4 * u + 3]};
            const v8bf bp = __builtin_bit_cast(v8bf, pb);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                u32x4 h, l;
                if (V_AHEAD) {
                    h = fvh[V_AHEAD ? db : 0][u];
                    l = fvl[V_AHEAD ? db : 0][u];
                } else {
                    v_frag(db, u, h, l);
                }
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, h), bp, o[db], 0, 0, 0);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, l), bp, o[db], 0, 0, 0);
            }
        }
    }
    if (valid) {
        float *orow = out + ((int64_t)b * N * H + head) * d + (int64_t)qi * hs;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int dim = 32 * db + 8 * a + 4 * hh;
                if (dim < d) {
                    const float4 t = {o[db][4 * a + 0], o[db][4 * a + 1], o[db][4 * a + 2], o[db][4 * a + 3]};
                    *reinterpret_cast<float4 *>(orow + dim) = t;
                }
            }
    }
}

template <class CF>
hipError_t launch_selfattn_cfg(const float *q, const float *k, const float *v, int32_t B, int32_t N,
                               int32_t H, int32_t d, int32_t bits, const float *scale_in, float *out,
                               float *scale_out, uint8_t *codes_dump, void *workspace,
                               hipStream_t st) {
    const int32_t n_tiles = (N + 31) / 32, BH = B * H;
    uint8_t *ws = static_cast<uint8_t *>(workspace);
    const float qk_scale = (float)(1.4426950408889634 / sqrt((double)d));
    if (scale_out) hipLaunchKernelGGL(k_fill_zero, dim3((B + 63) / 64), dim3(64), 0, st, scale_out, B);
    hipLaunchKernelGGL(k_selfattn_prep<CF>, dim3(n_tiles, H, B), dim3(256), 0, st, k, v, N, H, d,
                       qk_scale, scale_in, n_tiles, ws);
    const int32_t q_tiles = (N + 32 * kSWaves - 1) / (32 * kSWaves);
    const int64_t groups = ((int64_t)BH + 7) / 8;
    const dim3 grid((unsigned)(groups * q_tiles * 8));
    const size_t lds = (size_t)CF::STAGES * CF::TILE_BYTES;
    {
        hipError_t e = DGQ_ENSURE_LDS((k_selfattn<CF, true>), (int)lds);
        if (e == hipSuccess) e = DGQ_ENSURE_LDS((k_selfattn<CF, false>), (int)lds);
        if (e != hipSuccess) return e;
    }
    if (codes_dump)
        hipLaunchKernelGGL((k_selfattn<CF, true>), grid, dim3(64 * kSWaves), lds, st, q, BH, N, H, d, bits,
                           n_tiles, q_tiles, ws, scale_in, out, scale_out, codes_dump);
    else
        hipLaunchKernelGGL((k_selfattn<CF, false>), grid, dim3(64 * kSWaves), lds, st, q, BH, N, H, d, bits,
                           n_tiles, q_tiles, ws, scale_in, out, scale_out, codes_dump);
    return hipGetLastError();
}

// ======================================================================================
// Plain fp32 path (any head dim up to 256, any nk up to 128)
// ======================================================================================

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
    uint8_t *__restrict__ codes_dump, const float *__restrict__ scale_in) {
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
    const float s = scale_in ? scale_in[b] : scale[b];  // given, or this call's maximum
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

// Pass 2 of the attention on the integer codes of V^: the product of Section 3.3 as the shifts
// and adds Section 3.1 promises for the log quantizer.  With 4-bit codes A^q in 0..15 every
// quantized weight is s_b 2^-A^q = s_b 2^-15 (1 << (15 - A^q)), and V^ = s_v q_v + z_v with
// 8-bit q_v, so
//   sum_{j>=1} A^_ij V^_j = s_b 2^-15 ( s_v sum_j (q_v[j] << (15 - A^q_ij)) + z_v sum_j (1 << (15 - A^q_ij)) ),
// both sums exact in int32 (at most 127 keys x 255 x 2^15 < 2^31).  One thread per (query,
// head) as in k_xattn; V^'s codes wait in LDS as one dword per element, so the inner loop is
// one shift-and-add instruction per (key, dimension).  The <start> column stays in floating
// point: A_i0 times the reconstruction s_v q_v[0] + z_v.  The few floating-point operations
// that combine the integer sums run in double and round once.
template <int NKP>
__global__ __launch_bounds__(256) void k_xattn_intv(
    const float *__restrict__ q, const float *__restrict__ k, const uint8_t *__restrict__ vq,
    const float *__restrict__ vparams, const float *__restrict__ key_bias, int32_t N, int32_t H,
    int32_t d, int32_t dpad, int32_t nk, float inv_sqrt_d, float *__restrict__ out,
    const float *__restrict__ scale, uint8_t *__restrict__ codes_dump, int32_t *__restrict__ acc_dump) {
    extern __shared__ float kv[];  // [NKP][dpad]: K as floats, then V^'s codes as integers
    const int32_t b = blockIdx.z, h = blockIdx.y;
    const int32_t n_raw = blockIdx.x * 256 + threadIdx.x;
    const bool valid = n_raw < N;
    const int32_t n = valid ? n_raw : N - 1;
    const int64_t hs = (int64_t)H * d;

    stage_head<NKP>(k + ((int64_t)b * nk * H + h) * d, nk, d, dpad, hs, kv);
    __syncthreads();
    float L[NKP];
#pragma unroll
    for (int j = 0; j < NKP; ++j) L[j] = 0.0f;
    const float *qr = q + (((int64_t)b * N + n) * H + h) * d;
    for (int32_t t = 0; t < d; ++t) {
        const float qv = qr[t];
#pragma unroll
        for (int j = 0; j < NKP; ++j) L[j] = fmaf(qv, kv[j * dpad + t], L[j]);
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
    float sum = 0.0f;
#pragma unroll
    for (int j = 0; j < NKP; ++j) {
        L[j] = (L[j] - m) * kLog2e;
        sum += __builtin_amdgcn_exp2f(L[j]);
    }
    const float s = scale[b];
    const float l2s = __log2f(s), lse2 = __log2f(sum);
    const float a0 = __builtin_amdgcn_exp2f(L[0]) / sum;
    uint8_t *cd = codes_dump
                      ? codes_dump + ((((int64_t)b * H + h) * N + n) * (int64_t)(nk - 1))
                      : nullptr;
    // the shift of every key, four bits each: 15 - A^q (the <start> column and padding keys take none)
    uint32_t sh[NKP / 8];
#pragma unroll
    for (int w = 0; w < NKP / 8; ++w) sh[w] = 0;
    int32_t zsum = 0;
#pragma unroll
    for (int j = 1; j < NKP; ++j) {
        if (j < nk) {
            const float l2a = L[j] - lse2;
            float c = fminf(fmaxf(rintf(l2s - l2a), 0.0f), 15.0f);
            if (l2a < -150.0f) c = 15.0f;
            if (cd && valid) cd[j - 1] = (uint8_t)c;
            const uint32_t shift = 15u - (uint32_t)c;
            sh[j >> 3] |= shift << (4 * (j & 7));
            zsum += 1 << shift;
        }
    }

    // ---- V^'s codes replace K in LDS, one dword per element -------------------------------
    __syncthreads();
    int32_t *vi = reinterpret_cast<int32_t *>(kv);
    {
        const uint8_t *src = vq + ((int64_t)b * nk * H + h) * d;
        for (int32_t idx = threadIdx.x; idx < NKP * dpad; idx += 256) {
            const int32_t j = idx / dpad, t = idx - j * dpad;
            vi[idx] = (j < nk && t < d) ? (int32_t)src[(int64_t)j * hs + t] : 0;
        }
    }
    __syncthreads();
    const double sv = (double)vparams[((int64_t)b * H + h) * 2 + 0], zv = (double)vparams[((int64_t)b * H + h) * 2 + 1];
    const double tail = zv * (double)zsum;
    const double ws = (double)s * (1.0 / 32768.0);
    float *orow = out + (((int64_t)b * N + n) * H + h) * d;
    int32_t *arow = acc_dump ? acc_dump + (((int64_t)b * N + n) * H + h) * d : nullptr;
    for (int32_t t = 0; t < d; ++t) {
        int32_t acc = 0;
#pragma unroll
        for (int j = 1; j < NKP; ++j)
            acc += vi[j * dpad + t] << ((sh[j >> 3] >> (4 * (j & 7))) & 15u);  // padding keys hold code 0
        if (valid) {
            const float v0 = fmaf((float)sv, (float)vi[t], (float)zv);  // the fp32 reconstruction of V^_0
            orow[t] = (float)((double)a0 * (double)v0 + ws * (sv * (double)acc + tail));
            if (arow) arow[t] = acc;
        }
    }
}

// V^ of the product A^ V^ (Section 3.3): one workgroup per (prompt, head) finds the range
// of its [nk, d] slice, quantizes with s = (max - min) / 2^b, z = min (separate subtract
// and multiply, round to nearest even, clamp) and writes the reconstruction s q + z
// (one fused multiply-add, i.e. rounded once), optionally the codes and (s, z).
__global__ __launch_bounds__(256) void k_quantize_value(
    const float *v, int32_t nk, int32_t H, int32_t d, int32_t bits, float *vhat /* may be v */,
    uint8_t *__restrict__ codes, float *__restrict__ params) {
    __shared__ float red_mx[4], red_mn[4];
    const int32_t b = blockIdx.y, h = blockIdx.x;
    const int64_t base = ((int64_t)b * nk * H + h) * d, hs = (int64_t)H * d;
    const int32_t n = nk * d;
    float mx = -INFINITY, mn = INFINITY;
    for (int32_t i = threadIdx.x; i < n; i += 256) {
        const int32_t j = i / d, t = i - j * d;
        const float x = v[base + (int64_t)j * hs + t];
        mx = x > mx ? x : mx;
        mn = x < mn ? x : mn;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float a = __shfl_xor(mx, o, kWave), c = __shfl_xor(mn, o, kWave);
        mx = a > mx ? a : mx;
        mn = c < mn ? c : mn;
    }
    if ((threadIdx.x & 63) == 0) {
        red_mx[threadIdx.x >> 6] = mx;
        red_mn[threadIdx.x >> 6] = mn;
    }
    __syncthreads();
    mx = fmaxf(fmaxf(red_mx[0], red_mx[1]), fmaxf(red_mx[2], red_mx[3]));
    mn = fminf(fminf(red_mn[0], red_mn[1]), fminf(red_mn[2], red_mn[3]));
    const float levels = (float)(1 << bits), qmax = levels - 1.0f;
    const float s = mx > mn ? __fdiv_rn(__fsub_rn(mx, mn), levels) : 1.0f;
    const float inv = __fdiv_rn(1.0f, s);
    if (params && threadIdx.x == 0) {
        params[((int64_t)b * H + h) * 2 + 0] = s;
        params[((int64_t)b * H + h) * 2 + 1] = mn;
    }
    for (int32_t i = threadIdx.x; i < n; i += 256) {
        const int32_t j = i / d, t = i - j * d;
        const int64_t at = base + (int64_t)j * hs + t;
        const float u = __fmul_rn(__fsub_rn(v[at], mn), inv);
        float qf = fminf(fmaxf(rintf(u), 0.0f), qmax);  // NaN -> 0
        if (codes) codes[at] = (uint8_t)qf;
        vhat[at] = __fmaf_rn(s, qf, mn);
    }
}

template <int NKP>
hipError_t launch_passes(const float *q, const float *k, const float *v, const float *key_bias,
                         int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
                         float *out, float *scale_out, uint8_t *codes_dump,
                         const float *scale_in, hipStream_t st) {
    const int32_t dpad = (d + 3) / 4 * 4;
    const size_t lds = sizeof(float) * (size_t)NKP * dpad;
    const float inv_sqrt_d = (float)(1.0 / sqrt((double)d));
    const dim3 grid((N + 255) / 256, H, B);
    auto k1 = k_xattn<NKP, 1>;
    auto k2 = k_xattn<NKP, 2>;
    if (lds > 64 * 1024) {
        hipError_t e = DGQ_ENSURE_LDS((k_xattn<NKP, 1>), (int)lds);
        if (e != hipSuccess) return e;
        e = DGQ_ENSURE_LDS((k_xattn<NKP, 2>), (int)lds);
        if (e != hipSuccess) return e;
    }
    // scale_out accumulates a maximum: clear it with a fill kernel (capturable in a graph)
    // the first pass collects this call's maximum (with a given scale only if it is asked for)
    if (scale_out) {
        hipLaunchKernelGGL(k_fill_zero, dim3((B + 63) / 64), dim3(64), 0, st, scale_out, B);
        hipLaunchKernelGGL(k1, grid, dim3(256), lds, st, q, k, v, key_bias, N, H, d, dpad, nk, bits,
                           inv_sqrt_d, out, scale_out, codes_dump, nullptr);
    }
    hipLaunchKernelGGL(k2, grid, dim3(256), lds, st, q, k, v, key_bias, N, H, d, dpad, nk, bits,
                       inv_sqrt_d, out, scale_out, codes_dump, scale_in);
    return hipGetLastError();
}

}  // namespace

// The matrix-core path keeps one float (log2 of the soft-max denominator, shifted by the
// row maximum) per (prompt, head, query) between its two passes.
size_t xattn_workspace_min_bytes(int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk) {
    if (!mfma_shape(d, nk)) return 0;
    return xattn_lse_bytes(B, N, H);
}

// The row statistics plus one slot per piece of pass 1 (pairs + ranges, with room for a
// tuning build's larger range counts).
size_t xattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk) {
    if (!mfma_shape(d, nk)) return 0;
    return xattn_lse_bytes(B, N, H) + (sizeof(float) * ((size_t)B * H + 4096) + 255) / 256 * 256;
}

hipError_t launch_quantize_value(const float *v, int32_t B, int32_t nk, int32_t H, int32_t d,
                                 int32_t bits, float *vhat, uint8_t *codes, float *params,
                                 hipStream_t st) {
    hipLaunchKernelGGL(k_quantize_value, dim3(H, B), dim3(256), 0, st, v, nk, H, d, bits, vhat,
                       codes, params);
    return hipGetLastError();
}

template <int NKP>
hipError_t launch_intv_nkp(const float *q, const float *k, const uint8_t *vq, const float *vparams,
                           const float *key_bias, int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk,
                           float *out, float *scale_out, uint8_t *codes_dump, int32_t *acc_dump,
                           hipStream_t st) {
    const int32_t dpad = (d + 3) / 4 * 4;
    const size_t lds = sizeof(float) * (size_t)NKP * dpad;
    const float inv_sqrt_d = (float)(1.0 / sqrt((double)d));
    const dim3 grid((N + 255) / 256, H, B);
    if (lds > 64 * 1024) {
        hipError_t e = DGQ_ENSURE_LDS((k_xattn<NKP, 1>), (int)lds);
        if (e != hipSuccess) return e;
        e = DGQ_ENSURE_LDS((k_xattn_intv<NKP>), (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_fill_zero, dim3((B + 63) / 64), dim3(64), 0, st, scale_out, B);
    hipLaunchKernelGGL((k_xattn<NKP, 1>), grid, dim3(256), lds, st, q, k, static_cast<const float *>(nullptr),
                       key_bias, N, H, d, dpad, nk, 4, inv_sqrt_d, out, scale_out,
                       static_cast<uint8_t *>(nullptr), static_cast<const float *>(nullptr));
    hipLaunchKernelGGL((k_xattn_intv<NKP>), grid, dim3(256), lds, st, q, k, vq, vparams, key_bias, N, H, d,
                       dpad, nk, inv_sqrt_d, out, scale_out, codes_dump, acc_dump);
    return hipGetLastError();
}

hipError_t launch_xattn_intv(const float *q, const float *k, const uint8_t *vq, const float *vparams,
                             const float *key_bias, int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk,
                             float *out, float *scale_out, uint8_t *codes_dump, int32_t *acc_dump,
                             hipStream_t st) {
    if (nk <= 80)
        return launch_intv_nkp<80>(q, k, vq, vparams, key_bias, B, N, H, d, nk, out, scale_out, codes_dump,
                                   acc_dump, st);
    return launch_intv_nkp<128>(q, k, vq, vparams, key_bias, B, N, H, d, nk, out, scale_out, codes_dump,
                                acc_dump, st);
}

hipError_t launch_xattn(const float *q, const float *k, const float *v, const float *key_bias,
                        int32_t B, int32_t N, int32_t H, int32_t d, int32_t nk, int32_t bits,
                        float *out, float *scale_out, uint8_t *codes_dump, void *workspace,
                        size_t workspace_bytes, const float *scale_in, hipStream_t st) {
    if (mfma_shape(d, nk)) {
        float *lse2 = static_cast<float *>(workspace);
        const int ks = d <= 48 ? 3 : (d <= 64 ? 4 : (d <= 96 ? 6 : 10));
        const int nkb = nk + 2 <= 96 ? 3 : 4;
#define DGQ_XATTN_CASE(NKB, KS)                                                              \
    if (nkb == NKB && ks == KS)                                                              \
        return launch_mfma<XCfg<NKB, KS>>(q, k, v, key_bias, B, N, H, d, nk, bits, out,       \
                                          scale_out, codes_dump, lse2, workspace_bytes, scale_in, st);
        DGQ_XATTN_CASE(3, 3)
        DGQ_XATTN_CASE(3, 4)
        DGQ_XATTN_CASE(3, 6)
        DGQ_XATTN_CASE(3, 10)
        DGQ_XATTN_CASE(4, 3)
        DGQ_XATTN_CASE(4, 4)
        DGQ_XATTN_CASE(4, 6)
#undef DGQ_XATTN_CASE
    }
    if (nk <= 80)
        return launch_passes<80>(q, k, v, key_bias, B, N, H, d, nk, bits, out, scale_out,
                                 codes_dump, scale_in, st);
    return launch_passes<128>(q, k, v, key_bias, B, N, H, d, nk, bits, out, scale_out, codes_dump,
                              scale_in, st);
}

// K and V^T of every (prompt, head) pair in the matrix cores' pieces (see k_selfattn_prep).
static int selfattn_ks(int32_t d) {
    return d <= 16 ? 1 : (d <= 32 ? 2 : (d <= 48 ? 3 : (d <= 64 ? 4 : (d <= 80 ? 5 : 10))));
}

size_t selfattn_workspace_bytes(int32_t B, int32_t N, int32_t H, int32_t d) {
    if (d % 8 != 0 || d > 160 || d < 8) return 0;
    const size_t ks = (size_t)selfattn_ks(d), dv = 32 * ((ks + 1) / 2), pitch = 128 * ((ks + 3) / 4);
    const size_t n_tiles = ((size_t)N + 31) / 32;
    return (size_t)B * H * n_tiles * (2 * 32 * pitch + 2 * dv * 64);  // one tile image per 32 keys
}

hipError_t launch_selfattn(const float *q, const float *k, const float *v, int32_t B, int32_t N,
                           int32_t H, int32_t d, int32_t bits, const float *scale_in, float *out,
                           float *scale_out, uint8_t *codes_dump, void *workspace, hipStream_t st) {
    switch (selfattn_ks(d)) {
        case 1: return launch_selfattn_cfg<SCfg<1>>(q, k, v, B, N, H, d, bits, scale_in, out, scale_out, codes_dump, workspace, st);
        case 2: return launch_selfattn_cfg<SCfg<2>>(q, k, v, B, N, H, d, bits, scale_in, out, scale_out, codes_dump, workspace, st);
        case 3: return launch_selfattn_cfg<SCfg<3>>(q, k, v, B, N, H, d, bits, scale_in, out, scale_out, codes_dump, workspace, st);
        case 4: return launch_selfattn_cfg<SCfg<4>>(q, k, v, B, N, H, d, bits, scale_in, out, scale_out, codes_dump, workspace, st);
        case 5: return launch_selfattn_cfg<SCfg<5>>(q, k, v, B, N, H, d, bits, scale_in, out, scale_out, codes_dump, workspace, st);
        default: return launch_selfattn_cfg<SCfg<10>>(q, k, v, B, N, H, d, bits, scale_in, out, scale_out, codes_dump, workspace, st);
    }
}

}  // namespace dgq
