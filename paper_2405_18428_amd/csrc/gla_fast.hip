// fp16 MFMA engine for the output pass of the GLA recurrence in its chunk form, with the work of a chunk split
// between producer and consumer waves (DiG paper, Sec. 3.5: chunks of M = 64 tokens computed on-chip; recurrence
// of Sec. 3.1 Eq. (attn_gla) rows 1-3 with beta = 1; scan orders of Sec. 3.3 / Algorithm 1).
//
// Chunk form with a mid-chunk anchor.  Inside a chunk let b_j = sum_{i<=j} log2 alpha_i (inclusive, per key
// channel), b_m its value after the chunk's 32nd token and b_C after its last.  With
//     q~_j = q_j * 2^(b_j - b_m),   k~_i = k_i * 2^(b_m - b_i),   P = diag(2^b_m) S_0   (S_0 = state entering the chunk)
// unrolling the recurrence gives
//     o_j = sum_{i<=j} (q~_j . k~_i) v_i + q~_j P ,        S_C = diag(2^(b_C - b_m)) (P + K~^T V).
// Anchoring in the middle halves the exponent range of the gated operands, which is what lets them be single
// fp16 numbers (11 significant bits; one v_mfma_f32_16x16x32_f16 per product): as long as a channel decays by at
// most 2^-kMaxHalfDecay over either half of a chunk and the gated operands stay below kMaxOperand, every operand
// keeps fp16's full precision.  A span in which that does not hold raises its flag in the workspace and is
// recomputed by the bf16 hi/lo engine (gla_mfma.hip), which has the exponent range of fp32.
//
// A work-group of 8 waves walks the chunks of one span.  Waves 0..3 are producers, waves 4..7 consumers; wave w
// of either kind owns tokens 16w .. 16w+15 of every chunk.  The stages of a chunk cost about the same time and
// each of them is a chain of dependent instructions, so a wave that ran them one after the other would leave
// the vector, matrix and LDS pipes idle most of the time; with the two kinds of waves on the same SIMD a chunk
// costs the longer of the two halves instead of their sum.
// Producers fetch rows straight into the MFMA operand layout: lane (lm, g) = (lane % 16, lane / 16) holds, for
// token 16w + lm, the channels 16u + 4g .. 16u + 4g + 3 of every 16-channel unit u (16-byte pieces of log_alpha,
// 8-byte pieces of q and k).  Two units are the eight contraction slots of one 32-channel MFMA step.  The gate
// prefix sums are a 4-step DPP scan over the 16 lanes of a row plus the totals of the other waves' tiles,
// exchanged through LDS.  q~, k~ and v (as fp16) go to LDS, token-major, double-buffered.
// Consumers form the score tiles of their 16 tokens (transposed, so that the accumulators are the B operand of the
// next product), the output rows O^T = V^T A^T + P^T Q~^T, and the update of the state tiles they own (fp32 in
// accumulators for the whole span; token-contracted operands come from ds_read_b64_tr_b16), store the rows, and
// publish the state for the next chunk as an fp16 operand.
//
// One barrier per chunk: in iteration c the producers gate chunk c+1 (into the other LDS buffers), scan chunk c+2
// (tile totals into LDS) and issue the loads of log_alpha for chunk c+3 and of q, k, v for chunk c+2, while the
// consumers contract chunk c.
#include <type_traits>

#include "gla_common.h"
#include "gla_mfma_util.h"

namespace gla {
namespace {

typedef __attribute__((ext_vector_type(2))) _Float16 h16x2;
typedef __attribute__((ext_vector_type(4))) _Float16 h16x4;
typedef __attribute__((ext_vector_type(8))) _Float16 h16x8;

constexpr float kMaxHalfDecay = 11.f;    // log2: decay of a channel over half a chunk that the fp16 operands cover
constexpr float kMaxOperand = 16384.f;   // largest |v| taken as safe (fp16 overflows at 65504)
constexpr float kMaxInput = 8.f;         // largest |q|, |k|: times 2^kMaxHalfDecay still below kMaxOperand
constexpr float kMinInput = 0.00390625f; // a span whose largest |q|, |k| or |v| is below 2^-8 would sit in fp16's subnormals

__device__ inline uint32_t pack_f16(float lo, float hi) {
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, h16x2));
}
__device__ inline f32x4 mfma_h32(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h16x8, a), __builtin_bit_cast(h16x8, b), c, 0, 0, 0);
}
// a 16-channel step: the 32-channel MFMA with its upper four contraction slots zero.  (The 16-deep MFMA chained
// onto the accumulator of a 32-deep one gave wrong rows on MI355X with this compiler; one opcode for both.)
__device__ inline f32x4 mfma_h16(u32x2 a, u32x2 b, f32x4 c) {
    return mfma_h32(u32x4{a[0], a[1], 0u, 0u}, u32x4{b[0], b[1], 0u, 0u}, c);
}
// inclusive prefix sum over the 16 lanes of a DPP row
__device__ inline float row_scan16(float v) {
    v += dpp_move<0x111, 0xF, true>(v);  // row_shr:1
    v += dpp_move<0x112, 0xF, true>(v);  // row_shr:2
    v += dpp_move<0x114, 0xF, true>(v);  // row_shr:4
    v += dpp_move<0x118, 0xF, true>(v);  // row_shr:8
    return v;
}

// Four independent inclusive prefix sums over the 16 lanes of each DPP row, their steps interleaved: an
// instruction never reads a register written by one of the three before it, so no wait states are needed between
// the steps (a DPP read needs two after the instruction that wrote its source).  All 64 lanes must be active.
__device__ inline void row_scan16x4(float &a, float &b, float &c, float &d) {
    asm volatile(
        "s_nop 4\n\t"   // wait states a DPP read needs after a vector instruction wrote its source (2) or EXEC (5)
        "v_add_f32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %1, %1, %1 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %2, %2, %2 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %3, %3, %3 row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %1, %1, %1 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %2, %2, %2 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %3, %3, %3 row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %1, %1, %1 row_shr:4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %2, %2, %2 row_shr:4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %3, %3, %3 row_shr:4 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %1, %1, %1 row_shr:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %2, %2, %2 row_shr:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_f32_dpp %3, %3, %3 row_shr:8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1"      // and before whatever reads the results through DPP next
        : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// Head-size classes.  NK32 = 32-channel MFMA steps, TAIL = one more 16-channel step, NCT = 16-channel units
// (= row tiles of the state), NDV16 = 16-column tiles of the values.  Row strides (in 16-bit elements) are chosen so
// that the 8- and 16-byte reads of 16 neighbouring rows spread over the LDS banks.
template <int CLS>
struct FastCfg;
template <>
struct FastCfg<0> {   // dk <= 32, dv <= 64
    static constexpr int NK32 = 1, TAIL = 0, NCT = 2, NDV16 = 4, KST = 48, VS = 80, SST = 40;
    static constexpr int kOwned[4] = {4, 3, 1, 0};
};
template <>
struct FastCfg<1> {   // dk <= 48, dv <= 80
    static constexpr int NK32 = 1, TAIL = 1, NCT = 3, NDV16 = 5, KST = 48, VS = 80, SST = 56;
    static constexpr int kOwned[4] = {6, 5, 2, 2};
};
template <>
struct FastCfg<2> {   // dk <= 64, dv <= 128
    static constexpr int NK32 = 2, TAIL = 0, NCT = 4, NDV16 = 8, KST = 80, VS = 144, SST = 72;
    static constexpr int kOwned[4] = {12, 10, 5, 5};
};

template <int CLS>
struct FastLayout {
    using C = FastCfg<CLS>;
    static constexpr int kTot = 3 * 4 * 4 * (4 * C::NCT) * 4;            // float[3][tile][g][NV]
    static constexpr int kK = kChunk * C::KST * 2;                       // one buffer of k~ (and of q~)
    static constexpr int kV = kChunk * C::VS * 2;                        // one buffer of v
    static constexpr int kS = 16 * C::NDV16 * C::SST * 2;                // one buffer of P (fp16, [value column][slot])
    static constexpr int oTot = 0;
    static constexpr int oFlag = oTot + kTot;                            // int: the span left the fp16 range
    static constexpr int oZero = oFlag + 16;                             // float[g][NV] of zeros (a tile total that is not there)
    // two sets of operand buffers (k~, q~, v, P of one chunk each); chunk x uses set x % 2
    static constexpr int kSet = 2 * kK + kV + kS;
    static constexpr int oK = oZero + 4 * (4 * C::NCT) * 4;
    static constexpr int oQ = oK + kK;
    static constexpr int oV = oQ + kK;
    static constexpr int oS = oV + kV;
    static constexpr int kBytes = oK + 2 * kSet;
    // float[dk * dv] before the first chunk: in the second set, which nothing writes before chunk 1 is gated
    static constexpr int oChain = oK + kSet;
    static_assert(kSet >= 16 * C::NCT * 16 * C::NDV16 * 4, "the chained start state must fit");
    static_assert(kSet % 16 == 0 && kK % 16 == 0 && kV % 16 == 0, "16-byte LDS accesses");
};

template <int CLS>
__host__ __device__ constexpr int owned_start(int w) {
    int s = 0;
    for (int i = 0; i < w; ++i) s += FastCfg<CLS>::kOwned[i];
    return s;
}

constexpr int kFastThreads = 512;    // 4 producer waves + 4 consumer waves

// Last statement of a code path that exists once per consumer wave (W = compile-time wave index).  The paths end in
// the same instructions on different registers of the accumulator arrays; when the compiler merges such tails the
// arrays are addressed through a pointer that depends on the wave and leave the registers for scratch memory.
// A statement that differs between the copies keeps them apart.
#define WAVE_CODE_END(W) asm volatile("; end of the code of consumer wave %0" ::"n"(W))

// STATE: the span-state pass (phase 1 of the span plan): the same producers without q, the consumers only update
// their state tiles from a zero state and leave U_r (anchored at the end of the span) and log Gamma_r in the workspace.
// FUSE: the gates come from their bf16 pre-activations z (Eq. (gate_gla): log alpha = logsigmoid(z) / tau), formed by
// the producers where the plain kernel reads log_alpha: 72 instead of 144 bytes per token-head in either pass.
// (The output epilogue Swish(r) * LN(o) stays with the bf16 hi/lo kernel: the per-token normalisation divides by
// the spread of a row of o, and on rows whose outputs are small the error of the fp16 operands, 3e-3 of the RMS
// over all rows, came out at 2.7e-2 of the RMS of the normalised output at 1024 px, above the 2e-2 bar.)
template <int CLS, typename TOut, int MINW, bool STATE, bool FUSE>
__global__ __launch_bounds__(kFastThreads, MINW) void fast_span_kernel(Params p) {
    using C = FastCfg<CLS>;
    using L = FastLayout<CLS>;
    constexpr int NCT = C::NCT, NDV16 = C::NDV16, NK32 = C::NK32, KST = C::KST, VS = C::VS, SST = C::SST;
    constexpr bool TAIL = C::TAIL != 0;
    constexpr int NV = 4 * NCT;                       // gate values per lane and chunk
    constexpr int NVP = (2 * NDV16 + 3) / 4;          // 16-byte pieces of a v row per lane
    constexpr int SET = L::kSet / 2;                  // 16-bit elements from an operand buffer to its twin in the other set
    static_assert(2 * NK32 + (TAIL ? 1 : 0) == NCT, "units = slots of the MFMA steps");
    static_assert(owned_start<CLS>(4) == NCT * NDV16, "every state tile has an owner");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *s_tot = reinterpret_cast<float *>(smem + L::oTot);
    int *s_flag = reinterpret_cast<int *>(smem + L::oFlag);
    uint16_t *s_k = reinterpret_cast<uint16_t *>(smem + L::oK);
    uint16_t *s_q = reinterpret_cast<uint16_t *>(smem + L::oQ);
    uint16_t *s_v = reinterpret_cast<uint16_t *>(smem + L::oV);
    uint16_t *s_s = reinterpret_cast<uint16_t *>(smem + L::oS);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool consumer = w8 >= 4;                    // wave-uniform
    const int w = w8 & 3;                             // 16-token tile of every chunk
    const int lm = lane & 15;
    const int g = lane >> 4;

    // work-group -> (batch * head, span): contiguous ranges of spans per XCD; odd heads walk their spans
    // backwards when the span states are chained here (long and short chains then share a compute unit)
    int blk = blockIdx.x;
    {
        const int nb = gridDim.x;
        if ((nb & 7) == 0) blk = (blk & 7) * (nb >> 3) + (blk >> 3);
    }
    // spans per (batch, head) that this launch covers: the state pass leaves out the last one when the output
    // pass chains the span states itself (nothing reads that U)
    const int spans_here = (STATE && p.chain_in_output) ? p.nspans - 1 : p.nspans;
    const int bh = blk / spans_here;
    int sp_ = blk - bh * spans_here;
    if (!STATE && p.chain_in_output && (bh & 1)) sp_ = spans_here - 1 - sp_;
    const int sp = sp_;
    const int dk = p.dk, dv = p.dv, T = p.T;
    const int s_begin = sp * p.span_len;
    const int s_end = min(T, s_begin + p.span_len);
    const int nch = (s_end - s_begin + kChunk - 1) / kChunk;
    // only the last chunk of a span can hold rows that are not tokens (their pieces are then cleared)
    const int ragged_from = (s_end - s_begin) % kChunk != 0 ? nch - 1 : nch;

    const size_t base_k = slab_k(p, bh), base_v = slab_v(p, bh);

    if (tid == 0) *s_flag = 0;
    if (tid < 4 * NV) reinterpret_cast<float *>(smem + L::oZero)[tid] = 0.f;

    // Token of this lane's row (16 w + lm) as the wave moves from chunk to chunk.  The token of the next chunk's row
    // follows from the current one by a few additions (64 scan steps further: +-64 in a row scan; in a column scan
    // 64 / grid_h columns and 64 % grid_h rows further, with one wrap); a row past the end of the span stays on the
    // last token it had (loads stay in bounds; such rows are cleared or never stored).
    const int row_s0 = s_begin + 16 * w + lm;              // scan step of the lane's row in chunk 0
    auto row_is_token = [&](int x) { return row_s0 + x * kChunk < s_end; };
    int tok, tok_c = 0, tok_r = 0, walk_s = row_s0;
    {
        int s = min(row_s0, s_end - 1);
        tok = scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w);
        if (p.scan_dir >= 2) {
            if (p.scan_dir & 1) s = T - 1 - s;
            tok_c = s / p.grid_h;
            tok_r = s - tok_c * p.grid_h;
        }
    }
    const int col_dq = kChunk / p.grid_h, col_dr = kChunk - col_dq * p.grid_h;   // (uniform)
    auto next_row_token = [&]() {
        walk_s += kChunk;
        const bool ok = walk_s < s_end;
        if (p.scan_dir < 2) {
            const int t2 = (p.scan_dir & 1) ? tok - kChunk : tok + kChunk;
            tok = ok ? t2 : tok;
        } else {
            int c2, r2;
            if (p.scan_dir & 1) {
                c2 = tok_c - col_dq;
                r2 = tok_r - col_dr;
                if (r2 < 0) { r2 += p.grid_h; c2 -= 1; }
            } else {
                c2 = tok_c + col_dq;
                r2 = tok_r + col_dr;
                if (r2 >= p.grid_h) { r2 -= p.grid_h; c2 += 1; }
            }
            tok_c = ok ? c2 : tok_c;
            tok_r = ok ? r2 : tok_r;
            tok = ok ? r2 * p.grid_w + c2 : tok;
        }
    };

    bool bad = false;     // this lane saw something outside the fp16 range

    // Output pass: the consumers' chain (scores -> AV -> stores) sets the time of an iteration, the producers wait
    // at the barrier with slack; when both have an instruction ready on a SIMD the consumer's goes first.  (The
    // state pass has the shorter consumer side and measured no gain.)
    if (!STATE && consumer) __builtin_amdgcn_s_setprio(2);

    if (!consumer) {
        // =========================== producers ===========================
        const char *gq = static_cast<const char *>(p.q) + base_k * 2;
        const char *gk = static_cast<const char *>(p.k) + base_k * 2;
        const char *gv = static_cast<const char *>(p.v) + base_v * 2;
        // gate rows: fp32 log_alpha, or (FUSE) the bf16 pre-activations z, laid out like q and k
        const char *gla_ = FUSE ? static_cast<const char *>(p.z_gate) + base_k * 2
                                : reinterpret_cast<const char *>(p.log_alpha) + base_k * 4;
        const uint32_t dk2 = 2u * (uint32_t)p.st_k, dv2 = 2u * (uint32_t)p.st_v;   // bytes from one bf16 row to the next

        // unit u: channels 16u + 4g .. +3.  Every load is issued by every lane: a piece past the row repeats the
        // row's last piece (finite values of a real token) and its q, k are cleared on the way to LDS; what the
        // repeated gates and values then feed are channels whose k~ is zero and value columns that are never stored.
        // (only the last unit can reach past dk: dk > 16 (NCT - 1) in this head-size class)
        const uint32_t chb0 = 8u * (uint32_t)g;                                        // byte offset of unit 0's piece in a bf16 row
        const uint32_t chb_last = 2u * (uint32_t)min(16 * (NCT - 1) + 4 * g, dk - 4);  // ... of the last unit's
        const uint32_t mask_last = 16 * (NCT - 1) + 4 * g < dk ? 0xffffffffu : 0u;     // all ones where the last unit's channels exist
        uint32_t vpb[NVP];         // byte offset of the lane's i-th v piece (8 columns) in a bf16 row
#pragma unroll
        for (int i = 0; i < NVP; ++i) vpb[i] = 2u * (uint32_t)min(8 * (g + 4 * i), dv - 8);

        using GatePiece = std::conditional_t<FUSE, u32x2, f32x4>;
        GatePiece r_la[NCT];       // log_alpha (or z) pieces waiting for the scan
        float r_b[NV];             // scanned gates (log2, prefix inside the 16-token tile) waiting for the gate stage
        u32x2 r_q[NCT], r_k[NCT];  // raw q, k pieces waiting for the gate stage
        u32x4 r_v[NVP];            // v pieces on their way to LDS
        // fp16 range check of the span: largest half-chunk decay (log2), largest |q|, |k|, |v|
        float trk_q = 0.f, trk_k = 0.f, trk_v = 0.f;

        // the rows of the walker's current token
        auto issue_la = [&](GatePiece (&dst)[NCT]) {
            if constexpr (FUSE) {
                const uint32_t off = (uint32_t)tok * dk2 + chb0;
#pragma unroll
                for (int u = 0; u < NCT - 1; ++u) dst[u] = *reinterpret_cast<const u32x2 *>(gla_ + off + 32u * u);
                dst[NCT - 1] = *reinterpret_cast<const u32x2 *>(gla_ + (uint32_t)tok * dk2 + chb_last);
            } else {
                const uint32_t off = 2u * ((uint32_t)tok * dk2 + chb0);
#pragma unroll
                for (int u = 0; u < NCT - 1; ++u) dst[u] = *reinterpret_cast<const f32x4 *>(gla_ + off + 64u * u);
                dst[NCT - 1] = *reinterpret_cast<const f32x4 *>(gla_ + 2u * ((uint32_t)tok * dk2 + chb_last));
            }
        };
        auto issue_qk = [&](int tk) {
            const uint32_t off = (uint32_t)tk * dk2 + chb0;
#pragma unroll
            for (int u = 0; u < NCT - 1; ++u) {
                if constexpr (!STATE) r_q[u] = *reinterpret_cast<const u32x2 *>(gq + off + 32u * u);
                r_k[u] = *reinterpret_cast<const u32x2 *>(gk + off + 32u * u);
            }
            if constexpr (!STATE) r_q[NCT - 1] = *reinterpret_cast<const u32x2 *>(gq + (uint32_t)tk * dk2 + chb_last);
            r_k[NCT - 1] = *reinterpret_cast<const u32x2 *>(gk + (uint32_t)tk * dk2 + chb_last);
        };
        auto issue_v = [&](int tk) {   // (rows past the span keep the values of its last token: their k~ is zero)
#pragma unroll
            for (int i = 0; i < NVP; ++i) r_v[i] = *reinterpret_cast<const u32x4 *>(gv + (uint32_t)tk * dv2 + vpb[i]);
        };

        // scan: prefix sums of log2(alpha) inside this wave's tile, tile totals to LDS
        auto scan = [&](int x) {
            float *tot = s_tot + ((x % 3) * 4 + w) * 4 * NV + g * NV;
            if constexpr (FUSE) {
                // log2(alpha) = log2(sigmoid(z)) / tau = (min(t, 0) - log2(1 + 2^-|t|)) / tau with t = z log2(e)
                auto gate2 = [&](uint32_t pair, float &lo, float &hi) {
                    const float t0 = bf16_lo_as_float(pair) * kLog2e, t1 = bf16_hi_as_float(pair) * kLog2e;
                    lo = (fminf(t0, 0.f) - __builtin_amdgcn_logf(1.f + exp2_fast(-fabsf(t0)))) * p.inv_tau;
                    hi = (fminf(t1, 0.f) - __builtin_amdgcn_logf(1.f + exp2_fast(-fabsf(t1)))) * p.inv_tau;
                };
#pragma unroll
                for (int u = 0; u < NCT; ++u) {
                    gate2(r_la[u][0], r_b[4 * u], r_b[4 * u + 1]);
                    gate2(r_la[u][1], r_b[4 * u + 2], r_b[4 * u + 3]);
                }
            } else {
#pragma unroll
                for (int u = 0; u < NCT; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) r_b[4 * u + e] = r_la[u][e] * kLog2e;
            }
            if (x >= ragged_from) {
                const bool valid = row_is_token(x);
#pragma unroll
                for (int i = 0; i < NV; ++i) r_b[i] = valid ? r_b[i] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < NCT; ++u) row_scan16x4(r_b[4 * u], r_b[4 * u + 1], r_b[4 * u + 2], r_b[4 * u + 3]);
            if (lm == 15) {
#pragma unroll
                for (int u = 0; u < NCT; ++u)
                    *reinterpret_cast<f32x4 *>(tot + 4 * u) = f32x4{r_b[4 * u], r_b[4 * u + 1], r_b[4 * u + 2], r_b[4 * u + 3]};
            }
        };

        // gate: exponents relative to the mid-chunk anchor; q~ and k~ to LDS.
        // The prefix sums of this wave's tile are offset by sums of tile totals t0..t2: tiles 0, 1 lie before the anchor
        // (-(t0 + t1), -t1), tile 2 starts at it (0), tile 3 follows tile 2 (+t2): sign * (A + B) with A, B a tile's
        // totals or the row of zeros.  Nothing is clamped: an exponent outside the fp16 range gives non-finite
        // operands and outputs, and the span is then flagged and recomputed.
        const int tile_a = w == 0 ? 0 : -1, tile_b = w <= 1 ? 1 : (w == 3 ? 2 : -1);
        const float off_sign = w == 3 ? 1.f : -1.f;
        const float *s_zero = reinterpret_cast<const float *>(smem + L::oZero) + g * NV;
        auto gate = [&](int x) {
            const float *tot = s_tot + (x % 3) * 16 * NV + g * NV;      // + tile * 4 * NV
            const float *pa = tile_a >= 0 ? tot + tile_a * 4 * NV : s_zero;
            const float *pb = tile_b >= 0 ? tot + tile_b * 4 * NV : s_zero;
            uint16_t *krow = s_k + (x & 1) * SET + (16 * w + lm) * KST + 4 * g;
            uint16_t *qrow = s_q + (x & 1) * SET + (16 * w + lm) * KST + 4 * g;
            uint32_t keep_last = mask_last, keep = 0xffffffffu;
            const bool ragged = x >= ragged_from;       // (uniform)
            if (ragged) {
                const bool valid = row_is_token(x);
                keep = valid ? keep : 0u;
                keep_last = valid ? keep_last : 0u;
            }
#pragma unroll
            for (int u = 0; u < NCT; ++u) {
                const f32x4 ta = *reinterpret_cast<const f32x4 *>(pa + 4 * u);
                const f32x4 tb = *reinterpret_cast<const f32x4 *>(pb + 4 * u);
                uint32_t q0 = 0u, q1 = 0u, k0 = r_k[u][0], k1 = r_k[u][1];
                if constexpr (!STATE) {
                    q0 = r_q[u][0];
                    q1 = r_q[u][1];
                }
                if (u == NCT - 1) {
                    q0 &= keep_last; q1 &= keep_last; k0 &= keep_last; k1 &= keep_last;
                } else if (ragged) {
                    q0 &= keep; q1 &= keep; k0 &= keep; k1 &= keep;
                }
                float qx[4], kx[4];
                qx[0] = bf16_lo_as_float(q0); qx[1] = bf16_hi_as_float(q0); qx[2] = bf16_lo_as_float(q1); qx[3] = bf16_hi_as_float(q1);
                kx[0] = bf16_lo_as_float(k0); kx[1] = bf16_hi_as_float(k0); kx[2] = bf16_lo_as_float(k1); kx[3] = bf16_hi_as_float(k1);
                if constexpr (!STATE) {
                    trk_q = fmaxf(fmaxf(trk_q, fabsf(qx[0])), fabsf(qx[1]));
                    trk_q = fmaxf(fmaxf(trk_q, fabsf(qx[2])), fabsf(qx[3]));
                }
                trk_k = fmaxf(fmaxf(trk_k, fabsf(kx[0])), fabsf(kx[1]));
                trk_k = fmaxf(fmaxf(trk_k, fabsf(kx[2])), fabsf(kx[3]));
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float ex = fmaf(off_sign, ta[e] + tb[e], r_b[4 * u + e]);
                    if constexpr (!STATE) qx[e] *= exp2_fast(ex);
                    kx[e] *= exp2_fast(-ex);
                }
                if constexpr (!STATE)
                    *reinterpret_cast<u32x2 *>(qrow + 16 * u) = u32x2{pack_f16(qx[0], qx[1]), pack_f16(qx[2], qx[3])};
                *reinterpret_cast<u32x2 *>(krow + 16 * u) = u32x2{pack_f16(kx[0], kx[1]), pack_f16(kx[2], kx[3])};
            }
        };

        // v rows of chunk x: bf16 -> fp16 (exact inside fp16's range), to LDS
        auto park_v = [&](int x) {
            uint16_t *vrow = s_v + (x & 1) * SET + (16 * w + lm) * VS + 8 * g;
#pragma unroll
            for (int i = 0; i < NVP; ++i) {
                if (8 * (g + 4 * i) < 16 * NDV16) {
                    u32x4 h;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t x2 = r_v[i][j];
                        const float lo = bf16_lo_as_float(x2), hi = bf16_hi_as_float(x2);
                        trk_v = fmaxf(fmaxf(trk_v, fabsf(lo)), fabsf(hi));
                        h[j] = pack_f16(lo, hi);
                    }
                    *reinterpret_cast<u32x4 *>(vrow + 32 * i) = h;
                }
            }
        };

        // ---- the producers' loop ----
        // Iteration c runs beside the consumers' contraction of chunk c: gate and park chunk c + 1, scan chunk
        // c + 2, and refill the registers just read with the rows of chunks c + 2 (q, k, v) and c + 3 (log_alpha):
        // every load is issued as soon as the registers it fills have been read, one iteration before the stage
        // that reads them.
        // Filling the pipeline: everything the first stages need (log_alpha of chunks 0 and 1; q, k, v of chunk 0)
        // is requested at once, so the fill costs one trip to memory; chunk 0 is scanned, and after the barrier
        // that makes its tile totals visible the loop starts with iteration -1.  The loop is entered with no load
        // in flight, so the counts of younger loads that the waits inside it allow are those of the steady state.
        {
            // (requested in the order the loop leaves its loads in at the end of an iteration - q and k, the gates of
            // the chunk after, v: the compiler merges the two states at the loop's entry, and a gate row that
            // looked younger than a v row there would make every scan of the loop wait for the v rows requested
            // just before it)
            GatePiece la1[NCT];
            const int tok0 = tok;
            issue_la(r_la);
            issue_qk(tok0);
            next_row_token();
            issue_la(la1);
            issue_v(tok0);
            if constexpr (!STATE) {
                // with those loads in flight, the producers' half of the span-state chain
                if (p.chain_in_output && (sp > 0 || p.initial_state != nullptr)) {   // uniform
                    constexpr int kV4 = (16 * NCT * 16 * NDV16 / 4 + kFastThreads - 1) / kFastThreads;
                    constexpr int kRun = 8 / kV4 > 0 ? 8 / kV4 : 1;
                    chain_span_states<kFastThreads, kV4, kRun, false>(p, bh, sp, tid, reinterpret_cast<float *>(smem + L::oChain));
                }
            }
            scan(0);
#pragma unroll
            for (int u = 0; u < NCT; ++u) r_la[u] = la1[u];
        }
        __syncthreads();                    // tile totals of chunk 0 (and, for the consumers, the chained state)
        for (int c = -1; c < nch; ++c) {
            if (c + 1 < nch) gate(c + 1);
            const int tok_qkv = tok;        // token of chunk c + 2
            issue_qk(tok_qkv);
            if (c + 2 < nch) scan(c + 2);
            next_row_token();
            issue_la(r_la);                 // chunk c + 3
            if (c + 1 < nch) park_v(c + 1);
            issue_v(tok_qkv);
            __syncthreads();
        }

        // Outside the range: inputs so large or so small that the gated operands (within 2^kMaxHalfDecay of them)
        // overflow or lose their leading bits.  (Comparisons are written so that NaN fails them.)
        bad = !(trk_k <= kMaxInput) || !(trk_v <= kMaxOperand) || !(trk_k >= kMinInput) || !(trk_v >= kMinInput);
        if constexpr (!STATE) bad = bad || !(trk_q <= kMaxInput) || !(trk_q >= kMinInput);
    } else {
        // =========================== consumers ===========================
        char *gout = static_cast<char *>(p.out) + base_v * sizeof(TOut);
        float trk_o = 0.f;         // largest |output| (a non-finite one: an operand overflowed after all)
        float trk_e = 0.f;         // largest decay of a channel over half a chunk (log2)
        static_assert(C::kOwned[0] >= NCT, "consumer wave 0 owns a tile of every channel unit");
        f32x4 lg_sum[NCT];         // STATE, consumer wave 0: log2 of the span's total decay, channels 16 ct + 4 g + r
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) lg_sum[ct] = f32x4{0.f, 0.f, 0.f, 0.f};

        // ---- state tiles owned by this wave ----
        constexpr int MAXOWN = C::kOwned[0];
        f32x4 acc[MAXOWN];
#pragma unroll
        for (int i = 0; i < MAXOWN; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

        // ---- state entering the span ----
        if constexpr (!STATE) {
            const bool chain = p.chain_in_output && (sp > 0 || p.initial_state != nullptr);   // uniform
            const float *s0 = nullptr;
            if (p.nspans > 1 && !p.chain_in_output)
                s0 = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;      // as the carry kernel left it
            else if (p.nspans == 1 && p.initial_state != nullptr)
                s0 = p.initial_state + (size_t)bh * dk * dv;
            if (chain) {
                // (the producers do their half once the loads that fill the pipeline are on their way)
                constexpr int kV4 = (16 * NCT * 16 * NDV16 / 4 + kFastThreads - 1) / kFastThreads;
                constexpr int kRun = 8 / kV4 > 0 ? 8 / kV4 : 1;
                chain_span_states<kFastThreads, kV4, kRun, false>(p, bh, sp, tid, reinterpret_cast<float *>(smem + L::oChain));
                s0 = reinterpret_cast<const float *>(smem + L::oChain);      // (LDS is addressable through flat loads)
            }
            __syncthreads();               // the chained state is in LDS; so are the tile totals of chunk 0
            if (s0 != nullptr) {
                auto fetch = [&](auto wave_c) {
                    constexpr int W = decltype(wave_c)::value;
#pragma unroll
                    for (int i = 0; i < C::kOwned[W]; ++i) {
                        const int t = owned_start<CLS>(W) + i;
                        const int n = 16 * (t / NCT) + lm;
                        float x[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int c = 16 * (t % NCT) + 4 * g + r;
                            x[r] = (c < dk && n < dv) ? s0[min(c, dk - 1) * dv + min(n, dv - 1)] : 0.f;
                        }
                        acc[i] = f32x4{x[0], x[1], x[2], x[3]};
                    }
                };
                switch (w) {
                case 0: fetch(std::integral_constant<int, 0>{}); break;
                case 1: fetch(std::integral_constant<int, 1>{}); break;
                case 2: fetch(std::integral_constant<int, 2>{}); break;
                default: fetch(std::integral_constant<int, 3>{}); break;
                }
            }
        }

        // Owner step after chunk c (c = -1: before the first chunk): the tiles now hold P(c) + K~^T V; scale them by
        // 2^(b_C(c) - b_m(c) + b_m(c+1)) (anchor to anchor) and publish P(c+1) as the fp16 A operand of q~ P.
        auto publish = [&](auto wave_c, int c) {
            constexpr int W = decltype(wave_c)::value;
            constexpr int t_lo = owned_start<CLS>(W), t_hi = owned_start<CLS>(W + 1);
            const float *t_c = s_tot + ((c + 3) % 3) * 16 * NV + g * NV;        // totals of chunk c (c = -1: unused)
            const float *t_n = s_tot + ((c + 1) % 3) * 16 * NV + g * NV;        // totals of chunk c + 1
            uint16_t *srow = s_s + ((c + 1) & 1) * SET;
            (void)srow;
            f32x4 fac[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                bool used = false;
                for (int t = t_lo; t < t_hi; ++t) used = used || (t % NCT == ct);
                if (used) {
                    // second half of chunk c, first half of chunk c + 1 (the gates are <= 0, so the prefix sums are
                    // monotone and the halves' totals bound every exponent of the gated operands)
                    f32x4 h1 = f32x4{0.f, 0.f, 0.f, 0.f}, h0 = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (c >= 0)
                        h1 = *reinterpret_cast<const f32x4 *>(t_c + 2 * 4 * NV + 4 * ct) +
                             *reinterpret_cast<const f32x4 *>(t_c + 3 * 4 * NV + 4 * ct);
                    if (c + 1 < nch)
                        h0 = *reinterpret_cast<const f32x4 *>(t_n + 0 * 4 * NV + 4 * ct) +
                             *reinterpret_cast<const f32x4 *>(t_n + 1 * 4 * NV + 4 * ct);
#pragma unroll
                    for (int r = 0; r < 4; ++r) trk_e = fmaxf(fmaxf(trk_e, fabsf(h1[r])), fabsf(h0[r]));
                    // (whole-vector assignments: element-wise stores into these arrays keep them out of registers
                    // once the compiler merges the tails of the four wave-specific copies of this code)
                    const f32x4 hs = h1 + h0;
                    fac[ct] = f32x4{exp2_fast(hs[0]), exp2_fast(hs[1]), exp2_fast(hs[2]), exp2_fast(hs[3])};
                    if constexpr (STATE && W == 0) lg_sum[ct] = lg_sum[ct] + hs;   // over the span: log2 Gamma
                }
            }
#pragma unroll
            for (int i = 0; i < t_hi - t_lo; ++i) {
                const int t = t_lo + i;
                const int ct = t % NCT, nt = t / NCT;
                acc[i] = acc[i] * fac[ct];
                // slot of channel 16 ct + 4 g + r in a row of P: the 32-channel steps interleave two units per lane group
                if constexpr (!STATE) {
                    const int pos = (ct < 2 * NK32) ? 32 * (ct >> 1) + 8 * g + 4 * (ct & 1) : 32 * NK32 + 4 * g;
                    *reinterpret_cast<u32x2 *>(srow + (16 * nt + lm) * SST + pos) =
                        u32x2{pack_f16(acc[i][0], acc[i][1]), pack_f16(acc[i][2], acc[i][3])};
                } else {
                    (void)nt;
                }
            }
            WAVE_CODE_END(W);
        };

        const int tr_row = lm >> 2, tr_col = 4 * (lm & 3);   // transposing reads: token-in-4 and column quad of this lane

        auto contract = [&](auto wave_c, int c) {
            constexpr int W = decltype(wave_c)::value;
            constexpr int NQ = W / 2 + 1;                     // 32-token steps that hold causal tokens for this wave
            const uint16_t *kb = s_k + (c & 1) * SET;
            const uint16_t *vb = s_v + (c & 1) * SET;
            const uint16_t *sb = s_s + (c & 1) * SET;
            // ---- q~ of this wave's tokens: the B operand of the score tiles and of q~ P ----
            uint32_t qf[NCT][2];
            if constexpr (!STATE) {
                const uint16_t *qrow = s_q + (c & 1) * SET + (16 * W + lm) * KST + 4 * g;
#pragma unroll
                for (int u = 0; u < NCT; ++u) {
                    const u32x2 x = *reinterpret_cast<const u32x2 *>(qrow + 16 * u);
                    qf[u][0] = x[0];
                    qf[u][1] = x[1];
                }
            }
            // ---- score tiles, transposed: lane (lm, g) gets A[i = 16 W + lm][j = 16 jt + 4 g + r] ----
            f32x4 d[W + 1];
#pragma unroll
            for (int jt = 0; jt <= (STATE ? -1 : W); ++jt) {
                const uint16_t *krow = kb + (16 * jt + lm) * KST + 4 * g;
                d[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < NK32; ++ks) {
                    const u32x2 a0 = *reinterpret_cast<const u32x2 *>(krow + 32 * ks);
                    const u32x2 a1 = *reinterpret_cast<const u32x2 *>(krow + 32 * ks + 16);
                    d[jt] = mfma_h32(u32x4{a0[0], a0[1], a1[0], a1[1]},
                                     u32x4{qf[2 * ks][0], qf[2 * ks][1], qf[2 * ks + 1][0], qf[2 * ks + 1][1]},
                                     d[jt]);
                }
                if constexpr (TAIL) {
                    const u32x2 a = *reinterpret_cast<const u32x2 *>(krow + 32 * NK32);
                    d[jt] = mfma_h16(a, u32x2{qf[2 * NK32][0], qf[2 * NK32][1]}, d[jt]);
                }
            }
            if constexpr (!STATE) {
                // causal mask of the diagonal tile
                d[W] = f32x4{4 * g + 0 > lm ? 0.f : d[W][0], 4 * g + 1 > lm ? 0.f : d[W][1],
                             4 * g + 2 > lm ? 0.f : d[W][2], 4 * g + 3 > lm ? 0.f : d[W][3]};
            }
            u32x4 pa[NQ];                                     // A^T as the B operand of O^T += V^T A^T
#pragma unroll
            for (int q32 = 0; q32 < (STATE ? 0 : NQ); ++q32) {
                uint32_t hi0 = 0u, hi1 = 0u;
                if (2 * q32 + 1 <= W) {
                    hi0 = pack_f16(d[2 * q32 + 1][0], d[2 * q32 + 1][1]);
                    hi1 = pack_f16(d[2 * q32 + 1][2], d[2 * q32 + 1][3]);
                }
                pa[q32] = u32x4{pack_f16(d[2 * q32][0], d[2 * q32][1]), pack_f16(d[2 * q32][2], d[2 * q32][3]), hi0, hi1};
            }
            // ---- v fragments (contraction slot (g, e) of step q32 = token 32 q32 + 16 (e / 4) + 4 g + e % 4) ----
            const uint16_t *vrow = vb + (4 * g + tr_row) * VS + tr_col;
            auto v_frag = [&](int q32, int x) {
                const u32x2 lo = lds_read_tr(vrow + 32 * q32 * VS + 16 * x);
                const u32x2 hi = lds_read_tr(vrow + (32 * q32 + 16) * VS + 16 * x);
                return u32x4{lo[0], lo[1], hi[0], hi[1]};
            };
            // the fragments of the value-column tiles whose state tiles this wave owns are kept for the state update
            constexpr int t_lo = owned_start<CLS>(W), t_hi = owned_start<CLS>(W + 1);
            constexpr int NT_LO = t_lo / NCT, NT_HI = t_lo < t_hi ? (t_hi - 1) / NCT : NT_LO - 1;
            constexpr int NOWN = NT_HI - NT_LO + 1;
            u32x4 vown[2][NOWN > 0 ? NOWN : 1];
            // ---- O^T = V^T A^T + P^T Q~^T : lane (lm, g) accumulates O[i = 16 W + lm][n = 16 x + 4 g + r] ----
            f32x4 o[NDV16];
#pragma unroll
            for (int x = 0; x < NDV16; ++x) {
                o[x] = f32x4{0.f, 0.f, 0.f, 0.f};
                const bool owned_col = x >= NT_LO && x <= NT_HI;
#pragma unroll
                for (int q32 = 0; q32 < 2; ++q32) {
                    if ((!STATE && q32 < NQ) || owned_col) {
                        const u32x4 vf = v_frag(q32, x);
                        if constexpr (!STATE) {
                            if (q32 < NQ) o[x] = mfma_h32(vf, pa[q32], o[x]);
                        }
                        if (owned_col) vown[q32][owned_col ? x - NT_LO : 0] = vf;
                    }
                }
                if constexpr (!STATE) {
                    const uint16_t *srow = sb + (16 * x + lm) * SST;
#pragma unroll
                    for (int ks = 0; ks < NK32; ++ks) {
                        const u32x4 st = *reinterpret_cast<const u32x4 *>(srow + 32 * ks + 8 * g);
                        o[x] = mfma_h32(st, u32x4{qf[2 * ks][0], qf[2 * ks][1], qf[2 * ks + 1][0], qf[2 * ks + 1][1]},
                                        o[x]);
                    }
                    if constexpr (TAIL) {
                        const u32x2 st = *reinterpret_cast<const u32x2 *>(srow + 32 * NK32 + 4 * g);
                        o[x] = mfma_h16(st, u32x2{qf[2 * NK32][0], qf[2 * NK32][1]}, o[x]);
                    }
                }
            }
#pragma unroll
            for (int x = 0; x < (STATE ? 0 : NDV16); x += 2) {
                trk_o = fmaxf(fmaxf(trk_o, fabsf(o[x][0])), fabsf(o[x][1]));
                trk_o = fmaxf(fmaxf(trk_o, fabsf(o[x][2])), fabsf(o[x][3]));
                if (x + 1 < NDV16) {
                    trk_o = fmaxf(fmaxf(trk_o, fabsf(o[x + 1][0])), fabsf(o[x + 1][1]));
                    trk_o = fmaxf(fmaxf(trk_o, fabsf(o[x + 1][2])), fabsf(o[x + 1][3]));
                }
            }
            if (!STATE && (c < ragged_from || row_is_token(c))) {
                char *orow = gout + ((uint32_t)tok * (uint32_t)p.st_v + 4u * (uint32_t)g) * (uint32_t)sizeof(TOut);
#pragma unroll
                for (int x = 0; x < NDV16; ++x) {
                    if (4 * g + 16 * x < dv) {    // dv is a multiple of 8: all four columns or none
                        if constexpr (sizeof(TOut) == 4)
                            *reinterpret_cast<f32x4 *>(orow + 64 * x) = o[x];
                        else
                            *reinterpret_cast<u32x2 *>(orow + 32 * x) =
                                u32x2{pack_bf16(o[x][0], o[x][1]), pack_bf16(o[x][2], o[x][3])};
                    }
                }
            }
            // ---- state tiles of this wave: P + K~^T V ----
            if constexpr (t_lo < t_hi) {
                const uint16_t *ktr = kb + (4 * g + tr_row) * KST + tr_col;
                u32x4 kt[NCT][2];
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    bool used = false;
                    for (int t = t_lo; t < t_hi; ++t) used = used || (t % NCT == ct);
                    if (used) {
#pragma unroll
                        for (int q32 = 0; q32 < 2; ++q32) {
                            const u32x2 lo = lds_read_tr(ktr + 32 * q32 * KST + 16 * ct);
                            const u32x2 hi = lds_read_tr(ktr + (32 * q32 + 16) * KST + 16 * ct);
                            kt[ct][q32] = u32x4{lo[0], lo[1], hi[0], hi[1]};
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < t_hi - t_lo; ++i) {
                    const int t = t_lo + i;
                    acc[i] = mfma_h32(kt[t % NCT][0], vown[0][t / NCT - NT_LO], acc[i]);
                    acc[i] = mfma_h32(kt[t % NCT][1], vown[1][t / NCT - NT_LO], acc[i]);
                }
            }
            WAVE_CODE_END(W);
        };

        auto per_wave = [&](auto fn, int c) {
            switch (w) {
            case 0: fn(std::integral_constant<int, 0>{}, c); break;
            case 1: fn(std::integral_constant<int, 1>{}, c); break;
            case 2: fn(std::integral_constant<int, 2>{}, c); break;
            default: fn(std::integral_constant<int, 3>{}, c); break;
            }
        };

        if constexpr (STATE) __syncthreads();   // the tile totals of chunk 0 are in LDS
        per_wave(publish, -1);
        __syncthreads();

        for (int c = 0; c < nch; ++c) {
            per_wave(contract, c);
            per_wave(publish, c);
            if constexpr (!STATE) next_row_token();
            __syncthreads();
        }

        // a half-chunk decay beyond what fp16's exponent covers around the anchor, or a non-finite output / state
        if constexpr (STATE) {
#pragma unroll
            for (int i = 0; i < MAXOWN; ++i) {
                trk_o = fmaxf(fmaxf(trk_o, fabsf(acc[i][0])), fabsf(acc[i][1]));
                trk_o = fmaxf(fmaxf(trk_o, fabsf(acc[i][2])), fabsf(acc[i][3]));
            }
        }
        bad = !(trk_e <= kMaxHalfDecay) || !(trk_o <= 3.0e38f);

        float *dst = nullptr;
        if constexpr (STATE) {
            dst = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;      // U of the span (the last chunk's publish anchored it at the span's end)
            if (w == 0 && lm == 0) {                                         // the workspace keeps natural logarithms
                float *lg = p.ws_lgam + ((size_t)bh * p.nspans + sp) * dk;
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (16 * ct + 4 * g + r < dk) lg[16 * ct + 4 * g + r] = lg_sum[ct][r] * kLn2;
            }
        } else if ((p.nspans == 1 || p.chain_in_output) && sp == p.nspans - 1 && p.final_state != nullptr) {
            dst = p.final_state + (size_t)bh * dk * dv;
        }
        if (dst != nullptr) {
            auto put = [&](auto wave_c, int) {
                constexpr int W = decltype(wave_c)::value;
#pragma unroll
                for (int i = 0; i < C::kOwned[W]; ++i) {
                    const int t = owned_start<CLS>(W) + i;
                    const int n = 16 * (t / NCT) + lm;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int cch = 16 * (t % NCT) + 4 * g + r;
                        if (cch < dk && n < dv) dst[cch * dv + n] = acc[i][r];
                    }
                }
            };
            per_wave(put, 0);
        }
    }

    // ---- fp16 range flag of the span ----
    // (the state pass runs first and leaves out the last span of a head whose states the output pass chains)
    if (__any(bad) && lane == 0) atomicOr(s_flag, 1);
    __syncthreads();
    if (tid == 0) {
        int *flag = p.ws_fail + (size_t)bh * p.nspans + sp;
        if constexpr (STATE) {
            *flag = *s_flag;
            if (spans_here < p.nspans && sp == 0) p.ws_fail[(size_t)bh * p.nspans + p.nspans - 1] = 0;
        } else {
            *flag = *s_flag | (p.nspans > 1 ? *flag : 0);
        }
    }
}

template <int CLS, typename TOut, bool STATE, bool FUSE>
hipError_t launch_cls(const Params &p, hipStream_t stream) {
    using L = FastLayout<CLS>;
    constexpr int kGroupsPerCu = (160 * 1024) / L::kBytes;
    constexpr int MINW = kGroupsPerCu >= 2 ? 4 : 2;    // waves per SIMD: two resident groups of 8 waves, or one
    auto kernel = fast_span_kernel<CLS, TOut, MINW, STATE, FUSE>;
    static std::atomic<bool> configured[kMaxDevices] = {};
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), L::kBytes, configured);
    if (e != hipSuccess) return e;
    const int spans = (STATE && p.chain_in_output) ? p.nspans - 1 : p.nspans;
    if (spans <= 0) return hipSuccess;
    dim3 grid((unsigned)(p.B * p.H * spans)), block(kFastThreads);
    hipLaunchKernelGGL(kernel, grid, block, L::kBytes, stream, p);
    return hipGetLastError();
}

}  // namespace

// head-size class of a call, or -1: the producers fetch whole 16-channel units and clear only the last one's
// channels past dk, so the class must have exactly ceil(dk / 16) units
static int fast_class(const Params &p) {
    const int ndk16 = (p.dk + 15) / 16, ndv16 = (p.dv + 15) / 16;
    if (ndk16 == 2 && ndv16 <= 4) return 0;
    if (ndk16 == 3 && ndv16 <= 5) return 1;
    if (ndk16 == 4 && ndv16 <= 8) return 2;
    return -1;
}

bool fast_engine_supports(const Params &p) {
    if (!mfma_engine_supports(p) || fast_class(p) < 0) return false;
    // key-side recurrence, gates read or formed from their pre-activations: no output epilogue, no value-side gate,
    // no accumulation, no gate shift
    return !two_sided(p) && p.r_pre == nullptr && !p.accumulate && p.gate_shift == 0;
}

int fast_groups_per_cu(const Params &p) {
    switch (fast_class(p)) {
    case 0: return (160 * 1024) / FastLayout<0>::kBytes >= 2 ? 2 : 1;
    case 1: return (160 * 1024) / FastLayout<1>::kBytes >= 2 ? 2 : 1;
    default: return (160 * 1024) / FastLayout<2>::kBytes >= 2 ? 2 : 1;
    }
}

template <bool FUSE>
static hipError_t launch_output(const Params &p, hipStream_t stream) {
    const bool bf16_out = p.out_dtype == GLA_DT_BF16;
    switch (fast_class(p)) {
    case 0: return bf16_out ? launch_cls<0, uint16_t, false, FUSE>(p, stream) : launch_cls<0, float, false, FUSE>(p, stream);
    case 1: return bf16_out ? launch_cls<1, uint16_t, false, FUSE>(p, stream) : launch_cls<1, float, false, FUSE>(p, stream);
    case 2: return bf16_out ? launch_cls<2, uint16_t, false, FUSE>(p, stream) : launch_cls<2, float, false, FUSE>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fast_output(const Params &p, hipStream_t stream) {
    return p.z_gate != nullptr ? launch_output<true>(p, stream) : launch_output<false>(p, stream);
}

template <bool FUSE>
static hipError_t launch_state(const Params &p, hipStream_t stream) {
    switch (fast_class(p)) {
    case 0: return launch_cls<0, float, true, FUSE>(p, stream);
    case 1: return launch_cls<1, float, true, FUSE>(p, stream);
    case 2: return launch_cls<2, float, true, FUSE>(p, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_fast_state(const Params &p, hipStream_t stream) {
    return p.z_gate != nullptr ? launch_state<true>(p, stream) : launch_state<false>(p, stream);
}

}  // namespace gla
