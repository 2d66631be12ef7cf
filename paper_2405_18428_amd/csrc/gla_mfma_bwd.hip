// bf16 MFMA kernel for the state reads of the backward pass of the GLA recurrence
// (DiG paper, Sec. 3.1 Eq. (attn_gla) rows 1-3 with beta = 1, differentiated; chunks of M = 64
// tokens computed on-chip as in Sec. 3.5).
//
// It computes r_s[c] = sum_n S_s[c,n] w_s[n] for every scan step s of a span, where S follows
// S_s = diag(alpha_s) S_{s-1} + k_s^T v_s: with w = dO this is dq, and on the reversed recurrence
// of G = dL/dS (k, v := q, dO, gates shifted by one step) with w = v it is dk.
//
// Chunk form.  With b_j the inclusive sum of log_alpha inside the chunk (per key channel),
// k~_j = k_j exp(-b_j), E_j = exp(b_j) and S_0 the state entering the chunk,
//     S_j = diag(E_j) (S_0 + sum_{i<=j} k~_i^T v_i)
//     r_j = E_j * ( sum_{i<=j} (w_j . v_i) k~_i  +  S_0 w_j )          ("*" elementwise over channels)
//     S_C = diag(E_C) (S_0 + K~^T V)
// i.e. per chunk  P = tril(W V^T)  (plain bf16 operands, contraction over the value columns),
// R = E * (P K~ + W S_0^T),  S += K~^T V then scaled.  P, K~ and S_0 are split into a bf16 "hi" part
// and a bf16 "lo" remainder (three products where two split operands meet, two otherwise).
//
// One work-group of 4 waves walks the chunks of its span; wave i owns the 16 tokens 16i..16i+15 of a
// chunk (all channels of R) and the state tiles of the value-column tiles i, i+4.  The state is kept
// transposed, S^T[n][c], in fp32 accumulators: a lane then holds four consecutive value columns of one
// channel, which is (a) a 16-byte load from the [dk][dv] state the carry kernel left in the workspace,
// (b) an 8-byte LDS write of the bf16 parts as the channel-major rows that the S_0 term reads as its A
// operand, and (c) scaled by one exp(b_C) per lane.
// P is computed transposed (as in the forward kernel) so that its accumulator registers are the B
// operand of the next contraction: slot (g, e) of a 32-token step is token 32q + 16(e/4) + 4g + e%4,
// and K~ (contracted over tokens) is fetched in the same order by the transposing LDS read.
#include <type_traits>

#include "gla_common.h"
#include "gla_mfma_util.h"

namespace gla {
namespace {

template <int NDK8, int NDV16, bool DV, bool BETA = false>
struct RLayout {
    static constexpr int kDkp = NDK8 * 8;
    static constexpr int kDvp = NDV16 * 16;
    static constexpr int kNct = (NDK8 + 1) / 2;                           // 16-channel tiles
    // bf16 per row of K~: whole 16-channel tiles, an odd number of 16-byte units
    static constexpr int kChStride = (NDK8 % 4 == 0) ? kDkp + 8 : ((kDkp + 8 + 15) / 16) * 16 + 8;
    // bf16 per row of V, W and S_0: the columns, then an all-zero group of 8 (lanes whose column group lies
    // beyond the last one read that group); again an odd number of 16-byte units
    static constexpr int kVStride = kDvp + 8;
    static constexpr int kZeroCol = kDvp;
    static constexpr int kLaStride = kDkp + 4;                            // fp32 per row of log_alpha, then E
    static constexpr int kRowK = kChunk * kChStride * 2;
    static constexpr int kRowV = kChunk * kVStride * 2;
    static constexpr int kSt = 16 * kNct * kVStride * 2;

    static constexpr int oTok = 0;                                        // int[3][64]
    static constexpr int oTokG = oTok + 3 * kChunk * 4;                   // int[3][64]
    static constexpr int oGam = oTokG + 3 * kChunk * 4;                   // float[64] exp(b_C)
    static constexpr int oLa = oGam + 64 * 4;
    static constexpr int oKHi = oLa + kChunk * kLaStride * 4;
    static constexpr int oKLo = oKHi + kRowK;
    static constexpr int oV = oKLo + kRowK;
    static constexpr int oW = oV + kRowV;
    static constexpr int oStHi = oW + kRowV;
    static constexpr int oStLo = oStHi + kSt;
    static constexpr int oQHi = oStLo + kSt;                              // with DV: raw q rows, then q~ hi / lo
    static constexpr int oQLo = oQHi + kRowK;
    static constexpr int oEndAlpha = DV ? oQLo + kRowK : oStLo + kSt;
    // two-sided gate: raw log_beta rows, the bf16 remainders of the gated v and w rows, exp(c_C) per value column
    static constexpr int kLbStride = kDvp + 4;
    static constexpr int oLb = oEndAlpha;
    static constexpr int oVLo = oLb + kChunk * kLbStride * 4;
    static constexpr int oWLo = oVLo + kRowV;
    static constexpr int oGamB = oWLo + kRowV;                            // float[kDvp]
    static constexpr int kBytes = BETA ? oGamB + kDvp * 4 : oEndAlpha;
};

template <int N>
using int_c = std::integral_constant<int, N>;

// DV = also compute the outputs o_j = q_j S_j of the same recurrence (fp32 rows to p.out; p.q holds q):
//     o_j = sum_{i<=j} (q~_j . k~_i) v_i + q~_j S_0 ,   q~_j = q_j E_j
// as the forward kernel does, on the operands that are already in LDS.  In the backward pass the reversed
// recurrence of G needs both: dk as the row read against v, and dv = k G as the output with q := k.
// BETA = two-sided gate (p.log_beta): with c_j the inclusive sum of log_beta inside the chunk (per value column),
// F_j = exp(c_j), v~_i = v_i / F_i and w~_j = w_j * F_j,
//     r_j = E_j * ( sum_{i<=j} (w~_j . v~_i) k~_i + S_0 w~_j ),   S_C = diag(E_C) (S_0 + K~^T V~) diag(F_C):
// the same contractions with v~ and w~ (bf16 hi/lo pairs, all four products) in the places of v and w; with DV the
// outputs are o_j = F_j * (sum_{i<=j} (q~_j . k~_i) v~_i + q~_j S_0) (F_j is left in place of the raw log_beta row).
template <int NDK8, int NDV16, int MINW, bool DV, bool BETA = false>
__global__ __launch_bounds__(256, MINW) void mfma_row_read_kernel(Params p, const void *w_in, float *r_out) {
    using L = RLayout<NDK8, NDV16, DV, BETA>;
    constexpr int LBS = L::kLbStride;
    constexpr int NW = 4, NTHR = 256;
    constexpr int CHS = L::kChStride, VS = L::kVStride, LAS = L::kLaStride;
    constexpr int NCT = L::kNct;
    constexpr int KSV = (NDV16 * 2 + 3) / 4;        // 32-column steps of the contractions over value columns
    constexpr int TPW = (NDV16 + NW - 1) / NW;      // value-column tiles of the state per wave
    constexpr int NTB = 3;
    static_assert(16 * NCT <= CHS, "channel tiles must fit the operand row");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int *s_tok = reinterpret_cast<int *>(smem + L::oTok);
    int *s_tokg = reinterpret_cast<int *>(smem + L::oTokG);
    float *s_gam = reinterpret_cast<float *>(smem + L::oGam);
    float *s_la = reinterpret_cast<float *>(smem + L::oLa);
    uint16_t *s_khi = reinterpret_cast<uint16_t *>(smem + L::oKHi);
    uint16_t *s_klo = reinterpret_cast<uint16_t *>(smem + L::oKLo);
    uint16_t *s_v = reinterpret_cast<uint16_t *>(smem + L::oV);
    uint16_t *s_w = reinterpret_cast<uint16_t *>(smem + L::oW);
    uint16_t *s_sthi = reinterpret_cast<uint16_t *>(smem + L::oStHi);
    uint16_t *s_stlo = reinterpret_cast<uint16_t *>(smem + L::oStLo);
    uint16_t *s_qhi = reinterpret_cast<uint16_t *>(smem + L::oQHi);
    uint16_t *s_qlo = reinterpret_cast<uint16_t *>(smem + L::oQLo);
    float *s_lb = reinterpret_cast<float *>(smem + L::oLb);            // BETA only, like the three below
    uint16_t *s_vlo = reinterpret_cast<uint16_t *>(smem + L::oVLo);
    uint16_t *s_wlo = reinterpret_cast<uint16_t *>(smem + L::oWLo);
    float *s_gamb = reinterpret_cast<float *>(smem + L::oGamB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lm = lane & 15;
    const int g = lane >> 4;

    // contiguous ranges of spans per XCD (work-groups are dealt round-robin to the 8 XCDs)
    int blk = blockIdx.x;
    {
        const int nb = gridDim.x;
        if ((nb & 7) == 0) blk = (blk & 7) * (nb >> 3) + (blk >> 3);
    }
    const int bh = blk / p.nspans;
    int sp_ = blk - bh * p.nspans;
    // when the work-groups chain the span states themselves the cost grows with the span index: odd heads walk
    // their spans backwards, so that the two groups sharing a compute unit pair a long chain with a short one
    if (p.chain_in_output && (bh & 1)) sp_ = p.nspans - 1 - sp_;
    const int sp = sp_;
    const int dk = p.dk, dv = p.dv, T = p.T;
    const int s_begin = sp * p.span_len;
    const int s_end = min(T, s_begin + p.span_len);
    const int nch = (s_end - s_begin + kChunk - 1) / kChunk;

    const size_t base_k = slab_k(p, bh), base_v = slab_v(p, bh);
    const char *gk = static_cast<const char *>(p.k) + base_k * 2;
    const char *gv = static_cast<const char *>(p.v) + base_v * 2;
    const char *gw = static_cast<const char *>(w_in) + base_v * 2;
    const char *gla_ = reinterpret_cast<const char *>(p.log_alpha) + base_k * 4;
    char *gr = reinterpret_cast<char *>(r_out) + base_k * 4;
    const char *gq = static_cast<const char *>(p.q) + base_k * 2;
    const char *glb = reinterpret_cast<const char *>(p.log_beta) + base_v * 4;
    char *gout = static_cast<char *>(p.out) + base_v * 4;

    // ---- state tiles of this wave, transposed: acc[i][ct][r] = S[c = 16 ct + lm][n = 16 (w + 4 i) + 4 g + r] ----
    f32x4 acc[TPW][NCT];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) acc[i][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    // The state entering the span: what the carry kernel left in the workspace, or (chain_in_output) chained here
    // from the local states of the spans before it (chain_span_states: nearest span first, until the accumulated
    // decay makes the rest vanish in fp32); the result goes through LDS into the accumulator layout.
    {
        const bool chain = p.chain_in_output && sp > 0;   // uniform over the group
        if (chain) {
            constexpr int kV4 = (L::kDkp * L::kDvp / 4 + NTHR - 1) / NTHR;  // float4 per thread
            constexpr int kBudget = MINW >= 2 ? 32 : 64;                    // float4 in flight
            constexpr int kRun = kBudget / kV4 > 0 ? kBudget / kV4 : 1;     // spans in flight
            chain_span_states<NTHR, kV4, kRun, BETA>(p, bh, sp, tid, reinterpret_cast<float *>(smem));
        }
        __syncthreads();
        if (chain) {
            const float *s_chain = reinterpret_cast<const float *>(smem);
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int n = 16 * (w + NW * i) + 4 * g;
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    const int c = 16 * ct + lm;
                    if (c < dk && n < dv) acc[i][ct] = *reinterpret_cast<const f32x4 *>(s_chain + c * dv + n);
                }
            }
        }
        __syncthreads();
        if (!p.chain_in_output && p.nspans > 1) {
            const float *s0 = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int n = 16 * (w + NW * i) + 4 * g;
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    const int c = 16 * ct + lm;
                    if (c < dk && n < dv) acc[i][ct] = *reinterpret_cast<const f32x4 *>(s0 + c * dv + n);
                }
            }
        }
    }

    // ---- prologue: clear LDS (pads must read as zero), token maps of the first two chunks ----
    for (int i = tid; i < L::kBytes / 16; i += NTHR)
        reinterpret_cast<u32x4 *>(smem)[i] = u32x4{0, 0, 0, 0};
    __syncthreads();
    if (tid < 2 * kChunk) {
        const int s = s_begin + tid;
        const int sc = (s < s_end) ? s : s_begin;
        s_tok[tid] = scan_token(p.scan_dir, sc, T, p.grid_h, p.grid_w);
        s_tokg[tid] = scan_token(p.scan_dir, max(sc - p.gate_shift, 0), T, p.grid_h, p.grid_w);
    }
    __syncthreads();

    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): keeps later reads of acc from waiting on the row prefetch

    // ---- HBM pieces staged by this thread: the 16-byte pieces of log_alpha (8-byte pieces of k) of a chunk and the
    // 16-byte pieces of v and w are numbered row by row; slot m of a thread is piece tid + 256 m, so that a wave's
    // request covers neighbouring pieces of neighbouring rows.  Slots past the last piece repeat it (the load stays
    // in bounds; nothing is written to LDS for them) ----
    constexpr int kF = (kChunk * NDK8 * 2 + NTHR - 1) / NTHR;
    constexpr int kVF = (kChunk * NDV16 * 2 + NTHR - 1) / NTHR;
    const int pcs = dk >> 2, vpcs = dv >> 3;
    int frp[kF], fvrp[kVF];     // row << 8 | piece
#pragma unroll
    for (int m = 0; m < kF; ++m) {
        const int f = min(tid + NTHR * m, kChunk * pcs - 1);
        const int row = f / pcs;
        frp[m] = (row << 8) | (f - row * pcs);
    }
#pragma unroll
    for (int m = 0; m < kVF; ++m) {
        const int f = min(tid + NTHR * m, kChunk * vpcs - 1);
        const int row = f / vpcs;
        fvrp[m] = (row << 8) | (f - row * vpcs);
    }
    const uint32_t dk2 = 2u * (uint32_t)p.st_k, dv2 = 2u * (uint32_t)p.st_v;

    f32x4 r_la[kF];
    u32x2 r_k[kF];
    u32x2 r_q[DV ? kF : 1];
    u32x4 r_v[kVF], r_w[kVF];
    f32x4 r_lb[BETA ? kVF : 1][2];   // log_beta of the same 8 columns as the v piece
    auto load_chunk = [&](int chunk) {
        const int *tok = s_tok + (chunk % NTB) * kChunk;
        const int *tokg = s_tokg + (chunk % NTB) * kChunk;
#pragma unroll
        for (int m = 0; m < kF; ++m) {
            const int row = frp[m] >> 8;
            const uint32_t pc = 8u * (uint32_t)(frp[m] & 255);
            r_la[m] = *reinterpret_cast<const f32x4 *>(gla_ + 2u * ((uint32_t)tokg[row] * dk2 + pc));
            r_k[m] = *reinterpret_cast<const u32x2 *>(gk + (uint32_t)tok[row] * dk2 + pc);
            if constexpr (DV) r_q[m] = *reinterpret_cast<const u32x2 *>(gq + (uint32_t)tok[row] * dk2 + pc);
        }
#pragma unroll
        for (int m = 0; m < kVF; ++m) {
            const uint32_t e2 = (uint32_t)tok[fvrp[m] >> 8] * dv2 + 16u * (uint32_t)(fvrp[m] & 255);
            r_v[m] = *reinterpret_cast<const u32x4 *>(gv + e2);
            r_w[m] = *reinterpret_cast<const u32x4 *>(gw + e2);
            if constexpr (BETA) {
                const char *lbp = glb + 2u * ((uint32_t)tokg[fvrp[m] >> 8] * dv2 + 16u * (uint32_t)(fvrp[m] & 255));
                r_lb[m][0] = *reinterpret_cast<const f32x4 *>(lbp);
                r_lb[m][1] = *reinterpret_cast<const f32x4 *>(lbp + 16);
            }
        }
    };
    load_chunk(0);

    for (int chunk = 0; chunk < nch; ++chunk) {
        const int *tok = s_tok + (chunk % NTB) * kChunk;
        // ================= (a) registers -> LDS =================
        const int nvalid = min(kChunk, s_end - s_begin - chunk * kChunk);
        if (nvalid < kChunk) {   // rows past the span: no decay, no contribution
#pragma unroll
            for (int m = 0; m < kF; ++m) {
                if ((frp[m] >> 8) >= nvalid) {
                    r_la[m] = f32x4{0.f, 0.f, 0.f, 0.f};
                    r_k[m] = u32x2{0, 0};
                    if constexpr (DV) r_q[m] = u32x2{0, 0};
                }
            }
#pragma unroll
            for (int m = 0; m < kVF; ++m) {
                if ((fvrp[m] >> 8) >= nvalid) {
                    r_v[m] = u32x4{0, 0, 0, 0};
                    r_w[m] = u32x4{0, 0, 0, 0};
                    if constexpr (BETA) r_lb[m][0] = r_lb[m][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
#pragma unroll
        for (int m = 0; m < kF; ++m) {
            if (tid + NTHR * m < kChunk * pcs) {
                const int row = frp[m] >> 8, ch = 4 * (frp[m] & 255);
                *reinterpret_cast<f32x4 *>(s_la + row * LAS + ch) = r_la[m];
                *reinterpret_cast<u32x2 *>(s_khi + row * CHS + ch) = r_k[m];
                if constexpr (DV) *reinterpret_cast<u32x2 *>(s_qhi + row * CHS + ch) = r_q[m];
            }
        }
#pragma unroll
        for (int m = 0; m < kVF; ++m) {
            if (tid + NTHR * m < kChunk * vpcs) {
                const int row = fvrp[m] >> 8, col = 8 * (fvrp[m] & 255);
                *reinterpret_cast<u32x4 *>(s_v + row * VS + col) = r_v[m];
                *reinterpret_cast<u32x4 *>(s_w + row * VS + col) = r_w[m];
                if constexpr (BETA) {
                    *reinterpret_cast<f32x4 *>(s_lb + row * LBS + col) = r_lb[m][0];
                    *reinterpret_cast<f32x4 *>(s_lb + row * LBS + col + 4) = r_lb[m][1];
                }
            }
        }
        load_chunk(chunk + 1);   // past the span the clamped token map keeps the loads in bounds
        {
            // S_0 as bf16 hi/lo, channel-major
            const int ln = recompute_per_chunk(lane), lm2 = ln & 15, g2 = ln >> 4;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                if (w + NW * i < NDV16) {
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) {
                        u32x2 hi, lo;
                        SPLIT_PAIR(acc[i][ct][0], acc[i][ct][1], hi[0], lo[0]);
                        SPLIT_PAIR(acc[i][ct][2], acc[i][ct][3], hi[1], lo[1]);
                        const int off = (16 * ct + lm2) * VS + 16 * (w + NW * i) + 4 * g2;
                        *reinterpret_cast<u32x2 *>(s_sthi + off) = hi;
                        *reinterpret_cast<u32x2 *>(s_stlo + off) = lo;
                    }
                }
            }
        }
        if (w == NW - 1) {   // token map of the chunk loaded next time
            const int s = s_begin + (chunk + 2) * kChunk + lane;
            const int sc = (s < s_end) ? s : s_begin;
            s_tok[((chunk + 2) % NTB) * kChunk + lane] = scan_token(p.scan_dir, sc, T, p.grid_h, p.grid_w);
            s_tokg[((chunk + 2) % NTB) * kChunk + lane] =
                scan_token(p.scan_dir, max(sc - p.gate_shift, 0), T, p.grid_h, p.grid_w);
        }
        __syncthreads();

        // ================= (b) gates: lane = token, units of 4 channels dealt to the waves =================
        {
            const int j = lane;
            for (int u = w; u < pcs; u += NW) {
                const int c0 = 4 * u;
                const f32x4 x = *reinterpret_cast<const f32x4 *>(s_la + j * LAS + c0);
                const u32x2 kr = *reinterpret_cast<const u32x2 *>(s_khi + j * CHS + c0);
                float bb[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) bb[i] = x[i] * kLog2e;
                wave_inclusive_scan4(bb[0], bb[1], bb[2], bb[3]);
                f32x4 e;
#pragma unroll
                for (int i = 0; i < 4; ++i) e[i] = exp2_fast(bb[i]);
                u32x2 khi, klo;
                SPLIT_PAIR(bf16_lo_as_float(kr[0]) * exp2_fast(fminf(-bb[0], kMaxExp2)),
                           bf16_hi_as_float(kr[0]) * exp2_fast(fminf(-bb[1], kMaxExp2)), khi[0], klo[0]);
                SPLIT_PAIR(bf16_lo_as_float(kr[1]) * exp2_fast(fminf(-bb[2], kMaxExp2)),
                           bf16_hi_as_float(kr[1]) * exp2_fast(fminf(-bb[3], kMaxExp2)), khi[1], klo[1]);
                *reinterpret_cast<u32x2 *>(s_khi + j * CHS + c0) = khi;
                *reinterpret_cast<u32x2 *>(s_klo + j * CHS + c0) = klo;
                if constexpr (DV) {
                    const u32x2 qr = *reinterpret_cast<const u32x2 *>(s_qhi + j * CHS + c0);
                    u32x2 qhi, qlo;
                    SPLIT_PAIR(bf16_lo_as_float(qr[0]) * e[0], bf16_hi_as_float(qr[0]) * e[1], qhi[0], qlo[0]);
                    SPLIT_PAIR(bf16_lo_as_float(qr[1]) * e[2], bf16_hi_as_float(qr[1]) * e[3], qhi[1], qlo[1]);
                    *reinterpret_cast<u32x2 *>(s_qhi + j * CHS + c0) = qhi;
                    *reinterpret_cast<u32x2 *>(s_qlo + j * CHS + c0) = qlo;
                }
                *reinterpret_cast<f32x4 *>(s_la + j * LAS + c0) = e;      // E_j in place of the raw gates
                if (lane == 63) *reinterpret_cast<f32x4 *>(s_gam + c0) = e;
            }
            if constexpr (BETA) {
                // value side, 8-column units dealt from the last wave: v~ = v / F and w~ = w F as bf16 hi/lo
                for (int c0 = 8 * (NW - 1 - w); c0 < dv; c0 += 8 * NW) {
                    float cc[8];
#pragma unroll
                    for (int v4 = 0; v4 < 2; ++v4) {
                        const f32x4 x = *reinterpret_cast<const f32x4 *>(s_lb + j * LBS + c0 + 4 * v4);
#pragma unroll
                        for (int i = 0; i < 4; ++i) cc[4 * v4 + i] = x[i] * kLog2e;
                        wave_inclusive_scan4(cc[4 * v4], cc[4 * v4 + 1], cc[4 * v4 + 2], cc[4 * v4 + 3]);
                    }
                    const u32x4 vr = *reinterpret_cast<const u32x4 *>(s_v + j * VS + c0);
                    const u32x4 wr = *reinterpret_cast<const u32x4 *>(s_w + j * VS + c0);
                    u32x4 vh, vl, wh, wl;
                    float f[8];
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        f[2 * h] = exp2_fast(cc[2 * h]);
                        f[2 * h + 1] = exp2_fast(cc[2 * h + 1]);
                        SPLIT_PAIR(bf16_lo_as_float(vr[h]) * exp2_fast(fminf(-cc[2 * h], kMaxExp2)),
                                   bf16_hi_as_float(vr[h]) * exp2_fast(fminf(-cc[2 * h + 1], kMaxExp2)), vh[h], vl[h]);
                        SPLIT_PAIR(bf16_lo_as_float(wr[h]) * f[2 * h], bf16_hi_as_float(wr[h]) * f[2 * h + 1], wh[h], wl[h]);
                    }
                    *reinterpret_cast<u32x4 *>(s_v + j * VS + c0) = vh;
                    *reinterpret_cast<u32x4 *>(s_vlo + j * VS + c0) = vl;
                    *reinterpret_cast<u32x4 *>(s_w + j * VS + c0) = wh;
                    *reinterpret_cast<u32x4 *>(s_wlo + j * VS + c0) = wl;
                    if constexpr (DV) {
                        *reinterpret_cast<f32x4 *>(s_lb + j * LBS + c0) = f32x4{f[0], f[1], f[2], f[3]};
                        *reinterpret_cast<f32x4 *>(s_lb + j * LBS + c0 + 4) = f32x4{f[4], f[5], f[6], f[7]};
                    }
                    if (lane == 63) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) s_gamb[c0 + i] = f[i];
                    }
                }
            }
        }
        __syncthreads();

        // ================= (c) contractions =================
        const int ln = recompute_per_chunk(lane), lm3 = ln & 15, g3 = ln >> 4;
        int coln[KSV];   // column group of this lane in 32-column step ks; groups past the data alias the zero group
#pragma unroll
        for (int ks = 0; ks < KSV; ++ks) coln[ks] = (4 * ks + g3 < 2 * NDV16) ? 8 * (4 * ks + g3) : L::kZeroCol;
        const int tr_row = lm3 >> 2, tr_col = 4 * (lm3 & 3);
        auto contract = [&](auto wave_c) {
            constexpr int IT = decltype(wave_c)::value;   // 16-token tile of this wave
            constexpr int NQ = IT / 2 + 1;                // 32-token steps that hold tokens <= the tile's
            const int lm = lm3, g = g3;
            const uint16_t *krow_h = s_khi + (4 * g + tr_row) * CHS + tr_col;
            const uint16_t *krow_l = s_klo + (4 * g + tr_row) * CHS + tr_col;
            const uint16_t *vrow = s_v + (4 * g + tr_row) * VS + tr_col;
            const uint16_t *vrow_l = s_vlo + (4 * g + tr_row) * VS + tr_col;   // BETA
            u32x4 wf[KSV], wfl[BETA ? KSV : 1];
#pragma unroll
            for (int ks = 0; ks < KSV; ++ks) {
                wf[ks] = *reinterpret_cast<const u32x4 *>(s_w + (16 * IT + lm) * VS + coln[ks]);
                if constexpr (BETA) wfl[ks] = *reinterpret_cast<const u32x4 *>(s_wlo + (16 * IT + lm) * VS + coln[ks]);
            }
            u32x4 kth[2][NCT], ktl[2][NCT];   // K~ over tokens: [32-token step][channel tile]
            auto load_k = [&](int q) {
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    const u32x2 h0 = lds_read_tr(krow_h + 32 * q * CHS + 16 * ct);
                    const u32x2 h1 = lds_read_tr(krow_h + (32 * q + 16) * CHS + 16 * ct);
                    const u32x2 l0 = lds_read_tr(krow_l + 32 * q * CHS + 16 * ct);
                    const u32x2 l1 = lds_read_tr(krow_l + (32 * q + 16) * CHS + 16 * ct);
                    kth[q][ct] = u32x4{h0[0], h0[1], h1[0], h1[1]};
                    ktl[q][ct] = u32x4{l0[0], l0[1], l1[0], l1[1]};
                }
            };
            f32x4 rr[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) rr[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                u32x2 ph[2] = {u32x2{0, 0}, u32x2{0, 0}}, pl[2] = {u32x2{0, 0}, u32x2{0, 0}};
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int jt = 2 * q + u;
                    if (jt <= IT) {
                        // P^T tile: lane (lm, g) gets P[i = 16 IT + lm][j = 16 jt + 4 g + r]
                        f32x4 d = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int ks = 0; ks < KSV; ++ks) {
                            const u32x4 vf = *reinterpret_cast<const u32x4 *>(s_v + (16 * jt + lm) * VS + coln[ks]);
                            d = mfma(vf, wf[ks], d);
                            if constexpr (BETA) {
                                const u32x4 vfl = *reinterpret_cast<const u32x4 *>(s_vlo + (16 * jt + lm) * VS + coln[ks]);
                                d = mfma(vf, wfl[ks], d);
                                d = mfma(vfl, wf[ks], d);
                                d = mfma(vfl, wfl[ks], d);
                            }
                        }
                        if (jt == IT) {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (4 * g + r > lm) d[r] = 0.f;
                        }
                        SPLIT_PAIR(d[0], d[1], ph[u][0], pl[u][0]);
                        SPLIT_PAIR(d[2], d[3], ph[u][1], pl[u][1]);
                    }
                }
                load_k(q);
                const u32x4 bh_ = u32x4{ph[0][0], ph[0][1], ph[1][0], ph[1][1]};
                const u32x4 bl_ = u32x4{pl[0][0], pl[0][1], pl[1][0], pl[1][1]};
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    rr[ct] = mfma(kth[q][ct], bh_, rr[ct]);
                    rr[ct] = mfma(kth[q][ct], bl_, rr[ct]);
                    rr[ct] = mfma(ktl[q][ct], bh_, rr[ct]);
                }
            }
            // + W S_0^T
#pragma unroll
            for (int ks = 0; ks < KSV; ++ks) {
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    const int srow = (16 * ct + lm) * VS + coln[ks];
                    const u32x4 sh = *reinterpret_cast<const u32x4 *>(s_sthi + srow);
                    const u32x4 sl = *reinterpret_cast<const u32x4 *>(s_stlo + srow);
                    rr[ct] = mfma(sh, wf[ks], rr[ct]);
                    rr[ct] = mfma(sl, wf[ks], rr[ct]);
                    if constexpr (BETA) {
                        rr[ct] = mfma(sh, wfl[ks], rr[ct]);
                        rr[ct] = mfma(sl, wfl[ks], rr[ct]);
                    }
                }
            }
            // scale by E and store: lane (lm, g) holds channels 16 ct + 4 g .. + 3 of token 16 IT + lm
            const int row = 16 * IT + lm;
            if (row < nvalid) {
                char *orow = gr + ((uint32_t)tok[row] * (uint32_t)p.st_k + 4u * (uint32_t)g) * 4u;
#pragma unroll
                for (int ct = 0; ct < NCT; ++ct) {
                    if (16 * ct + 4 * g < dk) {   // dk is a multiple of 4: all four channels or none
                        const f32x4 e = *reinterpret_cast<const f32x4 *>(s_la + row * LAS + 16 * ct + 4 * g);
                        f32x4 o = rr[ct];
#pragma unroll
                        for (int r = 0; r < 4; ++r) o[r] *= e[r];
                        *reinterpret_cast<f32x4 *>(orow + 64 * ct) = o;
                    }
                }
            }
            if constexpr (DV) {
                // ---- outputs of the wave's 16 tokens: O^T[n][i], lane (lm, g) holds o[x][r] = O[i = 16 IT + lm][n = 16 x + 4 g + r]
                constexpr int NX = NDV16;
                constexpr int KS = (NDK8 + 3) / 4;            // 32-channel steps
                f32x4 o[NX];
#pragma unroll
                for (int x = 0; x < NX; ++x) o[x] = f32x4{0.f, 0.f, 0.f, 0.f};
                int colk[KS];   // channel group of this lane in step ks; groups past the data alias the all-zero group
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) colk[ks] = (4 * ks + g < NDK8) ? 8 * (4 * ks + g) : L::kDkp;
                u32x4 qfh[KS], qfl[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    qfh[ks] = *reinterpret_cast<const u32x4 *>(s_qhi + (16 * IT + lm) * CHS + colk[ks]);
                    qfl[ks] = *reinterpret_cast<const u32x4 *>(s_qlo + (16 * IT + lm) * CHS + colk[ks]);
                }
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    u32x2 ah[2] = {u32x2{0, 0}, u32x2{0, 0}}, al[2] = {u32x2{0, 0}, u32x2{0, 0}};
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int jt = 2 * q + u;
                        if (jt <= IT) {
                            // score tile, transposed: lane (lm, g) gets A[i = 16 IT + lm][j = 16 jt + 4 g + r]
                            f32x4 d = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int ks = 0; ks < KS; ++ks) {
                                const u32x4 kh = *reinterpret_cast<const u32x4 *>(s_khi + (16 * jt + lm) * CHS + colk[ks]);
                                const u32x4 kl = *reinterpret_cast<const u32x4 *>(s_klo + (16 * jt + lm) * CHS + colk[ks]);
                                d = mfma(kh, qfh[ks], d);
                                d = mfma(kh, qfl[ks], d);
                                d = mfma(kl, qfh[ks], d);
                            }
                            if (jt == IT) {
#pragma unroll
                                for (int r = 0; r < 4; ++r)
                                    if (4 * g + r > lm) d[r] = 0.f;
                            }
                            SPLIT_PAIR(d[0], d[1], ah[u][0], al[u][0]);
                            SPLIT_PAIR(d[2], d[3], ah[u][1], al[u][1]);
                        }
                    }
                    const u32x4 bh2 = u32x4{ah[0][0], ah[0][1], ah[1][0], ah[1][1]};
                    const u32x4 bl2 = u32x4{al[0][0], al[0][1], al[1][0], al[1][1]};
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        const u32x2 v0 = lds_read_tr(vrow + 32 * q * VS + 16 * x);
                        const u32x2 v1 = lds_read_tr(vrow + (32 * q + 16) * VS + 16 * x);
                        const u32x4 vf = u32x4{v0[0], v0[1], v1[0], v1[1]};
                        o[x] = mfma(vf, bh2, o[x]);
                        o[x] = mfma(vf, bl2, o[x]);
                        if constexpr (BETA) {
                            const u32x2 l0 = lds_read_tr(vrow_l + 32 * q * VS + 16 * x);
                            const u32x2 l1 = lds_read_tr(vrow_l + (32 * q + 16) * VS + 16 * x);
                            const u32x4 vfl = u32x4{l0[0], l0[1], l1[0], l1[1]};
                            o[x] = mfma(vfl, bh2, o[x]);
                            o[x] = mfma(vfl, bl2, o[x]);
                        }
                    }
                }
                // + Q~ S_0: the state rows (channel-major in LDS) are read transposed, so the channels of a 32-channel
                // step come in the slot order 16 (e/4) + 4 g + e%4; the q~ operand is read in that order too
                const uint16_t *strow_h = s_sthi + (4 * g + tr_row) * VS + tr_col;
                const uint16_t *strow_l = s_stlo + (4 * g + tr_row) * VS + tr_col;
#pragma unroll
                for (int q = 0; q < KS; ++q) {
                    const bool second = 32 * q + 16 < 16 * NCT;    // the step's upper 16 channels exist in the state rows
                    const uint16_t *qh = s_qhi + (16 * IT + lm) * CHS + 32 * q + 4 * g;
                    const uint16_t *ql = s_qlo + (16 * IT + lm) * CHS + 32 * q + 4 * g;
                    const u32x2 qh0 = *reinterpret_cast<const u32x2 *>(qh), ql0 = *reinterpret_cast<const u32x2 *>(ql);
                    u32x2 qh1 = u32x2{0, 0}, ql1 = u32x2{0, 0};
                    if (second) {
                        qh1 = *reinterpret_cast<const u32x2 *>(qh + 16);
                        ql1 = *reinterpret_cast<const u32x2 *>(ql + 16);
                    }
                    const u32x4 qsh = u32x4{qh0[0], qh0[1], qh1[0], qh1[1]}, qsl = u32x4{ql0[0], ql0[1], ql1[0], ql1[1]};
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        const u32x2 h0 = lds_read_tr(strow_h + 32 * q * VS + 16 * x);
                        const u32x2 l0 = lds_read_tr(strow_l + 32 * q * VS + 16 * x);
                        u32x2 h1 = u32x2{0, 0}, l1 = u32x2{0, 0};
                        if (second) {
                            h1 = lds_read_tr(strow_h + (32 * q + 16) * VS + 16 * x);
                            l1 = lds_read_tr(strow_l + (32 * q + 16) * VS + 16 * x);
                        }
                        const u32x4 sh = u32x4{h0[0], h0[1], h1[0], h1[1]}, sl = u32x4{l0[0], l0[1], l1[0], l1[1]};
                        o[x] = mfma(sh, qsh, o[x]);
                        o[x] = mfma(sh, qsl, o[x]);
                        o[x] = mfma(sl, qsh, o[x]);
                    }
                }
                if (row < nvalid) {
                    char *orow2 = gout + ((uint32_t)tok[row] * (uint32_t)p.st_v + 4u * (uint32_t)g) * 4u;
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        if (4 * g + 16 * x < dv) {
                            if constexpr (BETA) {   // row j of the outputs carries F_j per value column
                                const f32x4 f4 = *reinterpret_cast<const f32x4 *>(s_lb + row * LBS + 16 * x + 4 * g);
#pragma unroll
                                for (int r = 0; r < 4; ++r) o[x][r] *= f4[r];
                            }
                            *reinterpret_cast<f32x4 *>(orow2 + 64 * x) = o[x];
                        }
                    }
                }
            }
            // state update on this wave's tiles: S^T += V^T K~, then the chunk's decay per channel
#pragma unroll
            for (int q = NQ; q < 2; ++q) load_k(q);
            float gm[NCT];
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) gm[ct] = s_gam[16 * ct + lm];
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int nt = IT + NW * i;
                if (nt < NDV16) {
                    u32x4 vt[2], vtl[BETA ? 2 : 1];
#pragma unroll
                    for (int q = 0; q < 2; ++q) {
                        const u32x2 v0 = lds_read_tr(vrow + 32 * q * VS + 16 * nt);
                        const u32x2 v1 = lds_read_tr(vrow + (32 * q + 16) * VS + 16 * nt);
                        vt[q] = u32x4{v0[0], v0[1], v1[0], v1[1]};
                        if constexpr (BETA) {
                            const u32x2 l0 = lds_read_tr(vrow_l + 32 * q * VS + 16 * nt);
                            const u32x2 l1 = lds_read_tr(vrow_l + (32 * q + 16) * VS + 16 * nt);
                            vtl[q] = u32x4{l0[0], l0[1], l1[0], l1[1]};
                        }
                    }
                    f32x4 gb = f32x4{1.f, 1.f, 1.f, 1.f};     // BETA: decay of this lane's four value columns
                    if constexpr (BETA) gb = *reinterpret_cast<const f32x4 *>(s_gamb + 16 * nt + 4 * g);
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) {
                        f32x4 a = acc[i][ct];
#pragma unroll
                        for (int q = 0; q < 2; ++q) {
                            a = mfma(vt[q], kth[q][ct], a);
                            a = mfma(vt[q], ktl[q][ct], a);
                            if constexpr (BETA) {
                                a = mfma(vtl[q], kth[q][ct], a);
                                a = mfma(vtl[q], ktl[q][ct], a);
                            }
                        }
#pragma unroll
                        for (int r = 0; r < 4; ++r) a[r] *= BETA ? gm[ct] * gb[r] : gm[ct];
                        acc[i][ct] = a;
                    }
                }
            }
        };
        switch (w) {
        case 0: contract(int_c<0>{}); break;
        case 1: contract(int_c<1>{}); break;
        case 2: contract(int_c<2>{}); break;
        default: contract(int_c<3>{}); break;
        }
        __syncthreads();
    }
}

template <int NDK8, int NDV16, bool DV, bool BETA = false>
hipError_t launch_one(const Params &p, const void *w, float *r, hipStream_t stream) {
    using L = RLayout<NDK8, NDV16, DV, BETA>;
    constexpr int kGroupsPerCu = (160 * 1024) / L::kBytes;
    constexpr int MINW = kGroupsPerCu >= 2 ? 2 : 1;
    auto kernel = mfma_row_read_kernel<NDK8, NDV16, MINW, DV, BETA>;
    static std::atomic<bool> configured[kMaxDevices] = {};  // per instantiation and device
    {
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), L::kBytes, configured);
        if (e != hipSuccess) return e;
    }
    dim3 grid((unsigned)(p.B * p.H * p.nspans)), block(256);
    hipLaunchKernelGGL(kernel, grid, block, L::kBytes, stream, p, w, r);
    return hipGetLastError();
}

template <bool DV>
hipError_t launch_sizes(const Params &p, const void *w, float *r, hipStream_t stream) {
    const int ndk8 = (p.dk + 7) / 8, ndv16 = (p.dv + 15) / 16;
    if (p.log_beta != nullptr) {   // two-sided gate: the head sizes whose extra rows fit the LDS (dk <= 40, dv <= 80)
        if (ndk8 <= 4 && ndv16 <= 4) return launch_one<4, 4, DV, true>(p, w, r, stream);
        if (ndk8 <= 5 && ndv16 <= 5) return launch_one<5, 5, DV, true>(p, w, r, stream);
        return hipErrorInvalidConfiguration;
    }
    if (ndk8 <= 4 && ndv16 <= 4) return launch_one<4, 4, DV>(p, w, r, stream);
    if (ndk8 <= 5 && ndv16 <= 5) return launch_one<5, 5, DV>(p, w, r, stream);
    return launch_one<8, 8, DV>(p, w, r, stream);
}

}  // namespace

// Same conditions as the forward MFMA engine (bf16 rows, dk % 4 == 0, dv % 8 == 0, 32-bit offsets).
// with_outputs: also write o_j = q_j S_j (p.q, fp32 rows to p.out).
hipError_t launch_mfma_row_read(const Params &p, const void *w, float *r, hipStream_t stream, bool with_outputs) {
    return with_outputs ? launch_sizes<true>(p, w, r, stream) : launch_sizes<false>(p, w, r, stream);
}

}  // namespace gla
