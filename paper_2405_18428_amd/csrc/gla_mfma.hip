// bf16 MFMA engine for one span of the GLA recurrence in its chunk form
// (DiG paper, Sec. 3.5: chunks of M = 64 tokens computed on-chip; recurrence of
// Sec. 3.1 Eq. (attn_gla) rows 1-3 with beta = 1).
//
// With b_j = sum_{i<=j} log_alpha_i inside a chunk (inclusive, per key channel)
// and b_C its value at the chunk's last token, unrolling the recurrence gives
//     o_j  = sum_{i<=j} (q~_j . k~_i) v_i + q~_j S_0 ,   q~_j = q_j * exp(b_j),  k~_i = k_i * exp(-b_i)
//     S_C  = diag(exp(b_C)) (S_0 + K~^T V)
// i.e. four dense contractions per chunk, all on v_mfma_f32_16x16x32_bf16:
//     A^T = K~ Q~^T (causal tiles only),  O = A V + Q~ S_0,  S += K~^T V (then scaled by exp(b_C)).
// Every gated operand (q~, k~, A, S_0) is split into a bf16 "hi" part and a bf16
// "lo" remainder so that the products carry about 16 mantissa bits; v is used as
// given.  The state S lives in fp32 MFMA accumulators for the whole span.
// Exponentials run in base 2 (log_alpha is scaled by log2(e) once, before the scan).
//
// A work-group has NW = 4 waves in the output pass and 8 in the state pass; per chunk:
//   (a) registers prefetched from HBM -> LDS: raw log_alpha / q / k / v rows (all
//       token-major, 16- or 8-byte pieces), S_0 as bf16 hi/lo;
//   (b) lane = token: DPP wave scan of log_alpha per channel, exp2, gating, hi/lo
//       split, q~ and k~ written in place over the raw rows; the 32/NW-channel units
//       of a row are dealt to the waves round-robin, the channels past the last whole unit one by one;
//   (c) MFMA: in the output pass wave w owns output rows 16w..16w+15; in both passes the state
//       tiles of a wave lie in one 16-channel row tile (its K~ operand is read once per chunk).
// Operands whose contraction runs over tokens (V, and K~ in the state update) are
// fetched from the token-major rows with ds_read_b64_tr_b16, which hands lane i of
// a 16-lane group element i%4 of the 8 bytes read by lane 4e + i/4 (e = 0..3): 16
// lanes reading a 4-token x 16-column block each end up with 4 tokens of one column.
// The scan order only enters through the per-row token index in LDS.
#include <type_traits>

#include "gla_common.h"
#include "gla_mfma_util.h"

namespace gla {
namespace {

// LDS layout (byte offsets), sized by the padded head dimensions.
template <int MODE, int NDK8, int NDV16, bool BETA = false>
struct Layout {
    static constexpr int kDkp = NDK8 * 8;                                 // channels incl. padding to 8
    static constexpr int kDvp = NDV16 * 16;                               // value columns incl. padding to 16
    // bf16 per row of the channel-major operands: room for a multiple of 16 channels (the state update reads
    // 16-channel tiles) with one all-zero group of 8 after the data when dk is not a multiple of 32 (lanes whose
    // channel group lies beyond dk read that group instead of being masked), and an odd number of 16-byte units
    // per row so that the 16-byte operand reads of neighbouring rows fall into different LDS banks.
    static constexpr int kChStride = (NDK8 % 4 == 0) ? kDkp + 8 : ((kDkp + 8 + 15) / 16) * 16 + 8;
    static constexpr int kZeroCol = kDkp;                                 // first column of the all-zero group
    static constexpr int kVStride = kDvp + 8;                             // bf16 per row of V
    static constexpr int kLaStride = kDkp + 4;                            // fp32 per row of raw log_alpha
    static constexpr bool kOut = MODE == kModeOutput;
    static constexpr int kRowOp = kChunk * kChStride * 2;                 // one [64][channels] bf16 operand
    static constexpr int kV = kChunk * kVStride * 2;
    static constexpr int kSt = kDvp * kChStride * 2;

    static constexpr int oTok = 0;                                        // int[4][64] token of each row
    static constexpr int oTokG = oTok + 4 * kChunk * 4;                   // int[4][64] token whose gate the row uses
    static constexpr int oGam = oTokG + 4 * kChunk * 4;                   // float[64]  exp(b_C) of this chunk
    static constexpr int oLg = oGam + 64 * 4;                             // float[64]  sum of b_C over the span (base 2)
    static constexpr int oLa = oLg + 64 * 4;                              // raw log_alpha
    static constexpr int oKHi = oLa + kChunk * kLaStride * 4;             // raw k rows, then k~ hi in place
    static constexpr int oKLo = oKHi + kRowOp;
    static constexpr int oV = oKLo + kRowOp;
    static constexpr int oEndState = oV + kV;
    // output mode only
    static constexpr int oQHi = oEndState;                                // raw q rows, then q~ hi in place
    static constexpr int oQLo = oQHi + kRowOp;
    static constexpr int oStHi = oQLo + kRowOp;
    static constexpr int oStLo = oStHi + kSt;
    static constexpr int oLnW = oStLo + kSt;                              // float[kDvp] LayerNorm weight of this head
    static constexpr int oLnB = oLnW + kDvp * 4;                          // float[kDvp] LayerNorm bias
    static constexpr int oEndOut = oLnB + kDvp * 4;
    static constexpr int oEndAlpha = kOut ? oEndOut : oEndState;
    // two-sided gate only: raw log_beta rows (then exp(b^beta_j), the factor of output row j), the bf16 remainder
    // of the gated values, and per value column the chunk's total beta decay and its log summed over the span
    static constexpr int kLbStride = kDvp + 4;                            // fp32 per row of log_beta
    static constexpr int oLb = oEndAlpha;
    static constexpr int oVLo = oLb + kChunk * kLbStride * 4;
    static constexpr int oGamB = oVLo + kV;                               // float[kDvp]
    static constexpr int oLgB = oGamB + kDvp * 4;                         // float[kDvp]
    static constexpr int oEndBeta = oLgB + kDvp * 4;
    static constexpr int kBytes = BETA ? oEndBeta : oEndAlpha;
};

template <int N>
using int_c = std::integral_constant<int, N>;

// Which 16x16 tile of the dk x dv state is the i-th tile of wave w.  All tiles of a wave lie in one 16-channel row
// tile, so that its K~ operand is read once per chunk.  The output pass gives every row tile the same number of
// waves (the wave with the most score tiles then owns none); the state-only pass has nothing else to balance
// against and splits its waves over the row tiles as evenly as they divide (row tile ct: waves NW ct / NCT up to
// NW (ct + 1) / NCT), and the waves of a row tile take its value-column tiles in turn.
template <bool ROW_OWNED, int NW, int NCT, int NDV16>
struct TileMap {
    static_assert(ROW_OWNED || NW >= NCT, "state pass: at least one wave per row tile");
    static constexpr int WPC = (NW / NCT) > 0 ? NW / NCT : 1;  // waves sharing a row tile (the fewest, if uneven)
    static constexpr int kPerWave = (NDV16 + WPC - 1) / WPC;
    __host__ __device__ static constexpr int first_wave(int ct) { return NW * ct / NCT; }
    __host__ __device__ static constexpr int ct(int w, int = 0) {
        if (ROW_OWNED) return w / WPC;
        int c = 0;
        while (c + 1 < NCT && first_wave(c + 1) <= w) ++c;
        return c;
    }
    __host__ __device__ static constexpr int nt(int w, int i) {
        if (ROW_OWNED) return (w % WPC) + WPC * i;
        return (w - first_wave(ct(w))) + (first_wave(ct(w) + 1) - first_wave(ct(w))) * i;
    }
    __host__ __device__ static constexpr bool valid(int w, int i) {
        return ROW_OWNED ? (w / WPC < NCT && (w % WPC) + WPC * i < NDV16) : nt(w, i) < NDV16;
    }
    __host__ __device__ static constexpr int count(int w) {
        int n = 0;
        for (int i = 0; i < kPerWave; ++i) n += valid(w, i) ? 1 : 0;
        return n;
    }
};

// MINW = waves per SIMD the register budget must allow (4 -> 128 VGPRs, 2 -> 256 VGPRs).
// DEPTH = chunks of rows kept in flight from HBM (register sets; 2 only in the state pass).
// FUSE = the gate prologue (gates from bf16 pre-activations) and, in the output pass, the optional epilogue.
// ACC = the output pass adds its rows to the fp32 rows already in `out`.
// BETA = two-sided gate alpha_t^T beta_t (Eq. (gate_gla_2)): with c_j = sum_{i<=j} log beta_i inside a chunk, the
//        values are gated like the keys, v~_i = v_i exp(-c_i) (bf16 hi/lo), output row j is scaled by exp(c_j) and
//        state column n by exp(c_C[n]) per chunk.
template <int MODE, int NDK8, int NDV16, int NW, int MINW, int DEPTH, bool FUSE, bool ACC, typename TOut,
          bool BETA = false>
__global__ __launch_bounds__(NW * 64, MINW) void mfma_span_kernel(Params p) {
    using L = Layout<MODE, NDK8, NDV16, BETA>;
    constexpr bool OUT = MODE == kModeOutput;
    constexpr int NTHR = NW * 64;
    constexpr int CHS = L::kChStride;
    constexpr int VS = L::kVStride;
    constexpr int LAS = L::kLaStride;
    constexpr int KS = (NDK8 + 3) / 4;          // 32-channel steps of the channel contractions
    constexpr int NCT = (NDK8 + 1) / 2;         // 16-channel row tiles of the state
    using TM = TileMap<OUT, NW, NCT, NDV16>;
    constexpr int TPW = TM::kPerWave;           // state tiles per wave
    // With two sets in flight every row load is issued unconditionally (slots past the row or the span repeat a
    // valid piece), so that the number of younger loads is a constant and the waits can leave them in flight.
    constexpr bool UNCOND = OUT || DEPTH > 1;
    constexpr int NTB = DEPTH + 2;              // token-map buffers in LDS
    static_assert(NW == 4 || (NW == 8 && !OUT), "4 waves, or 8 in the state pass");
    static_assert(DEPTH == 1 || (DEPTH == 2 && !OUT), "two register sets only in the state pass");
    static_assert(NTB <= 4 && (DEPTH + 1) * kChunk <= NTHR, "token maps: four buffers, first ones filled in one go");
    static_assert(16 * NCT <= CHS, "state tiles must fit the operand row");
    static_assert(!ACC || (OUT && !FUSE && sizeof(TOut) == 4), "accumulation: plain output pass, fp32 rows");
    static_assert(!BETA || !ACC, "two-sided gate: no accumulation into existing rows");
    constexpr int LBS = L::kLbStride;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int *s_tok = reinterpret_cast<int *>(smem + L::oTok);
    int *s_tokg = reinterpret_cast<int *>(smem + L::oTokG);
    float *s_gam = reinterpret_cast<float *>(smem + L::oGam);
    float *s_lg = reinterpret_cast<float *>(smem + L::oLg);
    float *s_la = reinterpret_cast<float *>(smem + L::oLa);
    uint16_t *s_khi = reinterpret_cast<uint16_t *>(smem + L::oKHi);
    uint16_t *s_klo = reinterpret_cast<uint16_t *>(smem + L::oKLo);
    uint16_t *s_v = reinterpret_cast<uint16_t *>(smem + L::oV);
    uint16_t *s_qhi = reinterpret_cast<uint16_t *>(smem + L::oQHi);
    uint16_t *s_qlo = reinterpret_cast<uint16_t *>(smem + L::oQLo);
    uint16_t *s_sthi = reinterpret_cast<uint16_t *>(smem + L::oStHi);
    uint16_t *s_stlo = reinterpret_cast<uint16_t *>(smem + L::oStLo);
    float *s_lnw = reinterpret_cast<float *>(smem + L::oLnW);
    float *s_lnb = reinterpret_cast<float *>(smem + L::oLnB);
    float *s_lb = reinterpret_cast<float *>(smem + L::oLb);          // BETA only, like the three below
    uint16_t *s_vlo = reinterpret_cast<uint16_t *>(smem + L::oVLo);
    float *s_gamb = reinterpret_cast<float *>(smem + L::oGamB);
    float *s_lgb = reinterpret_cast<float *>(smem + L::oLgB);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave index, known uniform
    const int lm = lane & 15;
    const int g = lane >> 4;

    // Work-groups are dealt round-robin to the 8 XCDs; give each XCD a contiguous
    // range of spans so that neighbouring spans (which share cache lines in the
    // column scans) meet in one L2.
    int blk = blockIdx.x;
    {
        const int nb = gridDim.x;
        if ((nb & 7) == 0) blk = (blk & 7) * (nb >> 3) + (blk >> 3);
    }
    // spans per (batch, head) that this launch covers: the state pass leaves out the last one when the output
    // pass chains the span states itself (nothing reads that U)
    const int spans_here = (!OUT && p.chain_in_output) ? p.nspans - 1 : p.nspans;
    const int bh = blk / spans_here;
    int sp_ = blk - bh * spans_here;
    // Work-groups i and i + 32 of an XCD's range tend to share a compute unit.  When the output pass chains the
    // span states itself, the cost of that grows with the span index, so odd heads walk their spans backwards:
    // a compute unit then hosts a long and a short chain, and the group that ends first leaves it to the other.
    if (OUT && p.chain_in_output && (bh & 1)) sp_ = spans_here - 1 - sp_;
    const int sp = sp_;
    if constexpr (OUT) {
        // second opinion for the fp16 engine: a (batch, head) is recomputed if one of its spans raised its flag
        if (p.only_flagged) {
            int any = 0;
            for (int i = tid; i < p.fail_spans; i += NW * 64) any |= p.ws_fail[(size_t)bh * p.fail_spans + i];
            if (!__syncthreads_or(any)) return;   // (uniform over the group)
        }
    }
    const int dk = p.dk, dv = p.dv, T = p.T;
    const int s_begin = sp * p.span_len;
    const int s_end = min(T, s_begin + p.span_len);
    const int nch = (s_end - s_begin + kChunk - 1) / kChunk;

    // per-(batch, head) bases; everything below is a 32-bit byte offset from them
    const size_t base_k = slab_k(p, bh), base_v = slab_v(p, bh);
    const char *gq = static_cast<const char *>(p.q) + base_k * 2;
    const char *gk = static_cast<const char *>(p.k) + base_k * 2;
    const char *gv = static_cast<const char *>(p.v) + base_v * 2;
    const char *gla_ = reinterpret_cast<const char *>(p.log_alpha) + base_k * 4;
    const char *glb = reinterpret_cast<const char *>(p.log_beta) + base_v * 4;
    const char *gz = static_cast<const char *>(p.z_gate) + base_k * 2;
    const char *gzb = static_cast<const char *>(p.z_beta) + base_v * 2;
    const char *grp = static_cast<const char *>(p.r_pre) + base_v * 2;
    const bool epilogue = FUSE && OUT && p.r_pre != nullptr;   // uniform
    char *gout = static_cast<char *>(p.out) + base_v * sizeof(TOut);

    // ---- state tiles owned by this wave (TileMap) ----
    f32x4 acc[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- state entering the span, chained here from the local states of the spans before it ----
    // S_start(sp) = sum_{r < sp} diag(prod_{r < r' < sp} Gamma_r') U_r, summed from the nearest span backwards on
    // 4 consecutive state elements per thread (one key channel: dv % 4 == 0) until the accumulated decay makes the
    // remaining terms vanish in fp32 (chain_span_states); the result goes through LDS into the accumulator layout.
    if constexpr (OUT) {
        const bool chain = p.chain_in_output && (sp > 0 || p.initial_state != nullptr);  // uniform over the group
        if (chain) {
            constexpr int kV4 = (L::kDkp * L::kDvp / 4 + NTHR - 1) / NTHR;  // float4 per thread
            constexpr int kBudget = MINW >= 4 ? 16 : 32;                    // float4 in flight: 64 or 128 registers of U
            constexpr int kRun = kBudget / kV4 > 0 ? kBudget / kV4 : 1;     // spans in flight
            chain_span_states<NTHR, kV4, kRun, BETA>(p, bh, sp, tid, reinterpret_cast<float *>(smem));
        }
        __syncthreads();
        if (chain) {
            const float *s_chain = reinterpret_cast<const float *>(smem);
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                if (TM::valid(w, i)) {
                    const int n = 16 * TM::nt(w, i) + lm;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int c = 16 * TM::ct(w, i) + 4 * g + r;
                        if (c < dk && n < dv) acc[i][r] = s_chain[c * dv + n];
                    }
                }
            }
        }
        __syncthreads();
    }

    // ---- prologue: clear LDS (pads must read as zero), token maps of the first two chunks ----
    for (int i = tid; i < L::kBytes / 16; i += NTHR)
        reinterpret_cast<u32x4 *>(smem)[i] = u32x4{0, 0, 0, 0};
    __syncthreads();
    if constexpr (FUSE && OUT) {
        if (epilogue) {
            const int h = bh % p.H;
            for (int n = tid; n < dv; n += NTHR) {
                s_lnw[n] = p.ln_weight != nullptr ? p.ln_weight[h * dv + n] : 1.f;
                s_lnb[n] = p.ln_bias != nullptr ? p.ln_bias[h * dv + n] : 0.f;
            }
        }
    }
    if (tid < (DEPTH + 1) * kChunk) {
        const int s = s_begin + tid;
        const int sc = (s < s_end) ? s : s_begin;
        s_tok[tid] = scan_token(p.scan_dir, sc, T, p.grid_h, p.grid_w);
        s_tokg[tid] = scan_token(p.scan_dir, max(sc - p.gate_shift, 0), T, p.grid_h, p.grid_w);
    }
    __syncthreads();

    // ---- or the state entering the span as the carry kernel left it (single span: the caller's state) ----
    const float *s0 = nullptr;
    if (OUT && p.nspans > 1 && !p.chain_in_output)
        s0 = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;
    else if (OUT && p.nspans == 1 && p.initial_state != nullptr)
        s0 = p.initial_state + (size_t)bh * dk * dv;
    if (s0 != nullptr) {
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            if (TM::valid(w, i)) {
                const int n = 16 * TM::nt(w, i) + lm;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int c = 16 * TM::ct(w, i) + 4 * g + r;
                    if (c < dk && n < dv) acc[i][r] = s0[c * dv + n];
                }
            }
        }
    }
    // The start state must have landed before the chunk loop: the compiler's wait-count tracking would otherwise
    // make every later read of `acc` wait for all outstanding loads, i.e. for the prefetch of the next chunk.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

    // ---- which HBM pieces this thread stages (the same for every chunk) ----
    // A row of log_alpha is cut into 16-byte pieces (4 channels), a row of q or k into 8-byte pieces (the same
    // 4 channels), a row of v into 16-byte pieces (8 columns).  The pieces of a chunk are numbered row by row and
    // slot m of a thread is piece tid + NTHR m: the lanes of a wave then fetch neighbouring pieces of
    // neighbouring rows (one contiguous kilobyte when the scan visits rows that are neighbours in memory).
    // Slots past the last piece repeat it (the load stays in bounds; nothing is written to LDS for them).
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
    const uint32_t dk2 = 2u * (uint32_t)p.st_k, dv2 = 2u * (uint32_t)p.st_v;  // bytes from one bf16 row to the next

    f32x4 r_la[DEPTH][kF];
    u32x2 r_z[DEPTH][FUSE ? kF : 1];   // gate pre-activations (bf16) in place of log_alpha rows
    u32x2 r_k[DEPTH][kF];
    u32x2 r_q[DEPTH][OUT ? kF : 1];
    u32x4 r_v[DEPTH][kVF];
    f32x4 r_lb[DEPTH][BETA ? kVF : 1][2];   // log_beta of the same 8 columns as the v piece
    u32x4 r_zb[DEPTH][(BETA && FUSE) ? kVF : 1];   // or their pre-activations (bf16)

    // Rows past the end of a ragged last chunk carry the token of a valid row in s_tok (so the loads
    // stay in bounds) and are zeroed when they are written to LDS.
    auto load_chunk = [&](int chunk, auto set_c) {
        constexpr int S = decltype(set_c)::value;
        const int *tok = s_tok + (chunk % NTB) * kChunk;
        const int *tokg = s_tokg + (chunk % NTB) * kChunk;
#pragma unroll
        for (int m = 0; m < kF; ++m) {
            const int row = frp[m] >> 8;
            const uint32_t pc = 8u * (uint32_t)(frp[m] & 255);
            const uint32_t e2 = (uint32_t)tok[row] * dk2 + pc;
            const uint32_t eg = (uint32_t)tokg[row] * dk2 + pc;
            if constexpr (FUSE) r_z[S][m] = *reinterpret_cast<const u32x2 *>(gz + eg);
            else r_la[S][m] = *reinterpret_cast<const f32x4 *>(gla_ + 2u * eg);
            r_k[S][m] = *reinterpret_cast<const u32x2 *>(gk + e2);
            if constexpr (OUT) r_q[S][m] = *reinterpret_cast<const u32x2 *>(gq + e2);
        }
#pragma unroll
        for (int m = 0; m < kVF; ++m) {
            r_v[S][m] = *reinterpret_cast<const u32x4 *>(gv + (uint32_t)tok[fvrp[m] >> 8] * dv2 + 16u * (uint32_t)(fvrp[m] & 255));
            if constexpr (BETA && FUSE) {
                r_zb[S][m] = *reinterpret_cast<const u32x4 *>(gzb + (uint32_t)tokg[fvrp[m] >> 8] * dv2 + 16u * (uint32_t)(fvrp[m] & 255));
            } else if constexpr (BETA) {
                const char *lbp = glb + 2u * ((uint32_t)tokg[fvrp[m] >> 8] * dv2 + 16u * (uint32_t)(fvrp[m] & 255));
                r_lb[S][m][0] = *reinterpret_cast<const f32x4 *>(lbp);
                r_lb[S][m][1] = *reinterpret_cast<const f32x4 *>(lbp + 16);
            }
        }
    };

    // ---- gate work of this wave: whole UW-channel units w, w+NW, ..., then single left-over channels ----
    constexpr int UW = 32 / NW;                       // channels per unit: 16-byte LDS rows accesses for 4 waves
    const int nunits = dk / UW;
    const int upw = (nunits + NW - 1) / NW;           // units of the busiest wave
    const int left0 = UW * nunits;                    // first left-over channel (none with 4-channel units)
    const int lpw = (dk - left0 + NW - 1) / NW;       // left-over channels per wave
    constexpr int kMaxUnits = (kMaxDk / UW + NW - 1) / NW;
    constexpr int kMaxLeft = (UW - 4 + NW - 1) / NW;

    load_chunk(0, int_c<0>{});
    if constexpr (DEPTH == 2) {
        load_chunk(1, int_c<1>{});
    }

    auto process_chunk = [&](int chunk, auto set_c) {
        constexpr int S = decltype(set_c)::value;       // register set that holds this chunk's rows
        const int *tok = s_tok + (chunk % NTB) * kChunk;

        // ================= (a) registers -> LDS =================
        const int nvalid = min(kChunk, s_end - s_begin - chunk * kChunk);  // rows of this chunk that are tokens
        if constexpr (FUSE) {
            // log2(alpha) = log2(sigmoid(z)) / tau = (min(t, 0) - log2(1 + 2^-|t|)) / tau with t = z log2(e)
            auto gate2 = [&](uint32_t pair, float &lo, float &hi) {
                const float t0 = bf16_lo_as_float(pair) * kLog2e, t1 = bf16_hi_as_float(pair) * kLog2e;
                lo = (fminf(t0, 0.f) - __builtin_amdgcn_logf(1.f + exp2_fast(-fabsf(t0)))) * p.inv_tau;
                hi = (fminf(t1, 0.f) - __builtin_amdgcn_logf(1.f + exp2_fast(-fabsf(t1)))) * p.inv_tau;
            };
#pragma unroll
            for (int m = 0; m < kF; ++m) {
                f32x4 la;
                float a0, a1, a2, a3;
                gate2(r_z[S][m][0], a0, a1);
                gate2(r_z[S][m][1], a2, a3);
                la = f32x4{a0, a1, a2, a3};
                r_la[S][m] = la;
            }
            if constexpr (BETA) {
#pragma unroll
                for (int m = 0; m < kVF; ++m) {
                    float b0, b1, b2, b3, b4, b5, b6, b7;
                    gate2(r_zb[S][m][0], b0, b1);
                    gate2(r_zb[S][m][1], b2, b3);
                    gate2(r_zb[S][m][2], b4, b5);
                    gate2(r_zb[S][m][3], b6, b7);
                    r_lb[S][m][0] = f32x4{b0, b1, b2, b3};
                    r_lb[S][m][1] = f32x4{b4, b5, b6, b7};
                }
            }
        }
        if (nvalid < kChunk) {
#pragma unroll
            for (int m = 0; m < kF; ++m) {
                if ((frp[m] >> 8) >= nvalid) {
                    r_la[S][m] = f32x4{0.f, 0.f, 0.f, 0.f};
                    r_k[S][m] = u32x2{0, 0};
                    if constexpr (OUT) r_q[S][m] = u32x2{0, 0};
                }
            }
#pragma unroll
            for (int m = 0; m < kVF; ++m) {
                if ((fvrp[m] >> 8) >= nvalid) {
                    r_v[S][m] = u32x4{0, 0, 0, 0};
                    if constexpr (BETA) r_lb[S][m][0] = r_lb[S][m][1] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            }
        }
#pragma unroll
        for (int m = 0; m < kF; ++m) {
            if (tid + NTHR * m < kChunk * pcs) {
                const int row = frp[m] >> 8, ch = 4 * (frp[m] & 255);
                *reinterpret_cast<f32x4 *>(s_la + row * LAS + ch) = r_la[S][m];
                *reinterpret_cast<u32x2 *>(s_khi + row * CHS + ch) = r_k[S][m];
                if constexpr (OUT) *reinterpret_cast<u32x2 *>(s_qhi + row * CHS + ch) = r_q[S][m];
            }
        }
#pragma unroll
        for (int m = 0; m < kVF; ++m) {
            if (tid + NTHR * m < kChunk * vpcs) {
                *reinterpret_cast<u32x4 *>(s_v + (fvrp[m] >> 8) * VS + 8 * (fvrp[m] & 255)) = r_v[S][m];
                if constexpr (BETA) {
                    float *lrow = s_lb + (fvrp[m] >> 8) * LBS + 8 * (fvrp[m] & 255);
                    *reinterpret_cast<f32x4 *>(lrow) = r_lb[S][m][0];
                    *reinterpret_cast<f32x4 *>(lrow + 4) = r_lb[S][m][1];
                }
            }
        }
        // the rows of a later chunk start their trip from HBM into the set just emptied
        // (unconditional loads past the span: the clamped token map makes every lane read one row)
        if (UNCOND || chunk + DEPTH < nch) load_chunk(chunk + DEPTH, set_c);
        if constexpr (OUT) {
            // S_0 (state entering the chunk) as bf16 hi/lo, value-column-major for the B operand
            // (state rows past dk are exactly zero and land in the zero padding of the row)
            const int ln = recompute_per_chunk(lane), lm = ln & 15, g = ln >> 4;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                if (TM::valid(w, i)) {
                    u32x2 hi, lo;
                    SPLIT_PAIR(acc[i][0], acc[i][1], hi[0], lo[0]);
                    SPLIT_PAIR(acc[i][2], acc[i][3], hi[1], lo[1]);
                    const int off = (16 * TM::nt(w, i) + lm) * CHS + 16 * TM::ct(w, i) + 4 * g;
                    *reinterpret_cast<u32x2 *>(s_sthi + off) = hi;
                    *reinterpret_cast<u32x2 *>(s_stlo + off) = lo;
                }
            }
        }
        if (w == NW - 1 && (UNCOND || chunk + DEPTH + 1 < nch)) {  // token map of the chunk loaded next time, by the last wave
            const int s = s_begin + (chunk + DEPTH + 1) * kChunk + lane;
            const int sc = (s < s_end) ? s : s_begin;
            s_tok[((chunk + DEPTH + 1) % NTB) * kChunk + lane] = scan_token(p.scan_dir, sc, T, p.grid_h, p.grid_w);
            s_tokg[((chunk + DEPTH + 1) % NTB) * kChunk + lane] =
                scan_token(p.scan_dir, max(sc - p.gate_shift, 0), T, p.grid_h, p.grid_w);
        }
        __syncthreads();

        // ================= (b) gates: lane = token =================
        {
            const int j = lane;
#pragma unroll
            for (int ui = 0; ui < kMaxUnits; ++ui) {
                if (ui < upw && w + NW * ui < nunits) {
                    const int c0 = UW * (w + NW * ui);
                    float bb[UW];
#pragma unroll
                    for (int v4 = 0; v4 < UW / 4; ++v4) {
                        const f32x4 x = *reinterpret_cast<const f32x4 *>(s_la + j * LAS + c0 + 4 * v4);
#pragma unroll
                        for (int i = 0; i < 4; ++i) bb[4 * v4 + i] = FUSE ? x[i] : x[i] * kLog2e;
                        wave_inclusive_scan4(bb[4 * v4], bb[4 * v4 + 1], bb[4 * v4 + 2], bb[4 * v4 + 3]);
                    }
                    uint32_t kr[UW / 2], khi[UW / 2], klo[UW / 2];
#pragma unroll
                    for (int v2 = 0; v2 < UW / 4; ++v2) {
                        const u32x2 t = *reinterpret_cast<const u32x2 *>(s_khi + j * CHS + c0 + 4 * v2);
                        kr[2 * v2] = t[0];
                        kr[2 * v2 + 1] = t[1];
                    }
#pragma unroll
                    for (int h = 0; h < UW / 2; ++h)
                        SPLIT_PAIR(bf16_lo_as_float(kr[h]) * exp2_fast(fminf(-bb[2 * h], kMaxExp2)),
                                   bf16_hi_as_float(kr[h]) * exp2_fast(fminf(-bb[2 * h + 1], kMaxExp2)),
                                   khi[h], klo[h]);
#pragma unroll
                    for (int v2 = 0; v2 < UW / 4; ++v2) {
                        *reinterpret_cast<u32x2 *>(s_khi + j * CHS + c0 + 4 * v2) = u32x2{khi[2 * v2], khi[2 * v2 + 1]};
                        *reinterpret_cast<u32x2 *>(s_klo + j * CHS + c0 + 4 * v2) = u32x2{klo[2 * v2], klo[2 * v2 + 1]};
                    }
                    if constexpr (OUT) {
                        uint32_t qr[UW / 2], qhi[UW / 2], qlo[UW / 2];
                        float eq[UW];
#pragma unroll
                        for (int v2 = 0; v2 < UW / 4; ++v2) {
                            const u32x2 t = *reinterpret_cast<const u32x2 *>(s_qhi + j * CHS + c0 + 4 * v2);
                            qr[2 * v2] = t[0];
                            qr[2 * v2 + 1] = t[1];
                        }
#pragma unroll
                        for (int h = 0; h < UW / 2; ++h) {
                            eq[2 * h] = exp2_fast(bb[2 * h]);
                            eq[2 * h + 1] = exp2_fast(bb[2 * h + 1]);
                            SPLIT_PAIR(bf16_lo_as_float(qr[h]) * eq[2 * h], bf16_hi_as_float(qr[h]) * eq[2 * h + 1],
                                       qhi[h], qlo[h]);
                        }
#pragma unroll
                        for (int v2 = 0; v2 < UW / 4; ++v2) {
                            *reinterpret_cast<u32x2 *>(s_qhi + j * CHS + c0 + 4 * v2) = u32x2{qhi[2 * v2], qhi[2 * v2 + 1]};
                            *reinterpret_cast<u32x2 *>(s_qlo + j * CHS + c0 + 4 * v2) = u32x2{qlo[2 * v2], qlo[2 * v2 + 1]};
                        }
                        if (lane == 63) {  // the last token's exp(b) is the chunk's total decay
#pragma unroll
                            for (int v4 = 0; v4 < UW / 4; ++v4)
                                *reinterpret_cast<f32x4 *>(s_gam + c0 + 4 * v4) =
                                    f32x4{eq[4 * v4], eq[4 * v4 + 1], eq[4 * v4 + 2], eq[4 * v4 + 3]};
                        }
                    } else if (lane == 63) {
#pragma unroll
                        for (int v4 = 0; v4 < UW / 4; ++v4) {
                            f32x4 l0 = *reinterpret_cast<const f32x4 *>(s_lg + c0 + 4 * v4);
                            f32x4 g0;
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                g0[i] = exp2_fast(bb[4 * v4 + i]);
                                l0[i] += bb[4 * v4 + i];
                            }
                            *reinterpret_cast<f32x4 *>(s_gam + c0 + 4 * v4) = g0;
                            *reinterpret_cast<f32x4 *>(s_lg + c0 + 4 * v4) = l0;
                        }
                    }
                }
            }
#pragma unroll
            for (int li = 0; li < kMaxLeft; ++li) {
                const int c = left0 + w * lpw + li;
                if (li < lpw && c < dk) {
                    const float b = wave_inclusive_scan(FUSE ? s_la[j * LAS + c] : s_la[j * LAS + c] * kLog2e);
                    const float kx = bf16_bits_to_float(s_khi[j * CHS + c]) * exp2_fast(fminf(-b, kMaxExp2));
                    float qx = 0.f, e = 0.f;
                    if constexpr (OUT) {
                        e = exp2_fast(b);
                        qx = bf16_bits_to_float(s_qhi[j * CHS + c]) * e;
                    }
                    uint32_t h2, l2;
                    SPLIT_PAIR(kx, qx, h2, l2);
                    s_khi[j * CHS + c] = (uint16_t)(h2 & 0xffffu);
                    s_klo[j * CHS + c] = (uint16_t)(l2 & 0xffffu);
                    if constexpr (OUT) {
                        s_qhi[j * CHS + c] = (uint16_t)(h2 >> 16);
                        s_qlo[j * CHS + c] = (uint16_t)(l2 >> 16);
                        if (lane == 63) s_gam[c] = e;
                    } else if (lane == 63) {
                        s_gam[c] = exp2_fast(b);
                        s_lg[c] += b;
                    }
                }
            }
            if constexpr (BETA) {
                // value side: 8-column units dealt round-robin; v~ = v exp(-c) as bf16 hi/lo, exp(c) left in
                // place of the log_beta row, lane 63 holds the chunk's total
                for (int c0 = 8 * w; c0 < dv; c0 += 8 * NW) {
                    float cc[8];
#pragma unroll
                    for (int v4 = 0; v4 < 2; ++v4) {
                        const f32x4 x = *reinterpret_cast<const f32x4 *>(s_lb + j * LBS + c0 + 4 * v4);
#pragma unroll
                        for (int i = 0; i < 4; ++i) cc[4 * v4 + i] = FUSE ? x[i] : x[i] * kLog2e;
                        wave_inclusive_scan4(cc[4 * v4], cc[4 * v4 + 1], cc[4 * v4 + 2], cc[4 * v4 + 3]);
                    }
                    const u32x4 vr = *reinterpret_cast<const u32x4 *>(s_v + j * VS + c0);
                    u32x4 vh, vl;
                    float ev[8];
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        SPLIT_PAIR(bf16_lo_as_float(vr[h]) * exp2_fast(fminf(-cc[2 * h], kMaxExp2)),
                                   bf16_hi_as_float(vr[h]) * exp2_fast(fminf(-cc[2 * h + 1], kMaxExp2)),
                                   vh[h], vl[h]);
                        ev[2 * h] = exp2_fast(cc[2 * h]);
                        ev[2 * h + 1] = exp2_fast(cc[2 * h + 1]);
                    }
                    *reinterpret_cast<u32x4 *>(s_v + j * VS + c0) = vh;
                    *reinterpret_cast<u32x4 *>(s_vlo + j * VS + c0) = vl;
                    if constexpr (OUT) {
                        *reinterpret_cast<f32x4 *>(s_lb + j * LBS + c0) = f32x4{ev[0], ev[1], ev[2], ev[3]};
                        *reinterpret_cast<f32x4 *>(s_lb + j * LBS + c0 + 4) = f32x4{ev[4], ev[5], ev[6], ev[7]};
                    }
                    if (lane == 63) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            s_gamb[c0 + i] = ev[i];
                            if constexpr (!OUT) s_lgb[c0 + i] += cc[i];
                        }
                    }
                }
            }
        }
        __syncthreads();

        // ================= (c) contractions =================
        // One straight-line body per wave index: which tiles a wave owns is then known at compile time and the
        // LDS reads and MFMAs of different tiles can be interleaved freely.
        // The scheduler is fenced between batches: the LDS reads of batch k+1 are issued before the MFMAs of
        // batch k, so one wait covers a whole batch instead of one wait per operand.
        // per-lane LDS offsets (bf16 elements), derived afresh in every chunk: kept across the loop they would
        // occupy registers through the staging and gate stages as well
        const int ln = recompute_per_chunk(lane), lm = ln & 15, g = ln >> 4;
        // channel group read by this lane in 32-channel step ks; groups beyond dk alias the all-zero group
        int colk[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) colk[ks] = (4 * ks + g < NDK8) ? 8 * (4 * ks + g) : L::kZeroCol;
        // transposing reads: this lane supplies row lm/4 (of 4 tokens) and column quad lm%4 (of 16 columns)
        const int tr_row = lm >> 2, tr_col = 4 * (lm & 3);
        auto contract = [&](auto wave_c) {
            constexpr int W = decltype(wave_c)::value;
            constexpr int IT = W & 3;                       // 16-row output tile of this wave (output pass)
            constexpr int NTW = TM::count(W);               // state tiles of this wave

            // Contraction slot (g, e) of the 32-token step q32 is token 32 q32 + 16 (e/4) + 4g + e%4, for every
            // operand that is contracted over tokens (the layout in which the score tiles leave the MFMA).
            // ---- state-update operands: K~ (A operand) and V (B operand).  With row-owned tiles the K~ operand
            // is read once per chunk, and the V operand is the one the output rows were computed with.
            const uint16_t *krow_h = s_khi + (4 * g + tr_row) * CHS + tr_col;
            const uint16_t *krow_l = s_klo + (4 * g + tr_row) * CHS + tr_col;
            const uint16_t *vrow = s_v + (4 * g + tr_row) * VS + tr_col;
            const uint16_t *vrow_l = s_vlo + (4 * g + tr_row) * VS + tr_col;   // BETA: remainder of the gated values
            u32x2 ukh[1][2][2], ukl[1][2][2];               // [0][32-token step][half]: shared by the wave's tiles
            auto load_state_k = [&](int buf, int i) {
                const int ko = 16 * TM::ct(W, i);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    ukh[buf][ks][0] = lds_read_tr(krow_h + 32 * ks * CHS + ko);
                    ukh[buf][ks][1] = lds_read_tr(krow_h + (32 * ks + 16) * CHS + ko);
                    ukl[buf][ks][0] = lds_read_tr(krow_l + 32 * ks * CHS + ko);
                    ukl[buf][ks][1] = lds_read_tr(krow_l + (32 * ks + 16) * CHS + ko);
                }
            };
            // S = diag(exp(b_C)) (S + K~^T V) on state tile i; b0, b1 = V fragments of the two 32-token steps
            // (BETA: V~ hi with its remainders b0l, b1l, and column n of the tile also decays by exp(c_C[n]))
            auto update_state = [&](int kb, int i, const u32x4 &b0, const u32x4 &b1, const u32x4 &b0l,
                                    const u32x4 &b1l) {
                f32x4 a = acc[i];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const u32x4 b = ks == 0 ? b0 : b1;
                    const u32x4 kh = u32x4{ukh[kb][ks][0][0], ukh[kb][ks][0][1], ukh[kb][ks][1][0], ukh[kb][ks][1][1]};
                    a = mfma(kh, b, a);
                    a = mfma(u32x4{ukl[kb][ks][0][0], ukl[kb][ks][0][1], ukl[kb][ks][1][0], ukl[kb][ks][1][1]}, b, a);
                    if constexpr (BETA) {
                        a = mfma(kh, ks == 0 ? b0l : b1l, a);
                        a = mfma(u32x4{ukl[kb][ks][0][0], ukl[kb][ks][0][1], ukl[kb][ks][1][0], ukl[kb][ks][1][1]},
                                 ks == 0 ? b0l : b1l, a);
                    }
                }
                f32x4 gm = *reinterpret_cast<const f32x4 *>(s_gam + 16 * TM::ct(W, i) + 4 * g);
                if constexpr (BETA) {
                    const float gbn = s_gamb[16 * TM::nt(W, i) + lm];
#pragma unroll
                    for (int r = 0; r < 4; ++r) gm[r] *= gbn;
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) a[r] *= gm[r];
                acc[i] = a;
            };

            if constexpr (OUT) {
                constexpr int NX = NDV16;          // this wave's 16 output rows span all value-column tiles
                const uint16_t *qrow_h = s_qhi + (16 * IT + lm) * CHS, *qrow_l = s_qlo + (16 * IT + lm) * CHS;
                // When the last 32-channel step holds a single 8-channel group (dk = 33..40, or dk <= 8), its four
                // products hi*hi, hi*lo, lo*hi, lo*lo share one MFMA: lane groups g = 0..3 of the gated operand and
                // of S_0 read (hi, hi, lo, lo) of that channel group, those of Q~ read (hi, lo, hi, lo).
                // The "hi" arrays then hold the packed fragment of that step and the "lo" entry is unused.
                constexpr bool PT = NDK8 % 4 == 1;
                constexpr int TC = 32 * (KS - 1);  // first channel of the last step
                const uint16_t *ktail = (g >= 2 ? s_klo : s_khi) + TC;
                const uint16_t *qtail = ((g & 1) ? s_qlo : s_qhi) + TC;
                const uint16_t *sttail = (g >= 2 ? s_stlo : s_sthi) + TC;
                u32x4 qfh[KS], qfl[KS];            // Q~ fragments of this wave's 16 output rows
                u32x4 kfh[2][KS], kfl[2][KS];      // K~ fragments of two score tiles
                u32x2 vt[2][NX][2];                // V fragments of the two 32-token steps
                u32x2 vtl[2][BETA ? NX : 1][2];    // BETA: their remainders
                u32x4 sth[2][NX], stl[2][NX];      // S_0 fragments of one 32-channel step, two buffers
                u32x2 ph[2], pl[2];                // two score tiles as bf16 hi/lo (A operand of O += A V)
                f32x4 o[NX];
                auto load_ktile = [&](int u, int jt) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        if (PT && ks == KS - 1) {
                            kfh[u][ks] = *reinterpret_cast<const u32x4 *>(ktail + (16 * jt + lm) * CHS);
                        } else {
                            kfh[u][ks] = *reinterpret_cast<const u32x4 *>(s_khi + (16 * jt + lm) * CHS + colk[ks]);
                            kfl[u][ks] = *reinterpret_cast<const u32x4 *>(s_klo + (16 * jt + lm) * CHS + colk[ks]);
                        }
                    }
                };
                auto load_v = [&](int q32) {
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        vt[q32][x][0] = lds_read_tr(vrow + 32 * q32 * VS + 16 * x);
                        vt[q32][x][1] = lds_read_tr(vrow + (32 * q32 + 16) * VS + 16 * x);
                        if constexpr (BETA) {
                            vtl[q32][x][0] = lds_read_tr(vrow_l + 32 * q32 * VS + 16 * x);
                            vtl[q32][x][1] = lds_read_tr(vrow_l + (32 * q32 + 16) * VS + 16 * x);
                        }
                    }
                };
                auto v_frag = [&](int q32, int x) {
                    return u32x4{vt[q32][x][0][0], vt[q32][x][0][1], vt[q32][x][1][0], vt[q32][x][1][1]};
                };
                auto v_frag_lo = [&](int q32, int x) {   // (without BETA: unused by the callee)
                    if constexpr (BETA)
                        return u32x4{vtl[q32][x][0][0], vtl[q32][x][0][1], vtl[q32][x][1][0], vtl[q32][x][1][1]};
                    else
                        return v_frag(q32, x);
                };
                auto load_st = [&](int buf, int ks) {
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        if (PT && ks == KS - 1) {
                            sth[buf][x] = *reinterpret_cast<const u32x4 *>(sttail + (16 * x + lm) * CHS);
                        } else {
                            const int srow = (16 * x + lm) * CHS + colk[ks];
                            sth[buf][x] = *reinterpret_cast<const u32x4 *>(s_sthi + srow);
                            stl[buf][x] = *reinterpret_cast<const u32x4 *>(s_stlo + srow);
                        }
                    }
                };
                // score tile, transposed: lane (lm, g) gets A[i = 16 IT + lm][j = 16 jt + 4g + r]
                auto score_tile = [&](int u, int jt) {
                    f32x4 d = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        d = mfma(kfh[u][ks], qfh[ks], d);
                        if (PT && ks == KS - 1) continue;
                        d = mfma(kfh[u][ks], qfl[ks], d);
                        d = mfma(kfl[u][ks], qfh[ks], d);
                        d = mfma(kfl[u][ks], qfl[ks], d);
                    }
                    if (jt == IT) {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (4 * g + r > lm) d[r] = 0.f;
                    }
                    SPLIT_PAIR(d[0], d[1], ph[u][0], pl[u][0]);
                    SPLIT_PAIR(d[2], d[3], ph[u][1], pl[u][1]);
                };
                // O^T += V^T A^T : lane (lm, g) accumulates o[x][r] = O[i = 16 IT + lm][n = 16 x + 4g + r]
                auto av = [&](int q32) {
                    const u32x4 ah = u32x4{ph[0][0], ph[0][1], ph[1][0], ph[1][1]};
                    const u32x4 al = u32x4{pl[0][0], pl[0][1], pl[1][0], pl[1][1]};
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        const u32x4 b = v_frag(q32, x);
                        o[x] = mfma(b, ah, o[x]);
                        o[x] = mfma(b, al, o[x]);
                        if constexpr (BETA) {
                            o[x] = mfma(v_frag_lo(q32, x), ah, o[x]);
                            o[x] = mfma(v_frag_lo(q32, x), al, o[x]);
                        }
                    }
                };
                auto qs = [&](int buf, int ks) {
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        o[x] = mfma(sth[buf][x], qfh[ks], o[x]);
                        if (PT && ks == KS - 1) continue;
                        o[x] = mfma(sth[buf][x], qfl[ks], o[x]);
                        o[x] = mfma(stl[buf][x], qfh[ks], o[x]);
                        o[x] = mfma(stl[buf][x], qfl[ks], o[x]);
                    }
                };
                // what the state update still has to read: its K~ operand, and the second 32 tokens of V when the
                // causal part of this wave's rows ended before them
                auto load_state_first = [&]() {
                    if constexpr (NTW > 0) {
                        load_state_k(0, 0);
                        if constexpr (IT < 2) load_v(1);
                    }
                };

#pragma unroll
                for (int x = 0; x < NX; ++x) o[x] = f32x4{0.f, 0.f, 0.f, 0.f};
                // epilogue operand: this lane's four columns per tile of the output-gate pre-activations, fetched
                // now so that they have arrived when the rows are complete (rows past the span repeat a valid token)
                u32x2 rg[FUSE ? NX : 1];
                if constexpr (FUSE) {
                    if (epilogue) {
                        const char *rrow = grp + ((uint32_t)tok[16 * IT + lm] * (uint32_t)p.st_v + 4u * (uint32_t)g) * 2u;
#pragma unroll
                        for (int x = 0; x < NX; ++x)
                            rg[x] = (4 * g + 16 * x < dv) ? *reinterpret_cast<const u32x2 *>(rrow + 32 * x) : u32x2{0, 0};
                    }
                }
                // rows to add to, fetched now so that they have arrived when this chunk's rows are complete
                f32x4 prev[ACC ? NX : 1];
                if constexpr (ACC) {
                    const char *prow_ = gout + ((uint32_t)tok[16 * IT + lm] * (uint32_t)p.st_v + 4u * (uint32_t)g) * 4u;
#pragma unroll
                    for (int x = 0; x < NX; ++x)
                        prev[x] = (4 * g + 16 * x < dv) ? *reinterpret_cast<const f32x4 *>(prow_ + 64 * x)
                                                        : f32x4{0.f, 0.f, 0.f, 0.f};
                }
                ph[1] = u32x2{0, 0};
                pl[1] = u32x2{0, 0};
                // batch 0: Q~ and the first two score tiles' K~
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    if (PT && ks == KS - 1) {
                        qfh[ks] = *reinterpret_cast<const u32x4 *>(qtail + (16 * IT + lm) * CHS);
                    } else {
                        qfh[ks] = *reinterpret_cast<const u32x4 *>(qrow_h + colk[ks]);
                        qfl[ks] = *reinterpret_cast<const u32x4 *>(qrow_l + colk[ks]);
                    }
                }
                load_ktile(0, 0);
                if constexpr (IT >= 1) load_ktile(1, 1);
                __builtin_amdgcn_sched_barrier(0);
                load_v(0);
                score_tile(0, 0);
                if constexpr (IT >= 1) score_tile(1, 1);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (IT >= 2) {
                    load_ktile(0, 2);
                    if constexpr (IT >= 3) load_ktile(1, 3);
                    av(0);
                    __builtin_amdgcn_sched_barrier(0);
                    load_v(1);
                    ph[1] = u32x2{0, 0};
                    pl[1] = u32x2{0, 0};
                    score_tile(0, 2);
                    if constexpr (IT >= 3) score_tile(1, 3);
                    __builtin_amdgcn_sched_barrier(0);
                }
                load_st(0, 0);
                av(IT >= 2 ? 1 : 0);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (KS > 1) load_st(1, 1);
                else load_state_first();
                qs(0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (KS > 1) {
                    load_state_first();
                    qs(1, 1);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (BETA) {
                    // row j of the output carries exp(c_j) per value column
                    const float *erow = s_lb + (16 * IT + lm) * LBS + 4 * g;
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        if (4 * g + 16 * x < dv) {
                            const f32x4 e4 = *reinterpret_cast<const f32x4 *>(erow + 16 * x);
#pragma unroll
                            for (int r = 0; r < 4; ++r) o[x][r] *= e4[r];
                        }
                    }
                }
                if constexpr (FUSE) {
                    if (epilogue) {
                        // Swish(r) * LN(o): a token's row is spread over the four lanes lm, lm+16, lm+32, lm+48
                        // (columns past dv are exact zeros: they add nothing to the sum and are left out of the
                        // squares)
                        const float inv_n = 1.f / (float)dv;
                        float sum = 0.f;
#pragma unroll
                        for (int x = 0; x < NX; ++x) sum += (o[x][0] + o[x][1]) + (o[x][2] + o[x][3]);
                        sum += __shfl_xor(sum, 16);
                        sum += __shfl_xor(sum, 32);
                        const float mean = sum * inv_n;
                        float sq = 0.f;
#pragma unroll
                        for (int x = 0; x < NX; ++x) {
                            if (4 * g + 16 * x < dv) {
#pragma unroll
                                for (int r = 0; r < 4; ++r) {
                                    const float d = o[x][r] - mean;
                                    sq = fmaf(d, d, sq);
                                }
                            }
                        }
                        sq += __shfl_xor(sq, 16);
                        sq += __shfl_xor(sq, 32);
                        const float rstd = __builtin_amdgcn_rsqf(sq * inv_n + p.ln_eps);
#pragma unroll
                        for (int x = 0; x < NX; ++x) {
                            if (4 * g + 16 * x < dv) {
                                const f32x4 lw = *reinterpret_cast<const f32x4 *>(s_lnw + 16 * x + 4 * g);
                                const f32x4 lb = *reinterpret_cast<const f32x4 *>(s_lnb + 16 * x + 4 * g);
                                const float rv[4] = {bf16_lo_as_float(rg[x][0]), bf16_hi_as_float(rg[x][0]),
                                                     bf16_lo_as_float(rg[x][1]), bf16_hi_as_float(rg[x][1])};
#pragma unroll
                                for (int r = 0; r < 4; ++r) {
                                    const float sw = rv[r] * __builtin_amdgcn_rcpf(1.f + exp2_fast(-rv[r] * kLog2e));
                                    o[x][r] = fmaf((o[x][r] - mean) * rstd, lw[r], lb[r]) * sw;
                                }
                            }
                        }
                    }
                }
                if constexpr (ACC) {
#pragma unroll
                    for (int x = 0; x < NX; ++x) o[x] += prev[x];
                }
                const int row = 16 * IT + lm;
                if (row < nvalid) {
                    const int col0 = 4 * g;
                    char *orow = gout + ((uint32_t)tok[row] * (uint32_t)p.st_v + (uint32_t)col0) * (uint32_t)sizeof(TOut);
#pragma unroll
                    for (int x = 0; x < NX; ++x) {
                        if (col0 + 16 * x < dv) {  // dv is a multiple of 8: all four columns or none
                            if constexpr (sizeof(TOut) == 4)
                                *reinterpret_cast<f32x4 *>(orow + 64 * x) = o[x];
                            else
                                *reinterpret_cast<u32x2 *>(orow + 32 * x) =
                                    u32x2{pack_bf16(o[x][0], o[x][1]), pack_bf16(o[x][2], o[x][3])};
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < NTW; ++i)
                    update_state(0, i, v_frag(0, TM::nt(W, i)), v_frag(1, TM::nt(W, i)), v_frag_lo(0, TM::nt(W, i)),
                                 v_frag_lo(1, TM::nt(W, i)));
            } else {
                // state pass: K~ of the wave's row tile once, V of tile i+1 read while tile i is contracted
                u32x2 uv[2][2][2];                              // [buffer][32-token step][half]
                u32x2 uvl[BETA ? 2 : 1][2][2];                  // BETA: remainders of the gated values
                auto load_state_v = [&](int buf, int i) {
                    const int vo = 16 * TM::nt(W, i);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        uv[buf][ks][0] = lds_read_tr(vrow + 32 * ks * VS + vo);
                        uv[buf][ks][1] = lds_read_tr(vrow + (32 * ks + 16) * VS + vo);
                        if constexpr (BETA) {
                            uvl[buf][ks][0] = lds_read_tr(vrow_l + 32 * ks * VS + vo);
                            uvl[buf][ks][1] = lds_read_tr(vrow_l + (32 * ks + 16) * VS + vo);
                        }
                    }
                };
                if constexpr (NTW > 0) {
                    load_state_k(0, 0);
                    load_state_v(0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < NTW; ++i) {
                    if (i + 1 < NTW) load_state_v((i + 1) & 1, i + 1);
                    const int bf = i & 1;
                    const u32x4 v0 = u32x4{uv[bf][0][0][0], uv[bf][0][0][1], uv[bf][0][1][0], uv[bf][0][1][1]};
                    const u32x4 v1 = u32x4{uv[bf][1][0][0], uv[bf][1][0][1], uv[bf][1][1][0], uv[bf][1][1][1]};
                    if constexpr (BETA)
                        update_state(0, i, v0, v1,
                                     u32x4{uvl[bf][0][0][0], uvl[bf][0][0][1], uvl[bf][0][1][0], uvl[bf][0][1][1]},
                                     u32x4{uvl[bf][1][0][0], uvl[bf][1][0][1], uvl[bf][1][1][0], uvl[bf][1][1][1]});
                    else
                        update_state(0, i, v0, v1, v0, v1);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        switch (w) {
        case 0: contract(int_c<0>{}); break;
        case 1: contract(int_c<1>{}); break;
        case 2: contract(int_c<2>{}); break;
        case 3: contract(int_c<3>{}); break;
        case 4: if constexpr (NW > 4) contract(int_c<4>{}); break;
        case 5: if constexpr (NW > 4) contract(int_c<5>{}); break;
        case 6: if constexpr (NW > 4) contract(int_c<6>{}); break;
        default: if constexpr (NW > 4) contract(int_c<7>{}); break;
        }
        __syncthreads();
    };
    // Whole groups of DEPTH chunks in the loop, a last odd chunk after it: a conditional call inside the loop
    // would hide from the compiler which loads are still in flight at the loop head.
    int chunk = 0;
    for (; chunk + DEPTH <= nch; chunk += DEPTH) {
        process_chunk(chunk, int_c<0>{});
        if constexpr (DEPTH == 2) process_chunk(chunk + 1, int_c<1>{});
    }
    if constexpr (DEPTH == 2) {
        if (chunk < nch) process_chunk(chunk, int_c<0>{});
    }

    // ---- epilogue: the span's state ----
    float *dst = nullptr;
    if (!OUT)
        dst = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;
    else if ((p.nspans == 1 || p.chain_in_output) && sp == p.nspans - 1 && p.final_state != nullptr)
        dst = p.final_state + (size_t)bh * dk * dv;  // the last span ends in the final state
    if (dst != nullptr) {
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            if (TM::valid(w, i)) {
                const int n = 16 * TM::nt(w, i) + lm;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int c = 16 * TM::ct(w, i) + 4 * g + r;
                    if (c < dk && n < dv) dst[c * dv + n] = acc[i][r];
                }
            }
        }
    }
    // the workspace keeps natural logarithms
    if (!OUT && tid < dk) p.ws_lgam[((size_t)bh * p.nspans + sp) * dk + tid] = s_lg[tid] * kLn2;
    if constexpr (BETA && !OUT) {
        if (tid < dv) p.ws_lgam_b[((size_t)bh * p.nspans + sp) * dv + tid] = s_lgb[tid] * kLn2;
    }
}

template <int MODE, int NDK8, int NDV16, int DEPTH, bool FUSE, bool ACC, typename TOut, bool BETA>
hipError_t launch_depth(const Params &p, hipStream_t stream) {
    using L = Layout<MODE, NDK8, NDV16, BETA>;
    if constexpr (L::kBytes > 160 * 1024) {
        return hipErrorInvalidConfiguration;   // (two-sided gate at the largest head sizes: mfma_engine_supports says no)
    } else {
    // The state pass is light on registers and runs best with 8 waves (4 per SIMD at two work-groups per compute
    // unit); the output pass needs the 256-register budget of 4-wave groups for its operand batches.
    constexpr int NW = (MODE == kModeState) ? 8 : 4;
    // register cap: no tighter than the waves per SIMD that the LDS footprint lets a compute unit hold anyway
    constexpr int kGroupsPerCu = (160 * 1024) / L::kBytes;
    constexpr int kWavesPerSimd = kGroupsPerCu * NW / 4;
    constexpr int MINW = kWavesPerSimd >= 4 ? 4 : (kWavesPerSimd >= 2 ? 2 : 1);
    auto kernel = mfma_span_kernel<MODE, NDK8, NDV16, NW, MINW, DEPTH, FUSE, ACC, TOut, BETA>;
    static std::atomic<bool> configured[kMaxDevices] = {};  // per instantiation and device
    {
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), L::kBytes, configured);
        if (e != hipSuccess) return e;
    }
    const int spans = (MODE == kModeState && p.chain_in_output) ? p.nspans - 1 : p.nspans;
    dim3 grid((unsigned)(p.B * p.H * spans)), block(NW * 64);
    hipLaunchKernelGGL(kernel, grid, block, L::kBytes, stream, p);
    return hipGetLastError();
    }
}

template <int MODE, int NDK8, int NDV16, bool FUSE, bool ACC, typename TOut, bool BETA = false>
hipError_t launch_one(const Params &p, hipStream_t stream) {
    // Two chunks of rows in flight pay off in the state pass (short chunk period, registers to spare at the
    // smaller head sizes) once a span is long enough to amortise the second set's start-up.
    if constexpr (MODE == kModeState && NDK8 <= 5 && NDV16 <= 5) {
        if (!BETA && p.span_len >= 4 * kChunk)
            return launch_depth<MODE, NDK8, NDV16, 2, FUSE, ACC, TOut, false>(p, stream);
    }
    return launch_depth<MODE, NDK8, NDV16, 1, FUSE, ACC, TOut, BETA>(p, stream);
}

template <int MODE, int NDK8, int NDV16>
hipError_t launch_dt(const Params &p, hipStream_t stream) {
    if (p.z_gate != nullptr && p.z_beta != nullptr) {   // both gates from pre-activations (+ optional epilogue)
        if (MODE == kModeOutput && p.out_dtype == GLA_DT_BF16)
            return launch_one<MODE, NDK8, NDV16, true, false, uint16_t, true>(p, stream);
        return launch_one<MODE, NDK8, NDV16, true, false, float, true>(p, stream);
    }
    if (p.log_beta != nullptr) {   // two-sided gate from its logarithms (the host keeps it apart from the accumulation)
        if (MODE == kModeOutput && p.out_dtype == GLA_DT_BF16)
            return launch_one<MODE, NDK8, NDV16, false, false, uint16_t, true>(p, stream);
        return launch_one<MODE, NDK8, NDV16, false, false, float, true>(p, stream);
    }
    if (p.z_gate != nullptr) {
        if (MODE == kModeOutput && p.out_dtype == GLA_DT_BF16)
            return launch_one<MODE, NDK8, NDV16, true, false, uint16_t>(p, stream);
        return launch_one<MODE, NDK8, NDV16, true, false, float>(p, stream);
    }
    if constexpr (MODE == kModeOutput) {
        if (p.accumulate) return launch_one<MODE, NDK8, NDV16, false, true, float>(p, stream);   // host checks fp32 out
    }
    if (MODE == kModeOutput && p.out_dtype == GLA_DT_BF16)
        return launch_one<MODE, NDK8, NDV16, false, false, uint16_t>(p, stream);
    return launch_one<MODE, NDK8, NDV16, false, false, float>(p, stream);
}

template <int MODE>
hipError_t launch_mode(const Params &p, hipStream_t stream) {
    const int ndk8 = (p.dk + 7) / 8, ndv16 = (p.dv + 15) / 16;
    if (ndk8 <= 4 && ndv16 <= 4) return launch_dt<MODE, 4, 4>(p, stream);
    if (ndk8 <= 5 && ndv16 <= 5) return launch_dt<MODE, 5, 5>(p, stream);
    return launch_dt<MODE, 8, 8>(p, stream);
}

}  // namespace

bool mfma_engine_supports(const Params &p) {
    // two-sided gate: the extra rows (log_beta, remainder of the gated values) fit the LDS up to dk = 40, dv = 80
    if (two_sided(p) && (p.dk > 40 || p.dv > 80)) return false;
    // 32-bit byte offsets inside the view of one (batch, head)
    const long long slab = (long long)p.T * (p.st_k > p.st_v ? p.st_k : p.st_v) * 4;
    return p.qkv_dtype == GLA_DT_BF16 && p.dk % 4 == 0 && p.dv % 8 == 0 && p.dk <= kMaxDk && p.dv <= kMaxDv &&
           slab < (1LL << 31);
}

hipError_t launch_mfma_span(const Params &p, SpanMode mode, hipStream_t stream) {
    return mode == kModeState ? launch_mode<kModeState>(p, stream) : launch_mode<kModeOutput>(p, stream);
}

}  // namespace gla
