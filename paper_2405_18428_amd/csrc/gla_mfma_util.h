// Device helpers shared by the bf16 MFMA kernels (gfx950): the 16x16x32 bf16 MFMA, bf16 hi/lo splitting,
// the transposing LDS read, and the wave-wide prefix sum.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "gla_common.h"

namespace gla {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMaxExp2 = 120.f;       // clamp of -b (base 2) before exp2: keeps k~ finite

__device__ inline f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                   c, 0, 0, 0);
}

__device__ inline uint32_t pack_bf16(float lo, float hi) {
    f32x2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}
__device__ inline float bf16_lo_as_float(uint32_t packed) { return __builtin_bit_cast(float, packed << 16); }
__device__ inline float bf16_hi_as_float(uint32_t packed) { return __builtin_bit_cast(float, packed & 0xffff0000u); }
__device__ inline float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

typedef __attribute__((ext_vector_type(4))) short s16x4;
// Transposing 8-byte LDS read (see the header comment for the lane shuffle).
__device__ inline u32x2 lds_read_tr(const uint16_t *p) {
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    return __builtin_bit_cast(u32x2, __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)p));
}

// x0, x1 -> packed bf16 pair of the rounded values and packed pair of the remainders
struct HiLo {
    uint32_t hi, lo;
};
__device__ inline HiLo split_pair_val(float x0, float x1) {
    HiLo r;
    r.hi = pack_bf16(x0, x1);
    r.lo = pack_bf16(x0 - bf16_lo_as_float(r.hi), x1 - bf16_hi_as_float(r.hi));
    return r;
}
// (vector elements cannot bind to references, hence a macro for the two outputs)
#define SPLIT_PAIR(x0, x1, hi_out, lo_out)            \
    do {                                              \
        const HiLo hl_ = split_pair_val((x0), (x1));  \
        (hi_out) = hl_.hi;                            \
        (lo_out) = hl_.lo;                            \
    } while (0)

// Identity that the optimiser cannot see through: values derived from the result are recomputed where they are
// used instead of being hoisted out of the chunk loop and held in registers.
__device__ inline int recompute_per_chunk(int x) {
    asm volatile("" : "+v"(x));
    return x;
}

template <int CTRL, int ROW_MASK, bool BOUND>
__device__ inline float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK,
                                                                 0xF, BOUND));
}
// Inclusive prefix sum over the 64 lanes of a wave (lane = token).
__device__ inline float wave_inclusive_scan(float v) {
    v += dpp_move<0x111, 0xF, true>(v);  // row_shr:1
    v += dpp_move<0x112, 0xF, true>(v);  // row_shr:2
    v += dpp_move<0x114, 0xF, true>(v);  // row_shr:4
    v += dpp_move<0x118, 0xF, true>(v);  // row_shr:8   -> prefix inside each row of 16
    v += dpp_move<0x142, 0xA, false>(v); // row_bcast:15 into rows 1 and 3
    v += dpp_move<0x143, 0xC, false>(v); // row_bcast:31 into rows 2 and 3
    return v;
}

// Four independent inclusive prefix sums over the 64 lanes of a wave, their six DPP steps interleaved: every step
// is a single v_add_f32 with a DPP source (row_shr with out-of-row lanes reading zero; row_bcast writing only the
// rows named by row_mask), and an instruction never reads a register written by one of the three before it, so
// the chain of one sum hides behind the other three and no wait states are needed between the steps.
// All 64 lanes must be active.
__device__ inline void wave_inclusive_scan4(float &a, float &b, float &c, float &d) {
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
        "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_add_f32_dpp %2, %2, %2 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_add_f32_dpp %3, %3, %3 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %1, %1 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_add_f32_dpp %2, %2, %2 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "v_add_f32_dpp %3, %3, %3 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"      // and before whatever reads the results through DPP next
        : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// State entering span `sp` of (batch, head) `bh`, formed from the local states U_r and the log decays of the
// spans before it (phase 2 of the span plan, done by the work-group that needs the result):
//     S_start(sp) = U_{sp-1} + Gamma_{sp-1} U_{sp-2} + Gamma_{sp-1} Gamma_{sp-2} U_{sp-3} + ... (+ the decayed initial state)
// Each thread owns kV4 pieces of 4 consecutive state elements (one key channel each) and walks the spans from the
// nearest one backwards, 2 spans first, then kRun at a time (loads of a run issued together).  A thread stops
// when the decay accumulated on all its channels is below 2^-40 and it has summed something other than zero: a
// term that much smaller than the earlier states hold does not change an fp32 sum of terms of their size.
// With the gates of the DiG configurations a span of a few hundred tokens decays by more than that, so one or
// two spans are read whatever the span count.
// The result is written to s_chain[dk * dv] (LDS, row-major [dk][dv]).
// BETA (two-sided gate): element (c, n) also decays by the value-side sums of the spans (ws_lgam_b, per column n);
// the stopping rule stays the key-side one (the value side only makes the skipped terms smaller).
template <int NTHR, int kV4, int kRun, bool BETA = false>
__device__ inline void chain_span_states(const Params &p, int bh, int sp, int tid, float *s_chain) {
    const int dk = p.dk, dv = p.dv, ne = dk * dv, ne4 = ne >> 2;
    const float *ub = p.ws_state + (size_t)bh * p.nspans * ne;
    const float *lb = p.ws_lgam + (size_t)bh * p.nspans * dk;
    const float *lbb = BETA ? p.ws_lgam_b + (size_t)bh * p.nspans * dv : nullptr;
    int e4[kV4], ch[kV4], col[kV4];
#pragma unroll
    for (int m = 0; m < kV4; ++m) {
        e4[m] = min(tid + NTHR * m, ne4 - 1);  // threads past the end repeat the last piece
        ch[m] = (4 * e4[m]) / dv;
        col[m] = 4 * e4[m] - ch[m] * dv;       // first of the piece's four value columns (dv % 4 == 0)
    }
    f32x4 st[kV4];
    float wl[kV4];      // log2 of the weight of the next span to add
    f32x4 wb[BETA ? kV4 : 1];   // BETA: its value-side part per column
#pragma unroll
    for (int m = 0; m < kV4; ++m) {
        st[m] = f32x4{0.f, 0.f, 0.f, 0.f};
        wl[m] = 0.f;
        if constexpr (BETA) wb[m] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    auto run = [&](auto n_c, int r_hi) {   // spans r_hi, r_hi - 1, ..., r_hi - n + 1 (those below 0 do not exist)
        constexpr int N = decltype(n_c)::value;
        f32x4 u[N][kV4];
        float lg[N][kV4];
        f32x4 lgb[BETA ? N : 1][BETA ? kV4 : 1];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int r = max(r_hi - i, 0);     // loads past the first span repeat it
#pragma unroll
            for (int m = 0; m < kV4; ++m) {
                u[i][m] = *reinterpret_cast<const f32x4 *>(ub + (size_t)r * ne + 4 * e4[m]);
                lg[i][m] = lb[r * dk + ch[m]];
                if constexpr (BETA) lgb[i][m] = *reinterpret_cast<const f32x4 *>(lbb + r * dv + col[m]);
            }
        }
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if (r_hi - i >= 0) {
#pragma unroll
                for (int m = 0; m < kV4; ++m) {
                    if constexpr (BETA) {
#pragma unroll
                        for (int x = 0; x < 4; ++x) {
                            st[m][x] = fmaf(exp2_fast(wl[m] + wb[m][x]), u[i][m][x], st[m][x]);
                            wb[m][x] += lgb[i][m][x] * kLog2e;
                        }
                    } else {
                        const float wgt = exp2_fast(wl[m]);
#pragma unroll
                        for (int x = 0; x < 4; ++x) st[m][x] = fmaf(wgt, u[i][m][x], st[m][x]);
                    }
                    wl[m] += lg[i][m] * kLog2e;    // the workspace keeps natural logarithms
                }
            }
        }
    };
    // a piece goes on while its accumulated decay is above 2^-40, and also while everything it has summed is
    // exactly zero (all-zero k or v over the nearer spans, e.g. a padded tail: then even a strongly decayed
    // earlier state is the whole result)
    auto alive = [&]() {
        bool a = false;
#pragma unroll
        for (int m = 0; m < kV4; ++m)
            a = a || wl[m] > -40.f || (st[m][0] == 0.f && st[m][1] == 0.f && st[m][2] == 0.f && st[m][3] == 0.f);
        return a;
    };
    int r = sp - 1;
    if (r >= 0) {
        run(std::integral_constant<int, 2>{}, r);
        r -= 2;
    }
    while (r >= 0 && alive()) {
        run(std::integral_constant<int, kRun>{}, r);
        r -= kRun;
    }
    if (p.initial_state != nullptr && alive()) {   // every span was walked: the caller's state, decayed by all of them
#pragma unroll
        for (int m = 0; m < kV4; ++m) {
            const f32x4 s0 = *reinterpret_cast<const f32x4 *>(p.initial_state + (size_t)bh * ne + 4 * e4[m]);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                float wlx = wl[m];
                if constexpr (BETA) wlx += wb[m][x];
                st[m][x] = fmaf(exp2_fast(wlx), s0[x], st[m][x]);
            }
        }
    }
#pragma unroll
    for (int m = 0; m < kV4; ++m)
        if (tid + NTHR * m < ne4) *reinterpret_cast<f32x4 *>(s_chain + 4 * e4[m]) = st[m];
}

}  // namespace
}  // namespace gla
