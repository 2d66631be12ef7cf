// Device helpers shared by the bf16 MFMA kernels (gfx950): the 16x16x32 bf16 MFMA, bf16 hi/lo splitting,
// the transposing LDS read, and the wave-wide prefix sum.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

}  // namespace
}  // namespace gla
