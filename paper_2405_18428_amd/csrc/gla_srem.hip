// 3x3 depth-wise convolution of the spatial reorient & enhancement module of the DiG block
// (DiG paper, Sec. 3.3 and Algorithm 1: DWConv2d on the 2-D token matrix, identity-initialised).
//
// Tensors stay in canonical row-major token order, [B, T, D] with the D channels of a token contiguous.
// The paper transposes / flips the sequence between blocks, so later blocks convolve the transposed and / or
// reversed token matrix; `orient` names that order and only changes which kernel tap meets which neighbour:
//   order 0 (row-major)              tap (dy, dx) meets the neighbour at ( dy,  dx)
//   order 1 (reversed)                                                    (-dy, -dx)
//   order 2 (column-major)                                                ( dx,  dy)
//   order 3 (column-major reversed)                                       (-dx, -dy)
// A thread owns VEC channels (4 when D allows: 8-byte bf16 pieces) of a strip of kStrip tokens of a grid row and
// walks kRows rows of that strip from top to bottom.  The lanes of a wave cover 64 neighbouring channel groups of
// the same tokens (contiguous addresses); the kWaves waves of a work-group take neighbouring strips and share the weights
// of their 64 channel groups, which are fetched once, coalesced, into LDS (a lane's 9 x VEC weights are VEC*36
// bytes apart from its neighbour's in memory) and then held in registers.  The window is three rows of
// kStrip + 2 pieces; the row below it is requested before the arithmetic of the current row starts, so loads and
// arithmetic overlap inside every wave and an input row is fetched once per band of kRows rows.  Coordinates are
// clamped and pieces outside the matrix cleared by an AND mask (zero padding, no branches).  HBM-bound.
#include "gla_common.h"

namespace gla {
namespace {

constexpr int kStrip = 4;      // output tokens per thread and grid row
constexpr int kRows = 8;       // grid rows a wave walks
constexpr int kWaves = 2;      // strips per work-group (2560 waves on the 2048 px shape: small groups spread evenly)
constexpr int kAhead = 1;      // rows requested ahead of the window (2 and 3 measured no faster)
constexpr int kRing = kAhead + 3;
constexpr int kThreads = 64 * kWaves;

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ inline uint32_t pack_bf16(float lo, float hi) {   // round to nearest even, two at a time
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// VEC consecutive elements as they lie in memory
template <typename T, int VEC> struct Raw;
template <> struct Raw<float, 1> { float v; };
template <> struct Raw<uint16_t, 1> { uint16_t v; };
template <> struct Raw<float, 4> { f32x4 v; };
template <> struct Raw<uint16_t, 4> { u32x2 v; };

template <typename T, int VEC>
__device__ inline Raw<T, VEC> load_raw(const void *base, size_t e) {
    return *reinterpret_cast<const Raw<T, VEC> *>(static_cast<const T *>(base) + e);
}
__device__ inline void to_floats(const Raw<float, 1> &r, float (&x)[1]) { x[0] = r.v; }
__device__ inline void to_floats(const Raw<uint16_t, 1> &r, float (&x)[1]) { x[0] = bf16_bits_to_float(r.v); }
__device__ inline void to_floats(const Raw<float, 4> &r, float (&x)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = r.v[i];
}
__device__ inline void to_floats(const Raw<uint16_t, 4> &r, float (&x)[4]) {
    x[0] = __builtin_bit_cast(float, r.v[0] << 16);
    x[1] = __builtin_bit_cast(float, r.v[0] & 0xffff0000u);
    x[2] = __builtin_bit_cast(float, r.v[1] << 16);
    x[3] = __builtin_bit_cast(float, r.v[1] & 0xffff0000u);
}

// keeps (mask = all ones) or clears (mask = 0) a piece without a branch
__device__ inline void and_mask(Raw<float, 1> &r, uint32_t m) { r.v = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, r.v) & m); }
__device__ inline void and_mask(Raw<uint16_t, 1> &r, uint32_t m) { r.v = (uint16_t)(r.v & m); }
__device__ inline void and_mask(Raw<float, 4> &r, uint32_t m) {
    const u32x4 bits = __builtin_bit_cast(u32x4, r.v) & u32x4{m, m, m, m};
    r.v = __builtin_bit_cast(f32x4, bits);
}
__device__ inline void and_mask(Raw<uint16_t, 4> &r, uint32_t m) { r.v = r.v & u32x2{m, m}; }

template <typename T, int VEC>
__device__ inline void store_vec(void *base, size_t e, const float (&x)[VEC]) {
    if constexpr (VEC == 1) {
        if constexpr (sizeof(T) == 4) static_cast<float *>(base)[e] = x[0];
        else static_cast<uint16_t *>(base)[e] = float_to_bf16_bits(x[0]);
    } else if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(base) + e) = f32x4{x[0], x[1], x[2], x[3]};
    } else {
        *reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(base) + e) = u32x2{pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
    }
}

template <typename TIn, typename TOut, int VEC>
__global__ __launch_bounds__(kThreads) void srem_dwconv_kernel(const void *x, const float *w, const float *bias,
                                                               void *y, int B, int gh, int gw, int D, int orient) {
    __shared__ __attribute__((aligned(16))) float s_w[64 * VEC * 9];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int ncg = D / VEC;
    // Work-groups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of (strip, channel block)
    // pairs, i.e. a band of grid rows, so that the three uses of a row by vertically neighbouring strips meet in
    // one L2.
    const int gx = (ncg + 63) / 64;
    int blk = blockIdx.x;
    {
        const int nb = gridDim.x;
        if ((nb & 7) == 0) blk = (blk & 7) * (nb >> 3) + (blk >> 3);
    }
    const int bx = blk % gx, by = blk / gx;
    const int cg0 = bx * 64;
    const int ncg_here = min(64, ncg - cg0);
    // A wave walks kRows grid rows of its strip from top to bottom.  Three rows (r-1, r, r+1; columns c0-1..c0+kStrip)
    // are held as raw pieces; the row after them is requested before the arithmetic of the current output row starts
    // and has arrived when the window moves down, so that loads and arithmetic overlap inside every wave and each
    // input row is fetched once per band instead of three times.  Coordinates are clamped (lanes and waves without
    // work repeat a valid piece) and pieces outside the matrix are cleared afterwards (zero padding).
    // (strip index and everything derived from it are uniform over the wave: scalar arithmetic; addresses are
    // a 64-bit base of the (batch, channel group) plus 32-bit byte offsets, row part + column part)
    const int nstrips = (gw + kStrip - 1) / kStrip;
    const int nbands = (gh + kRows - 1) / kRows;
    const uint32_t nsid = (uint32_t)B * (uint32_t)nbands * (uint32_t)nstrips;          // < 2^31 (host check)
    const uint32_t sid = (uint32_t)__builtin_amdgcn_readfirstlane(by * kWaves + wv);   // (band, strip) of this wave
    const bool active = lane < ncg_here && sid < nsid;
    const uint32_t sidc = sid < nsid ? sid : nsid - 1;
    const uint32_t q1 = sidc / (uint32_t)nstrips;
    const int cs = (int)(sidc - q1 * (uint32_t)nstrips);
    const int b = (int)(q1 / (uint32_t)nbands);
    const int r0 = (int)(q1 - (uint32_t)b * (uint32_t)nbands) * kRows;
    const int ch = (cg0 + (lane < ncg_here ? lane : 0)) * VEC;
    const int c0 = cs * kStrip;
    const size_t img = (size_t)b * gh * gw * D + ch;                 // element offset of (b, token 0, ch)
    const char *xin = static_cast<const char *>(x) + img * sizeof(TIn);
    char *yout = static_cast<char *>(y) + img * sizeof(TOut);
    const uint32_t pitch = (uint32_t)D * (uint32_t)sizeof(TIn);     // bytes from a token to the next
    const uint32_t opitch = (uint32_t)D * (uint32_t)sizeof(TOut);
    uint32_t coloff[kStrip + 2];
#pragma unroll
    for (int t = 0; t < kStrip + 2; ++t) coloff[t] = (uint32_t)min(max(c0 + t - 1, 0), gw - 1) * pitch;
    auto load_row = [&](int rr, Raw<TIn, VEC> (&dst)[kStrip + 2]) {
        const uint32_t rowoff = (uint32_t)(min(max(rr, 0), gh - 1) * gw) * pitch;
#pragma unroll
        for (int t = 0; t < kStrip + 2; ++t) dst[t] = *reinterpret_cast<const Raw<TIn, VEC> *>(xin + (rowoff + coloff[t]));
    };
    Raw<TIn, VEC> win[kRing][kStrip + 2];    // rows r-1, r, r+1 and the kAhead rows in flight, rotating
#pragma unroll
    for (int m = 0; m < kAhead + 2; ++m) load_row(r0 - 1 + m, win[m]);
    // weights of the block's channel groups: one contiguous piece of the [D, 3, 3] array
    {
        const float *src = w + (size_t)cg0 * VEC * 9;
        const int n = ncg_here * VEC * 9;
        if constexpr (VEC == 4) {   // n is a multiple of 4 and src 16-byte aligned (144 bytes per channel group)
            for (int i = tid; i < n / 4; i += kThreads)
                reinterpret_cast<f32x4 *>(s_w)[i] = reinterpret_cast<const f32x4 *>(src)[i];
        } else {
            for (int i = tid; i < n; i += kThreads) s_w[i] = src[i];
        }
    }
    __syncthreads();
    if (!active) return;

    // weights of this thread's channels, indexed by the canonical offset (oy, ox) of the neighbour; the tap that
    // meets it is (dy, dx) = (a oy + b ox, b oy + a ox) with (a, b) = (1,0), (-1,0), (0,1), (0,-1) for the four orders
    const int ta = orient == 0 ? 1 : (orient == 1 ? -1 : 0);
    const int tb = orient == 2 ? 1 : (orient == 3 ? -1 : 0);
    float wt[3][3][VEC];
#pragma unroll
    for (int oy = -1; oy <= 1; ++oy) {
#pragma unroll
        for (int ox = -1; ox <= 1; ++ox) {
            const int dy = ta * oy + tb * ox, dx = tb * oy + ta * ox;
            const int tap = (dy + 1) * 3 + (dx + 1);
#pragma unroll
            for (int i = 0; i < VEC; ++i) wt[oy + 1][ox + 1][i] = s_w[(lane * VEC + i) * 9 + tap];
        }
    }
    float bv[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) bv[i] = bias != nullptr ? bias[ch + i] : 0.f;

#pragma unroll
    for (int ri = 0; ri < kRows; ++ri) {
        const int r = r0 + ri;
        if (r >= gh) break;                                   // uniform: the last band may be short
        if (ri + kAhead < kRows) load_row(r + 1 + kAhead, win[(ri + 2 + kAhead) % kRing]);   // in flight during the arithmetic of kAhead rows
        float acc[kStrip][VEC];
#pragma unroll
        for (int t = 0; t < kStrip; ++t)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[t][i] = bv[i];
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            const bool row_in = (r + j - 1 >= 0) && (r + j - 1 < gh);
#pragma unroll
            for (int t = 0; t < kStrip + 2; ++t) {
                const int c = c0 + t - 1;
                // a piece outside the matrix was fetched from a clamped position: clear it (zero padding);
                // the cleared copy is a temporary, the window keeps the fetched bytes (a clamped bottom row is a
                // real row for the output rows above it)
                Raw<TIn, VEC> piece = win[(ri + j) % kRing][t];
                and_mask(piece, (row_in && c >= 0 && c < gw) ? 0xffffffffu : 0u);
                float xv[VEC];
                to_floats(piece, xv);
                // this piece is the left / middle / right neighbour of outputs t, t-1, t-2
#pragma unroll
                for (int o = 0; o < 3; ++o) {
                    const int tt = t - o;          // output token index in the strip
                    if (tt >= 0 && tt < kStrip) {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc[tt][i] = fmaf(wt[j][o][i], xv[i], acc[tt][i]);
                    }
                }
            }
        }
        char *yrow = yout + (size_t)((uint32_t)(r * gw + c0) * opitch);
#pragma unroll
        for (int t = 0; t < kStrip; ++t)
            if (c0 + t < gw) store_vec<TOut, VEC>(yrow + (uint32_t)t * opitch, 0, acc[t]);
    }
}

template <typename TIn, typename TOut, int VEC>
hipError_t launch_vec(const void *x, const float *w, const float *bias, void *y, int B, int gh, int gw, int D,
                      int orient, hipStream_t stream) {
    const long long nstrips = (long long)B * ((gh + kRows - 1) / kRows) * ((gw + kStrip - 1) / kStrip);
    const long long nblocks = (long long)((D / VEC + 63) / 64) * ((nstrips + kWaves - 1) / kWaves);
    dim3 grid((unsigned)nblocks), block(kThreads);
    hipLaunchKernelGGL((srem_dwconv_kernel<TIn, TOut, VEC>), grid, block, 0, stream, x, w, bias, y, B, gh, gw, D,
                       orient);
    return hipGetLastError();
}

template <typename TIn, typename TOut>
hipError_t launch_types(const void *x, const float *w, const float *bias, void *y, int B, int gh, int gw, int D,
                        int orient, hipStream_t stream) {
    // 4 channels per thread (8-byte bf16 pieces) when the channel count allows it
    if (D % 4 == 0) return launch_vec<TIn, TOut, 4>(x, w, bias, y, B, gh, gw, D, orient, stream);
    return launch_vec<TIn, TOut, 1>(x, w, bias, y, B, gh, gw, D, orient, stream);
}

}  // namespace

hipError_t launch_srem_dwconv(const void *x, const float *w, const float *bias, void *y, int B, int gh, int gw, int D,
                              int orient, int x_dtype, int y_dtype, hipStream_t stream) {
    const bool xb = x_dtype == GLA_DT_BF16, yb = y_dtype == GLA_DT_BF16;
    if (xb && yb) return launch_types<uint16_t, uint16_t>(x, w, bias, y, B, gh, gw, D, orient, stream);
    if (xb) return launch_types<uint16_t, float>(x, w, bias, y, B, gh, gw, D, orient, stream);
    if (yb) return launch_types<float, uint16_t>(x, w, bias, y, B, gh, gw, D, orient, stream);
    return launch_types<float, float>(x, w, bias, y, B, gh, gw, D, orient, stream);
}

}  // namespace gla
