// Kernels that exist only for the backward pass of the GLA recurrence
// (DiG paper, Sec. 3.1 Eq. (attn_gla) rows 1-3 with beta = 1, differentiated).
//
// With S_s the state after scan step s and G_s = dL/dS_s (which obeys the same kind
// of recurrence walked backwards, G_s = q_s^T dO_s + diag(alpha_{s+1}) G_{s+1}):
//     dq_s[c] = sum_n S_s[c,n] dO_s[n]        dk_s[c] = sum_n G_s[c,n] v_s[n]
//     dv_s    = k_s G_s                        (a forward pass with q, k, v := k, q, dO)
//     dlog_alpha_s = sum_{s' >= s} (q_s' * dq_s' - k_s' * dk_s')      (reverse cumulative sum)
// dq and dk read the state along its value axis, which the forward engines (they read
// it along the key axis) do not do; row_read_kernel does: it walks one span token by
// token in fp32 with the state rows in registers, thread c of a wave owning row c
// of half of the value columns.  The state entering the span comes from the span
// plan of the forward pass (span-state pass + carry kernel).
//
// (A first, plain-ALU rendering: the chunk form of these reads on the MFMA units is the next step.)
#include "gla_common.h"

namespace gla {
namespace {

constexpr int kTile = 16;          // tokens staged per round
constexpr int kRowWaves = 2;       // waves per work-group; each owns half of the value columns
constexpr int kColsPerWave = kMaxDv / kRowWaves;

typedef __attribute__((ext_vector_type(4))) float f32x4;

template <typename T> __device__ inline float load_elem(const void *base, size_t idx);
template <> __device__ inline float load_elem<float>(const void *base, size_t idx) {
    return static_cast<const float *>(base)[idx];
}
template <> __device__ inline float load_elem<uint16_t>(const void *base, size_t idx) {
    return bf16_bits_to_float(static_cast<const uint16_t *>(base)[idx]);
}

// r_s[c] = sum_n S_s[c,n] w_s[n] for the scan steps of one span; S follows (p.k, p.v, p.log_alpha).
// p.q is not used; `w` has the layout of p.v, `r` (fp32) that of p.k.
// A tile of kTile tokens is staged in LDS (alpha and k per channel; v and w interleaved in groups of four
// columns, as fp32), then walked token by token: the rows v_s and w_s are the same for all lanes and are read
// as broadcasts, 16 bytes of each per ds_read_b128 pair.
template <typename TIn>
__global__ __launch_bounds__(kRowWaves * 64) void row_read_kernel(Params p, const void *w, float *r) {
    __shared__ float s_a[kTile][kMaxDk];
    __shared__ float s_k[kTile][kMaxDk];
    __shared__ __attribute__((aligned(16))) float s_vw[kTile][kMaxDv / 4][8];   // [token][column quad][v0..v3, w0..w3]
    __shared__ float s_r[kRowWaves][kTile][kMaxDk];
    __shared__ int s_tok[kTile];
    __shared__ int s_tokg[kTile];

    const int tid = threadIdx.x;
    const int c = tid & 63;                                     // state row (key channel) of this lane
    const int half = __builtin_amdgcn_readfirstlane(tid >> 6);  // which value columns
    const int bh = blockIdx.x / p.nspans;
    const int sp = blockIdx.x - bh * p.nspans;
    const int dk = p.dk, dv = p.dv, T = p.T;
    const int s_begin = sp * p.span_len;
    const int s_end = min(T, s_begin + p.span_len);
    const size_t base_k = slab_k(p, bh), base_v = slab_v(p, bh);
    const size_t st_k = (size_t)p.st_k, st_v = (size_t)p.st_v;
    // column quads of this wave: [quad_lo, quad_hi)
    const int nquads = (dv + 3) / 4;
    const int per_wave = (nquads + kRowWaves - 1) / kRowWaves;
    const int quad_lo = half * per_wave;
    const int quad_hi = min(nquads, quad_lo + per_wave);
    const bool row_active = c < dk;

    float S[kColsPerWave];
#pragma unroll
    for (int n = 0; n < kColsPerWave; ++n) S[n] = 0.f;
    if (p.nspans > 1 && row_active) {
        const float *s0 = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv + (size_t)c * dv;
#pragma unroll
        for (int n = 0; n < kColsPerWave; ++n)
            if (4 * quad_lo + n < dv && n < 4 * (quad_hi - quad_lo)) S[n] = s0[4 * quad_lo + n];
    }

    for (int t0 = s_begin; t0 < s_end; t0 += kTile) {
        __syncthreads();
        if (tid < kTile) {
            const int s = min(t0 + tid, s_end - 1);
            s_tok[tid] = (t0 + tid < s_end) ? scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w) : -1;
            s_tokg[tid] = scan_token(p.scan_dir, max(s - p.gate_shift, 0), T, p.grid_h, p.grid_w);
        }
        __syncthreads();
        // stage alpha and k of the tile (a step past the span leaves the state alone) ...
        if (row_active) {
            for (int j = half; j < kTile; j += kRowWaves) {
                const int n = s_tok[j];
                s_a[j][c] = n >= 0 ? expf(p.log_alpha[base_k + (size_t)s_tokg[j] * st_k + c]) : 1.f;
                s_k[j][c] = n >= 0 ? load_elem<TIn>(p.k, base_k + (size_t)n * st_k + c) : 0.f;
            }
        }
        // ... and its rows of v and w, zero past dv and past the span
        for (int idx = tid; idx < kTile * 4 * nquads; idx += kRowWaves * 64) {
            const int j = idx / (4 * nquads), col = idx - j * 4 * nquads;
            const int n = s_tok[j];
            float x = 0.f, y = 0.f;
            if (n >= 0 && col < dv) {
                x = load_elem<TIn>(p.v, base_v + (size_t)n * st_v + col);
                y = load_elem<TIn>(w, base_v + (size_t)n * st_v + col);
            }
            s_vw[j][col >> 2][col & 3] = x;
            s_vw[j][col >> 2][4 + (col & 3)] = y;
        }
        __syncthreads();
        for (int j = 0; j < kTile; ++j) {
            const float a = s_a[j][c], kc = s_k[j][c];
            float acc = 0.f;
#pragma unroll
            for (int qd = 0; qd < kColsPerWave / 4; ++qd) {
                if (quad_lo + qd < quad_hi) {   // uniform
                    const f32x4 vq = *reinterpret_cast<const f32x4 *>(&s_vw[j][quad_lo + qd][0]);
                    const f32x4 wq = *reinterpret_cast<const f32x4 *>(&s_vw[j][quad_lo + qd][4]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        S[4 * qd + i] = fmaf(a, S[4 * qd + i], kc * vq[i]);
                        acc = fmaf(S[4 * qd + i], wq[i], acc);
                    }
                }
            }
            s_r[half][j][c] = acc;
        }
        __syncthreads();
        // sum the partial reads of the waves and store the tile
        for (int idx = tid; idx < kTile * dk; idx += kRowWaves * 64) {
            const int j = idx / dk, cc = idx - j * dk;
            const int n = s_tok[j];
            if (n >= 0) {
                float x = 0.f;
#pragma unroll
                for (int h = 0; h < kRowWaves; ++h) x += s_r[h][j][cc];
                r[base_k + (size_t)n * st_k + cc] = x;
            }
        }
    }
}

// ---- dlog_alpha: reverse cumulative sum over the scan order of (q * dq - k * dk), in two kernels ----
// Spans of kDgSpan scan steps.  Kernel 1: inside each span, lane = scan step, a wave scan from the span's last
// step backwards per channel, written at the canonical token index, and the span's total.  Kernel 2: every
// span adds the totals of the spans after it.
constexpr int kDgSpan = 128;       // scan steps per work-group (2 waves of 64 lanes)

template <int CTRL, int ROW_MASK, bool BOUND>
__device__ inline float dpp_move(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK,
                                                                 0xF, BOUND));
}
__device__ inline float wave_inclusive_scan(float v) {
    v += dpp_move<0x111, 0xF, true>(v);  // row_shr:1
    v += dpp_move<0x112, 0xF, true>(v);  // row_shr:2
    v += dpp_move<0x114, 0xF, true>(v);  // row_shr:4
    v += dpp_move<0x118, 0xF, true>(v);  // row_shr:8
    v += dpp_move<0x142, 0xA, false>(v); // row_bcast:15
    v += dpp_move<0x143, 0xC, false>(v); // row_bcast:31
    return v;
}

// Row j of the tile is scan step (span end - 1 - j): prefix sums over j are suffix sums over the scan.
template <typename TIn>
__global__ __launch_bounds__(kDgSpan) void dg_local_kernel(Params p, const float *dq, const float *dk_grad,
                                                          float *dg, float *totals, int ndg) {
    __shared__ float s_x[kDgSpan][kMaxDk + 1];   // odd row length: lane = row accesses hit distinct banks
    __shared__ float s_wave[kDgSpan / 64][kMaxDk];
    __shared__ int s_tok[kDgSpan];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int bh = blockIdx.x / ndg, sp = blockIdx.x - bh * ndg;
    const int dk = p.dk, T = p.T;
    const size_t base_k = slab_k(p, bh), st_k = (size_t)p.st_k;
    const int s_last = min(T, (sp + 1) * kDgSpan) - 1;
    {
        const int s = s_last - tid;
        s_tok[tid] = s >= sp * kDgSpan ? scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w) : -1;
    }
    __syncthreads();
    // the terms q * dq - k * dk, rows read channel by channel (neighbouring lanes, neighbouring addresses)
    for (int idx = tid; idx < kDgSpan * dk; idx += kDgSpan) {
        const int j = idx / dk, c = idx - j * dk;
        const int n = s_tok[j];
        float x = 0.f;
        if (n >= 0) {
            const size_t e = base_k + (size_t)n * st_k + c;
            x = load_elem<TIn>(p.q, e) * dq[e] - load_elem<TIn>(p.k, e) * dk_grad[e];
        }
        s_x[j][c] = x;
    }
    __syncthreads();
    for (int c = 0; c < dk; ++c) {
        const float x = wave_inclusive_scan(s_x[tid][c]);
        s_x[tid][c] = x;
        if (lane == 63) s_wave[wv][c] = x;
    }
    __syncthreads();
    for (int idx = tid; idx < kDgSpan * dk; idx += kDgSpan) {
        const int j = idx / dk, c = idx - j * dk;
        float x = s_x[j][c];
        for (int u = 0; u < (j >> 6); ++u) x += s_wave[u][c];   // the waves that hold later scan steps
        const int n = s_tok[j];
        if (n >= 0) dg[base_k + (size_t)n * st_k + c] = x;
        if (j == kDgSpan - 1) totals[((size_t)bh * ndg + sp) * dk + c] = x;
    }
}

__global__ __launch_bounds__(kDgSpan) void dg_offset_kernel(Params p, float *dg, const float *totals, int ndg) {
    __shared__ float s_off[kMaxDk];
    __shared__ int s_tok[kDgSpan];
    const int tid = threadIdx.x;
    const int bh = blockIdx.x / ndg, sp = blockIdx.x - bh * ndg;
    const int dk = p.dk, T = p.T;
    if (sp == ndg - 1) return;   // nothing after the last span (uniform)
    if (tid < dk) {
        float x = 0.f;
        for (int r = sp + 1; r < ndg; ++r) x += totals[((size_t)bh * ndg + r) * dk + tid];
        s_off[tid] = x;
    }
    {
        const int s = sp * kDgSpan + tid;
        s_tok[tid] = s < T ? scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w) : -1;
    }
    __syncthreads();
    const size_t base_k = slab_k(p, bh), st_k = (size_t)p.st_k;
    for (int idx = tid; idx < kDgSpan * dk; idx += kDgSpan) {
        const int j = idx / dk, c = idx - j * dk;
        const int n = s_tok[j];
        if (n >= 0) dg[base_k + (size_t)n * st_k + c] += s_off[c];
    }
}

}  // namespace

hipError_t launch_row_read(const Params &p, const void *w, float *r, hipStream_t stream) {
    dim3 grid((unsigned)(p.B * p.H * p.nspans)), block(kRowWaves * 64);
    if (p.qkv_dtype == GLA_DT_BF16)
        hipLaunchKernelGGL((row_read_kernel<uint16_t>), grid, block, 0, stream, p, w, r);
    else
        hipLaunchKernelGGL((row_read_kernel<float>), grid, block, 0, stream, p, w, r);
    return hipGetLastError();
}

int dg_spans(int T) { return (T + kDgSpan - 1) / kDgSpan; }

hipError_t launch_dlog_alpha(const Params &p, const float *dq, const float *dk_grad, float *dg, float *totals,
                             hipStream_t stream) {
    const int ndg = dg_spans(p.T);
    dim3 grid((unsigned)(p.B * p.H * ndg)), block(kDgSpan);
    if (p.qkv_dtype == GLA_DT_BF16)
        hipLaunchKernelGGL((dg_local_kernel<uint16_t>), grid, block, 0, stream, p, dq, dk_grad, dg, totals, ndg);
    else
        hipLaunchKernelGGL((dg_local_kernel<float>), grid, block, 0, stream, p, dq, dk_grad, dg, totals, ndg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ndg > 1) hipLaunchKernelGGL(dg_offset_kernel, grid, block, 0, stream, p, dg, totals, ndg);
    return hipGetLastError();
}

}  // namespace gla
