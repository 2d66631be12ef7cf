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
// The rows v_s and w_s (the vector the state is read with) are the same for all lanes,
// so they are fetched with scalar loads and feed the vector ALU as scalar operands.
#include "gla_common.h"

namespace gla {
namespace {

constexpr int kTile = 16;          // tokens staged per round
constexpr int kRowWaves = 2;       // waves per work-group; each owns half of the value columns
constexpr int kColsPerWave = kMaxDv / kRowWaves;
constexpr int kColStep = 16;       // value columns whose scalars are in flight at once

typedef const __attribute__((address_space(4))) uint32_t *const_u32;   // constant address space: scalar loads
typedef const __attribute__((address_space(4))) float *const_f32;

template <typename TIn> struct ScalarRow;
// 16 neighbouring columns of a bf16 row as 8 uniform dwords
// (ncols, the number of columns that exist from col0 on, is even for bf16: no dword straddles the row end)
template <> struct ScalarRow<uint16_t> {
    uint32_t w[kColStep / 2];
    __device__ void load(const void *row, int col0, int ncols) {
        const_u32 p = (const_u32)(uintptr_t)(static_cast<const uint16_t *>(row) + col0);
        if (ncols >= kColStep) {
#pragma unroll
            for (int i = 0; i < kColStep / 2; ++i) w[i] = p[i];
        } else {
#pragma unroll
            for (int i = 0; i < kColStep / 2; ++i) w[i] = (2 * i < ncols) ? p[i] : 0u;
        }
    }
    __device__ float get(int i) const {
        const uint32_t x = w[i >> 1];
        return __builtin_bit_cast(float, (i & 1) ? (x & 0xffff0000u) : (x << 16));
    }
};
template <> struct ScalarRow<float> {
    float w[kColStep];
    __device__ void load(const void *row, int col0, int ncols) {
        const_f32 p = (const_f32)(uintptr_t)(static_cast<const float *>(row) + col0);
        if (ncols >= kColStep) {
#pragma unroll
            for (int i = 0; i < kColStep; ++i) w[i] = p[i];
        } else {
#pragma unroll
            for (int i = 0; i < kColStep; ++i) w[i] = (i < ncols) ? p[i] : 0.f;
        }
    }
    __device__ float get(int i) const { return w[i]; }
};

template <typename T> __device__ inline float load_elem(const void *base, size_t idx);
template <> __device__ inline float load_elem<float>(const void *base, size_t idx) {
    return static_cast<const float *>(base)[idx];
}
template <> __device__ inline float load_elem<uint16_t>(const void *base, size_t idx) {
    return bf16_bits_to_float(static_cast<const uint16_t *>(base)[idx]);
}

// r_s[c] = sum_n S_s[c,n] w_s[n] for the scan steps of one span; S follows (p.k, p.v, p.log_alpha).
// p.q is not used; `w` has the layout of p.v, `r` (fp32) that of p.k.  Scalar loads are dword loads: bf16 rows
// must start on 4-byte boundaries and have an even number of columns (checked by the host).
template <typename TIn>
__global__ __launch_bounds__(kRowWaves * 64) void row_read_kernel(Params p, const void *w, float *r) {
    __shared__ float s_a[kTile][kMaxDk];
    __shared__ float s_k[kTile][kMaxDk];
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
    // columns of this wave: [col_lo, col_hi), walked in steps of kColStep (the last step may be partial)
    const int per_wave = ((dv + kRowWaves * kColStep - 1) / (kRowWaves * kColStep)) * kColStep;
    const int col_lo = half * per_wave;
    const int col_hi = min(dv, col_lo + per_wave);
    const bool row_active = c < dk;

    float S[kColsPerWave];
#pragma unroll
    for (int n = 0; n < kColsPerWave; ++n) S[n] = 0.f;
    if (p.nspans > 1 && row_active) {
        const float *s0 = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv + (size_t)c * dv;
#pragma unroll
        for (int n = 0; n < kColsPerWave; ++n)
            if (col_lo + n < col_hi) S[n] = s0[col_lo + n];
    }

    for (int t0 = s_begin; t0 < s_end; t0 += kTile) {
        __syncthreads();
        if (tid < kTile) {
            const int s = min(t0 + tid, s_end - 1);
            s_tok[tid] = (t0 + tid < s_end) ? scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w) : -1;
            s_tokg[tid] = scan_token(p.scan_dir, max(s - p.gate_shift, 0), T, p.grid_h, p.grid_w);
        }
        __syncthreads();
        // stage alpha and k of the tile: thread (half, c) takes tokens half, half + 2, ...
        if (row_active) {
            for (int j = half; j < kTile; j += kRowWaves) {
                const int n = s_tok[j];
                if (n >= 0) {
                    s_a[j][c] = expf(p.log_alpha[base_k + (size_t)s_tokg[j] * st_k + c]);
                    s_k[j][c] = load_elem<TIn>(p.k, base_k + (size_t)n * st_k + c);
                }
            }
        }
        __syncthreads();
        for (int j = 0; j < kTile; ++j) {
            const int n = __builtin_amdgcn_readfirstlane(s_tok[j]);
            if (n < 0) break;
            const float a = s_a[j][c], kc = s_k[j][c];
            const char *vrow = static_cast<const char *>(p.v) + (base_v + (size_t)n * st_v) * sizeof(TIn);
            const char *wrow = static_cast<const char *>(w) + (base_v + (size_t)n * st_v) * sizeof(TIn);
            float acc = 0.f;
#pragma unroll
            for (int n0 = 0; n0 < kColsPerWave; n0 += kColStep) {
                if (col_lo + n0 < col_hi) {   // uniform
                    ScalarRow<TIn> vs, ws;
                    vs.load(vrow, col_lo + n0, col_hi - col_lo - n0);
                    ws.load(wrow, col_lo + n0, col_hi - col_lo - n0);
#pragma unroll
                    for (int i = 0; i < kColStep; ++i) {
                        if (col_lo + n0 + i < col_hi) {   // uniform
                            S[n0 + i] = fmaf(a, S[n0 + i], kc * vs.get(i));
                            acc = fmaf(S[n0 + i], ws.get(i), acc);
                        }
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
constexpr int kDgSpan = 256;       // scan steps per work-group (4 waves of 64 lanes)

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

template <typename TIn>
__global__ __launch_bounds__(kDgSpan) void dg_local_kernel(Params p, const float *dq, const float *dk_grad,
                                                          float *dg, float *totals, int ndg) {
    __shared__ float s_wave[kDgSpan / 64][kMaxDk];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int bh = blockIdx.x / ndg, sp = blockIdx.x - bh * ndg;
    const int dk = p.dk, T = p.T;
    const size_t base_k = slab_k(p, bh), st_k = (size_t)p.st_k;
    // thread tid handles scan step s = span end - 1 - tid: prefix sums over tid are suffix sums over s
    const int s_last = min(T, (sp + 1) * kDgSpan) - 1;
    const int s = s_last - tid;
    const bool valid = s >= sp * kDgSpan;
    const int n = scan_token(p.scan_dir, valid ? s : s_last, T, p.grid_h, p.grid_w);
    const size_t row = base_k + (size_t)n * st_k;
    for (int c = 0; c < dk; ++c) {
        float x = 0.f;
        if (valid)
            x = load_elem<TIn>(p.q, row + c) * dq[row + c] - load_elem<TIn>(p.k, row + c) * dk_grad[row + c];
        x = wave_inclusive_scan(x);
        if (lane == 63) s_wave[wv][c] = x;
        __syncthreads();
        float before = 0.f;   // the waves that hold later scan steps
        for (int u = 0; u < wv; ++u) before += s_wave[u][c];
        x += before;
        if (valid) dg[row + c] = x;
        if (tid == kDgSpan - 1) totals[((size_t)bh * ndg + sp) * dk + c] = x;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kDgSpan) void dg_offset_kernel(Params p, float *dg, const float *totals, int ndg) {
    __shared__ float s_off[kMaxDk];
    const int tid = threadIdx.x;
    const int bh = blockIdx.x / ndg, sp = blockIdx.x - bh * ndg;
    const int dk = p.dk, T = p.T;
    if (sp == ndg - 1) return;   // nothing after the last span (uniform)
    if (tid < dk) {
        float x = 0.f;
        for (int r = sp + 1; r < ndg; ++r) x += totals[((size_t)bh * ndg + r) * dk + tid];
        s_off[tid] = x;
    }
    __syncthreads();
    const int s = sp * kDgSpan + tid;
    if (s >= T) return;
    const int n = scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w);
    float *row = dg + slab_k(p, bh) + (size_t)n * p.st_k;
    for (int c = 0; c < dk; ++c) row[c] += s_off[c];
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
