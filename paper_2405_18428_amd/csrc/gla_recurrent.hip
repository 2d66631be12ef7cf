// Token-by-token fp32 engine for one span of the GLA recurrence
// (DiG paper, Sec. 3.1 Eq. (attn_gla) rows 1-3; the value-side gate beta of Eq. (gate_gla_2) is optional).
//
// One work-group walks the scan steps of its span in order.  Thread n owns
// column n of the dk x dv state in registers; q, k and alpha = exp(log_alpha) of
// a tile of tokens are staged in LDS and read as wave-wide broadcasts.  There is
// no factorised decay here, so any gate value (alpha down to 0) is exact; this
// engine serves fp32 inputs, odd head sizes, and as the fallback of the MFMA
// engine.
#include "gla_common.h"

namespace gla {
namespace {

constexpr int kThreads = 128;  // >= kMaxDv
constexpr int kTile = 16;      // tokens staged per round

template <typename T> __device__ inline float load_elem(const void *base, size_t idx);
template <> __device__ inline float load_elem<float>(const void *base, size_t idx) {
    return static_cast<const float *>(base)[idx];
}
template <> __device__ inline float load_elem<uint16_t>(const void *base, size_t idx) {
    return bf16_bits_to_float(static_cast<const uint16_t *>(base)[idx]);
}
template <typename T> __device__ inline void store_elem(void *base, size_t idx, float x);
template <> __device__ inline void store_elem<float>(void *base, size_t idx, float x) {
    static_cast<float *>(base)[idx] = x;
}
template <> __device__ inline void store_elem<uint16_t>(void *base, size_t idx, float x) {
    static_cast<uint16_t *>(base)[idx] = float_to_bf16_bits(x);
}

// BETA: the gate is alpha_t^T beta_t (log_beta given); otherwise diag(alpha_t).
template <int MODE, typename TIn, typename TOut, bool BETA>
__global__ __launch_bounds__(kThreads) void recurrent_span_kernel(Params p) {
    __shared__ float s_b[BETA ? kTile : 1][BETA ? kMaxDv : 1];   // log_beta rows of the tile
    __shared__ float s_q[kTile][kMaxDk];
    __shared__ float s_k[kTile][kMaxDk];
    __shared__ float s_a[kTile][kMaxDk];
    __shared__ float s_v[kTile][kMaxDv];
    __shared__ float s_o[kTile][kMaxDv];   // rows of o awaiting the epilogue
    __shared__ float s_lsum[2][kMaxDk];
    __shared__ int s_tok[kTile];
    __shared__ int s_tokg[kTile];   // token whose gate the scan step uses (the previous step's with gate_shift)

    const int tid = threadIdx.x;
    const int bh = blockIdx.x / p.nspans;
    const int sp = blockIdx.x - bh * p.nspans;
    const int dk = p.dk, dv = p.dv, T = p.T;
    const int s_begin = sp * p.span_len;
    const int s_end = min(T, s_begin + p.span_len);
    const size_t base_k = slab_k(p, bh), base_v = slab_v(p, bh);
    const size_t st_k = (size_t)p.st_k, st_v = (size_t)p.st_v;
    const bool col_active = tid < dv;
    const bool epilogue = MODE == kModeOutput && p.r_pre != nullptr;   // uniform
    const float *lnw = p.ln_weight != nullptr ? p.ln_weight + (size_t)(bh % p.H) * dv : nullptr;
    const float *lnb = p.ln_bias != nullptr ? p.ln_bias + (size_t)(bh % p.H) * dv : nullptr;

    float S[kMaxDk];
#pragma unroll
    for (int c = 0; c < kMaxDk; ++c) S[c] = 0.f;
    // state entering the span: from the carry kernel, or (single span) the caller's initial state
    const float *s0 = nullptr;
    if (MODE == kModeOutput && p.nspans > 1)
        s0 = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;
    else if (MODE == kModeOutput && p.initial_state != nullptr)
        s0 = p.initial_state + (size_t)bh * dk * dv;
    if (s0 != nullptr && col_active) {
#pragma unroll
        for (int c = 0; c < kMaxDk; ++c)
            if (c < dk) S[c] = s0[(size_t)c * dv + tid];
    }

    // staging role: channel sc, token rows sj, sj+2, ...
    const int sc = tid & 63;
    const int sj = tid >> 6;
    float lsum = 0.f;
    float lsum_b = 0.f;     // BETA: summed log_beta of this thread's column

    for (int t0 = s_begin; t0 < s_end; t0 += kTile) {
        __syncthreads();
        if (tid < kTile) {
            int s = t0 + tid;
            s_tok[tid] = (s < s_end) ? scan_token(p.scan_dir, s, T, p.grid_h, p.grid_w) : -1;
            s_tokg[tid] = scan_token(p.scan_dir, max(min(s, s_end - 1) - p.gate_shift, 0), T, p.grid_h, p.grid_w);
        }
        __syncthreads();
        if (sc < dk) {
            for (int j = sj; j < kTile; j += 2) {
                int n = s_tok[j];
                if (n >= 0) {
                    size_t e = base_k + (size_t)n * st_k + sc;
                    float g;
                    if (p.z_gate != nullptr) {   // Eq. (gate_gla): log alpha = logsigmoid(z) / tau
                        const float z = load_elem<TIn>(p.z_gate, base_k + (size_t)s_tokg[j] * st_k + sc);
                        g = (fminf(z, 0.f) - log1pf(expf(-fabsf(z)))) * p.inv_tau;
                    } else {
                        g = p.log_alpha[base_k + (size_t)s_tokg[j] * st_k + sc];
                    }
                    lsum += g;
                    s_a[j][sc] = expf(g);
                    s_k[j][sc] = load_elem<TIn>(p.k, e);
                    if (MODE == kModeOutput) s_q[j][sc] = load_elem<TIn>(p.q, e);
                }
            }
        }
        for (int idx = tid; idx < kTile * dv; idx += kThreads) {
            int j = idx / dv, n2 = idx - j * dv;
            int n = s_tok[j];
            if (n >= 0) {
                s_v[j][n2] = load_elem<TIn>(p.v, base_v + (size_t)n * st_v + n2);
                if constexpr (BETA) {
                    const size_t eb = base_v + (size_t)s_tokg[j] * st_v + n2;
                    if (p.z_beta != nullptr) {   // Eq. (gate_gla_2): log beta = logsigmoid(z) / tau
                        const float z = load_elem<TIn>(p.z_beta, eb);
                        s_b[j][n2] = (fminf(z, 0.f) - log1pf(expf(-fabsf(z)))) * p.inv_tau;
                    } else {
                        s_b[j][n2] = p.log_beta[eb];
                    }
                }
            }
        }
        __syncthreads();
        if (col_active) {
            for (int j = 0; j < kTile; ++j) {
                int n = s_tok[j];
                if (n < 0) break;
                float vn = s_v[j][tid];
                float o = 0.f;
                float bn = 1.f;
                if constexpr (BETA) {
                    const float lb = s_b[j][tid];
                    lsum_b += lb;
                    bn = expf(lb);
                }
#pragma unroll
                for (int c = 0; c < kMaxDk; ++c) {
                    if (c < dk) {
                        S[c] = fmaf(BETA ? s_a[j][c] * bn : s_a[j][c], S[c], s_k[j][c] * vn);
                        if (MODE == kModeOutput) o = fmaf(s_q[j][c], S[c], o);
                    }
                }
                if (MODE == kModeOutput) {
                    if (epilogue) {
                        s_o[j][tid] = o;
                    } else {
                        const size_t e = base_v + (size_t)n * st_v + tid;
                        if (p.accumulate) o += static_cast<const float *>(p.out)[e];   // fp32 rows (host checks)
                        store_elem<TOut>(p.out, e, o);
                    }
                }
            }
        }
        if (epilogue) {
            // Eq. (attn_gla) rows 4-5 up to the projection: Swish(r) * LN(o), 8 threads per token of the tile
            __syncthreads();
            const int j = tid >> 3, sub = tid & 7;
            const int n = s_tok[j];
            const float inv_n = 1.f / (float)dv;
            float sum = 0.f;
            for (int c = sub; c < dv; c += 8) sum += s_o[j][c];
            sum += __shfl_xor(sum, 1);
            sum += __shfl_xor(sum, 2);
            sum += __shfl_xor(sum, 4);
            const float mean = sum * inv_n;
            float sq = 0.f;
            for (int c = sub; c < dv; c += 8) {
                const float d = s_o[j][c] - mean;
                sq = fmaf(d, d, sq);
            }
            sq += __shfl_xor(sq, 1);
            sq += __shfl_xor(sq, 2);
            sq += __shfl_xor(sq, 4);
            const float rstd = 1.f / sqrtf(sq * inv_n + p.ln_eps);
            if (n >= 0) {
                for (int c = sub; c < dv; c += 8) {
                    const size_t e = base_v + (size_t)n * st_v + c;
                    const float r = load_elem<TIn>(p.r_pre, e);
                    const float y = (s_o[j][c] - mean) * rstd * (lnw != nullptr ? lnw[c] : 1.f) + (lnb != nullptr ? lnb[c] : 0.f);
                    store_elem<TOut>(p.out, e, y * (r / (1.f + expf(-r))));
                }
            }
        }
    }

    if (MODE == kModeState) {
        // U of this span and the log of its total decay
        if (col_active) {
            float *u = p.ws_state + ((size_t)bh * p.nspans + sp) * dk * dv;
#pragma unroll
            for (int c = 0; c < kMaxDk; ++c)
                if (c < dk) u[(size_t)c * dv + tid] = S[c];
            if constexpr (BETA) p.ws_lgam_b[((size_t)bh * p.nspans + sp) * dv + tid] = lsum_b;
        }
        s_lsum[sj][sc] = lsum;
        __syncthreads();
        if (tid < dk)
            p.ws_lgam[((size_t)bh * p.nspans + sp) * dk + tid] = s_lsum[0][tid] + s_lsum[1][tid];
    } else if (p.nspans == 1 && p.final_state != nullptr && col_active) {
        float *f = p.final_state + (size_t)bh * dk * dv;
#pragma unroll
        for (int c = 0; c < kMaxDk; ++c)
            if (c < dk) f[(size_t)c * dv + tid] = S[c];
    }
}

template <int MODE, bool BETA>
hipError_t dispatch_gate(const Params &p, hipStream_t stream) {
    dim3 grid((unsigned)(p.B * p.H * p.nspans)), block(kThreads);
    const bool in_bf16 = p.qkv_dtype == GLA_DT_BF16;
    const bool out_bf16 = p.out_dtype == GLA_DT_BF16;
    if (in_bf16 && out_bf16)
        hipLaunchKernelGGL((recurrent_span_kernel<MODE, uint16_t, uint16_t, BETA>), grid, block, 0, stream, p);
    else if (in_bf16)
        hipLaunchKernelGGL((recurrent_span_kernel<MODE, uint16_t, float, BETA>), grid, block, 0, stream, p);
    else if (out_bf16)
        hipLaunchKernelGGL((recurrent_span_kernel<MODE, float, uint16_t, BETA>), grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL((recurrent_span_kernel<MODE, float, float, BETA>), grid, block, 0, stream, p);
    return hipGetLastError();
}

template <int MODE>
hipError_t dispatch(const Params &p, hipStream_t stream) {
    return two_sided(p) ? dispatch_gate<MODE, true>(p, stream) : dispatch_gate<MODE, false>(p, stream);
}

}  // namespace

hipError_t launch_recurrent_span(const Params &p, SpanMode mode, hipStream_t stream) {
    return mode == kModeState ? dispatch<kModeState>(p, stream) : dispatch<kModeOutput>(p, stream);
}

}  // namespace gla
