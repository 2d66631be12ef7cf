// Shared declarations of the GLA library (host + gfx950 device code).
//
// The operation is the gated recurrence of the DiG paper, Sec. 3.1 Eq. (attn_gla)
// rows 1-3 with beta = 1:  S_t = diag(alpha_t) S_{t-1} + k_t^T v_t,  o_t = q_t S_t,
// evaluated span by span (Sec. 3.5: chunks that are computed on-chip):
//   phase 1  every span computes, from a zero state, its local state U and the
//            log of its total decay, log Gamma = sum of log_alpha over the span;
//   phase 2  the spans of one (batch, head) are chained:
//            S_start(r+1) = diag(Gamma_r) S_start(r) + U_r;
//   phase 3  every span recomputes its tokens from S_start(r) and writes o_t.
// Phase 2 is a kernel of its own, or (MFMA engine, up to 128 spans per head) the start
// of phase 3: each work-group then chains the U of the spans before its own.
// The backward pass, the gate prologue / output epilogue, the sums over scan orders and
// the SREM convolution reuse this plan and these parameters.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stdint.h>
#include <stddef.h>

#include "../../include/gla.h"

namespace gla {

constexpr int kChunk = 64;      // tokens per chunk (the paper's M)
constexpr int kMaxDk = 64;
constexpr int kMaxDv = 128;

enum SpanMode : int {
    kModeState = 0,   // phase 1: no outputs, write U and log Gamma of the span
    kModeOutput = 1   // phase 3 (or the single pass): write outputs
};

struct Params {
    const void *q, *k, *v;
    const float *log_alpha;
    void *out;
    float *final_state;     // may be null
    const float *initial_state;  // [B*H, dk, dv] state before the first scan step, or null (zero)
    // element strides of the [B,H,T,d] tensors: q, k, log_alpha (suffix k) and v, out (suffix v)
    long long sb_k, sh_k, sb_v, sh_v;   // batch, head
    int st_k, st_v;                     // token (row) stride
    float *ws_state;        // [B*H, nspans, dk, dv]  U_r after phase 1, S_start(r) after phase 2
    float *ws_lgam;         // [B*H, nspans, dk]      log Gamma_r
    int B, H, T, dk, dv, grid_h, grid_w, scan_dir;
    int nspans;             // spans per (batch, head)
    int span_len;           // tokens per span, a multiple of kChunk
    int gate_shift;         // 1: scan step s uses the log_alpha row of the token visited at step s-1 (the
                            //    reverse-mode recurrence dS_s = diag(alpha_{s+1}) dS_{s+1} + q_s^T dO_s walked backwards)
    int chain_in_output;    // 1: no phase-2 kernel; the output pass chains U_0..U_{r-1} itself and phase 1
                            //    skips the last span of every (batch, head) (nobody reads its U)
    int qkv_dtype, out_dtype;
    int accumulate;         // 1: the output pass adds its rows to what `out` (fp32) holds (sums over scan orders)
    // gate prologue (Eq. (gate_gla)): if z_gate is set, log_alpha is not read; the gate of a row is
    // logsigmoid(z) * inv_tau, z in the element type of q, k, v and laid out like log_alpha
    const void *z_gate;
    float inv_tau;
    // output epilogue (Eq. (attn_gla) rows 4-5 up to the output projection): if r_pre is set, the stored row is
    // Swish(r_pre) * LN(o) with LN over the dv entries of the head; r_pre in the element type of q, k, v and laid
    // out like v; ln_weight / ln_bias: [H, dv] fp32 or null (1 and 0)
    const void *r_pre;
    const float *ln_weight, *ln_bias;
    float ln_eps;
    // value-side gate (Eq. (gate_gla_2)): if log_beta is set ([B,H,T,dv] fp32, laid out like v), the state element
    // (c, n) decays by alpha_t[c] * beta_t[n]; token-by-token engine only
    const float *log_beta;
    const void *z_beta;     // or (with z_gate) its pre-activation: log beta = logsigmoid(z_beta) * inv_tau, like v
    float *ws_lgam_b;       // [B*H, nspans, dv]  summed log_beta of each span (phase 1 -> phase 2)
    // fp16 engine (gla_fast.hip): one flag per span, raised by its passes when the span's gates or operands leave
    // the range its fp16 operands cover; with only_flagged the bf16 hi/lo output pass (launched with one span per
    // head) recomputes the (batch, head) sequences that have a raised flag and leaves the others alone
    int *ws_fail;           // [B*H, nspans of the fp16 engine's plan]
    int only_flagged;
    int fail_spans;         // flags per (batch, head) when only_flagged is set
};

// the gate has a value-side factor
__host__ __device__ inline bool two_sided(const Params &p) { return p.log_beta != nullptr || p.z_beta != nullptr; }

// Scan step s -> canonical token index (Sec. 3.3 / Algorithm 1 orders).
__host__ __device__ inline int scan_token(int scan_dir, int s, int T, int grid_h, int grid_w) {
    if (scan_dir & 1) s = T - 1 - s;
    if (scan_dir < 2) return s;
    int c = s / grid_h;
    int r = s - c * grid_h;
    return r * grid_w + c;
}

// bf16 <-> fp32 on raw bit patterns (round to nearest even; inputs are finite).
__host__ __device__ inline float bf16_bits_to_float(uint16_t b) {
    union { uint32_t u; float f; } x;
    x.u = ((uint32_t)b) << 16;
    return x.f;
}
__host__ __device__ inline uint16_t float_to_bf16_bits(float f) {
    union { uint32_t u; float f; } x;
    x.f = f;
    uint32_t u = x.u;
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Element offset of the (batch, head) slab `bh` in the dk-sized / dv-sized tensors.
__host__ __device__ inline size_t slab_k(const Params &p, int bh) {
    return (size_t)(bh / p.H) * (size_t)p.sb_k + (size_t)(bh % p.H) * (size_t)p.sh_k;
}
__host__ __device__ inline size_t slab_v(const Params &p, int bh) {
    return (size_t)(bh / p.H) * (size_t)p.sb_v + (size_t)(bh % p.H) * (size_t)p.sh_v;
}

// Raises a kernel's dynamic-LDS limit once per device and kernel (`done` is the caller's per-kernel flag array,
// indexed by device ordinal; the attribute is per device).
constexpr int kMaxDevices = 64;
inline hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<bool> (&done)[kMaxDevices]) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices || !done[dev]) {
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < kMaxDevices) done[dev] = true;
    }
    return hipSuccess;
}

// Launchers (defined in the .hip files); each enqueues on `stream` and returns
// hipGetLastError().
hipError_t launch_recurrent_span(const Params &p, SpanMode mode, hipStream_t stream);
hipError_t launch_mfma_span(const Params &p, SpanMode mode, hipStream_t stream);
hipError_t launch_carry(const Params &p, hipStream_t stream);
bool mfma_engine_supports(const Params &p);
// fp16 output pass with the pipelined chunk loop (gla_fast.hip): what it covers, how many of its work-groups a
// compute unit holds, and its launcher
bool fast_engine_supports(const Params &p);
int fast_groups_per_cu(const Params &p);
hipError_t launch_fast_output(const Params &p, hipStream_t stream);
hipError_t launch_fast_state(const Params &p, hipStream_t stream);   // its span-state pass (phase 1)
// backward-only kernels: r_s[c] = sum_n S_s[c,n] w_s[n] over the states of (p.k, p.v, p.log_alpha); and
// dlog_alpha = reverse cumulative sum of q * dq - k * dk (totals: [B*H, dg_spans(T), dk] floats of scratch)
hipError_t launch_row_read(const Params &p, const void *w, float *r, hipStream_t stream);
// the same on the MFMA units (chunk form); needs what mfma_engine_supports() checks
hipError_t launch_mfma_row_read(const Params &p, const void *w, float *r, hipStream_t stream,
                                bool with_outputs = false);   // with_outputs: also o_j = q_j S_j (p.q) to p.out, fp32
hipError_t launch_dlog_alpha(const Params &p, const float *dq, const float *dk_grad, float *dg, float *totals,
                             hipStream_t stream);
int dg_spans(int T);
// 3x3 depth-wise convolution of the SREM on [B, T, D] tokens (gla_srem.hip)
hipError_t launch_srem_dwconv(const void *x, const float *w, const float *bias, void *y, int B, int gh, int gw, int D,
                              int orient, int x_dtype, int y_dtype, hipStream_t stream);

}  // namespace gla
