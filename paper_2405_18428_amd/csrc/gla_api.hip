// Host side of the C ABI declared in include/gla.h: argument validation, launch
// plan, library-owned scratch for gla_fwd, and the timing aid.
#include <atomic>
#include <mutex>
#include <vector>

#include "gla_common.h"

namespace gla {
namespace {

constexpr int kVersion = 330;  // 0.3.3

// process-wide options (gla_set_option): atomics, so that a setter on one host thread and calls on another do not
// race on them; a call reads them as it goes, so options are meant to be set between calls, not during one
std::atomic<int> g_opt_chunks_per_span{0};
std::atomic<int> g_opt_engine{GLA_ENGINE_AUTO};
std::atomic<int> g_opt_carry{GLA_CARRY_AUTO};
std::atomic<int> g_opt_bwd_split{0};
std::atomic<int> g_opt_range_fallback{1};

// Most spans per (batch, head) that the output pass chains by itself: work-group r reads the r local states
// before it, so the reads grow with the square of the span count while a carry kernel's grow linearly.
constexpr int kMaxChainedSpans = 128; // beyond this the reads of a slowly decaying chain outgrow the carry kernel

struct Scratch {
    void *ptr = nullptr;
    size_t bytes = 0;
};
std::mutex g_scratch_mutex;
Scratch g_scratch[64];  // indexed by HIP device ordinal

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t workspace_bytes(int B, int H, int T, int dk, int dv) {
    // upper bound: one span per chunk
    size_t nspans = ((size_t)T + kChunk - 1) / kChunk;
    size_t bh = (size_t)B * H;
    size_t state = align_up(bh * nspans * dk * dv * sizeof(float), 256);
    size_t lgam = align_up(bh * nspans * dk * sizeof(float), 256);
    size_t lgam_b = align_up(bh * nspans * dv * sizeof(float), 256);   // value-side gate sums (two-sided gate only)
    size_t flags = align_up(bh * nspans * sizeof(int), 256);           // fp16 engine: one range flag per span
    return state + lgam + lgam_b + flags;
}

// what a plan of `nspans` spans per (batch, head) really uses (the three arrays that choose_engine_and_plan lays out)
size_t plan_workspace_bytes(size_t bh, size_t nspans, int dk, int dv) {
    return align_up(bh * nspans * dk * dv * sizeof(float), 256) + align_up(bh * nspans * dk * sizeof(float), 256) +
           align_up(bh * nspans * dv * sizeof(float), 256) + align_up(bh * nspans * sizeof(int), 256);
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int validate(const void *q, const void *k, const void *v, const float *log_alpha,
             int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
             int qkv_dtype, int out_dtype, const void *out, const float *final_state) {
    if (!q || !k || !v || !log_alpha || !out) return GLA_ERR_NULL;
    if (B <= 0 || H <= 0 || T <= 0 || dk <= 0 || dv <= 0 || grid_h <= 0 || grid_w <= 0) return GLA_ERR_SHAPE;
    if ((long long)grid_h * grid_w != (long long)T) return GLA_ERR_SHAPE;
    if (scan_dir < 0 || scan_dir > 3) return GLA_ERR_SHAPE;
    if (qkv_dtype != GLA_DT_F32 && qkv_dtype != GLA_DT_BF16) return GLA_ERR_SHAPE;
    if (out_dtype != GLA_DT_F32 && out_dtype != GLA_DT_BF16) return GLA_ERR_SHAPE;
    if ((long long)B * H > 0x7fffffffLL / (((long long)T + kChunk - 1) / kChunk)) return GLA_ERR_SHAPE;
    if (dk > kMaxDk || dv > kMaxDv) return GLA_ERR_UNSUPPORTED;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(log_alpha) || misaligned(out) ||
        (final_state && misaligned(final_state)))
        return GLA_ERR_ALIGN;
    return GLA_OK;
}

// Chooses how many 64-token chunks one work-group walks.  Long spans amortise
// the state traffic of phases 1-3 (about 4 * dk * dv * 4 bytes per span) and the
// per-work-group prologue; short spans give the 256 compute units more
// work-groups.  Two resident work-groups per compute unit is the sweet spot
// measured on MI355X for the output pass.
int plan_chunks_per_span(int bh, int nchunks, bool mfma_engine, int groups_per_cu = 2, bool fp16_engine = false) {
    int cps = g_opt_chunks_per_span;
    if (cps <= 0 && fp16_engine) {
        // fp16 engine: a work-group spends about three chunk periods on its prologue (span-state chain, pipeline
        // fill) whatever the span length, and a chunk period is about 0.62 as long when the group has its compute
        // unit to itself (measured on MI355X: 1024 / 2048 / 4096 chunks of DiG-XL/2 and 1176 of DiG-S/2 at 1792 px
        // with 1..16 chunks per span).  Cost of a plan in chunk periods: rounds of resident groups x (cps + 3) x
        // (1 if two groups share a compute unit, else 0.62); the cheapest plan wins, ties go to the shorter span.
        const long long total = (long long)bh * nchunks;
        double best = 0.0;
        for (int c = 1; c <= nchunks; ++c) {
            const long long groups = (long long)bh * ((nchunks + c - 1) / c);
            const long long resident = 256LL * groups_per_cu;
            const double rounds = (double)((groups + resident - 1) / resident);
            const double period = (groups_per_cu >= 2 && groups > 256) ? 1.0 : 0.62;
            const double cost = rounds * (c + 3) * period;
            if (cps <= 0 || cost < best - 1e-9) {
                best = cost;
                cps = c;
            }
            if (groups <= 128 && total > 128) break;   // longer spans only idle more compute units
        }
    }
    if (cps <= 0) {
        // no more work-groups than are resident at once (two per compute unit); sequences of up to four chunks are
        // walked in one pass (a second kernel costs more than the chunks it would save)
        const long long resident_groups = 256LL * groups_per_cu;
        cps = (int)(((long long)bh * nchunks + resident_groups - 1) / resident_groups);
        if (cps < 1) cps = 1;
        if (mfma_engine && nchunks <= 4) cps = nchunks;
    }
    if (cps > nchunks) cps = nchunks;
    return cps;
}

// Engine for the span passes (p.qkv_dtype, sizes and strides must be set) and the span plan with its workspace.
// use_fast (optional): the caller is the plain forward pass and would take the fp16 output pass where it covers
// the call; on return, whether it does (the span plan is then sized for that kernel's residency).
int choose_engine_and_plan(Params &p, void *workspace, bool &use_mfma, bool *use_fast = nullptr) {
    if (g_opt_engine == GLA_ENGINE_RECURRENT) {
        use_mfma = false;
    } else if (g_opt_engine == GLA_ENGINE_MFMA || g_opt_engine == GLA_ENGINE_MFMA_FP16) {
        if (!mfma_engine_supports(p)) return GLA_ERR_UNSUPPORTED;
        use_mfma = true;
    } else {
        use_mfma = mfma_engine_supports(p);
    }
    bool fast = false;
    if (use_fast != nullptr) {
        fast = use_mfma && g_opt_engine != GLA_ENGINE_MFMA && fast_engine_supports(p);
        if (g_opt_engine == GLA_ENGINE_MFMA_FP16 && !fast) return GLA_ERR_UNSUPPORTED;
        *use_fast = fast;
    }
    const int nchunks = (p.T + kChunk - 1) / kChunk;
    // short sequences are one span on the bf16 hi/lo kernel: a single pass, and no launch for the range fallback
    if (fast && nchunks <= 4 && g_opt_engine != GLA_ENGINE_MFMA_FP16 && g_opt_chunks_per_span <= 0) {
        fast = false;
        *use_fast = false;
    }
    const int cps = plan_chunks_per_span(p.B * p.H, nchunks, use_mfma, fast ? fast_groups_per_cu(p) : 2, fast);
    p.span_len = cps * kChunk;
    p.nspans = (nchunks + cps - 1) / cps;
    const size_t bh = (size_t)p.B * p.H;
    p.ws_state = static_cast<float *>(workspace);
    p.ws_lgam = reinterpret_cast<float *>(static_cast<char *>(workspace) +
                                          align_up(bh * p.nspans * p.dk * p.dv * sizeof(float), 256));
    p.ws_lgam_b = reinterpret_cast<float *>(reinterpret_cast<char *>(p.ws_lgam) +
                                            align_up(bh * p.nspans * p.dk * sizeof(float), 256));
    p.ws_fail = reinterpret_cast<int *>(reinterpret_cast<char *>(p.ws_lgam_b) +
                                        align_up(bh * p.nspans * p.dv * sizeof(float), 256));
    return GLA_OK;
}

void set_dense_bhtd_strides(Params &p) {
    p.st_k = p.dk; p.sh_k = (long long)p.T * p.dk; p.sb_k = (long long)p.H * p.T * p.dk;
    p.st_v = p.dv; p.sh_v = (long long)p.T * p.dv; p.sb_v = (long long)p.H * p.T * p.dv;
}

size_t bwd_totals_bytes(int B, int H, int T, int dk) {
    return align_up((size_t)B * H * dg_spans(T) * dk * sizeof(float), 256);
}

// Backward pass (see gla_bwd_kernels.hip for the formulas): three walks over the sequence on the span plan of
// the forward pass, then the reverse cumulative sum for the gate gradient.
int run_bwd(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
            int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
            float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
            void *workspace, size_t ws_bytes, hipStream_t stream,
            const void *fwd_workspace = nullptr, size_t fwd_ws_bytes = 0, int layout = GLA_LAYOUT_BHTD) {
    if (!d_out || !dq || !dk_grad || !dv_grad || !dlog_alpha) return GLA_ERR_NULL;
    if (layout != GLA_LAYOUT_BHTD && layout != GLA_LAYOUT_BTHD) return GLA_ERR_SHAPE;
    int st = validate(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                      qkv_dtype, GLA_DT_F32, dv_grad, nullptr);
    if (st != GLA_OK) return st;
    if (misaligned(d_out) || misaligned(dq) || misaligned(dk_grad) || misaligned(dlog_alpha)) return GLA_ERR_ALIGN;
    const size_t state_bytes = workspace_bytes(B, H, T, dk, dv);
    if (!workspace || misaligned(workspace) || ws_bytes < state_bytes + bwd_totals_bytes(B, H, T, dk))
        return GLA_ERR_WORKSPACE;
    float *totals = reinterpret_cast<float *>(static_cast<char *>(workspace) + state_bytes);
    if (fwd_workspace && (misaligned(fwd_workspace) || fwd_ws_bytes < state_bytes || fwd_workspace == workspace))
        return GLA_ERR_WORKSPACE;

    Params base{};
    base.B = B; base.H = H; base.T = T; base.dk = dk; base.dv = dv;
    base.grid_h = grid_h; base.grid_w = grid_w;
    base.qkv_dtype = qkv_dtype; base.out_dtype = GLA_DT_F32;
    if (layout == GLA_LAYOUT_BHTD) {
        set_dense_bhtd_strides(base);
    } else {  // [B,T,H,d]: the heads of one token are neighbours (gradients in the same order)
        base.st_k = H * dk; base.sh_k = dk; base.sb_k = (long long)T * H * dk;
        base.st_v = H * dv; base.sh_v = dv; base.sb_v = (long long)T * H * dv;
    }
    bool use_mfma;
    st = choose_engine_and_plan(base, workspace, use_mfma);
    if (st != GLA_OK) return st;
    // MFMA engine with few spans per head: every kernel that needs the state entering its span chains the local
    // states itself (as the forward output pass does); otherwise the carry kernel chains them in place
    base.chain_in_output = use_mfma && base.nspans > 1 &&
                           (g_opt_carry == GLA_CARRY_IN_OUTPUT_PASS ||
                            (g_opt_carry == GLA_CARRY_AUTO && base.nspans <= kMaxChainedSpans));
    auto span = [&](const Params &p, SpanMode mode) {
        return use_mfma ? launch_mfma_span(p, mode, stream) : launch_recurrent_span(p, mode, stream);
    };
    auto row_read = [&](const Params &p, const void *w, float *r) {
        return use_mfma ? launch_mfma_row_read(p, w, r, stream) : launch_row_read(p, w, r, stream);
    };
    auto states = [&](const Params &p) {   // span-local states, then chained in place
        if (p.nspans <= 1) return hipSuccess;
        hipError_t e = span(p, kModeState);
        if (e != hipSuccess || p.chain_in_output) return e;
        return launch_carry(p, stream);
    };

    // 1. states of the forward recurrence (k, v, log_alpha); dq_s = S_s dO_s
    Params pa = base;
    pa.k = k; pa.v = v; pa.log_alpha = log_alpha; pa.scan_dir = scan_dir; pa.gate_shift = 0;
    if (fwd_workspace && pa.nspans > 1) {
        // The forward call on the same tensors ran this very state pass.  Its workspace holds either the chained
        // states S_start(r) (carry kernel) or the local states U_r and log Gamma_r (chained inside its output
        // pass), by the rule that also sets base.chain_in_output.
        Params pf = base;
        bool same_engine, fwd_fast = false;
        if (choose_engine_and_plan(pf, const_cast<void *>(fwd_workspace), same_engine, &fwd_fast) != GLA_OK)
            return GLA_ERR_HIP;
        // either way the states are read where they are: the row-read kernel chains local states itself.
        // The walk adopts the forward call's span plan (its output pass may have been sized differently).
        pa.ws_state = pf.ws_state;
        pa.ws_lgam = pf.ws_lgam;
        pa.nspans = pf.nspans;
        pa.span_len = pf.span_len;
        pa.chain_in_output = use_mfma && pa.nspans > 1 &&
                             (g_opt_carry == GLA_CARRY_IN_OUTPUT_PASS ||
                              (g_opt_carry == GLA_CARRY_AUTO && pa.nspans <= kMaxChainedSpans));
    } else if (states(pa) != hipSuccess) {
        return GLA_ERR_HIP;
    }
    if (row_read(pa, d_out, dq) != hipSuccess) return GLA_ERR_HIP;

    // 2. states of the reversed recurrence G_s = q_s^T dO_s + diag(alpha_{s+1}) G_{s+1}: the forward recurrence
    //    with k, v := q, dO, walked from the last scan step, each step using the previous step's gate
    Params pb = base;
    pb.q = k; pb.k = q; pb.v = d_out; pb.log_alpha = log_alpha; pb.scan_dir = scan_dir ^ 1; pb.gate_shift = 1;
    pb.out = dv_grad;
    if (states(pb) != hipSuccess) return GLA_ERR_HIP;
    if (use_mfma && !g_opt_bwd_split) {
        // one walk over the chunks of G for both dk_s = G_s v_s (row read) and dv_s = k_s G_s (outputs with q := k)
        if (launch_mfma_row_read(pb, v, dk_grad, stream, true) != hipSuccess) return GLA_ERR_HIP;
    } else {
        if (span(pb, kModeOutput) != hipSuccess) return GLA_ERR_HIP;             // dv_s = k_s G_s
        if (row_read(pb, v, dk_grad) != hipSuccess) return GLA_ERR_HIP;          // dk_s = G_s v_s
    }

    // 3. dlog_alpha = reverse cumulative sum of q * dq - k * dk along the scan
    Params pc = base;
    pc.q = q; pc.k = k; pc.scan_dir = scan_dir;
    if (launch_dlog_alpha(pc, dq, dk_grad, dlog_alpha, totals, stream) != hipSuccess) return GLA_ERR_HIP;
    return GLA_OK;
}

// Backward pass with the two-sided gate alpha_t^T beta_t.  Same walks as run_bwd; the adjoint state obeys
// G_s = q_s^T dO_s + (alpha_{s+1}^T beta_{s+1}) * G_{s+1}.  Every kernel runs on the engine the forward call would
// take.  The value-side gate gradient is the reverse cumulative sum of o * dO - v * dv, so the outputs o are
// recomputed first (fp32, in the workspace).
size_t bwd_gates_out_bytes(int B, int H, int T, int dv) { return align_up((size_t)B * H * T * dv * sizeof(float), 256); }

int run_bwd_gates(const void *q, const void *k, const void *v, const float *log_alpha, const float *log_beta,
                  const void *d_out, const float *out_fwd, int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha, float *dlog_beta,
                  void *workspace, size_t ws_bytes, hipStream_t stream) {
    if (!log_beta || !d_out || !dq || !dk_grad || !dv_grad || !dlog_alpha || !dlog_beta) return GLA_ERR_NULL;
    int st = validate(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                      qkv_dtype, GLA_DT_F32, dv_grad, nullptr);
    if (st != GLA_OK) return st;
    if (misaligned(log_beta) || misaligned(d_out) || misaligned(out_fwd) || misaligned(dq) || misaligned(dk_grad) || misaligned(dlog_alpha) ||
        misaligned(dlog_beta))
        return GLA_ERR_ALIGN;
    const size_t state_bytes = workspace_bytes(B, H, T, dk, dv);
    const size_t totals_bytes = bwd_totals_bytes(B, H, T, dk > dv ? dk : dv);
    if (!workspace || misaligned(workspace) ||
        ws_bytes < state_bytes + totals_bytes + bwd_gates_out_bytes(B, H, T, dv))
        return GLA_ERR_WORKSPACE;
    float *totals = reinterpret_cast<float *>(static_cast<char *>(workspace) + state_bytes);
    float *o_buf = reinterpret_cast<float *>(static_cast<char *>(workspace) + state_bytes + totals_bytes);

    Params base{};
    base.B = B; base.H = H; base.T = T; base.dk = dk; base.dv = dv;
    base.grid_h = grid_h; base.grid_w = grid_w;
    base.qkv_dtype = qkv_dtype; base.out_dtype = GLA_DT_F32;
    base.log_alpha = log_alpha; base.log_beta = log_beta;
    set_dense_bhtd_strides(base);
    bool use_mfma;
    st = choose_engine_and_plan(base, workspace, use_mfma);
    if (st != GLA_OK) return st;
    // as in run_bwd: with the MFMA engine and few spans every kernel chains the span states it needs itself
    base.chain_in_output = use_mfma && base.nspans > 1 &&
                           (g_opt_carry == GLA_CARRY_IN_OUTPUT_PASS ||
                            (g_opt_carry == GLA_CARRY_AUTO && base.nspans <= kMaxChainedSpans));
    auto span = [&](const Params &p, SpanMode mode) {
        return use_mfma ? launch_mfma_span(p, mode, stream) : launch_recurrent_span(p, mode, stream);
    };
    auto states = [&](const Params &p) {
        if (p.nspans <= 1) return hipSuccess;
        hipError_t e = span(p, kModeState);
        if (e != hipSuccess || p.chain_in_output) return e;
        return launch_carry(p, stream);
    };
    // value-axis reads of the state: chunk form on the MFMA units where the engine covers the case
    auto row_read = [&](const Params &p, const void *w, float *r) {
        return use_mfma ? launch_mfma_row_read(p, w, r, stream) : launch_row_read(p, w, r, stream);
    };

    // 1. forward recurrence: states entering the spans, the outputs o (for the value-side gate gradient),
    //    dq_s = S_s dO_s
    Params pa = base;
    pa.q = q; pa.k = k; pa.v = v; pa.scan_dir = scan_dir; pa.gate_shift = 0; pa.out = o_buf;
    if (states(pa) != hipSuccess) return GLA_ERR_HIP;
    if (!out_fwd && span(pa, kModeOutput) != hipSuccess) return GLA_ERR_HIP;   // (the caller may still hold o)
    if (row_read(pa, d_out, dq) != hipSuccess) return GLA_ERR_HIP;

    // 2. adjoint recurrence (k, v := q, dO; walked from the last scan step, each step with the previous step's
    //    gates): dv_s = k_s G_s (outputs with q := k), dk_s = G_s v_s
    Params pb = base;
    pb.q = k; pb.k = q; pb.v = d_out; pb.scan_dir = scan_dir ^ 1; pb.gate_shift = 1; pb.out = dv_grad;
    if (states(pb) != hipSuccess) return GLA_ERR_HIP;
    if (use_mfma && !g_opt_bwd_split) {
        // one walk over the chunks of G for both dk (row read) and dv (outputs with q := k)
        if (launch_mfma_row_read(pb, v, dk_grad, stream, true) != hipSuccess) return GLA_ERR_HIP;
    } else {
        if (span(pb, kModeOutput) != hipSuccess) return GLA_ERR_HIP;
        if (row_read(pb, v, dk_grad) != hipSuccess) return GLA_ERR_HIP;
    }

    // 3. gate gradients: reverse cumulative sums of q * dq - k * dk (key side) and of dO * o - v * dv (value
    //    side: the same kernels over the dv columns, with dO, v in the places of q, k)
    Params pc = base;
    pc.q = q; pc.k = k; pc.scan_dir = scan_dir;
    if (launch_dlog_alpha(pc, dq, dk_grad, dlog_alpha, totals, stream) != hipSuccess) return GLA_ERR_HIP;
    Params pd = base;
    pd.q = d_out; pd.k = v; pd.scan_dir = scan_dir;
    pd.dk = dv; pd.st_k = base.st_v; pd.sh_k = base.sh_v; pd.sb_k = base.sb_v;
    if (launch_dlog_alpha(pd, out_fwd ? out_fwd : o_buf, dv_grad, dlog_beta, totals, stream) != hipSuccess)
        return GLA_ERR_HIP;
    return GLA_OK;
}

// arguments of the gate prologue and the output epilogue (gla_fwd_fused)
struct FusedArgs {
    const void *z;
    float tau;
    const void *r_pre;
    const float *ln_weight, *ln_bias;
    float ln_eps;
    const void *z_beta;     // pre-activation of the value-side gate, or null (beta = 1)
};

struct PhaseEvents {
    hipEvent_t ev[4];
};

int run(const void *q, const void *k, const void *v, const float *log_alpha,
        int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
        int qkv_dtype, int out_dtype, void *out, float *final_state,
        void *workspace, size_t ws_bytes, hipStream_t stream, PhaseEvents *events,
        int layout = GLA_LAYOUT_BHTD, const float *initial_state = nullptr, const FusedArgs *fused = nullptr,
        int accumulate = 0, const float *log_beta = nullptr, bool plan_sized_workspace = false) {
    // with the gate prologue the gate rows are z (checked like log_alpha: non-null, aligned)
    int st = validate(q, k, v, fused ? static_cast<const float *>(fused->z) : log_alpha, B, H, T, dk, dv,
                      grid_h, grid_w, scan_dir, qkv_dtype, out_dtype, out, final_state);
    if (st != GLA_OK) return st;
    if (fused) {
        if (!(fused->tau > 0.f) || !(fused->ln_eps >= 0.f)) return GLA_ERR_SHAPE;
        if (misaligned(fused->r_pre) || misaligned(fused->ln_weight) || misaligned(fused->ln_bias) ||
            misaligned(fused->z_beta))
            return GLA_ERR_ALIGN;
    }
    if (layout != GLA_LAYOUT_BHTD && layout != GLA_LAYOUT_BTHD) return GLA_ERR_SHAPE;
    if (initial_state && misaligned(initial_state)) return GLA_ERR_ALIGN;
    if (log_beta && misaligned(log_beta)) return GLA_ERR_ALIGN;
    // plan_sized_workspace: the buffer is checked against what the launch plan of this call uses (below)
    // instead of the bound over all plans
    if (!workspace || misaligned(workspace) ||
        (!plan_sized_workspace && ws_bytes < workspace_bytes(B, H, T, dk, dv)))
        return GLA_ERR_WORKSPACE;

    Params p{};
    p.log_beta = log_beta;
    p.q = q; p.k = k; p.v = v; p.log_alpha = log_alpha; p.out = out; p.final_state = final_state;
    p.B = B; p.H = H; p.T = T; p.dk = dk; p.dv = dv;
    p.grid_h = grid_h; p.grid_w = grid_w; p.scan_dir = scan_dir;
    p.qkv_dtype = qkv_dtype; p.out_dtype = out_dtype;
    p.initial_state = initial_state;
    if (accumulate && out_dtype != GLA_DT_F32) return GLA_ERR_UNSUPPORTED;
    if (accumulate && (log_beta || (fused && fused->z_beta))) return GLA_ERR_UNSUPPORTED;
    p.accumulate = accumulate;
    if (fused) {
        p.log_alpha = nullptr;
        p.z_gate = fused->z;
        p.inv_tau = 1.f / fused->tau;
        p.r_pre = fused->r_pre;
        p.ln_weight = fused->ln_weight;
        p.ln_bias = fused->ln_bias;
        p.ln_eps = fused->ln_eps;
        p.z_beta = fused->z_beta;
    }
    if (layout == GLA_LAYOUT_BHTD) {
        p.st_k = dk; p.sh_k = (long long)T * dk; p.sb_k = (long long)H * T * dk;
        p.st_v = dv; p.sh_v = (long long)T * dv; p.sb_v = (long long)H * T * dv;
    } else {  // [B,T,H,d]: the heads of one token are neighbours
        p.st_k = H * dk; p.sh_k = dk; p.sb_k = (long long)T * H * dk;
        p.st_v = H * dv; p.sh_v = dv; p.sb_v = (long long)T * H * dv;
    }

    bool use_mfma, use_fast = false;
    st = choose_engine_and_plan(p, workspace, use_mfma, &use_fast);
    if (st != GLA_OK) return st;
    if (plan_sized_workspace && ws_bytes < plan_workspace_bytes((size_t)B * H, (size_t)p.nspans, dk, dv))
        return GLA_ERR_WORKSPACE;
    auto span = [&](SpanMode mode) {
        return use_mfma ? launch_mfma_span(p, mode, stream) : launch_recurrent_span(p, mode, stream);
    };
    auto mark = [&](int i) {
        if (events) (void)hipEventRecord(events->ev[i], stream);
    };

    p.chain_in_output = use_mfma && p.nspans > 1 &&
                        (g_opt_carry == GLA_CARRY_IN_OUTPUT_PASS ||
                         (g_opt_carry == GLA_CARRY_AUTO && p.nspans <= kMaxChainedSpans));

    hipError_t e = hipSuccess;
    mark(0);
    if (p.nspans > 1) {
        e = use_fast ? launch_fast_state(p, stream) : span(kModeState);
        if (e != hipSuccess) return GLA_ERR_HIP;
    }
    mark(1);
    if (p.nspans > 1 && !p.chain_in_output) {
        e = launch_carry(p, stream);
        if (e != hipSuccess) return GLA_ERR_HIP;
    }
    mark(2);
    if (use_fast) {
        // fp16 output pass; the spans whose gates or operands leave its range raise their flags and are
        // recomputed by the bf16 hi/lo pass (work-groups of unflagged spans return at once)
        e = launch_fast_output(p, stream);
        if (e != hipSuccess) return GLA_ERR_HIP;
        if (g_opt_range_fallback) {
            // one work-group per (batch, head) walks the whole sequence from the caller's initial state; those of
            // heads without a raised flag return at once
            Params pf = p;
            pf.fail_spans = p.nspans;
            pf.only_flagged = 1;
            pf.nspans = 1;
            pf.span_len = ((p.T + kChunk - 1) / kChunk) * kChunk;
            pf.chain_in_output = 0;
            e = launch_mfma_span(pf, kModeOutput, stream);
        }
    } else {
        e = span(kModeOutput);
    }
    if (e != hipSuccess) return GLA_ERR_HIP;
    mark(3);
    return GLA_OK;
}

// ---- gla_fwd_static: the workspace of the span plan in a file-scope device array ----
// Host code never uses the array's name as an address: the device address is asked for once per device
// (hipGetSymbolAddress with that device current) and kept; every GPU holds its own copy of the array.
constexpr size_t kStaticScratchBytes = GLA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_static_mutex;
void *g_static_ptr[kMaxDevices] = {};

// bytes the launch plan of a dense [B,H,T,d] bf16 -> fp32 call uses (host arithmetic only)
size_t static_plan_bytes(int B, int H, int T, int dk, int dv) {
    Params p{};
    p.B = B; p.H = H; p.T = T; p.dk = dk; p.dv = dv;
    p.qkv_dtype = GLA_DT_BF16; p.out_dtype = GLA_DT_F32;
    set_dense_bhtd_strides(p);
    bool use_mfma;
    alignas(256) static unsigned char layout_base[256];   // only offsets from it are formed, nothing is accessed
    bool use_fast = false;
    if (choose_engine_and_plan(p, layout_base, use_mfma, &use_fast) != GLA_OK) return ~(size_t)0;
    return plan_workspace_bytes((size_t)B * H, (size_t)p.nspans, dk, dv);
}

}  // namespace
}  // namespace gla

using namespace gla;

extern "C" {

int gla_fwd_static(const void *q, const void *k, const void *v, const float *log_alpha,
                   int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                   float *out, float *final_state, gla_stream_t stream) {
    int st = validate(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                      GLA_DT_BF16, GLA_DT_F32, out, final_state);
    if (st != GLA_OK) return st;
    if (static_plan_bytes(B, H, T, dk, dv) > kStaticScratchBytes) return GLA_ERR_WORKSPACE;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GLA_ERR_HIP;
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_static_mutex);
        if (!g_static_ptr[dev]) {
            void *sym = nullptr;
            if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return GLA_ERR_HIP;
            g_static_ptr[dev] = sym;
        }
        ws = g_static_ptr[dev];
    }
    return run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir, GLA_DT_BF16, GLA_DT_F32,
               out, final_state, ws, kStaticScratchBytes, static_cast<hipStream_t>(stream), nullptr,
               GLA_LAYOUT_BHTD, nullptr, nullptr, 0, nullptr, /*plan_sized_workspace=*/true);
}

int gla_fwd_gates(const void *q, const void *k, const void *v, const float *log_alpha, const float *log_beta,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, int out_dtype, int layout, const float *initial_state,
                  void *out, float *final_state, void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    if (!log_beta) return GLA_ERR_NULL;
    return run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype, out_dtype,
               out, final_state, workspace, workspace_bytes_, static_cast<hipStream_t>(stream), nullptr,
               layout, initial_state, nullptr, 0, log_beta);
}

int gla_fwd_ex(const void *q, const void *k, const void *v, const float *log_alpha,
               int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
               int qkv_dtype, int out_dtype, void *out, float *final_state,
               void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    return run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype, out_dtype,
               out, final_state, workspace, workspace_bytes_, static_cast<hipStream_t>(stream), nullptr);
}

int gla_fwd_layout(const void *q, const void *k, const void *v, const float *log_alpha,
                   int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                   int qkv_dtype, int out_dtype, int layout, const float *initial_state,
                   void *out, float *final_state,
                   void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    return run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype, out_dtype,
               out, final_state, workspace, workspace_bytes_, static_cast<hipStream_t>(stream), nullptr,
               layout, initial_state);
}

int gla_fwd_fused(const void *q, const void *k, const void *v, const void *z_alpha, float tau,
                  const void *r_pre, const float *ln_weight, const float *ln_bias, float ln_eps,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, int out_dtype, void *out, float *final_state,
                  void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    const FusedArgs fused{z_alpha, tau, r_pre, ln_weight, ln_bias, ln_eps, nullptr};
    return run(q, k, v, nullptr, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype, out_dtype,
               out, final_state, workspace, workspace_bytes_, static_cast<hipStream_t>(stream), nullptr,
               GLA_LAYOUT_BHTD, nullptr, &fused);
}

int gla_fwd_fused_gates(const void *q, const void *k, const void *v, const void *z_alpha, const void *z_beta, float tau,
                        const void *r_pre, const float *ln_weight, const float *ln_bias, float ln_eps,
                        int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                        int qkv_dtype, int out_dtype, void *out, float *final_state,
                        void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    if (!z_beta) return GLA_ERR_NULL;
    const FusedArgs fused{z_alpha, tau, r_pre, ln_weight, ln_bias, ln_eps, z_beta};
    return run(q, k, v, nullptr, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype, out_dtype,
               out, final_state, workspace, workspace_bytes_, static_cast<hipStream_t>(stream), nullptr,
               GLA_LAYOUT_BHTD, nullptr, &fused);
}

int gla_srem_dwconv(const void *x, const float *weight, const float *bias, int B, int grid_h, int grid_w, int D,
                    int orient, int x_dtype, int y_dtype, void *y, gla_stream_t stream) {
    if (!x || !weight || !y) return GLA_ERR_NULL;
    if (B <= 0 || grid_h <= 0 || grid_w <= 0 || D <= 0 || orient < 0 || orient > 3) return GLA_ERR_SHAPE;
    if ((x_dtype != GLA_DT_F32 && x_dtype != GLA_DT_BF16) || (y_dtype != GLA_DT_F32 && y_dtype != GLA_DT_BF16))
        return GLA_ERR_SHAPE;
    // 32-bit byte offsets inside one batch element, 31-bit strip and work-group counts
    if ((long long)grid_h * grid_w * D * 4 >= (1LL << 32) || (long long)B * grid_h * grid_w >= (1LL << 31))
        return GLA_ERR_UNSUPPORTED;
    if (x == y) return GLA_ERR_SHAPE;   // neighbours are read after a token is written: not in place
    if (misaligned(x) || misaligned(y) || misaligned(weight) || misaligned(bias)) return GLA_ERR_ALIGN;
    if (launch_srem_dwconv(x, weight, bias, y, B, grid_h, grid_w, D, orient, x_dtype, y_dtype,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
        return GLA_ERR_HIP;
    return GLA_OK;
}

int gla_fwd_multi(const void *q, const void *k, const void *v, const float *log_alpha,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, unsigned scan_mask,
                  int qkv_dtype, float *out, void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    if (scan_mask == 0u || scan_mask > 15u) return GLA_ERR_SHAPE;
    int first = 1;
    for (int d = 0; d < 4; ++d) {
        if (!(scan_mask & (1u << d))) continue;
        // the first scan order writes `out`, the others add to it; the workspace is reused in stream order
        const int st = run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, d, qkv_dtype, GLA_DT_F32, out,
                           nullptr, workspace, workspace_bytes_, static_cast<hipStream_t>(stream), nullptr,
                           GLA_LAYOUT_BHTD, nullptr, nullptr, first ? 0 : 1);
        if (st != GLA_OK) return st;   // argument errors show on the first pass, before any launch
        first = 0;
    }
    return GLA_OK;
}

int gla_bwd(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
            int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
            float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
            void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    return run_bwd(q, k, v, log_alpha, d_out, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype,
                   dq, dk_grad, dv_grad, dlog_alpha, workspace, workspace_bytes_, static_cast<hipStream_t>(stream));
}

size_t gla_bwd_gates_workspace_bytes(int B, int H, int T, int dk, int dv, int qkv_dtype) {
    (void)qkv_dtype;
    if (B <= 0 || H <= 0 || T <= 0 || dk <= 0 || dv <= 0) return 0;
    return workspace_bytes(B, H, T, dk, dv) + bwd_totals_bytes(B, H, T, dk > dv ? dk : dv) +
           bwd_gates_out_bytes(B, H, T, dv);
}

int gla_bwd_gates(const void *q, const void *k, const void *v, const float *log_alpha, const float *log_beta,
                  const void *d_out, const float *out_fwd, int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha, float *dlog_beta,
                  void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    return run_bwd_gates(q, k, v, log_alpha, log_beta, d_out, out_fwd, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype,
                         dq, dk_grad, dv_grad, dlog_alpha, dlog_beta, workspace, workspace_bytes_,
                         static_cast<hipStream_t>(stream));
}

size_t gla_bwd_workspace_bytes(int B, int H, int T, int dk, int dv, int qkv_dtype) {
    if (B <= 0 || H <= 0 || T <= 0 || dk <= 0 || dv <= 0) return 0;
    if (qkv_dtype != GLA_DT_F32 && qkv_dtype != GLA_DT_BF16) return 0;
    return workspace_bytes(B, H, T, dk, dv) + bwd_totals_bytes(B, H, T, dk);
}

int gla_fwd(const void *q, const void *k, const void *v, const float *log_alpha,
            int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
            float *out, float *final_state, gla_stream_t stream) {
    int st = validate(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir,
                      GLA_DT_BF16, GLA_DT_F32, out, final_state);
    if (st != GLA_OK) return st;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GLA_ERR_HIP;
    const size_t need = workspace_bytes(B, H, T, dk, dv);
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        Scratch &s = g_scratch[dev];
        if (s.bytes < need) {
            if (s.ptr) {
                // earlier calls may still be reading the old buffer
                if (hipDeviceSynchronize() != hipSuccess) return GLA_ERR_HIP;
                (void)hipFree(s.ptr);
                s.ptr = nullptr;
                s.bytes = 0;
            }
            void *fresh = nullptr;
            if (hipMalloc(&fresh, need) != hipSuccess) return GLA_ERR_HIP;
            s.ptr = fresh;
            s.bytes = need;
        }
        ws = s.ptr;
    }
    return run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir, GLA_DT_BF16, GLA_DT_F32,
               out, final_state, ws, need, static_cast<hipStream_t>(stream), nullptr);
}

int gla_bwd_reuse(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
                  const void *fwd_workspace, size_t fwd_workspace_bytes,
                  float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
                  void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    if (!fwd_workspace) return GLA_ERR_NULL;
    return run_bwd(q, k, v, log_alpha, d_out, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype,
                   dq, dk_grad, dv_grad, dlog_alpha, workspace, workspace_bytes_, static_cast<hipStream_t>(stream),
                   fwd_workspace, fwd_workspace_bytes);
}

int gla_bwd_layout(const void *q, const void *k, const void *v, const float *log_alpha, const void *d_out,
                   int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir, int qkv_dtype,
                   int layout, const void *fwd_workspace, size_t fwd_workspace_bytes,
                   float *dq, float *dk_grad, float *dv_grad, float *dlog_alpha,
                   void *workspace, size_t workspace_bytes_, gla_stream_t stream) {
    return run_bwd(q, k, v, log_alpha, d_out, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype,
                   dq, dk_grad, dv_grad, dlog_alpha, workspace, workspace_bytes_, static_cast<hipStream_t>(stream),
                   fwd_workspace, fwd_workspace_bytes, layout);
}

size_t gla_fwd_workspace_bytes(int B, int H, int T, int dk, int dv, int qkv_dtype) {
    if (B <= 0 || H <= 0 || T <= 0 || dk <= 0 || dv <= 0) return 0;
    if (qkv_dtype != GLA_DT_F32 && qkv_dtype != GLA_DT_BF16) return 0;
    return workspace_bytes(B, H, T, dk, dv);
}

namespace {
// register-resident MFMA loop: eight independent accumulator chains per wave, operands never change
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, float *sink) {
    typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
    typedef __attribute__((ext_vector_type(4))) float f32x4_t;
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
    const uint32_t seed = 0x3f803f80u + (threadIdx.x & 3);   // bf16 pairs near 1.0
    const bf16x8_t a = __builtin_bit_cast(bf16x8_t, u32x4_t{seed, seed, seed, seed});
    const bf16x8_t b = __builtin_bit_cast(bf16x8_t, u32x4_t{seed ^ 1u, seed, seed ^ 1u, seed});
    f32x4_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (s == 12345.678f) sink[threadIdx.x] = s;   // keeps the loop alive; never true for these operands
}
}  // namespace

int gla_calibrate_mfma(double *tflops, gla_stream_t stream) {
    if (!tflops) return GLA_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *sink = nullptr;
    if (hipMalloc(&sink, 4096) != hipSuccess) return GLA_ERR_HIP;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int status = GLA_OK;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) status = GLA_ERR_HIP;
    constexpr int kGroups = 256 * 8, kIters = 4096;     // 8 work-groups of 4 waves per compute unit
    if (status == GLA_OK) {
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(kGroups), dim3(256), 0, s, 64, sink);   // warm-up
        (void)hipEventRecord(e0, s);
        hipLaunchKernelGGL(mfma_rate_kernel, dim3(kGroups), dim3(256), 0, s, kIters, sink);
        (void)hipEventRecord(e1, s);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(s) != hipSuccess) status = GLA_ERR_HIP;
    }
    if (status == GLA_OK) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.f)) {
            status = GLA_ERR_HIP;
        } else {
            const double flops = (double)kGroups * 4 /*waves*/ * kIters * 8 /*chains*/ * (2.0 * 16 * 16 * 32);
            *tflops = flops / (ms * 1e-3) / 1e12;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(sink);
    return status;
}

int gla_fwd_timed(const void *q, const void *k, const void *v, const float *log_alpha,
                  int B, int H, int T, int dk, int dv, int grid_h, int grid_w, int scan_dir,
                  int qkv_dtype, int out_dtype, void *out, float *final_state,
                  void *workspace, size_t workspace_bytes_, gla_stream_t stream,
                  int iters, float *phase_ms) {
    if (!phase_ms) return GLA_ERR_NULL;
    if (iters <= 0 || iters > 4096) return GLA_ERR_SHAPE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<PhaseEvents> evs((size_t)iters);
    int created = 0;
    int status = GLA_OK;
    for (int i = 0; i < iters && status == GLA_OK; ++i) {
        for (int j = 0; j < 4; ++j) {
            if (hipEventCreate(&evs[i].ev[j]) != hipSuccess) { status = GLA_ERR_HIP; break; }
            ++created;
        }
    }
    int done = 0;
    for (int i = 0; i < iters && status == GLA_OK; ++i) {
        status = run(q, k, v, log_alpha, B, H, T, dk, dv, grid_h, grid_w, scan_dir, qkv_dtype, out_dtype,
                     out, final_state, workspace, workspace_bytes_, s, &evs[i]);
        if (status == GLA_OK) ++done;
    }
    if (hipStreamSynchronize(s) != hipSuccess && status == GLA_OK) status = GLA_ERR_HIP;
    double sum[4] = {0, 0, 0, 0};
    if (status == GLA_OK) {
        for (int i = 0; i < done; ++i) {
            float ms = 0.f;
            for (int j = 0; j < 3; ++j) {
                if (hipEventElapsedTime(&ms, evs[i].ev[j], evs[i].ev[j + 1]) != hipSuccess) status = GLA_ERR_HIP;
                sum[j] += ms;
            }
            if (hipEventElapsedTime(&ms, evs[i].ev[0], evs[i].ev[3]) != hipSuccess) status = GLA_ERR_HIP;
            sum[3] += ms;
        }
    }
    for (int n = 0; n < created; ++n) (void)hipEventDestroy(evs[n / 4].ev[n % 4]);
    if (status == GLA_OK)
        for (int j = 0; j < 4; ++j) phase_ms[j] = (float)(sum[j] / done);
    return status;
}

int gla_set_option(int option, int value) {
    switch (option) {
    case GLA_OPT_CHUNKS_PER_SPAN:
        if (value < 0 || value > 65536) return GLA_ERR_SHAPE;
        g_opt_chunks_per_span = value;
        return GLA_OK;
    case GLA_OPT_ENGINE:
        if (value < GLA_ENGINE_AUTO || value > GLA_ENGINE_MFMA_FP16) return GLA_ERR_SHAPE;
        g_opt_engine = value;
        return GLA_OK;
    case GLA_OPT_CARRY:
        if (value < GLA_CARRY_AUTO || value > GLA_CARRY_IN_OUTPUT_PASS) return GLA_ERR_SHAPE;
        g_opt_carry = value;
        return GLA_OK;
    case GLA_OPT_BWD_SPLIT:
        if (value < 0 || value > 1) return GLA_ERR_SHAPE;
        g_opt_bwd_split = value;
        return GLA_OK;
    case GLA_OPT_RANGE_FALLBACK:
        if (value < 0 || value > 1) return GLA_ERR_SHAPE;
        g_opt_range_fallback = value;
        return GLA_OK;
    default:
        return GLA_ERR_SHAPE;
    }
}

int gla_get_option(int option) {
    switch (option) {
    case GLA_OPT_CHUNKS_PER_SPAN: return g_opt_chunks_per_span;
    case GLA_OPT_ENGINE: return g_opt_engine;
    case GLA_OPT_CARRY: return g_opt_carry;
    case GLA_OPT_BWD_SPLIT: return g_opt_bwd_split;
    case GLA_OPT_RANGE_FALLBACK: return g_opt_range_fallback;
    default: return -1;
    }
}

int gla_block_scan_dir(int block, int schedule) {
    // the order entering block l is the composition of the operators after blocks 1 .. l-1; both schedules walk
    // the four orders with period four
    static const int kBlockProcess[4] = {GLA_SCAN_ROW_FWD, GLA_SCAN_ROW_REV, GLA_SCAN_COL_REV, GLA_SCAN_COL_FWD};
    static const int kBlockScan[4] = {GLA_SCAN_ROW_FWD, GLA_SCAN_COL_FWD, GLA_SCAN_COL_REV, GLA_SCAN_ROW_REV};
    if (block < 1) return -1;
    if (schedule == GLA_SCHEDULE_BLOCK_PROCESS) return kBlockProcess[(block - 1) & 3];
    if (schedule == GLA_SCHEDULE_BLOCK_SCAN) return kBlockScan[(block - 1) & 3];
    return -1;
}

const char *gla_status_string(int status) {
    switch (status) {
    case GLA_OK: return "ok";
    case GLA_ERR_NULL: return "a required pointer is NULL";
    case GLA_ERR_SHAPE: return "invalid size, grid, enum value or option";
    case GLA_ERR_UNSUPPORTED: return "head size, element type or engine not supported";
    case GLA_ERR_ALIGN: return "a base pointer is not 16-byte aligned";
    case GLA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GLA_ERR_HIP: return "the HIP runtime reported an error";
    default: return "unknown status";
    }
}

int gla_version(void) { return kVersion; }

}  // extern "C"
