// Kernels that exist only for the backward pass of the GLA recurrence
// (DiG paper, Sec. 3.1 Eq. (attn_gla) rows 1-3 with beta = 1, differentiated).
//
// With S_s the state after scan step s and G_s = dL/dS_s (which obeys the same kind
// of recurrence walked backwards, G_s = q_s^T dO_s + diag(alpha_{s+1}) G_{s+1}):
//     dq_s[c] = sum_n S_s[c,n] dO_s[n]        dk_s[c] = sum_n G_s[c,n] v_s[n]
//     dv_s    = k_s G_s                        (a forward pass with q, k, v := k, q, dO)
//     dlog_alpha_s = sum_{s' >= s} (q_s' * dq_s' - k_s' * dk_s')      (reverse cumulative sum)
// dq and dk read the state along its value axis, which the forward engines (they read
// it along the key axis) do not do.  For bf16 inputs with head sizes the MFMA engine
// takes, that read runs in chunk form on the MFMA units (gla_mfma_bwd.hip).  The
// row_read_kernel of this file covers everything else (fp32 inputs, odd head sizes):
// it walks one span token by token in fp32 with the state rows in registers, thread c
// of a wave owning row c of half of the value columns.  The state entering the span
// comes from the span plan of the forward pass (span-state pass + carry kernel).
// The two kernels of the gate gradient (the reverse cumulative sum) serve both paths.
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
// columns, as fp32; fetched one tile ahead), then walked token by token: the rows v_s and w_s are the same for all lanes and are read
// as broadcasts, 16 bytes of each per ds_read_b128 pair.
// BETA: the state element (c, n) decays by alpha[c] * beta[n] (two-sided gate, p.log_beta).
template <typename TIn, bool BETA>
__global__ __launch_bounds__(kRowWaves * 64) void row_read_kernel(Params p, const void *w, float *r) {
    __shared__ __attribute__((aligned(16))) float s_bq[BETA ? kTile : 1][BETA ? kMaxDv / 4 : 1][4];   // beta per column
    __shared__ float s_a[kTile][kMaxDk];
    __shared__ float s_k[kTile][kMaxDk];
    __shared__ __attribute__((aligned(16))) float s_vw[kTile][kMaxDv / 4][8];   // [token][column quad][v0..v3, w0..w3]
    __shared__ float s_r[kRowWaves][kTile][kMaxDk];
    __shared__ int s_tok[kTile];

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

    // The rows of a tile are fetched into registers one tile ahead (the loads of tile t + 1 are in flight while
    // tile t is walked) and reach LDS, gates exponentiated, at the start of their own round.  Slots: the key side
    // has token rows half, half + 2, ... of channel c; the value side has (token row, column quad) pairs
    // tid, tid + 128, ... as 8- or 16-byte pieces when the row pitch allows it, element by element otherwise.
    constexpr int kKSlots = kTile / kRowWaves;
    constexpr int kVSlots = kTile * (kMaxDv / 4) / (kRowWaves * 64);
    const bool vec = (dv % 4 == 0) && (st_v % 4 == 0) && (base_v % 4 == 0);   // uniform
    float ra[kKSlots], rk[kKSlots];
    f32x4 rv[kVSlots], rw[kVSlots], rb[kVSlots];
    auto fetch = [&](int t0) {
#pragma unroll
        for (int m = 0; m < kKSlots; ++m) {
            const int j = half + kRowWaves * m;
            const bool valid = t0 + j < s_end;
            const int sc = min(t0 + j, s_end - 1);
            ra[m] = 0.f;      // a step past the span leaves the state alone: alpha = 1, k = 0
            rk[m] = 0.f;
            if (valid && row_active) {
                const int n = scan_token(p.scan_dir, sc, T, p.grid_h, p.grid_w);
                const int ng = scan_token(p.scan_dir, max(sc - p.gate_shift, 0), T, p.grid_h, p.grid_w);
                ra[m] = p.log_alpha[base_k + (size_t)ng * st_k + c];
                rk[m] = load_elem<TIn>(p.k, base_k + (size_t)n * st_k + c);
            }
        }
#pragma unroll
        for (int m = 0; m < kVSlots; ++m) {
            const int idx = tid + kRowWaves * 64 * m;
            const int j = idx / nquads, col = 4 * (idx - j * nquads);
            rv[m] = rw[m] = rb[m] = f32x4{0.f, 0.f, 0.f, 0.f};     // zero past dv and past the span (beta = 1)
            if (j < kTile && t0 + j < s_end) {
                const int sc = t0 + j;
                const int n = scan_token(p.scan_dir, sc, T, p.grid_h, p.grid_w);
                const size_t e = base_v + (size_t)n * st_v + col;
                size_t eg = e;
                if (BETA) eg = base_v + (size_t)scan_token(p.scan_dir, max(sc - p.gate_shift, 0), T, p.grid_h, p.grid_w) * st_v + col;
                if (vec) {
                    if constexpr (sizeof(TIn) == 4) {
                        rv[m] = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(p.v) + e);
                        rw[m] = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(w) + e);
                    } else {
                        const uint2 tv = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(p.v) + e);
                        const uint2 tw = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(w) + e);
                        rv[m] = f32x4{__builtin_bit_cast(float, tv.x << 16), __builtin_bit_cast(float, tv.x & 0xffff0000u),
                                      __builtin_bit_cast(float, tv.y << 16), __builtin_bit_cast(float, tv.y & 0xffff0000u)};
                        rw[m] = f32x4{__builtin_bit_cast(float, tw.x << 16), __builtin_bit_cast(float, tw.x & 0xffff0000u),
                                      __builtin_bit_cast(float, tw.y << 16), __builtin_bit_cast(float, tw.y & 0xffff0000u)};
                    }
                    if constexpr (BETA) rb[m] = *reinterpret_cast<const f32x4 *>(p.log_beta + eg);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (col + i < dv) {
                            rv[m][i] = load_elem<TIn>(p.v, e + i);
                            rw[m][i] = load_elem<TIn>(w, e + i);
                            if constexpr (BETA) rb[m][i] = p.log_beta[eg + i];
                        }
                    }
                }
            }
        }
    };
    fetch(s_begin);

    for (int t0 = s_begin; t0 < s_end; t0 += kTile) {
        __syncthreads();
        if (tid < kTile)
            s_tok[tid] = (t0 + tid < s_end) ? scan_token(p.scan_dir, t0 + tid, T, p.grid_h, p.grid_w) : -1;
        if (row_active) {
#pragma unroll
            for (int m = 0; m < kKSlots; ++m) {
                s_a[half + kRowWaves * m][c] = expf(ra[m]);
                s_k[half + kRowWaves * m][c] = rk[m];
            }
        }
#pragma unroll
        for (int m = 0; m < kVSlots; ++m) {
            const int idx = tid + kRowWaves * 64 * m;
            const int j = idx / nquads, qd = idx - j * nquads;
            if (j < kTile) {
                *reinterpret_cast<f32x4 *>(&s_vw[j][qd][0]) = rv[m];
                *reinterpret_cast<f32x4 *>(&s_vw[j][qd][4]) = rw[m];
                if constexpr (BETA)
                    *reinterpret_cast<f32x4 *>(&s_bq[j][qd][0]) =
                        f32x4{expf(rb[m][0]), expf(rb[m][1]), expf(rb[m][2]), expf(rb[m][3])};
            }
        }
        if (t0 + kTile < s_end) fetch(t0 + kTile);
        __syncthreads();
        for (int j = 0; j < kTile; ++j) {
            const float a = s_a[j][c], kc = s_k[j][c];
            float acc = 0.f;
#pragma unroll
            for (int qd = 0; qd < kColsPerWave / 4; ++qd) {
                if (quad_lo + qd < quad_hi) {   // uniform
                    const f32x4 vq = *reinterpret_cast<const f32x4 *>(&s_vw[j][quad_lo + qd][0]);
                    const f32x4 wq = *reinterpret_cast<const f32x4 *>(&s_vw[j][quad_lo + qd][4]);
                    f32x4 bq = f32x4{1.f, 1.f, 1.f, 1.f};
                    if constexpr (BETA) bq = *reinterpret_cast<const f32x4 *>(&s_bq[j][quad_lo + qd][0]);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        S[4 * qd + i] = fmaf(BETA ? a * bq[i] : a, S[4 * qd + i], kc * vq[i]);
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
// Spans of kDgSpan scan steps, one work-group each.  Kernel 1 stages the span's terms in LDS channel-major
// (rows read from HBM in pieces of PW channels, neighbouring lanes neighbouring pieces), scans every channel
// with lane = scan step counted from the span's last step backwards, and writes the sums at the canonical
// token index together with the span's total.  Kernel 2 adds to every span the totals of the spans after it.
constexpr int kDgSpan = 256;       // scan steps per work-group
constexpr int kDgThreads = 256;    // one lane per scan step in the scan stage
constexpr int kDgBatch = 3;        // pieces per thread whose loads are in flight together
constexpr int kDgRow = kDgSpan + 1;  // floats per channel row in LDS

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

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// PW consecutive elements starting at element index e, as floats (PW = 4: e is a multiple of 4 and 16-byte
// aligned in fp32, 8-byte aligned in bf16)
template <typename TIn, int PW>
__device__ inline void load_piece(const void *base, size_t e, float (&x)[PW]) {
    if constexpr (PW == 1) {
        x[0] = load_elem<TIn>(base, e);
    } else if constexpr (sizeof(TIn) == 4) {
        const f32x4 t = *reinterpret_cast<const f32x4 *>(static_cast<const float *>(base) + e);
#pragma unroll
        for (int i = 0; i < 4; ++i) x[i] = t[i];
    } else {
        const u32x2 t = *reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(base) + e);
        x[0] = __builtin_bit_cast(float, t[0] << 16);
        x[1] = __builtin_bit_cast(float, t[0] & 0xffff0000u);
        x[2] = __builtin_bit_cast(float, t[1] << 16);
        x[3] = __builtin_bit_cast(float, t[1] & 0xffff0000u);
    }
}
template <int PW>
__device__ inline void store_piece(float *dst, const float (&x)[PW]) {
    if constexpr (PW == 1) dst[0] = x[0];
    else *reinterpret_cast<f32x4 *>(dst) = f32x4{x[0], x[1], x[2], x[3]};
}

// Walks the (row, piece) pairs tid, tid + kDgThreads, ... of a [kDgSpan][pcs] tile without divisions.
struct PieceWalk {
    int j, pc, dj, dpc, pcs;
    __device__ PieceWalk(int tid, int pcs_) : pcs(pcs_) {
        j = tid / pcs;
        pc = tid - j * pcs;
        dj = kDgThreads / pcs;
        dpc = kDgThreads - dj * pcs;
    }
    __device__ void next() {
        j += dj;
        pc += dpc;
        if (pc >= pcs) {
            pc -= pcs;
            ++j;
        }
    }
};

// Row j of the tile is scan step (span end - 1 - j): prefix sums over j are suffix sums over the scan.
template <typename TIn, int PW>
__global__ __launch_bounds__(kDgThreads) void dg_local_kernel(Params p, const float *dq, const float *dk_grad,
                                                             float *dg, float *totals, int ndg) {
    extern __shared__ float s_dyn[];
    const int dk = p.dk, T = p.T;
    float *s_x = s_dyn;                                   // [dk][kDgRow]
    float *s_wave = s_dyn + dk * kDgRow;                  // [4][dk] sums of the waves, then their exclusive prefix
    int *s_tok = reinterpret_cast<int *>(s_wave + 4 * dk);  // [kDgSpan]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int bh = blockIdx.x / ndg, sp = blockIdx.x - bh * ndg;
    const size_t base_k = slab_k(p, bh), st_k = (size_t)p.st_k;
    const int s_last = min(T, (sp + 1) * kDgSpan) - 1;
    const int nrows = s_last - sp * kDgSpan + 1;          // scan steps in this span (>= 1)
    s_tok[tid] = scan_token(p.scan_dir, max(s_last - tid, sp * kDgSpan), T, p.grid_h, p.grid_w);
    __syncthreads();

    const int pcs = dk / PW, npieces = kDgSpan * pcs;
    {
        PieceWalk wk(tid, pcs);
        for (int idx0 = tid; idx0 < npieces; idx0 += kDgThreads * kDgBatch) {
            float x[kDgBatch][PW];
            int jj[kDgBatch], cc[kDgBatch];
#pragma unroll
            for (int b = 0; b < kDgBatch; ++b) {   // rows past the span or the tile repeat a valid row
                jj[b] = wk.j;
                cc[b] = PW * wk.pc;
                const size_t e = base_k + (size_t)s_tok[min(wk.j, kDgSpan - 1)] * st_k + cc[b];
                float xq[PW], xk[PW], xdq[PW], xdk[PW];
                load_piece<TIn, PW>(p.q, e, xq);
                load_piece<TIn, PW>(p.k, e, xk);
                load_piece<float, PW>(dq, e, xdq);
                load_piece<float, PW>(dk_grad, e, xdk);
#pragma unroll
                for (int i = 0; i < PW; ++i) x[b][i] = xq[i] * xdq[i] - xk[i] * xdk[i];
                wk.next();
            }
#pragma unroll
            for (int b = 0; b < kDgBatch; ++b) {
                if (jj[b] < kDgSpan) {
#pragma unroll
                    for (int i = 0; i < PW; ++i) s_x[(cc[b] + i) * kDgRow + jj[b]] = jj[b] < nrows ? x[b][i] : 0.f;
                }
            }
        }
    }
    __syncthreads();
    for (int c = 0; c < dk; ++c) {
        const float x = wave_inclusive_scan(s_x[c * kDgRow + tid]);
        s_x[c * kDgRow + tid] = x;
        if (lane == 63) s_wave[wv * dk + c] = x;
    }
    __syncthreads();
    if (tid < dk) {   // what the waves holding later scan steps add to a wave; the sum of all is the span's total
        float run = 0.f;
#pragma unroll
        for (int u = 0; u < kDgThreads / 64; ++u) {
            const float t = s_wave[u * dk + tid];
            s_wave[u * dk + tid] = run;
            run += t;
        }
        totals[((size_t)bh * ndg + sp) * dk + tid] = run;
    }
    __syncthreads();
    {
        PieceWalk wk(tid, pcs);
        for (int idx = tid; idx < npieces; idx += kDgThreads) {
            const int j = wk.j, c0 = PW * wk.pc;
            if (j < nrows) {
                float x[PW];
#pragma unroll
                for (int i = 0; i < PW; ++i) x[i] = s_x[(c0 + i) * kDgRow + j] + s_wave[(j >> 6) * dk + c0 + i];
                store_piece<PW>(dg + base_k + (size_t)s_tok[j] * st_k + c0, x);
            }
            wk.next();
        }
    }
}

template <int PW>
__global__ __launch_bounds__(kDgThreads) void dg_offset_kernel(Params p, float *dg, const float *totals, int ndg) {
    __shared__ float s_off[kMaxDv];   // (the value-side gate gradient runs this kernel over dv columns)
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
    const int nrows = min(T, (sp + 1) * kDgSpan) - sp * kDgSpan;
    s_tok[tid] = scan_token(p.scan_dir, min(sp * kDgSpan + tid, T - 1), T, p.grid_h, p.grid_w);
    __syncthreads();
    const size_t base_k = slab_k(p, bh), st_k = (size_t)p.st_k;
    const int pcs = dk / PW, npieces = kDgSpan * pcs;
    PieceWalk wk(tid, pcs);
    for (int idx = tid; idx < npieces; idx += kDgThreads) {
        const int j = wk.j, c0 = PW * wk.pc;
        if (j < nrows) {
            float *dst = dg + base_k + (size_t)s_tok[j] * st_k + c0;
            float x[PW];
            load_piece<float, PW>(dst, 0, x);
#pragma unroll
            for (int i = 0; i < PW; ++i) x[i] += s_off[c0 + i];
            store_piece<PW>(dst, x);
        }
        wk.next();
    }
}

constexpr size_t kDgLdsMax = ((size_t)kMaxDv * kDgRow + 4 * kMaxDv + kDgSpan) * 4;   // up to dv columns (log_beta)

template <typename TIn, int PW>
hipError_t launch_dg(const Params &p, const float *dq, const float *dk_grad, float *dg, float *totals, int ndg,
                     hipStream_t stream) {
    auto kernel = dg_local_kernel<TIn, PW>;
    static std::atomic<bool> configured[kMaxDevices] = {};  // per instantiation and device
    {
        hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), (int)kDgLdsMax, configured);
        if (e != hipSuccess) return e;
    }
    const size_t lds = ((size_t)p.dk * kDgRow + 4 * p.dk + kDgSpan) * 4;
    dim3 grid((unsigned)(p.B * p.H * ndg)), block(kDgThreads);
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, p, dq, dk_grad, dg, totals, ndg);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (ndg > 1) hipLaunchKernelGGL(dg_offset_kernel<PW>, grid, block, 0, stream, p, dg, totals, ndg);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_row_read(const Params &p, const void *w, float *r, hipStream_t stream) {
    dim3 grid((unsigned)(p.B * p.H * p.nspans)), block(kRowWaves * 64);
    const bool bf16 = p.qkv_dtype == GLA_DT_BF16;
    if (p.log_beta != nullptr) {
        if (bf16) hipLaunchKernelGGL((row_read_kernel<uint16_t, true>), grid, block, 0, stream, p, w, r);
        else hipLaunchKernelGGL((row_read_kernel<float, true>), grid, block, 0, stream, p, w, r);
    } else {
        if (bf16) hipLaunchKernelGGL((row_read_kernel<uint16_t, false>), grid, block, 0, stream, p, w, r);
        else hipLaunchKernelGGL((row_read_kernel<float, false>), grid, block, 0, stream, p, w, r);
    }
    return hipGetLastError();
}

int dg_spans(int T) { return (T + kDgSpan - 1) / kDgSpan; }

hipError_t launch_dlog_alpha(const Params &p, const float *dq, const float *dk_grad, float *dg, float *totals,
                             hipStream_t stream) {
    const int ndg = dg_spans(p.T);
    const bool bf16 = p.qkv_dtype == GLA_DT_BF16;
    // rows in 4-channel pieces (16-byte fp32 accesses) when the channel count and the row pitch allow it
    if (p.dk % 4 == 0 && p.st_k % 4 == 0)
        return bf16 ? launch_dg<uint16_t, 4>(p, dq, dk_grad, dg, totals, ndg, stream)
                    : launch_dg<float, 4>(p, dq, dk_grad, dg, totals, ndg, stream);
    return bf16 ? launch_dg<uint16_t, 1>(p, dq, dk_grad, dg, totals, ndg, stream)
                : launch_dg<float, 1>(p, dq, dk_grad, dg, totals, ndg, stream);
}

}  // namespace gla
