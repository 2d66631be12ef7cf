// Phase 2 of the span plan: chain the spans of each (batch, head).
//
// Every span r has produced, from a zero state, its local state U_r and
// log Gamma_r (the summed log_alpha of its tokens).  Because the recurrence of
// Sec. 3.1 Eq. (attn_gla) is linear in S, the state entering span r+1 is
//     S_start(r+1) = diag(Gamma_r) S_start(r) + U_r ,   S_start(0) = the caller's initial state (or 0)
// (with the value-side gate of Eq. (gate_gla_2), element (c, n) decays by Gamma_r[c] times the product of beta[n]
// over the span, whose logarithm phase 1 left in ws_lgam_b).
// Each of the dk*dv state elements is an independent scalar recurrence over the
// spans; the buffer is rewritten in place (U_r becomes S_start(r)) and the value
// after the last span is the final state.
//
// The kernel is bound by the latency of its loads, so the spans of one element
// are cut into kGroups runs handled by kGroups threads: each thread loads its
// whole run at once, composes it (product of the Gammas, state from zero),
// the runs are chained through LDS, and each thread then replays its run from
// its true start state.
#include "gla_common.h"

namespace gla {
namespace {

constexpr int kElems = 64;    // state elements per work-group (one wave wide: coalesced rows)
constexpr int kGroups = 4;    // runs of spans per element
constexpr int kRun = 16;      // spans per run and pass
constexpr int kCarryThreads = kElems * kGroups;

__global__ __launch_bounds__(kCarryThreads) void carry_kernel(Params p) {
    __shared__ float s_gam[kGroups][kElems];
    __shared__ float s_u[kGroups][kElems];

    // (batch, head) on grid.x, whose limit is 2^31 - 1; the blocks of elements (at most 128) on grid.y
    const int bh = blockIdx.x;
    const int el = threadIdx.x % kElems;
    const int grp = threadIdx.x / kElems;
    const int ne = p.dk * p.dv;
    const int e = min((int)blockIdx.y * kElems + el, ne - 1);  // threads past the end repeat the last element
    const bool writer = (int)blockIdx.y * kElems + el < ne;
    const int c = e / p.dv;
    float *st = p.ws_state + (size_t)bh * p.nspans * ne + e;
    const float *lg = p.ws_lgam + (size_t)bh * p.nspans * p.dk + c;
    const float *lgb = two_sided(p) ? p.ws_lgam_b + (size_t)bh * p.nspans * p.dv + (e - c * p.dv) : nullptr;

    // state entering the current pass of kGroups * kRun spans; the first pass starts from the caller's state
    float carry = p.initial_state ? p.initial_state[(size_t)bh * ne + e] : 0.f;
    for (int r0 = 0; r0 < p.nspans; r0 += kGroups * kRun) {
        const int first = r0 + grp * kRun;
        float u[kRun], gam[kRun];
#pragma unroll
        for (int i = 0; i < kRun; ++i) {
            const int r = first + i;
            const bool ok = r < p.nspans;
            u[i] = ok ? st[(size_t)r * ne] : 0.f;
            gam[i] = ok ? expf(lg[(size_t)r * p.dk] + (lgb != nullptr ? lgb[(size_t)r * p.dv] : 0.f)) : 1.f;
        }
        // the run composed from a zero state
        float gprod = 1.f, ulocal = 0.f;
#pragma unroll
        for (int i = 0; i < kRun; ++i) {
            ulocal = fmaf(gam[i], ulocal, u[i]);
            gprod *= gam[i];
        }
        s_gam[grp][el] = gprod;
        s_u[grp][el] = ulocal;
        __syncthreads();
        // state entering this thread's run, and the state after the whole pass
        float s = carry, pass_end = carry;
#pragma unroll
        for (int q = 0; q < kGroups; ++q) {
            const float gq = s_gam[q][el], uq = s_u[q][el];
            if (q < grp) s = fmaf(gq, s, uq);
            pass_end = fmaf(gq, pass_end, uq);
        }
        carry = pass_end;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kRun; ++i) {
            const int r = first + i;
            if (r < p.nspans) {
                if (writer) st[(size_t)r * ne] = s;
                s = fmaf(gam[i], s, u[i]);
            }
        }
    }
    if (p.final_state != nullptr && writer && grp == 0) p.final_state[(size_t)bh * ne + e] = carry;
}

}  // namespace

hipError_t launch_carry(const Params &p, hipStream_t stream) {
    dim3 grid((unsigned)(p.B * p.H), (unsigned)((p.dk * p.dv + kElems - 1) / kElems));
    hipLaunchKernelGGL(carry_kernel, grid, dim3(kCarryThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace gla
