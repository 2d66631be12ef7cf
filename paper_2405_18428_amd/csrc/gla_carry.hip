// Phase 2 of the span plan: chain the spans of each (batch, head).
//
// Every span r has produced, from a zero state, its local state U_r and
// log Gamma_r (the summed log_alpha of its tokens).  Because the recurrence of
// Sec. 3.1 Eq. (attn_gla) is linear in S, the state entering span r+1 is
//     S_start(r+1) = diag(Gamma_r) S_start(r) + U_r ,   S_start(0) = 0.
// Each of the dk*dv state elements is an independent scalar recurrence over the
// spans, so one thread carries one element; the buffer is rewritten in place
// (U_r becomes S_start(r)) and the value after the last span is the final state.
#include "gla_common.h"

namespace gla {
namespace {

constexpr int kCarryThreads = 256;

constexpr int kBatch = 32;  // spans whose loads are in flight together

__global__ __launch_bounds__(kCarryThreads) void carry_kernel(Params p) {
    const int bh = blockIdx.y;
    const int e = blockIdx.x * kCarryThreads + threadIdx.x;
    const int ne = p.dk * p.dv;
    if (e >= ne) return;
    const int c = e / p.dv;
    float *st = p.ws_state + (size_t)bh * p.nspans * ne + e;
    const float *lg = p.ws_lgam + (size_t)bh * p.nspans * p.dk + c;
    float s = 0.f;
    for (int r0 = 0; r0 < p.nspans; r0 += kBatch) {
        // all loads of a batch are issued before the first dependent multiply-add
        float u[kBatch], gl[kBatch];
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int r = min(r0 + i, p.nspans - 1);
            u[i] = st[(size_t)r * ne];
            gl[i] = lg[(size_t)r * p.dk];
        }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            if (r0 + i < p.nspans) {
                st[(size_t)(r0 + i) * ne] = s;
                s = fmaf(expf(gl[i]), s, u[i]);
            }
        }
    }
    if (p.final_state != nullptr) p.final_state[(size_t)bh * ne + e] = s;
}

}  // namespace

hipError_t launch_carry(const Params &p, hipStream_t stream) {
    dim3 grid((unsigned)((p.dk * p.dv + kCarryThreads - 1) / kCarryThreads), (unsigned)(p.B * p.H));
    hipLaunchKernelGGL(carry_kernel, grid, dim3(kCarryThreads), 0, stream, p);
    return hipGetLastError();
}

}  // namespace gla
