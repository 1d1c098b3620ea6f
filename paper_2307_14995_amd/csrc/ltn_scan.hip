// Sequence-parallel form of the decayed linear-attention pass (arXiv 2307.14995, Sec. 3.3:
// the recurrence kv_t = lambda kv_{t-1} + k_t^T v_t is linear in the state, so a chain cut
// into segments needs only each segment's end state from a zero start and a scan over
// them).  This file holds the scan: with L[g] the end state of segment g computed from a
// zero state and len(g) its token count,
//
//     S[0] = initial state,     S[g+1] = lambda^len(g) S[g] + L[g].
//
// One thread per state element and (pass, chain); the segments are walked in order.  The
// states array [count][chains][segs][D*D] is rewritten in place from L[.] to S[.] (the
// state at each segment's start); the state after the last segment goes to kv_out.
#include "ltn_kernels.h"

namespace ltn {
namespace {

__global__ __launch_bounds__(256)
void segment_scan_kernel(float* __restrict__ states, const float* __restrict__ kv_in, float* __restrict__ kv_out,
                         const float* __restrict__ decay, int count, int chains, int H, int segs,
                         long long seg_len, long long N, int DD) {
    const long long total = (long long)count * chains * DD;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int e = (int)(idx % DD);
    const long long pc = idx / DD;
    const int chain = (int)(pc % chains);
    const int pass = (int)(pc / chains);
    const float lam = decay[chain % H];
    const float lam_full = decay_pow(lam, (int)seg_len);
    float* s = states + (size_t)pc * segs * DD + e;
    float run = (pass == 0 && kv_in) ? kv_in[(size_t)chain * DD + e] : 0.0f;
    for (int g = 0; g < segs; ++g) {
        const long long left = N - (long long)g * seg_len;
        const bool last = g + 1 == segs;
        // the last segment's end state exists only if someone asked for the final state
        const float local = (!last || kv_out) ? s[(size_t)g * DD] : 0.0f;
        s[(size_t)g * DD] = run;
        run = fmaf(left >= seg_len ? lam_full : decay_pow(lam, (int)left), run, local);
    }
    if (pass == 0 && kv_out) kv_out[(size_t)chain * DD + e] = run;
}

}  // namespace

hipError_t launch_segment_scan(float* states, const float* kv_in, float* kv_out, const float* decay,
                               int count, int chains, int H, int segs, long long seg_len, long long N,
                               int D, hipStream_t stream, int DC) {
    if (DC == 0) DC = D;
    const long long total = (long long)count * chains * D * DC;
    if (total <= 0 || segs < 1 || seg_len <= 0 || seg_len > 0x7fffffffLL) return hipErrorInvalidValue;
    const long long wgs = (total + 255) / 256;
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(segment_scan_kernel, dim3((unsigned)wgs), dim3(256), 0, stream,
                       states, kv_in, kv_out, decay, count, chains, H, segs, seg_len, N, D * DC);
    return hipGetLastError();
}

}  // namespace ltn
