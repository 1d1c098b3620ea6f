// Recurrent decode of Lightning Attention (arXiv 2307.14995, Sec. 3.3, Algorithm 2), per
// (batch, head), for S >= 1 consecutive tokens in one call:
//     kv <- lambda kv + k_s^T v_s   (fp32),   o_s = q_s kv   (the updated state),  s = 0..S-1
// The state is read once, kept in registers over the S iterations and written once, so a
// call moves 2 D^2 fp32 values per chain whatever S is; with S = 1 (one token per call) the
// step is bound by HBM bandwidth (about half a FLOP per byte).  Plain fp32 vector code with
// 16-byte accesses; one workgroup per chain, each thread owns four adjacent state
// columns of a strided set of rows, and the partial dot products per column are reduced
// through LDS.  Queries and keys have DK features, values and outputs DV (the state is
// [DK x DV]); the two differ only behind the LRPE-d expansion of Eq. 1.
#include "ltn_kernels.h"

namespace ltn {
namespace {

// Threads per workgroup, at least max(DK, DV) (one thread per q/k/v feature).  128 threads
// per 128 x 128 state: measured best on MI355X for the 2048-chain decode workload (39.4 us
// per step against 41.9 with 256 and 39.9 with 1024); larger states keep the same number of
// state values per thread, smaller ones the 128 threads.
constexpr int threads_for(int DK, int DV) {
    return (DK == 96 && DV == 96) ? 96 : (DK * DV / 128 < 128 ? 128 : DK * DV / 128);   // 96: 24 threads per row
}

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short h) {
    return __uint_as_float(((unsigned int)h) << 16);
}

__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {   // round to nearest even
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

template <int DK, int DV, bool BF16>
__global__ __launch_bounds__(threads_for(DK, DV))
void decode_kernel(const void* __restrict__ q, const void* __restrict__ k, const void* __restrict__ v,
                   void* __restrict__ o, float* __restrict__ kv, const float* __restrict__ decay, int H,
                   int steps) {
    constexpr int kThreads = threads_for(DK, DV);
    constexpr int TX = DV / 4;            // threads across one state row (float4 each)
    constexpr int TY = kThreads / TX;     // rows in flight per sweep
    constexpr int IT = DK / TY;           // sweeps
    static_assert(kThreads >= DK && kThreads >= DV && kThreads % TX == 0 && DK % TY == 0, "thread layout");
    __shared__ float qs[DK], ks[DK], vs[DV];
    __shared__ float4 part[TY][TX];

    const int chain = blockIdx.x;
    const int tid = threadIdx.x;
    const float lam = decay[chain % H];
    const int tx = tid % TX, ty = tid / TX;
    float4* S = (float4*)(kv + (size_t)chain * DK * DV);
    float4 s[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) s[it] = S[(size_t)(ty + TY * it) * TX + tx];

    for (int step = 0; step < steps; ++step) {
        if (tid < DK) {
            const size_t e = ((size_t)chain * steps + step) * DK + tid;
            if (BF16) {
                qs[tid] = bf16_bits_to_f32(((const unsigned short*)q)[e]);
                ks[tid] = bf16_bits_to_f32(((const unsigned short*)k)[e]);
            } else {
                qs[tid] = ((const float*)q)[e];
                ks[tid] = ((const float*)k)[e];
            }
        }
        if (tid < DV) {
            const size_t e = ((size_t)chain * steps + step) * DV + tid;
            vs[tid] = BF16 ? bf16_bits_to_f32(((const unsigned short*)v)[e]) : ((const float*)v)[e];
        }
        __syncthreads();
        const float4 vv = *(const float4*)(&vs[4 * tx]);
        float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int i = ty + TY * it;
            const float ki = ks[i], qi = qs[i];
            s[it].x = fmaf(lam, s[it].x, ki * vv.x);
            s[it].y = fmaf(lam, s[it].y, ki * vv.y);
            s[it].z = fmaf(lam, s[it].z, ki * vv.z);
            s[it].w = fmaf(lam, s[it].w, ki * vv.w);
            acc.x = fmaf(qi, s[it].x, acc.x);
            acc.y = fmaf(qi, s[it].y, acc.y);
            acc.z = fmaf(qi, s[it].z, acc.z);
            acc.w = fmaf(qi, s[it].w, acc.w);
        }
        part[ty][tx] = acc;
        __syncthreads();                  // also: everyone is done with qs/ks/vs of this step
        if (tid < DV) {
            const int cx = tid / 4, comp = tid % 4;
            float sum = 0.f;
#pragma unroll
            for (int y = 0; y < TY; ++y) sum += ((const float*)&part[y][cx])[comp];
            const size_t e = ((size_t)chain * steps + step) * DV + tid;
            if (BF16) ((unsigned short*)o)[e] = f32_to_bf16_bits(sum);
            else ((float*)o)[e] = sum;
        }
        // the next step's first barrier separates these reads of `part` from its next writes
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) S[(size_t)(ty + TY * it) * TX + tx] = s[it];
}

}  // namespace

hipError_t launch_decode(const void* q, const void* k, const void* v, void* o, float* kv,
                         const float* decay, int chains, int H, int steps, int DK, int DV, int is_bf16,
                         hipStream_t stream) {
    if (chains <= 0 || steps <= 0) return hipSuccess;
    const dim3 grid((unsigned)chains);
#define LTN_DECODE(dk, dv)                                                                              \
    if (DK == dk && DV == dv) {                                                                         \
        const dim3 block(threads_for(dk, dv));                                                          \
        if (is_bf16) hipLaunchKernelGGL((decode_kernel<dk, dv, true>), grid, block, 0, stream, q, k, v, o, kv, decay, H, steps);  \
        else hipLaunchKernelGGL((decode_kernel<dk, dv, false>), grid, block, 0, stream, q, k, v, o, kv, decay, H, steps);         \
        return hipGetLastError();                                                                       \
    }
    LTN_DECODE(128, 128) LTN_DECODE(64, 64) LTN_DECODE(96, 96) LTN_DECODE(256, 256) LTN_DECODE(256, 128) LTN_DECODE(128, 64)
#undef LTN_DECODE
    return hipErrorInvalidValue;
}

}  // namespace ltn
