// Recurrent decode of Lightning Attention (arXiv 2307.14995, Sec. 3.3, Algorithm 2), per
// (batch, head), for S >= 1 consecutive tokens in one call:
//     kv <- lambda kv + k_s^T v_s   (fp32),   o_s = q_s kv   (the updated state),  s = 0..S-1
// The state is read once, kept in registers over the S iterations and written once, so a
// call moves 2 D^2 fp32 values per chain whatever S is; with S = 1 (one token per call) the
// step is bound by HBM bandwidth (about half a FLOP per byte).  Plain fp32 vector code with
// 16-byte accesses; one 128-thread workgroup per chain, each thread owns four adjacent state
// columns of a strided set of rows, and the D partial dot products per column are reduced
// through LDS.
#include "ltn_kernels.h"

namespace ltn {
namespace {

// 128 threads: measured best on MI355X for the 2048-chain decode workload (39.4 us per step
// against 41.9 with 256 and 39.9 with 1024); must be >= D (one thread per q/k/v feature).
constexpr int kThreads = 128;

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short h) {
    return __uint_as_float(((unsigned int)h) << 16);
}

__device__ __forceinline__ unsigned short f32_to_bf16_bits(float f) {   // round to nearest even
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

template <int D, bool BF16>
__global__ __launch_bounds__(kThreads)
void decode_kernel(const void* __restrict__ q, const void* __restrict__ k, const void* __restrict__ v,
                   void* __restrict__ o, float* __restrict__ kv, const float* __restrict__ decay, int H,
                   int steps) {
    constexpr int TX = D / 4;             // threads across one state row (float4 each)
    constexpr int TY = kThreads / TX;     // rows in flight per sweep
    constexpr int IT = D / TY;            // sweeps
    __shared__ float qs[D], ks[D], vs[D];
    __shared__ float4 part[TY][TX];

    const int chain = blockIdx.x;
    const int tid = threadIdx.x;
    const float lam = decay[chain % H];
    const int tx = tid % TX, ty = tid / TX;
    float4* S = (float4*)(kv + (size_t)chain * D * D);
    float4 s[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) s[it] = S[(size_t)(ty + TY * it) * TX + tx];

    for (int step = 0; step < steps; ++step) {
        if (tid < D) {
            const size_t e = ((size_t)chain * steps + step) * D + tid;
            if (BF16) {
                qs[tid] = bf16_bits_to_f32(((const unsigned short*)q)[e]);
                ks[tid] = bf16_bits_to_f32(((const unsigned short*)k)[e]);
                vs[tid] = bf16_bits_to_f32(((const unsigned short*)v)[e]);
            } else {
                qs[tid] = ((const float*)q)[e];
                ks[tid] = ((const float*)k)[e];
                vs[tid] = ((const float*)v)[e];
            }
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
        if (tid < D) {
            const int cx = tid / 4, comp = tid % 4;
            float sum = 0.f;
#pragma unroll
            for (int y = 0; y < TY; ++y) sum += ((const float*)&part[y][cx])[comp];
            const size_t e = ((size_t)chain * steps + step) * D + tid;
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
                         const float* decay, int chains, int H, int steps, int D, int is_bf16,
                         hipStream_t stream) {
    if (chains <= 0 || steps <= 0) return hipSuccess;
    const dim3 grid((unsigned)chains), block(kThreads);
    if (D == 128 && is_bf16) hipLaunchKernelGGL((decode_kernel<128, true>), grid, block, 0, stream, q, k, v, o, kv, decay, H, steps);
    else if (D == 128) hipLaunchKernelGGL((decode_kernel<128, false>), grid, block, 0, stream, q, k, v, o, kv, decay, H, steps);
    else if (D == 64 && is_bf16) hipLaunchKernelGGL((decode_kernel<64, true>), grid, block, 0, stream, q, k, v, o, kv, decay, H, steps);
    else if (D == 64) hipLaunchKernelGGL((decode_kernel<64, false>), grid, block, 0, stream, q, k, v, o, kv, decay, H, steps);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ltn
