// Measurement aid, not part of the attention path: a bare streaming-read kernel that pulls
// bytes the way the pass kernels' tile pipeline does -- every wave of a 512-thread workgroup
// keeps eight wave-wide 1 KB loads in flight (64 KB per compute unit), either straight into
// LDS (global_load_lds_dwordx4) or into registers -- so that the report can put "what this
// machine gives such a pipeline" next to the 8 TB/s peak and next to the kernels' own rates.
// Each workgroup walks its own contiguous region `iters` times; regions of 64 KB stay in L2,
// of 512 KB in the memory-side cache, of 16 MB come from HBM.
#include "ltn_bf16_tiles.h"

namespace ltn {
namespace {

template <int MODE>
__global__ __launch_bounds__(512)
void probe_stream_kernel(const char* __restrict__ base, size_t per_wg, int iters, unsigned* __restrict__ sink) {
    __shared__ __attribute__((aligned(1024))) char smem[8 * 8 * 1024];    // 8 waves x 8 slots x 1 KB
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const char* p = base + (size_t)blockIdx.x * per_wg;
    const unsigned lds0 = lds_address(smem) + (unsigned)wave * 8192u;
    const size_t steps = per_wg / 65536;          // one step = 8 loads per wave = 64 KB per workgroup
    u32x4 acc = {0, 0, 0, 0};
    for (int it = 0; it < iters; ++it)
        for (size_t c = 0; c < steps; ++c) {
            const char* q = p + c * 65536 + wave * 1024 + lane * 16;
            if (MODE == 0) {
#pragma unroll
                for (int s = 0; s < 8; ++s) dma16(lds0 + s * 1024, q + s * 8192);
                wait_dma<0>();
            } else {
                u32x4 r[8];
#pragma unroll
                for (int s = 0; s < 8; ++s) r[s] = *(const u32x4*)(q + s * 8192);
#pragma unroll
                for (int s = 0; s < 8; ++s) acc ^= r[s];
            }
        }
    if (MODE == 0) acc = *(const u32x4*)(smem + wave * 8192 + lane * 16);
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;   // keeps the loads alive
}

}  // namespace

// `buf` holds at least wgs * per_wg bytes; per_wg is a multiple of 64 KB.
hipError_t launch_probe_stream(const void* buf, size_t per_wg, int wgs, int iters, int to_registers, unsigned* sink,
                               hipStream_t stream) {
    if (!buf || !sink || wgs <= 0 || iters <= 0 || per_wg == 0 || per_wg % 65536 != 0) return hipErrorInvalidValue;
    if (to_registers)
        hipLaunchKernelGGL(probe_stream_kernel<1>, dim3((unsigned)wgs), dim3(512), 0, stream, (const char*)buf, per_wg, iters, sink);
    else
        hipLaunchKernelGGL(probe_stream_kernel<0>, dim3((unsigned)wgs), dim3(512), 0, stream, (const char*)buf, per_wg, iters, sink);
    return hipGetLastError();
}

}  // namespace ltn
