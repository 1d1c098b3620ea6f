// fp32 kernel for one decayed linear-attention pass (same block recurrence as the
// bf16 MFMA kernel, plain fp32 FMAs, no reduced-precision step anywhere).
//
//   P    = (A_i B_i^T) (.) M,       M[r,c] = lambda^(r-c) for r >= c else 0
//   O_i  = P C_i + diag(lambda^(r+1)) A_i S_i
//   S_i+1 = lambda^len S_i + sum_c lambda^(len-1-c) b_c^T c_c
//
// (arXiv 2307.14995, Sec. 3.2.1 / Eq. 1; Sec. 3.3 Algorithm 2 in block form.)
// One 256-thread workgroup per (chain, value-column slice); tiles and the fp32
// state live in LDS.  This path exists for fp32 callers and the fp32 parity
// configuration; the throughput path is the bf16 kernel.
#include "ltn_kernels.h"

namespace ltn {
namespace {

constexpr int kThreads = 256;

// GATED (full-width slices, one pass): the block's output rows are complete, so the token
// mixer's epilogue (Sec. 3.1.2 Eq. 3 with the SimpleRMSNorm of Sec. 3.1.3 per head),
// y = o / sqrt(mean(o^2) + eps) (.) u, is applied to them from an LDS copy.
template <int D, int DV, int B, bool GATED>
__global__ __launch_bounds__(kThreads)
void pass_f32_kernel(const PassBatch pb, const int nsplit) {
    static_assert(!GATED || DV == D, "the gated epilogue needs complete output rows");
    constexpr int DP = D + 1;     // padded pitches: conflict-free column walks
    constexpr int BP = B + 1;
    __shared__ float As[B * DP];
    __shared__ float Bs[B * DP];
    __shared__ float Cs[B * DV];
    __shared__ float Ps[B * BP];
    __shared__ float St[D * DV];
    __shared__ float pw[B + 1];   // lambda^0 .. lambda^B
    __shared__ float Os[GATED ? B * DV : 1];
    __shared__ float rstd[GATED ? B : 1];

    const int tid = threadIdx.x;
    int chain, within;
    map_workgroup(blockIdx.x, pb.count * nsplit, pb.chains, chain, within);
    const int pi = within / nsplit;
    const int split = within - pi * nsplit;
    const PassArgs P = pb.p[pi];
    const int rev = P.rev;
    const long long N = pb.N;
    const float lam = pb.decay[chain % pb.H];

    const size_t chain_off = (size_t)chain * (size_t)N * D;
    const float* Ap = (const float*)P.a + chain_off;
    const float* Bp = (const float*)P.b + chain_off;
    const float* Cp = (const float*)P.c + chain_off + (size_t)split * DV;
    float* Op = P.out ? (float*)P.out + chain_off + (size_t)split * DV : nullptr;
    const float* Up = GATED ? (const float*)P.gate + chain_off : nullptr;
    float* Yp = GATED ? (float*)P.gated_out + chain_off : nullptr;

    for (int n = tid; n <= B; n += kThreads) pw[n] = decay_pow(lam, n);
    for (int e = tid; e < D * DV; e += kThreads) {
        const int i = e / DV, j = e % DV;
        St[e] = P.state_in ? P.state_in[(size_t)chain * D * D + (size_t)i * D + split * DV + j] : 0.0f;
    }
    __syncthreads();

    for (long long t0 = 0; t0 < N; t0 += B) {
        const int len = (N - t0 < B) ? (int)(N - t0) : B;
        // ---- load tiles (rows past the end are zero)
        for (int e = tid; e < B * D; e += kThreads) {
            const int r = e / D, i = e % D;
            const long long t = t0 + r;
            const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
            const bool ok = r < len;
            As[r * DP + i] = ok ? Ap[gr * D + i] : 0.0f;
            Bs[r * DP + i] = ok ? Bp[gr * D + i] : 0.0f;
        }
        for (int e = tid; e < B * DV; e += kThreads) {
            const int r = e / DV, j = e % DV;
            const long long t = t0 + r;
            const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
            Cs[e] = (r < len) ? Cp[gr * D + j] : 0.0f;
        }
        __syncthreads();
        // ---- masked scores
        for (int e = tid; e < B * B; e += kThreads) {
            const int r = e / B, c = e % B;
            float acc = 0.0f;
            if (c <= r) {
#pragma unroll 8
                for (int i = 0; i < D; ++i) acc = fmaf(As[r * DP + i], Bs[c * DP + i], acc);
                acc *= pw[r - c];
            }
            Ps[r * BP + c] = acc;
        }
        __syncthreads();
        // ---- outputs
        for (int e = tid; e < B * DV; e += kThreads) {
            const int r = e / DV, j = e % DV;
            float intra = 0.0f, inter = 0.0f;
            for (int c = 0; c <= r; ++c) intra = fmaf(Ps[r * BP + c], Cs[c * DV + j], intra);
#pragma unroll 8
            for (int i = 0; i < D; ++i) inter = fmaf(As[r * DP + i], St[i * DV + j], inter);
            const float o = fmaf(pw[r + 1], inter, intra);
            if (GATED) Os[e] = o;
            if (r < len && Op) {
                const long long t = t0 + r;
                const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
                Op[gr * D + j] = o;
            }
        }
        __syncthreads();
        if constexpr (GATED) {
            if (tid < len) {
                float ss = 0.0f;
                for (int j = 0; j < DV; ++j) {
                    const float o = Os[tid * DV + (j + tid) % DV];   // skewed walk: no bank conflicts
                    ss = fmaf(o, o, ss);
                }
                rstd[tid] = 1.0f / sqrtf(ss * (1.0f / D) + P.eps);
            }
            __syncthreads();
            for (int e = tid; e < len * DV; e += kThreads) {
                const int r = e / DV, j = e % DV;
                const long long t = t0 + r;
                const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
                Yp[gr * D + j] = Os[e] * rstd[r] * Up[gr * D + j];
            }
        }
        // ---- state update (each thread owns its state entries: no hazard inside the step)
        for (int e = tid; e < D * DV; e += kThreads) {
            const int i = e / DV, j = e % DV;
            float acc = 0.0f;
            for (int c = 0; c < len; ++c) acc = fmaf(pw[len - 1 - c] * Bs[c * DP + i], Cs[c * DV + j], acc);
            St[e] = fmaf(pw[len], St[e], acc);
        }
        __syncthreads();
    }

    if (P.state_out) {
        for (int e = tid; e < D * DV; e += kThreads) {
            const int i = e / DV, j = e % DV;
            P.state_out[(size_t)chain * D * D + (size_t)i * D + split * DV + j] = St[e];
        }
    }
}

template <int D, int DV, int B, bool GATED = false>
hipError_t launch_t(const PassBatch& pb, hipStream_t stream) {
    const int nsplit = D / DV;
    const long long wgs = (long long)pb.chains * pb.count * nsplit;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pass_f32_kernel<D, DV, B, GATED>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, pb, nsplit);
    return hipGetLastError();
}

__global__ void state_copy_kernel(const float* __restrict__ in, float* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in ? in[i] : 0.0f;
}

}  // namespace

hipError_t launch_pass_f32(const PassBatch& pb, int D, int dv, int block, hipStream_t stream) {
    if (pb.p[0].gate) {                    // gated epilogue: one pass, complete output rows
        if (pb.count != 1 || dv != D || !pb.p[0].gated_out) return hipErrorInvalidValue;
#define LTN_F32_GATED(d, b) if (D == d && block == b) return launch_t<d, d, b, true>(pb, stream)
        LTN_F32_GATED(64, 16); LTN_F32_GATED(64, 32); LTN_F32_GATED(64, 64);
        LTN_F32_GATED(128, 16); LTN_F32_GATED(128, 32);
#undef LTN_F32_GATED
        return hipErrorInvalidValue;
    }
#define LTN_F32_CASE(d, v, b) if (D == d && dv == v && block == b) return launch_t<d, v, b>(pb, stream)
    LTN_F32_CASE(64, 64, 16); LTN_F32_CASE(64, 64, 32); LTN_F32_CASE(64, 64, 64);
    LTN_F32_CASE(64, 32, 16); LTN_F32_CASE(64, 32, 32); LTN_F32_CASE(64, 32, 64);
    LTN_F32_CASE(128, 128, 16); LTN_F32_CASE(128, 128, 32);
    LTN_F32_CASE(128, 64, 16); LTN_F32_CASE(128, 64, 32);
#undef LTN_F32_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_state_copy(const float* kv_in, float* kv_out, size_t n, hipStream_t stream) {
    if (n == 0 || kv_in == kv_out) return hipSuccess;
    const unsigned grid = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    hipLaunchKernelGGL(state_copy_kernel, dim3(grid), dim3(256), 0, stream, kv_in, kv_out, n);
    return hipGetLastError();
}

}  // namespace ltn
