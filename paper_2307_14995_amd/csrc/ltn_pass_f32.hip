// fp32 kernel for one decayed linear-attention pass (same block recurrence as the
// bf16 MFMA kernel, plain fp32 FMAs, no reduced-precision step anywhere).
//
//   P    = (A_i B_i^T) (.) M,       M[r,c] = lambda^(r-c) for r >= c else 0
//   O_i  = P C_i + diag(lambda^(r+1)) A_i S_i
//   S_i+1 = lambda^len S_i + sum_c lambda^(len-1-c) b_c^T c_c
//
// (arXiv 2307.14995, Sec. 3.2.1 / Eq. 1; Sec. 3.3 Algorithm 2 in block form.)
// One 256-thread workgroup per (chain, value-column slice).  Tiles live in LDS; every
// product is register-tiled (a thread owns a small rectangle of the result and walks the
// contraction with 16-byte LDS reads), the state rectangle of a thread stays in its
// registers for the whole sequence and is mirrored to LDS once per block for the
// A_i S_i product.  Plain passes with D in {64, 128} run on the matrix cores instead
// (ltn_pass_f32_mfma.hip); this kernel serves what that one does not have: the gated
// epilogue, unequal query/key and value widths, and heads of 96 and 256 features.
#include "ltn_kernels.h"

namespace ltn {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float4 ld4(const float* p) { return *(const float4*)p; }

// GATED (full-width slices, one pass): the block's output rows are complete, so the token
// mixer's epilogue (Sec. 3.1.2 Eq. 3 with the SimpleRMSNorm of Sec. 3.1.3 per head),
// y = o / sqrt(mean(o^2) + eps) (.) u, is applied to them from an LDS copy.
// A and B have D features per token; C and the output have DC (equal to D except around
// the LRPE-d expansion of Eq. 1, where queries and keys are twice as wide as values); the
// state is [D x DC].
// DR: features per token that A and B really have in memory (D, or 96 computed as 128 with
// the tiles' last columns zero and the state's last rows unused).
template <int D, int DV, int B, bool GATED, int DC = D, int DR = D>
__global__ __launch_bounds__(kThreads)
void pass_f32_kernel(const PassBatch pb, const int nsplit) {
    static_assert(!GATED || (DV == D && DC == D), "the gated epilogue needs complete output rows");
    static_assert(B % 16 == 0 && D % 64 == 0 && DV % 32 == 0 && DV <= DC && DC % DV == 0, "tile shapes");
    constexpr int DP = D + 4;     // row pitch of A and B tiles: 16-byte aligned rows, shifted banks
    constexpr int BP = B + 1;
    __shared__ __attribute__((aligned(16))) float As[B * DP];
    __shared__ __attribute__((aligned(16))) float Bs[B * DP];
    __shared__ __attribute__((aligned(16))) float Cs[B * DV];
    __shared__ float Ps[B * BP];
    __shared__ __attribute__((aligned(16))) float St[D * DV];
    __shared__ float pw[B + 1];   // lambda^0 .. lambda^B
    __shared__ __attribute__((aligned(16))) float Os[GATED ? B * DV : 4];
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

    const size_t ab_off = (size_t)chain * (size_t)N * DR;
    const size_t chain_off = (size_t)chain * (size_t)N * DC;
    const float* Ap = (const float*)P.a + ab_off;
    const float* Bp = (const float*)P.b + ab_off;
    const float* Cp = (const float*)P.c + chain_off + (size_t)split * DV;
    float* Op = P.out ? (float*)P.out + chain_off + (size_t)split * DV : nullptr;
    const float* Up = GATED ? (const float*)P.gate + chain_off : nullptr;
    float* Yp = GATED ? (float*)P.gated_out + chain_off : nullptr;

    // thread rectangles
    //   scores: rows sy*SR.., columns sx*SR.. of the B x B tile          (16 x 16 threads)
    //   output: rows oy + OY*m, columns 4*ox..+3 of the B x DV tile      (OY x DV/4 threads)
    //   state : rows uy*UR.., columns ux*UC.. of the D x DV state        (16 x 16 threads)
    constexpr int SR = B / 16;
    const int sy = tid >> 4, sx = tid & 15;
    constexpr int OX = DV / 4, OY = kThreads / OX, OM = (B + OY - 1) / OY;
    const int ox = tid % OX, oy = tid / OX;
    constexpr int UR = D / 16, UC = DV / 16;
    static_assert(UR % 4 == 0 && UC % 2 == 0, "vector reads of the state rectangle");
    const int uy = tid >> 4, ux = tid & 15;

    for (int n = tid; n <= B; n += kThreads) pw[n] = decay_pow(lam, n);
    float st[UR][UC];             // this thread's rectangle of the running state
#pragma unroll
    for (int a = 0; a < UR; ++a)
#pragma unroll
        for (int b = 0; b < UC; ++b) {
            const int i = uy * UR + a, j = ux * UC + b;
            st[a][b] = (P.state_in && (DR == D || i < DR))
                           ? P.state_in[(size_t)chain * DR * DC + (size_t)i * DC + split * DV + j] : 0.0f;
            St[i * DV + j] = st[a][b];
        }
    __syncthreads();

    for (long long t0 = 0; t0 < N; t0 += B) {
        const int len = (N - t0 < B) ? (int)(N - t0) : B;
        // ---- load tiles with 16-byte accesses (rows past the end are zero)
        for (int e = tid; e < B * (D / 4); e += kThreads) {
            const int r = e / (D / 4), i4 = e % (D / 4);
            const long long t = t0 + r;
            const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
            const bool ok = r < len && (DR == D || 4 * i4 < DR);
            const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
            *(float4*)&As[r * DP + 4 * i4] = ok ? ld4(Ap + gr * DR + 4 * i4) : z;
            *(float4*)&Bs[r * DP + 4 * i4] = ok ? ld4(Bp + gr * DR + 4 * i4) : z;
        }
        for (int e = tid; e < B * (DV / 4); e += kThreads) {
            const int r = e / (DV / 4), j4 = e % (DV / 4);
            const long long t = t0 + r;
            const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
            *(float4*)&Cs[r * DV + 4 * j4] = (r < len) ? ld4(Cp + gr * DC + 4 * j4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        __syncthreads();

        // ---- masked scores: an SR x SR rectangle per thread, skipped when above the diagonal
        {
            const int r0 = sy * SR, c0 = sx * SR;
            float acc[SR][SR];
#pragma unroll
            for (int a = 0; a < SR; ++a)
#pragma unroll
                for (int b = 0; b < SR; ++b) acc[a][b] = 0.0f;
            if (c0 <= r0 + SR - 1) {
#pragma unroll 4
                for (int i = 0; i < D; i += 4) {
                    float4 av[SR], bv[SR];
#pragma unroll
                    for (int a = 0; a < SR; ++a) av[a] = ld4(&As[(r0 + a) * DP + i]);
#pragma unroll
                    for (int b = 0; b < SR; ++b) bv[b] = ld4(&Bs[(c0 + b) * DP + i]);
#pragma unroll
                    for (int a = 0; a < SR; ++a)
#pragma unroll
                        for (int b = 0; b < SR; ++b) {
                            acc[a][b] = fmaf(av[a].x, bv[b].x, acc[a][b]);
                            acc[a][b] = fmaf(av[a].y, bv[b].y, acc[a][b]);
                            acc[a][b] = fmaf(av[a].z, bv[b].z, acc[a][b]);
                            acc[a][b] = fmaf(av[a].w, bv[b].w, acc[a][b]);
                        }
                }
            }
#pragma unroll
            for (int a = 0; a < SR; ++a)
#pragma unroll
                for (int b = 0; b < SR; ++b) {
                    const int r = r0 + a, c = c0 + b;
                    Ps[r * BP + c] = (c <= r) ? acc[a][b] * pw[r - c] : 0.0f;
                }
        }
        __syncthreads();

        // ---- outputs: rows oy + OY*m, four value columns per thread
        {
            float4 intra[OM], inter[OM];
#pragma unroll
            for (int m = 0; m < OM; ++m) {
                intra[m] = make_float4(0.f, 0.f, 0.f, 0.f);
                inter[m] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll 4
            for (int c = 0; c < len; ++c) {                       // P C (P is zero above the diagonal)
                const float4 cv = ld4(&Cs[c * DV + 4 * ox]);
#pragma unroll
                for (int m = 0; m < OM; ++m) {
                    const int r = oy + OY * m;
                    const float p = (r < B) ? Ps[r * BP + c] : 0.0f;
                    intra[m].x = fmaf(p, cv.x, intra[m].x);
                    intra[m].y = fmaf(p, cv.y, intra[m].y);
                    intra[m].z = fmaf(p, cv.z, intra[m].z);
                    intra[m].w = fmaf(p, cv.w, intra[m].w);
                }
            }
#pragma unroll 4
            for (int i = 0; i < D; i += 4) {                      // A S
                const float4 s0 = ld4(&St[(i + 0) * DV + 4 * ox]);
                const float4 s1 = ld4(&St[(i + 1) * DV + 4 * ox]);
                const float4 s2 = ld4(&St[(i + 2) * DV + 4 * ox]);
                const float4 s3 = ld4(&St[(i + 3) * DV + 4 * ox]);
#pragma unroll
                for (int m = 0; m < OM; ++m) {
                    const int r = oy + OY * m;
                    const float4 a = (r < B) ? ld4(&As[r * DP + i]) : make_float4(0.f, 0.f, 0.f, 0.f);
                    inter[m].x = fmaf(a.x, s0.x, fmaf(a.y, s1.x, fmaf(a.z, s2.x, fmaf(a.w, s3.x, inter[m].x))));
                    inter[m].y = fmaf(a.x, s0.y, fmaf(a.y, s1.y, fmaf(a.z, s2.y, fmaf(a.w, s3.y, inter[m].y))));
                    inter[m].z = fmaf(a.x, s0.z, fmaf(a.y, s1.z, fmaf(a.z, s2.z, fmaf(a.w, s3.z, inter[m].z))));
                    inter[m].w = fmaf(a.x, s0.w, fmaf(a.y, s1.w, fmaf(a.z, s2.w, fmaf(a.w, s3.w, inter[m].w))));
                }
            }
#pragma unroll
            for (int m = 0; m < OM; ++m) {
                const int r = oy + OY * m;
                if (r < B) {
                    const float q = pw[r + 1];
                    const float4 o = make_float4(fmaf(q, inter[m].x, intra[m].x), fmaf(q, inter[m].y, intra[m].y),
                                                 fmaf(q, inter[m].z, intra[m].z), fmaf(q, inter[m].w, intra[m].w));
                    if (GATED) *(float4*)&Os[r * DV + 4 * ox] = o;
                    if (r < len && Op) {
                        const long long t = t0 + r;
                        const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
                        *(float4*)(Op + gr * DC + 4 * ox) = o;
                    }
                }
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
            for (int e = tid; e < len * (DV / 4); e += kThreads) {
                const int r = e / (DV / 4), j4 = e % (DV / 4);
                const long long t = t0 + r;
                const size_t gr = (size_t)(rev ? (N - 1 - t) : t);
                const float4 o = ld4(&Os[r * DV + 4 * j4]);
                const float4 u = ld4(Up + gr * D + 4 * j4);
                const float s = rstd[r];
                *(float4*)(Yp + gr * D + 4 * j4) = make_float4(o.x * s * u.x, o.y * s * u.y, o.z * s * u.z, o.w * s * u.w);
            }
        }

        // ---- state update on the thread's own rectangle (registers), mirrored to LDS
        {
            const float decay_all = pw[len];
#pragma unroll
            for (int a = 0; a < UR; ++a)
#pragma unroll
                for (int b = 0; b < UC; ++b) st[a][b] *= decay_all;
#pragma unroll 4
            for (int c = 0; c < len; ++c) {
                const float w = pw[len - 1 - c];
                float bv[UR], cv[UC];
#pragma unroll
                for (int a = 0; a < UR; a += 4) {
                    const float4 x = ld4(&Bs[c * DP + uy * UR + a]);
                    bv[a] = x.x * w; bv[a + 1] = x.y * w; bv[a + 2] = x.z * w; bv[a + 3] = x.w * w;
                }
#pragma unroll
                for (int b = 0; b < UC; b += 2) {
                    const float2 x = *(const float2*)&Cs[c * DV + ux * UC + b];
                    cv[b] = x.x; cv[b + 1] = x.y;
                }
#pragma unroll
                for (int a = 0; a < UR; ++a)
#pragma unroll
                    for (int b = 0; b < UC; ++b) st[a][b] = fmaf(bv[a], cv[b], st[a][b]);
            }
            // every thread has read the old LDS copy (outputs above, before the last barrier)
#pragma unroll
            for (int a = 0; a < UR; ++a)
#pragma unroll
                for (int b = 0; b < UC; ++b) St[(uy * UR + a) * DV + ux * UC + b] = st[a][b];
        }
        __syncthreads();
    }

    if (P.state_out) {
#pragma unroll
        for (int a = 0; a < UR; ++a)
#pragma unroll
            for (int b = 0; b < UC; ++b) {
                const int i = uy * UR + a, j = ux * UC + b;
                if (DR == D || i < DR) P.state_out[(size_t)chain * DR * DC + (size_t)i * DC + split * DV + j] = st[a][b];
            }
    }
}

template <int D, int DV, int B, bool GATED = false, int DC = D, int DR = D>
hipError_t launch_t(const PassBatch& pb, hipStream_t stream) {
    const int nsplit = DC / DV;
    const long long wgs = (long long)pb.chains * pb.count * nsplit;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pass_f32_kernel<D, DV, B, GATED, DC, DR>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, pb, nsplit);
    return hipGetLastError();
}

__global__ void state_copy_kernel(const float* __restrict__ in, float* __restrict__ out, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) out[i] = in ? in[i] : 0.0f;
}

}  // namespace

hipError_t launch_pass_f32(const PassBatch& pb, int D, int dv, int block, hipStream_t stream, int DC) {
    if (DC != 0 && DC != D) {              // queries/keys and values of different widths (plain pass only)
        if (pb.p[0].gate) return hipErrorInvalidValue;
#define LTN_F32_DC(d, v, c, b) if (D == d && dv == v && DC == c && block == b) return launch_t<d, v, b, false, c>(pb, stream)
        LTN_F32_DC(256, 64, 128, 16); LTN_F32_DC(128, 128, 256, 16); LTN_F32_DC(128, 64, 256, 16);
        LTN_F32_DC(128, 64, 64, 16); LTN_F32_DC(128, 64, 64, 32);
        LTN_F32_DC(64, 128, 128, 16); LTN_F32_DC(64, 128, 128, 32); LTN_F32_DC(64, 64, 128, 16); LTN_F32_DC(64, 64, 128, 32);
#undef LTN_F32_DC
        return hipErrorInvalidValue;
    }
    if (!pb.p[0].gate && pb.segs == 1 && !pb.state_only && pass_f32_mfma_supports(D, dv, block))
        return launch_pass_f32_mfma(pb, D, dv, block, stream);       // the matrix-core kernel
    if (D == 96) {                         // computed as 128 with zero tile columns, 32-column slices
        if (pb.p[0].gate || dv != 32) return hipErrorInvalidValue;
        if (block == 16) return launch_t<128, 32, 16, false, 96, 96>(pb, stream);
        if (block == 32) return launch_t<128, 32, 32, false, 96, 96>(pb, stream);
        return hipErrorInvalidValue;
    }
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
    LTN_F32_CASE(256, 64, 16);
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
