// Input side of the token mixer for queries and keys (arXiv 2307.14995): the activation of
// Sec. 3.1.2 Eq. 2, phi = swish, z = x sigma(x), and the position encoding of Sec. 3.1.1
// Eq. 1, LRPE-d, in the separable form that keeps the attention linear: with one learnable
// angle per head and feature, theta[h, d], and p the token's absolute position,
//
//     y = [ z (.) cos(theta p) | z (.) sin(theta p) ]          (2D features per token)
//
// for queries and keys alike, so that y_q(t) . y_k(s) = sum_d z_q[d] z_k[d] cos(theta_d (t - s)),
// the real part of Eq. 1's phase.  Without theta, y = z (D features).  The derivative:
//
//     dz = dy_c cos + dy_s sin,   dx = dz phi'(x),   phi'(x) = sigma (1 + x (1 - sigma)),
//     dtheta[h, d] = sum over batch and tokens of  p z (dy_s cos - dy_c sin).
//
// Streaming kernels, 16 bytes per lane and access.  A workgroup handles 64 tokens of one
// head for every batch entry, so a (token, feature) pair's sine and cosine are computed
// once and reused over the batch.  The angle theta p is formed in fp64 and reduced there to a
// fraction of a turn in [-1/2, 1/2] (positions reach 10^4 .. 10^6: an fp32 product would
// lose the phase); sine and cosine of the fraction come from the hardware's turn-based
// v_sin_f32 / v_cos_f32, the sigmoid from v_exp_f32 and v_rcp_f32 -- with the library
// routines instead, these kernels are bound by the vector ALUs, not by HBM.
// dtheta is reduced without atomics: every thread sums its few tokens (times the batch) in
// fp32, the workgroup adds its threads' sums in a fixed order in fp64 through LDS and writes
// one partial, and a second kernel adds the partials in order -- bitwise reproducible.
#include "ltn_kernels.h"

namespace ltn {
namespace {

constexpr int kThreads = 256;
constexpr int kTok = 64;                 // tokens per workgroup

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;

// sigma(x) = 1 / (1 + 2^(-x log2 e)); exp2 overflows to +inf for very negative x, whose
// reciprocal is the right limit 0.
__device__ __forceinline__ float sigmoid(float x) {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

// E consecutive features of one token, 16 bytes in either dtype.
template <bool BF16>
struct Vec {
    static constexpr int E = BF16 ? 8 : 4;
    float v[E];
    __device__ __forceinline__ void load(const void* base, size_t elem) {
        if constexpr (BF16) {
            const uint4 w = *(const uint4*)((const unsigned short*)base + elem);
            const unsigned int u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[2 * i] = __uint_as_float(u[i] << 16);
                v[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
            }
        } else {
            const float4 w = *(const float4*)((const float*)base + elem);
            v[0] = w.x; v[1] = w.y; v[2] = w.z; v[3] = w.w;
        }
    }
    __device__ __forceinline__ void store(void* base, size_t elem) const {
        if constexpr (BF16) {
            f32x8 f;
#pragma unroll
            for (int i = 0; i < 8; ++i) f[i] = v[i];
            union { bf16x8 h; uint4 w; } cv;
            cv.h = __builtin_convertvector(f, bf16x8);       // round to nearest even
            *(uint4*)((unsigned short*)base + elem) = cv.w;
        } else {
            *(float4*)((float*)base + elem) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
};

template <int D, bool BF16, bool BWD>
__global__ __launch_bounds__(kThreads)
void prologue_kernel(const void* __restrict__ x, const float* __restrict__ theta, const void* __restrict__ dy,
                     void* __restrict__ out, double* __restrict__ partials, int act, int Bt, int H,
                     long long N, long long pos0, int nchunks) {
    using V = Vec<BF16>;
    constexpr int E = V::E;
    constexpr int TX = D / E;                 // threads across one token's features
    constexpr int TY = kThreads / TX;         // tokens in flight
    __shared__ double red[BWD ? TY : 1][BWD ? D : 1];

    const int chunk = blockIdx.x % nchunks;
    const int h = blockIdx.x / nchunks;
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    const int d0 = tx * E;
    const bool lrpe = theta != nullptr;
    const int W = lrpe ? 2 * D : D;           // features per token of y / dy

    float th[E];
#pragma unroll
    for (int e = 0; e < E; ++e) th[e] = lrpe ? theta[(size_t)h * D + d0 + e] : 0.0f;
    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.0f;

    const long long t0 = (long long)chunk * kTok;
    for (int r = ty; r < kTok && t0 + r < N; r += TY) {
        const long long t = t0 + r;
        const double p = (double)(pos0 + t);
        const float pf = (float)p;
        float cs[E], sn[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            if (lrpe) {
                const double turns = (double)th[e] * p * 0.15915494309189535;   // theta p / 2 pi
                const float frac = (float)(turns - rint(turns));                 // in [-1/2, 1/2]
                sn[e] = __builtin_amdgcn_sinf(frac);
                cs[e] = __builtin_amdgcn_cosf(frac);
            } else {
                cs[e] = 1.0f;
                sn[e] = 0.0f;
            }
        }
        for (int b = 0; b < Bt; ++b) {
            const size_t row = ((size_t)b * H + h) * (size_t)N + (size_t)t;
            V xv;
            xv.load(x, row * D + d0);
            float z[E], dphi[E];
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float s = sigmoid(xv.v[e]);
                z[e] = act ? xv.v[e] * s : xv.v[e];
                dphi[e] = act ? s * (1.0f + xv.v[e] * (1.0f - s)) : 1.0f;
            }
            if constexpr (!BWD) {
                V yc;
#pragma unroll
                for (int e = 0; e < E; ++e) yc.v[e] = z[e] * cs[e];
                yc.store(out, row * W + d0);
                if (lrpe) {
                    V ys;
#pragma unroll
                    for (int e = 0; e < E; ++e) ys.v[e] = z[e] * sn[e];
                    ys.store(out, row * W + D + d0);
                }
            } else {
                V gc, gs, dx;
                gc.load(dy, row * W + d0);
                if (lrpe) gs.load(dy, row * W + D + d0);
#pragma unroll
                for (int e = 0; e < E; ++e) {
                    const float g_s = lrpe ? gs.v[e] : 0.0f;
                    dx.v[e] = (gc.v[e] * cs[e] + g_s * sn[e]) * dphi[e];
                    acc[e] = fmaf(pf, z[e] * (g_s * cs[e] - gc.v[e] * sn[e]), acc[e]);
                }
                dx.store(out, row * D + d0);
            }
        }
    }

    if constexpr (BWD) {
        if (partials) {                       // uniform: every thread of every workgroup
#pragma unroll
            for (int e = 0; e < E; ++e) red[ty][d0 + e] = (double)acc[e];
            __syncthreads();
            if (threadIdx.x < D) {
                double s = 0.0;
                for (int y = 0; y < TY; ++y) s += red[y][threadIdx.x];
                partials[((size_t)chunk * H + h) * D + threadIdx.x] = s;
            }
        }
    }
}

// dtheta[h, d] = sum of the partials over chunks, in a fixed order: a workgroup takes 16
// (h, d) columns; 16 threads per column each add every 16th chunk, then one adds the 16 sums.
__global__ __launch_bounds__(256)
void prologue_reduce_kernel(const double* __restrict__ partials, float* __restrict__ dtheta,
                            int nchunks, int HD) {
    __shared__ double red[16][16];
    const int col = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int i = blockIdx.x * 16 + col;
    double s = 0.0;
    if (i < HD)
        for (int c = grp; c < nchunks; c += 16) s += partials[(size_t)c * HD + i];
    red[grp][col] = s;
    __syncthreads();
    if (grp == 0 && i < HD) {
        double t = 0.0;
#pragma unroll
        for (int g = 0; g < 16; ++g) t += red[g][col];
        dtheta[i] = (float)t;
    }
}

template <int D, bool BF16, bool BWD>
hipError_t launch_t(const void* x, const float* theta, const void* dy, void* out, double* partials, int act,
                    int Bt, int H, long long N, long long pos0, int nchunks, hipStream_t stream) {
    hipLaunchKernelGGL((prologue_kernel<D, BF16, BWD>), dim3((unsigned)(nchunks * H)), dim3(kThreads), 0, stream,
                       x, theta, dy, out, partials, act, Bt, H, N, pos0, nchunks);
    return hipGetLastError();
}

}  // namespace

long long prologue_partial_count(long long N) { return (N + kTok - 1) / kTok; }

hipError_t launch_prologue(const void* x, const float* theta, const void* dy, void* out, float* dtheta,
                           double* partials, int act, int Bt, int H, long long N, int D, long long pos0,
                           int is_bf16, int is_bwd, hipStream_t stream) {
    if (Bt <= 0 || H <= 0 || N <= 0) return hipSuccess;
    const long long nch = prologue_partial_count(N);
    if (nch * H > 0x7fffffffLL) return hipErrorInvalidValue;
    const int nchunks = (int)nch;
    double* part = (is_bwd && theta && dtheta) ? partials : nullptr;
    if (is_bwd && theta && dtheta && !partials) return hipErrorInvalidValue;
    hipError_t e = hipErrorInvalidValue;
#define LTN_PRO(d, bf, bw) \
    if (D == d && (is_bf16 != 0) == bf && (is_bwd != 0) == bw) \
        e = launch_t<d, bf, bw>(x, theta, dy, out, part, act, Bt, H, N, pos0, nchunks, stream)
    LTN_PRO(64, true, false); LTN_PRO(64, true, true); LTN_PRO(64, false, false); LTN_PRO(64, false, true);
    LTN_PRO(128, true, false); LTN_PRO(128, true, true); LTN_PRO(128, false, false); LTN_PRO(128, false, true);
#undef LTN_PRO
    if (e != hipSuccess) return e;
    if (part) {
        const int HD = H * D;
        hipLaunchKernelGGL(prologue_reduce_kernel, dim3((unsigned)((HD + 15) / 16)), dim3(256), 0, stream,
                           part, dtheta, nchunks, HD);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace ltn
