// Gated SimpleRMSNorm on rows (arXiv 2307.14995, Sec. 3.1.2 Eq. 3: O = Norm(.) (.) U, with
// the SimpleRMSNorm of Sec. 3.1.3 taken per head over its D features):
//
//     y = x / sqrt(mean(x^2) + eps) (.) u
//
// and its derivative.  The forward of this map is normally fused into the attention
// forward (the gated epilogue of the pass kernels); these stand-alone kernels serve the
// backward (which needs the stored attention output x) and callers that hold x already.
// Streaming kernels, HBM-bound: every lane owns 16 bytes of one row, a row's lanes are
// neighbours in one wave and reduce with cross-lane shuffles (rows of 96 features take 16 or 32
// lanes of which 12 or 24 hold data); fp32 arithmetic.
#include "ltn_kernels.h"

namespace ltn {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;

template <bool BF16> struct Vec;            // the 16 bytes of one lane as fp32 values
template <> struct Vec<true> {
    static constexpr int N = 8;
    float v[8];
    __device__ __forceinline__ void load(const void* p) {
        union { u32x4 u; bf16x8 h; } c;
        c.u = *(const u32x4*)p;
        const f32x8 f = __builtin_convertvector(c.h, f32x8);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = f[i];
    }
    __device__ __forceinline__ void store(void* p) const {
        f32x8 f;
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = v[i];
        union { u32x4 u; bf16x8 h; } c;
        c.h = __builtin_convertvector(f, bf16x8);
        *(u32x4*)p = c.u;
    }
};
template <> struct Vec<false> {
    static constexpr int N = 4;
    float v[4];
    __device__ __forceinline__ void load(const void* p) {
        const float4 f = *(const float4*)p;
        v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
    }
    __device__ __forceinline__ void store(void* p) const { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }
};

template <int LPR>
__device__ __forceinline__ float row_sum(float x) {   // sum over the LPR neighbouring lanes of a row
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
    return x;
}

constexpr int kThreads = 256;

template <int D, bool BF16, bool BWD>
__global__ __launch_bounds__(kThreads)
void gate_kernel(const char* __restrict__ x, const char* __restrict__ u, const char* __restrict__ dy,
                 char* __restrict__ o0, char* __restrict__ o1, float eps, long long rows) {
    using V = Vec<BF16>;
    constexpr int ACT = D / V::N;                 // lanes that hold a piece of the row
    constexpr int LPR = ACT <= 8 ? 8 : (ACT <= 16 ? 16 : (ACT <= 32 ? 32 : 64));   // lanes given to a row (96 features: 12 of 16, 24 of 32)
    constexpr int RPW = kThreads / LPR;           // rows per workgroup step
    static_assert(D % V::N == 0 && ACT <= 64, "a row's lanes sit in one wave");
    const int sub = threadIdx.x % LPR;
    const bool live = sub < ACT;                  // idle lanes of a row contribute zeros and store nothing
    long long r = (long long)blockIdx.x * RPW + threadIdx.x / LPR;
    const long long stride = (long long)gridDim.x * RPW;
    // every lane of a wave runs the same number of steps (the shuffles need all of a
    // row's lanes); rows past the end are skipped as whole rows
    for (; r < rows; r += stride) {
        const size_t off = ((size_t)r * ACT + (live ? sub : 0)) * 16;
        V xv, uv;
        xv.load(x + off);
        uv.load(u + off);
        if (!live) {
#pragma unroll
            for (int i = 0; i < V::N; ++i) xv.v[i] = 0.f;
        }
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < V::N; ++i) ss = fmaf(xv.v[i], xv.v[i], ss);
        if constexpr (!BWD) {
            ss = row_sum<LPR>(ss);
            const float rstd = 1.0f / sqrtf(ss * (1.0f / D) + eps);
            V yv;
#pragma unroll
            for (int i = 0; i < V::N; ++i) yv.v[i] = xv.v[i] * rstd * uv.v[i];
            if (live) yv.store(o0 + off);
        } else {
            V gv;
            gv.load(dy + off);
            float dot = 0.f;
#pragma unroll
            for (int i = 0; i < V::N; ++i) dot = fmaf(gv.v[i] * uv.v[i], xv.v[i], dot);
            ss = row_sum<LPR>(ss);
            dot = row_sum<LPR>(dot);
            const float rstd = 1.0f / sqrtf(ss * (1.0f / D) + eps);
            const float mean = dot * rstd * (1.0f / D);       // mean of (dy u) (.) (x rstd)
            V dx, du;
#pragma unroll
            for (int i = 0; i < V::N; ++i) {
                const float n = xv.v[i] * rstd;
                du.v[i] = gv.v[i] * n;
                dx.v[i] = (gv.v[i] * uv.v[i] - n * mean) * rstd;
            }
            if (live) {
                dx.store(o0 + off);
                du.store(o1 + off);
            }
        }
    }
}

template <int D, bool BF16, bool BWD>
hipError_t launch_gate_t(const void* x, const void* u, const void* dy, void* o0, void* o1, float eps,
                         long long rows, hipStream_t stream) {
    constexpr int ACT = D / Vec<BF16>::N;
    constexpr int RPW = kThreads / (ACT <= 8 ? 8 : (ACT <= 16 ? 16 : (ACT <= 32 ? 32 : 64)));
    long long wgs = (rows + RPW - 1) / RPW;
    if (wgs > 256 * 16) wgs = 256 * 16;           // grid-stride beyond 16 workgroups per compute unit
    if (wgs <= 0) return hipSuccess;
    hipLaunchKernelGGL((gate_kernel<D, BF16, BWD>), dim3((unsigned)wgs), dim3(kThreads), 0, stream,
                       (const char*)x, (const char*)u, (const char*)dy, (char*)o0, (char*)o1, eps, rows);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gate(const void* x, const void* u, const void* dy, void* o0, void* o1, float eps,
                       long long rows, int D, int is_bf16, int is_bwd, hipStream_t stream) {
#define LTN_GATE_CASE(d, b, w) \
    if (D == d && (is_bf16 != 0) == b && (is_bwd != 0) == w) return launch_gate_t<d, b, w>(x, u, dy, o0, o1, eps, rows, stream)
    LTN_GATE_CASE(128, true, false); LTN_GATE_CASE(128, true, true);
    LTN_GATE_CASE(128, false, false); LTN_GATE_CASE(128, false, true);
    LTN_GATE_CASE(64, true, false); LTN_GATE_CASE(64, true, true);
    LTN_GATE_CASE(64, false, false); LTN_GATE_CASE(64, false, true);
    LTN_GATE_CASE(96, true, false); LTN_GATE_CASE(96, true, true);
    LTN_GATE_CASE(96, false, false); LTN_GATE_CASE(96, false, true);
    LTN_GATE_CASE(256, true, false); LTN_GATE_CASE(256, true, true);
    LTN_GATE_CASE(256, false, false); LTN_GATE_CASE(256, false, true);
#undef LTN_GATE_CASE
    return hipErrorInvalidValue;
}

}  // namespace ltn
