// The paper's own tiling of Lightning Attention (arXiv 2307.14995, App. B, Algorithm 3), as
// a second bf16 forward kernel for gfx950, kept for comparison with the state recurrence:
// for every block i of 64 queries, loop over ALL key/value blocks j <= i,
//
//     O_i = sum_{j <= i} ((Q_i K_j^T) (.) M_ij) V_j,     M_ij[r,c] = lambda^(64(i-j) + r - c)  (0 above the diagonal of j = i)
//
// with the mask generated on chip (the listing reads it from memory).  Cost grows with the
// square of the sequence length; nothing is carried between query blocks, so the grid is
// one workgroup per (chain, query block) and needs no sequential sweep.
//
// One workgroup = 256 threads = 4 waves; wave w owns query rows 16w..16w+15 of the block and,
// as in the pass kernels, forms the transposed scores P^T with 16x16x32 bf16 MFMA (their
// accumulator layout is the B operand of the next MFMA) and the transposed output
// O^T += V_j^T P^T.  K_j and V_j tiles stream global -> LDS directly through a two-stage
// ring (80 KB of LDS per workgroup: two workgroups per compute unit); the key blocks are
// walked from j = i downwards, so the block decay lambda^(64(i-j-1)) is a running product.
// Only non-negative powers of lambda are formed.
#include "ltn_bf16_tiles.h"

#include <type_traits>

namespace ltn {
namespace {

constexpr int kTiledThreads = 256;

template <int D, int W>
__device__ __forceinline__ void tiled_wave(const char* qp, const char* kp, const char* vp, char* op,
                                           long long N, int i, float lam, char* smem, unsigned lds0, int lane) {
    using F = Swz<D>;
    constexpr int KS = D / 32, NT = D / 16, RB = F::RB, FB = F::BYTES;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;

    // Decay of the transposed score entry (key 16kt + 4g + jx of block j, row 16W + i16 of
    // block i): lambda^(64(i-j) + 16(W-kt) + d0 - jx), d0 = i16 - 4g, split into non-negative
    // powers:  diagonal block, kt = W:  mdiag[jx] = lambda^(d0-jx) (0 above the diagonal)
    //          diagonal block, kt < W:  moff[jx] * lambda^(16(W-kt-1)),  moff[jx] = lambda^(16+d0-jx)
    //          j < i:                   moff[jx] * cblk[kt] * lambda^(64(i-j-1)),  cblk[kt] = lambda^(48+16(W-kt))
    const int d0 = i16 - 4 * g;
    float mdiag[4], moff[4], cblk[4];
#pragma unroll
    for (int jx = 0; jx < 4; ++jx) {
        mdiag[jx] = (d0 - jx >= 0) ? decay_pow(lam, d0 - jx) : 0.0f;
        moff[jx] = decay_pow(lam, 16 + d0 - jx);
    }
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) cblk[kt] = decay_pow(lam, 48 + 16 * (W - kt));
    const float lam16 = decay_pow(lam, 16), lam32 = decay_pow(lam, 32), lam64 = decay_pow(lam, 64);

    int row_off[KS], ctr[NT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) row_off[ks] = F::off(i16, 4 * ks + g);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int col = 16 * nt + 4 * (i16 & 3);
        ctr[nt] = F::off(4 * g + (i16 >> 2), col >> 3) + (col & 4) * 2;
    }

    TileDma<D> dma;
    dma.init(W, lane, ROW);
    auto valid_of = [&](int b) {
        const long long left = N - (long long)b * kBlock;
        return left < kBlock ? (int)left : kBlock;
    };
    auto fetch_kv = [&](int j, int stage) {
        const unsigned lds = lds0 + (unsigned)(FB + stage * 2 * FB);
        const long long o = (long long)j * kBlock * ROW;
        dma.issue(kp + o, lds, W, valid_of(j));
        dma.issue(vp + o, lds + FB, W, valid_of(j));
    };

    dma.issue(qp + (long long)i * kBlock * ROW, lds0, W, valid_of(i));
    fetch_kv(i, 0);
    wait_dma<0>();
    __syncthreads();

    Frag Af[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Af[ks].u = *(const u32x4*)(smem + (16 * W) * RB + row_off[ks]);
    f32x4 oi[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) oi[nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one key/value block: scores against key tiles 0..KT-1, masked, then O^T += V^T P^T
    auto block = [&](const char* ktile, const char* vtile, auto diag_tag, float f) {
        constexpr bool DIAG = decltype(diag_tag)::value;
        constexpr int KT = DIAG ? W + 1 : 4;         // the diagonal block is causal
        f32x4 sacc[KT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) sacc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                Frag a;
                a.u = *(const u32x4*)(ktile + (16 * kt) * RB + row_off[ks]);
                sacc[kt] = mfma16(a.v, Af[ks].v, sacc[kt]);
            }
        bf16x4 Pt[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            f32x4 m = f32x4{0.f, 0.f, 0.f, 0.f};
            if (kt < KT) {
                float sc;
                if (DIAG) sc = (kt == W) ? 1.0f : ((W - kt == 1) ? 1.0f : ((W - kt == 2) ? lam16 : lam32));
                else sc = cblk[kt] * f;
#pragma unroll
                for (int jx = 0; jx < 4; ++jx)
                    m[jx] = sacc[kt < KT ? kt : 0][jx] * ((DIAG && kt == W) ? mdiag[jx] : moff[jx] * sc);
            }
            Pt[kt] = to_bf16(m);
        }
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            if (2 * p < KT) {
                Frag b;
                b.b[0] = Pt[2 * p];
                b.b[1] = Pt[2 * p + 1];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    Frag vf;
                    vf.h[0] = lds_tr16(vtile + (32 * p) * RB + ctr[nt]);
                    vf.h[1] = lds_tr16(vtile + (32 * p + 16) * RB + ctr[nt]);
                    oi[nt] = mfma16(vf.v, b.v, oi[nt]);
                }
            }
        }
    };

    float f = 1.0f;                        // lambda^(64 (i - j - 1)) for j < i, a running product
    for (int jj = 0; jj <= i; ++jj) {
        const int stage = jj & 1;
        if (jj < i) fetch_kv(i - jj - 1, stage ^ 1);     // that stage was last read before the previous barrier
        const char* ktile = smem + FB + stage * 2 * FB;
        if (jj == 0) {
            block(ktile, ktile + FB, std::true_type{}, 1.0f);
        } else {
            block(ktile, ktile + FB, std::false_type{}, f);
            f *= lam64;
        }
        if (jj < i) {
            wait_dma<0>();
            __syncthreads();
        }
    }

    const bool row_ok = (16 * W + i16) < valid_of(i);
    store_strip<NT>(oi, op + ((long long)i * kBlock + 16 * W + i16) * ROW + (8 * g) * 2, row_ok);
}

template <int D>
__global__ __launch_bounds__(kTiledThreads)
void tiled_fwd_bf16_kernel(const char* __restrict__ q, const char* __restrict__ k, const char* __restrict__ v,
                           char* __restrict__ o, const float* __restrict__ decay, int chains, int H,
                           long long N, int T) {
    __shared__ __attribute__((aligned(1024))) char smem[5 * Swz<D>::BYTES];   // Q tile + 2 x {K, V}
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // query blocks with the most key blocks first; consecutive workgroups take different chains,
    // so a chain's workgroups share an XCD (and its L2) whenever chains is a multiple of 8
    const int slot = blockIdx.x;
    const int i = T - 1 - slot / chains;
    const int chain = slot % chains;
    const size_t off = (size_t)chain * (size_t)N * D * 2;
    const float lam = decay[chain % H];
    const unsigned lds0 = lds_address(smem);
    switch (wave) {
        case 0: tiled_wave<D, 0>(q + off, k + off, v + off, o + off, N, i, lam, smem, lds0, tid & 63); break;
        case 1: tiled_wave<D, 1>(q + off, k + off, v + off, o + off, N, i, lam, smem, lds0, tid & 63); break;
        case 2: tiled_wave<D, 2>(q + off, k + off, v + off, o + off, N, i, lam, smem, lds0, tid & 63); break;
        default: tiled_wave<D, 3>(q + off, k + off, v + off, o + off, N, i, lam, smem, lds0, tid & 63); break;
    }
}

}  // namespace

hipError_t launch_tiled_fwd_bf16(const void* q, const void* k, const void* v, void* o, const float* decay,
                                 int chains, int H, long long N, int D, hipStream_t stream) {
    const long long T = (N + kBlock - 1) / kBlock;
    const long long wgs = (long long)chains * T;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (D == 128)
        hipLaunchKernelGGL((tiled_fwd_bf16_kernel<128>), dim3((unsigned)wgs), dim3(kTiledThreads), 0, stream,
                           (const char*)q, (const char*)k, (const char*)v, (char*)o, decay, chains, H, N, (int)T);
    else if (D == 64)
        hipLaunchKernelGGL((tiled_fwd_bf16_kernel<64>), dim3((unsigned)wgs), dim3(kTiledThreads), 0, stream,
                           (const char*)q, (const char*)k, (const char*)v, (char*)o, decay, chains, H, N, (int)T);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ltn
