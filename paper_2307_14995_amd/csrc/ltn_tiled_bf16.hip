// The paper's own tiling of Lightning Attention (arXiv 2307.14995, App. B, Algorithms 3 and
// 4), as bf16 comparison kernels for gfx950 next to the state recurrence.
//
// Forward (Algorithm 3): for every block i of 64 queries, loop over ALL key/value blocks
// j <= i,
//
//     O_i = sum_{j <= i} ((Q_i K_j^T) (.) M_ij) V_j,     M_ij[r,c] = lambda^(64(i-j) + r - c)  (0 above the diagonal of j = i)
//
// with the mask generated on chip (the listing reads it from memory).
//
// Backward (Algorithm 4, read with its misprints corrected: dK_j accumulates dA_ij^T Q_i and
// dQ_i accumulates dA_ij K_j): with A_ij = (Q_i K_j^T) (.) M_ij and dA_ij = (dO_i V_j^T) (.) M_ij,
//
//     dV_j = sum_{i >= j} A_ij^T dO_i,    dK_j = sum_{i >= j} dA_ij^T Q_i,    dQ_i = sum_{j <= i} dA_ij K_j.
//
// The listing keeps K_j, V_j on chip in its outer loop, walks i in the inner loop and adds
// into dQ_i in memory.  Here one workgroup per key/value block j does exactly that for dK_j
// and dV_j (both accumulated on chip over the inner loop, Q_i and dO_i tiles fetched once for
// the two of them); dQ_i is produced by a second kind of workgroup, one per query block i
// looping over j <= i, which forms dA_ij again instead of a read-modify-write of dQ in memory
// (no atomics, results reproducible).  Both kinds run in one launch.
//
// All of these are one tile loop: "own" rows X (16 per wave, fragments in registers) against
// streamed tile pairs (Y_j, Z_j),
//
//     out[own rows] = sum_j ((X Y_j^T) (.) M) Z_j,
//
// forward: (X, Y, Z) = (Q, K, V); dQ: (dO, V, K); and on the reversed token axis (row
// N-1-t, which turns "i >= j" into "j <= i" with the same mask) dV: (K, Q, dO), dK: (V, dO, Q).
//
// One workgroup = 256 threads = 4 waves; wave w owns rows 16w..16w+15 of its block and, as
// in the pass kernels, forms the transposed scores P^T with 16x16x32 bf16 MFMA (their
// accumulator layout is the B operand of the next MFMA) and the transposed output
// out^T += Z_j^T P^T.  The streamed tiles go global -> LDS directly through a two-stage ring
// (80 KB of LDS per workgroup: two workgroups per compute unit); the streamed blocks are
// walked from the diagonal block outwards, so the block decay lambda^(64(i-j-1)) is a running
// product.  Cost grows with the square of the sequence length.  Only non-negative powers of
// lambda are formed.
#include "ltn_bf16_tiles.h"

#include <type_traits>

namespace ltn {
namespace {

constexpr int kTiledThreads = 256;

// What one workgroup computes.  NOUT = 1: out0 = sum_j ((own0 Y^T)(.)M) Z.  NOUT = 2 (the
// fused dK_j / dV_j workgroup): additionally out1 = sum_j ((own1 Z^T)(.)M) Y -- the same
// streamed tiles with their roles swapped.
struct TiledJob {
    const char* own[2];
    const char* y;
    const char* z;
    char* out[2];
    long long N;
    int i;                // block index along the (possibly reversed) token axis
    int rev;              // 1: tile row r of block b is tensor row N-1-(64b+r)
    float lam;
};

template <int D, int W, int NOUT>
__device__ __forceinline__ void tiled_wave(const TiledJob& job, char* smem, unsigned lds0, int lane) {
    using F = Swz<D>;
    constexpr int KS = D / 32, NT = D / 16, RB = F::RB, FB = F::BYTES;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    const int i = job.i;
    const long long N = job.N;
    const float lam = job.lam;

    // Decay of the transposed score entry (streamed row 16kt + 4g + jx of block j, own row
    // 16W + i16 of block i): lambda^(64(i-j) + 16(W-kt) + d0 - jx), d0 = i16 - 4g, split into
    // non-negative powers:
    //   diagonal block, kt = W:  mdiag[jx] = lambda^(d0-jx) (0 above the diagonal)
    //   diagonal block, kt < W:  moff[jx] * lambda^(16(W-kt-1)),  moff[jx] = lambda^(16+d0-jx)
    //   j < i:                   moff[jx] * cblk[kt] * lambda^(64(i-j-1)),  cblk[kt] = lambda^(48+16(W-kt))
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

    // tile row r of block b is tensor row 64b + r (or N-1-64b-r): a base address per block and
    // a signed row stride
    const long long rs = job.rev ? -ROW : ROW;
    const long long row0 = job.rev ? (N - 1) * ROW : 0;
    TileDma<D> dma;
    dma.init(W, lane, rs);
    auto valid_of = [&](int b) {
        const long long left = N - (long long)b * kBlock;
        return left < kBlock ? (int)left : kBlock;
    };
    auto block_base = [&](const char* p, int b) { return p + row0 + (long long)b * kBlock * rs; };
    auto fetch_yz = [&](int j, int stage) {
        const unsigned lds = lds0 + (unsigned)(FB + stage * 2 * FB);
        dma.issue(block_base(job.y, j), lds, W, valid_of(j));
        dma.issue(block_base(job.z, j), lds + FB, W, valid_of(j));
    };

    // own rows: through LDS slot 0 into registers, one operand after the other
    Frag Af[NOUT][KS];
    dma.issue(block_base(job.own[0], i), lds0, W, valid_of(i));
    fetch_yz(i, 0);
    wait_dma<0>();
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Af[0][ks].u = *(const u32x4*)(smem + (16 * W) * RB + row_off[ks]);
    if constexpr (NOUT == 2) {
        __syncthreads();                   // every wave has read its rows of the first operand
        dma.issue(block_base(job.own[1], i), lds0, W, valid_of(i));
        wait_dma<0>();
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) Af[1][ks].u = *(const u32x4*)(smem + (16 * W) * RB + row_off[ks]);
    }

    f32x4 acc[NOUT][NT];
#pragma unroll
    for (int o = 0; o < NOUT; ++o)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[o][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one streamed block: scores of the own rows against tile rows 0..KT-1 (x 16), masked, then
    // out^T += ztile^T P^T
    auto block = [&](const char* ytile, const char* ztile, const Frag (&af)[KS], f32x4 (&oi)[NT], auto diag_tag,
                     float f) {
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
                a.u = *(const u32x4*)(ytile + (16 * kt) * RB + row_off[ks]);
                sacc[kt] = mfma16(a.v, af[ks].v, sacc[kt]);
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
                    vf.h[0] = lds_tr16(ztile + (32 * p) * RB + ctr[nt]);
                    vf.h[1] = lds_tr16(ztile + (32 * p + 16) * RB + ctr[nt]);
                    oi[nt] = mfma16(vf.v, b.v, oi[nt]);
                }
            }
        }
    };

    float f = 1.0f;                        // lambda^(64 (i - j - 1)) for j < i, a running product
    for (int jj = 0; jj <= i; ++jj) {
        const int stage = jj & 1;
        if (jj < i) fetch_yz(i - jj - 1, stage ^ 1);     // that stage was last read before the previous barrier
        const char* ytile = smem + FB + stage * 2 * FB;
        const char* ztile = ytile + FB;
        if (jj == 0) {
            block(ytile, ztile, Af[0], acc[0], std::true_type{}, 1.0f);
            if constexpr (NOUT == 2) block(ztile, ytile, Af[1], acc[1], std::true_type{}, 1.0f);
        } else {
            block(ytile, ztile, Af[0], acc[0], std::false_type{}, f);
            if constexpr (NOUT == 2) block(ztile, ytile, Af[1], acc[1], std::false_type{}, f);
            f *= lam64;
        }
        if (jj < i) {
            wait_dma<0>();
            __syncthreads();
        }
    }

    const bool row_ok = (16 * W + i16) < valid_of(i);
    const long long r = (long long)i * kBlock + 16 * W + i16;
    const long long out_off = (job.rev ? N - 1 - r : r) * ROW + (8 * g) * 2;
#pragma unroll
    for (int o = 0; o < NOUT; ++o) store_strip<NT>(acc[o], job.out[o] + out_off, row_ok);
}

template <int D, int NOUT>
__device__ __forceinline__ void tiled_workgroup(const TiledJob& job, char* smem) {
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned lds0 = lds_address(smem);
    switch (wave) {
        case 0: tiled_wave<D, 0, NOUT>(job, smem, lds0, tid & 63); break;
        case 1: tiled_wave<D, 1, NOUT>(job, smem, lds0, tid & 63); break;
        case 2: tiled_wave<D, 2, NOUT>(job, smem, lds0, tid & 63); break;
        default: tiled_wave<D, 3, NOUT>(job, smem, lds0, tid & 63); break;
    }
}

template <int D>
__global__ __launch_bounds__(kTiledThreads)
void tiled_fwd_bf16_kernel(const char* __restrict__ q, const char* __restrict__ k, const char* __restrict__ v,
                           char* __restrict__ o, const float* __restrict__ decay, int chains, int H,
                           long long N, int T) {
    __shared__ __attribute__((aligned(1024))) char smem[5 * Swz<D>::BYTES];   // own tile + 2 x {Y, Z}
    // query blocks with the most key blocks first; consecutive workgroups take different chains,
    // so a chain's workgroups share an XCD (and its L2) whenever chains is a multiple of 8
    const int slot = blockIdx.x;
    const int chain = slot % chains;
    const size_t off = (size_t)chain * (size_t)N * D * 2;
    TiledJob job;
    job.own[0] = q + off; job.own[1] = nullptr;
    job.y = k + off; job.z = v + off;
    job.out[0] = o + off; job.out[1] = nullptr;
    job.N = N;
    job.i = T - 1 - slot / chains;
    job.rev = 0;
    job.lam = decay[chain % H];
    tiled_workgroup<D, 1>(job, smem);
}

// Algorithm 4.  Workgroups [0, chains*T): key/value block j = one block of the reversed token
// axis, dK_j and dV_j together (twice the tile work of the other kind, so they come first);
// workgroups [chains*T, 2*chains*T): query block i, dQ_i.  Within a kind, blocks with the
// longest inner loop first.
template <int D>
__global__ __launch_bounds__(kTiledThreads)
void tiled_bwd_bf16_kernel(const char* __restrict__ q, const char* __restrict__ k, const char* __restrict__ v,
                           const char* __restrict__ d_o, char* __restrict__ dq, char* __restrict__ dk,
                           char* __restrict__ dv, const float* __restrict__ decay, int chains, int H,
                           long long N, int T) {
    __shared__ __attribute__((aligned(1024))) char smem[5 * Swz<D>::BYTES];
    const int per_kind = chains * T;
    const int kind = blockIdx.x >= per_kind;
    const int slot = blockIdx.x - kind * per_kind;
    const int chain = slot % chains;
    const size_t off = (size_t)chain * (size_t)N * D * 2;
    TiledJob job;
    job.N = N;
    job.i = T - 1 - slot / chains;
    job.lam = decay[chain % H];
    if (kind == 0) {
        // reversed axis: dV = sum ((K Q^T)(.)M) dO,  dK = sum ((V dO^T)(.)M) Q
        job.own[0] = k + off; job.own[1] = v + off;
        job.y = q + off; job.z = d_o + off;
        job.out[0] = dv + off; job.out[1] = dk + off;
        job.rev = 1;
        tiled_workgroup<D, 2>(job, smem);
    } else {
        // dQ = sum ((dO V^T)(.)M) K
        job.own[0] = d_o + off; job.own[1] = nullptr;
        job.y = v + off; job.z = k + off;
        job.out[0] = dq + off; job.out[1] = nullptr;
        job.rev = 0;
        tiled_workgroup<D, 1>(job, smem);
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

hipError_t launch_tiled_bwd_bf16(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk,
                                 void* dv, const float* decay, int chains, int H, long long N, int D,
                                 hipStream_t stream) {
    const long long T = (N + kBlock - 1) / kBlock;
    const long long wgs = 2 * (long long)chains * T;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (D == 128)
        hipLaunchKernelGGL((tiled_bwd_bf16_kernel<128>), dim3((unsigned)wgs), dim3(kTiledThreads), 0, stream,
                           (const char*)q, (const char*)k, (const char*)v, (const char*)d_o, (char*)dq, (char*)dk,
                           (char*)dv, decay, chains, H, N, (int)T);
    else if (D == 64)
        hipLaunchKernelGGL((tiled_bwd_bf16_kernel<64>), dim3((unsigned)wgs), dim3(kTiledThreads), 0, stream,
                           (const char*)q, (const char*)k, (const char*)v, (const char*)d_o, (char*)dq, (char*)dk,
                           (char*)dv, decay, chains, H, N, (int)T);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ltn
