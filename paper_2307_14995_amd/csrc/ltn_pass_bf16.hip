// bf16 MFMA kernel for one decayed linear-attention pass on gfx950 (MI355X).
//
// What it computes (arXiv 2307.14995, Sec. 3.2.1 with the decay mask of Eq. 1;
// recurrence of Sec. 3.3, Algorithm 2, taken 64 tokens at a time): for each chain
// (batch, head) and a slice of DV value columns,
//
//   per block i of 64 tokens, with S_i the running [D x DV] state:
//     P    = (A_i B_i^T) (.) M,       M[r,c] = lambda^(r-c) for r >= c else 0
//     O_i  = P C_i + diag(lambda^(r+1)) A_i S_i
//     S_i+1 = lambda^len S_i + (diag(lambda^(len-1-c)) B_i)^T C_i
//
// (A,B,C) = (Q,K,V) gives the forward output; the gradient passes reuse the same
// kernel with permuted operands and, for dK/dV, a reversed token axis.
//
// Work split inside a 256-thread workgroup (4 wavefronts of 64 lanes):
//   * wave w owns the 16 query rows 16w..16w+15 of the block.  It forms the
//     transposed score tiles P^T[key tile][its rows] with 16x16x32 bf16 MFMA, so
//     the fp32 accumulators already sit in the lane layout the next MFMA wants as
//     its B operand: the masked scores never leave registers.
//   * the output is produced transposed (O^T = C^T P^T + S^T A^T) so every lane
//     holds four consecutive output features of one token -> 8-byte stores.
//   * wave w owns state rows [w*D/4, (w+1)*D/4) in fp32 accumulators for the whole
//     sequence; after each update it publishes a bf16 copy to LDS (double
//     buffered), which all waves read as the A operand of S^T A^T.
//   * B and C tiles are staged global -> registers -> LDS one block ahead (double
//     buffered, padded rows: conflict-free 16-byte reads); operands that must be
//     read "down the token axis" (C for P C, B^T and C for the state update) use
//     the LDS transpose read ds_read_b64_tr_b16.
//   * one workgroup barrier per block.
// Only non-negative powers of lambda are formed.
#include "ltn_kernels.h"

namespace ltn {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;

union Frag {          // one 16x16x32 MFMA operand: 8 bf16 per lane
    bf16x8 v;
    uint4 u;
    s16x4 h[2];
    bf16x4 b[2];
};

__device__ __forceinline__ s16x4 lds_tr16(const char* p) {
    // 16 lanes give the addresses of a 4 x 16 tile of 16-bit elements (lane s: row
    // s/4, columns 4(s%4)..+3); lane i receives column i of that tile, rows 0..3.
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(p));
}

__device__ __forceinline__ f32x4 mfma16(const bf16x8& a, const bf16x8& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x4 to_bf16(const f32x4& x) {
    return __builtin_convertvector(x, bf16x4);
}

constexpr int kBlock = 64;
constexpr int kThreads = 256;

template <int D, int DV>
struct Cfg {
    static constexpr int KS = D / 32;          // k-steps of a D-long contraction
    static constexpr int MT = D / 64;          // 16-row state tiles owned per wave
    static constexpr int NT = DV / 16;         // 16-column tiles of the value slice
    static constexpr int KP = D * 2 + 16;      // LDS row pitch of the B tile / state copy (bytes)
    static constexpr int VP = DV * 2 + 16;     // LDS row pitch of the C tile (bytes)
    static constexpr int KC = D / 32;          // 16-byte chunks of B staged per thread
    static constexpr int VC = (DV >= 32) ? DV / 32 : 1;
    static constexpr int KB = 0;                       // B tile, 2 buffers
    static constexpr int VB = 2 * kBlock * KP;         // C tile, 2 buffers
    static constexpr int SB = VB + 2 * kBlock * VP;    // bf16 state copy [DV][D], 2 buffers
    static constexpr int TOTAL = SB + 2 * DV * KP;
};

template <int D, int DV>
__global__ __launch_bounds__(kThreads, 1)
void pass_bf16_kernel(const PassBatch pb, const int nsplit) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, MT = C::MT, NT = C::NT, KP = C::KP, VP = C::VP;
    __shared__ __attribute__((aligned(16))) char smem[C::TOTAL];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;          // wave = query-row strip
    const int g = lane >> 4;         // 16-lane group
    const int i16 = lane & 15;

    int chain, within;
    map_workgroup(blockIdx.x, pb.count * nsplit, pb.chains, chain, within);
    const int pi = within / nsplit;
    const int split = within - pi * nsplit;
    const PassArgs P = pb.p[pi];
    const int rev = P.rev;
    const long long N = pb.N;
    const int T = (int)((N + kBlock - 1) / kBlock);
    const float lam = pb.decay[chain % pb.H];

    const size_t chain_off = (size_t)chain * (size_t)N * D * 2;
    const char* Ap = (const char*)P.a + chain_off;
    const char* Bp = (const char*)P.b + chain_off;
    const char* Cp = (const char*)P.c + chain_off + (size_t)split * DV * 2;
    char* Op = (char*)P.out + chain_off + (size_t)split * DV * 2;
    constexpr size_t ROW = (size_t)D * 2;

    // ---- per-lane decay constants (non-negative exponents only)
    const float qscale = decay_pow(lam, 16 * w + i16 + 1);     // lambda^(r+1), r = row in block
    const int d0 = i16 - 4 * g;                                 // (row - key) inside a diagonal tile, j = 0
    float mdiag[4], moff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        mdiag[j] = (d0 - j >= 0) ? decay_pow(lam, d0 - j) : 0.0f;
        moff[j] = decay_pow(lam, 16 + d0 - j);                  // 16 + d0 - j >= 1
    }
    const float lam16 = decay_pow(lam, 16), lam32 = decay_pow(lam, 32);
    float ksc[2][8];                                            // lambda^(len-1-token), token per MFMA k-slot
    float lamB;
    auto set_block_len = [&](int len) {
        lamB = decay_pow(lam, len);
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int tok = 32 * p + 16 * (j >> 2) + 4 * g + (j & 3);
                ksc[p][j] = (tok < len) ? decay_pow(lam, len - 1 - tok) : 0.0f;
            }
    };
    set_block_len(kBlock);

    // ---- state: wave w owns rows [dk0, dk0 + D/4) x all DV columns, fp32
    const int dk0 = w * (D / 4);
    f32x4 st[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (P.state_in) {
                const float* s = P.state_in + (size_t)chain * D * D + (size_t)split * DV;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    st[mt][nt][j] = s[(size_t)(dk0 + 16 * mt + 4 * g + j) * D + 16 * nt + i16];
            } else {
                st[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    auto publish_state = [&](int buf) {
        char* sb = smem + C::SB + buf * (DV * KP);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                *(bf16x4*)(sb + (16 * nt + i16) * KP + (dk0 + 16 * mt + 4 * g) * 2) = to_bf16(st[mt][nt]);
    };

    // ---- staging of the next block: global -> registers
    uint4 kst[C::KC], vst[C::VC];
    Frag Qf[KS], Qn[KS];
    auto grow = [&](long long t) -> size_t { return (size_t)(rev ? (N - 1 - t) : t); };
    auto load_block = [&](int blk) {
        const long long t0 = (long long)blk * kBlock;
#pragma unroll
        for (int c = 0; c < C::KC; ++c) {
            const int id = c * kThreads + tid;
            const int r = id / (D / 8), ch = id % (D / 8);
            const long long t = t0 + r;
            kst[c] = (t < N) ? *(const uint4*)(Bp + grow(t) * ROW + ch * 16) : uint4{0, 0, 0, 0};
        }
#pragma unroll
        for (int c = 0; c < C::VC; ++c) {
            const int id = c * kThreads + tid;
            const int r = id / (DV / 8), ch = id % (DV / 8);
            const long long t = t0 + r;
            const bool ok = (t < N) && (r < kBlock);
            vst[c] = ok ? *(const uint4*)(Cp + grow(t) * ROW + ch * 16) : uint4{0, 0, 0, 0};
        }
        const long long tq = t0 + 16 * w + i16;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            Qn[ks].u = (tq < N) ? *(const uint4*)(Ap + grow(tq) * ROW + (32 * ks + 8 * g) * 2)
                                : uint4{0, 0, 0, 0};
    };
    auto stage_to_lds = [&](int buf) {
        char* kb = smem + C::KB + buf * (kBlock * KP);
        char* vb = smem + C::VB + buf * (kBlock * VP);
#pragma unroll
        for (int c = 0; c < C::KC; ++c) {
            const int id = c * kThreads + tid;
            *(uint4*)(kb + (id / (D / 8)) * KP + (id % (D / 8)) * 16) = kst[c];
        }
#pragma unroll
        for (int c = 0; c < C::VC; ++c) {
            const int id = c * kThreads + tid;
            const int r = id / (DV / 8);
            if (r < kBlock) *(uint4*)(vb + r * VP + (id % (DV / 8)) * 16) = vst[c];
        }
    };

    // ---- prologue
    load_block(0);
    publish_state(0);
    stage_to_lds(0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) Qf[ks] = Qn[ks];
    __syncthreads();

    for (int blk = 0; blk < T; ++blk) {
        const int cur = blk & 1;
        const long long t0 = (long long)blk * kBlock;
        const char* kb = smem + C::KB + cur * (kBlock * KP);
        const char* vb = smem + C::VB + cur * (kBlock * VP);
        const char* sb = smem + C::SB + cur * (DV * KP);

        if (blk + 1 < T) load_block(blk + 1);          // in flight during this block's math
        const long long rem = N - t0;
        if (rem < kBlock) set_block_len((int)rem);      // short last block only

        // -- transposed masked scores P^T[key tile kt][own 16 rows], kept in registers
        bf16x4 Pt[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            if (kt <= w) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    Frag a;
                    a.u = *(const uint4*)(kb + (16 * kt + i16) * KP + (32 * ks + 8 * g) * 2);
                    acc = mfma16(a.v, Qf[ks].v, acc);
                }
                if (kt == w) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] *= mdiag[j];
                } else {
                    const int dlt = w - kt;             // 1..3, wave-uniform
                    const float s = (dlt == 1) ? 1.0f : ((dlt == 2) ? lam16 : lam32);
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[j] *= moff[j] * s;
                }
                Pt[kt] = to_bf16(acc);
            } else {
                Pt[kt] = bf16x4{0, 0, 0, 0};
            }
        }

        // -- C-tile operands read down the token axis (used by P C and by the state update)
        Frag Vf[2][NT];
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const char* a0 = vb + (32 * p + 4 * g + (i16 >> 2)) * VP + (16 * nt + 4 * (i16 & 3)) * 2;
                Vf[p][nt].h[0] = lds_tr16(a0);
                Vf[p][nt].h[1] = lds_tr16(a0 + 16 * VP);
            }

        // -- intra-block output (transposed): O^T += C^T P^T
        f32x4 oi[NT], oe[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            oi[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            oe[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            if (2 * p <= w) {
                Frag b;
                b.b[0] = Pt[2 * p];
                b.b[1] = Pt[2 * p + 1];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) oi[nt] = mfma16(Vf[p][nt].v, b.v, oi[nt]);
            }
        }

        // -- inter-block output: S^T A^T with the published bf16 state
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Frag a;
                a.u = *(const uint4*)(sb + (16 * nt + i16) * KP + (32 * ks + 8 * g) * 2);
                oe[nt] = mfma16(a.v, Qf[ks].v, oe[nt]);
            }

        // -- combine and store: lane holds token (16w + i16), features 16nt + 4g .. +3
        {
            const long long t = t0 + 16 * w + i16;
            if (t < N) {
                char* orow = Op + grow(t) * ROW + (4 * g) * 2;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    f32x4 r;
#pragma unroll
                    for (int j = 0; j < 4; ++j) r[j] = oi[nt][j] + qscale * oe[nt][j];
                    *(bf16x4*)(orow + 32 * nt) = to_bf16(r);
                }
            }
        }

        // -- state update: S <- lambda^len S + (decayed B)^T C
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) st[mt][nt][j] *= lamB;
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const char* a0 = kb + (32 * p + 4 * g + (i16 >> 2)) * KP + (dk0 + 16 * mt + 4 * (i16 & 3)) * 2;
                Frag a;
                a.h[0] = lds_tr16(a0);
                a.h[1] = lds_tr16(a0 + 16 * KP);
                f32x8 af = __builtin_convertvector(a.v, f32x8);
#pragma unroll
                for (int j = 0; j < 8; ++j) af[j] *= ksc[p][j];
                a.v = __builtin_convertvector(af, bf16x8);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) st[mt][nt] = mfma16(a.v, Vf[p][nt].v, st[mt][nt]);
            }

        // -- publish for the next block, then hand over the staged tiles
        if (blk + 1 < T) {
            publish_state(cur ^ 1);
            stage_to_lds(cur ^ 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) Qf[ks] = Qn[ks];
        }
        __syncthreads();
    }

    if (P.state_out) {
        float* s = P.state_out + (size_t)chain * D * D + (size_t)split * DV;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    s[(size_t)(dk0 + 16 * mt + 4 * g + j) * D + 16 * nt + i16] = st[mt][nt][j];
    }
}

template <int D, int DV>
hipError_t launch_t(const PassBatch& pb, hipStream_t stream) {
    const int nsplit = D / DV;
    const long long wgs = (long long)pb.chains * pb.count * nsplit;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pass_bf16_kernel<D, DV>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, pb, nsplit);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pass_bf16(const PassBatch& pb, int D, int dv, hipStream_t stream) {
    if (D == 128 && dv == 128) return launch_t<128, 128>(pb, stream);
    if (D == 128 && dv == 64) return launch_t<128, 64>(pb, stream);
    if (D == 128 && dv == 32) return launch_t<128, 32>(pb, stream);
    if (D == 64 && dv == 64) return launch_t<64, 64>(pb, stream);
    if (D == 64 && dv == 32) return launch_t<64, 32>(pb, stream);
    return hipErrorInvalidValue;
}

}  // namespace ltn
