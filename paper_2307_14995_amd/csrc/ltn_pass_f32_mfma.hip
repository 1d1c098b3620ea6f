// fp32 MFMA kernel for one decayed linear-attention pass on gfx950: the same block recurrence
// as the bf16 kernel (arXiv 2307.14995, Sec. 3.2.1 / Eq. 1; Sec. 3.3 Algorithm 2 in block
// form), every product on the matrix cores in full fp32 (v_mfma_f32_16x16x4_f32: fp32
// operands, fp32 accumulation -- no reduced-precision step anywhere):
//
//   P    = (A_i B_i^T) (.) M,       M[r,c] = lambda^(r-c) for r >= c else 0
//   O_i  = P C_i + diag(lambda^(r+1)) A_i S_i
//   S_i+1 = lambda^len S_i + sum_c lambda^(len-1-c) b_c^T c_c
//
// One 512-thread workgroup (8 waves, two per SIMD, in two roles so that one role's LDS waits
// hide under the other's MFMAs) per (chain, pass, slice of DV value columns), blocks of B tokens.
//   * Output waves 0..3: wave w owns the token strip (w mod B/16) and a group of value-column tiles.
//     It forms the transposed scores P^T[keys][its 16 tokens]; their accumulator layout (lane
//     holds keys 4g..4g+3 of a token) is the B operand of the next product with the
//     contraction index permuted (k-slot g of step j <-> key 4g + j), so the masked scores stay
//     in registers, and the output comes out transposed: a lane ends up with four consecutive
//     output features of one token = one 16-byte store.
//   * Operands whose contraction index is contiguous in LDS (feature index of the A and B
//     tiles, key-feature index of the transposed state copy) are read 16 bytes per lane, one
//     read feeding four MFMAs; operands contracted over the token index (C in P C, B and C in
//     the state update) are read 4 bytes per lane.  Row pitches are 4 floats more than a
//     multiple of 64, which makes both kinds of read conflict-free.
//   * State waves 4..7: wave 4 + u owns state rows [u D/4, (u+1) D/4) x DV in accumulators for
//     the whole sequence; once per block the new state goes to LDS transposed ([dv][dk], 16-byte
//     writes) for the next block's A_i S_i.
//   * The next block's tiles are fetched into registers by the output waves (the state waves'
//     work is the longer one between two barriers) while the current block is computed, and
//     written to LDS between two barriers at the end of the block.
// Only non-negative powers of lambda are formed.
#include "ltn_kernels.h"

namespace ltn {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kMThreads = 512;

__device__ __forceinline__ v4f mfma4(float a, float b, v4f c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

template <int D, int DV, int B>
struct FCfg {
    static constexpr int TS = B / 16;              // token strips of a block
    static constexpr int VG = 4 / TS;              // value-column groups the 4 waves split into
    static constexpr int NT = DV / 16;             // 16-column tiles of the slice
    static constexpr int NTW = NT / VG;            // ... per wave in the output part
    static constexpr int MT = D / 64;              // 16-row state tiles per wave
    static constexpr int KC = D / 16;              // 16-feature chunks of a D-long contraction
    static constexpr int PA = D + 4;               // row pitch (floats) of the A and B tiles and of the state copy
    static constexpr int PC = DV + 4;              // row pitch of the C tile
    static constexpr int A_OFF = 0, B_OFF = B * PA, C_OFF = 2 * B * PA, S_OFF = C_OFF + B * PC, PW_OFF = S_OFF + DV * PA;
    static constexpr int FLOATS = PW_OFF + B + 4;
    static_assert(B == 16 || B == 32 || B == 64, "block lengths");
    static_assert(D == 64 || D == 128, "head dims of this kernel");
    static_assert(NT % VG == 0 && NTW >= 1, "every wave needs a value-column tile");
    static_assert(FLOATS * 4 <= 163840, "LDS per workgroup");
    // prefetch registers of the output waves (they fetch the tiles; the state waves' work is the
    // longer one between two barriers): 16-byte pieces per thread and tile (the last round of a
    // tile may be partial)
    static constexpr int FT = kMThreads / 2;       // threads of waves 0..3
    static constexpr int EA = B * (D / 4), EC = B * (DV / 4);
    static constexpr int LA = (EA + FT - 1) / FT, LC = (EC + FT - 1) / FT;
};

// The whole pass as one wave runs it; STRIP (the wave's token strip in the output part) is a
// compile-time constant, so causal tile skipping and the choice of decay constants cost no
// branches or indexed register reads inside a block.
template <int D, int DV, int B, int STRIP, bool STATE>
__device__ __forceinline__ void pass_f32_mfma_wave(const PassBatch& pb, const int nsplit, float* smem, const int wave) {
    using C = FCfg<D, DV, B>;
    constexpr int TS = C::TS, NT = C::NT, NTW = C::NTW, MT = C::MT, KC = C::KC, PA = C::PA, PC = C::PC;
    constexpr int strip = STRIP;
    float* As = smem + C::A_OFF;
    float* Bs = smem + C::B_OFF;
    float* Cs = smem + C::C_OFF;
    float* St = smem + C::S_OFF;          // transposed state copy [dv][dk]
    float* pw = smem + C::PW_OFF;         // lambda^0 .. lambda^B

    const int tid = threadIdx.x;
    const int lane = tid & 63, g = lane >> 4, i16 = lane & 15;
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
    float* Op = (float*)P.out + chain_off + (size_t)split * DV;
    const float* sin_p = P.state_in ? P.state_in + (size_t)chain * D * D + (size_t)split * DV : nullptr;
    float* sout_p = P.state_out ? P.state_out + (size_t)chain * D * D + (size_t)split * DV : nullptr;

    for (int n = tid; n <= B; n += kMThreads) pw[n] = decay_pow(lam, n);

    // output waves: value-column tiles of this wave (its strip is STRIP)
    const int vg = wave / TS;
    const int nt0 = vg * NTW;
    // state waves: rows dkb .. dkb + D/4 of the state
    const int dkb = (wave & 3) * (D / 4);

    // running state, fp32 accumulators: S[dkb + 16mt + 4g + j][16nt + i16]
    v4f st[STATE ? MT : 1][STATE ? NT : 1];
    if constexpr (STATE) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    st[mt][nt][j] = sin_p ? sin_p[(size_t)(dkb + 16 * mt + 4 * g + j) * D + 16 * nt + i16] : 0.0f;
    }

    auto publish_state = [&]() {
        if constexpr (STATE) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    *(v4f*)&St[(16 * nt + i16) * PA + dkb + 16 * mt + 4 * g] = st[mt][nt];
        }
    };

    // tile prefetch through registers (output waves: tid < FT)
    v4f ra[STATE ? 1 : C::LA], rb[STATE ? 1 : C::LA], rc[STATE ? 1 : C::LC];
    auto fetch = [&](long long t0) {
        if constexpr (STATE) return;
        const long long left = N - t0;
#pragma unroll
        for (int i = 0; i < (STATE ? 0 : C::LA); ++i) {
            const int e = tid + i * C::FT, r = e / (D / 4), c4 = e % (D / 4);
            const bool ok = e < C::EA && r < left;
            const size_t gr = (size_t)(rev ? (N - 1 - (t0 + r)) : (t0 + r));
            ra[i] = ok ? *(const v4f*)(Ap + gr * D + 4 * c4) : v4f{0.f, 0.f, 0.f, 0.f};
            rb[i] = ok ? *(const v4f*)(Bp + gr * D + 4 * c4) : v4f{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < (STATE ? 0 : C::LC); ++i) {
            const int e = tid + i * C::FT, r = e / (DV / 4), c4 = e % (DV / 4);
            const bool ok = e < C::EC && r < left;
            const size_t gr = (size_t)(rev ? (N - 1 - (t0 + r)) : (t0 + r));
            rc[i] = ok ? *(const v4f*)(Cp + gr * D + 4 * c4) : v4f{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto commit = [&]() {
        if constexpr (STATE) return;
#pragma unroll
        for (int i = 0; i < (STATE ? 0 : C::LA); ++i) {
            const int e = tid + i * C::FT, r = e / (D / 4), c4 = e % (D / 4);
            if (e < C::EA) {
                *(v4f*)&As[r * PA + 4 * c4] = ra[i];
                *(v4f*)&Bs[r * PA + 4 * c4] = rb[i];
            }
        }
#pragma unroll
        for (int i = 0; i < (STATE ? 0 : C::LC); ++i) {
            const int e = tid + i * C::FT, r = e / (DV / 4), c4 = e % (DV / 4);
            if (e < C::EC) *(v4f*)&Cs[r * PC + 4 * c4] = rc[i];
        }
    };

    fetch(0);
    commit();
    publish_state();
    __syncthreads();

    // decay constants of this lane's score entries: key 16kt + 4g + j against token 16 strip + i16
    float mdiag[4], moff[STRIP > 0 ? STRIP : 1][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int e = i16 - 4 * g - j;
        mdiag[j] = e >= 0 ? pw[e] : 0.0f;
#pragma unroll
        for (int d = 1; d <= STRIP; ++d) moff[d - 1][j] = pw[16 * d + e];  // 16 d + e >= 1
    }
    const float qscale = pw[16 * strip + i16 + 1];

    for (long long t0 = 0; t0 < N; t0 += B) {
        const int len = (N - t0 < B) ? (int)(N - t0) : B;
        const bool more = t0 + B < N;
        if (more) fetch(t0 + B);

        // ------------------------------------------------ output waves
        if constexpr (!STATE) {
            v4f af[KC];
#pragma unroll
            for (int c = 0; c < KC; ++c) af[c] = *(const v4f*)&As[(16 * strip + i16) * PA + 16 * c + 4 * g];

            v4f pt[STRIP + 1];           // masked P^T tiles kt <= strip
#pragma unroll
            for (int kt = 0; kt <= STRIP; ++kt) pt[kt] = v4f{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int kt = 0; kt <= STRIP; ++kt) {
                    const v4f b4 = *(const v4f*)&Bs[(16 * kt + i16) * PA + 16 * c + 4 * g];
#pragma unroll
                    for (int j = 0; j < 4; ++j) pt[kt] = mfma4(b4[j], af[c][j], pt[kt]);
                }
#pragma unroll
            for (int kt = 0; kt <= STRIP; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j) pt[kt][j] *= (kt == STRIP) ? mdiag[j] : moff[kt < STRIP ? STRIP - kt - 1 : 0][j];

            v4f oi[NTW], oe[NTW];
#pragma unroll
            for (int n = 0; n < NTW; ++n) {
                oi[n] = v4f{0.f, 0.f, 0.f, 0.f};
                oe[n] = v4f{0.f, 0.f, 0.f, 0.f};
            }
            // intra-block part: C^T P^T (contraction over the keys of tiles kt <= strip)
#pragma unroll
            for (int kt = 0; kt <= STRIP; ++kt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int n = 0; n < NTW; ++n)
                        oi[n] = mfma4(Cs[(16 * kt + 4 * g + j) * PC + 16 * (nt0 + n) + i16], pt[kt][j], oi[n]);
            // inter-block part: S^T A^T with the state copy of the block's start
#pragma unroll
            for (int c = 0; c < KC; ++c)
#pragma unroll
                for (int n = 0; n < NTW; ++n) {
                    const v4f s4 = *(const v4f*)&St[(16 * (nt0 + n) + i16) * PA + 16 * c + 4 * g];
#pragma unroll
                    for (int j = 0; j < 4; ++j) oe[n] = mfma4(s4[j], af[c][j], oe[n]);
                }
            // the lane holds features 16 nt + 4g .. +3 of token 16 strip + i16
            const int r = 16 * strip + i16;
            if (r < len) {
                const size_t gr = (size_t)(rev ? (N - 1 - (t0 + r)) : (t0 + r));
#pragma unroll
                for (int n = 0; n < NTW; ++n) {
                    v4f o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] = fmaf(qscale, oe[n][j], oi[n][j]);
                    *(v4f*)(Op + gr * D + 16 * (nt0 + n) + 4 * g) = o;
                }
            }
        }

        // ------------------------------------------------ state waves
        if constexpr (STATE) if (more || sout_p) {
            const float lam_len = pw[len];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int j = 0; j < 4; ++j) st[mt][nt][j] *= lam_len;
#pragma unroll
            for (int q = 0; q < TS; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int key = 16 * q + 4 * g + j;
                    const float w = key < len ? pw[len - 1 - key] : 0.0f;
                    float bv[MT], cv[NT];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) bv[mt] = Bs[key * PA + dkb + 16 * mt + i16] * w;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) cv[nt] = Cs[key * PC + 16 * nt + i16];
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) st[mt][nt] = mfma4(bv[mt], cv[nt], st[mt][nt]);
                }
        }

        if (more) {
            __syncthreads();             // every wave is done with this block's tiles and state copy
            commit();
            publish_state();
            __syncthreads();
        }
    }

    if constexpr (STATE) if (sout_p) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    sout_p[(size_t)(dkb + 16 * mt + 4 * g + j) * D + 16 * nt + i16] = st[mt][nt][j];
    }
}

template <int D, int DV, int B>
__global__ __launch_bounds__(kMThreads)
void pass_f32_mfma_kernel(const PassBatch pb, const int nsplit) {
    using C = FCfg<D, DV, B>;
    __shared__ __attribute__((aligned(16))) float smem[C::FLOATS];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the dispatch is a uniform branch
    if (wave >= 4) {
        pass_f32_mfma_wave<D, DV, B, 0, true>(pb, nsplit, smem, wave);
        return;
    }
    const int strip = wave % C::TS;
    if constexpr (C::TS == 1) {
        pass_f32_mfma_wave<D, DV, B, 0, false>(pb, nsplit, smem, wave);
    } else if constexpr (C::TS == 2) {
        if (strip == 0) pass_f32_mfma_wave<D, DV, B, 0, false>(pb, nsplit, smem, wave);
        else pass_f32_mfma_wave<D, DV, B, 1, false>(pb, nsplit, smem, wave);
    } else {
        switch (strip) {
            case 0: pass_f32_mfma_wave<D, DV, B, 0, false>(pb, nsplit, smem, wave); break;
            case 1: pass_f32_mfma_wave<D, DV, B, 1, false>(pb, nsplit, smem, wave); break;
            case 2: pass_f32_mfma_wave<D, DV, B, 2, false>(pb, nsplit, smem, wave); break;
            default: pass_f32_mfma_wave<D, DV, B, 3, false>(pb, nsplit, smem, wave); break;
        }
    }
}

template <int D, int DV, int B>
hipError_t launch_m(const PassBatch& pb, hipStream_t stream) {
    const int nsplit = D / DV;
    const long long wgs = (long long)pb.chains * pb.count * nsplit;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pass_f32_mfma_kernel<D, DV, B>), dim3((unsigned)wgs), dim3(kMThreads), 0, stream, pb, nsplit);
    return hipGetLastError();
}

}  // namespace

bool pass_f32_mfma_supports(int D, int dv, int block) {
    if (D == 64) return (block == 64 && (dv == 64 || dv == 32 || dv == 16)) || (block == 32 && (dv == 64 || dv == 32)) ||
                        (block == 16 && dv == 64);
    if (D == 128) return (block == 32 && (dv == 128 || dv == 64 || dv == 32)) || (block == 16 && (dv == 128 || dv == 64));
    return false;
}

// Plain passes only (no gated epilogue, equal widths, whole chains), D in {64, 128}.
hipError_t launch_pass_f32_mfma(const PassBatch& pb, int D, int dv, int block, hipStream_t stream) {
    if (pb.segs != 1 || pb.state_only) return hipErrorInvalidValue;
    for (int i = 0; i < pb.count; ++i)
        if (pb.p[i].gate || !pb.p[i].out) return hipErrorInvalidValue;
#define LTN_F32M(d, v, b) if (D == d && dv == v && block == b) return launch_m<d, v, b>(pb, stream)
    LTN_F32M(64, 64, 64); LTN_F32M(64, 32, 64); LTN_F32M(64, 16, 64);
    LTN_F32M(64, 64, 32); LTN_F32M(64, 32, 32);
    LTN_F32M(64, 64, 16);
    LTN_F32M(128, 128, 32); LTN_F32M(128, 64, 32); LTN_F32M(128, 32, 32);
    LTN_F32M(128, 128, 16); LTN_F32M(128, 64, 16);
#undef LTN_F32M
    return hipErrorInvalidValue;
}

}  // namespace ltn
