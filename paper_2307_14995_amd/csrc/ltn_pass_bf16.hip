// bf16 MFMA kernels for Lightning Attention on gfx950 (MI355X).
//
// Building block: the decayed linear-attention pass (arXiv 2307.14995, Sec. 3.2.1 with
// the decay mask of Eq. 1; recurrence of Sec. 3.3, Algorithm 2, taken 64 tokens at a
// time).  For each chain (batch, head) and a slice of DV value columns, per block i of
// 64 tokens, with S_i the running [D x DV] state (A, B have D features; C and the output
// have DC, equal to D except around the LRPE-d expansion of Eq. 1, where queries and keys
// are twice as wide as values):
//
//     P    = (A_i B_i^T) (.) M,       M[r,c] = lambda^(r-c) for r >= c else 0
//     O_i  = P C_i + diag(lambda^(r+1)) A_i S_i
//     S_i+1 = lambda^len S_i + (diag(lambda^(len-1-c)) B_i)^T C_i
//
// (A,B,C) = (Q,K,V) gives the forward output O; the gradients are the same pass with
// permuted operands, dQ = pass(dO,V,K), and on a reversed token axis dV = pass(K,Q,dO),
// dK = pass(V,dO,Q) (derivative of the definition; App. B Algorithm 4 corrected).
//
// One workgroup = one pass over one chain for a slice of DV value columns: 512 threads =
// 8 wavefronts in two roles (two waves per SIMD, so one role's LDS/VALU latencies hide
// under the other's MFMAs):
//
//   * output waves 0..3: wave w owns token rows 16w..16w+15 of the block.  It forms the
//     transposed score tiles P^T[key tile][its rows] with 16x16x32 bf16 MFMA; the fp32
//     accumulators already sit in the lane layout the next MFMA wants as its B operand
//     (the contraction index is permuted identically on both operands), so the masked
//     scores never leave registers.  The output is produced transposed
//     (O^T = C^T P^T + S^T A^T): every lane holds groups of four consecutive output
//     features of one token; lane-row swaps regroup them into 16-byte stores.
//   * state waves 4..7: wave u owns state rows [u*D/4, (u+1)*D/4) x DV in fp32
//     accumulators for the whole sequence, applies S <- lambda^len S + (decayed B)^T C
//     and publishes a bf16 copy [dv][dk] to LDS (double buffered), which the output waves
//     read as the A operand of S^T A^T.
//   * all three operand tiles go global -> LDS directly (global_load_lds_dwordx4: no
//     registers, every wave-wide load covers 1 KB of consecutive addresses; wave-uniform base
//     in scalar registers plus a 32-bit lane offset) into a ring of 2-4 stages (as many as fit
//     beside the two state copies), so one to three blocks of loads are always in flight per
//     workgroup; one barrier per block.  The loads are issued by output waves 0 and 1: the
//     state waves' chain (update, publish) is the longest between two barriers, a burst of
//     40-48 wave-wide loads holds its issuer for 600-1600 cycles, and those two waves have the
//     fewest causal score tiles.  They wait for a block with an exact vmcnt that counts their
//     own stores in between (VMEM operations of a wave retire in issue order), never for the
//     stores themselves.  In the register-fed layout (256 features) all four output waves
//     share the loads; in the gated pass the gate values are loaded from assembly too, ahead
//     of the block's tile loads, and counted with them.  LDS rows are unpadded; the 16-byte chunk
//     index is XOR-swizzled with the row so that row reads, transpose reads
//     (ds_read_b64_tr_b16, for operands needed "down the token axis") and the state-copy
//     writes spread over the banks.  Rows past the end of a short last block are fetched
//     from a small buffer of zeros; tile columns past the end of a tensor's rows (heads of 96
//     features in 128-wide tiles) are cleared once and masked out of every load.
//   * wave role and strip are compile-time constants of the code each wave runs, so
//     causal tile skipping costs no branches inside a block.
// Only non-negative powers of lambda are formed.
//
// Two variations of the same workgroup: the gated epilogue (full-width slices: the token
// mixer's y = SRMSNorm(o) (.) u of Eq. 3 applied to the fp32 output rows before they are
// stored) and the state-only sweep of the sequence-parallel form (a chain cut into
// segments: only the state waves work, and only the segment's end state is written).
#include "ltn_bf16_tiles.h"

namespace ltn {
namespace {

constexpr int kThreads = 512;

template <int D, int DV>
struct Cfg {
    static constexpr int KS = D / 32;          // k-steps of a D-long contraction
    static constexpr int MT = D / 64;          // 16-row state tiles owned per state wave
    static constexpr int NT = DV / 16;         // 16-column tiles of the value slice
    using F = Swz<D>;                          // full-width tiles and state copies [DV][D]
    // the C tile in LDS: DV columns, or the next power of two with the rest zero-filled (96 -> 128)
    static constexpr int CW = DV == 96 ? 128 : DV;
    using V = Swz<CW>;
    static constexpr int SBYTES = DV * F::RB;  // one bf16 state copy
    // pass body: ring of PST stages {A tile, B tile, C tile}, then two state copies.
    // AREG (256 query/key features, the LRPE-d expansion of Eq. 1): two 32 KB tiles per
    // stage would leave room for one stage only, so the A tile stays out of LDS -- every
    // output wave fetches its own 16 rows of A straight into registers, two blocks ahead --
    // and a stage is {B tile, C tile}.
    static constexpr bool AREG = D == 256;
    static constexpr int BOFF = AREG ? 0 : F::BYTES;        // B tile inside a stage
    static constexpr int COFF = BOFF + F::BYTES;            // C tile inside a stage
    static constexpr int PSTAGE = COFF + V::BYTES;
    static constexpr int PST = (4 * PSTAGE + 2 * SBYTES <= 163840) ? 4 : ((3 * PSTAGE + 2 * SBYTES <= 163840) ? 3 : 2);
    static constexpr int P_SB = PST * PSTAGE;
    static constexpr int PASS_TOTAL = P_SB + 2 * SBYTES;
    static_assert(PASS_TOTAL <= 163840, "LDS per workgroup");
    // Plain pass: the tile loads are issued by output waves 0 .. FW-1 -- the waves with the
    // fewest causal score tiles, which reach the block's barrier long before the state waves do;
    // the texture addresser takes 16 cycles per wave-wide 1 KB load, and whoever issues a
    // block's 40-48 loads in a burst stands still for that long.
    static constexpr int FW = 2;
    // AREG layout: all four output waves share the B and C tile loads (each also fetches its own
    // A fragments); the state waves' update and publish are the longer chain there.
    static constexpr int AFW = 4;
};

// MODE of a workgroup: the plain pass, the pass with the gated epilogue, or the
// state-only sweep of the sequence-parallel form (no outputs: only the segment's end state).
enum { kPlain = 0, kGated = 1, kStateOnly = 2 };


// Register prefetch loads of the AREG output waves are issued from inline assembly and
// waited for with explicit vmcnt counts: left to the compiler, loads that rotate through
// register sets two blocks ahead make its wait-count bookkeeping wait for every load right
// after issuing it.  The destination is an in/out operand and every load is unconditional,
// so a register set is one variable updated in place and the compiler has no reason to copy
// it (a copy made between issue and wait would read stale data).
__device__ __forceinline__ void gload16(u32x4& r, const char* p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(r) : "v"(p) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm8(u32x4 (&r)[8]) {
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
                 : "n"(N) : "memory");
}

// lambda^n for 0 <= n <= 64 without one fp64 powering loop per constant: every lane powers
// once (lambda^lane, and lambda^64), the rest are cross-lane reads.  Same values as
// decay_pow(lam, n), bit for bit.  All 64 lanes must call get() together.
struct DecayTable {
    float mine, p64;
    __device__ __forceinline__ void init(float lam, int lane) {
        mine = decay_pow(lam, lane);
        p64 = decay_pow(lam, 64);
    }
    __device__ __forceinline__ float get(int n) const {
        const float v = __shfl(mine, n & 63, 64);
        return n >= 64 ? p64 : v;
    }
};

// Per-lane decay constants of an output wave (non-negative exponents only).
template <int W>
struct OutConsts {
    float qscale, mdiag[4], moff[4], lam16, lam32;
    __device__ __forceinline__ void init(float lam, int g, int i16) {
        DecayTable tb;
        tb.init(lam, 16 * g + i16);
        qscale = tb.get(16 * W + i16 + 1);               // lambda^(r+1), r = row in block
        const int d0 = i16 - 4 * g;                      // (row - key) in a diagonal tile at j = 0
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float md = tb.get(d0 - j >= 0 ? d0 - j : 0);
            mdiag[j] = (d0 - j >= 0) ? md : 0.0f;
            moff[j] = tb.get(16 + d0 - j);               // 16 + d0 - j >= 1
        }
        lam16 = tb.get(16);
        lam32 = tb.get(32);
    }
};

// Per-lane byte offsets into swizzled tiles (computed once per wave).
//   row[ks]  : 16-byte row read of a full-width tile / state copy: row i16, chunk 4ks + g
//   ctr[nt]  : transpose read of the C operand: token row 4g + s/4, columns c0 + 16nt + 4(s%4)
template <int D, int DV, int CCOLS>
struct ReadOffs {
    int row[D / 32];
    int ctr[DV / 16];
    __device__ __forceinline__ void init(int g, int i16, int c0) {
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks) row[ks] = Swz<D>::off(i16, 4 * ks + g);
#pragma unroll
        for (int nt = 0; nt < DV / 16; ++nt) {
            const int col = c0 + 16 * nt + 4 * (i16 & 3);
            ctr[nt] = Swz<CCOLS>::off(4 * g + (i16 >> 2), col >> 3) + (col & 4) * 2;
        }
    }
};

// One pass's output for the token strip of output wave W in the current block:
//   out^T[DV x 16] = Ct^T P^T + diag(qscale) S^T A^T,   P^T = (Bt A^T) (.) M^T
//   btile : full-width B tile in LDS (rows = tokens);  ctile : tile holding the C operand
//   (CCOLS columns wide);  scopy : bf16 state copy [DV][D];  Af : A fragments of the strip
//   out   : global address of this lane's token row, slice column 8g
//   GATED (full-width slices only): the strip's rows are complete output rows, so the
//   token mixer's epilogue (Sec. 3.1.2 Eq. 3 with the SimpleRMSNorm of Sec. 3.1.3 per head),
//   y = o / sqrt(mean(o^2) + eps) (.) u, is applied before anything is stored; gate/yout are
//   this lane's addresses in U and Y (same position as out), out may be null.
//   uq (GATED): the gate values of this lane's token, loads issued by the caller from assembly
//   before the block's tile loads; GWAIT = the VMEM operations the wave issued after them.
template <int D, int DV, int W, int CCOLS, bool GATED = false, int DROW = D, int GWAIT = 0>
__device__ __forceinline__ void output_pass(const char* btile, const char* ctile, const char* scopy,
                                            const Frag (&Af)[D / 32], const OutConsts<W>& k,
                                            const ReadOffs<D, DV, CCOLS>& ro, char* out, bool store,
                                            u32x4* uq = nullptr, char* yout = nullptr, float eps = 0.f) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, NT = C::NT, RB = C::F::RB, CRB = Swz<CCOLS>::RB;
    static_assert(!GATED || DV == DROW, "the gated epilogue needs complete output rows (DROW features)");

    // -- transposed scores P^T[key tile kt <= W][own 16 rows]
    f32x4 sacc[W + 1];
#pragma unroll
    for (int kt = 0; kt <= W; ++kt) sacc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kt = 0; kt <= W; ++kt) {
            Frag a;
            a.u = *(const u32x4*)(btile + (16 * kt) * RB + ro.row[ks]);
            sacc[kt] = mfma16(a.v, Af[ks].v, sacc[kt]);
        }

    // -- inter-block part (independent of the scores): S^T A^T with the published state
    f32x4 oi[NT], oe[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        oi[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        oe[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            Frag a;
            a.u = *(const u32x4*)(scopy + (16 * nt) * RB + ro.row[ks]);
            oe[nt] = mfma16(a.v, Af[ks].v, oe[nt]);
        }

    // -- mask the scores, round to bf16: they are B operands as they stand
    bf16x4 Pt[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
        if (kt < W) {
            const float sc = (W - kt == 1) ? 1.0f : ((W - kt == 2) ? k.lam16 : k.lam32);
            f32x4 m;
#pragma unroll
            for (int j = 0; j < 4; ++j) m[j] = sacc[kt < W ? kt : 0][j] * (k.moff[j] * sc);
            Pt[kt] = to_bf16(m);
        } else if (kt == W) {
            f32x4 m;
#pragma unroll
            for (int j = 0; j < 4; ++j) m[j] = sacc[W][j] * k.mdiag[j];
            Pt[kt] = to_bf16(m);
        } else {
            Pt[kt] = bf16x4{0, 0, 0, 0};
        }
    }

    // -- intra-block part (transposed): C^T P^T, C read down the token axis
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        if (2 * p <= W) {
            Frag b;
            b.b[0] = Pt[2 * p];
            b.b[1] = Pt[2 * p + 1];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                Frag vf;
                vf.h[0] = lds_tr16(ctile + (32 * p) * CRB + ro.ctr[nt]);
                vf.h[1] = lds_tr16(ctile + (32 * p + 16) * CRB + ro.ctr[nt]);
                oi[nt] = mfma16(vf.v, b.v, oi[nt]);
            }
        }
    }

    // -- combine and store (the strip is regrouped into 16-byte stores)
    if constexpr (!GATED) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j) oi[nt][j] += k.qscale * oe[nt][j];
        store_strip<NT>(oi, out, store);
    } else {
        // the same regrouping on fp32 values, after the row's mean square: the four lanes of
        // a token (one per lane row) each hold a quarter of its D features
        float ss = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                oi[nt][j] += k.qscale * oe[nt][j];
                ss = fmaf(oi[nt][j], oi[nt][j], ss);
            }
        {   // sum over the four lane rows: swapping two copies leaves both halves' parts side by side
            auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(ss), __float_as_uint(ss), false, false);
            ss = __uint_as_float(s[0]) + __uint_as_float(s[1]);
            auto t = __builtin_amdgcn_permlane16_swap(__float_as_uint(ss), __float_as_uint(ss), false, false);
            ss = __uint_as_float(t[0]) + __uint_as_float(t[1]);
        }
        const float rstd = 1.0f / sqrtf(ss * (1.0f / DROW) + eps);
        wait_dma<GWAIT>();                 // the gate values have arrived
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) asm volatile("" : "+v"(uq[p]));
#pragma unroll
        for (int p = 0; p < NT / 2; ++p) {
            float x[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float lo = oi[2 * p][j], hi = oi[2 * p + 1][j];
                auto s = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
                auto t = __builtin_amdgcn_permlane16_swap(s[0], s[1], false, false);
                x[j] = __uint_as_float(t[0]);
                x[4 + j] = __uint_as_float(t[1]);
            }
            Frag uf, of, yf;
            uf.u = uq[p];
            const f32x8 ug = __builtin_convertvector(uf.v, f32x8);
            f32x8 xo, xy;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                xo[j] = x[j];
                xy[j] = x[j] * rstd * ug[j];
            }
            yf.v = __builtin_convertvector(xy, bf16x8);
            if (store) *(u32x4*)(yout + 64 * p) = yf.u;
            if (out) {
                of.v = __builtin_convertvector(xo, bf16x8);
                if (store) *(u32x4*)(out + 64 * p) = of.u;
            }
        }
    }
}

// What a state wave needs per lane: decay factors for the B^T fragments
// (lambda^(len-1-token) per MFMA k-slot, lambda^len for the state) and swizzled offsets.
template <int D, int DV, int CCOLS>
struct StateConsts {
    float ksc[2][8], lamB;
    int btr[D / 64];     // transpose read of B^T: token row 4g + s/4, columns dk0 + 16mt + 4(s%4)
    int ctr[DV / 16];    // transpose read of C:   token row 4g + s/4, columns c0 + 16nt + 4(s%4)
    int pub[D / 64];     // 8-byte write into a state copy: row i16, columns dk0 + 16mt + 4g
    __device__ __forceinline__ void set_block_len(float lam, int len, int lane) {   // whole wave together
        const int g = lane >> 4;
        DecayTable tb;
        tb.init(lam, lane);
        lamB = tb.get(len);
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int tok = 32 * p + 16 * (j >> 2) + 4 * g + (j & 3);
                const float v = tb.get(tok < len ? len - 1 - tok : 0);
                ksc[p][j] = (tok < len) ? v : 0.0f;
            }
    }
    __device__ __forceinline__ void init_offsets(int g, int i16, int dk0, int c0) {
#pragma unroll
        for (int mt = 0; mt < D / 64; ++mt) {
            const int col = dk0 + 16 * mt + 4 * (i16 & 3);
            btr[mt] = Swz<D>::off(4 * g + (i16 >> 2), col >> 3) + (col & 4) * 2;
            const int pc = dk0 + 16 * mt + 4 * g;
            pub[mt] = Swz<D>::off(i16, pc >> 3) + (pc & 4) * 2;
        }
#pragma unroll
        for (int nt = 0; nt < DV / 16; ++nt) {
            const int col = c0 + 16 * nt + 4 * (i16 & 3);
            ctr[nt] = Swz<CCOLS>::off(4 * g + (i16 >> 2), col >> 3) + (col & 4) * 2;
        }
    }
};

// S[dk0 .. dk0 + D/4, :] <- lambda^len S + (decayed Bt)^T Ct for the rows this state wave owns.
template <int D, int DV, int CCOLS>
__device__ __forceinline__ void state_update(f32x4 (&st)[D / 64][DV / 16], const char* btile, const char* ctile,
                                             const StateConsts<D, DV, CCOLS>& k) {
    using C = Cfg<D, DV>;
    constexpr int MT = C::MT, NT = C::NT, RB = C::F::RB, CRB = Swz<CCOLS>::RB;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j) st[mt][nt][j] *= k.lamB;
#pragma unroll
    for (int p = 0; p < 2; ++p) {          // 32 tokens per step
        Frag Vf[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            Vf[nt].h[0] = lds_tr16(ctile + (32 * p) * CRB + k.ctr[nt]);
            Vf[nt].h[1] = lds_tr16(ctile + (32 * p + 16) * CRB + k.ctr[nt]);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            Frag a;
            a.h[0] = lds_tr16(btile + (32 * p) * RB + k.btr[mt]);
            a.h[1] = lds_tr16(btile + (32 * p + 16) * RB + k.btr[mt]);
            f32x8 af = __builtin_convertvector(a.v, f32x8);
#pragma unroll
            for (int j = 0; j < 8; ++j) af[j] *= k.ksc[p][j];
            a.v = __builtin_convertvector(af, bf16x8);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) st[mt][nt] = mfma16(a.v, Vf[nt].v, st[mt][nt]);
        }
    }
}

template <int D, int DV, int CCOLS>
__device__ __forceinline__ void publish_state(const f32x4 (&st)[D / 64][DV / 16], char* scopy,
                                              const StateConsts<D, DV, CCOLS>& k) {
    using C = Cfg<D, DV>;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt)
            *(bf16x4*)(scopy + (16 * nt) * C::F::RB + k.pub[mt]) = to_bf16(st[mt][nt]);
}

struct Chain {            // what every wave of the workgroup knows about its problem
    const char* a;        // pass body: operands offset to this chain (c/out also to the slice)
    const char* b;
    const char* c;
    char* out;
    const char* gate;        // gated epilogue: U and Y, offset like out (out may then be null)
    char* y;
    float eps;
    const float* state_in;   // offset to this chain and column slice, or nullptr
    float* state_out;
    long long N;
    int T;                // number of 64-token blocks
    int last_valid;       // tokens in the last block (1..64)
    int rev;
    float lam;
};

// =============================================================== pass body

// "Block blk + 1 has landed" for a wave that issues, per block and in this order, G gate loads,
// L tile loads (for block blk + PST - 1) and S stores, after PST - 1 blocks' tile loads up front:
// the operations it issued after that block's loads.
template <int PST, int L, int S, int G>
__device__ __forceinline__ void wait_block(int blk) {
    static_assert(PST >= 2 && PST <= 4, "ring depths");
    if constexpr (PST == 2) {
        wait_dma<S>();
    } else if constexpr (PST == 3) {
        if (blk == 0) wait_dma<L + S + G>(); else wait_dma<L + 2 * S + G>();
    } else {
        if (blk == 0) wait_dma<2 * L + S + G>();
        else if (blk == 1) wait_dma<2 * L + 2 * S + 2 * G>();
        else wait_dma<2 * L + 3 * S + 2 * G>();
    }
}

template <int D, int DV, int DC, int W, int MODE, int DR>
__device__ __forceinline__ void pass_output_wave(const Chain& ch, char* smem, unsigned lds0, int lane) {
    using C = Cfg<D, DV>;
    constexpr bool GATED = MODE == kGated;
    constexpr bool SO = MODE == kStateOnly;          // nothing to produce: tile loads and barriers only
    constexpr int KS = C::KS;
    constexpr long long ROW = DC * 2;      // the output's row (and U's, Y's)
    const long long step = ch.rev ? -(long long)kBlock * ROW : (long long)kBlock * ROW;

    // Tile pipeline (issuing waves only): block b lives in ring stage b % PST; the loads of
    // block b + PST - 1 go out right after the barrier that frees their stage.  This wave's
    // VMEM operations retire in issue order, loads and stores alike, so "block b + 1 has
    // landed" is a vmcnt of exactly the operations issued after its loads: the NT/2 stores of
    // every block since and the loads of the PST - 2 blocks behind it.
    constexpr bool ISSUER = W < C::FW;
    constexpr bool NOA = SO || C::AREG;              // the A tile is not fetched into LDS
    constexpr int L = ISSUER ? ((NOA ? 1 : 2) * TileDmaU<D>::NI + TileDmaU<C::CW>::NI) / C::FW : 0;   // loads per block, this wave
    constexpr int S = SO ? 0 : C::NT / 2;            // stores per block and output tensor, this wave
    constexpr int G = GATED ? C::NT / 2 : 0;         // gate loads per block, issued before the block's tile loads
    static_assert((C::PST - 2) * (L + G) + (C::PST - 1) * (GATED ? 2 : 1) * S <= 63, "vmcnt field");
    constexpr long long AROW = DR * 2;
    TileDmaU<D, DR> dab;                              // A and B tiles: same shape, same offsets
    TileDmaU<C::CW, DV> dcc;
    const char* pa0 = nullptr;
    const char* pb0 = nullptr;
    const char* pc0 = nullptr;
    if constexpr (ISSUER) {
        dab.init(lane, AROW, ch.rev);
        dcc.init(lane, ROW, ch.rev);
        pa0 = ch.a + (ch.rev ? (ch.N - 1) * AROW : 0);
        pb0 = ch.b + (ch.rev ? (ch.N - 1) * AROW : 0);
        pc0 = ch.c + (ch.rev ? (ch.N - 1) * ROW : 0);
    }
    const long long astep = ch.rev ? -(long long)kBlock * AROW : (long long)kBlock * AROW;
    auto fetch = [&](int b, int stage) {
        if constexpr (ISSUER) {
            b = b < ch.T ? b : ch.T - 1;   // past the end: re-read the last block into a free stage
            const int valid = (b + 1 == ch.T) ? ch.last_valid : kBlock;
            const unsigned lds = lds0 + (unsigned)(stage * C::PSTAGE);
            const char* pa = pa0 + (long long)b * astep;
            const char* pb = pb0 + (long long)b * astep;
            const char* pc = pc0 + (long long)b * step;
            if (valid == kBlock) {
                if constexpr (!NOA) dab.template issue_full<C::FW, W>(pa, AROW, ch.rev, lds);
                dab.template issue_full<C::FW, W>(pb, AROW, ch.rev, lds + C::BOFF);
                dcc.template issue_full<C::FW, W>(pc, ROW, ch.rev, lds + C::COFF);
            } else {
                if constexpr (!NOA) dab.template issue_partial<C::FW, W>(pa, AROW, ch.rev, lds, valid, lane);
                dab.template issue_partial<C::FW, W>(pb, AROW, ch.rev, lds + C::BOFF, valid, lane);
                dcc.template issue_partial<C::FW, W>(pc, ROW, ch.rev, lds + C::COFF, valid, lane);
            }
        }
    };
    const bool two_outputs = GATED && ch.out;          // the gated pass stores Y and, if asked, O
    auto wait_next = [&](int blk) {        // block blk + 1 has landed (this wave's part)
        if constexpr (ISSUER) {
            if (two_outputs) wait_block<C::PST, L, 2 * S, G>(blk);
            else wait_block<C::PST, L, S, G>(blk);
        }
    };
    if constexpr (ISSUER) {                // blocks 0 .. PST-2 in flight, block 0 landed
#pragma unroll
        for (int b = 0; b < C::PST - 1; ++b) fetch(b, b);
        wait_dma<(C::PST - 2) * L>();
    }

    if constexpr (SO) {
        __syncthreads();
        int stage = 0;
        for (int blk = 0; blk + 1 < ch.T; ++blk) {
            if constexpr (ISSUER) {
                int fs = stage + C::PST - 1;
                if (fs >= C::PST) fs -= C::PST;
                fetch(blk + C::PST - 1, fs);
                wait_next(blk);
            }
            __syncthreads();
            stage = (stage + 1 == C::PST) ? 0 : stage + 1;
        }
        if constexpr (ISSUER) wait_dma<0>();
        return;
    }

    const int g = lane >> 4, i16 = lane & 15;
    OutConsts<W> k;
    k.init(ch.lam, g, i16);
    ReadOffs<D, DV, C::CW> ro;
    ro.init(g, i16, 0);

    // this lane's token row (16W + i16) of block 0
    const long long r0 = ch.rev ? (ch.N - 1 - (16 * W + i16)) : (long long)(16 * W + i16);
    const long long lane_off = r0 * ROW + (8 * g) * 2;
    char* po = ch.out ? ch.out + lane_off : nullptr;
    const char* pu = GATED ? ch.gate + lane_off : nullptr;
    char* py = GATED ? ch.y + lane_off : nullptr;
    u32x4 uq[GATED ? G : 1];
#pragma unroll
    for (int p = 0; p < (GATED ? G : 1); ++p) uq[p] = u32x4{0, 0, 0, 0};

    __syncthreads();                       // block 0 tiles and the initial state copy are in LDS
    int stage = 0;
    for (int blk = 0; blk < ch.T; ++blk) {
        const bool more = blk + 1 < ch.T;
        const bool row_ok = (16 * W + i16) < ((blk + 1 == ch.T) ? ch.last_valid : kBlock);
        const long long bo = (long long)blk * step;
        if constexpr (GATED) {             // gate values of this lane's token: issued first, used last
#pragma unroll
            for (int p = 0; p < G; ++p) gload16(uq[p], (more || row_ok) ? pu + bo + 64 * p : (const char*)kZeros);
        }
        if constexpr (ISSUER) {
            int fs = stage + C::PST - 1;   // stage of block blk + PST - 1 (free since the last barrier)
            if (fs >= C::PST) fs -= C::PST;
            fetch(blk + C::PST - 1, fs);
        }
        const char* st = smem + stage * C::PSTAGE;
        Frag Af[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) Af[ks].u = *(const u32x4*)(st + (16 * W) * C::F::RB + ro.row[ks]);
        // with more blocks to come every lane stores (the count above relies on it)
        output_pass<D, DV, W, C::CW, GATED, DC, L>(st + C::BOFF, st + C::COFF,
                                            smem + C::P_SB + (blk & 1) * C::SBYTES, Af, k, ro,
                                            po ? po + bo : nullptr, more || row_ok,
                                            uq, GATED ? py + bo : nullptr, ch.eps);
        if (more) {
            wait_next(blk);
            __syncthreads();
        }
        stage = (stage + 1 == C::PST) ? 0 : stage + 1;
    }
    if constexpr (ISSUER) wait_dma<0>();   // nothing may land in LDS after this workgroup is gone
}

// Output wave of the AREG layout: as pass_output_wave, but the A fragments of its 16 rows
// come straight from global memory into three rotating register sets, two blocks ahead, and
// every output wave issues a quarter of the B and C tile loads.
template <int D, int DV, int DC, int W>
__device__ __forceinline__ void areg_output_wave(const Chain& ch, char* smem, unsigned lds0, int lane) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, NT = C::NT;
    static_assert(KS == 8, "register sets of eight fragments");
    constexpr long long AROW = D * 2, ROW = DC * 2;
    const int g = lane >> 4, i16 = lane & 15;
    OutConsts<W> k;
    k.init(ch.lam, g, i16);
    ReadOffs<D, DV, C::CW> ro;
    ro.init(g, i16, 0);

    const long long r0 = ch.rev ? (ch.N - 1 - (16 * W + i16)) : (long long)(16 * W + i16);
    const long long astep = ch.rev ? -(long long)kBlock * AROW : (long long)kBlock * AROW;
    const long long step = ch.rev ? -(long long)kBlock * ROW : (long long)kBlock * ROW;
    const char* pa = ch.a + r0 * AROW + (8 * g) * 2;
    char* po = ch.out + r0 * ROW + (8 * g) * 2;
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };

    struct Set { u32x4 f[KS]; };
    auto load_a = [&](Set& s, int b) {
        b = b < ch.T ? b : ch.T - 1;       // past the end: re-read the last block (ignored)
        const bool ok = (16 * W + i16) < valid_of(b);
        const char* p = pa + (long long)b * astep;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) gload16(s.f[ks], ok ? p + ks * 64 : (const char*)kZeros);
    };
    // Tile pipeline: per block this wave issues, in this order, its L loads of the B and C tiles
    // of block blk + PST - 1, the KS loads of set(blk + 2) and the NT/2 stores of block blk; all
    // of them retire in issue order.
    constexpr int L = (TileDmaU<D>::NI + TileDmaU<C::CW>::NI) / C::AFW;
    static_assert(W < C::AFW && TileDmaU<D>::NI % C::AFW == 0 && TileDmaU<C::CW>::NI % C::AFW == 0, "even shares");
    TileDmaU<D> dbb;
    TileDmaU<C::CW> dcc;
    dbb.init(lane, AROW, ch.rev);
    dcc.init(lane, ROW, ch.rev);
    const char* pb0 = ch.b + (ch.rev ? (ch.N - 1) * AROW : 0);
    const char* pc0 = ch.c + (ch.rev ? (ch.N - 1) * ROW : 0);
    auto fetch = [&](int b, int stage) {
        b = b < ch.T ? b : ch.T - 1;       // past the end: re-read the last block into a free stage
        const int valid = valid_of(b);
        const unsigned lds = lds0 + (unsigned)(stage * C::PSTAGE);
        const char* pb = pb0 + (long long)b * astep;
        const char* pc = pc0 + (long long)b * step;
        if (valid == kBlock) {
            dbb.template issue_full<C::AFW, W>(pb, AROW, ch.rev, lds + C::BOFF);
            dcc.template issue_full<C::AFW, W>(pc, ROW, ch.rev, lds + C::COFF);
        } else {
            dbb.template issue_partial<C::AFW, W>(pb, AROW, ch.rev, lds + C::BOFF, valid, lane);
            dcc.template issue_partial<C::AFW, W>(pc, ROW, ch.rev, lds + C::COFF, valid, lane);
        }
    };
    // Set(blk) was issued two blocks ago; since then this wave issued the NT/2 stores of
    // each of two blocks, the KS loads of set(blk+1) and one block's tile loads.
    constexpr int kAfter = NT + KS + L;
    // The tiles of block blk + 1 went out PST - 1 blocks ago, before that block's set and stores.
    constexpr int kTilesAfter = (C::PST - 1) * (KS + NT / 2) + (C::PST - 2) * L;
    static_assert(kAfter <= 63 && kTilesAfter <= 63, "vmcnt field");

    auto do_block = [&](int blk, int stage, Set& cur_set, Set& incoming) {
        const bool more = blk + 1 < ch.T;
        const bool row_ok = (16 * W + i16) < valid_of(blk);
        wait_vm8<kAfter>(cur_set.f);
        Frag Af[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) Af[ks].u = cur_set.f[ks];
        int fs = stage + C::PST - 1;       // stage of block blk + PST - 1 (free since the last barrier)
        if (fs >= C::PST) fs -= C::PST;
        fetch(blk + C::PST - 1, fs);
        load_a(incoming, blk + 2);
        const char* st = smem + stage * C::PSTAGE;
        // with more blocks to come every lane stores (the counts above rely on it)
        output_pass<D, DV, W, C::CW>(st + C::BOFF, st + C::COFF, smem + C::P_SB + (blk & 1) * C::SBYTES, Af, k, ro,
                                  po + (long long)blk * step, more || row_ok);
        if (more) {
            wait_dma<kTilesAfter>();       // block blk + 1 has landed (this wave's part)
            __syncthreads();
        }
    };

    Set s0, s1, s2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s0.f[ks] = s1.f[ks] = s2.f[ks] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < C::PST - 1; ++b) fetch(b, b);      // tiles of blocks 0 .. PST-2
    load_a(s0, 0);
    load_a(s1, 1);
    wait_vm8<0>(s0.f);                     // blocks 0 and 1 are retired here, so the
    wait_vm8<0>(s1.f);                     // steady-state count is safe for them too
    __syncthreads();                       // block 0 tiles and the initial state copy are in LDS

    int stage = 0;
    auto next = [&]() { stage = (stage + 1 == C::PST) ? 0 : stage + 1; };
    for (int blk = 0; blk < ch.T; blk += 3) {
        do_block(blk, stage, s0, s2); next();
        if (blk + 1 < ch.T) { do_block(blk + 1, stage, s1, s0); next(); }
        if (blk + 2 < ch.T) { do_block(blk + 2, stage, s2, s1); next(); }
    }
    // the last two prefetches were never consumed: retire them before the registers die (and
    // with them every tile load: nothing may land in LDS after this workgroup is gone)
    wait_vm8<0>(s0.f);
    wait_vm8<0>(s1.f);
    wait_vm8<0>(s2.f);
}

// DR: features per token that A and B really have in memory (D, or 96 computed as 128 with
// the tiles' last columns zero-filled and the state's last rows unused).
template <int D, int DV, int DC, int MODE, int DR>
__device__ __forceinline__ void pass_state_wave(const Chain& ch, char* smem, int lane, int u) {
    using C = Cfg<D, DV>;
    constexpr int MT = C::MT, NT = C::NT;
    constexpr bool SO = MODE == kStateOnly;          // no published state copies
    const int g = lane >> 4, i16 = lane & 15;
    const int dk0 = u * (D / 4);
    StateConsts<D, DV, C::CW> k;
    k.set_block_len(ch.lam, kBlock, lane);
    k.init_offsets(g, i16, dk0, 0);

    // running state, fp32
    f32x4 st[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (ch.state_in) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = dk0 + 16 * mt + 4 * g + j;
                    st[mt][nt][j] = (DR == D || row < DR) ? ch.state_in[(size_t)row * DC + 16 * nt + i16] : 0.0f;
                }
            } else {
                st[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }

    // prologue: the initial state copy published (the output waves run the tile pipeline:
    // block b lives in ring stage b % PST)
    if constexpr (!SO) publish_state<D, DV, C::CW>(st, smem + C::P_SB, k);
    __syncthreads();

    int stage = 0;                                   // stage of block blk
    for (int blk = 0; blk < ch.T; ++blk) {
        const bool more = blk + 1 < ch.T;
        if (!more) {
            if (!ch.state_out) break;                // the last update only feeds the returned state
            if (ch.last_valid != kBlock) k.set_block_len(ch.lam, ch.last_valid, lane);
        }
        const char* tb = smem + stage * C::PSTAGE;
        state_update<D, DV, C::CW>(st, tb + C::BOFF, tb + C::COFF, k);
        if (more) {
            if constexpr (!SO) publish_state<D, DV, C::CW>(st, smem + C::P_SB + ((blk + 1) & 1) * C::SBYTES, k);
            __syncthreads();
        }
        stage = (stage + 1 == C::PST) ? 0 : stage + 1;
    }

    if (ch.state_out) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = dk0 + 16 * mt + 4 * g + j;
                    if (DR == D || row < DR) ch.state_out[(size_t)row * DC + 16 * nt + i16] = st[mt][nt][j];
                }
    }
}

template <int D, int DV, int DC, int MODE, int DR>
__device__ __forceinline__ void pass_body(const PassBatch& pb, int nsplit, int xcd_ids, int wg, char* smem,
                                          unsigned lds0, int wave, int lane) {
    constexpr bool GATED = MODE == kGated;
    // (chain, segment) pairs are dealt to workgroups like chains; with one segment per
    // chain the pair index is the chain index
    int vchain, within;
    bool mine = map_workgroup_padded(wg, pb.count * nsplit, pb.chains * pb.segs, xcd_ids, vchain, within);
    if (pb.pairs_first && pb.count == 3 && nsplit == 1 && xcd_ids) {
        // Backward at full width: passes 0 and 1 of a chain walk the token axis together and
        // share two operands, pass 2 walks the other way.  Ids: all (pass 0, pass 1) pairs
        // first, a chain's pair side by side on one XCD, then every pass 2.  With more
        // workgroups than compute units the pairs still meet in L2 and the late-starting
        // rounds are filled with pass-2 workgroups, which share nothing with anyone
        // (measured on MI355X, 96..256 chains: 0..3 % faster than chain-major ids when backward
        // launches follow each other, no different when they alternate with forward launches).
        const int nch = (pb.chains * pb.segs + 7) / 8 * 8;       // chain slots of the launch
        const int xcd = wg & 7, slot = wg >> 3;
        if (wg < 2 * nch) {
            within = slot & 1;
            vchain = (slot >> 1) * 8 + xcd;
        } else {
            within = 2;
            vchain = (slot - (nch >> 2)) * 8 + xcd;
        }
        mine = vchain < pb.chains * pb.segs;
    }
    if (!mine) return;                     // a padding workgroup: the whole workgroup leaves before any barrier
    const int chain = vchain / pb.segs;
    const int seg = vchain - chain * pb.segs;
    if (MODE == kStateOnly && seg + 1 == pb.segs && !pb.need_last) return;   // nobody consumes this end state
    const int pi = within / nsplit;
    const int split = within - pi * nsplit;
    const PassArgs P = pb.p[pi];

    // the segment's tokens [seg_start, seg_start + n) of the pass's (possibly reversed) token
    // axis are rows [row0, row0 + n) of the tensors
    const long long seg_start = (long long)seg * pb.seg_len;
    const long long n = (pb.segs > 1 && pb.N - seg_start > pb.seg_len) ? pb.seg_len : pb.N - seg_start;
    const long long row0 = P.rev ? (pb.N - seg_start - n) : seg_start;

    Chain ch;
    const size_t first_row = (size_t)chain * (size_t)pb.N + (size_t)row0;
    const size_t ab_off = first_row * DR * 2;           // A, B: DR features per token
    const size_t chain_off = first_row * DC * 2;        // C, out (U, Y): DC features per token
    const size_t col_off = (size_t)split * DV * 2;
    ch.a = (const char*)P.a + ab_off;
    ch.b = (const char*)P.b + ab_off;
    ch.c = (const char*)P.c + chain_off + col_off;
    ch.out = P.out ? (char*)P.out + chain_off + col_off : nullptr;
    ch.gate = GATED ? (const char*)P.gate + chain_off : nullptr;
    ch.y = GATED ? (char*)P.gated_out + chain_off : nullptr;
    ch.eps = P.eps;
    ch.state_in = P.state_in ? P.state_in + (size_t)vchain * DR * DC + (size_t)split * DV : nullptr;
    ch.state_out = P.state_out ? P.state_out + (size_t)vchain * DR * DC + (size_t)split * DV : nullptr;
    ch.N = n;
    ch.T = (int)((n + kBlock - 1) / kBlock);
    ch.last_valid = (int)(n - (long long)(ch.T - 1) * kBlock);
    ch.rev = P.rev;
    ch.lam = pb.decay[chain % pb.H];

    if constexpr (DR != D || Cfg<D, DV>::CW != DV) {
        // Tiles wider than the tensors' rows: their loads leave the surplus chunks alone, which
        // hold zeros from here on (cleared once, in every ring stage, before the first load).
        using C = Cfg<D, DV>;
        static_assert(!C::AREG, "stages with an A tile");
        constexpr int ZA = (D - DR) / 8, ZC = (C::CW - DV) / 8;      // surplus chunks per row
        constexpr int kPerStage = kBlock * (2 * ZA + ZC);
        for (int i = wave * 64 + lane; i < C::PST * kPerStage; i += kThreads) {
            const int stage = i / kPerStage, j = i % kPerStage;
            int off;
            if (j < 2 * kBlock * ZA) {
                const int t = j / (kBlock * ZA), q = j % (kBlock * ZA);   // tile A or B, row and chunk
                off = (t ? C::BOFF : 0) + C::F::off(q / ZA, DR / 8 + q % ZA);
            } else {
                const int q = j - 2 * kBlock * ZA;
                off = C::COFF + C::V::off(q / (ZC ? ZC : 1), DV / 8 + q % (ZC ? ZC : 1));
            }
            *(u32x4*)(smem + stage * C::PSTAGE + off) = u32x4{0, 0, 0, 0};
        }
        __syncthreads();
    }
    if constexpr (Cfg<D, DV>::AREG) {
        static_assert(MODE != kGated && DR == D, "the register-fed layout has no gated epilogue");
        switch (wave) {
            case 0: case 1: case 2: case 3:
                if constexpr (MODE == kStateOnly) {    // tile loads (waves 0 .. FW-1) and barriers only
                    if (wave == 0) pass_output_wave<D, DV, DC, 0, MODE, DR>(ch, smem, lds0, lane);
                    else if (wave == 1) pass_output_wave<D, DV, DC, 1, MODE, DR>(ch, smem, lds0, lane);
                    else if (wave == 2) pass_output_wave<D, DV, DC, 2, MODE, DR>(ch, smem, lds0, lane);
                    else pass_output_wave<D, DV, DC, 3, MODE, DR>(ch, smem, lds0, lane);
                } else {
                    if (wave == 0) areg_output_wave<D, DV, DC, 0>(ch, smem, lds0, lane);
                    else if (wave == 1) areg_output_wave<D, DV, DC, 1>(ch, smem, lds0, lane);
                    else if (wave == 2) areg_output_wave<D, DV, DC, 2>(ch, smem, lds0, lane);
                    else areg_output_wave<D, DV, DC, 3>(ch, smem, lds0, lane);
                }
                break;
            default: pass_state_wave<D, DV, DC, MODE, DR>(ch, smem, lane, wave - 4); break;
        }
    } else {
        switch (wave) {
            case 0: pass_output_wave<D, DV, DC, 0, MODE, DR>(ch, smem, lds0, lane); break;
            case 1: pass_output_wave<D, DV, DC, 1, MODE, DR>(ch, smem, lds0, lane); break;
            case 2: pass_output_wave<D, DV, DC, 2, MODE, DR>(ch, smem, lds0, lane); break;
            case 3: pass_output_wave<D, DV, DC, 3, MODE, DR>(ch, smem, lds0, lane); break;
            default: pass_state_wave<D, DV, DC, MODE, DR>(ch, smem, lane, wave - 4); break;
        }
    }
}

// =============================================================== kernels

template <int D, int DV, int MODE, int DC = D, int DR = D>
__global__ __launch_bounds__(kThreads)
void pass_bf16_kernel(const PassBatch pb, const int nsplit, const int xcd_ids) {
    __shared__ __attribute__((aligned(1024))) char smem[Cfg<D, DV>::PASS_TOTAL];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: role dispatch is a uniform branch
    pass_body<D, DV, DC, MODE, DR>(pb, nsplit, xcd_ids, blockIdx.x, smem, lds_address(smem), wave, tid & 63);
}

template <int D, int DV, int MODE = kPlain, int DC = D, int DR = D>
hipError_t launch_t(const PassBatch& pb, hipStream_t stream) {
    static_assert(DV <= DC && DC % DV == 0, "value-column slices tile the C operand");
    static_assert(DC == D || MODE != kGated || (D == 128 && DC == 96 && DR == 96 && DV == 96),
                  "unequal widths: no gated epilogue (heads of 96 features computed as 128 have one)");
    const int nsplit = DC / DV;
    const long long nch = (long long)pb.chains * pb.segs;
    const int per_chain = pb.count * nsplit;
    const long long wgs = launch_chain_slots(nch, per_chain) * per_chain;
    if (wgs <= 0 || wgs > 0x7fffffffLL || pb.segs < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL((pass_bf16_kernel<D, DV, MODE, DC, DR>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, pb, nsplit,
                       (int)xcd_ids_fit(nch, per_chain));
    return hipGetLastError();
}

}  // namespace

hipError_t launch_pass_bf16(const PassBatch& pb, int D, int dv, hipStream_t stream, int DC) {
    if (DC != 0 && DC != D) {              // queries/keys and values of different widths (plain pass only)
        if (pb.p[0].gate) return hipErrorInvalidValue;
        if (pb.state_only) {               // segment end states: one slice width per shape
            if (D == 256 && dv == 64 && DC == 128) return launch_t<256, 64, kStateOnly, 128>(pb, stream);
            if (D == 128 && dv == 128 && DC == 256) return launch_t<128, 128, kStateOnly, 256>(pb, stream);
            if (D == 128 && dv == 64 && DC == 64) return launch_t<128, 64, kStateOnly, 64>(pb, stream);
            if (D == 64 && dv == 64 && DC == 128) return launch_t<64, 64, kStateOnly, 128>(pb, stream);
            return hipErrorInvalidValue;
        }
#define LTN_BF16_DC(d, v, c) if (D == d && dv == v && DC == c) return launch_t<d, v, kPlain, c>(pb, stream)
        LTN_BF16_DC(256, 64, 128); LTN_BF16_DC(256, 32, 128);
        LTN_BF16_DC(128, 128, 256); LTN_BF16_DC(128, 64, 256); LTN_BF16_DC(128, 32, 256);
        LTN_BF16_DC(128, 64, 64); LTN_BF16_DC(128, 32, 64);
        LTN_BF16_DC(64, 64, 128); LTN_BF16_DC(64, 32, 128);
#undef LTN_BF16_DC
        return hipErrorInvalidValue;
    }
    if (D == 96) {                         // computed as 128 with zero-filled tile columns: 32-column slices or all 96
        if (dv != 32 && dv != 96) return hipErrorInvalidValue;
        if (pb.p[0].gate) {                // gated epilogue: one pass, all 96 columns of a row in one workgroup
            if (pb.count != 1 || dv != 96 || !pb.p[0].gated_out || pb.state_only) return hipErrorInvalidValue;
            return launch_t<128, 96, kGated, 96, 96>(pb, stream);
        }
        if (pb.state_only) return dv == 32 ? launch_t<128, 32, kStateOnly, 96, 96>(pb, stream) : hipErrorInvalidValue;
        if (dv == 96) return launch_t<128, 96, kPlain, 96, 96>(pb, stream);
        return launch_t<128, 32, kPlain, 96, 96>(pb, stream);
    }
    if (pb.p[0].gate) {                    // gated epilogue: one pass, complete output rows
        if (pb.count != 1 || dv != D || !pb.p[0].gated_out || pb.state_only) return hipErrorInvalidValue;
        if (D == 128) return launch_t<128, 128, kGated>(pb, stream);
        if (D == 64) return launch_t<64, 64, kGated>(pb, stream);
        return hipErrorInvalidValue;
    }
    if (pb.state_only) {                   // segment end states only (sequence-parallel form)
        if (D == 256 && dv == 64) return launch_t<256, 64, kStateOnly>(pb, stream);
        if (D == 128 && dv == 128) return launch_t<128, 128, kStateOnly>(pb, stream);
        if (D == 128 && dv == 64) return launch_t<128, 64, kStateOnly>(pb, stream);
        if (D == 64 && dv == 64) return launch_t<64, 64, kStateOnly>(pb, stream);
        return hipErrorInvalidValue;
    }
    if (D == 256 && dv == 64) return launch_t<256, 64>(pb, stream);
    if (D == 256 && dv == 32) return launch_t<256, 32>(pb, stream);
    if (D == 128 && dv == 128) return launch_t<128, 128>(pb, stream);
    if (D == 128 && dv == 64) return launch_t<128, 64>(pb, stream);
    if (D == 128 && dv == 32) return launch_t<128, 32>(pb, stream);
    if (D == 64 && dv == 64) return launch_t<64, 64>(pb, stream);
    if (D == 64 && dv == 32) return launch_t<64, 32>(pb, stream);
    return hipErrorInvalidValue;
}

}  // namespace ltn
