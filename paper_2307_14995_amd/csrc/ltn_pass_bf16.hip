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
// A workgroup is 512 threads = 8 wavefronts with two roles, two waves per SIMD, so
// that one role's LDS and VALU latencies hide under the other's MFMAs:
//   * output waves 0..3: wave w owns query rows 16w..16w+15 of the block.  It forms
//     the transposed score tiles P^T[key tile][its rows] with 16x16x32 bf16 MFMA; the
//     fp32 accumulators already sit in the lane layout the next MFMA wants as its B
//     operand (the contraction index is permuted identically on both operands), so
//     the masked scores never leave registers.  The output is produced transposed
//     (O^T = C^T P^T + S^T A^T): every lane holds four consecutive output features of
//     one token -> 8-byte stores.  A fragments come straight from global memory.
//   * state waves 4..7: wave u owns state rows [u*D/4, (u+1)*D/4) x DV in fp32
//     accumulators for the whole sequence, applies S <- lambda^len S + (decayed B)^T C
//     and publishes a bf16 copy [dv][dk] to LDS, which the output waves read as the A
//     operand of S^T A^T.  These waves also stage the next block's B and C tiles
//     global -> registers -> LDS.
//   * LDS tiles and the state copy are double buffered: one barrier per block.  Row
//     pitches are 32 bytes over a multiple of 256 (measured best for the 16-byte
//     row reads and for the transpose reads).  Operands read "down the token axis"
//     (C for P C, B^T and C for the state update) use ds_read_b64_tr_b16.
//   * wave role and strip are compile-time constants of the code each wave runs, so
//     causal tile skipping costs no branches inside a block.
// Only non-negative powers of lambda are formed.
#include "ltn_kernels.h"

namespace ltn {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

union Frag {          // one 16x16x32 MFMA operand: 8 bf16 per lane
    bf16x8 v;
    u32x4 u;
    s16x4 h[2];
    bf16x4 b[2];
};

// Global prefetch loads are issued from inline assembly and waited for with explicit
// vmcnt counts.  Left to the compiler, the loads that rotate through register sets two
// blocks ahead make its wait-count bookkeeping give up at the loop header and wait for
// every load right after issuing it (measured: the kernel then runs at memory latency,
// not bandwidth).  VMEM operations retire in issue order, so "vmcnt(n)" with n = the
// number of VMEM operations issued after the wanted loads is exact; a smaller n is safe.
// The destination is an in/out operand and every prefetch load is unconditional, so a
// register set is one variable updated in place: the compiler has no reason to copy it
// (a copy made between issue and wait would read stale data).
__device__ __forceinline__ void gload16(u32x4& r, const char* p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(r) : "v"(p) : "memory");
}
// wait until at most N VMEM operations are outstanding; the operands tie the wait to the
// registers it protects so that no use of them can be scheduled above it
template <int N>
__device__ __forceinline__ void wait_vm(u32x4& a) { asm volatile("s_waitcnt vmcnt(%1)" : "+v"(a) : "n"(N) : "memory"); }
template <int N>
__device__ __forceinline__ void wait_vm(u32x4& a, u32x4& b) { asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory"); }
template <int N, int CNT>
__device__ __forceinline__ void wait_vm_all(u32x4 (&r)[CNT]) {
    static_assert(CNT >= 1 && CNT <= 4, "register sets of 1..4 fragments");
    if constexpr (CNT == 1) wait_vm<N>(r[0]);
    else if constexpr (CNT == 2) wait_vm<N>(r[0], r[1]);
    else if constexpr (CNT == 3) { wait_vm<N>(r[0], r[1]); wait_vm<N>(r[2]); }
    else { wait_vm<N>(r[0], r[1]); wait_vm<N>(r[2], r[3]); }
}

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
constexpr int kThreads = 512;
constexpr int kStageThreads = 256;     // the four state waves

template <int D, int DV>
struct Cfg {
    static constexpr int KS = D / 32;          // k-steps of a D-long contraction
    static constexpr int MT = D / 64;          // 16-row state tiles owned per state wave
    static constexpr int NT = DV / 16;         // 16-column tiles of the value slice
    static constexpr int KP = D * 2 + 32;      // LDS row pitch of the B tile / state copy (bytes)
    static constexpr int VP = DV * 2 + 32;     // LDS row pitch of the C tile (bytes)
    static constexpr int KC = D / 32;          // 16-byte chunks of B staged per staging thread
    static constexpr int VC = DV / 32;         // 16-byte chunks of C staged per staging thread
    static constexpr int KBYTES = kBlock * KP;
    static constexpr int VBYTES = kBlock * VP;
    static constexpr int SBYTES = DV * KP;
    static constexpr int KB = 0;                       // B tile, 2 buffers
    static constexpr int AB = 2 * KBYTES;              // A tile, 2 buffers
    static constexpr int VB = 4 * KBYTES;              // C tile, 2 buffers
    static constexpr int SB = VB + 2 * VBYTES;         // bf16 state copy [DV][D], 2 buffers
    static constexpr int TOTAL = SB + 2 * SBYTES;
};

struct Chain {            // what every wave of the workgroup knows about its problem
    const char* a;        // operands offset to this chain (and value-column slice for c/out)
    const char* b;
    const char* c;
    char* out;
    const float* state_in;   // offset to this chain and column slice, or nullptr
    float* state_out;
    long long N;
    int T;                // number of 64-token blocks
    int last_valid;       // tokens in the last block (1..64)
    int rev;
    float lam;
};

// ------------------------------------------------------------------ output waves

template <int D, int DV, int W>
__device__ __forceinline__ void run_output_wave(const Chain& ch, char* smem, int lane) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, NT = C::NT, KP = C::KP, VP = C::VP;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    const float lam = ch.lam;

    // decay constants (non-negative exponents only)
    const float qscale = decay_pow(lam, 16 * W + i16 + 1);      // lambda^(r+1), r = row in block
    const int d0 = i16 - 4 * g;                                  // (row - key) in a diagonal tile at j = 0
    float mdiag[4], moff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        mdiag[j] = (d0 - j >= 0) ? decay_pow(lam, d0 - j) : 0.0f;
        moff[j] = decay_pow(lam, 16 + d0 - j);                   // 16 + d0 - j >= 1
    }
    const float lam16 = decay_pow(lam, 16), lam32 = decay_pow(lam, 32);

    // output cursor for this lane's token row (16W + i16) of block 0
    const long long r0 = ch.rev ? (ch.N - 1 - (16 * W + i16)) : (long long)(16 * W + i16);
    const long long step = ch.rev ? -(long long)kBlock * ROW : (long long)kBlock * ROW;
    char* po = ch.out + r0 * ROW + (4 * g) * 2;
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };

    // Output waves issue no global loads: their stores retire in issue order with any
    // load that follows, and a store's acknowledgement is slow enough to stall a
    // prefetch queued behind it.  All loads belong to the state waves.
    __syncthreads();                       // block 0 tiles and the initial state copy are in LDS

    for (int blk = 0; blk < ch.T; ++blk) {
        const int cur = blk & 1;
        const bool more = blk + 1 < ch.T;
        const int valid = valid_of(blk);
        const char* kb = smem + C::KB + cur * C::KBYTES;
        const char* ab = smem + C::AB + cur * C::KBYTES;
        const char* vb = smem + C::VB + cur * C::VBYTES;
        const char* sb = smem + C::SB + cur * C::SBYTES;

        // -- own A fragments (rows past the end of the last block were staged as zeros)
        Frag Qf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            Qf[ks].u = *(const u32x4*)(ab + (16 * W + i16) * KP + (32 * ks + 8 * g) * 2);

        // -- transposed scores P^T[key tile kt <= W][own 16 rows]
        f32x4 sacc[W + 1];
#pragma unroll
        for (int kt = 0; kt <= W; ++kt) sacc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
        const char* ka = kb + i16 * KP + (8 * g) * 2;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kt = 0; kt <= W; ++kt) {
                Frag a;
                a.u = *(const u32x4*)(ka + (16 * kt) * KP + (32 * ks) * 2);
                sacc[kt] = mfma16(a.v, Qf[ks].v, sacc[kt]);
            }

        // -- inter-block output (independent of the scores): S^T A^T with the published state
        f32x4 oi[NT], oe[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            oi[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            oe[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const char* sa = sb + i16 * KP + (8 * g) * 2;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                Frag a;
                a.u = *(const u32x4*)(sa + (16 * nt) * KP + (32 * ks) * 2);
                oe[nt] = mfma16(a.v, Qf[ks].v, oe[nt]);
            }

        // -- mask the scores, round to bf16: they are B operands as they stand
        bf16x4 Pt[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            if (kt < W) {
                const float sc = (W - kt == 1) ? 1.0f : ((W - kt == 2) ? lam16 : lam32);
                f32x4 m;
#pragma unroll
                for (int j = 0; j < 4; ++j) m[j] = sacc[kt < W ? kt : 0][j] * (moff[j] * sc);
                Pt[kt] = to_bf16(m);
            } else if (kt == W) {
                f32x4 m;
#pragma unroll
                for (int j = 0; j < 4; ++j) m[j] = sacc[W][j] * mdiag[j];
                Pt[kt] = to_bf16(m);
            } else {
                Pt[kt] = bf16x4{0, 0, 0, 0};
            }
        }

        // -- intra-block output (transposed): O^T += C^T P^T, C read down the token axis
        const char* va = vb + (4 * g + (i16 >> 2)) * VP + (4 * (i16 & 3)) * 2;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            if (2 * p <= W) {
                Frag b;
                b.b[0] = Pt[2 * p];
                b.b[1] = Pt[2 * p + 1];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    Frag vf;
                    vf.h[0] = lds_tr16(va + (32 * p) * VP + (16 * nt) * 2);
                    vf.h[1] = lds_tr16(va + (32 * p + 16) * VP + (16 * nt) * 2);
                    oi[nt] = mfma16(vf.v, b.v, oi[nt]);
                }
            }
        }

        // -- combine and store: lane holds token (16W + i16), features 16nt + 4g .. +3
        if (more || (16 * W + i16) < valid) {     // every lane stores in a full block
            char* p = po + (long long)blk * step;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                f32x4 r;
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = oi[nt][j] + qscale * oe[nt][j];
                *(bf16x4*)(p + 32 * nt) = to_bf16(r);
            }
        }
        if (more) __syncthreads();
    }
}

// ------------------------------------------------------------------ state waves

template <int D, int DV>
__device__ __forceinline__ void run_state_wave(const Chain& ch, char* smem, int lane, int u) {
    using C = Cfg<D, DV>;
    constexpr int MT = C::MT, NT = C::NT, KP = C::KP, VP = C::VP;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    const int stid = u * 64 + lane;                 // 0..255 among the staging threads
    const int dk0 = u * (D / 4);
    const float lam = ch.lam;

    // lambda^(len-1-token) per MFMA k-slot, and lambda^len
    float ksc[2][8], lamB;
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

    // running state, fp32
    f32x4 st[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (ch.state_in) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    st[mt][nt][j] = ch.state_in[(size_t)(dk0 + 16 * mt + 4 * g + j) * D + 16 * nt + i16];
            } else {
                st[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    auto publish_state = [&](int buf) {
        char* sb = smem + C::SB + buf * C::SBYTES;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                *(bf16x4*)(sb + (16 * nt + i16) * KP + (dk0 + 16 * mt + 4 * g) * 2) = to_bf16(st[mt][nt]);
    };

    // staging cursors: this thread's first chunk of the B tile and of the C tile, block 0
    constexpr int KRPC = kStageThreads / (D / 8);    // tile rows covered per chunk index
    constexpr int VRPC = kStageThreads / (DV / 8);
    const int krow = stid / (D / 8), kch = stid % (D / 8);
    const int vrow = stid / (DV / 8), vch = stid % (DV / 8);
    const long long rs = ch.rev ? -ROW : ROW;        // byte stride between consecutive block rows
    const long long step = ch.rev ? -(long long)kBlock * ROW : (long long)kBlock * ROW;
    const char* pk = ch.b + (ch.rev ? (ch.N - 1 - krow) : (long long)krow) * ROW + kch * 16;
    const char* pa = ch.a + (ch.rev ? (ch.N - 1 - krow) : (long long)krow) * ROW + kch * 16;
    const char* pv = ch.c + (ch.rev ? (ch.N - 1 - vrow) : (long long)vrow) * ROW + vch * 16;
    // Two staging register sets: block b+1 is "ready" (landed or landing) while block b+2
    // is being fetched, so two blocks of loads are in flight per workgroup.  Loads are
    // unconditional; rows past the end of the last block read its last valid row and are
    // zeroed when staged.
    struct Stage { u32x4 a[C::KC]; u32x4 k[C::KC]; u32x4 v[C::VC]; };
    constexpr int kLoads = 2 * C::KC + C::VC;          // VMEM loads per block per thread
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };
    auto load_tiles = [&](Stage& t, int b) {
        b = b < ch.T ? b : ch.T - 1;       // past the end: re-read the last block (ignored)
        const int valid = valid_of(b);
        const char* k0 = pk + (long long)b * step;
        const char* a0 = pa + (long long)b * step;
        const char* v0 = pv + (long long)b * step;
#pragma unroll
        for (int c = 0; c < C::KC; ++c) {
            int r = c * KRPC + krow;
            r = (r < valid ? r : valid - 1) - krow;
            gload16(t.k[c], k0 + (long long)r * rs);
            gload16(t.a[c], a0 + (long long)r * rs);
        }
#pragma unroll
        for (int c = 0; c < C::VC; ++c) {
            int r = c * VRPC + vrow;
            r = (r < valid ? r : valid - 1) - vrow;
            gload16(t.v[c], v0 + (long long)r * rs);
        }
    };
    auto wait_tiles = [&](Stage& t, bool newer_in_flight) {
        // the loads of the following block are always issued after these
        if (newer_in_flight) { wait_vm_all<kLoads>(t.k); wait_vm_all<kLoads>(t.a); wait_vm_all<kLoads>(t.v); }
        else { wait_vm_all<0>(t.k); wait_vm_all<0>(t.a); wait_vm_all<0>(t.v); }
    };
    auto stage_to_lds = [&](const Stage& t, int buf, int valid) {
        char* kb = smem + C::KB + buf * C::KBYTES;
        char* ab = smem + C::AB + buf * C::KBYTES;
        char* vb = smem + C::VB + buf * C::VBYTES;
#pragma unroll
        for (int c = 0; c < C::KC; ++c) {
            const bool ok = c * KRPC + krow < valid;
            *(u32x4*)(kb + (c * KRPC + krow) * KP + kch * 16) = ok ? t.k[c] : u32x4{0, 0, 0, 0};
            *(u32x4*)(ab + (c * KRPC + krow) * KP + kch * 16) = ok ? t.a[c] : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int c = 0; c < C::VC; ++c)
            *(u32x4*)(vb + (c * VRPC + vrow) * VP + vch * 16) = (c * VRPC + vrow < valid) ? t.v[c] : u32x4{0, 0, 0, 0};
    };

    auto do_block = [&](int blk, Stage& ready, Stage& incoming) -> bool {
        const int cur = blk & 1;
        const bool more = blk + 1 < ch.T;
        const char* kb = smem + C::KB + cur * C::KBYTES;
        const char* vb = smem + C::VB + cur * C::VBYTES;

        load_tiles(incoming, blk + 2);     // global -> registers, two blocks ahead
        if (!more) {
            if (!ch.state_out) return false;   // the last update only feeds the returned state
            if (ch.last_valid != kBlock) set_block_len(ch.last_valid);
        }

        // -- C operand down the token axis, all four key tiles
        Frag Vf[2][NT];
        const char* va = vb + (4 * g + (i16 >> 2)) * VP + (4 * (i16 & 3)) * 2;
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                Vf[p][nt].h[0] = lds_tr16(va + (32 * p) * VP + (16 * nt) * 2);
                Vf[p][nt].h[1] = lds_tr16(va + (32 * p + 16) * VP + (16 * nt) * 2);
            }

        // -- S <- lambda^len S + (decayed B)^T C
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) st[mt][nt][j] *= lamB;
        const char* kt0 = kb + (4 * g + (i16 >> 2)) * KP + (dk0 + 4 * (i16 & 3)) * 2;
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                Frag a;
                a.h[0] = lds_tr16(kt0 + (32 * p) * KP + (16 * mt) * 2);
                a.h[1] = lds_tr16(kt0 + (32 * p + 16) * KP + (16 * mt) * 2);
                f32x8 af = __builtin_convertvector(a.v, f32x8);
#pragma unroll
                for (int j = 0; j < 8; ++j) af[j] *= ksc[p][j];
                a.v = __builtin_convertvector(af, bf16x8);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) st[mt][nt] = mfma16(a.v, Vf[p][nt].v, st[mt][nt]);
            }

        if (more) {
            publish_state(cur ^ 1);
            wait_tiles(ready, true);
            stage_to_lds(ready, cur ^ 1, valid_of(blk + 1));
            __syncthreads();
        }
        return more;
    };

    // prologue: block 0 tiles and the initial state copy into buffer 0; block 1 in flight
    Stage sa_, sb_;
#pragma unroll
    for (int c = 0; c < C::KC; ++c) sa_.k[c] = sb_.k[c] = sa_.a[c] = sb_.a[c] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < C::VC; ++c) sa_.v[c] = sb_.v[c] = u32x4{0, 0, 0, 0};
    load_tiles(sa_, 0);
    publish_state(0);
    wait_tiles(sa_, false);
    stage_to_lds(sa_, 0, valid_of(0));
    load_tiles(sa_, 1);
    __syncthreads();

    for (int blk = 0; blk < ch.T; blk += 2) {
        if (!do_block(blk, sa_, sb_)) break;
        if (!do_block(blk + 1, sb_, sa_)) break;
    }
    // prefetches past the last block were never consumed: retire them before the registers die
    wait_tiles(sa_, false);
    wait_tiles(sb_, false);

    if (ch.state_out) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    ch.state_out[(size_t)(dk0 + 16 * mt + 4 * g + j) * D + 16 * nt + i16] = st[mt][nt][j];
    }
}

template <int D, int DV>
__global__ __launch_bounds__(kThreads)
void pass_bf16_kernel(const PassBatch pb, const int nsplit) {
    using C = Cfg<D, DV>;
    __shared__ __attribute__((aligned(16))) char smem[C::TOTAL];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: role dispatch is a uniform branch

    int chain, within;
    map_workgroup(blockIdx.x, pb.count * nsplit, pb.chains, chain, within);
    const int pi = within / nsplit;
    const int split = within - pi * nsplit;
    const PassArgs P = pb.p[pi];

    Chain ch;
    const size_t chain_off = (size_t)chain * (size_t)pb.N * D * 2;
    const size_t col_off = (size_t)split * DV * 2;
    ch.a = (const char*)P.a + chain_off;
    ch.b = (const char*)P.b + chain_off;
    ch.c = (const char*)P.c + chain_off + col_off;
    ch.out = (char*)P.out + chain_off + col_off;
    ch.state_in = P.state_in ? P.state_in + (size_t)chain * D * D + (size_t)split * DV : nullptr;
    ch.state_out = P.state_out ? P.state_out + (size_t)chain * D * D + (size_t)split * DV : nullptr;
    ch.N = pb.N;
    ch.T = (int)((pb.N + kBlock - 1) / kBlock);
    ch.last_valid = (int)(pb.N - (long long)(ch.T - 1) * kBlock);
    ch.rev = P.rev;
    ch.lam = pb.decay[chain % pb.H];

    switch (wave) {
        case 0: run_output_wave<D, DV, 0>(ch, smem, lane); break;
        case 1: run_output_wave<D, DV, 1>(ch, smem, lane); break;
        case 2: run_output_wave<D, DV, 2>(ch, smem, lane); break;
        case 3: run_output_wave<D, DV, 3>(ch, smem, lane); break;
        default: run_state_wave<D, DV>(ch, smem, lane, wave - 4); break;
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
    if (D == 128 && dv == 64) return launch_t<128, 64>(pb, stream);
    if (D == 128 && dv == 32) return launch_t<128, 32>(pb, stream);
    if (D == 64 && dv == 64) return launch_t<64, 64>(pb, stream);
    if (D == 64 && dv == 32) return launch_t<64, 32>(pb, stream);
    return hipErrorInvalidValue;
}

}  // namespace ltn
