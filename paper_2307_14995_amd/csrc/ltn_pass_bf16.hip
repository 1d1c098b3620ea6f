// bf16 MFMA kernels for Lightning Attention on gfx950 (MI355X).
//
// Building block: the decayed linear-attention pass (arXiv 2307.14995, Sec. 3.2.1 with
// the decay mask of Eq. 1; recurrence of Sec. 3.3, Algorithm 2, taken 64 tokens at a
// time).  For each chain (batch, head) and a slice of DV value columns, per block i of
// 64 tokens, with S_i the running [D x DV] state:
//
//     P    = (A_i B_i^T) (.) M,       M[r,c] = lambda^(r-c) for r >= c else 0
//     O_i  = P C_i + diag(lambda^(r+1)) A_i S_i
//     S_i+1 = lambda^len S_i + (diag(lambda^(len-1-c)) B_i)^T C_i
//
// (A,B,C) = (Q,K,V) gives the forward output O; the gradients are the same pass with
// permuted operands, dQ = pass(dO,V,K), and on a reversed token axis dV = pass(K,Q,dO),
// dK = pass(V,dO,Q) (derivative of the definition; App. B Algorithm 4 corrected).
//
// Two workgroup bodies, both 512 threads = 8 wavefronts in two roles (two waves per
// SIMD, so one role's LDS/VALU latencies hide under the other's MFMAs):
//
//   pass body    one pass for a DV-column slice: forward, and dQ in the backward.
//   dK/dV body   both reversed-axis passes for one half of the columns.  They share all
//                four operand tiles (Q and dO are each the B operand of one pass and the C
//                operand of the other; K and V are the A operands), so a chain's tokens
//                are read once for two gradients instead of twice.
//
//   * output waves 0..3: wave w owns token rows 16w..16w+15 of the block.  It forms the
//     transposed score tiles P^T[key tile][its rows] with 16x16x32 bf16 MFMA; the fp32
//     accumulators already sit in the lane layout the next MFMA wants as its B operand
//     (the contraction index is permuted identically on both operands), so the masked
//     scores never leave registers.  The output is produced transposed
//     (O^T = C^T P^T + S^T A^T): every lane holds four consecutive output features of
//     one token -> 8-byte stores.
//   * state waves 4..7: wave u owns state rows [u*D/4, (u+1)*D/4) x DV in fp32
//     accumulators for the whole sequence, applies S <- lambda^len S + (decayed B)^T C
//     and publishes a bf16 copy [dv][dk] to LDS, which the output waves read as the A
//     operand of S^T A^T.  These waves also stage the coming blocks' tiles
//     global -> registers -> LDS, two blocks ahead.
//   * LDS tiles and state copies are double buffered: one barrier per block.  Row
//     pitches are 32 bytes over a multiple of 256 (measured best for the 16-byte row
//     reads and the transpose reads).  Operands read "down the token axis" (C for P C,
//     B^T and C for the state update) use ds_read_b64_tr_b16.
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
    static constexpr int KP = D * 2 + 32;      // LDS row pitch of a full-width tile / state copy (bytes)
    static constexpr int VP = DV * 2 + 32;     // LDS row pitch of a DV-wide C tile (bytes)
    static constexpr int KC = D / 32;          // 16-byte chunks of a full tile staged per staging thread
    static constexpr int VC = DV / 32;         // 16-byte chunks of a DV-wide tile staged per staging thread
    static constexpr int KBYTES = kBlock * KP;
    static constexpr int VBYTES = kBlock * VP;
    static constexpr int SBYTES = DV * KP;
    // pass body: B tile, C tile (DV wide), state copy; two buffers each
    static constexpr int KB = 0;
    static constexpr int VB = 2 * KBYTES;
    static constexpr int SB = VB + 2 * VBYTES;
    static constexpr int PASS_TOTAL = SB + 2 * SBYTES;
    // dK/dV body: Q tile, dO tile (full width), two state copies; two buffers each
    static constexpr int QB = 0;
    static constexpr int GB = 2 * KBYTES;
    static constexpr int S1B = 4 * KBYTES;
    static constexpr int S2B = S1B + 2 * SBYTES;
    static constexpr int KV_TOTAL = S2B + 2 * SBYTES;
    static constexpr int KRPC = kStageThreads / (D / 8);    // tile rows covered per chunk index
    static constexpr int VRPC = kStageThreads / (DV / 8);
};

// Per-lane decay constants of an output wave (non-negative exponents only).
template <int W>
struct OutConsts {
    float qscale, mdiag[4], moff[4], lam16, lam32;
    __device__ __forceinline__ void init(float lam, int g, int i16) {
        qscale = decay_pow(lam, 16 * W + i16 + 1);      // lambda^(r+1), r = row in block
        const int d0 = i16 - 4 * g;                      // (row - key) in a diagonal tile at j = 0
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            mdiag[j] = (d0 - j >= 0) ? decay_pow(lam, d0 - j) : 0.0f;
            moff[j] = decay_pow(lam, 16 + d0 - j);       // 16 + d0 - j >= 1
        }
        lam16 = decay_pow(lam, 16);
        lam32 = decay_pow(lam, 32);
    }
};

// One pass's output for the token strip of output wave W in the current block:
//   out^T[DV x 16] = Ct^T P^T + diag(qscale) S^T A^T,   P^T = (Bt A^T) (.) M^T
//   btile : full-width B tile in LDS (rows = tokens)
//   ctile : C tile in LDS, already offset to this slice's first column; pitch CP
//   scopy : bf16 state copy [DV][D] in LDS
//   Af    : A fragments of the strip (zero for rows past the end)
//   out   : global address of this lane's token row, slice column 4g
template <int D, int DV, int W, int CP>
__device__ __forceinline__ void output_pass(const char* btile, const char* ctile, const char* scopy,
                                            const Frag (&Af)[D / 32], const OutConsts<W>& k,
                                            char* out, bool store, int g, int i16) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, NT = C::NT, KP = C::KP;

    // -- transposed scores P^T[key tile kt <= W][own 16 rows]
    f32x4 sacc[W + 1];
#pragma unroll
    for (int kt = 0; kt <= W; ++kt) sacc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
    const char* ka = btile + i16 * KP + (8 * g) * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int kt = 0; kt <= W; ++kt) {
            Frag a;
            a.u = *(const u32x4*)(ka + (16 * kt) * KP + (32 * ks) * 2);
            sacc[kt] = mfma16(a.v, Af[ks].v, sacc[kt]);
        }

    // -- inter-block part (independent of the scores): S^T A^T with the published state
    f32x4 oi[NT], oe[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        oi[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        oe[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const char* sa = scopy + i16 * KP + (8 * g) * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            Frag a;
            a.u = *(const u32x4*)(sa + (16 * nt) * KP + (32 * ks) * 2);
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
    const char* va = ctile + (4 * g + (i16 >> 2)) * CP + (4 * (i16 & 3)) * 2;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        if (2 * p <= W) {
            Frag b;
            b.b[0] = Pt[2 * p];
            b.b[1] = Pt[2 * p + 1];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                Frag vf;
                vf.h[0] = lds_tr16(va + (32 * p) * CP + (16 * nt) * 2);
                vf.h[1] = lds_tr16(va + (32 * p + 16) * CP + (16 * nt) * 2);
                oi[nt] = mfma16(vf.v, b.v, oi[nt]);
            }
        }
    }

    // -- combine and store: lane holds one token, features 16nt + 4g .. +3
    if (store) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            f32x4 r;
#pragma unroll
            for (int j = 0; j < 4; ++j) r[j] = oi[nt][j] + k.qscale * oe[nt][j];
            *(bf16x4*)(out + 32 * nt) = to_bf16(r);
        }
    }
}

// Decay factors a state wave applies to the B^T fragments: lambda^(len-1-token) per MFMA
// k-slot, and lambda^len for the state itself.
struct StateConsts {
    float ksc[2][8], lamB;
    __device__ __forceinline__ void set_block_len(float lam, int len, int g) {
        lamB = decay_pow(lam, len);
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int tok = 32 * p + 16 * (j >> 2) + 4 * g + (j & 3);
                ksc[p][j] = (tok < len) ? decay_pow(lam, len - 1 - tok) : 0.0f;
            }
    }
};

// S[dk0 .. dk0 + D/4, :] <- lambda^len S + (decayed Bt)^T Ct for the rows this state wave owns.
//   btile : full-width B tile (rows = tokens); ctile : C tile offset to the slice, pitch CP
template <int D, int DV, int CP>
__device__ __forceinline__ void state_update(f32x4 (&st)[D / 64][DV / 16], const char* btile, const char* ctile,
                                             const StateConsts& k, int dk0, int g, int i16) {
    using C = Cfg<D, DV>;
    constexpr int MT = C::MT, NT = C::NT, KP = C::KP;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j) st[mt][nt][j] *= k.lamB;
    const char* va = ctile + (4 * g + (i16 >> 2)) * CP + (4 * (i16 & 3)) * 2;
    const char* kt0 = btile + (4 * g + (i16 >> 2)) * KP + (dk0 + 4 * (i16 & 3)) * 2;
#pragma unroll
    for (int p = 0; p < 2; ++p) {          // 32 tokens per step
        Frag Vf[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            Vf[nt].h[0] = lds_tr16(va + (32 * p) * CP + (16 * nt) * 2);
            Vf[nt].h[1] = lds_tr16(va + (32 * p + 16) * CP + (16 * nt) * 2);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            Frag a;
            a.h[0] = lds_tr16(kt0 + (32 * p) * KP + (16 * mt) * 2);
            a.h[1] = lds_tr16(kt0 + (32 * p + 16) * KP + (16 * mt) * 2);
            f32x8 af = __builtin_convertvector(a.v, f32x8);
#pragma unroll
            for (int j = 0; j < 8; ++j) af[j] *= k.ksc[p][j];
            a.v = __builtin_convertvector(af, bf16x8);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) st[mt][nt] = mfma16(a.v, Vf[nt].v, st[mt][nt]);
        }
    }
}

template <int D, int DV>
__device__ __forceinline__ void publish_state(const f32x4 (&st)[D / 64][DV / 16], char* scopy, int dk0, int g, int i16) {
    using C = Cfg<D, DV>;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < C::NT; ++nt)
            *(bf16x4*)(scopy + (16 * nt + i16) * C::KP + (dk0 + 16 * mt + 4 * g) * 2) = to_bf16(st[mt][nt]);
}

// A full-width tile (64 rows x D) staged by the 256 staging threads: KC chunks per thread.
template <int D, int DV>
struct TileRegs {
    u32x4 r[Cfg<D, DV>::KC];
};
// global -> registers; rows >= valid read row valid-1 instead (zeroed when staged)
template <int D, int DV>
__device__ __forceinline__ void load_full_tile(TileRegs<D, DV>& t, const char* p0, int krow, long long rs, int valid) {
    using C = Cfg<D, DV>;
#pragma unroll
    for (int c = 0; c < C::KC; ++c) {
        int r = c * C::KRPC + krow;
        r = (r < valid ? r : valid - 1) - krow;
        gload16(t.r[c], p0 + (long long)r * rs);
    }
}
template <int D, int DV>
__device__ __forceinline__ void stage_full_tile(const TileRegs<D, DV>& t, char* tile, int krow, int kch, int valid) {
    using C = Cfg<D, DV>;
#pragma unroll
    for (int c = 0; c < C::KC; ++c)
        *(u32x4*)(tile + (c * C::KRPC + krow) * C::KP + kch * 16) =
            (c * C::KRPC + krow < valid) ? t.r[c] : u32x4{0, 0, 0, 0};
}

struct Chain {            // what every wave of the workgroup knows about its problem
    const char* a;        // pass body: operands offset to this chain (c/out also to the slice)
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

// =============================================================== pass body

template <int D, int DV, int W>
__device__ __forceinline__ void pass_output_wave(const Chain& ch, char* smem, int lane) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, NT = C::NT;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    OutConsts<W> k;
    k.init(ch.lam, g, i16);

    // cursors for this lane's token row (16W + i16) of block 0
    const long long r0 = ch.rev ? (ch.N - 1 - (16 * W + i16)) : (long long)(16 * W + i16);
    const long long rs = ch.rev ? -ROW : ROW;
    const long long step = kBlock * rs;
    const char* pa = ch.a + r0 * ROW + (8 * g) * 2;
    char* po = ch.out + r0 * ROW + (4 * g) * 2;
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };

    // A fragments straight from global memory (only this wave needs them): three rotating
    // register sets, loaded two blocks ahead.
    struct ASet { u32x4 a[KS]; };
    auto load_a = [&](ASet& s, int b) {
        b = b < ch.T ? b : ch.T - 1;       // past the end: re-read the last block (ignored)
        const int row = 16 * W + i16, valid = valid_of(b);
        long long off = (long long)b * step;
        if (row >= valid) off -= (long long)(row - (valid - 1)) * rs;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) gload16(s.a[ks], pa + off + ks * 64);
    };
    // Set(blk) was issued two blocks ago; since then this wave issued the NT stores of
    // each of two blocks and the KS loads of set(blk+1).
    constexpr int kAfter = 2 * NT + KS;

    auto do_block = [&](int blk, ASet& cur_set, ASet& incoming) {
        const int cur = blk & 1;
        const bool more = blk + 1 < ch.T;
        const bool row_ok = (16 * W + i16) < valid_of(blk);
        wait_vm_all<kAfter>(cur_set.a);
        Frag Af[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {      // rows past the end are zeroed in place (landed data)
            if (!row_ok) cur_set.a[ks] = u32x4{0, 0, 0, 0};
            Af[ks].u = cur_set.a[ks];
        }
        load_a(incoming, blk + 2);
        output_pass<D, DV, W, C::VP>(smem + C::KB + cur * C::KBYTES, smem + C::VB + cur * C::VBYTES,
                                     smem + C::SB + cur * C::SBYTES, Af, k,
                                     po + (long long)blk * step, more || row_ok, g, i16);
        if (more) __syncthreads();
    };

    ASet s0, s1, s2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s0.a[ks] = s1.a[ks] = s2.a[ks] = u32x4{0, 0, 0, 0};
    load_a(s0, 0);
    load_a(s1, 1);
    wait_vm_all<0>(s0.a);                  // blocks 0 and 1 are retired here, so the
    wait_vm_all<0>(s1.a);                  // steady-state count is safe for them too
    __syncthreads();                       // block 0 tiles and the initial state copy are in LDS

    for (int blk = 0; blk < ch.T; blk += 3) {
        do_block(blk, s0, s2);
        if (blk + 1 < ch.T) do_block(blk + 1, s1, s0);
        if (blk + 2 < ch.T) do_block(blk + 2, s2, s1);
    }
    // the last two prefetches were never consumed: retire them before the registers die
    wait_vm_all<0>(s0.a);
    wait_vm_all<0>(s1.a);
    wait_vm_all<0>(s2.a);
}

template <int D, int DV>
__device__ __forceinline__ void pass_state_wave(const Chain& ch, char* smem, int lane, int u) {
    using C = Cfg<D, DV>;
    constexpr int MT = C::MT, NT = C::NT;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    const int stid = u * 64 + lane;                 // 0..255 among the staging threads
    const int dk0 = u * (D / 4);
    StateConsts k;
    k.set_block_len(ch.lam, kBlock, g);

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

    // staging cursors: this thread's first chunk of each tile, block 0
    const int krow = stid / (D / 8), kch = stid % (D / 8);
    const int vrow = stid / (DV / 8), vch = stid % (DV / 8);
    const long long rs = ch.rev ? -ROW : ROW;        // byte stride between consecutive block rows
    const long long step = ch.rev ? -(long long)kBlock * ROW : (long long)kBlock * ROW;
    const char* pk = ch.b + (ch.rev ? (ch.N - 1 - krow) : (long long)krow) * ROW + kch * 16;
    const char* pv = ch.c + (ch.rev ? (ch.N - 1 - vrow) : (long long)vrow) * ROW + vch * 16;

    // Two staging register sets: block b+1 is "ready" (landed or landing) while block b+2
    // is being fetched, so two blocks of loads are in flight per workgroup.  Loads are
    // unconditional; past the last block they re-read it (ignored).
    struct Stage { TileRegs<D, DV> k; u32x4 v[C::VC]; };
    constexpr int kLoads = C::KC + C::VC;              // VMEM loads per block per thread
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };
    auto load_tiles = [&](Stage& t, int b) {
        b = b < ch.T ? b : ch.T - 1;
        const int valid = valid_of(b);
        load_full_tile<D, DV>(t.k, pk + (long long)b * step, krow, rs, valid);
        const char* v0 = pv + (long long)b * step;
#pragma unroll
        for (int c = 0; c < C::VC; ++c) {
            int r = c * C::VRPC + vrow;
            r = (r < valid ? r : valid - 1) - vrow;
            gload16(t.v[c], v0 + (long long)r * rs);
        }
    };
    auto wait_tiles = [&](Stage& t, bool newer_in_flight) {
        // the loads of the following block are always issued after these
        if (newer_in_flight) { wait_vm_all<kLoads>(t.k.r); wait_vm_all<kLoads>(t.v); }
        else { wait_vm_all<0>(t.k.r); wait_vm_all<0>(t.v); }
    };
    auto stage_to_lds = [&](const Stage& t, int buf, int valid) {
        stage_full_tile<D, DV>(t.k, smem + C::KB + buf * C::KBYTES, krow, kch, valid);
        char* vb = smem + C::VB + buf * C::VBYTES;
#pragma unroll
        for (int c = 0; c < C::VC; ++c)
            *(u32x4*)(vb + (c * C::VRPC + vrow) * C::VP + vch * 16) =
                (c * C::VRPC + vrow < valid) ? t.v[c] : u32x4{0, 0, 0, 0};
    };

    auto do_block = [&](int blk, Stage& ready, Stage& incoming) -> bool {
        const int cur = blk & 1;
        const bool more = blk + 1 < ch.T;
        load_tiles(incoming, blk + 2);     // global -> registers, two blocks ahead
        if (!more) {
            if (!ch.state_out) return false;   // the last update only feeds the returned state
            if (ch.last_valid != kBlock) k.set_block_len(ch.lam, ch.last_valid, g);
        }
        state_update<D, DV, C::VP>(st, smem + C::KB + cur * C::KBYTES, smem + C::VB + cur * C::VBYTES, k, dk0, g, i16);
        if (more) {
            publish_state<D, DV>(st, smem + C::SB + (cur ^ 1) * C::SBYTES, dk0, g, i16);
            wait_tiles(ready, true);
            stage_to_lds(ready, cur ^ 1, valid_of(blk + 1));
            __syncthreads();
        }
        return more;
    };

    // prologue: block 0 tiles and the initial state copy into buffer 0; block 1 in flight
    Stage sa_, sb_;
#pragma unroll
    for (int c = 0; c < C::KC; ++c) sa_.k.r[c] = sb_.k.r[c] = u32x4{0, 0, 0, 0};
#pragma unroll
    for (int c = 0; c < C::VC; ++c) sa_.v[c] = sb_.v[c] = u32x4{0, 0, 0, 0};
    load_tiles(sa_, 0);
    publish_state<D, DV>(st, smem + C::SB, dk0, g, i16);
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
__device__ __forceinline__ void pass_body(const PassBatch& pb, int nsplit, int wg, char* smem, int wave, int lane) {
    int chain, within;
    map_workgroup(wg, pb.count * nsplit, pb.chains, chain, within);
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
        case 0: pass_output_wave<D, DV, 0>(ch, smem, lane); break;
        case 1: pass_output_wave<D, DV, 1>(ch, smem, lane); break;
        case 2: pass_output_wave<D, DV, 2>(ch, smem, lane); break;
        case 3: pass_output_wave<D, DV, 3>(ch, smem, lane); break;
        default: pass_state_wave<D, DV>(ch, smem, lane, wave - 4); break;
    }
}

// =============================================================== dK/dV body
//
// Both reversed-axis gradient passes for one half (DV = D/2 columns) of a chain:
//   dV[:, half] = pass_rev(A = K, B = Q,  C = dO[:, half])   state S1 = sum decayed q^T dO[half]
//   dK[:, half] = pass_rev(A = V, B = dO, C = Q[:, half])    state S2 = sum decayed dO^T q[half]
// Q and dO tiles live in LDS (full width: each is the B operand of one pass and, through a
// column offset, the C operand of the other); K and V are only A operands, so each output
// wave fetches its own 16 rows of them straight from global memory, two blocks ahead.

struct KvChain {
    const char* q;        // offset to this chain
    const char* k;
    const char* v;
    const char* g;        // dO
    char* dk;             // offset to this chain and column half
    char* dv;
    long long N;
    int T, last_valid, half;
    float lam;
};

template <int D, int DV, int W>
__device__ __forceinline__ void kv_output_wave(const KvChain& ch, char* smem, int lane) {
    using C = Cfg<D, DV>;
    constexpr int KS = C::KS, NT = C::NT, KP = C::KP;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    OutConsts<W> k;
    k.init(ch.lam, g, i16);

    // reversed token axis: local row r of block b is global row N-1-(64b + r)
    const long long r0 = ch.N - 1 - (16 * W + i16);
    constexpr long long step = -(long long)kBlock * ROW;
    const char* pk = ch.k + r0 * ROW + (8 * g) * 2;
    const char* pv = ch.v + r0 * ROW + (8 * g) * 2;
    char* pdk = ch.dk + r0 * ROW + (4 * g) * 2;
    char* pdv = ch.dv + r0 * ROW + (4 * g) * 2;
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };

    // A fragments of both passes: three rotating register sets, loaded two blocks ahead.
    struct ASet { u32x4 k[KS]; u32x4 v[KS]; };
    auto load_a = [&](ASet& s, int b) {
        b = b < ch.T ? b : ch.T - 1;       // past the end: re-read the last block (ignored)
        const int row = 16 * W + i16, valid = valid_of(b);
        long long off = (long long)b * step;
        if (row >= valid) off += (long long)(row - (valid - 1)) * ROW;   // reversed axis: previous local row is +ROW
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            gload16(s.k[ks], pk + off + ks * 64);
            gload16(s.v[ks], pv + off + ks * 64);
        }
    };
    // Set(blk) was issued two blocks ago; since then this wave issued the 2*NT stores of
    // each of two blocks and the 2*KS loads of set(blk+1).
    constexpr int kAfter = 4 * NT + 2 * KS;
    static_assert(kAfter <= 63, "vmcnt field");

    auto do_block = [&](int blk, ASet& cur_set, ASet& incoming) {
        const int cur = blk & 1;
        const bool more = blk + 1 < ch.T;
        const int valid = valid_of(blk);
        const bool row_ok = (16 * W + i16) < valid;
        wait_vm_all<kAfter>(cur_set.k);
        wait_vm_all<kAfter>(cur_set.v);
        Frag Kf[KS], Vf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {      // rows past the end are zeroed in place (landed data)
            if (!row_ok) cur_set.k[ks] = cur_set.v[ks] = u32x4{0, 0, 0, 0};
            Kf[ks].u = cur_set.k[ks];
            Vf[ks].u = cur_set.v[ks];
        }
        load_a(incoming, blk + 2);

        const char* qt = smem + C::QB + cur * C::KBYTES;
        const char* gt = smem + C::GB + cur * C::KBYTES;
        const long long o = (long long)blk * step;
        const bool store = more || row_ok;
        // dV = pass(K, Q, dO[:, half])
        output_pass<D, DV, W, KP>(qt, gt + ch.half * DV * 2, smem + C::S1B + cur * C::SBYTES, Kf, k, pdv + o, store, g, i16);
        // dK = pass(V, dO, Q[:, half])
        output_pass<D, DV, W, KP>(gt, qt + ch.half * DV * 2, smem + C::S2B + cur * C::SBYTES, Vf, k, pdk + o, store, g, i16);
        if (more) __syncthreads();
    };

    ASet s0, s1, s2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        s0.k[ks] = s0.v[ks] = s1.k[ks] = s1.v[ks] = s2.k[ks] = s2.v[ks] = u32x4{0, 0, 0, 0};
    load_a(s0, 0);
    load_a(s1, 1);
    wait_vm_all<0>(s0.k); wait_vm_all<0>(s0.v);      // blocks 0 and 1 are retired here, so the
    wait_vm_all<0>(s1.k); wait_vm_all<0>(s1.v);      // steady-state count is safe for them too
    __syncthreads();                                 // block 0 tiles and state copies are in LDS

    for (int blk = 0; blk < ch.T; blk += 3) {
        do_block(blk, s0, s2);
        if (blk + 1 < ch.T) do_block(blk + 1, s1, s0);
        if (blk + 2 < ch.T) do_block(blk + 2, s2, s1);
    }
    // the last two prefetches were never consumed: retire them before the registers die
    wait_vm_all<0>(s0.k); wait_vm_all<0>(s0.v);
    wait_vm_all<0>(s1.k); wait_vm_all<0>(s1.v);
    wait_vm_all<0>(s2.k); wait_vm_all<0>(s2.v);
}

template <int D, int DV>
__device__ __forceinline__ void kv_state_wave(const KvChain& ch, char* smem, int lane, int u) {
    using C = Cfg<D, DV>;
    constexpr int MT = C::MT, NT = C::NT, KP = C::KP;
    constexpr long long ROW = D * 2;
    const int g = lane >> 4, i16 = lane & 15;
    const int stid = u * 64 + lane;
    const int dk0 = u * (D / 4);
    StateConsts k;
    k.set_block_len(ch.lam, kBlock, g);      // a short last block never updates the states

    f32x4 st1[MT][NT], st2[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            st1[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            st2[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    const int krow = stid / (D / 8), kch = stid % (D / 8);
    constexpr long long rs = -ROW;                   // reversed token axis
    constexpr long long step = -(long long)kBlock * ROW;
    const char* pq = ch.q + (ch.N - 1 - krow) * ROW + kch * 16;
    const char* pg = ch.g + (ch.N - 1 - krow) * ROW + kch * 16;

    struct Stage { TileRegs<D, DV> q, g; };
    constexpr int kLoads = 2 * C::KC;
    auto valid_of = [&](int b) { return (b + 1 == ch.T) ? ch.last_valid : kBlock; };
    auto load_tiles = [&](Stage& t, int b) {
        b = b < ch.T ? b : ch.T - 1;
        const int valid = valid_of(b);
        load_full_tile<D, DV>(t.q, pq + (long long)b * step, krow, rs, valid);
        load_full_tile<D, DV>(t.g, pg + (long long)b * step, krow, rs, valid);
    };
    auto wait_tiles = [&](Stage& t, bool newer_in_flight) {
        if (newer_in_flight) { wait_vm_all<kLoads>(t.q.r); wait_vm_all<kLoads>(t.g.r); }
        else { wait_vm_all<0>(t.q.r); wait_vm_all<0>(t.g.r); }
    };
    auto stage_to_lds = [&](const Stage& t, int buf, int valid) {
        stage_full_tile<D, DV>(t.q, smem + C::QB + buf * C::KBYTES, krow, kch, valid);
        stage_full_tile<D, DV>(t.g, smem + C::GB + buf * C::KBYTES, krow, kch, valid);
    };

    // One staging set, fetched one block ahead: a block of this body carries two passes'
    // worth of math, so one block time already covers the load latency, and the registers
    // of a second set are needed for the second state.
    Stage sa_;
#pragma unroll
    for (int c = 0; c < C::KC; ++c) sa_.q.r[c] = sa_.g.r[c] = u32x4{0, 0, 0, 0};
    load_tiles(sa_, 0);
    publish_state<D, DV>(st1, smem + C::S1B, dk0, g, i16);
    publish_state<D, DV>(st2, smem + C::S2B, dk0, g, i16);
    wait_tiles(sa_, false);
    stage_to_lds(sa_, 0, valid_of(0));
    __syncthreads();

    for (int blk = 0; blk + 1 < ch.T; ++blk) {     // no state is returned: the last block needs no update
        const int cur = blk & 1;
        load_tiles(sa_, blk + 1);
        const char* qt = smem + C::QB + cur * C::KBYTES;
        const char* gt = smem + C::GB + cur * C::KBYTES;
        // S1 <- lambda^64 S1 + (decayed Q)^T dO[:, half];   S2 <- lambda^64 S2 + (decayed dO)^T Q[:, half]
        state_update<D, DV, KP>(st1, qt, gt + ch.half * DV * 2, k, dk0, g, i16);
        publish_state<D, DV>(st1, smem + C::S1B + (cur ^ 1) * C::SBYTES, dk0, g, i16);
        state_update<D, DV, KP>(st2, gt, qt + ch.half * DV * 2, k, dk0, g, i16);
        publish_state<D, DV>(st2, smem + C::S2B + (cur ^ 1) * C::SBYTES, dk0, g, i16);
        wait_tiles(sa_, false);
        stage_to_lds(sa_, cur ^ 1, valid_of(blk + 1));
        __syncthreads();
    }
}

template <int D, int DV>
__device__ __forceinline__ void kv_body(const BwdBatch& bb, int wg, char* smem, int wave, int lane) {
    // two halves of a chain sit 8 workgroup ids apart (same XCD, shared L2) when possible
    int chain, half;
    map_workgroup(wg, 2, bb.chains, chain, half);
    KvChain ch;
    const size_t chain_off = (size_t)chain * (size_t)bb.N * D * 2;
    ch.q = (const char*)bb.q + chain_off;
    ch.k = (const char*)bb.k + chain_off;
    ch.v = (const char*)bb.v + chain_off;
    ch.g = (const char*)bb.d_o + chain_off;
    ch.dk = (char*)bb.dk + chain_off + (size_t)half * DV * 2;
    ch.dv = (char*)bb.dv + chain_off + (size_t)half * DV * 2;
    ch.N = bb.N;
    ch.T = (int)((bb.N + kBlock - 1) / kBlock);
    ch.last_valid = (int)(bb.N - (long long)(ch.T - 1) * kBlock);
    ch.half = half;
    ch.lam = bb.decay[chain % bb.H];
    switch (wave) {
        case 0: kv_output_wave<D, DV, 0>(ch, smem, lane); break;
        case 1: kv_output_wave<D, DV, 1>(ch, smem, lane); break;
        case 2: kv_output_wave<D, DV, 2>(ch, smem, lane); break;
        case 3: kv_output_wave<D, DV, 3>(ch, smem, lane); break;
        default: kv_state_wave<D, DV>(ch, smem, lane, wave - 4); break;
    }
}

// =============================================================== kernels

template <int D, int DV>
__global__ __launch_bounds__(kThreads)
void pass_bf16_kernel(const PassBatch pb, const int nsplit) {
    __shared__ __attribute__((aligned(16))) char smem[Cfg<D, DV>::PASS_TOTAL];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: role dispatch is a uniform branch
    pass_body<D, DV>(pb, nsplit, blockIdx.x, smem, wave, tid & 63);
}

// Backward in one launch: the first 2*chains workgroups run the dK/dV body, the
// remaining 2*chains run the dQ pass (DV = D/2 slices) as the first ones drain.
template <int D>
__global__ __launch_bounds__(kThreads)
void bwd_bf16_kernel(const BwdBatch bb) {
    constexpr int DV = D / 2;
    using C = Cfg<D, DV>;
    constexpr int LDS = C::KV_TOTAL > C::PASS_TOTAL ? C::KV_TOTAL : C::PASS_TOTAL;
    __shared__ __attribute__((aligned(16))) char smem[LDS];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wg = blockIdx.x;
    if (wg < 2 * bb.chains) {
        kv_body<D, DV>(bb, wg, smem, wave, tid & 63);
    } else {
        PassBatch pb = {};
        pb.p[0] = PassArgs{bb.d_o, bb.v, bb.k, bb.dq, nullptr, nullptr, 0};
        pb.count = 1;
        pb.decay = bb.decay;
        pb.chains = bb.chains;
        pb.H = bb.H;
        pb.N = bb.N;
        pass_body<D, DV>(pb, 2, wg - 2 * bb.chains, smem, wave, tid & 63);
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

hipError_t launch_bwd_bf16(const BwdBatch& bb, int D, hipStream_t stream) {
    const long long wgs = 4LL * bb.chains;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (D == 128) hipLaunchKernelGGL((bwd_bf16_kernel<128>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, bb);
    else if (D == 64) hipLaunchKernelGGL((bwd_bf16_kernel<64>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, bb);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ltn
