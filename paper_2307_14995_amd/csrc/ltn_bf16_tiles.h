// Device-side building blocks shared by the bf16 MFMA kernels of this library (gfx950):
// MFMA operand fragments, direct global -> LDS tile loads, the swizzled LDS tile layout and
// the regrouped 16-byte output stores.  Internal; included by the kernel sources only.
#pragma once
#include <type_traits>
#include <utility>
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

// Source of rows past the end of a short last block.
static __device__ __attribute__((aligned(256))) const unsigned char kZeros[256] = {};

// Direct global -> LDS loads are issued from inline assembly and waited for with explicit
// vmcnt counts (the compiler does not model their LDS side).  VMEM operations retire in
// issue order, so "vmcnt(n)" with n = the number of VMEM operations this wave issued after
// the wanted ones is exact; a smaller n is safe.
// Direct global -> LDS load: the wave writes 64 consecutive 16-byte LDS slots starting at
// the wave-uniform LDS byte address `lds`; lane i fills slot i from its own global address.
__device__ __forceinline__ void dma16(unsigned lds, const char* g) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds), "v"(g) : "memory", "m0");
}
// The same load with a wave-uniform 64-bit base (scalar registers) and a 32-bit unsigned
// per-lane byte offset: no per-lane 64-bit address arithmetic at the point of issue.
__device__ __forceinline__ void dma16s(unsigned lds, const char* base, unsigned off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds), "v"(off), "s"(base) : "memory", "m0");
}
// The same with only the lanes of `mask` taking part (wave-uniform; all 64 lanes are active at
// the call): the other lanes' LDS slots are left as they are.  EXEC is put back inside the
// statement.
__device__ __forceinline__ void dma16s_masked(unsigned lds, const char* base, unsigned off, unsigned long long mask) {
    unsigned long long saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %4\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved) : "s"(lds), "v"(off), "s"(base), "s"(mask) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_dma() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

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

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(const F& f, std::integer_sequence<int, Is...>) {
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(const F& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// Unpadded row-major LDS tile of COLS bf16 columns whose 16-byte chunks are XOR-swizzled
// with the row: chunk c of row r lives at chunk position c ^ key(r).  The key is built so
// that (i) 8 consecutive rows put a given 32-byte chunk pair on 8 different bank groups
// (what a transpose read or an 8-byte state-copy write touches per half wave) and (ii) 16
// consecutive rows put a given 16-byte chunk on 16 different ones (a 16-byte row read per
// quarter wave).  Adding a multiple of 16 rows does not change the key, so row-block
// offsets stay compile-time immediates.
template <int COLS>
struct Swz {
    static constexpr int RB = COLS * 2;        // bytes per row
    static constexpr int CPR = RB / 16;        // chunks per row
    static constexpr int RPB = RB >= 256 ? 1 : 256 / RB;   // rows per 256 bytes (one pass over the banks)
    static constexpr int KC = CPR < 16 ? CPR : 16;         // chunk positions the key permutes (a bank pass)
    static constexpr int BYTES = kBlock * RB;  // a 64-row tile
    static constexpr int NI = BYTES / 1024;    // wave-wide direct loads per tile
    static_assert(COLS == 256 || COLS == 128 || COLS == 64 || COLS == 32, "tile widths");
    __host__ __device__ static constexpr int key(int r) {
        // q: index of the row's 256-byte group member
        return (((r / RPB) % (KC / 2)) << 1) | (((r / RPB) / (KC / 2)) & 1);
    }
    __device__ static __forceinline__ int off(int r, int c) { return r * RB + ((c ^ key(r)) << 4); }
};

// Direct global -> LDS fetch of one 64-row tile of COLS columns by four waves (u = 0..3),
// every lane with a full 64-bit address (the quadratic comparison kernels; the pass kernel uses
// TileDmaU below).
// Wave u issues the wave-wide loads j = u, u+4, ...; load j fills LDS slots 64j .. 64j+63
// (slot s = row s / CPR, chunk position s % CPR).  `src[i]` is this lane's byte offset
// from the block's first row for its i-th load; `row[i]` the tile row it fetches.
// REAL < COLS: the tensor's rows hold only REAL features; the tile's remaining columns are
// filled with zeros (a row index of kBlock marks such a slot: it is never below `valid`).
template <int COLS, int REAL = COLS>
struct TileDma {
    static_assert(Swz<COLS>::NI % 4 == 0, "every state wave issues the same number of loads");
    static_assert(REAL % 8 == 0 && REAL <= COLS, "whole 16-byte chunks");
    static constexpr int PER_WAVE = Swz<COLS>::NI / 4;
    long long src[PER_WAVE];
    int row[PER_WAVE];
    __device__ __forceinline__ void init(int u, int lane, long long row_stride) {
        using S = Swz<COLS>;
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const int slot = 64 * (u + 4 * i) + lane;
            const int r = slot / S::CPR;
            const int c = (slot % S::CPR) ^ S::key(r);
            row[i] = (REAL < COLS && c * 8 >= REAL) ? kBlock : r;
            src[i] = (long long)r * row_stride + c * 16;
        }
    }
    // base: global address of the block's row 0 (plus the slice's column offset);
    // lds: LDS byte address of the tile; rows >= valid come from the zero buffer
    __device__ __forceinline__ void issue(const char* base, unsigned lds, int u, int valid) const {
#pragma unroll
        for (int i = 0; i < PER_WAVE; ++i) {
            const char* g = (row[i] < valid) ? base + src[i] : (const char*)kZeros;
            dma16(lds + 1024u * (unsigned)(u + 4 * i), g);
        }
    }
};

// The same fetch in scalar-base form for any subset of waves.  The per-lane part of a load's
// address repeats every 16 rows (the swizzle key does), so a tile needs only NV = CPR / 4
// per-lane offsets; the 16-row group and the block sit in the wave-uniform base address.  Load
// j = m NV + v (m: 16-row group, v < NV) fills LDS slots 64j .. 64j+63 as above; of NW issuing
// waves, wave W_ takes the loads with j % NW == W_ (NI / NW loads per tile and wave).
// REAL < COLS: the tensor's rows hold only REAL features.  The lanes of the tile's remaining
// chunks take no part in a load, so those chunks keep what they hold: zeros written once by
// the workgroup before its first load.
template <int COLS, int REAL = COLS>
struct TileDmaU {
    using S = Swz<COLS>;
    static constexpr int NV = S::CPR / 4;
    static constexpr int NI = S::NI;
    static_assert(NV >= 1 && NI == 4 * NV, "four 16-row groups per tile");
    static_assert(REAL % 8 == 0 && REAL <= COLS, "whole 16-byte chunks");
    // lanes of load v (of any 16-row group) whose chunk holds real features
    __host__ __device__ static constexpr unsigned long long real_lanes(int v) {
        unsigned long long m = 0;
        for (int lane = 0; lane < 64; ++lane) {
            const int slot = 64 * v + lane;
            const int c = (slot % S::CPR) ^ S::key(slot / S::CPR);
            if (c * 8 < REAL) m |= 1ull << lane;
        }
        return m;
    }
    template <int V>
    __device__ __forceinline__ void load(unsigned lds, const char* grp) const {
        if constexpr (REAL == COLS) {
            dma16s(lds, grp, off[V]);
        } else {
            constexpr unsigned long long m = real_lanes(V);
            dma16s_masked(lds, grp, off[V], m);
        }
    }
    unsigned off[NV];     // (row within its 16-row group, from the group's lowest-address row) * pitch + chunk * 16
    __device__ __forceinline__ void init(int lane, long long pitch, int rev) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int slot = 64 * v + lane;
            const int rr = slot / S::CPR;                       // 0..15
            const int c = (slot % S::CPR) ^ S::key(rr);
            off[v] = (unsigned)((rev ? 15 - rr : rr) * pitch + c * 16);
        }
    }
    // row0: wave-uniform global address of the block's row 0 (plus the slice's column offset);
    // rows follow at +pitch, or at -pitch on a reversed token axis.  All kBlock rows are read.
    template <int NW, int W_>
    __device__ __forceinline__ void issue_full(const char* row0, long long pitch, int rev, unsigned lds) const {
        static_assert(NI % NW == 0, "every issuing wave takes the same number of loads");
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const char* grp = row0 + (rev ? -(long long)(16 * m + 15) * pitch : (long long)(16 * m) * pitch);
            static_for<NV>([&](auto vc) {
                constexpr int v = decltype(vc)::value;
                if ((m * NV + v) % NW == W_) load<v>(lds + 1024u * (unsigned)(m * NV + v), grp);
            });
        }
    }
    // The same loads for a short last block: rows >= valid come from the zero buffer.
    template <int NW, int W_>
    __device__ __forceinline__ void issue_partial(const char* row0, long long pitch, int rev, unsigned lds, int valid,
                                                  int lane) const {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const char* grp = row0 + (rev ? -(long long)(16 * m + 15) * pitch : (long long)(16 * m) * pitch);
            static_for<NV>([&](auto vc) {
                constexpr int v = decltype(vc)::value;
                if ((m * NV + v) % NW == W_) {
                    constexpr unsigned long long rl = real_lanes(v);
                    const int r = 16 * m + (64 * v + lane) / S::CPR;
                    const bool real = REAL == COLS || ((rl >> lane) & 1);
                    dma16(lds + 1024u * (unsigned)(m * NV + v), (r < valid && real) ? grp + off[v] : (const char*)kZeros);
                }
            });
        }
    }
};

// The output strip of a wave is produced transposed: the lane holds, for its token (lane
// % 16), features 16nt + 4g .. +3 of every 16-feature tile nt (g = lane / 16).  Two lane-row
// swaps per tile pair (rows of 16 lanes: first between the wave's halves, then between
// neighbouring rows) regroup them so that the lane holds the eight consecutive features
// 32p + 8g .. +7 of its token: one 16-byte store per tile pair, and the four lanes of a
// token write 64 contiguous bytes.  `out`: the lane's token row, column 8g.
template <int NT>
__device__ __forceinline__ void store_strip(const f32x4 (&r)[NT], char* out, bool store) {
    unsigned w[NT][2];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        union { bf16x4 h; unsigned u[2]; } cv;
        cv.h = to_bf16(r[nt]);
        w[nt][0] = cv.u[0];
        w[nt][1] = cv.u[1];
    }
#pragma unroll
    for (int p = 0; p < NT / 2; ++p) {
        u32x4 q;
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            auto s = __builtin_amdgcn_permlane32_swap(w[2 * p][d], w[2 * p + 1][d], false, false);
            auto t = __builtin_amdgcn_permlane16_swap(s[0], s[1], false, false);
            q[d] = t[0];
            q[2 + d] = t[1];
        }
        if (store) *(u32x4*)(out + 64 * p) = q;
    }
}

__device__ __forceinline__ unsigned lds_address(const char* p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) char*)p;
}

}  // namespace
}  // namespace ltn
