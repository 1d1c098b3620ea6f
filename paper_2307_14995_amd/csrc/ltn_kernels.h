// Internal launcher interface between the C-ABI layer and the gfx950 kernels.
// Not installed; the public boundary is include/ltn_attn.h.
#pragma once
#include <hip/hip_runtime.h>

namespace ltn {

// One "decayed linear-attention pass":
//   out[t,:] = sum_{s<=t} lambda^(t-s) (a_t . b_s) c_s  (+ lambda^(t+1) a_t state_in)
// evaluated blockwise with a running state  S <- lambda^len S + (decayed b)^T c.
// With rev = 1 the token axis is traversed from the last token to the first, which
// turns the sum into  sum_{s>=t} lambda^(s-t) (a_t . b_s) c_s  (the anti-causal pass
// the gradients dK and dV need).  The forward pass and the three gradients of
// Lightning Attention (arXiv 2307.14995, Sec. 3.2.1 / App. B) are four such passes:
//   O  = pass(Q,  K,  V)        dQ = pass(dO, V,  K)
//   dV = pass(K,  Q,  dO, rev)  dK = pass(V,  dO, Q, rev)
struct PassArgs {
    const void* a;        // [chains, N, D]  "query-like" operand
    const void* b;        // [chains, N, D]  "key-like" operand
    const void* c;        // [chains, N, D]  "value-like" operand
    void* out;            // [chains, N, D]
    const float* state_in;  // [chains, D, D] fp32 or nullptr (zero)
    float* state_out;       // [chains, D, D] fp32 or nullptr
    int rev;              // 0: first token -> last; 1: last -> first
    // Gated, normalised epilogue (arXiv 2307.14995 Eq. 3 with the SimpleRMSNorm of
    // Sec. 3.1.3 per head): when gate != nullptr the pass also writes
    //   gated_out[t,:] = out[t,:] / sqrt(mean(out[t,:]^2) + eps) (.) gate[t,:]
    // and `out` itself may be nullptr.  Needs full-width slices (dv = D), one pass.
    const void* gate;     // [chains, N, D] or nullptr
    void* gated_out;      // [chains, N, D]
    float eps;
};

struct PassBatch {
    PassArgs p[3];
    int count;            // 1..3 passes run concurrently in one launch
    const float* decay;   // [H]
    int chains;           // Bt * H
    int H;
    long long N;
    // Sequence-parallel form: every chain is cut into `segs` segments of seg_len tokens
    // (a multiple of 64; the last may be shorter) along the pass's own token order, each
    // handled by its own workgroups.  state_in / state_out then hold one state per
    // (chain, segment): [chains * segs, D, D].  segs = 1: the whole chain, seg_len unused.
    int segs;
    long long seg_len;
    int state_only;       // 1: compute only each segment's end state from a zero state
    int need_last;        // state_only: also for the last segment of a chain
    // count == 3 only: passes 0 and 1 read the same token rows at the same time (same direction,
    // two shared operands) and pass 2 does not; lets the bf16 kernel order workgroup ids for that
    int pairs_first;
};

// bf16 MFMA kernel, block length 64.  D in {64,96,128,256}; dv = value columns per workgroup
// (D, D/2 or, for D = 128, D/4; 64 or 32 for D = 256 and 32 for D = 96, plain pass only).
// DC (0: = D): features per token of c and out when they differ from those of a and b
// (the LRPE-d expansion of Eq. 1 doubles the query/key width): a, b [chains, N, D];
// c, out [chains, N, DC]; states [chains, D, DC]; dv slices DC.  Plain pass, or the state-only
// sweep with dv = 64 (128 for (128,256)).  (D, DC) in {(256,128), (128,256), (128,64), (64,128)}.
hipError_t launch_pass_bf16(const PassBatch& pb, int D, int dv, hipStream_t stream, int DC = 0);
// Forward by the quadratic tiling of App. B Algorithm 3 (comparison kernel), bf16, zero
// initial state, D in {64,128}.
hipError_t launch_tiled_fwd_bf16(const void* q, const void* k, const void* v, void* o, const float* decay,
                                 int chains, int H, long long N, int D, hipStream_t stream);
// Gradients by the tiling of App. B Algorithm 4 (comparison kernel), bf16, D in {64,128}: one
// workgroup per key/value block (dK, dV) and one per query block (dQ), in one launch.
hipError_t launch_tiled_bwd_bf16(const void* q, const void* k, const void* v, const void* d_o, void* dq, void* dk,
                                 void* dv, const float* decay, int chains, int H, long long N, int D,
                                 hipStream_t stream);
// fp32 kernel.  D in {64,96,128,256}, block in {16,32,64}, D*block <= 4096 (D = 256: dv = 64;
// D = 96: dv = 32, block 16 or 32).
hipError_t launch_pass_f32(const PassBatch& pb, int D, int dv, int block, hipStream_t stream, int DC = 0);
// fp32 MFMA kernel (v_mfma_f32_16x16x4_f32) for plain passes with D in {64,128}: the
// (D, dv, block) combinations pass_f32_mfma_supports() accepts; launch_pass_f32 routes those
// here and keeps its plain-FMA kernel for the rest (gated epilogue, unequal widths, 96, 256).
bool pass_f32_mfma_supports(int D, int dv, int block);
hipError_t launch_pass_f32_mfma(const PassBatch& pb, int D, int dv, int block, hipStream_t stream);
// Turns the segment-local end states L[pass][chain][g] in `states` (as written by a
// state_only launch) into the states at each segment's start, in place:
//   S[0] = kv_in (pass 0 only) or 0,   S[g+1] = lambda^len(g) S[g] + L[g],
// and writes the state after the last segment to kv_out (pass 0) when given.
hipError_t launch_segment_scan(float* states, const float* kv_in, float* kv_out, const float* decay,
                               int count, int chains, int H, int segs, long long seg_len, long long N,
                               int D, hipStream_t stream, int DC = 0 /* 0: = D; states are [D x DC] */);
// kv[c] (or zeros if null) -> kv_out[c], n floats.
hipError_t launch_state_copy(const float* kv_in, float* kv_out, size_t n, hipStream_t stream);
// `steps` consecutive decode steps per chain (q, k: [chains, steps, DK]; v, o: [chains,
// steps, DV]; kv: [chains, DK, DV]), see ltn_attn_decode_steps.  (DK, DV) in {(128,128),
// (64,64), (256,128), (128,64)}.
hipError_t launch_decode(const void* q, const void* k, const void* v, void* o, float* kv,
                         const float* decay, int chains, int H, int steps, int DK, int DV, int is_bf16,
                         hipStream_t stream);

// Input side of the token mixer for queries and keys (see ltn_prologue.hip): swish (Eq. 2)
// and the LRPE-d expansion of Eq. 1.  is_bwd = 0: y from x.  is_bwd = 1: dx from (x, dy)
// and, with theta and dtheta given, dtheta[H, D] through `partials` (device scratch of
// prologue_partial_count(N) * H * D doubles).
long long prologue_partial_count(long long N);
hipError_t launch_prologue(const void* x, const float* theta, const void* dy, void* out, float* dtheta,
                           double* partials, int act, int Bt, int H, long long N, int D, long long pos0,
                           int is_bf16, int is_bwd, hipStream_t stream);

// Gated SimpleRMSNorm on `rows` rows of D features (see ltn_gate.hip).  is_bwd = 0:
// o0 = y (dy, o1 unused); is_bwd = 1: o0 = dx, o1 = du.
hipError_t launch_gate(const void* x, const void* u, const void* dy, void* o0, void* o1, float eps,
                       long long rows, int D, int is_bf16, int is_bwd, hipStream_t stream);

// Streaming-read probe (see ltn_probe.hip): wgs workgroups each read their own per_wg bytes
// (a multiple of 64 KB) of `buf` `iters` times, to LDS directly or to registers.
hipError_t launch_probe_stream(const void* buf, size_t per_wg, int wgs, int iters, int to_registers, unsigned* sink,
                               hipStream_t stream);

// lambda^n, n >= 0, by binary powering in fp64 (only multiplications: exact up to
// rounding, lambda = 0 gives 0^0 = 1, no transcendental).  Never called with n < 0.
__device__ __forceinline__ float decay_pow(float lam, int n) {
    double base = (double)lam, r = 1.0;
    while (n > 0) {
        if (n & 1) r *= base;
        base *= base;
        n >>= 1;
    }
    return (float)r;
}

// Workgroup index -> (pass, chain, split).  Consecutive workgroup ids are dealt
// round-robin to the 8 XCDs, each with a private L2; all workgroups that read the
// same chain's tokens (its passes and value-column splits) are therefore given
// ids that are congruent mod 8, so re-reads of a chain's tiles hit one L2.
__device__ __forceinline__ void map_workgroup(int wg, int per_chain, int chains,
                                              int& chain, int& within) {
    if ((chains & 7) == 0) {
        const int xcd = wg & 7, slot = wg >> 3;
        chain = (slot / per_chain) * 8 + xcd;
        within = slot % per_chain;
    } else {
        chain = wg / per_chain;
        within = wg % per_chain;
    }
}

// The same dealing for a number of chains that is no multiple of 8: the launch is padded to
// 8 * ceil(chains / 8) chain slots and the workgroups of the empty ones leave at once.  That
// puts ceil(chains / 8) * per_chain workgroups on the first XCDs, so it is used only while
// those fit an XCD's 32 compute units (xcd_ids_fit); otherwise ids stay chain-major.
inline bool xcd_ids_fit(long long chains, int per_chain) {
    return per_chain > 1 && ((chains & 7) == 0 || (chains + 7) / 8 * per_chain <= 32);
}
inline long long launch_chain_slots(long long chains, int per_chain) {
    return xcd_ids_fit(chains, per_chain) ? (chains + 7) / 8 * 8 : chains;
}
// xcd_ids: xcd_ids_fit(chains, per_chain), computed by the host.  False: the workgroup is a
// padding one and has nothing to do.
__device__ __forceinline__ bool map_workgroup_padded(int wg, int per_chain, int chains, int xcd_ids,
                                                     int& chain, int& within) {
    if (xcd_ids) {
        const int xcd = wg & 7, slot = wg >> 3;
        chain = (slot / per_chain) * 8 + xcd;
        within = slot % per_chain;
    } else {
        chain = wg / per_chain;
        within = wg % per_chain;
    }
    return chain < chains;
}

}  // namespace ltn
