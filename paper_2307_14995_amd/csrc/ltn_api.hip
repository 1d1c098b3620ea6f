// C-ABI layer of the Lightning Attention library: argument validation (host only,
// before any launch), choice of block length and value-column split, and dispatch
// to the gfx950 kernels.  See include/ltn_attn.h for the contract.
#include "../../include/ltn_attn.h"
#include "ltn_kernels.h"

#include <atomic>
#include <cstdint>
#include <mutex>

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Test-only overrides of the launch plan (ltn_attn_set_debug_plan); 0 = the library's choice.
std::atomic<int> g_debug_dv{0};
std::atomic<int> g_debug_segs{0};

// A tensor argument as a byte range.  Outputs are written while inputs are still being
// read (tile loads run up to three blocks ahead of the stores), so any overlap between an
// output and an input, or between two outputs, is rejected, not only equal base pointers.
struct Span { const void* p; size_t bytes; };

bool spans_overlap(const Span& a, const Span& b) {
    if (!a.p || !b.p || a.bytes == 0 || b.bytes == 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a.p), b0 = reinterpret_cast<uintptr_t>(b.p);
    return a0 < b0 + b.bytes && b0 < a0 + a.bytes;
}

// true when some output overlaps an input or another output
bool outputs_alias(const Span* outs, int n_out, const Span* ins, int n_in) {
    for (int a = 0; a < n_out; ++a) {
        for (int b = 0; b < n_in; ++b)
            if (spans_overlap(outs[a], ins[b])) return true;
        for (int b = a + 1; b < n_out; ++b)
            if (spans_overlap(outs[a], outs[b])) return true;
    }
    return false;
}

size_t esize_of(ltn_dtype dtype) { return dtype == LTN_BF16 ? 2 : 4; }

// Value columns handled per workgroup.  Every value-column slice of a chain recomputes
// that chain's score tiles and re-reads its first two operands through L2, and a compute
// unit holds one workgroup: the split is the deepest one whose workgroups still fit one
// round of the 256 compute units; when even full-width slices need more than one round,
// full width (fewest re-reads).  Among the splits that fit one round, bf16 takes the deepest
// whose workgroups of one chain can be given ids on one XCD (count passes x slices per chain,
// ltn::xcd_ids_fit): slices that meet in one L2 beat a deeper split that does not (20 chains,
// backward: 32-column slices 0.101 ms, 64-column 0.066 ms; 42 chains: 64-column 0.120 ms,
// full width 0.110 ms).  Measured on MI355X for 8..256 chains, forward and backward.
// ltn_attn_set_debug_plan (test only) overrides the choice.
// chain_passes = chains (x segments) x count; count = passes per chain in the launch.
int pick_dv(long long chain_passes, int D, ltn_dtype dtype, int blk, int count = 1) {
    if (D == 96) {                         // three 32-column slices, or all 96 columns in one workgroup
        if (dtype != LTN_BF16) return 32;
        if (const int v = g_debug_dv.load(std::memory_order_relaxed)) {
            if (v == 32 || v == 96) return v;
        }
        // three slices per pass while a chain's workgroups can share an XCD within one round
        return (chain_passes * 3 <= 256 && ltn::xcd_ids_fit(chain_passes / count, count * 3)) ? 32 : 96;
    }
    // D = 256: the state copies of more than 64 columns do not fit the LDS
    const int hi = (D == 256) ? 64 : D;
    int lo = (dtype == LTN_BF16) ? 32 : (D == 256 ? 64 : D / 2);
    // fp32 on the matrix cores: a quarter of the columns too where its kernel has them
    if (dtype == LTN_F32 && ((D == 128 && blk == 32) || (D == 64 && blk == 64))) lo = D / 4;
    if (const int v = g_debug_dv.load(std::memory_order_relaxed)) {
        if ((v == D || v == D / 2 || v == D / 4 || v == D / 8) && v >= lo && v <= hi) return v;
    }
    int fits = 0;
    for (int dv = lo; dv <= hi; dv *= 2) {
        if (chain_passes * (D / dv) > 256) continue;
        if (dtype != LTN_BF16 || count * (D / dv) == 1 || ltn::xcd_ids_fit(chain_passes / count, count * (D / dv))) return dv;
        if (!fits) fits = dv;
    }
    if (fits) return fits;
    // More than one round even at full width.  The fp32 matrix-core kernel is bound by its MFMA
    // and LDS latencies, and two of its half-width workgroups fit one compute unit (76 KB of LDS
    // each), so half width runs 5-7 % faster there (measured: 1B and 7B shapes, backward); the
    // memory-bound bf16 kernel keeps full width (fewest re-reads).
    if (dtype == LTN_F32 && D == 128 && blk == 32) return D / 2;
    return hi;
}

// The same rule for a pass whose value side has DC columns and whose kernels exist for
// slices of lo .. hi columns (powers of two).
int pick_dv_range(long long chain_passes, int DC, int lo, int hi) {
    for (int dv = lo; dv <= hi; dv *= 2)
        if (chain_passes * (DC / dv) <= 256) return dv;
    return hi;
}

ltn_status check_common(int Bt, int H, long long N, int D, int block, ltn_dtype dtype, int* blk_out) {
    if (Bt < 0 || H < 0 || N < 0 || D <= 0 || block < 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (D != 64 && D != 96 && D != 128 && D != 256) return LTN_ERR_UNSUPPORTED;
    const int blk = block ? block : ltn_attn_pick_block(D, dtype);
    if (dtype == LTN_BF16) {
        if (blk != 64) return LTN_ERR_UNSUPPORTED;
    } else {
        if (blk != 16 && blk != 32 && blk != 64) return LTN_ERR_UNSUPPORTED;
        if ((long long)(D == 96 ? 128 : D) * blk > 4096) return LTN_ERR_UNSUPPORTED;   // 96 is computed as 128
    }
    if ((long long)Bt * H > 0x3fffffffLL) return LTN_ERR_SHAPE;
    *blk_out = blk;
    return LTN_OK;
}

// Sequence-parallel plan.  With few chains even the deepest value-column split leaves
// compute units idle and makes every workgroup re-read A and B; cutting each chain into
// segments instead gives full-width workgroups to all compute units at the price of one
// extra read of B and C (the state-only sweep) and two more launches.  Measured on MI355X
// (2 .. 64 chains, N = 2048 .. 65536, forward and backward, every segment count): pays when a
// chain can be cut at least 8 ways into segments of at least 512 tokens without exceeding one
// round of compute units, from 5 ways on when the segments are at least 1024 tokens long
// (33 .. 51 passes of long chains: the forward of 36 .. 48 chains at N = 8192 runs 17-29 % faster
// cut 5 .. 7 ways, the backward of 12 .. 16 chains 11-16 %), and 4 ways in the backward of about
// 20 chains with segments of at least 2048 tokens (13-19 %); never otherwise.
// bf16 kernels only.  Heads of 256 features always need four 64-column workgroups per chain
// and segment, heads of 96 three of 32; there the form pays from 3 segments of at least 512
// tokens on (measured: 2 .. 32 chains, N = 2048 .. 32768, forward and backward; heads of 96
// features have a second cut for their 96-column workgroups, in place), for the gated
// pass from 4 segments of at least 512 tokens on, and from 2 when they are at least 2048 tokens
// long (measured: 4 .. 100 chains, N = 2048 .. 16384, 64 / 96 / 128 features).
// ltn_attn_set_debug_plan (test only) forces a segment count.
struct SegPlan { int segs; long long seg_len; };
constexpr long long kMinSegsFullWidth = 4;   // measured: 2 segments lose to one workgroup per chain

SegPlan cut_chain(long long N, long long want) {
    SegPlan plan = {1, 0};
    if (want <= 1) return plan;
    long long len = (N + want - 1) / want;
    len = (len + 63) / 64 * 64;
    const long long segs = (N + len - 1) / len;
    if (segs <= 1 || segs > 0x7fff) return plan;
    plan.segs = (int)segs;
    plan.seg_len = len;
    return plan;
}

// paired_chains: the number of chains when the passes are the three of a backward (whose
// (dV, dK) workgroups sit side by side on one XCD at full width), else 0.
SegPlan pick_segments(long long chain_passes, long long N, int D, ltn_dtype dtype, bool full_width = false,
                      long long paired_chains = 0) {
    SegPlan plan = {1, 0};
    if (dtype != LTN_BF16 || chain_passes <= 0 || N <= 64) return plan;
    // D = 256: every (chain, segment) still needs four 64-column workgroups; D = 96: three of 32
    const long long per_seg = (D == 256) ? 4 : ((D == 96 && !full_width) ? 3 : 1);
    long long want = 256 / (per_seg * chain_passes);
    bool whole_rows = per_seg == 1;        // one workgroup per chain, pass and segment
    // a pass that must keep full-width slices has no column split to fall back on
    if (want > N / 512) want = N / 512;       // segments of at least 512 tokens
    if (full_width) {
        // from 4 ways on; 2 or 3 ways when the segments stay at least 2048 tokens long (not for 96
        // features, whose state-only sweep runs three workgroups per segment; for 128 features
        // only when that leaves an eighth of the compute units free: at 128 chains the second
        // read of K and V costs more than the idle half of the chip)
        const bool few_ok = D != 96 && want >= 2 && N / want >= 2048 && (D == 64 || chain_passes * want <= 224);
        if (want < kMinSegsFullWidth && !few_ok) want = 1;
    } else if (per_seg > 1) {
        if (want < 3) want = 1;
        if (D == 96) {
            // Workgroup ids deal (chain, segment) pairs to the 8 XCDs of 32 compute units and keep
            // a pair's three slices on one XCD: an XCD's share must not exceed its units (11
            // pairs per XCD -- 252 workgroups -- ran 30 % slower than 10).
            while (want > 1 && (chain_passes * want + 7) / 8 * 3 > 32) --want;
            if (want < 3) want = 1;
            // Heads of 96 features also have one 96-column workgroup per chain and segment
            // (pick_dv takes it when three 32-column slices each would need more than one round).
            // From 12 chain passes on, cutting for that width pays from 8 segments on -- of at
            // least 768 tokens, or 512 where the rule above finds nothing to cut -- and from 5
            // segments of at least 1024 tokens (measured: 4 .. 32 chains, N = 4096 .. 32768,
            // forward and backward, every segment count).
            if (chain_passes >= 12) {
                long long all = 256 / chain_passes;
                if (all > N / 512) all = N / 512;
                if (all >= 5) {
                    const long long len = N / all;
                    if ((all >= 8 && (len >= 768 || want == 1)) || len >= 1024) {
                        want = all;
                        whole_rows = true;
                    }
                }
            }
        }
    } else if (want < 8) {
        // 5 .. 7 ways: segments of at least 1024 tokens; 4 ways: the backward alone, segments of at
        // least 2048 tokens, when its (dV, dK) pairs can sit side by side (chains x 4 a multiple of 8)
        // (heads of 64 features, whose blocks cost half as much: 512 and 1024 tokens)
        const long long few_len = D == 64 ? 512 : 1024;
        const bool few = want >= 5 && N / want >= few_len;
        const bool four = want == 4 && paired_chains > 0 && (paired_chains * 4) % 8 == 0 && N / want >= 2 * few_len;
        if (!few && !four) want = 1;
    }
    if (paired_chains > 0 && want >= 6 && whole_rows) {
        // The backward's workgroup ids pair a chain's (dV, dK) passes on one XCD only when
        // chains x segments is a multiple of 8: up to a quarter fewer segments for that
        // (measured, 4 / 5 / 6 / 12 chains: 21 -> 20, 17 -> 16, 14 -> 12, 7 -> 6 segments run
        // 9-15 % faster).
        for (long long w = want; w >= 2 && 4 * w >= 3 * want; --w) {
            const SegPlan p = cut_chain(N, w);
            if (p.segs > 1 && (paired_chains * p.segs) % 8 == 0) {
                want = w;
                break;
            }
        }
    }
    if (const int v = g_debug_segs.load(std::memory_order_relaxed)) want = v;
    return cut_chain(N, want);
}

// full_width: the pass carries the gated epilogue, which needs complete output rows in one
// workgroup (slices of all D value columns).
ltn_status run_passes(ltn::PassBatch& pb, int D, int blk, ltn_dtype dtype, void* workspace, hipStream_t stream,
                      bool full_width = false) {
    const long long chain_passes = (long long)pb.chains * pb.count;
    const SegPlan plan = pick_segments(chain_passes, pb.N, D, dtype, full_width,
                                       (pb.pairs_first && pb.count == 3) ? pb.chains : 0);
    pb.segs = 1;
    if (plan.segs == 1) {
        const int dv = full_width ? D : pick_dv(chain_passes, D, dtype, blk, pb.count);
        const hipError_t e = (dtype == LTN_BF16) ? ltn::launch_pass_bf16(pb, D, dv, stream)
                                                 : ltn::launch_pass_f32(pb, D, dv, blk, stream);
        return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
    }
    // three launches: segment end states from zero, scan, then the pass proper per segment
    if (!workspace) return LTN_ERR_NULL;
    float* states = static_cast<float*>(workspace);
    const size_t per_pass = (size_t)pb.chains * plan.segs * D * D;
    const float* kv_in = pb.p[0].state_in;
    float* kv_out = pb.p[0].state_out;
    ltn::PassBatch sweep = pb;
    sweep.segs = plan.segs;
    sweep.seg_len = plan.seg_len;
    sweep.state_only = 1;
    sweep.need_last = kv_out != nullptr;
    for (int i = 0; i < pb.count; ++i) {
        sweep.p[i].out = nullptr;
        sweep.p[i].gate = nullptr;
        sweep.p[i].gated_out = nullptr;
        sweep.p[i].state_in = nullptr;
        sweep.p[i].state_out = states + i * per_pass;
    }
    if (ltn::launch_pass_bf16(sweep, D, D == 256 ? 64 : (D == 96 ? 32 : D), stream) != hipSuccess) return LTN_ERR_LAUNCH;
    if (ltn::launch_segment_scan(states, kv_in, kv_out, pb.decay, pb.count, pb.chains, pb.H, plan.segs,
                                 plan.seg_len, pb.N, D, stream) != hipSuccess)
        return LTN_ERR_LAUNCH;
    ltn::PassBatch main = pb;
    main.segs = plan.segs;
    main.seg_len = plan.seg_len;
    for (int i = 0; i < pb.count; ++i) {
        main.p[i].state_in = states + i * per_pass;
        main.p[i].state_out = nullptr;
    }
    const int dv = full_width ? D : pick_dv(chain_passes * plan.segs, D, dtype, blk, pb.count);
    return ltn::launch_pass_bf16(main, D, dv, stream) == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

// Scratch of ltn_attn_fwd_static: device memory that belongs to the library's code object,
// so that entry point needs no allocation and no caller workspace.  Every GPU the library
// runs on holds its own copy at its own address until the process ends; in host code the
// array's name is only a handle for hipGetSymbolAddress, never an address to pass on.
constexpr size_t kScratchBytes = (size_t)LTN_ATTN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up once per device).
ltn_status scratch_on_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LTN_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LTN_ERR_LAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LTN_OK;
}

}  // namespace

extern "C" {

ltn_status ltn_attn_set_debug_plan(int dv, int segs) {
    if (dv != 0 && dv != 16 && dv != 32 && dv != 64 && dv != 96 && dv != 128 && dv != 256) return LTN_ERR_SHAPE;
    if (segs < 0 || segs > 4096) return LTN_ERR_SHAPE;
    g_debug_dv.store(dv, std::memory_order_relaxed);
    g_debug_segs.store(segs, std::memory_order_relaxed);
    return LTN_OK;
}

ltn_status ltn_attn_query_plan(int Bt, int H, long long N, int D, ltn_dtype dtype, int call,
                               int* dv_out, int* segs_out) {
    if (!dv_out || !segs_out) return LTN_ERR_NULL;
    if (Bt <= 0 || H <= 0 || N <= 0 || call < 0 || call > 2) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (D != 64 && D != 96 && D != 128 && D != 256) return LTN_ERR_UNSUPPORTED;
    const long long chain_passes = (long long)Bt * H * (call == 1 ? 3 : 1);
    const SegPlan plan = pick_segments(chain_passes, N, D, dtype, call == 2, call == 1 ? (long long)Bt * H : 0);
    *segs_out = plan.segs;
    *dv_out = (call == 2) ? D : pick_dv(chain_passes * plan.segs, D, dtype, ltn_attn_pick_block(D, dtype), call == 1 ? 3 : 1);
    return LTN_OK;
}

int ltn_attn_pick_block(int D, ltn_dtype dtype) {
    if (D != 64 && D != 96 && D != 128 && D != 256) return 0;
    if (dtype == LTN_BF16) return 64;
    if (dtype == LTN_F32) return D == 64 ? 64 : (D == 256 ? 16 : 32);
    return 0;
}

size_t ltn_attn_workspace_bytes(int Bt, int H, long long N, int D, int block, ltn_dtype dtype, int call) {
    (void)block;
    if (Bt <= 0 || H <= 0 || N <= 0 || (D != 64 && D != 96 && D != 128 && D != 256) || call < 0 || call > 2) return 0;
    const long long chains = (long long)Bt * H;
    const int count = (call == 1) ? 3 : 1;
    const size_t state = (size_t)D * D * sizeof(float);                                   // one fp32 state per segment
    const SegPlan plan = pick_segments(chains * count, N, D, dtype, call == 2, call == 1 ? chains : 0);
    size_t need = plan.segs == 1 ? 0 : (size_t)count * (size_t)chains * (size_t)plan.segs * state;
    if (call == 2) {
        // the gated forward may run as the plain forward followed by the gate kernel (when the
        // attention output is stored anyway): room for whichever plan needs more
        const SegPlan plain = pick_segments(chains, N, D, dtype, false);
        const size_t alt = plain.segs == 1 ? 0 : (size_t)chains * (size_t)plain.segs * state;
        if (alt > need) need = alt;
    }
    return need;
}

ltn_status ltn_attn_check_decay(const float* decay_host, int H) {
    if (!decay_host) return LTN_ERR_NULL;
    if (H < 0) return LTN_ERR_SHAPE;
    for (int h = 0; h < H; ++h)
        if (!(decay_host[h] >= 0.0f && decay_host[h] <= 1.0f)) return LTN_ERR_DECAY;
    return LTN_OK;
}

const char* ltn_status_str(ltn_status s) {
    switch (s) {
        case LTN_OK: return "LTN_OK";
        case LTN_ERR_NULL: return "LTN_ERR_NULL: a required pointer is NULL";
        case LTN_ERR_SHAPE: return "LTN_ERR_SHAPE: bad size or workspace too small";
        case LTN_ERR_UNSUPPORTED: return "LTN_ERR_UNSUPPORTED: shape/dtype/block not supported, or an output overlaps an input or another output";
        case LTN_ERR_ALIGN: return "LTN_ERR_ALIGN: tensor pointer not 16-byte aligned";
        case LTN_ERR_DECAY: return "LTN_ERR_DECAY: decay value outside [0, 1]";
        case LTN_ERR_LAUNCH: return "LTN_ERR_LAUNCH: HIP launch failed";
        case LTN_ERR_SCRATCH: return "LTN_ERR_SCRATCH: the call needs more scratch than the library's static buffer holds";
        default: break;
    }
    return "LTN_ERR_?: unknown status";
}

// Shared body of ltn_attn_fwd and ltn_attn_fwd_gated (u == nullptr: plain forward).
static ltn_status fwd_common(const void* q, const void* k, const void* v, const void* u, void* o, void* y,
                             const float* decay, const float* kv_in, float* kv_out, float eps,
                             int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                             void* workspace, size_t workspace_bytes, void* stream, bool gated) {
    const bool empty = (Bt == 0 || H == 0 || N == 0);   // no token is read or written
    if (!decay || (!empty && (!q || !k || !v || (gated ? (!u || !y) : !o)))) return LTN_ERR_NULL;
    int blk = 0;
    const ltn_status cs = check_common(Bt, H, N, D, block, dtype, &blk);
    if (cs != LTN_OK) return cs;
    if (gated && !(eps >= 0.0f)) return LTN_ERR_SHAPE;
    // 256 features (and 96 in fp32): no kernel holds a complete output row of these widths in one
    // workgroup, so the epilogue is applied to the stored attention output by the gate kernel; a
    // caller that does not want o stored has no fused form to fall back on
    const bool unfused_only = gated && (D == 256 || (D == 96 && dtype != LTN_BF16));
    if (unfused_only && !o && !empty) return LTN_ERR_UNSUPPORTED;
    const size_t need_ws = ltn_attn_workspace_bytes(Bt, H, N, D, block, dtype, gated ? 2 : 0);
    if (workspace_bytes < need_ws) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(u) || !aligned16(y) ||
        !aligned16(kv_in) || !aligned16(kv_out) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    const long long chains = (long long)Bt * H;
    if (!empty) {
        const size_t tb = (size_t)chains * (size_t)N * D * esize_of(dtype), sb = (size_t)chains * D * D * sizeof(float);
        // kv_out may be kv_in itself (a state updated in place); any other overlap is refused
        const Span ins[5] = {{q, tb}, {k, tb}, {v, tb}, {u, tb}, {kv_in == kv_out ? nullptr : kv_in, sb}};
        const Span outs[4] = {{o, tb}, {y, tb}, {kv_out, sb}, {workspace, need_ws}};
        if (outputs_alias(outs, 4, ins, 5)) return LTN_ERR_UNSUPPORTED;
    }
    if (chains == 0) return LTN_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (N == 0) {
        if (!kv_out) return LTN_OK;
        if (kv_in && kv_in != kv_out && spans_overlap({kv_in, (size_t)chains * D * D * sizeof(float)},
                                                      {kv_out, (size_t)chains * D * D * sizeof(float)}))
            return LTN_ERR_UNSUPPORTED;
        return ltn::launch_state_copy(kv_in, kv_out, (size_t)chains * D * D, st) == hipSuccess
                   ? LTN_OK : LTN_ERR_LAUNCH;
    }
    ltn::PassBatch pb = {};
    pb.segs = 1;
    pb.count = 1;
    pb.decay = decay;
    pb.chains = (int)chains;
    pb.H = H;
    pb.N = N;
    pb.p[0] = ltn::PassArgs{q, k, v, o, kv_in, kv_out, 0, gated ? u : nullptr, gated ? y : nullptr, eps};
    if (!gated) return run_passes(pb, D, blk, dtype, workspace, st);
    if (unfused_only) {
        pb.p[0].gate = nullptr;
        pb.p[0].gated_out = nullptr;
        const ltn_status s1 = run_passes(pb, D, blk, dtype, workspace, st);
        if (s1 != LTN_OK) return s1;
        return ltn::launch_gate(o, u, nullptr, y, nullptr, eps, chains * N, D, dtype == LTN_BF16, 0, st) == hipSuccess
                   ? LTN_OK : LTN_ERR_LAUNCH;
    }
    // The fused epilogue needs complete output rows in one workgroup, i.e. full-width slices
    // (one workgroup per chain, or per chain segment).  With few chains that can leave
    // compute units idle; when the caller wants the attention output stored anyway
    // (training), the plain forward at its usual split followed by the gate kernel on the
    // stored output is then the faster way to the same result (measured on MI355X: below
    // about 192 chains).
    if (o && dtype == LTN_BF16 && chains < 192) {
        pb.p[0].gate = nullptr;
        pb.p[0].gated_out = nullptr;
        const ltn_status s1 = run_passes(pb, D, blk, dtype, workspace, st);
        if (s1 != LTN_OK) return s1;
        return ltn::launch_gate(o, u, nullptr, y, nullptr, eps, chains * N, D, 1, 0, st) == hipSuccess
                   ? LTN_OK : LTN_ERR_LAUNCH;
    }
    return run_passes(pb, D, blk, dtype, workspace, st, true);
}

ltn_status ltn_attn_fwd(const void* q, const void* k, const void* v, void* o,
                        const float* decay, const float* kv_in, float* kv_out,
                        int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                        void* workspace, size_t workspace_bytes, void* stream) {
    return fwd_common(q, k, v, nullptr, o, nullptr, decay, kv_in, kv_out, 0.0f, Bt, H, N, D, block, dtype,
                      workspace, workspace_bytes, stream, false);
}

ltn_status ltn_attn_fwd_static(const void* q, const void* k, const void* v, void* o,
                               const float* decay, const float* kv_in, float* kv_out,
                               int Bt, int H, long long N, int D, int block, ltn_dtype dtype, void* stream) {
    // the plan (and so the scratch it needs) is the one ltn_attn_fwd would take
    if (ltn_attn_workspace_bytes(Bt, H, N, D, block, dtype, 0) > kScratchBytes) return LTN_ERR_SCRATCH;
    void* ws = nullptr;
    const ltn_status s = scratch_on_current_device(&ws);
    if (s != LTN_OK) return s;
    // Nothing in the scratch has to start at zero: the scan reads exactly the segment end
    // states that the state-only sweep of the same call has written.
    return fwd_common(q, k, v, nullptr, o, nullptr, decay, kv_in, kv_out, 0.0f, Bt, H, N, D, block, dtype,
                      ws, kScratchBytes, stream, false);
}

ltn_status ltn_attn_fwd_gated(const void* q, const void* k, const void* v, const void* u, void* o, void* y,
                              const float* decay, const float* kv_in, float* kv_out, float eps,
                              int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                              void* workspace, size_t workspace_bytes, void* stream) {
    return fwd_common(q, k, v, u, o, y, decay, kv_in, kv_out, eps, Bt, H, N, D, block, dtype,
                      workspace, workspace_bytes, stream, true);
}

ltn_status ltn_attn_fwd_tiled(const void* q, const void* k, const void* v, void* o, const float* decay,
                              int Bt, int H, long long N, int D, ltn_dtype dtype, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || N == 0);
    if (!decay || (!empty && (!q || !k || !v || !o))) return LTN_ERR_NULL;
    if (Bt < 0 || H < 0 || N < 0 || D <= 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_BF16 || (D != 64 && D != 128)) return LTN_ERR_UNSUPPORTED;
    if ((long long)Bt * H > 0x3fffffffLL) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) ||
        (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    if (!empty) {
        const size_t tb = (size_t)Bt * H * (size_t)N * D * esize_of(dtype);
        const Span ins[3] = {{q, tb}, {k, tb}, {v, tb}};
        const Span outs[1] = {{o, tb}};
        if (outputs_alias(outs, 1, ins, 3)) return LTN_ERR_UNSUPPORTED;
    }
    if (empty) return LTN_OK;
    return ltn::launch_tiled_fwd_bf16(q, k, v, o, decay, Bt * H, H, N, D, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

ltn_status ltn_attn_bwd_tiled(const void* q, const void* k, const void* v, const void* d_o,
                              void* dq, void* dk, void* dv, const float* decay,
                              int Bt, int H, long long N, int D, ltn_dtype dtype, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || N == 0);
    if (!decay || (!empty && (!q || !k || !v || !d_o || !dq || !dk || !dv))) return LTN_ERR_NULL;
    if (Bt < 0 || H < 0 || N < 0 || D <= 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_BF16 || (D != 64 && D != 128)) return LTN_ERR_UNSUPPORTED;
    if ((long long)Bt * H > 0x3fffffffLL) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv) || (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    if (empty) return LTN_OK;
    const size_t tb = (size_t)Bt * H * (size_t)N * D * esize_of(dtype);
    const Span ins[4] = {{q, tb}, {k, tb}, {v, tb}, {d_o, tb}};
    const Span outs[3] = {{dq, tb}, {dk, tb}, {dv, tb}};
    if (outputs_alias(outs, 3, ins, 4)) return LTN_ERR_UNSUPPORTED;
    return ltn::launch_tiled_bwd_bf16(q, k, v, d_o, dq, dk, dv, decay, Bt * H, H, N, D,
                                      static_cast<hipStream_t>(stream)) == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

static ltn_status gate_common(const void* x, const void* u, const void* d_y, void* o0, void* o1, float eps,
                              long long rows, int D, ltn_dtype dtype, void* stream, bool bwd) {
    if (rows < 0 || D <= 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (D != 64 && D != 96 && D != 128 && D != 256) return LTN_ERR_UNSUPPORTED;
    if (!(eps >= 0.0f)) return LTN_ERR_SHAPE;
    if (rows == 0) return LTN_OK;
    if (!x || !u || !o0 || (bwd && (!d_y || !o1))) return LTN_ERR_NULL;
    if (!aligned16(x) || !aligned16(u) || !aligned16(d_y) || !aligned16(o0) || !aligned16(o1)) return LTN_ERR_ALIGN;
    {
        const size_t tb = (size_t)rows * D * esize_of(dtype);
        const Span ins[3] = {{x, tb}, {u, tb}, {d_y, tb}};
        const Span outs[2] = {{o0, tb}, {bwd ? o1 : nullptr, tb}};
        if (outputs_alias(outs, 2, ins, 3)) return LTN_ERR_UNSUPPORTED;
    }
    const hipError_t e = ltn::launch_gate(x, u, d_y, o0, o1, eps, rows, D, dtype == LTN_BF16, bwd,
                                          static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

ltn_status ltn_gate_fwd(const void* x, const void* u, void* y, float eps,
                        long long rows, int D, ltn_dtype dtype, void* stream) {
    return gate_common(x, u, nullptr, y, nullptr, eps, rows, D, dtype, stream, false);
}

ltn_status ltn_gate_bwd(const void* x, const void* u, const void* d_y, void* d_x, void* d_u, float eps,
                        long long rows, int D, ltn_dtype dtype, void* stream) {
    return gate_common(x, u, d_y, d_x, d_u, eps, rows, D, dtype, stream, true);
}

ltn_status ltn_attn_bwd(const void* q, const void* k, const void* v, const void* d_o,
                        void* dq, void* dk, void* dv, const float* decay,
                        int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                        void* workspace, size_t workspace_bytes, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || N == 0);
    if (!decay || (!empty && (!q || !k || !v || !d_o || !dq || !dk || !dv))) return LTN_ERR_NULL;
    int blk = 0;
    const ltn_status cs = check_common(Bt, H, N, D, block, dtype, &blk);
    if (cs != LTN_OK) return cs;
    const size_t need_ws = ltn_attn_workspace_bytes(Bt, H, N, D, block, dtype, 1);
    if (workspace_bytes < need_ws) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    const long long chains = (long long)Bt * H;
    if (!empty) {
        const size_t tb = (size_t)chains * (size_t)N * D * esize_of(dtype);
        const Span ins[4] = {{q, tb}, {k, tb}, {v, tb}, {d_o, tb}};
        const Span outs[4] = {{dq, tb}, {dk, tb}, {dv, tb}, {workspace, need_ws}};
        if (outputs_alias(outs, 4, ins, 4)) return LTN_ERR_UNSUPPORTED;
    }
    if (chains == 0 || N == 0) return LTN_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The three gradients are three decayed linear-attention passes with permuted
    // operands (derivative of O = ((Q K^T)(.)M) V; App. B Algorithm 4 corrected):
    //   dQ = ((dO V^T)(.)M)   K   -> pass(dO, V, K), first token -> last
    //   dV = ((Q K^T)(.)M)^T  dO  -> pass(K, Q, dO), last token -> first
    //   dK = ((dO V^T)(.)M)^T Q   -> pass(V, dO, Q), last token -> first
    ltn::PassBatch pb = {};
    pb.segs = 1;
    pb.count = 3;
    pb.decay = decay;
    pb.chains = (int)chains;
    pb.H = H;
    pb.N = N;
    pb.p[0] = ltn::PassArgs{k, q, d_o, dv, nullptr, nullptr, 1};
    pb.p[1] = ltn::PassArgs{v, d_o, q, dk, nullptr, nullptr, 1};
    pb.p[2] = ltn::PassArgs{d_o, v, k, dq, nullptr, nullptr, 0};
    pb.pairs_first = 1;
    return run_passes(pb, D, blk, dtype, workspace, st);
}

ltn_status ltn_attn_decode_steps(const void* q, const void* k, const void* v, void* o,
                                 float* kv, const float* decay,
                                 int Bt, int H, int S, int D, ltn_dtype dtype, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || S == 0);   // no token is read, the state is not touched
    if (!decay || (!empty && (!q || !k || !v || !o || !kv))) return LTN_ERR_NULL;
    if (Bt < 0 || H < 0 || S < 0 || D <= 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (D != 64 && D != 96 && D != 128 && D != 256) return LTN_ERR_UNSUPPORTED;
    if ((long long)Bt * H > 0x3fffffffLL) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(kv) ||
        (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    const int chains = Bt * H;
    if (!empty) {
        const size_t tb = (size_t)chains * S * D * esize_of(dtype);
        const Span ins[3] = {{q, tb}, {k, tb}, {v, tb}};
        const Span outs[2] = {{o, tb}, {kv, (size_t)chains * D * D * sizeof(float)}};
        if (outputs_alias(outs, 2, ins, 3)) return LTN_ERR_UNSUPPORTED;
    }
    if (empty) return LTN_OK;
    const hipError_t e = ltn::launch_decode(q, k, v, o, kv, decay, chains, H, S, D, D, dtype == LTN_BF16,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

ltn_status ltn_attn_decode_step(const void* q, const void* k, const void* v, void* o,
                                float* kv, const float* decay,
                                int Bt, int H, int D, ltn_dtype dtype, void* stream) {
    return ltn_attn_decode_steps(q, k, v, o, kv, decay, Bt, H, 1, D, dtype, stream);
}

// ---------------------------------------------------------------------------------------
// Query/key width Dk = 2 Dv (behind the LRPE-d expansion) and the input side itself.
// ---------------------------------------------------------------------------------------

static ltn_status check_dkdv(int Bt, int H, long long N, int Dk, int Dv, int block, ltn_dtype dtype, int* blk_out) {
    if (Bt < 0 || H < 0 || N < 0 || Dk <= 0 || Dv <= 0 || block < 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (!((Dk == 256 && Dv == 128) || (Dk == 128 && Dv == 64))) return LTN_ERR_UNSUPPORTED;
    int blk = block;
    if (dtype == LTN_BF16) {
        if (blk == 0) blk = 64;
        if (blk != 64) return LTN_ERR_UNSUPPORTED;
    } else {
        if (blk == 0) blk = Dk == 256 ? 16 : 32;
        if (blk != 16 && !(blk == 32 && Dk == 128)) return LTN_ERR_UNSUPPORTED;
    }
    if ((long long)Bt * H > 0x3fffffffLL) return LTN_ERR_SHAPE;
    *blk_out = blk;
    return LTN_OK;
}

// Slices the bf16 kernels exist for behind a DA-wide query/key side: 32..64 for 256 (its state
// copies fill the LDS beyond that) and for 64, 32..min(DC,128) otherwise; the state-only sweep
// of the sequence-parallel form uses the widest of them.
static int dkdv_hi(int DA, int DC) { return (DA == 256 || DA == 64) ? 64 : (DC < 128 ? DC : 128); }

// Sequence-parallel plan of a launch of `chain_passes` passes of shape (DA, DC): as for equal
// widths (pick_segments), with DC / hi workgroups per chain segment.  bf16 only.
static SegPlan pick_segments_dkdv(long long chain_passes, long long N, int DA, int DC, ltn_dtype dtype) {
    SegPlan plan = {1, 0};
    if (dtype != LTN_BF16 || chain_passes <= 0 || N <= 64) return plan;
    const long long per_seg = DC / dkdv_hi(DA, DC);
    long long want = 256 / (per_seg * chain_passes);
    if (want > N / 512) want = N / 512;       // segments of at least 512 tokens (measured: 2 .. 32 chains, N = 2048 .. 16384)
    if (want < kMinSegsFullWidth) want = 1;
    if (const int v = g_debug_segs.load(std::memory_order_relaxed)) want = v;
    if (want <= 1) return plan;
    long long len = (N + want - 1) / want;
    len = (len + 63) / 64 * 64;
    const long long segs = (N + len - 1) / len;
    if (segs <= 1 || segs > 0x7fff) return plan;
    plan.segs = (int)segs;
    plan.seg_len = len;
    return plan;
}

// One launch of `pb` (passes of one shape): a, b with DA features, c and out with DC; cut into
// segments (state-only sweep, scan, per-segment pass) when the plan says so.
static ltn_status run_dkdv(ltn::PassBatch& pb, int DA, int DC, int blk, ltn_dtype dtype, void* workspace, hipStream_t st) {
    const long long chain_passes = (long long)pb.chains * pb.count;
    pb.segs = 1;
    hipError_t e;
    if (dtype != LTN_BF16) {
        const int lo = 64, hi = (DA == 256) ? 64 : (DC < 128 ? DC : 128);
        e = ltn::launch_pass_f32(pb, DA, pick_dv_range(chain_passes, DC, lo, hi), blk, st, DC);
        return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
    }
    const int hi = dkdv_hi(DA, DC);
    const SegPlan plan = pick_segments_dkdv(chain_passes, pb.N, DA, DC, dtype);
    if (plan.segs == 1) {
        e = ltn::launch_pass_bf16(pb, DA, pick_dv_range(chain_passes, DC, 32, hi), st, DC);
        return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
    }
    if (!workspace) return LTN_ERR_NULL;
    float* states = static_cast<float*>(workspace);
    const size_t per_pass = (size_t)pb.chains * plan.segs * DA * DC;
    const float* kv_in = pb.p[0].state_in;
    float* kv_out = pb.p[0].state_out;
    ltn::PassBatch sweep = pb;
    sweep.segs = plan.segs;
    sweep.seg_len = plan.seg_len;
    sweep.state_only = 1;
    sweep.need_last = kv_out != nullptr;
    for (int i = 0; i < pb.count; ++i) {
        sweep.p[i].out = nullptr;
        sweep.p[i].state_in = nullptr;
        sweep.p[i].state_out = states + i * per_pass;
    }
    if (ltn::launch_pass_bf16(sweep, DA, hi, st, DC) != hipSuccess) return LTN_ERR_LAUNCH;
    if (ltn::launch_segment_scan(states, kv_in, kv_out, pb.decay, pb.count, pb.chains, pb.H, plan.segs, plan.seg_len,
                                 pb.N, DA, st, DC) != hipSuccess)
        return LTN_ERR_LAUNCH;
    ltn::PassBatch main = pb;
    main.segs = plan.segs;
    main.seg_len = plan.seg_len;
    for (int i = 0; i < pb.count; ++i) {
        main.p[i].state_in = states + i * per_pass;
        main.p[i].state_out = nullptr;
    }
    e = ltn::launch_pass_bf16(main, DA, pick_dv_range(chain_passes * plan.segs, DC, 32, hi), st, DC);
    return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

size_t ltn_attn_workspace_bytes_dkdv(int Bt, int H, long long N, int Dk, int Dv, ltn_dtype dtype, int call) {
    if (Bt <= 0 || H <= 0 || N <= 0 || call < 0 || call > 1) return 0;
    if (!((Dk == 256 && Dv == 128) || (Dk == 128 && Dv == 64))) return 0;
    const long long chains = (long long)Bt * H;
    const size_t state = (size_t)Dk * Dv * sizeof(float);
    // forward and the dV pass: (Dk, Dv), one pass per chain; dK and dQ: (Dv, Dk), two; the two
    // launches of the backward follow each other on the stream and share the workspace
    const SegPlan a = pick_segments_dkdv(chains, N, Dk, Dv, dtype);
    size_t need = a.segs > 1 ? (size_t)chains * a.segs * state : 0;
    if (call == 1) {
        const SegPlan b = pick_segments_dkdv(2 * chains, N, Dv, Dk, dtype);
        const size_t nb = b.segs > 1 ? (size_t)2 * chains * b.segs * state : 0;
        if (nb > need) need = nb;
    }
    return need;
}

ltn_status ltn_attn_fwd_dkdv(const void* q, const void* k, const void* v, void* o,
                             const float* decay, const float* kv_in, float* kv_out,
                             int Bt, int H, long long N, int Dk, int Dv, int block, ltn_dtype dtype,
                             void* workspace, size_t workspace_bytes, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || N == 0);
    if (!decay || (!empty && (!q || !k || !v || !o))) return LTN_ERR_NULL;
    int blk = 0;
    const ltn_status cs = check_dkdv(Bt, H, N, Dk, Dv, block, dtype, &blk);
    if (cs != LTN_OK) return cs;
    const size_t need_ws = ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, dtype, 0);
    if (workspace_bytes < need_ws) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(kv_in) ||
        !aligned16(kv_out) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    const long long chains = (long long)Bt * H;
    if (!empty) {
        const size_t qb = (size_t)chains * (size_t)N * Dk * esize_of(dtype), vb = (size_t)chains * (size_t)N * Dv * esize_of(dtype);
        const size_t sb = (size_t)chains * Dk * Dv * sizeof(float);
        const Span ins[4] = {{q, qb}, {k, qb}, {v, vb}, {kv_in == kv_out ? nullptr : kv_in, sb}};
        const Span outs[3] = {{o, vb}, {kv_out, sb}, {workspace, need_ws}};
        if (outputs_alias(outs, 3, ins, 4)) return LTN_ERR_UNSUPPORTED;
    }
    if (chains == 0) return LTN_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (N == 0) {
        if (!kv_out) return LTN_OK;
        return ltn::launch_state_copy(kv_in, kv_out, (size_t)chains * Dk * Dv, st) == hipSuccess
                   ? LTN_OK : LTN_ERR_LAUNCH;
    }
    ltn::PassBatch pb = {};
    pb.segs = 1;
    pb.count = 1;
    pb.decay = decay;
    pb.chains = (int)chains;
    pb.H = H;
    pb.N = N;
    pb.p[0] = ltn::PassArgs{q, k, v, o, kv_in, kv_out, 0};
    return run_dkdv(pb, Dk, Dv, blk, dtype, workspace, st);
}

ltn_status ltn_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o,
                             void* dq, void* dk, void* dv, const float* decay,
                             int Bt, int H, long long N, int Dk, int Dv, int block, ltn_dtype dtype,
                             void* workspace, size_t workspace_bytes, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || N == 0);
    if (!decay || (!empty && (!q || !k || !v || !d_o || !dq || !dk || !dv))) return LTN_ERR_NULL;
    int blk = 0;
    const ltn_status cs = check_dkdv(Bt, H, N, Dk, Dv, block, dtype, &blk);
    if (cs != LTN_OK) return cs;
    const size_t need_ws = ltn_attn_workspace_bytes_dkdv(Bt, H, N, Dk, Dv, dtype, 1);
    if (workspace_bytes < need_ws) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(d_o) || !aligned16(dq) ||
        !aligned16(dk) || !aligned16(dv) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    const long long chains = (long long)Bt * H;
    if (!empty) {
        const size_t qb = (size_t)chains * (size_t)N * Dk * esize_of(dtype), vb = (size_t)chains * (size_t)N * Dv * esize_of(dtype);
        const Span ins[4] = {{q, qb}, {k, qb}, {v, vb}, {d_o, vb}};
        const Span outs[4] = {{dq, qb}, {dk, qb}, {dv, vb}, {workspace, need_ws}};
        if (outputs_alias(outs, 4, ins, 4)) return LTN_ERR_UNSUPPORTED;
    }
    if (chains == 0 || N == 0) return LTN_OK;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The same three passes as ltn_attn_bwd; they come in two shapes, hence two launches:
    //   dV = pass(K, Q, dO), last token -> first:  Dk-wide a, b;  Dv-wide c, out
    //   dK = pass(V, dO, Q) (last -> first), dQ = pass(dO, V, K):  Dv-wide a, b;  Dk-wide c, out
    ltn::PassBatch pb = {};
    pb.segs = 1;
    pb.decay = decay;
    pb.chains = (int)chains;
    pb.H = H;
    pb.N = N;
    pb.count = 1;
    pb.p[0] = ltn::PassArgs{k, q, d_o, dv, nullptr, nullptr, 1};
    const ltn_status s1 = run_dkdv(pb, Dk, Dv, blk, dtype, workspace, st);
    if (s1 != LTN_OK) return s1;
    pb.count = 2;
    pb.p[0] = ltn::PassArgs{v, d_o, q, dk, nullptr, nullptr, 1};
    pb.p[1] = ltn::PassArgs{d_o, v, k, dq, nullptr, nullptr, 0};
    return run_dkdv(pb, Dv, Dk, blk, dtype, workspace, st);
}

ltn_status ltn_attn_decode_steps_dkdv(const void* q, const void* k, const void* v, void* o,
                                      float* kv, const float* decay,
                                      int Bt, int H, int S, int Dk, int Dv, ltn_dtype dtype, void* stream) {
    const bool empty = (Bt == 0 || H == 0 || S == 0);
    if (!decay || (!empty && (!q || !k || !v || !o || !kv))) return LTN_ERR_NULL;
    if (Bt < 0 || H < 0 || S < 0 || Dk <= 0 || Dv <= 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (!((Dk == 256 && Dv == 128) || (Dk == 128 && Dv == 64))) return LTN_ERR_UNSUPPORTED;
    if ((long long)Bt * H > 0x3fffffffLL) return LTN_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(kv) ||
        (reinterpret_cast<uintptr_t>(decay) & 3u))
        return LTN_ERR_ALIGN;
    if (!empty) {
        const size_t qb = (size_t)Bt * H * S * Dk * esize_of(dtype), vb = (size_t)Bt * H * S * Dv * esize_of(dtype);
        const Span ins[3] = {{q, qb}, {k, qb}, {v, vb}};
        const Span outs[2] = {{o, vb}, {kv, (size_t)Bt * H * Dk * Dv * sizeof(float)}};
        if (outputs_alias(outs, 2, ins, 3)) return LTN_ERR_UNSUPPORTED;
    }
    if (empty) return LTN_OK;
    const hipError_t e = ltn::launch_decode(q, k, v, o, kv, decay, Bt * H, H, S, Dk, Dv, dtype == LTN_BF16,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

ltn_status ltn_probe_stream_read(const void* buf, size_t buf_bytes, size_t bytes_per_workgroup, int workgroups,
                                 int iters, int to_registers, unsigned* sink, void* stream) {
    if (!buf || !sink) return LTN_ERR_NULL;
    if (workgroups <= 0 || iters <= 0 || bytes_per_workgroup == 0 || bytes_per_workgroup % 65536 != 0) return LTN_ERR_SHAPE;
    if (bytes_per_workgroup > buf_bytes / (size_t)workgroups) return LTN_ERR_SHAPE;      // every region inside the buffer
    if (!aligned16(buf) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return LTN_ERR_ALIGN;
    return ltn::launch_probe_stream(buf, bytes_per_workgroup, workgroups, iters, to_registers, sink,
                                    static_cast<hipStream_t>(stream)) == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

size_t ltn_prologue_workspace_bytes(int Bt, int H, long long N, int D) {
    if (Bt <= 0 || H <= 0 || N <= 0 || D <= 0) return 0;
    return (size_t)ltn::prologue_partial_count(N) * (size_t)H * (size_t)D * sizeof(double);
}

static ltn_status prologue_common(const void* x, const float* theta, const void* d_y, void* out, float* d_theta,
                                  int act, int Bt, int H, long long N, int D, long long pos0, ltn_dtype dtype,
                                  void* workspace, size_t workspace_bytes, void* stream, bool bwd) {
    if (Bt < 0 || H < 0 || N < 0 || D <= 0 || pos0 < 0) return LTN_ERR_SHAPE;
    if (dtype != LTN_F32 && dtype != LTN_BF16) return LTN_ERR_UNSUPPORTED;
    if (D != 64 && D != 128) return LTN_ERR_UNSUPPORTED;
    if ((long long)Bt * H > 0x3fffffffLL || pos0 + N > (1LL << 40)) return LTN_ERR_SHAPE;
    const bool empty = (Bt == 0 || H == 0 || N == 0);
    if (d_theta && !theta) return LTN_ERR_NULL;
    if (!empty && (!x || !out || (bwd && !d_y))) return LTN_ERR_NULL;
    const bool want_dtheta = bwd && theta && d_theta;
    if (want_dtheta && !empty) {
        if (workspace_bytes < ltn_prologue_workspace_bytes(Bt, H, N, D)) return LTN_ERR_SHAPE;
        if (!workspace) return LTN_ERR_NULL;
    }
    if (!aligned16(x) || !aligned16(d_y) || !aligned16(out) || !aligned16(workspace) ||
        (reinterpret_cast<uintptr_t>(theta) & 3u) || (reinterpret_cast<uintptr_t>(d_theta) & 3u))
        return LTN_ERR_ALIGN;
    if (!empty) {
        // x and d_x have D features per token; y and d_y have 2D behind the expansion, D without it
        const size_t xb = (size_t)Bt * H * (size_t)N * D * esize_of(dtype), yb = theta ? 2 * xb : xb;
        const size_t hb = (size_t)H * D * sizeof(float);
        const Span ins[3] = {{x, xb}, {d_y, yb}, {theta, hb}};
        const Span outs[3] = {{out, bwd ? xb : yb}, {d_theta, hb},
                              {want_dtheta ? workspace : nullptr, ltn_prologue_workspace_bytes(Bt, H, N, D)}};
        if (outputs_alias(outs, 3, ins, 3)) return LTN_ERR_UNSUPPORTED;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (empty) {
        // no token contributes: the angle gradient is zero
        if (want_dtheta && H > 0)
            return ltn::launch_state_copy(nullptr, d_theta, (size_t)H * D, st) == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
        return LTN_OK;
    }
    const hipError_t e = ltn::launch_prologue(x, theta, d_y, out, d_theta, static_cast<double*>(workspace), act != 0,
                                              Bt, H, N, D, pos0, dtype == LTN_BF16, bwd, st);
    return e == hipSuccess ? LTN_OK : LTN_ERR_LAUNCH;
}

ltn_status ltn_prologue_fwd(const void* x, const float* theta, void* y, int act,
                            int Bt, int H, long long N, int D, long long pos0, ltn_dtype dtype, void* stream) {
    return prologue_common(x, theta, nullptr, y, nullptr, act, Bt, H, N, D, pos0, dtype, nullptr, 0, stream, false);
}

ltn_status ltn_prologue_bwd(const void* x, const float* theta, const void* d_y, void* d_x, float* d_theta, int act,
                            int Bt, int H, long long N, int D, long long pos0, ltn_dtype dtype,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return prologue_common(x, theta, d_y, d_x, d_theta, act, Bt, H, N, D, pos0, dtype, workspace, workspace_bytes,
                           stream, true);
}

}  // extern "C"
