/*
 * ltn_attn.h -- C ABI of the MI355X (gfx950) Lightning Attention library.
 *
 * Lightning Attention is causal linear attention with a per-head exponential
 * decay (arXiv 2307.14995, Sec. 3.2.1; decay mask from Eq. 1 without the LRPE
 * phase, as Sec. 3.3 drops it):
 *
 *     O = ((Q K^T) (.) M_h) V,   M_h[t,s] = lambda_h^(t-s) for t >= s, else 0,
 *
 * with no 1/sqrt(d) scale, no softmax and no normaliser (Sec. 3.1.3).  The
 * library evaluates it blockwise: a masked intra-block tile product plus a
 * decay-scaled product with a running D x D state, the block form of the
 * recurrence  kv_t = lambda kv_{t-1} + k_t^T v_t,  o_t = q_t kv_t
 * (Sec. 3.3, Algorithm 2).
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers into caller-owned memory.  The
 *     library never allocates, frees or keeps a pointer after the call returns.
 *   - Tensors are contiguous row-major [Bt, H, N, D] (batch, head, token,
 *     feature) in `dtype` (fp32, or bf16 stored as 16-bit words).  `decay` is a
 *     device array of H fp32 values lambda_h in [0, 1]; values are not read on
 *     the host (use ltn_attn_check_decay on a host copy to validate them).
 *   - States are fp32 [Bt, H, D, D] with kv[b,h,i,j] = sum_s w_s k_s[i] v_s[j]
 *     (row = key feature, column = value feature).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  Calls return without synchronising.
 *   - Outputs are fully overwritten; inputs are never written.  An output whose
 *     bytes overlap an input's or another output's (not only equal base
 *     pointers; the workspace counts as an output) is rejected
 *     (LTN_ERR_UNSUPPORTED).  The one exception: kv_out may be kv_in itself.
 *   - Errors are return codes only.  Argument errors are detected on the host
 *     before anything is launched.  Bt == 0 or H == 0 is a successful no-op; when
 *     Bt * H * N == 0 the token tensors are not touched and may be NULL.
 *   - Arithmetic: bf16 tensors use bf16 MFMA with fp32 accumulation and an fp32
 *     running state; fp32 tensors use fp32 arithmetic throughout (fp32 MFMA for plain
 *     passes with D in {64, 128}, fp32 multiply-adds elsewhere).  Only
 *     non-negative powers of lambda are ever formed, so lambda = 0 and
 *     lambda = 1 are exact and strong decays cannot overflow (the failure mode
 *     Sec. 3.3 describes for the factorised form of Algorithm 1).
 *   - Supported shapes: D in {64, 96, 128, 256} for ltn_attn_fwd, ltn_attn_bwd, the decode
 *     steps, the gate kernels and the gated forward (which for 256 features, and for 96 in
 *     fp32, needs its `o` argument); D in {64, 128} for the tiled comparison kernels; N >= 0
 *     arbitrary (a short last block
 *     is handled on chip; the paper's listings assume block | N).
 *     `block` is the intra-block tile length: 0 lets the library choose
 *     (ltn_attn_pick_block); bf16 supports 64; fp32 supports 16, 32 and 64
 *     with D * block <= 4096 (D = 96 counts as 128 there: its tiles are 128 wide
 *     on chip, the last columns zero).
 *   - Results are bitwise reproducible run to run for fixed arguments (no
 *     floating-point atomics).
 */
#ifndef LTN_ATTN_H
#define LTN_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LTN_OK = 0,
    LTN_ERR_NULL = 1,        /* a required pointer is NULL                          */
    LTN_ERR_SHAPE = 2,       /* negative size, or workspace too small               */
    LTN_ERR_UNSUPPORTED = 3, /* D / block / dtype combination not built, aliasing   */
    LTN_ERR_ALIGN = 4,       /* a tensor pointer is not 16-byte aligned             */
    LTN_ERR_DECAY = 5,       /* ltn_attn_check_decay: a value outside [0, 1] or NaN */
    LTN_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch                  */
    LTN_ERR_SCRATCH = 7,     /* ltn_attn_fwd_static: needs more than the static scratch */
    /* not status codes: they make every int a valid value of the type, so that a caller
     * (or a foreign-function binding) passing an unknown code is an error path, not
     * undefined behaviour in a C++ implementation */
    LTN_STATUS_INT_MIN_ = -2147483647 - 1, LTN_STATUS_INT_MAX_ = 2147483647
} ltn_status;

typedef enum { LTN_F32 = 0, LTN_BF16 = 1,
               LTN_DTYPE_INT_MIN_ = -2147483647 - 1, LTN_DTYPE_INT_MAX_ = 2147483647 /* as above */
} ltn_dtype;

/*
 * Forward pass (Sec. 3.2.1; App. B Algorithm 3 computes the same O with a
 * quadratic tile loop -- this library uses the linear-cost block recurrence).
 *
 *   o[b,h,t,:] = sum_{s<=t} lambda_h^(t-s) (q_t . k_s) v_s  +  lambda_h^(t+1) q_t kv_in[b,h]
 *
 *   q, k, v  in : device, [Bt,H,N,D] dtype
 *   o        out: device, [Bt,H,N,D] dtype
 *   decay    in : device, [H] fp32
 *   kv_in    in : device, [Bt,H,D,D] fp32, or NULL for a zero initial state
 *   kv_out   out: device, [Bt,H,D,D] fp32, or NULL; receives the state after the
 *                 last token (kv_{N-1} of Algorithm 2); may alias kv_in
 *   workspace   : device scratch of at least ltn_attn_workspace_bytes(...) bytes
 *                 (may be NULL when that is 0)
 * N == 0 copies kv_in (or zeros) to kv_out and does nothing else.
 */
ltn_status ltn_attn_fwd(const void* q, const void* k, const void* v, void* o,
                        const float* decay, const float* kv_in, float* kv_out,
                        int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * ltn_attn_fwd for callers that cannot allocate device memory and so have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, results (bit for bit) and errors as ltn_attn_fwd, without
 * the workspace pair: where ltn_attn_fwd would use a workspace (few long chains, cut into
 * segments), this entry point uses a scratch buffer of LTN_ATTN_STATIC_SCRATCH_BYTES that
 * is part of the library's device code (every GPU the library runs on holds one copy
 * until the process ends).  It calls no hipMalloc / hipFree and no allocating routine.
 *   - A call whose plan needs more scratch than that returns LTN_ERR_SCRATCH and launches
 *     nothing (the library's own plans need at most 16 MiB: 256 segment states of 64 KB).
 *   - The device that owns `stream` must be the current device.  The first call on a
 *     device looks up the buffer's address (once per device); make that call outside graph
 *     capture.
 *   - All calls on one GPU share the one buffer: calls that overlap in time on the same GPU
 *     (different streams, different threads) race and must be serialised by the caller.
 *     Its contents are scratch and mean nothing between calls.
 */
#define LTN_ATTN_STATIC_SCRATCH_BYTES (16u << 20)
ltn_status ltn_attn_fwd_static(const void* q, const void* k, const void* v, void* o,
                               const float* decay, const float* kv_in, float* kv_out,
                               int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                               void* stream);

/*
 * Forward pass with the token mixer's epilogue fused in (Sec. 3.1.2, Eq. 3:
 * O = Norm(Q K^T V) (.) U, with the SimpleRMSNorm of Sec. 3.1.3,
 * SRMSNorm(x) = x / (|x|_2 / sqrt(d)), taken per head over its D features):
 *
 *   o as in ltn_attn_fwd;   y[b,h,t,:] = o[b,h,t,:] / sqrt(mean_d(o[b,h,t,:]^2) + eps) (.) u[b,h,t,:]
 *
 * The normalisation and the gate are applied to the fp32 attention output while
 * it is still on chip, so an inference caller (o == NULL) never writes or re-reads
 * the attention output; a training caller passes `o` as well, because the
 * derivative of the epilogue (ltn_gate_bwd) needs it.
 *
 *   u     in : device, [Bt,H,N,D] dtype  (the gate)
 *   o     out: device, [Bt,H,N,D] dtype, or NULL
 *   y     out: device, [Bt,H,N,D] dtype
 * (With few chains and `o` requested, the library may instead run the plain forward and
 * apply the epilogue to the stored o in a second kernel; y then derives from o rounded
 * to `dtype`, so the two forms of the call agree to rounding, not bit for bit.  For D = 256,
 * and for D = 96 in fp32, that is the only form: no kernel there holds a complete output row
 * in one workgroup, so `o` must be given -- LTN_ERR_UNSUPPORTED otherwise.)
 *   eps   >= 0, added to the mean square under the root (0 is the printed formula:
 *         an all-zero output row then yields NaN, as the formula does)
 * Other arguments, layout and errors as for ltn_attn_fwd.
 */
ltn_status ltn_attn_fwd_gated(const void* q, const void* k, const void* v, const void* u, void* o, void* y,
                              const float* decay, const float* kv_in, float* kv_out, float eps,
                              int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same epilogue on its own, row by row (Sec. 3.1.2 Eq. 3, Sec. 3.1.3):
 *   y[r,:] = x[r,:] / sqrt(mean(x[r,:]^2) + eps) (.) u[r,:]
 * and its derivative: with n = x / sqrt(mean(x^2) + eps) and g = d_y (.) u,
 *   d_u = d_y (.) n,    d_x = (g - n * mean(g (.) n)) / sqrt(mean(x^2) + eps).
 * In training, d_x is the d_o handed to ltn_attn_bwd.
 *
 *   x, u, d_y in : device, [rows, D] dtype (for attention tensors rows = Bt*H*N)
 *   y, d_x, d_u out: device, [rows, D] dtype; must not alias an input or each other
 *   D in {64, 96, 128, 256}; fp32 arithmetic inside for either dtype.
 */
ltn_status ltn_gate_fwd(const void* x, const void* u, void* y, float eps,
                        long long rows, int D, ltn_dtype dtype, void* stream);
ltn_status ltn_gate_bwd(const void* x, const void* u, const void* d_y, void* d_x, void* d_u, float eps,
                        long long rows, int D, ltn_dtype dtype, void* stream);

/*
 * The same forward output by the paper's own evaluation order (App. B, Algorithm 3): every
 * block of 64 queries loops over all key/value blocks up to its own, with the decay mask
 * tile generated on chip.  Quadratic in N; kept as a comparison kernel (where on the N axis
 * it loses to the state recurrence of ltn_attn_fwd is part of the report), zero initial
 * state, no state output, bf16 only (LTN_ERR_UNSUPPORTED otherwise).
 *
 *   q, k, v in : device, [Bt,H,N,D] bf16      o out: device, [Bt,H,N,D] bf16
 */
ltn_status ltn_attn_fwd_tiled(const void* q, const void* k, const void* v, void* o, const float* decay,
                              int Bt, int H, long long N, int D, ltn_dtype dtype, void* stream);

/*
 * The gradients by the paper's own evaluation order (App. B, Algorithm 4, with its misprints
 * corrected as in ltn_attn_bwd): one workgroup per block of 64 keys/values keeps K_j, V_j on
 * chip, loops over all query blocks i >= j and accumulates dK_j and dV_j; dQ_i comes from a
 * second kind of workgroup that loops over j <= i and forms dA_ij = (dO_i V_j^T) (.) M_ij
 * again, in place of the listing's read-modify-write of dQ_i in memory (no atomics).
 * Quadratic in N; a comparison kernel like ltn_attn_fwd_tiled, bf16 only, D in {64, 128}.
 *
 *   q, k, v, d_o in : device, [Bt,H,N,D] bf16      dq, dk, dv out: device, [Bt,H,N,D] bf16
 */
ltn_status ltn_attn_bwd_tiled(const void* q, const void* k, const void* v, const void* d_o,
                              void* dq, void* dk, void* dv, const float* decay,
                              int Bt, int H, long long N, int D, ltn_dtype dtype, void* stream);

/*
 * Backward pass: gradients of the definition above (App. B Algorithm 4 read
 * with its misprints corrected: dK = dA^T Q, dQ accumulates dA K).  With
 * A = (Q K^T)(.)M and dA = (dO V^T)(.)M:  dQ = dA K, dK = dA^T Q, dV = A^T dO.
 * Nothing saved by the forward is needed (the paper trains with activation
 * recomputation, Sec. 3.2): inputs are q, k, v and d_o only, zero initial state.
 *
 *   q, k, v, d_o in : device, [Bt,H,N,D] dtype
 *   dq, dk, dv   out: device, [Bt,H,N,D] dtype
 */
ltn_status ltn_attn_bwd(const void* q, const void* k, const void* v, const void* d_o,
                        void* dq, void* dk, void* dv, const float* decay,
                        int Bt, int H, long long N, int D, int block, ltn_dtype dtype,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * One recurrent decode step (Sec. 3.3, Algorithm 2, one loop iteration):
 *     kv <- lambda_h kv + k^T v   (in place),   o = q kv   (the updated state)
 *
 *   q, k, v in : device, [Bt,H,D] dtype       o out: device, [Bt,H,D] dtype
 *   kv  in/out : device, [Bt,H,D,D] fp32
 */
ltn_status ltn_attn_decode_step(const void* q, const void* k, const void* v, void* o,
                                float* kv, const float* decay,
                                int Bt, int H, int D, ltn_dtype dtype, void* stream);

/*
 * S consecutive decode steps in one call (Algorithm 2, S loop iterations): the state is
 * read once, kept on chip over the S tokens and written once, for callers that hold
 * several tokens per sequence (a short prompt tail, drafted tokens).
 *     for s = 0..S-1:  kv <- lambda_h kv + k_s^T v_s,   o_s = q_s kv
 *
 *   q, k, v in : device, [Bt,H,S,D] dtype     o out: device, [Bt,H,S,D] dtype
 *   kv  in/out : device, [Bt,H,D,D] fp32      S == 0 is a successful no-op
 * All arithmetic is fp32 whatever `dtype` is, and the result is bit for bit that of S
 * single-token calls.  The loop is bound by its fp32 multiply-adds from about 8 tokens per
 * call on: a caller with more tokens per sequence than that (bf16 tensors) gets the same
 * state and outputs, to rounding, faster from ltn_attn_fwd(q, k, v, o, ..., kv_in = kv,
 * kv_out = kv, N = S), which evaluates the S iterations blockwise with bf16 MFMA
 * (measured on MI355X, 2048 chains: 16 tokens 66 us against 101 us, 64 tokens 79 us
 * against 312 us).  The library does not switch by itself because the two differ in
 * rounding.
 */
ltn_status ltn_attn_decode_steps(const void* q, const void* k, const void* v, void* o,
                                 float* kv, const float* decay,
                                 int Bt, int H, int S, int D, ltn_dtype dtype, void* stream);

/*
 * Input side of the token mixer, applied to queries and to keys (one call per tensor):
 * the activation of Sec. 3.1.2 Eq. 2 (Q = phi(X W_q), K = phi(X W_k), phi = swish,
 * z = x / (1 + exp(-x))) and the position encoding of Sec. 3.1.1 Eq. 1 (LRPE-d),
 *
 *     a[t,s] = q_t^T k_s lambda^(t-s) exp(i theta (t-s)).
 *
 * The paper prints the complex form only; this library reads it with one real learnable
 * angle per head and feature, theta[h,d], acting feature by feature, and the real part as
 * the score: a[t,s] = lambda^(t-s) sum_d q_t[d] k_s[d] cos(theta[h,d] (t-s)).  It "can be
 * decomposed with respect to s and t separately" (Sec. 3.1.1): with p the absolute position
 * of a token,
 *
 *     y[b,h,t,:] = [ z (.) cos(theta_h p) | z (.) sin(theta_h p) ],     p = pos0 + t,
 *
 * for queries and keys alike gives y_q(t) . y_k(s) = that score without the decay, so the
 * attention entry points for Dk = 2 Dv below finish the job.  Only differences of positions
 * matter; pos0 lets a later chunk (chunked prefill, decode) continue an earlier one.
 *
 *   x      in : device, [Bt,H,N,D] dtype
 *   theta  in : device, [H,D] fp32, or NULL: no position encoding, y = z with D features
 *   y      out: device, [Bt,H,N,2D] dtype ([Bt,H,N,D] when theta is NULL)
 *   act       : nonzero applies swish, 0 passes x through (z = x)
 *   pos0      : absolute position of token 0, 0 <= pos0, pos0 + N <= 2^40
 * D in {64, 128}.  The angle theta p is formed and reduced in fp64, everything else in fp32;
 * outputs are rounded once to `dtype`.
 */
ltn_status ltn_prologue_fwd(const void* x, const float* theta, void* y, int act,
                            int Bt, int H, long long N, int D, long long pos0,
                            ltn_dtype dtype, void* stream);

/*
 * Derivative of ltn_prologue_fwd for one tensor:
 *     dz = dy_c (.) cos + dy_s (.) sin,   dx = dz (.) phi'(x),
 *     d_theta[h,d] = sum over b and t of  p z (dy_s cos - dy_c sin)
 * (the caller adds the d_theta of the query call and of the key call: theta is shared).
 *
 *   x, theta, act, pos0 : as given to the forward
 *   d_y     in : device, [Bt,H,N,2D] dtype ([Bt,H,N,D] when theta is NULL)
 *   d_x     out: device, [Bt,H,N,D] dtype
 *   d_theta out: device, [H,D] fp32, overwritten; NULL skips it (and must be NULL when
 *                theta is NULL)
 *   workspace  : device scratch of ltn_prologue_workspace_bytes(...) bytes, needed only
 *                when d_theta is wanted (the sum is taken in a fixed order, in fp64, through
 *                per-workgroup partial sums: reproducible, no atomics)
 */
ltn_status ltn_prologue_bwd(const void* x, const float* theta, const void* d_y, void* d_x,
                            float* d_theta, int act,
                            int Bt, int H, long long N, int D, long long pos0, ltn_dtype dtype,
                            void* workspace, size_t workspace_bytes, void* stream);

size_t ltn_prologue_workspace_bytes(int Bt, int H, long long N, int D);

/*
 * Forward, gradients and decode with query/key width Dk different from the value width
 * Dv -- what the attention sees behind the LRPE-d expansion above (Dk = 2 Dv).  Same
 * definition, same conventions and the same kernels as ltn_attn_fwd / ltn_attn_bwd /
 * ltn_attn_decode_steps (Sec. 3.2.1; Sec. 3.3 Algorithm 2 never uses that the widths agree):
 *
 *   q, k, dq, dk : [Bt,H,N,Dk]        v, o, d_o, dv : [Bt,H,N,Dv]
 *   kv_in, kv_out, kv : fp32 [Bt,H,Dk,Dv]  (row = key feature, column = value feature)
 *   decode: q, k [Bt,H,S,Dk];  v, o [Bt,H,S,Dv]
 *
 * Supported: (Dk, Dv) in {(256,128), (128,64)}; equal widths go through the entry points
 * above (LTN_ERR_UNSUPPORTED here).  block: 0 = library's choice; bf16 64; fp32 16, or 32
 * when Dk = 128.  workspace: device scratch of ltn_attn_workspace_bytes_dkdv(...) bytes (0
 * unless few chains meet a long sequence, as for ltn_attn_fwd / ltn_attn_bwd; call = 0 for
 * the forward, 1 for the backward); too small -> LTN_ERR_SHAPE, NULL when needed ->
 * LTN_ERR_NULL.
 */
ltn_status ltn_attn_fwd_dkdv(const void* q, const void* k, const void* v, void* o,
                             const float* decay, const float* kv_in, float* kv_out,
                             int Bt, int H, long long N, int Dk, int Dv, int block,
                             ltn_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

ltn_status ltn_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* d_o,
                             void* dq, void* dk, void* dv, const float* decay,
                             int Bt, int H, long long N, int Dk, int Dv, int block,
                             ltn_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

size_t ltn_attn_workspace_bytes_dkdv(int Bt, int H, long long N, int Dk, int Dv, ltn_dtype dtype, int call);

ltn_status ltn_attn_decode_steps_dkdv(const void* q, const void* k, const void* v, void* o,
                                      float* kv, const float* decay,
                                      int Bt, int H, int S, int Dk, int Dv,
                                      ltn_dtype dtype, void* stream);

/* Block length the library uses for (D, dtype) when `block` is 0; 0 if unsupported.
 * The paper leaves the block sizes B_r, B_c of its tiling as inputs (App. B, Algorithms 3
 * and 4); the result does not depend on them beyond rounding.  bf16: 64 for every D (a
 * 128-token block does not leave room for two pipeline stages in the 160 KB of LDS, a
 * 32-token block doubles the per-token cost of reading the state copy); fp32: the largest
 * of 16, 32, 64 whose tiles fit. */
int ltn_attn_pick_block(int D, ltn_dtype dtype);

/* The launch plan the library takes for these arguments (call as in
 * ltn_attn_workspace_bytes): value columns per workgroup in *dv, segments per chain in
 * *segs (1 = whole chains).  For reports that need to name the kernel variant that ran. */
ltn_status ltn_attn_query_plan(int Bt, int H, long long N, int D, ltn_dtype dtype, int call,
                               int* dv, int* segs);

/* TEST ONLY.  Forces the launch plan of ltn_attn_fwd / ltn_attn_bwd / ltn_attn_fwd_gated for
 * the whole process until called again: dv = value columns per workgroup (0 = the library's
 * choice; a value the kernels do not have for a given D is ignored), segs = segments per
 * chain (0 = the library's choice, 1 = never cut).  It exists so that the parity tests can
 * reach every kernel variant at small sizes; it also changes what
 * ltn_attn_workspace_bytes returns.  Not thread-safe against concurrent calls into the
 * library.  LTN_ERR_SHAPE for values outside {0, 16, 32, 64, 96, 128, 256} / [0, 4096]. */
ltn_status ltn_attn_set_debug_plan(int dv, int segs);

/* Scratch bytes a call needs for these arguments: call = 0 for ltn_attn_fwd, 1 for
 * ltn_attn_bwd, 2 for ltn_attn_fwd_gated.  A smaller workspace makes the call fail with
 * LTN_ERR_SHAPE; a NULL one with LTN_ERR_NULL when bytes are needed.  It is 0 except
 * when few chains meet a long sequence: then every chain is cut into segments that run
 * in parallel (the recurrence of Sec. 3.3 is linear in the state, so the segments' end
 * states can be computed from zero and combined by a scan), and the workspace holds one
 * fp32 D x D state per (pass, chain, segment).  For ltn_attn_fwd_gated the figure covers
 * both of its forms (fused, and plain forward followed by the gate kernel).  Contents are
 * scratch: undefined before and after the call. */
size_t ltn_attn_workspace_bytes(int Bt, int H, long long N, int D, int block,
                                ltn_dtype dtype, int call);

/* Measurement aid (no attention arithmetic): `workgroups` workgroups of 512 threads each read
 * their own contiguous bytes_per_workgroup bytes (a multiple of 64 KB) of `buf` `iters`
 * times, eight 1 KB loads in flight per wave, straight into LDS (to_registers = 0, the way the
 * attention kernels fetch their tiles) or into registers (1).  The benchmark's report times
 * it to state what rate this machine gives such a pipeline out of L2, the memory-side cache
 * and HBM, next to the published 8 TB/s.  buf: device, buf_bytes >= workgroups *
 * bytes_per_workgroup, read only; sink: device, one word, written only if the data matches a
 * magic pattern (it keeps the loads alive). */
ltn_status ltn_probe_stream_read(const void* buf, size_t buf_bytes, size_t bytes_per_workgroup, int workgroups,
                                 int iters, int to_registers, unsigned* sink, void* stream);

/* Host-side validation of a HOST copy of the decay array: LTN_OK if every value
 * is in [0, 1], LTN_ERR_DECAY otherwise (Eq. 2 gives values in (0, 1]; the last
 * layer uses exactly 1). */
ltn_status ltn_attn_check_decay(const float* decay_host, int H);

/* Static, human-readable name of a status code. */
const char* ltn_status_str(ltn_status s);

#ifdef __cplusplus
}
#endif
#endif /* LTN_ATTN_H */
