/*
 * la.h - C ABI of the MI355X (gfx950) Lightning Attention library.
 *
 * The library computes causal linear attention with a per-head decay rate,
 * forward and backward, with the tiled algorithm of Lightning Attention:
 * each sequence block is split into an intra-block part computed as a masked
 * left product and an inter-block part computed as a right product against a
 * running d x d state (Alg. 3/4; with decay Alg. 5/6 and App. C).
 *
 * Result definition (per batch b and head h, lambda = lambda[h], rows t, s):
 *
 *     O[t]  = sum_{s <= t} lambda^(t-s) (Q[t] . K[s]) V[s]          (App. A)
 *     dQ[t] = sum_{s <= t} lambda^(t-s) (dO[t] . V[s]) K[s]
 *     dK[s] = sum_{t >= s} lambda^(t-s) (dO[t] . V[s]) Q[t]
 *     dV[s] = sum_{t >= s} lambda^(t-s) (Q[t] . K[s]) dO[t]         (App. C)
 *
 * No 1/sqrt(d) scaling and no normalisation are applied (Sec. 3.1); lambda
 * is a constant and receives no gradient (Sec. 4.1).
 *
 * Conventions common to every entry point
 *   - Tensor arguments are DEVICE pointers owned by the caller, contiguous
 *     [B, H, n, d] with d fastest, 16-byte aligned.  Outputs are fully
 *     overwritten (never accumulated into).  Inputs and outputs must not alias.
 *   - `lambda` is a HOST pointer to H floats; it is read during the call and
 *     need not outlive it.  Every entry must be finite with 0 < lambda <= 1.
 *   - d is 64 or 128; B, H, n >= 1; H <= LA_MAX_HEADS; n <= LA_MAX_SEQ_LEN.  n need not be a
 *     multiple of the tile length: the tail behaves as if zero-padded, which
 *     is exact.
 *   - dt = LA_BF16: tensors are bfloat16; contractions use bf16 operands with
 *     fp32 accumulation and the running state is kept in fp32.
 *     dt = LA_F32: tensors and all arithmetic are fp32.
 *   - `workspace` is a DEVICE pointer to at least la_workspace_bytes(...)
 *     bytes, 256-byte aligned, owned by the caller; it may be NULL when that
 *     query returns 0.  Its contents are scratch (segment states) and need
 *     not be initialised or preserved.  The library itself allocates nothing.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Work is enqueued on it and the call returns without synchronising.
 *   - The return value is an la_status; nothing is thrown, errno is untouched.
 *     On any error nothing has been enqueued, except LA_ERR_LAUNCH, which
 *     reports a failed kernel launch part-way through the call.
 *   - Calls are thread-safe (no global mutable state apart from the optional
 *     profiling hooks below) and results are bitwise reproducible from run to
 *     run: no atomics are used in any reduction.  The environment is never read.
 *   - Every entry point that takes a stream only launches kernels on it (no memory-set or
 *     copy nodes, no events unless the profiling hooks are on), so calls can be recorded
 *     into a HIP graph by stream capture and replayed.  The first launch of each kernel in
 *     a process sets a function attribute (its dynamic LDS size): make one ordinary call
 *     of the same entry point and shape before capturing.
 *   - The launch planner is written for MI355X: it assumes 256 compute units when it
 *     decides whether, and how finely, a sequence is cut into segments.  On a part
 *     with another count the results are the same, only the occupancy differs.
 */
#ifndef LA_H
#define LA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LA_MAX_HEADS 256
#define LA_MAX_SEQ_LEN 1073741823   /* 2^30 - 1: longer n gives LA_ERR_SHAPE */

/* (the two bounds only widen the enum's range to that of int, so that any value a caller
 * passes can be inspected and refused with LA_ERR_DTYPE) */
typedef enum { LA_F32 = 0, LA_BF16 = 1, LA_DTYPE_MIN_ = -2147483647 - 1, LA_DTYPE_MAX_ = 2147483647 } la_dtype;

typedef enum {
    LA_OK = 0,
    LA_ERR_NULL = -1,       /* a required pointer is NULL                       */
    LA_ERR_SHAPE = -2,      /* B, H, n < 1, H > LA_MAX_HEADS, or d not 64 / 128  */
    LA_ERR_DTYPE = -3,      /* dt is not LA_F32 or LA_BF16                      */
    LA_ERR_LAMBDA = -4,     /* a decay rate is not finite or not in (0, 1]      */
    LA_ERR_WORKSPACE = -5,  /* workspace NULL / misaligned / too small          */
    LA_ERR_LAUNCH = -6,     /* a HIP launch failed                              */
    LA_ERR_ALIGN = -7,      /* a tensor pointer is not 16-byte aligned          */
    LA_ERR_TOO_LARGE = -8   /* la_fwd_static: needs more than its static scratch */
} la_status;

/*
 * Bytes of device scratch that la_fwd (is_bwd = 0) or la_bwd (is_bwd != 0)
 * needs for this problem size.  The scratch holds the d x d fp32 states at
 * segment boundaries when a sequence is cut into segments so that a small
 * B*H still fills the GPU (the block recurrence of App. C, "KV_t" and
 * "dKV_t", applied at segment instead of block granularity); la_bwd needs twice
 * what la_fwd needs.  Returns 0 when
 * no scratch is needed or when the arguments are invalid.  Pure host
 * arithmetic: callable without a GPU.
 */
size_t la_workspace_bytes(int B, int H, int n, int d, la_dtype dt, int is_bwd);

/*
 * Forward pass (Alg. 5; Alg. 3 when lambda = 1):
 *     O = lightning_attention(Q, K, V, lambda).
 * Q, K, V: inputs; O: output; all [B, H, n, d] of type dt, device memory.
 */
int la_fwd(const void *Q, const void *K, const void *V,
           const float *lambda /* host, [H] */,
           void *O,
           int B, int H, int n, int d, la_dtype dt,
           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * la_fwd for callers that cannot allocate and have no workspace to give: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and
 * bit-identical results, but the segment states live in a buffer of
 * LA_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy per GPU
 * the library runs on, held until the process ends) instead of a caller workspace.  The
 * call allocates nothing and calls no allocating routine; its first use on a device looks
 * up that buffer's address (hipGetSymbolAddress), later calls reuse it.  The device the
 * tensors and `hip_stream` belong to must be the current device.
 * A problem for which la_workspace_bytes(B, H, n, d, dt, 0) exceeds
 * LA_STATIC_SCRATCH_BYTES is refused with LA_ERR_TOO_LARGE and nothing is enqueued.
 * (The planner cuts a problem into fewer than 768 (scan, segment) pieces of 64 KB at
 * d = 128 and fewer than 1280 of 16 KB at d = 64, so 64 MiB holds every plan it makes by
 * itself, whatever B, H and n.)
 * All calls on one GPU share that GPU's buffer: calls that may overlap in time on one GPU
 * (different streams, different threads) race and must be serialised by the caller.
 * Nothing in the buffer needs clearing between calls.
 */
#define LA_STATIC_SCRATCH_BYTES (64u << 20)
int la_fwd_static(const void *Q, const void *K, const void *V,
                  const float *lambda /* host, [H] */,
                  void *O,
                  int B, int H, int n, int d, la_dtype dt, void *hip_stream);

/*
 * Backward pass (Alg. 6; Alg. 4 when lambda = 1): given dO = dLoss/dO,
 * writes dQ, dK, dV.  Takes no saved forward context and not O (the
 * algorithm lists O among its loads but never uses it); the forward state
 * it needs is recomputed.
 */
int la_bwd(const void *Q, const void *K, const void *V,
           const float *lambda /* host, [H] */,
           const void *dO,
           void *dQ, void *dK, void *dV,
           int B, int H, int n, int d, la_dtype dt,
           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward pass that reuses what the forward pass already computed.  When a sequence
 * is cut into segments (la_workspace_bytes(..., 0) > 0), la_fwd leaves the segment
 * states of scan(Q, K, V) in its workspace; the dQ scan of the backward pass needs
 * exactly their transposes (App. C: both are the KV state at segment boundaries).
 * `fwd_workspace` is the buffer a completed la_fwd call with the same Q, K, V, lambda,
 * B, H, n, d, dt used, unmodified since; it is only read.  `workspace` then needs only
 * la_workspace_bytes(..., is_bwd = 0) bytes (the reverse states) and must be a
 * different buffer.  Results equal la_bwd's up to the rounding order of those states.
 * When no segmentation is needed (that query returns 0) both may be NULL and this is
 * la_bwd.  A training step that keeps the forward workspace saves half of the
 * backward pre-pass.
 */
int la_bwd_saved(const void *Q, const void *K, const void *V,
                 const float *lambda /* host, [H] */,
                 const void *dO,
                 void *dQ, void *dK, void *dV,
                 const void *fwd_workspace,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward pass with a carried state (the next step after la_fwd / la_bwd: the
 * paper's inference use, Sec. 3.1, where only the d x d state K^T V is kept
 * between calls; the recurrence is App. A's with kv_0 = kv_in):
 *     kv_{-1} = kv_in ;  kv_t = lambda kv_{t-1} + k_t v_t^T ;  o_t^T = q_t^T kv_t ;
 *     kv_out = kv_{n-1}.
 * kv_in, kv_out: DEVICE pointers to [B, H, d, d] fp32 (rows = key feature,
 * columns = value feature), 16-byte aligned; either may be NULL (zero state in,
 * no state out); they may be the same buffer.  Everything else as la_fwd; with
 * both NULL this is la_fwd.  Long prompts can be fed in pieces of any length.
 */
int la_fwd_state(const void *Q, const void *K, const void *V,
                 const float *lambda /* host, [H] */,
                 void *O, const float *kv_in, float *kv_out,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One decode token (App. A, recurrence form), for every (batch, head):
 *     kv <- lambda kv + k v^T ;  o = q^T kv.
 * q, k, v: inputs [B, H, d] of type dt; o: output [B, H, d] of type dt;
 * kv: [B, H, d, d] fp32, updated IN PLACE; all DEVICE pointers, kv 16-byte
 * aligned.  fp32 arithmetic whatever dt is.  Needs no workspace.
 */
int la_decode_step(const void *q, const void *k, const void *v,
                   const float *lambda /* host, [H] */,
                   float *kv, void *o,
                   int B, int H, int d, la_dtype dt, void *hip_stream);

/*
 * Gated, normalised output stage of the attention block (Sec. 4.2, "Gating
 * Mechanism" and "Tensor Normalization"), the step that follows la_fwd in the
 * paper's GLA:
 *     Y = SRMSNorm(O) * U ,   SRMSNorm(x) = x / sqrt(mean(x^2) + eps) ,
 * the mean running, per token, over all H*d features of O (the heads
 * concatenated); the paper's formula is eps = 0.  O, U: inputs, Y: output, all
 * [B, H, n, d] of type dt (DEVICE); fp32 arithmetic inside.  eps must be finite
 * and >= 0 (else LA_ERR_LAMBDA).  B <= 65535.  Needs no workspace.
 */
int la_gate_norm_fwd(const void *O, const void *U, void *Y, float eps,
                     int B, int H, int n, int d, la_dtype dt, void *hip_stream);

/*
 * Backward of la_gate_norm_fwd: with r = sqrt(mean(O^2) + eps), dN = dY * U:
 *     dU = dY * O / r ,   dO = dN / r - O * mean(dN * O) / r^3 .
 * O, U, dY: inputs; dO, dU: outputs; all [B, H, n, d] of type dt (DEVICE).
 * The dO written here is what la_bwd takes as its dO argument.
 */
int la_gate_norm_bwd(const void *O, const void *U, const void *dY, void *dO, void *dU, float eps,
                     int B, int H, int n, int d, la_dtype dt, void *hip_stream);

/*
 * Forward and backward with the activation of the query / key projections
 * fused in (Sec. 4.2, "Gating Mechanism": Q = phi(X W_q), K = phi(X W_k), phi =
 * Swish, read as phi(x) = x * sigmoid(x)).  Qp, Kp are the pre-activations:
 *     la_fwd_swish:  O = lightning_attention(phi(Qp), phi(Kp), V, lambda)
 *     la_bwd_swish:  with (dQ, dK, dV) the gradients la_bwd gives for Q = phi(Qp),
 *                    K = phi(Kp):  dQp = dQ * phi'(Qp),  dKp = dK * phi'(Kp),  dV.
 * phi is evaluated in fp32 while a tile is staged and rounded to dt before the
 * contractions (what they would see had phi(Qp), phi(Kp) been stored); phi',
 * in fp32, multiplies the result tile as it is stored.  Neither activated
 * tensor ever exists in memory.  Arguments, workspace and errors as la_fwd / la_bwd.
 */
int la_fwd_swish(const void *Qp, const void *Kp, const void *V,
                 const float *lambda /* host, [H] */,
                 void *O,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

int la_bwd_swish(const void *Qp, const void *Kp, const void *V,
                 const float *lambda /* host, [H] */,
                 const void *dO,
                 void *dQp, void *dKp, void *dV,
                 int B, int H, int n, int d, la_dtype dt,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Attention whose query / key feature is wider than its value feature, d_k = m d_v
 * (m = 1..4), as the cos / sin features of LRPE-d give (Sec. 4.1, "Position
 * Encoding": the phase factor exp(i theta (t-s)) of the score q_t^T k_s lambda^(t-s)
 * exp(i theta (t-s)) splits into a factor in t and a factor in s, so with
 * x~_t = [x_t cos(t theta), x_t sin(t theta)] its real part is the plain score
 * q~_t^T k~_s lambda^(t-s) over 2d features):
 *     O[t] = sum_{s <= t} lambda^(t-s) (Qw[t] . Kw[s]) V[s]
 * and its gradients.  Qw, Kw, dQw, dKw: [B, H, n, dk]; V, O, dO, dV: [B, H, n, dv];
 * dv is 64 or 128.  The scores add over the m slices of dv features, so the result
 * is accumulated over m scans of slices (the KV state is m states of dv x dv); O and
 * dV are read back and rounded to dt between slices.  Exception: la_fwd_wide in bf16 with
 * dk = 256, dv = 128 on a problem the planner does not cut into segments
 * (la_workspace_bytes(B, H, n, dv, dt, 0) == 0) runs ONE kernel that holds the whole
 * 256 x 128 state: one pass over Qw, Kw, V, no intermediate rounding of O.  Workspace as
 * la_fwd / la_bwd with d = dv.  The rotation itself (and theta's gradient) is the caller's.
 */
int la_fwd_wide(const void *Qw, const void *Kw, const void *V,
                const float *lambda /* host, [H] */,
                void *O,
                int B, int H, int n, int dk, int dv, la_dtype dt,
                void *workspace, size_t workspace_bytes, void *hip_stream);

int la_bwd_wide(const void *Qw, const void *Kw, const void *V,
                const float *lambda /* host, [H] */,
                const void *dO,
                void *dQw, void *dKw, void *dV,
                int B, int H, int n, int dk, int dv, la_dtype dt,
                void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * LRPE-d rotation (Sec. 4.1, "Position Encoding"; the decomposition of
 * exp(i theta (t - s)) over t and s): for row t (counted from 0) of every (batch, head),
 *     Xw[t] = [ X[t] * cos(t theta_h) , X[t] * sin(t theta_h) ]        ([B, H, n, 2d])
 * with theta a DEVICE pointer to [H, d] fp32 angles in radians (one per head and
 * feature; it is a learnable parameter of the model, so it lives on the device).
 * la_fwd_wide / la_bwd_wide on the rotated Q and K give LRPE-d's attention.
 * Backward:  dX[t] = dXw_c[t] cos(t theta) + dXw_s[t] sin(t theta)  and
 *     dtheta[h, i] (+)= sum_{b, t} t X[t, i] (dXw_s[t, i] cos(t theta_i) - dXw_c[t, i] sin(t theta_i)),
 * dtheta: DEVICE [H, d] fp32, overwritten, or added to when accumulate_dtheta != 0
 * (query and key share theta: rotate both, accumulate the second call).  The
 * reduction uses no atomics: `workspace` (DEVICE, 256-byte aligned, at least
 * la_lrpe_workspace_bytes(...) bytes, contents scratch) holds per-tile partial sums
 * that a second kernel adds in a fixed order.  B * H <= 65535.
 */
size_t la_lrpe_workspace_bytes(int B, int H, int n, int d);
int la_lrpe_rotate_fwd(const void *X, const float *theta /* device, [H, d] */, void *Xw,
                       int B, int H, int n, int d, la_dtype dt, void *hip_stream);
int la_lrpe_rotate_bwd(const void *X, const float *theta /* device, [H, d] */, const void *dXw,
                       void *dX, float *dtheta /* device, [H, d] */, int accumulate_dtheta,
                       void *workspace, size_t workspace_bytes,
                       int B, int H, int n, int d, la_dtype dt, void *hip_stream);

/*
 * la_fwd / la_bwd on tensors that are not contiguous [B, H, n, d]: the slab of
 * (batch b, head h) starts b * batch_stride + h * head_stride elements after the
 * pointer and its rows (d contiguous elements each) are row_stride elements apart.
 * Contiguous [B, H, n, d] is {H n d, n d, d}; the [B, n, H, d] a projection GEMM
 * writes is {n H d, d, H d}; Q, K, V packed as [B, n, 3, H, d] are three pointers d * H
 * elements apart with {3 n H d, d, 3 H d}.  This is the paper's own situation: its
 * layers produce Q, K, V as [B, n, H d] (Sec. 4.2, Q = phi(X W_q) ...) and the
 * attention runs per head.  Q, K, V share one layout; O (forward), dO, and dQ, dK, dV
 * (backward) have their own.  Strides are in elements, multiples of 8, row_stride
 * >= d (else LA_ERR_ALIGN / LA_ERR_SHAPE); outputs must not overlap anything.
 * Everything else as la_fwd / la_bwd: the same kernels with explicit strides, and the same
 * results bit for bit as la_fwd / la_bwd on contiguous copies of the tensors.
 */
typedef struct la_layout {
    long long batch_stride, head_stride, row_stride;
} la_layout;

int la_fwd_strided(const void *Q, const void *K, const void *V,
                   const float *lambda /* host, [H] */,
                   void *O,
                   const la_layout *qkv_layout, const la_layout *o_layout,
                   int B, int H, int n, int d, la_dtype dt,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

int la_bwd_strided(const void *Q, const void *K, const void *V,
                   const float *lambda /* host, [H] */,
                   const void *dO,
                   void *dQ, void *dK, void *dV,
                   const la_layout *qkv_layout, const la_layout *do_layout,
                   const la_layout *grad_layout,
                   int B, int H, int n, int d, la_dtype dt,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Static, human-readable text for an la_status value. */
const char *la_strerror(int status);

/*
 * Plan introspection (host arithmetic only): the tile length (the paper's
 * "block size B"), the segment length in tokens and the number of segments per
 * (batch, head) scan that la_fwd / la_bwd will use for this problem.  Any
 * output pointer may be NULL.  Returns an la_status.
 */
int la_plan(int B, int H, int n, int d, la_dtype dt,
            int *tile_len, int *segment_len, int *segments);

/*
 * Optional profiling hooks for benchmarks.  While enabled, every la_fwd /
 * la_bwd call brackets each launch of its block-scan kernel (the kernel that
 * runs the loops of Alg. 5 / Alg. 6) with HIP events on the call's stream.
 * la_profile_enable(1) creates the events (the only place where the library
 * creates anything; the forward / backward calls only record into them) and may
 * return LA_ERR_LAUNCH if that fails; la_profile_enable(0) stops recording.
 * la_profile_collect waits for the recorded events, adds up the elapsed times and
 * launch counts recorded since the last collect, and clears them.
 * Not thread-safe; meant for a single benchmarking thread.  At most
 * LA_PROFILE_MAX_LAUNCHES launches are recorded between collects; further
 * launches run normally but are not timed.
 */
#define LA_PROFILE_MAX_LAUNCHES 4096
int la_profile_enable(int on);
int la_profile_collect(double *scan_kernel_ms, int *scan_kernel_launches);

#ifdef __cplusplus
}
#endif
#endif /* LA_H */
