/*
 * linfusion.h -- C ABI of the MI355X (gfx950) LinFusion token mixer.
 *
 * The operation is the normalized, non-causal generalized linear attention that LinFusion
 * substitutes for self-attention (Sec. 2.3 normalization, Eq. 5; Sec. 2.4 non-causality,
 * Prop. 2 and Prop. 3: Y = f'(X) g'(X)^T X with rows normalised to sum to one).  Per
 * (batch b, head h), with Q, K, V in R^{N x d}, a non-negative elementwise feature map phi
 * applied to Q and K, and eps >= 0:
 *
 *     S     = sum_j phi(k_j)^T v_j          (d x d state, g'(X)^T X of Prop. 2)
 *     z     = sum_j phi(k_j)                (normalizer state, non-causal Z of Eq. 5)
 *     out_i = phi(q_i) S / (phi(q_i) . z + eps)
 *
 * (Sections of the paper are cited by position: 2.1 Preliminary, 2.2 Overview, 2.3 Normalization-Aware
 * Mamba, 2.4 Non-Causal Mamba, 2.5 Training Objectives, 3.1 Implementation Details, 3.2 Main Results,
 * 3.3 Empirical Extensions.)
 *
 * Every step (feature map, state reduction, combine, apply, normalize) runs in this
 * library's own HIP kernels.  There is no CPU fallback: on a machine without a gfx950
 * device every compute entry point returns LINFUSION_ERR_DEVICE.
 *
 * Conventions shared by all entry points
 *   - q, k, v, out: DEVICE pointers to contiguous [B, H, N, d] tensors, d fastest, all of the
 *     same element type; `out` has the element type of the inputs.  Base pointers must be
 *     16-byte aligned.  `out` must not overlap k or v; out == q (exact alias) is allowed.
 *     (linfusion_attn_fwd_strided takes other layouts, e.g. the token-major [B, N, H*d].)
 *   - The caller owns every buffer and keeps it alive until the work enqueued on `stream`
 *     has completed.  Calls are asynchronous: they enqueue on `stream` (a hipStream_t passed
 *     as void*; NULL = the default stream) and return without synchronising.
 *   - Results are run-to-run bit-identical for identical arguments (fixed-order reductions,
 *     no floating-point atomics).
 *   - Return value: LINFUSION_OK or a negative LINFUSION_ERR_* code.  All argument checks
 *     happen before anything is enqueued.  Nothing is printed, nothing aborts.
 *   - Supported head widths: d in {8, 16, 24, 32, 40, 48, 56, 64} for every dtype; for fp16 and bf16 also
 *     d = 80 and d = 160 (the deeper levels of the SD-v1.5 UNet: 640 and 1280 channels over 8 heads) and
 *     d = 96, 128.  Widths above 80 run on the three-kernel path only (LINFUSION_FLAG_FORCE_FUSED ->
 *     LINFUSION_ERR_UNSUPPORTED).
 *   - Arithmetic: every sum over tokens or channels is accumulated in fp32; the state is rescaled by a power of
 *     two before it becomes a 16-bit matrix-core operand.  Operands are rounded once to fp16 for fp16 tensors
 *     (relative 2^-12 each); carried as two bf16 levels (about 16 bits) for bf16 tensors, except in the apply
 *     kernel of the widths above 80, which multiplies bf16 tensors as fp16 operands after scaling every query
 *     row into fp16's range (the factor cancels in Eq. 5's ratio); fp32 tensors never pass through 16-bit
 *     products of fewer than 24 bits.  The result is rounded once, to nearest even, to the tensors' type.
 */
#ifndef LINFUSION_H_
#define LINFUSION_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of q, k, v, out */
#define LINFUSION_DTYPE_F32 0
#define LINFUSION_DTYPE_F16 1
#define LINFUSION_DTYPE_BF16 2

/* feature maps phi (Sec. 2.3: a non-negative activation on the key / query branches) */
#define LINFUSION_PHI_ELU_PLUS_ONE 0 /* x > 0 ? x + 1 : exp(x)   (default) */
#define LINFUSION_PHI_RELU 1         /* max(x, 0)                 (test aid) */
#define LINFUSION_PHI_IDENTITY 2     /* x; caller guarantees q, k >= 0 (test aid) */

/* flags for linfusion_attn_fwd_ex */
#define LINFUSION_FLAG_NONE 0u
#define LINFUSION_FLAG_UNNORMALIZED 1u /* out_i = phi(q_i) S, the un-normalized arm of Tab. 2 */
#define LINFUSION_FLAG_FORCE_SPLIT 2u  /* always take the three-kernel split-N path */
#define LINFUSION_FLAG_FORCE_FUSED 4u  /* take the single-launch path whenever the shape allows it */
#define LINFUSION_FLAG_FORCE_SOLO 8u   /* take the replicated-state launch whenever the shape allows it */

#define LINFUSION_OK 0
#define LINFUSION_ERR_INVALID (-1)     /* NULL pointer, B/H/N/d <= 0, eps < 0 or NaN, bad flags */
#define LINFUSION_ERR_UNSUPPORTED (-2) /* d, dtype or feature_map outside the supported sets */
#define LINFUSION_ERR_MISALIGNED (-3)  /* a tensor or workspace pointer is not 16-byte aligned */
#define LINFUSION_ERR_WORKSPACE (-4)   /* workspace_bytes below linfusion_attn_workspace_bytes() */
#define LINFUSION_ERR_HIP (-5)         /* a HIP runtime call or kernel launch failed */
#define LINFUSION_ERR_DEVICE (-6)      /* no HIP device, or the current device is not gfx950 */
#define LINFUSION_ERR_OVERLAP (-7)     /* an output overlaps an input it must not, another output, or the workspace */
#define LINFUSION_ERR_TIMEOUT (-8)     /* a single-launch call gave up waiting at its internal barrier */

/*
 * General entry point: the whole hot path (feature map -> split-N state reduction ->
 * deterministic combine -> apply + normalize) for one [B, H, N, d] problem.
 *
 * Three launch shapes compute it.  The replicated-state launch is one kernel without any exchange between
 * workgroups: every workgroup reduces the whole state of its head by itself and applies it to its share
 * of the queries; no workspace is touched, nothing can time out, and it may be captured into a HIP graph.
 * It is taken only when LINFUSION_FLAG_FORCE_SOLO asks for it (d <= 64): on MI355X the repeated reduction,
 * bound by one compute unit's vector rate, made it slower than three launches at every measured size
 * (36 against 22 us at 4096 tokens of 8 x 40 fp16; a tie below 256 tokens).
 * The split path enqueues three kernels (state reduction,
 * combine, apply).  The single-launch path runs the same three phases in one kernel whose
 * workgroups meet at two per-head barriers; it is chosen automatically where it measured
 * faster (16-bit heads of 56 or 64 channels with about 128 MB to 1 GB of tensor traffic, where
 * draining and refilling the chip between kernels costs a visible share), can be forced or
 * forbidden with the flags, and is used only
 * when all of its workgroups are resident at once (otherwise the call falls back to the split
 * path).  Its barrier waits are bounded: if a wait ever expires (which needs another workload
 * to hold the device's compute units for seconds) the kernel ends early, `out` is incomplete,
 * and linfusion_attn_last_error reports LINFUSION_ERR_TIMEOUT.
 *
 *   dtype            LINFUSION_DTYPE_*; accumulation is fp32 for every dtype.
 *   feature_map      LINFUSION_PHI_*.
 *   eps              added once to the denominator phi(q_i).z, after the dot product.
 *   flags            LINFUSION_FLAG_* (bitwise or).
 *   workspace        DEVICE scratch of at least linfusion_attn_workspace_bytes(...) bytes,
 *                    16-byte aligned, owned by the caller, contents undefined before and after.
 *                    Calls that share a workspace must be ordered on one stream.
 *   stream           hipStream_t (NULL = default stream).
 *
 * Never allocates, never synchronises; may be recorded into a HIP graph (while `stream` is being
 * captured the split path is taken whatever the flags say: the single launch's barrier tickets are
 * per call and must not be replayed).
 */
int linfusion_attn_fwd_ex(const void* q, const void* k, const void* v, void* out,
                          int B, int H, long long N, int d,
                          int dtype, int feature_map, float eps, unsigned flags,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * linfusion_attn_fwd_ex on tensors that are views into larger buffers, so that the layer around
 * the mixer needs no permute or copy: the UNet's token-major activations [B, N, H*d] (Sec. 2.2, Overview:
 * the module replaces self-attention inside each transformer block, whose q/k/v projections emit
 * that layout), or q, k, v sliced out of one fused projection output.
 *
 * Each *_strides array holds HOST values, in ELEMENTS: {batch stride, head stride, token stride}.
 * The d channels of one token of one head are always contiguous.  q has its own strides, k and v
 * share one set, out has its own.  Examples for element (b, h, n, c):
 *     contiguous [B, H, N, d]  : {H*N*d, N*d, d}
 *     token-major [B, N, H*d]  : {N*H*d, d, H*d}
 *     k, v inside [B, N, 2, H, d] : {N*2*H*d, d, 2*H*d} with k = base, v = base + H*d
 * A NULL array means contiguous [B, H, N, d].
 *
 * Requirements: every stride is >= 0 and a multiple of 16 bytes (8 elements for the 16-bit types,
 * 4 for fp32), so that with 16-byte aligned base pointers every token row is 16-byte aligned;
 * token stride below 2^24 * 16 bytes (else LINFUSION_ERR_INVALID).  Input strides may be 0 (one
 * k, v shared by all heads, say).  The rows of `out` must not overlap one another
 * (LINFUSION_ERR_OVERLAP).  Overlap between tensors is judged on the byte range each view spans from
 * its first to its last element: the range of `out` must be disjoint from those of k and v and
 * from that of q, except that out == q with identical strides (in place) is allowed.
 * Everything else is as for linfusion_attn_fwd_ex (same workspace size, same two launch paths).
 * Speed: 16-bit tensors whose heads are neighbours in memory (head stride == d) and whose head rows are
 * not whole 128-byte lines (d = 40, say) are moved in groups of 4 or 8 heads as whole contiguous row
 * pieces once the problem is large enough for that to pay (about 24 MB of tensor traffic); they then
 * run as fast as the contiguous layout.  Results there may differ from the contiguous call's in the
 * last bits (another summation order); they stay run-to-run identical.
 */
int linfusion_attn_fwd_strided(const void* q, const void* k, const void* v, void* out,
                               int B, int H, long long N, int d,
                               int dtype, int feature_map, float eps, unsigned flags,
                               const long long q_strides[3], const long long kv_strides[3],
                               const long long out_strides[3],
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Benchmark aid: linfusion_attn_fwd_strided that also records four caller-created hipEvent_t
 * (passed as void*) on `stream`: events[0] before the state reduction, [1] after it, [2] after
 * the combine (and the packing of the states into apply operands, where the row-piece kernels run),
 * [3] after apply, so a harness can time each kernel of one call.  The stride
 * arrays may be NULL (contiguous).
 */
int linfusion_attn_fwd_profile(const void* q, const void* k, const void* v, void* out,
                               int B, int H, long long N, int d,
                               int dtype, int feature_map, float eps, unsigned flags,
                               const long long q_strides[3], const long long kv_strides[3],
                               const long long out_strides[3],
                               void* workspace, size_t workspace_bytes, void* stream,
                               void* events[4]);

/*
 * Backward pass of the mixer: gradients of a scalar loss with respect to q, k and v, given
 * dout = d loss / d out.  (Training by distillation, Sec. 2.5 (Training Objectives), Eq. 8, differentiates through every
 * LinFusion module; the paper gives no formula, so the operation is defined as the derivative of the
 * forward definition above.)  With P = phi(K), R = phi(Q), S = P^T V, z = P^T 1, den_i = r_i . z + eps:
 *
 *     u_i = S dout_i ,  go_i = (r_i . u_i) / den_i            (= dout_i . out_i)
 *     dq_i = ((u_i - go_i z) / den_i) * phi'(q_i)
 *     dS = sum_i r_i^T (dout_i / den_i) ,  dz = -sum_i r_i go_i / den_i
 *     dk_j = (dS v_j + dz) * phi'(k_j) ,   dv_j = dS^T p_j
 *
 * (LINFUSION_FLAG_UNNORMALIZED: den = 1, go = 0.)  phi' at 0 is the one-sided value 1 for elu+1 and 0
 * for relu.  The forward output is not an input: dout . out is recomputed in fp32.
 *
 *   state           NULL, or a DEVICE pointer to the fp32 forward state of these q, k, v ([B*H][d*d + d]: S
 *                   row-major then z, as linfusion_attn_state writes it and as a forward call leaves it in
 *                   its workspace at linfusion_attn_workspace_state_offset(...)): saves the pass over k, v.
 *                   16-byte aligned; must not overlap dq, dk, dv or `workspace`.
 *   q, k, v, dout   DEVICE pointers, contiguous [B, H, N, d].  fp16, bf16: d in {8, ..., 64 step 8, 80}; fp16 also
 *                   d in {96, 128, 160} (bf16 there -> LINFUSION_ERR_UNSUPPORTED); fp32: d in {8, ..., 64 step 8}.
 *                   fp16 above 80 and fp32 run a pass composed of the forward's kernels with three temporaries of
 *                   the tensors' type in the workspace, sixteen launches: there so that every level of the UNet
 *                   and every type has a gradient, not for speed.
 *   dq, dk, dv      DEVICE pointers, same shape and type; must not overlap any input or each other.
 *   flags           LINFUSION_FLAG_NONE or LINFUSION_FLAG_UNNORMALIZED (anything else -> ERR_INVALID).
 *   workspace       DEVICE scratch of at least linfusion_attn_bwd_workspace_bytes(...) bytes, 16-byte
 *                   aligned, caller-owned, contents undefined before and after.
 * Enqueues six kernels (four when `state` is given) on `stream`; never allocates, never synchronises.  Results are run-to-run identical.
 */
int linfusion_attn_bwd(const void* q, const void* k, const void* v, const void* dout, const float* state,
                       void* dq, void* dk, void* dv,
                       int B, int H, long long N, int d,
                       int dtype, int feature_map, float eps, unsigned flags,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * linfusion_attn_bwd on strided views: q; k and v (one layout); dout; dq; dk and dv (one layout) are each
 * addressed by element strides {batch, head, token} with contiguous channels, as in
 * linfusion_attn_fwd_strided (a NULL stride array = contiguous [B, H, N, d]).  Rows must be 16-byte aligned;
 * dq and dk / dv rows must be disjoint, and the byte span of every output must be disjoint from the spans of
 * the inputs, of the other outputs and of the workspace (so three gradients interleaved in one buffer are not
 * accepted).  Same arithmetic and order as the contiguous call: dense strides give bit-identical results.
 * Speed: where the heads of a token are neighbours in memory (head stride == d, the UNet's [B, N, H*d]), a head's
 * row is no whole number of 128-byte lines (d * 2 % 128 != 0: d = 40, 80, ...), H is a multiple of 4 and a tensor
 * has 24 MB or more, the gradients come from kernels that move whole row pieces of four or eight neighbouring
 * heads: the forward state (when not handed in), dQ, dK and dV for every width up to 56 and 80, the state gradient
 * too for fp16 up to d = 48 (token-major 8 x 40 at 2 M tokens: fp16 2.2 ms, against 7.0 ms on the per-head kernels
 * and 2.3 ms contiguous; bf16 3.5 against 8.2 and 3.2 ms).  These kernels sum the state and its gradient over the tiles in another order
 * than the per-head kernels, so the gradients may differ from the contiguous call's in the last bit; they stay
 * run-to-run identical.  Head counts that are no multiple of 4 run the per-head kernels on partial lines, at a
 * fraction of the contiguous speed; d = 64 token-major does not suffer.
 */
int linfusion_attn_bwd_strided(const void* q, const void* k, const void* v, const void* dout, const float* state,
                               void* dq, void* dk, void* dv,
                               int B, int H, long long N, int d,
                               int dtype, int feature_map, float eps, unsigned flags,
                               const long long q_strides[3], const long long kv_strides[3],
                               const long long dout_strides[3], const long long dq_strides[3],
                               const long long dkv_strides[3],
                               void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of device scratch linfusion_attn_bwd needs; pure host function; 0 for rejected arguments. */
size_t linfusion_attn_bwd_workspace_bytes(int B, int H, long long N, int d, int dtype);

/*
 * The mixer fed directly by the two-branch MLPs f' and g' that produce its queries and keys (Sec. 3.1 (Implementation Details),
 * implementation details: a linear branch, started from the softmax layer's W_Q / W_K, plus one
 * Linear-LayerNorm-LeakyReLU block, started at zero, the two results added; Prop. 2 names the functions):
 *
 *     q_i = a_q,i + LeakyReLU(gamma_q * (t_q,i - mean_i) / sqrt(var_i + ln_eps) + beta_q)      (k likewise)
 *     out = mixer(q, k, v)                          as linfusion_attn_fwd_ex, per head, Eq. 5 / Prop. 2
 *
 * a_* is the result of the linear branch and t_* the result of the second branch's Linear for the same
 * tokens (both GEMMs are the caller's); mean_i and var_i (mean squared deviation) run over all C = H*d
 * channels of token i.  q and k are formed inside the state-reduction and apply kernels and never exist in
 * memory: where one workgroup can hold whole token rows (H = 8 with d <= 48, H = 4 with d <= 64 or 80) the
 * call reads five tensors and writes one; for every other shape a pass over t_q and t_k first leaves the
 * rows' LayerNorm statistics (8 bytes per token and branch) in the workspace, two tensor reads more, and the
 * reduction and apply kernels work on groups of four heads, on single heads, or (d > 80) on the wide kernels.
 *
 *   a_q, t_q, a_k, t_k, v   DEVICE pointers, token-major contiguous [B, N, H*d] (head h owns channels
 *                           h*d .. h*d+d-1 of a token), fp16 or bf16, 16-byte aligned.
 *   out                     DEVICE pointer, same layout and type; must not overlap any input.
 *   gamma_*, beta_*         DEVICE pointers to H*d fp32 values each (the LayerNorms' affine).
 *   H, d                    any H >= 1 with B*H <= 65535 and B <= 32767; d in {8, ..., 64 step 8, 80, 96, 128, 160};
 *                           LINFUSION_DTYPE_F32 and every other width -> LINFUSION_ERR_UNSUPPORTED.
 *   eps                     as linfusion_attn_fwd_ex.  ln_eps > 0 (finite), 0 <= slope <= 1: the LayerNorm's
 *                           epsilon (inside the square root) and the LeakyReLU's negative slope; the paper
 *                           names neither, the common defaults are 1e-5 and 0.01.
 *   flags                   LINFUSION_FLAG_NONE or LINFUSION_FLAG_UNNORMALIZED (anything else -> ERR_INVALID).
 *   workspace               DEVICE scratch of at least linfusion_attn_mlp_workspace_bytes(...) bytes,
 *                           16-byte aligned, caller-owned, contents undefined before and after.
 *   events                  NULL, or four hipEvent_t created by the caller (passed as void*), recorded on
 *                           `stream` before the first kernel, after the state reduction, after combine +
 *                           operand packing, and after apply.
 * Enqueues four kernels (five with the statistics pass) on `stream`; never allocates, never synchronises; run-to-run identical results.
 * Errors as linfusion_attn_fwd_ex (first failing check wins; nothing is enqueued on an error).
 */
int linfusion_attn_fwd_mlp(const void* a_q, const void* t_q, const void* a_k, const void* t_k, const void* v,
                           void* out,
                           const float* gamma_q, const float* beta_q, const float* gamma_k, const float* beta_k,
                           int B, int H, long long N, int d,
                           int dtype, int feature_map, float eps, float ln_eps, float slope, unsigned flags,
                           void* workspace, size_t workspace_bytes, void* stream, void* events[4]);

/*
 * linfusion_attn_fwd_mlp on strided token rows (Sec. 3.1 (Implementation Details): the five branch results are usually column blocks of
 * one projection's output, [B, N, 5 C] say, and need no copy to become dense).
 *   in_strides      HOST array {batch, token}: element strides shared by a_q, t_q, a_k, t_k and v, whose
 *                   [b][n] row is C = H * d contiguous elements at base + b * batch + n * token.
 *   out_strides     HOST array {batch, token} of out; rows must not intersect (token >= C, batch >=
 *                   (N - 1) * token + C, else LINFUSION_ERR_OVERLAP).
 * Strides are multiples of 8 elements (16 bytes; else LINFUSION_ERR_MISALIGNED), non-negative, token >= C for
 * the inputs, token < 2^27 and the spanned extent below 2^45 elements (else LINFUSION_ERR_INVALID).  The inputs
 * may interleave in one buffer; the extent out spans must not overlap the extent any input spans.  Either
 * array NULL = dense [B, N, C].  Everything else, the workspace size included, as linfusion_attn_fwd_mlp, whose
 * results this call reproduces bit for bit on the same values.
 */
int linfusion_attn_fwd_mlp_strided(const void* a_q, const void* t_q, const void* a_k, const void* t_k, const void* v,
                                   void* out,
                                   const float* gamma_q, const float* beta_q, const float* gamma_k,
                                   const float* beta_k,
                                   int B, int H, long long N, int d,
                                   int dtype, int feature_map, float eps, float ln_eps, float slope, unsigned flags,
                                   const long long in_strides[2], const long long out_strides[2],
                                   void* workspace, size_t workspace_bytes, void* stream, void* events[4]);

/* Bytes of device scratch linfusion_attn_fwd_mlp needs; pure host function; 0 for rejected arguments. */
size_t linfusion_attn_mlp_workspace_bytes(int B, int H, long long N, int d, int dtype);

/*
 * The mixer with a feature width d_qk of q and k different from the value width d_v (Prop. 3: with
 * vector-valued attention weights f' and g' map to d' * r channels while the values keep theirs; the
 * computational form is that of Prop. 2 with a d_qk x d_v state):
 *
 *     S = sum_j phi(k_j)^T v_j  (d_qk x d_v),  z = sum_j phi(k_j)  (d_qk),
 *     out_i = phi(q_i) S / (phi(q_i) . z + eps)                      (d_v)
 *
 *   q, k            DEVICE pointers, contiguous [B, H, N, d_qk]; v, out: contiguous [B, H, N, d_v]; fp16 or
 *                   bf16 (LINFUSION_DTYPE_F32 -> LINFUSION_ERR_UNSUPPORTED); 16-byte aligned; out must not
 *                   overlap an input.
 *   d_qk, d_v       d_v in {40, 64}, d_qk in {16, 32, 40, 64, 80}, d_qk != d_v (equal widths are
 *                   linfusion_attn_fwd_ex's); anything else -> LINFUSION_ERR_UNSUPPORTED.
 *   flags           LINFUSION_FLAG_NONE or LINFUSION_FLAG_UNNORMALIZED (anything else -> ERR_INVALID).
 *   workspace       DEVICE scratch of at least linfusion_attn_qv_workspace_bytes(...) bytes, 16-byte
 *                   aligned, caller-owned, contents undefined before and after.
 *   events          NULL, or four hipEvent_t created by the caller (passed as void*), recorded on `stream`
 *                   before the state reduction, after it, after the combine, and after apply.
 * Enqueues three kernels on `stream`; never allocates, never synchronises; run-to-run identical results.
 */
int linfusion_attn_fwd_qv(const void* q, const void* k, const void* v, void* out,
                          int B, int H, long long N, int d_qk, int d_v,
                          int dtype, int feature_map, float eps, unsigned flags,
                          void* workspace, size_t workspace_bytes, void* stream, void* events[4]);

/* Bytes of device scratch linfusion_attn_fwd_qv needs; pure host function; 0 for rejected arguments. */
size_t linfusion_attn_qv_workspace_bytes(int B, int H, long long N, int d_qk, int d_v, int dtype);

/*
 * Synchronises `stream` and reports whether the most recent single-launch call that used this
 * workspace for this shape completed: LINFUSION_OK, LINFUSION_ERR_TIMEOUT, or an argument / HIP
 * error code.  The answer is read from records the single-launch kernels keep inside the workspace
 * itself, so calls on other workspaces, streams or threads do not disturb it.  (The split path
 * cannot time out and leaves the records alone; a workspace no single-launch call has used
 * reports LINFUSION_OK.)
 */
int linfusion_attn_last_error(const void* workspace, size_t workspace_bytes,
                              int B, int H, long long N, int d, int dtype, void* stream);

/*
 * Byte offset, inside the workspace of linfusion_attn_fwd_ex / _fwd_strided, at which a completed forward
 * call of this shape has left the head states ([B*H][d*d + d] fp32, S row-major then z).  A later call
 * with the same workspace overwrites them.  Pure host function; 0 for rejected arguments.
 */
size_t linfusion_attn_workspace_state_offset(int B, int H, long long N, int d, int dtype);

/*
 * Bytes of device scratch linfusion_attn_fwd_ex needs for this shape; 0 for arguments the forward
 * call would reject.  Host function of its arguments and of the current device's compute-unit count
 * (launch sizes follow it; 256, one whole MI355X, is assumed while no device is visible).  No
 * environment variable enters unless tuning has been switched on (linfusion_set_tuning).
 */
size_t linfusion_attn_workspace_bytes(int B, int H, long long N, int d, int dtype);

/*
 * Convenience entry points with the signature of the method's token mixer
 * (q, k, v -> out for phi, eps).  Element type: fp16 for linfusion_attn_fwd and _f16, bf16 for
 * _bf16, fp32 for _f32.  They use a library-owned scratch buffer per device that is allocated
 * with hipMalloc on first use (and re-allocated when a later call needs more), so the first
 * call per device -- and any call that grows the buffer -- synchronises that device.  Calls
 * on one device must be issued from one thread at a time and ordered on one stream.  They always
 * take the three-kernel path, which cannot time out (the caller has no workspace to ask
 * linfusion_attn_last_error about).
 */
int linfusion_attn_fwd(const void* q, const void* k, const void* v, void* out,
                       int B, int H, long long N, int d, int feature_map, float eps, void* stream);
int linfusion_attn_fwd_f16(const void* q, const void* k, const void* v, void* out,
                           int B, int H, long long N, int d, int feature_map, float eps, void* stream);
int linfusion_attn_fwd_bf16(const void* q, const void* k, const void* v, void* out,
                            int B, int H, long long N, int d, int feature_map, float eps, void* stream);
int linfusion_attn_fwd_f32(const void* q, const void* k, const void* v, void* out,
                           int B, int H, long long N, int d, int feature_map, float eps, void* stream);

/*
 * linfusion_attn_fwd_ex for callers that cannot allocate and have no workspace to hand over: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch the kernels need (the
 * partial states of the split-N reduction, the combined states, the apply operands of the row-piece kernels)
 * lives in a fixed array inside the library's device image, linfusion_attn_static_scratch_bytes() = 16 MiB per
 * device, held until the process ends.  The call allocates nothing, frees nothing and synchronises nothing.
 *
 *   q, k, v, out, B, H, N, d, dtype, feature_map, eps, stream: as linfusion_attn_fwd_ex (contiguous [B, H, N, d]).
 *   flags        LINFUSION_FLAG_NONE or LINFUSION_FLAG_UNNORMALIZED; the three-kernel path always runs
 *                (LINFUSION_FLAG_FORCE_FUSED -> LINFUSION_ERR_INVALID), so results equal those of
 *                linfusion_attn_fwd_ex with LINFUSION_FLAG_FORCE_SPLIT bit for bit.
 * Shapes whose three-kernel scratch exceeds the array are rejected with LINFUSION_ERR_WORKSPACE before anything
 * is enqueued (the need is that of the three-kernel path alone, well below linfusion_attn_workspace_bytes, which
 * also covers the single launch).  On a whole MI355X: widths up to 64 fit for B*H up to a few hundred, d = 80
 * for B*H up to about 64; the wide widths (96, 128, 160) exceed it for all but tiny shapes -- for those use
 * linfusion_attn_fwd_ex.  Every call on a device uses that device's one array: calls on one device
 * must be ordered on one stream (or otherwise not overlap in time); overlapping calls race on the scratch.
 * Nothing in the array has to start at zero -- every word a kernel reads was written earlier in the same call
 * -- so contents left by an earlier call, of whatever shape, are harmless.
 * linfusion_init (optional) resolves the array's device address for the current device ahead of time, so that
 * the first linfusion_attn_fwd_static call does not; it allocates nothing either.
 */
int linfusion_attn_fwd_static(const void* q, const void* k, const void* v, void* out,
                              int B, int H, long long N, int d,
                              int dtype, int feature_map, float eps, unsigned flags, void* stream);
size_t linfusion_attn_static_scratch_bytes(void);
int linfusion_init(void);

/*
 * State-only entry point (the reduction half of Prop. 2; also what an N-sharded deployment
 * exchanges between devices, Sec. 3.3 (Empirical Extensions, distributed parallel inference: "constant communication cost")): writes, per (b, h),
 * the fp32 state S as [d][d] row-major (row = feature index of phi(K), column = value
 * channel) followed by z as [d], i.e. state_out is a DEVICE buffer of B*H*(d*d+d) floats.
 * Same workspace contract as linfusion_attn_fwd_ex.
 */
int linfusion_attn_state(const void* k, const void* v, float* state_out,
                         int B, int H, long long N, int d, int dtype, int feature_map,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Frees the library-owned scratch buffers (synchronises).  Optional; safe to call twice. */
void linfusion_release(void);

/* Static string for a status code. */
const char* linfusion_status_string(int status);

/* major * 10000 + minor * 100 + patch */
int linfusion_version(void);

/*
 * Measurement aids (no arithmetic of the method): what plain streaming and plain launching reach on the
 * device, for the roofline figures of the benchmark to be compared with.
 *
 * linfusion_hbm_probe enqueues one kernel that reads `reads` (0..3) streams a, b, c and writes `writes` (0 or 1)
 * stream d of `bytes` bytes each (a multiple of 16), every byte once, with 256-thread workgroups, 128-bit
 * non-temporal accesses and `workgroups` workgroups that sweep the streams in one moving window -- the access
 * pattern of the state reduction (reads = 2, writes = 0) and of apply (reads = 1, writes = 1).  With reads > 0
 * the written (or, with writes = 0, discarded) value is the xor of the streams read.  All pointers DEVICE,
 * 16-byte aligned; unused ones may be NULL; `sink`: DEVICE pointer to two 32-bit words (required when
 * writes = 0).
 * linfusion_launch_probe enqueues `launches` (1..1024) kernels of `workgroups` x 256 threads that do nothing,
 * back to back on `stream`: the cost of a dependent chain of launches by itself.
 * Both return LINFUSION_OK or LINFUSION_ERR_INVALID / _MISALIGNED / _DEVICE / _HIP; never allocate or synchronise.
 */
int linfusion_hbm_probe(int reads, int writes, const void* a, const void* b, const void* c, void* d,
                        size_t bytes, int workgroups, unsigned* sink, void* stream);
int linfusion_launch_probe(int launches, int workgroups, unsigned* sink, void* stream);

/*
 * Development switch.  The LINFUSION_* environment variables (launch shapes, forced kernel routes, the
 * single launch's poll limit: aids for sweeps and tests) are consulted only while tuning is on; it is
 * off unless LINFUSION_TUNE=1 was in the environment when the library was first used or this function
 * switched it on.  With tuning off no call reads the environment and launch plans and workspace sizes
 * depend on the shape and the device alone.
 */
void linfusion_set_tuning(int on);

/*
 * Introspection for benchmarks and tests (host only, no device work): the launch plan the
 * forward call will use for this shape.  plan[0] = path (0 = split-N three-kernel path,
 * 1 = single launch with barriers, 2 = replicated-state launch), plan[1] = state-reduction workgroups per
 * head, plan[2] = apply workgroups per head (on the single-launch paths both are its workgroups per head),
 * plan[3] = tokens per tile.  Returns LINFUSION_OK or an error code.
 */
int linfusion_attn_plan(int B, int H, long long N, int d, int dtype, unsigned flags, int plan[4]);

/*
 * Name of the kernel that will run the apply step for this shape on contiguous tensors ("apply16_dma",
 * "apply16_packed", "apply32", "apply16_wide", "apply16_wave", or "fused16" / "fused32" / "solo16" / "solo32" when a single
 * launch is chosen);
 * an empty string for rejected arguments.  Static storage.  For benchmarks and profile summaries.
 */
const char* linfusion_attn_apply_kernel(int B, int H, long long N, int d, int dtype, unsigned flags);

#ifdef __cplusplus
}
#endif
#endif /* LINFUSION_H_ */
