/*
 * lory.h - C ABI of the MI355X (gfx950) Lory causal-segment expert-merging
 * MoE FFN layer.
 *
 * The layer (paper Section 3.1, Eq. 2 and Algorithm 1; merged FFN of
 * Section 2.2, Eq. 1; SwiGLU experts per Section 4.1):
 *   a sequence of L tokens is cut into N = L/T segments of T tokens; the
 *   routing weights of segment k are softmax(R(mean hidden state of segment
 *   k-1)), the first segment routes on its own mean; the E SwiGLU experts are
 *   merged in parameter space with those weights; the merged FFN is applied
 *   to every token of the segment.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers on the current HIP device,
 *     row-major contiguous (last index fastest), 16-byte aligned.
 *   - The caller owns every buffer, including the workspace; the library
 *     never allocates, frees or keeps a pointer past the call.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only
 *     enqueue work on that stream and return; no implicit synchronisation.
 *   - Return value is a lory_status; nothing throws or aborts.  All argument
 *     checks happen before the first launch; on any error return no output
 *     buffer has been written.
 *   - `dtype` names the storage type of X, R, the expert stacks, Y, dY, dX
 *     and the saved activations: LORY_F32 (fp32 arithmetic throughout) or
 *     LORY_BF16 (bf16 operands, fp32 accumulation on the matrix cores).
 *     Routing weights w / dw and hbar are always fp32.
 *   - Host-side state (the slab budget, the optional event timing, one-time
 *     kernel attribute set-up) is process-global and unsynchronised: calls
 *     into the library from several host threads must be serialised by the
 *     caller.  Workspace sizes depend on the slab budget in force when
 *     lory_workspace_bytes is called; keep it unchanged until the call that
 *     uses the workspace has returned.
 *   - Shape rules: every dimension > 0, L % T == 0 (the paper's listing uses
 *     N = L // T with a reshape, so a ragged tail has no defined meaning),
 *     E <= 64.  LORY_BF16 additionally needs d % 64 == 0, d_ff % 64 == 0 and
 *     T % 64 == 0 (MFMA tile granularity).
 */
#ifndef LORY_H
#define LORY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LORY_OK = 0,
    LORY_ERR_NULL = 1,      /* a required pointer is NULL */
    LORY_ERR_SHAPE = 2,     /* a dimension is <= 0, L % T != 0, or a granularity rule is violated */
    LORY_ERR_DTYPE = 3,     /* unknown dtype value */
    LORY_ERR_ALIGN = 4,     /* a pointer is not 16-byte aligned */
    LORY_ERR_WORKSPACE = 5, /* workspace_bytes is smaller than lory_workspace_bytes() reports */
    LORY_ERR_DEVICE = 6     /* a HIP call or kernel launch failed */
} lory_status;

typedef enum { LORY_F32 = 0, LORY_BF16 = 1 } lory_dtype;

typedef enum { LORY_PASS_FWD = 0, LORY_PASS_BWD = 1, LORY_PASS_DENSE = 2 } lory_pass;

/* Problem statement of Algorithm 1: x is B x L x d, E experts, segment
 * length T; d_ff is the FFN width (the paper's d'). */
typedef struct {
    int32_t B, L, T, d, d_ff, E;
    int32_t dtype; /* lory_dtype */
} lory_shape;

/* Static string for a status code (never NULL). */
const char *lory_status_string(int status);

/* Library version, "major.minor". */
const char *lory_version(void);

/*
 * Tuning knob (process-global, host-only): upper bound in bytes for the
 * transient slab through which merged parameters and per-segment weight
 * gradients pass (Eq. 2's theta_bar is produced and consumed block by block).
 * Default 6 GiB: on MI355X large blocks (few, long launches that fill all 256
 * CUs) measured faster than blocks sized for the 256 MB memory-side cache; the
 * LORY_SLAB_MB environment variable sets the initial value.  Changes what
 * lory_workspace_bytes reports, so set it before sizing a workspace.
 * Returns LORY_ERR_SHAPE for values below 64 KiB.
 */
int lory_set_slab_budget(size_t bytes);

/*
 * Tuning knob (process-global, host-only): which LORY_BF16 shapes run their
 * token contractions with the merge INSIDE the GEMM (Eq. 2's theta_bar formed
 * tile by tile on chip and consumed there: no merged parameter reaches HBM, in
 * the forward or in the backward's re-merge) instead of the slab pipeline.
 *   0  never
 *   1  where it measured faster (default): T <= 64 and E <= 16, shape fitting
 *      the kernel.  The fused kernel is bound by the L2 -> CU path at about the
 *      same rate for every segment length, while the slab pipeline's HBM
 *      traffic grows with the number of segments
 *   2  wherever the shape fits the kernel: T in {64, 128, 256}, E <= 32,
 *      B*L a multiple of 1024 (512 for T <= 128), no Wbar_save given
 *   3  as 2, and the backward also keeps the per-segment weight gradients on
 *      chip (expert gradients and routing-weight inner products accumulated by
 *      the kernel that forms X_s^T dG_s; no gradient slab in HBM) where that
 *      kernel takes the shape: E <= 16, T a multiple of 64, B*L/T a multiple of
 *      8, bf16 gradients that overwrite (other calls use the slab pipeline for
 *      this stage).  Measured slower than the slab pipeline at every shape tried;
 *      it exists to be measured
 * The LORY_FUSED environment variable sets the initial value.  Changes what
 * lory_workspace_bytes reports (forward pass), so set it before sizing a
 * workspace.  Returns LORY_ERR_SHAPE for other values.
 */
int lory_set_fused_merge(int mode);

/*
 * Optional timing of the hot path's kernels, by class, with HIP events on the
 * caller's stream (the measurement model is the paper's Appendix B: GEMM work
 * 6*tokens*d*d_ff per pass direction, merge-class work 6*E*d*d_ff per segment
 * and pass).  lory_profile_enable(1) makes every later launch record a pair
 * of events tagged with that launch's algorithmic FLOPs and bytes;
 * lory_profile_read waits for the recorded events, sums them per class into
 * out[0..*n_out) (at most max_out entries; classes without launches are
 * skipped) and clears the records.  Host-side state is process-global and not
 * thread-safe.  The event objects (4096, i.e. 2048 timed launches between two
 * reads; further launches go untimed) are created by lory_profile_enable(1),
 * never inside a launch, and reused.
 */
typedef struct {
    char name[32];   /* kernel class, e.g. "gemm_gate_up", "merge", "scatter_dots" */
    int32_t launches;
    double ms;       /* summed event time of the launches */
    double flops;    /* summed algorithmic floating-point operations */
    double bytes;    /* summed algorithmic HBM bytes (reads + writes) */
} lory_kernel_stat;
int lory_profile_enable(int on);
int lory_profile_read(lory_kernel_stat *out, int max_out, int *n_out);

/*
 * Bytes of device workspace that lory_merged_ffn_fwd (pass = LORY_PASS_FWD),
 * lory_merged_ffn_bwd (pass = LORY_PASS_BWD) or lory_dense_ffn_fwd (pass =
 * LORY_PASS_DENSE, shape as that call takes it) needs for this shape.  The
 * workspace holds only transient data (merged-weight slabs, per-segment
 * weight-gradient slabs, activations between the two projections, partial
 * router-weight gradients); its contents are undefined before and after a
 * call.  Host-only: touches no device.
 */
int lory_workspace_bytes(const lory_shape *shape, int pass, size_t *bytes_out);

/*
 * Bytes of the optional "merged parameters saved for the backward" buffer
 * (Wbar_save of lory_merged_ffn_fwd / lory_merged_ffn_bwd): 3 * S * d * d_ff
 * elements of dtype, or 0 when this shape does not support it (LORY_F32, or
 * more segments than one merge launch handles: S > 256, or S > 128 when
 * E > 32).  The paper's own implementation keeps the merged FFN parameters of
 * every segment in memory (Appendix G.2 mentions the cost); here that is an
 * opt-in trade of memory for one re-merge of the expert stack.  Host-only.
 */
int lory_merged_save_bytes(const lory_shape *shape, size_t *bytes_out);

/*
 * Causal segment routing (Section 3.1, Eq. 2; Algorithm 1).
 *   hbar[b,k,:] = (1/T) sum of X[b, kT .. kT+T-1, :]
 *   e[b,k,:]    = softmax(hbar[b,k,:] . R)        (no bias, temperature 1)
 *   w[b,0,:]    = e[b,0,:]       (the first segment routes on itself)
 *   w[b,k,:]    = e[b,k-1,:]     for 1 <= k < N   (shift by one segment)
 * in:  X [B, L, d] (dtype), R [d, E] (dtype)
 * out: w [B*N, E] fp32, rows sum to 1; hbar_opt [B*N, d] fp32 or NULL.
 * The stop gradient on the first segment only matters for the router
 * backward (lory_route_bwd).  Mean, logits and softmax
 * are computed in fp32 for both dtypes.  Needs no workspace.
 */
int lory_route(const lory_shape *shape, const void *X, const void *R,
               float *w, float *hbar_opt, void *stream);

/*
 * Router backward: the chain rule through lory_route (Section 3.1, Eq. 2),
 * with the stop gradient Algorithm 1 puts on the first segment's own routing
 * weights.  With e[b,j] = softmax(hbar[b,j] R) (read back as w[b,j+1]):
 *   de[b,j] = dw[b,j+1] for j < N-1, and 0 for the last segment of a sequence
 *             (dw[b,0] is not used: w[b,0] is a stopped copy of e[b,0])
 *   dz[b,j] = e[b,j] * (de[b,j] - <e[b,j], de[b,j]>)
 *   dR      = sum over all segments of hbar[b,j]^T dz[b,j]
 *   dX[b, jT+t, :] += (dz[b,j] R^T) / T          for every token t of segment j
 * in:     R [d, E] (dtype); w [B*N, E] and hbar [B*N, d] fp32 exactly as
 *         lory_route wrote them; dw [B*N, E] fp32 (from lory_merged_ffn_bwd)
 * in/out: dX [B, L, d] (dtype): the FFN path's input gradient, to which the
 *         router path is added in place (bf16: one more rounding per element)
 * out:    dR [d, E] fp32, overwritten, or added to when accumulate_dR = 1
 * Sums run in a fixed order (bit-reproducible).  Needs no workspace.
 * lory_route + lory_merged_ffn_fwd, then lory_merged_ffn_bwd + this call, are
 * the whole layer of Algorithm 1 and its gradient.
 */
int lory_route_bwd(const lory_shape *shape, const void *R, const float *w, const float *hbar,
                   const float *dw, void *dX, float *dR, int accumulate_dR, void *stream);

/*
 * Prompt-only routing at inference (Section 3.1, "Prompt-only routing during
 * inference"; Appendix G.1): one routing decision per sequence and layer from
 * the mean hidden state of the whole prompt, and the merged FFN it selects,
 * materialised once and then used like a dense FFN for the whole generation.
 *   w[b,:]   = softmax(mean over the prompt tokens of X_prompt[b] . R)
 *   Wx_bar_b = sum_e w[b,e] Wx[e]      x in {gate, up, down}
 * shape: L = rows per sequence of X_prompt (any length > 0) and T = L (one
 *        segment per sequence; anything else is LORY_ERR_SHAPE);
 *        LORY_BF16 needs d % 64 == 0 and d_ff % 64 == 0 only.
 * in:  X_prompt [B, L, d], R [d, E], Wg, Wu [E, d, d_ff], Wd [E, d_ff, d] (dtype);
 *      prompt_len_opt: NULL (every prompt has L tokens) or B int32 on the
 *      device, 4-byte aligned: sequence b's prompt is the first prompt_len[b]
 *      rows of X_prompt[b], the rest is padding that is never read (the mean
 *      is what lets the router take prompts of different lengths); values
 *      are clamped to 1 .. L
 * out: w [B, E] fp32; Wbar: 3 * B * d * d_ff elements of dtype, laid out
 *      [Wg_bar | Wu_bar | Wd_bar], each [B, rows, cols] like one expert matrix
 *      (the layout of Wbar_save).  Needs no workspace.
 * Per-segment routing at inference, the other mode the paper evaluates, is
 * lory_route + lory_merged_ffn_fwd as in training.
 */
int lory_prompt_merge(const lory_shape *shape, const void *X_prompt, const int32_t *prompt_len_opt,
                      const void *R, const void *Wg, const void *Wu, const void *Wd,
                      float *w, void *Wbar, void *stream);

/*
 * Dense SwiGLU FFN of every sequence with its own merged parameters, i.e. the
 * generation phase after lory_prompt_merge (or after a lory_merged_ffn_fwd
 * with T = L that filled Wbar_save):
 *   Y[b] = (G * sigmoid(G) (.) U) Wd_bar_b,  G = X[b] Wg_bar_b, U = X[b] Wu_bar_b
 * shape: L = tokens per sequence in this call (1 for a decode step), T = L.
 * in:  X [B, L, d] (dtype); Wbar as lory_prompt_merge wrote it
 * out: Y [B, L, d] (dtype)
 * LORY_BF16 with L % 64 == 0 runs on the batched matrix-core GEMMs; every other
 * case runs HBM-bound kernels that read each weight once per 8 tokens.
 * workspace: lory_workspace_bytes(shape, LORY_PASS_DENSE).
 */
int lory_dense_ffn_fwd(const lory_shape *shape, const void *X, const void *Wbar, void *Y,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * lory_dense_ffn_fwd for callers that cannot allocate device memory or carry
 * a workspace: code under HIP graph capture, tight serving loops (one decode
 * step per call), harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results; what lory_dense_ffn_fwd keeps in the
 * caller's workspace (partial sums of the K splits, or the activation block of
 * the matrix-core path) lives in a 16 MiB array in device memory that the
 * library itself holds (one copy per GPU, for the life of the process).
 * Returns LORY_ERR_WORKSPACE, before any launch, when
 * lory_workspace_bytes(shape, LORY_PASS_DENSE) exceeds 16 MiB (16777216 bytes):
 * at d = 2048, d_ff = 5632 a decode step of one token per sequence needs about
 * 6 MiB and two tokens per sequence about 12 MiB, whatever the batch (the K
 * split shrinks as the batch grows); larger calls take lory_dense_ffn_fwd.
 * The call allocates nothing and clears nothing (the kernels write every
 * value of the array before they read it).  All calls on one GPU share that
 * GPU's array: calls that overlap on one GPU (different streams, or different
 * host threads) race; calls on one stream do not.
 */
int lory_dense_ffn_fwd_static(const lory_shape *shape, const void *X, const void *Wbar, void *Y,
                              void *stream);

/*
 * Merged FFN forward (Eq. 1 / Eq. 2 with SwiGLU experts):
 *   for every segment s (S = B*N of them, T tokens each):
 *     Wg_bar = sum_e w[s,e] Wg[e],  Wu_bar, Wd_bar likewise
 *     G = X_s Wg_bar, U = X_s Wu_bar, A = G*sigmoid(G) (.) U, Y_s = A Wd_bar
 * in:  X [B, L, d]; w [S, E] fp32 (any rows: lory_route's output, one-hot,
 *      uniform ...); Wg, Wu [E, d, d_ff]; Wd [E, d_ff, d]
 * out: Y [B, L, d]; G_save, U_save [B*L, d_ff] (dtype) or both NULL;
 *      Wbar_save: NULL, or lory_merged_save_bytes() bytes that receive the
 *      merged parameters of all segments, laid out [Wg_bar | Wu_bar | Wd_bar],
 *      each [S, rows, cols] like one expert matrix (LORY_ERR_SHAPE if the
 *      shape does not support it).
 * Without Wbar_save the merged parameters are transient: they are produced
 * block by block into a slab inside the workspace and consumed from there by
 * the projections.  The slab is bounded by lory_set_slab_budget; with the
 * default budget of 6 GiB and a shape whose S * d * d_ff * 2 * 2 bytes fit, one
 * block is a whole matrix for all S segments (gate and up together at the
 * headline shape: 2.95 GB resident while the projections run).
 */
int lory_merged_ffn_fwd(const lory_shape *shape, const void *X, const float *w,
                        const void *Wg, const void *Wu, const void *Wd,
                        void *Y, void *G_save, void *U_save, void *Wbar_save,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * Merged FFN backward with w treated as an independent input (chain rule on
 * theta_bar = sum_e w_e theta_e, Eq. 2).  Per segment s, given dY_s:
 *   dA = dY Wd_bar^T;  dWd_bar = A^T dY
 *   dG = dA (.) U (.) sig(G)(1 + G(1 - sig(G)));  dU = dA (.) G sig(G)
 *   dWg_bar = X^T dG;  dWu_bar = X^T dU;  dX = dG Wg_bar^T + dU Wu_bar^T
 *   dWx[e] = sum_s w[s,e] dWx_bar(s);   dw[s,e] = sum_x <Wx[e], dWx_bar(s)>
 * in:  X, w, Wg, Wu, Wd as for the forward; dY [B, L, d];
 *      G_save, U_save from the forward, or both NULL to recompute them;
 *      Wbar_save from the forward (same shape, same w), or NULL to re-merge
 * out: dX [B, L, d] (FFN path only; the router path's contribution through
 *      the segment mean is not included); dWg, dWu [E, d, d_ff] and
 *      dWd [E, d_ff, d] in grad_dtype (LORY_F32, or for LORY_BF16 shapes also
 *      LORY_BF16); dw [S, E] fp32 for all segments including the first.
 *      accumulate = 0 overwrites dWg/dWu/dWd, 1 adds to them.  dX and dw are
 *      always overwritten.
 * The per-segment weight gradients dWx_bar are transient: they pass, one
 * block of d_ff columns at a time, through the slab inside the workspace
 * (bf16; bounded by lory_set_slab_budget - with the default budget and the
 * headline shape one block is all of d_ff, i.e. dWd_bar, dWg_bar and dWu_bar of
 * all S segments, 4.4 GB, are resident between the weight-gradient GEMMs and
 * the scatter).  Reductions across workgroups use a fixed order: two calls on
 * the same inputs give bit-identical results.
 */
int lory_merged_ffn_bwd(const lory_shape *shape, const void *X, const float *w,
                        const void *Wg, const void *Wu, const void *Wd,
                        const void *dY, const void *G_save, const void *U_save,
                        const void *Wbar_save,
                        void *dX, void *dWg, void *dWu, void *dWd,
                        int grad_dtype, int accumulate, float *dw,
                        void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LORY_H */
