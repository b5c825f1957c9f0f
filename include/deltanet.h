/*
 * deltanet.h - C ABI of the MI355X (gfx950) chunkwise-parallel DeltaNet layer.
 *
 * The operation is the DeltaNet token mixer of "Parallelizing Linear Transformers with the Delta
 * Rule over Sequence Length": per (sequence, head) chain, with a state S in R^{d_k x d_v},
 *
 *     S_t = S_{t-1} + beta_t k_t (v_t - S_{t-1}^T k_t)^T ,   o_t = S_t^T q_t
 *
 * (section 2.2, the delta update rule and read-out; section 3.1 writes the same update as a
 * generalized Householder transition S_{t-1}(I - beta k k^T) + beta v k^T; the state is kept in the
 * orientation of the paper's pseudocode listing, d_k rows by d_v columns).  It is evaluated in the
 * chunkwise-parallel form of section 3.2 (Eq. 8-9: inter-chunk state carry plus causal intra-chunk
 * output) with the per-chunk WY factors W, U built by the UT transform (Eq. 10-11).  No scale
 * factor is applied to q; normalising q, k and squashing beta are the caller's job.
 *
 * Conventions common to every call
 *  - All data pointers are DEVICE pointers unless a name ends in _host.  The caller owns every
 *    buffer; the library never allocates, frees or synchronises.  All work is enqueued on
 *    `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *  - Dense layout: q,k [B,L,H,d_k]; v,o,do [B,L,H,d_v]; beta [B,L,H]; states [B,H,d_k,d_v].
 *    Packed layout (cu_seqlens != NULL): B must be 1, L is the total token count, sequence n
 *    covers rows cu_seqlens[n] .. cu_seqlens[n+1]-1, the state is reset at every sequence start and
 *    states are [num_seqs,H,d_k,d_v].  All tensors are contiguous and row-major.
 *  - q,k,v,beta,o,do,dq,dk,dv have element type `dtype` (fp32, or bf16 with fp32 accumulation);
 *    states, state gradients and dbeta are always fp32.
 *  - Every data pointer must be 16-byte aligned.
 *  - `workspace` is caller-provided device scratch of at least deltanet_workspace_bytes();
 *    its contents are undefined afterwards.  (For few long sequences the passes cut the sequences into
 *    segments that are scanned side by side; the per-segment states this needs are part of that size.)
 *  - Return value: DN_OK (0) or a negative dn_status.  All validation happens before the first
 *    launch; on a validation error nothing has been enqueued.  No exceptions, no abort.
 *  - Packed layout without cu_seqlens_host: nothing can be validated on the host; the kernels then work on the
 *    running maximum of the device array held inside [0, L] (the array itself if it is valid), so a malformed array
 *    gives meaningless results but no access outside the tensors or the workspace.
 *  - A tensor without rows (B * L == 0) may come with a NULL pointer; final_state is then initial_state (or zero).
 *  - Sequences of length 0 are allowed in the packed layout; lengths need not be multiples of
 *    the chunk size (a ragged last chunk is handled exactly, as beta = 0 leaves the state
 *    unchanged, section 2.2).
 */
#ifndef DELTANET_H_
#define DELTANET_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DN_F32 = 0, DN_BF16 = 1 } dn_dtype;

typedef enum {
    DN_OK = 0,
    DN_ERR_NULL = -1,        /* a required pointer is NULL */
    DN_ERR_SHAPE = -2,       /* a size is non-positive or inconsistent */
    DN_ERR_UNSUPPORTED = -3, /* (dtype, d_k, d_v, chunk) has no compiled kernel */
    DN_ERR_ALIGN = -4,       /* a data pointer is not 16-byte aligned */
    DN_ERR_WORKSPACE = -5,   /* workspace is NULL or too small */
    DN_ERR_CUSEQLENS = -6,   /* cu_seqlens_host is not 0 = c[0] <= c[1] <= ... <= c[N] = L */
    DN_ERR_LAUNCH = -7       /* the HIP runtime reported an error at launch */
} dn_status;

typedef struct {
    int32_t B, L, H, d_k, d_v;
    int32_t chunk;                   /* C of section 3.2; 64 is the compiled value */
    int32_t dtype;                   /* dn_dtype */
    int32_t num_seqs;                /* packed layout only: N */
    const int32_t *cu_seqlens;       /* DEVICE int32 [N+1], or NULL for the dense layout */
    const int32_t *cu_seqlens_host;  /* optional HOST copy of the same array; if given it is
                                        validated (DN_ERR_CUSEQLENS) and never dereferenced later */
} dn_shape;

/* Bytes of device scratch that deltanet_fwd (want_bwd = 0) or deltanet_bwd (want_bwd != 0) needs
 * for this shape.  Host-only; touches no device. */
int deltanet_workspace_bytes(const dn_shape *shape, int want_bwd, size_t *out_bytes);

/*
 * Forward pass (Eq. 8-11).  initial_state may be NULL (zeros).  final_state may be NULL (not
 * written).  Outputs: o (element type dtype), final_state (fp32).
 * Compiled (d_k, d_v): fp32 (64,64), (32,64), (64,32); bf16 (128,128), (64,64), (64,128), (128,64)
 * and (256,256); every entry point below runs at each of them.
 */
int deltanet_fwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                 const float *initial_state, void *o, float *final_state, void *workspace,
                 size_t workspace_bytes, void *hip_stream);

/*
 * deltanet_fwd for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as deltanet_fwd, minus the workspace: the
 * scratch the pass needs is a device array of DN_STATIC_SCRATCH_BYTES that is part of the library (every GPU the
 * library runs on holds its own copy until the process ends).  The call allocates and frees nothing.  Shapes whose
 * deltanet_workspace_bytes(shape, 0) exceeds DN_STATIC_SCRATCH_BYTES are refused with DN_ERR_WORKSPACE before anything
 * is enqueued (one C x C tile per chunk and head: 36 MiB covers 16 384 tokens x 16 heads in bf16, half as many in
 * fp32).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it; calls on one stream, or otherwise ordered, do not.  Nothing in the array needs clearing
 * between calls.
 */
#define DN_STATIC_SCRATCH_BYTES (36u << 20)
int deltanet_fwd_static(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                        const float *initial_state, void *o, float *final_state, void *hip_stream);

/*
 * Backward pass: exact gradient of  sum(o * d_o) + sum(final_state * dfinal_state)  with respect to
 * q, k, v, beta and initial_state.  Self-contained: chunk states are recomputed from the inputs
 * (section 3.2, "hidden states recomputed during the backward pass"), so nothing from the forward
 * call has to be kept.  dfinal_state may be NULL (zeros); dinitial_state may be NULL (not written).
 * Outputs: dq, dk, dv (element type dtype), dbeta (fp32, shape of beta), dinitial_state (fp32).
 */
int deltanet_bwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                 const float *initial_state, const void *d_o, const float *dfinal_state, void *dq,
                 void *dk, void *dv, float *dbeta, float *dinitial_state, void *workspace,
                 size_t workspace_bytes, void *hip_stream);

/*
 * The same forward and backward pass for a training step that keeps the forward pass's per-chunk
 * results instead of recomputing them (the other side of the trade section 3.2 describes: with
 * hundreds of GB of HBM the chunk states of a layer, d_k * d_v * 2 bytes per 64 tokens and head in
 * bf16, are cheap to keep, and the backward pass then skips the UT transform and the forward scan).
 * deltanet_fwd_save computes what deltanet_fwd computes and leaves T and (I + A)^-1 of Eq. 10, the
 * chunk-initial states and U - W S of Eq. 8 in `saved`; deltanet_bwd_saved computes what deltanet_bwd
 * computes from the same q, k, v, beta and that buffer, which it also uses as scratch (afterwards the
 * buffer can serve another deltanet_fwd_save, not another deltanet_bwd_saved).  `saved` is
 * caller-provided device memory of deltanet_workspace_bytes(shape, 1) bytes; its layout is private to
 * the library, and it must stay untouched between the two calls.  The initial state is not an argument
 * of deltanet_bwd_saved: it is the first saved chunk state.  Everything else is as for deltanet_fwd /
 * deltanet_bwd; head sizes without a backward pass return DN_ERR_UNSUPPORTED.
 */
int deltanet_fwd_save(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                      const float *initial_state, void *o, float *final_state, void *saved, size_t saved_bytes,
                      void *hip_stream);
int deltanet_bwd_saved(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                       const void *d_o, const float *dfinal_state, void *dq, void *dk, void *dv, float *dbeta,
                       float *dinitial_state, void *saved, size_t saved_bytes, void *hip_stream);

/*
 * The same passes with the layer's prologue fused into the load path (section 3.3, "Feature map and
 * normalization", and the writing strength of section 2.2): the caller hands over the pre-activations
 * q_pre, k_pre (layouts and element type of q, k) and the logits beta_logit (layout and element type of
 * beta), and the kernels form
 *
 *     q_t = SiLU(q_pre_t) / ||SiLU(q_pre_t)||_2 ,  k_t likewise,  beta_t = sigmoid(beta_logit_t)
 *
 * per token and head (fp32 arithmetic, result rounded to the element type).  The kernel that builds T
 * maps q and k once and leaves them in the workspace for the chain scans; the backward's chunk kernel
 * maps its tiles on their way to the LDS and sends dq, dk back through the map on their way out, so at head
 * sizes up to 128 the gradients never reach HBM in the mapped coordinates and no separate elementwise pass runs
 * in either direction.  At head size 256 the way back is not fused: the chunk kernel writes dq, dk in the mapped
 * coordinates (element type dtype) and one more kernel per tensor takes them through the map in place, so those
 * two gradients are rounded to the element type twice.  A row whose SiLU image is exactly zero maps to zero (the
 * paper gives no epsilon).
 * deltanet_fused_bwd returns the gradients with respect to q_pre, k_pre and beta_logit (through the
 * normalisation, the SiLU and the sigmoid) in dq_pre, dk_pre (element type dtype) and dbeta_logit
 * (fp32); dv and dinitial_state are as for deltanet_bwd.  Workspace (and `saved`) sizes come from
 * deltanet_fused_workspace_bytes: the plain sizes plus the mapped q and k.  deltanet_fused_fwd_save /
 * deltanet_fused_bwd_saved are the pair that keeps the forward pass's per-chunk results, as
 * deltanet_fwd_save / deltanet_bwd_saved.  Everything else is as for the plain calls.
 */
int deltanet_fused_workspace_bytes(const dn_shape *shape, int want_bwd, size_t *out_bytes);
int deltanet_fused_fwd(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v, const void *beta_logit,
                       const float *initial_state, void *o, float *final_state, void *workspace, size_t workspace_bytes,
                       void *hip_stream);
int deltanet_fused_bwd(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v, const void *beta_logit,
                       const float *initial_state, const void *d_o, const float *dfinal_state, void *dq_pre, void *dk_pre,
                       void *dv, float *dbeta_logit, float *dinitial_state, void *workspace, size_t workspace_bytes,
                       void *hip_stream);
int deltanet_fused_fwd_save(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v,
                            const void *beta_logit, const float *initial_state, void *o, float *final_state, void *saved,
                            size_t saved_bytes, void *hip_stream);
int deltanet_fused_bwd_saved(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v,
                             const void *beta_logit, const void *d_o, const float *dfinal_state, void *dq_pre, void *dk_pre,
                             void *dv, float *dbeta_logit, float *dinitial_state, void *saved, size_t saved_bytes,
                             void *hip_stream);

/*
 * Forward pass in the recurrent (token-serial) form: the delta-rule update and read-out of
 * section 2.2 applied one token after the other, state in fp32 registers, no chunking, no matrix
 * cores and no workspace.  It computes the same o and final_state as deltanet_fwd (fp32 arithmetic
 * on the fp32 or bf16 inputs) and is what a decoder calls with L = 1 per step, handing
 * final_state back in as initial_state; it is also the baseline the paper's chunkwise form is
 * timed against (section 3.3).  Same layouts, pointer rules and return codes as deltanet_fwd.
 * Compiled for d_k in {32, 64, 128, 256} and any d_v that is a multiple of 16, both dtypes
 * (else DN_ERR_UNSUPPORTED).  `chunk` is not used but must hold a supported value.
 * initial_state may be NULL (zeros); final_state may be NULL (not written); the two may alias.
 */
int deltanet_recurrent_fwd(const dn_shape *shape, const void *q, const void *k, const void *v,
                           const void *beta, const float *initial_state, void *o, float *final_state,
                           void *hip_stream);

/*
 * Gated variant: the last row of the paper's overview table of linear recurrent models (section 6),
 * which its limitations section names as the way to add the decay DeltaNet lacks.  A scalar decay
 * alpha_t = exp(g_t) per token and head multiplies the transition,
 *
 *     S_t = alpha_t (S_{t-1} - beta_t k_t (S_{t-1}^T k_t)^T) + beta_t k_t v_t^T ,   o_t = S_t^T q_t
 *
 * (state orientation as above; g = 0 is the plain delta rule).  g is fp32 [B,L,H] (packed: [L,H]),
 * g <= 0 expected; inside one chunk of 64 tokens the sum of |g| must stay below about 160 (a mean alpha
 * of about 0.08), as the kernels work with exp(+-(sum g) / 2) in fp32.  Evaluated chunkwise like
 * deltanet_fwd / deltanet_bwd: with gamma_i the running product of alpha inside a chunk, taken relative
 * to the chunk's geometric middle, S_i / gamma_i follows the plain delta rule on the values
 * v_i / gamma_i, so Eq. 8-11 apply unchanged to rescaled rows.  In bf16 the gate gradient dg, a
 * difference of nearly equal sums of rounded gradients, loses relative accuracy as the decay grows.  deltanet_gated_bwd also
 * returns dg (fp32, shape of g).  Workspace sizes come from deltanet_gated_workspace_bytes; everything
 * else (layouts, nullable states, return codes) is as for the plain calls.
 * deltanet_gated_recurrent_fwd is the token-serial form (decode steps), as deltanet_recurrent_fwd.
 */
int deltanet_gated_workspace_bytes(const dn_shape *shape, int want_bwd, size_t *out_bytes);
int deltanet_gated_fwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                       const float *g, const float *initial_state, void *o, float *final_state, void *workspace,
                       size_t workspace_bytes, void *hip_stream);
int deltanet_gated_bwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                       const float *g, const float *initial_state, const void *d_o, const float *dfinal_state,
                       void *dq, void *dk, void *dv, float *dbeta, float *dg, float *dinitial_state, void *workspace,
                       size_t workspace_bytes, void *hip_stream);
int deltanet_gated_recurrent_fwd(const dn_shape *shape, const void *q, const void *k, const void *v,
                                 const void *beta, const float *g, const float *initial_state, void *o,
                                 float *final_state, void *hip_stream);
/* The gated pair that keeps the forward pass's per-chunk results, as deltanet_fwd_save / deltanet_bwd_saved;
 * `saved` holds deltanet_gated_workspace_bytes(shape, 1) bytes. */
int deltanet_gated_fwd_save(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                            const float *g, const float *initial_state, void *o, float *final_state, void *saved,
                            size_t saved_bytes, void *hip_stream);
int deltanet_gated_bwd_saved(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                             const float *g, const void *d_o, const float *dfinal_state, void *dq, void *dk, void *dv,
                             float *dbeta, float *dg, float *dinitial_state, void *saved, size_t saved_bytes,
                             void *hip_stream);

/*
 * Measurement aid (not part of the method): per-kernel device time.  After
 * deltanet_profile_enable(1), every kernel launch of deltanet_fwd / deltanet_bwd is bracketed by a
 * pair of HIP events recorded on the launch stream.  deltanet_profile_collect waits for those
 * events, sums the elapsed milliseconds per kernel name into `out` (at most max_entries distinct
 * kernels; HOST memory), stores the number of entries and forgets the records.  Events cost a few
 * microseconds per launch, so whole-pass timings should be taken with profiling disabled.
 */
typedef struct {
    char name[96];    /* kernel name with its template arguments, as written in the source */
    double total_ms;  /* summed device time between the two events */
    int32_t launches;
} dn_kernel_time;
int deltanet_profile_enable(int on);
int deltanet_profile_collect(dn_kernel_time *out, int max_entries, int *num_entries);

/*
 * Process-wide options (each 0 by default).
 *  DN_OPT_STREAMED_CHUNK_KERNEL: the backward pass of the plain delta rule in bf16 (head sizes up to 128) takes the chunk
 *    kernel that reads the chunk states in blocks of 32 state columns and rebuilds U - W S of Eq. 8 and its gradient on
 *    chip instead of reading them back from the scans, which then do not store them: 13 % fewer bytes through HBM per
 *    training step, and on MI355X a slower step (the blocks take more barrier intervals than they save in traffic).
 *    Same results to within rounding.  deltanet_fwd_save and the deltanet_bwd_saved that follows it must run under the
 *    same setting.  Unknown options return DN_ERR_UNSUPPORTED.
 */
typedef enum { DN_OPT_STREAMED_CHUNK_KERNEL = 0 } dn_option;
int deltanet_set_option(int option, int value);

/*
 * Measurement aid (not part of the method): one launch of a probe kernel that repeats, `iters` times, ONE of the LDS
 * access patterns the kernels are built from (pattern 0..17: operand-fragment reads in both storage orders, accumulator
 * and register tiles written to LDS, row-segment reads; the list is in csrc/dn_lds_probe.hip), so that a profiler's LDS
 * counters can be read per pattern.  256 workgroups of 512 threads, no global memory traffic.  iters in [0, 2^20];
 * DN_ERR_UNSUPPORTED for an unknown pattern.  The launch is enqueued on hip_stream.
 */
int deltanet_lds_probe(int pattern, int iters, void *hip_stream);

/* Static, NUL-terminated description of a dn_status value. */
const char *deltanet_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DELTANET_H_ */
