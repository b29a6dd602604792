/*
 * gka.h -- C ABI of libgka: the Gated KalmaNet (GKA) layer forward pass on AMD MI355X (gfx950).
 *
 * The library evaluates, for every (batch, head) pair and token t, the recurrence of the paper's
 * Eq. (CH) (Section 4.1, "Forward Recurrence"):
 *
 *     H_t = gamma_t H_{t-1} + k_t k_t^T,      U_t = gamma_t U_{t-1} + v_t k_t^T,
 *     xhat_t = CH(H_t + lambda_t I, q_t, r),  y_t = U_t xhat_t,
 *
 * where CH is r passes of the Chebyshev Iteration (Algorithm 1) with eigenvalue bounds
 * L = ||H_t||_F + lambda_t and mu = lambda_t (Section 4.1, "Adaptive Regularization").
 * gka_forward processes whole sequences chunk-wise (Section 4.2.1); gka_decode_step advances
 * stored states by one token, gka_decode_tokens by a few.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers. The caller owns every buffer; the library never
 *     allocates, frees or synchronises. All work is enqueued on the given HIP stream
 *     (a hipStream_t passed as void*; NULL is the default stream).
 *   - Every call returns a gka_status. Argument errors are detected on the host before any
 *     kernel is launched, and leave all buffers untouched.
 *   - Value preconditions are NOT checked: gamma in [0, 1], lambda > 0, finite inputs.
 *     Gates below exp(-100), including 0, are treated as exp(-100) by gka_forward: such a gate wipes
 *     the state (to within 4e-44 of its magnitude). This is how packed variable-length sequences are
 *     run: concatenate them along T and give the first token of every sequence a gate of 0.
 *   - State layout: H[b][h][i][j] (d_k x d_k) and U[b][h][i_v][j_k] (d_v x d_k, U = sum v k^T),
 *     row-major float32.
 */
#ifndef GKA_H_
#define GKA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    GKA_OK = 0,
    GKA_ERR_NULL = 1,         /* a required pointer is NULL                                   */
    GKA_ERR_SHAPE = 2,        /* non-positive or inconsistent size / stride                   */
    GKA_ERR_UNSUPPORTED = 3,  /* head dimension, chunk, dtype or compute mode not supported   */
    GKA_ERR_WORKSPACE = 4,    /* workspace NULL, misaligned or smaller than the query says    */
    GKA_ERR_LAUNCH = 5,       /* a HIP call or kernel launch reported an error                */
    GKA_ERR_STATIC_SCRATCH = 6 /* gka_forward_static: the problem needs more than GKA_STATIC_SCRATCH_BYTES */
} gka_status;

typedef enum { GKA_F32 = 0, GKA_BF16 = 1 } gka_dtype;

/* Arithmetic of the matrix products.
 * GKA_COMPUTE_F32 : float32 operands on the float32 MFMA path (required for GKA_F32 tensors).
 * GKA_COMPUTE_BF16: bf16 operands with float32 accumulation on the bf16 MFMA path; the Chebyshev
 *                   iterate, the residual and all per-token scalars stay float32.
 * GKA_COMPUTE_BF16_SPLIT: the bf16 MFMA path for ill-conditioned systems (lambda_t orders of magnitude below
 *                   ||H_t||_F, where the iteration amplifies the rounding of its operands): the chunk's initial state
 *                   H_[n], the update of the iterate and the masked intra-chunk products enter their products as
 *                   bf16 value + bf16 remainder, about 2.6 times the products of GKA_COMPUTE_BF16 and a fraction of the cost of GKA_COMPUTE_F32. (Appendix
 *                   B.1 leaves the precision of the matrix products to the implementation.) gka_forward only, and only
 *                   what the fused kernel covers (see gka_path); GKA_ERR_UNSUPPORTED otherwise. */
typedef enum { GKA_COMPUTE_F32 = 0, GKA_COMPUTE_BF16 = 1, GKA_COMPUTE_BF16_SPLIT = 2 } gka_compute;

/* Which part of gka_forward to enqueue. The forward pass has two phases (Section 4.2.1): first the
 * chunk initial states H_[n], U_[n] are computed and stored in the workspace (this phase also writes
 * H_final / U_final), then every chunk is solved independently from its stored state (this phase writes
 * o and fro_out). GKA_PHASE_SOLVE alone is valid only on a workspace that still holds the states of a
 * GKA_PHASE_STATES (or GKA_PHASE_ALL) call with the same parameters and inputs; it exists so that
 * callers can overlap the two phases. A single phase can be requested only when the problem is small
 * enough to be processed as one launch of each kernel (otherwise GKA_ERR_UNSUPPORTED). */
typedef enum { GKA_PHASE_ALL = 0, GKA_PHASE_STATES = 1, GKA_PHASE_SOLVE = 2 } gka_phase;

/* Which elements of a stored H state carry it. H_t is symmetric, so a decode cache needs only one triangle.
 * GKA_STATE_FULL          : all d x d elements are read and written.
 * GKA_STATE_H_LOWER_BLOCKS: only the 32 x 32 blocks on and below the block diagonal are: element [i][j] with
 *                           j < 32 (i / 32 + 1). gka_decode_step and gka_decode_tokens neither read nor write the
 *                           other elements of H_state (the buffer keeps its [d,d] shape; those elements keep
 *                           whatever they held), which removes 3/8 (d = 128) or 1/4 (d = 64) of the traffic of H;
 *                           gka_forward reads H_init the same way (its H_final is always written in full, which
 *                           is valid under either layout). U states are not symmetric and are always full. */
typedef enum { GKA_STATE_FULL = 0, GKA_STATE_H_LOWER_BLOCKS = 1 } gka_state_layout;

/* Which kernels gka_forward runs.
 * GKA_PATH_AUTO     : the library's choice (the fused kernel where it applies, else the two-phase kernels; token by
 *                     token where there are no chunk-wise kernels).
 * GKA_PATH_TWO_PHASE: chunk initial states H_[n], U_[n] of Section 4.2.1 are computed and stored in the workspace
 *                     first, then every chunk is solved independently. d = 64, 128: all dtypes and variants; d = 16,
 *                     32: GKA_BF16 tensors with GKA_COMPUTE_BF16, all variants, GKA_PHASE_ALL (kernels of their own,
 *                     whose matrix products cover a whole state in one instruction).
 * GKA_PATH_FUSED    : one kernel walks the chunks of a pair in order with H and U in registers, so that no chunk state
 *                     crosses HBM. Available for GKA_BF16 tensors with GKA_COMPUTE_BF16 (or _SPLIT), d = 128, with or without
 *                     the layer's variants (beta, alpha, the rule for lambda) but without xhat_out, GKA_PHASE_ALL;
 *                     GKA_ERR_UNSUPPORTED otherwise.
 * GKA_PATH_RECURRENT: Eq. (CH) token by token, one workgroup per (batch, head) pair with the states in registers (the
 *                     kernel of gka_decode_tokens), float32 arithmetic whatever p->compute says. Every head dimension,
 *                     dtype, stride and variant, with xhat_out and fro_out; GKA_PHASE_ALL only. It is the only path
 *                     for d = 256 and for float32 tensors or operands at d = 16 and 32 (what GKA_PATH_AUTO selects
 *                     there) and its parallelism is the number of pairs: meant for short sequences over many heads
 *                     and as a float32 cross-check of the chunk-wise kernels, not for long sequences over few
 *                     pairs. Gates are used as given (no floor at exp(-100)). */
typedef enum { GKA_PATH_AUTO = 0, GKA_PATH_TWO_PHASE = 1, GKA_PATH_FUSED = 2, GKA_PATH_RECURRENT = 3 } gka_path;

typedef struct {
    int32_t B;            /* batch (gka_decode_step: number of sequences)                      */
    int32_t H;            /* heads                                                             */
    int32_t T;            /* tokens per sequence (ignored by gka_decode_step); any T >= 1      */
    int32_t d_k;          /* head dimension of q, k: 16, 32, 64, 128 or 256 (gka_backward and    */
                          /*   gka_forward_sketched: 64 or 128; which kernels run: see gka_path)  */
    int32_t d_v;          /* head dimension of v, o: must equal d_k                            */
    int32_t chunk;        /* chunk size C of Section 4.2.1: 64 (T need not be a multiple)      */
    int32_t n_iter;       /* r of Algorithm 1 = number of loop passes; 0 returns U_t xi_0      */
    int32_t io_dtype;     /* gka_dtype of q, k, v, o                                           */
    int32_t compute;      /* gka_compute                                                       */
    int32_t phase;        /* gka_phase; GKA_PHASE_ALL (0) for a complete forward pass          */
    int64_t stride_b;     /* element strides of q, k, v, o between batches, tokens and heads;  */
    int64_t stride_t;     /*   the head dimension is contiguous. 0,0,0 selects the packed      */
    int64_t stride_h;     /*   [B,T,H,d] layout of the paper's tensors (Appendix D). Explicit  */
                          /*   strides: multiples of 4 elements (of 8 for GKA_COMPUTE_BF16,    */
                          /*   where stride_t must also stay below 2^23); q, k, v, o 16-byte   */
                          /*   aligned                                                          */
    /* Variants of the layer (Section 4.1 "Adaptive Regularization" and its Remark, Section 4.3). With
     * lambda_scale = 0 and both pointers NULL the call is Eq. (CH) as printed. */
    float   lambda_scale; /* a > 0 of lambda_t = a ||H_t||_F; used when the lambda argument is NULL     */
    int32_t state_layout; /* gka_state_layout of H_state / H_init: 0 = every element is read and written   */
    const float *beta;    /* DEVICE pointer or NULL (= 1): write gate beta_t in [0,1] of the            */
                          /*   beta-augmented recurrence H_t = gamma_t H_{t-1} + beta_t k_t k_t^T,      */
                          /*   U_t = gamma_t U_{t-1} + beta_t v_t k_t^T; [B,T,H] ([B,H] for decode)     */
    const float *alpha;   /* DEVICE pointer or NULL (= 1): alpha-connection, the readout becomes        */
                          /*   y_t = U_t (alpha_t xhat_t + (1 - alpha_t) q_t); same shape as beta       */
    float *xhat_out;      /* DEVICE pointer or NULL: gka_forward also writes the solve's result            */
                          /*   xhat_t = CH(H_t + lambda_t I, q_t, r) here, packed [B,T,H,d_k] float32       */
                          /*   (before the alpha-connection). With q := an incoming gradient this is the    */
                          /*   solve of the backward pass, CH(H_t + lambda_t I, dxhat_t, r) (Section 4.2.2). */
                          /*   Ignored by the decode entry points.                                          */
    /* Launch plan of gka_forward (0 everywhere = the library's choices; results do not depend on these beyond
     * rounding). They exist so that callers and tests can bound the workspace or force short walks. */
    int64_t slab_state_bytes; /* two-phase kernels: bytes of chunk states one launch pair keeps in the workspace  */
                              /*   (0 = 1 GiB); larger problems run as several launches, states carried in fp32   */
    int32_t walk_chunks;      /* fused kernel: chunks one workgroup walks (rounded up to an even number); the     */
                              /*   sequence is cut into such segments, whose start states come from a summary     */
                              /*   launch. 0 = as few segments as fill the GPU                                    */
    int32_t path;             /* gka_path                                                                         */
} gka_params;

/* Bytes of scratch gka_forward needs for these parameters (0 if they are invalid). The buffer must
 * be 256-byte aligned. It holds the chunk initial states H_[n], U_[n] of Section 4.2.1 in the
 * operand layout of the solve kernel, for one batch of (batch, head) pairs and one slab of consecutive
 * chunks at a time: large problems are processed as a sequence of such launches, the running states
 * carried from slab to slab in float32, so that the workspace stays bounded (about 1 GiB of chunk
 * states; p->slab_state_bytes overrides that budget). The fused kernel (gka_path) needs only the segment summaries
 * of its chunk walk; the query returns the larger of the two sizes. The chunk-wise kernels of d = 16 and 32 keep four
 * d x d float32 states per chunk. The token-by-token path (GKA_PATH_RECURRENT) keeps
 * its states in registers: 256 bytes, plus one U state per pair at d = 256. Its contents after a call are unspecified. */
size_t gka_forward_workspace_bytes(const gka_params *p);

/* Whole-sequence forward, Eq. (CH).
 *   q, k     [B,T,H,d_k]  io_dtype           v  [B,T,H,d_v]  io_dtype
 *   gate     [B,T,H] float32, gamma_t        lambda [B,T,H] float32, lambda_t > 0, or NULL with
 *                                             p->lambda_scale > 0 (lambda_t = lambda_scale ||H_t||_F)
 *   o        [B,T,H,d_v]  io_dtype (written)
 *   H_init   [B,H,d_k,d_k], U_init [B,H,d_v,d_k] float32, or NULL for zero initial states;
 *            gamma of the first token multiplies the initial state
 *   H_final, U_final      same shapes, written if not NULL (state after the last token)
 *   fro_out  [B,T,H] float32 ||H_t||_F, written if not NULL
 *   workspace, workspace_bytes: see gka_forward_workspace_bytes
 * gate and lambda are packed [B,T,H] regardless of the q/k/v strides. */
gka_status gka_forward(const gka_params *p,
                       const void *q, const void *k, const void *v,
                       const float *gate, const float *lambda,
                       void *o,
                       const float *H_init, const float *U_init,
                       float *H_final, float *U_final,
                       float *fro_out,
                       void *workspace, size_t workspace_bytes,
                       void *hip_stream);

/* gka_forward for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc. The same arguments as gka_forward without the
 * workspace, the same kernels and the same results; the scratch that the kernels need (segment summaries of the chunk
 * walk and the parked states, 196,612 bytes per workgroup) lives in an array of GKA_STATIC_SCRATCH_BYTES
 * that the library's code object reserves on every GPU it is loaded on, until the process ends. The call allocates
 * and frees nothing, on the device or through any library.
 *   Supported: what the fused kernels cover (see gka_path: GKA_BF16 tensors, GKA_COMPUTE_BF16 or _SPLIT, d = 128, no
 *   xhat_out, GKA_PHASE_ALL, path not GKA_PATH_TWO_PHASE), else GKA_ERR_UNSUPPORTED.
 *   Size limit: (number of (batch, head) pairs) x (segments of the chunk walk) x 196,612 bytes (+ padding) must not
 *   exceed GKA_STATIC_SCRATCH_BYTES: at most 341 workgroups. The library cuts the walk into ceil(256 / (B H))
 *   segments (fewer for short sequences); p->walk_chunks >= ceil(T / 64) asks for a single segment, with which any
 *   B H <= 341 fits. Larger: GKA_ERR_STATIC_SCRATCH, nothing is launched.
 *   Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race and
 *   give wrong results; calls on one stream, or ordered by events, are safe. Nothing in the array needs clearing
 *   between calls: every word a call reads it has written before.
 *   Under stream capture the call records kernel launches only. The first call on a device looks up the array's address
 *   and sets kernel attributes: make it outside a capture. */
#define GKA_STATIC_SCRATCH_BYTES (64u << 20)
gka_status gka_forward_static(const gka_params *p,
                              const void *q, const void *k, const void *v,
                              const float *gate, const float *lambda,
                              void *o,
                              const float *H_init, const float *U_init,
                              float *H_final, float *U_final,
                              float *fro_out,
                              void *hip_stream);

/* gka_forward for profiling: the same work with the same arguments, bracketed per phase by HIP events on the
 * given stream. Unlike every other entry point this one creates and destroys events and BLOCKS until the work
 * has finished. It returns the time spent in the chunk-state phase and in the per-chunk solve phase
 * (milliseconds, summed over the launches of this call) and the number of solve-kernel launches the call was
 * split into (batches of pairs and slabs of chunks, see gka_forward_workspace_bytes). Host pointers:
 * ms_states, ms_solve, n_solve_launches. */
gka_status gka_forward_profile(const gka_params *p,
                               const void *q, const void *k, const void *v,
                               const float *gate, const float *lambda,
                               void *o,
                               const float *H_init, const float *U_init,
                               float *H_final, float *U_final,
                               float *fro_out,
                               void *workspace, size_t workspace_bytes,
                               void *hip_stream,
                               float *ms_states, float *ms_solve, int32_t *n_solve_launches);

/* One recurrent step of Eq. (CH) on stored states (T is ignored).
 *   H_state [B,H,d_k,d_k], U_state [B,H,d_v,d_k] float32, updated IN PLACE
 *   q, k [B,H,d_k], v [B,H,d_v] io_dtype (packed); gate, lambda [B,H] float32 (lambda NULL as in gka_forward)
 *   o [B,H,d_v] io_dtype (written)
 * The arithmetic is float32 for either compute mode. Every head dimension of gka_params; the block-lower layout of H
 * up to d = 128 (d = 16 and 32 are a single block: the layout is the full one). */
gka_status gka_decode_step(const gka_params *p,
                           float *H_state, float *U_state,
                           const void *q, const void *k, const void *v,
                           const float *gate, const float *lambda,
                           void *o, void *hip_stream);

/* Several recurrent steps of Eq. (CH) on stored states in one call: the T = p->T next tokens of every sequence
 * (short continuations: speculative or multi-token decoding, the tail of a prompt). The result equals T calls of
 * gka_decode_step, but the states cross HBM once per call instead of once per token; each (sequence, head) pair
 * is advanced by one workgroup, token after token, in float32. For long segments gka_forward (with H_init /
 * H_final) is the faster path: its work runs on the matrix cores.
 *   H_state [B,H,d_k,d_k], U_state [B,H,d_v,d_k] float32, updated IN PLACE to the state after the last token
 *   q, k [B,T,H,d_k], v [B,T,H,d_v] io_dtype, packed (explicit strides: GKA_ERR_UNSUPPORTED);
 *   gate, lambda (NULL as in gka_forward), p->beta, p->alpha [B,T,H] float32
 *   o [B,T,H,d_v] io_dtype (written)
 * T <= 0: GKA_ERR_SHAPE. */
gka_status gka_decode_tokens(const gka_params *p,
                             float *H_state, float *U_state,
                             const void *q, const void *k, const void *v,
                             const float *gate, const float *lambda,
                             void *o, void *hip_stream);

/* Backward pass of the layer by implicit differentiation (Section 4.2.2 "Backward Pass", Appendix B.2): given
 * dy_t = dL/dy_t, the gradients at q, k, v, the gates and lambda (and at the write gate and the alpha-connection if
 * they are in use). The forward solve's result is treated as the exact solution of its system and both solves run
 * r passes of Algorithm 1 (dq_t = CH(H_t + lambda_t I, dxhat_t, r)), as in the paper. The two solves run on the
 * forward kernels; the reverse recurrences of Section 4.2.2 are six gated-linear-attention readouts (seven on bf16
 * tensors, where the output is read out again from the stored operand for the gate gradient), four of them
 * walking the sequence backwards (one kernel with the state in registers for GKA_BF16 tensors, the forward kernels
 * on reversed copies for GKA_F32 tensors), plus a few elementwise kernels: about five times the cost of gka_forward
 * with bf16 tensors and operands; the paper's chunk-wise backward kernels are not reproduced.
 *   Supported: lambda given or NULL with p->lambda_scale > 0 (the rule lambda_t = a ||H_t||_F, whose w_t H_t terms
 *   of the Lemma in Section 4.2.2 cost two more readouts), zero initial states (gka_backward_from_state takes
 *   others), p->beta and p->alpha as in gka_forward. Explicit strides apply to q, k, v and dy (multiples of 16
 *   bytes; they are copied into the packed layout first: four more tensors of workspace); the gradients are always
 *   written packed. Packed sequences (a gate of 0 at a sequence's first token) are handled:
 *   dgate at such a gate is written as 0 (the formula divides by the gate), and the cumulative sum behind dgate
 *   restarts there.
 *   q, k, v, dy  [B,T,H,d] io_dtype, 16-byte aligned;  gate, lambda [B,T,H] float32
 *   dq, dk, dv   [B,T,H,d] float32, 16-byte aligned (written);  dgate [B,T,H] float32 (written)
 *   dlambda, dbeta, dalpha [B,T,H] float32, each written if not NULL (dlambda only when lambda is given)
 *   workspace: gka_backward_workspace_bytes(p) bytes, 256-byte aligned (about 24 tensors of the size of q in
 *   io_dtype plus the forward workspace); contents unspecified afterwards. */
size_t gka_backward_workspace_bytes(const gka_params *p);
gka_status gka_backward(const gka_params *p,
                        const void *q, const void *k, const void *v,
                        const float *gate, const float *lambda,
                        const void *dy,
                        float *dq, float *dk, float *dv, float *dgate,
                        float *dlambda, float *dbeta, float *dalpha,
                        void *workspace, size_t workspace_bytes,
                        void *hip_stream);

/* gka_backward for a sequence that continues from given states (chunked training over a long sequence, a prefix
 * cached elsewhere): the forward pass starts from H_init, U_init as gka_forward does (the first gate multiplies them),
 * and the gradients at the two states are returned as well,
 *     dH_init = gamma_0 sum_t M[0,t] dL/dH_t (partial),   dU_init = gamma_0 sum_t M[0,t] dy_t xt_t^T
 * (Section 4.2.2: the accumulated gradients of the reverse recurrences at the first token, times its gate; with the rule
 * lambda_t = a ||H_t||_F the -c_t H_t terms of the Lemma are included). dH_init is the partial derivative with respect
 * to every element of H_init taken as independent, like the paper's dL/dH_t: it is not symmetrised.
 *   H_init [B,H,d,d], U_init [B,H,d,d] float32, both or neither (NULL: zero states, as gka_backward)
 *   dH_init, dU_init [B,H,d,d] float32, each written if not NULL
 *   Supported: GKA_BF16 tensors, GKA_STATE_FULL (else GKA_ERR_UNSUPPORTED); everything else as gka_backward, whose
 *   workspace query also serves this call. */
gka_status gka_backward_from_state(const gka_params *p,
                                   const void *q, const void *k, const void *v,
                                   const float *gate, const float *lambda,
                                   const void *dy,
                                   const float *H_init, const float *U_init,
                                   float *dq, float *dk, float *dv, float *dgate,
                                   float *dlambda, float *dbeta, float *dalpha,
                                   float *dH_init, float *dU_init,
                                   void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/* Forward pass with latent sketching (appendix "Latent Sketching for Approximate Solutions"): the normal equations
 * are projected into the subspace spanned by the rows of a sketch matrix S, solved there, and the solution is
 * projected back:
 *     z_t = CH(S H_t S^T + lambda_t I, S q_t, r),   xhat_t = S^T z_t,   y_t = U_t xhat_t,
 * with S H_t S^T = sum_i eta_{t,i} (S k_i)(S k_i)^T and the bounds of Section 4.1 taken in the subspace
 * (L = ||S H_t S^T||_F + lambda_t, mu = lambda_t; lambda NULL: lambda_t = p->lambda_scale ||S H_t S^T||_F). The paper
 * gives no formulas for this variant; this is the reading the library and its test oracle share. U_t is the full
 * state of Eq. (CH); sketched keys are not renormalised.
 *   S        [d_s, d_k] float32, 16-byte aligned (one sketch for all heads) or, with sketch_per_head != 0,
 *            [H, d_s, d_k]; 1 <= d_s <= 64
 *   q, k, v, o, gate, lambda, p->beta: as in gka_forward; p->alpha must be NULL
 *   Supported: GKA_BF16 tensors with GKA_COMPUTE_BF16, packed layout, zero initial states (else GKA_ERR_UNSUPPORTED;
 *   d_s out of range: GKA_ERR_SHAPE).
 *   workspace: gka_forward_sketched_workspace_bytes(p, d_s) bytes, 256-byte aligned; contents unspecified afterwards.
 * Up to d_s = 32 the solve has kernels of its own (a 32 x 32 state per chunk, every operand of a pass in registers);
 * above, it runs on the forward kernels in 64 sketched dimensions (rows of zeros are appended to S, which changes
 * nothing). The readout is a separate kernel that keeps its state in registers and, for d = 128, works in the
 * sketched space: y_t = (U_t S^T) z_t with the d_v x 32 or d_v x 64 state built from the stored sketched keys. */
size_t gka_forward_sketched_workspace_bytes(const gka_params *p, int d_s);
gka_status gka_forward_sketched(const gka_params *p,
                                const void *q, const void *k, const void *v,
                                const float *gate, const float *lambda,
                                const float *S, int d_s, int sketch_per_head,
                                void *o,
                                void *workspace, size_t workspace_bytes,
                                void *hip_stream);

const char *gka_status_string(gka_status s);

/* Library version: major * 10000 + minor * 100 + patch. */
int gka_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GKA_H_ */
