/*
 * lsm.h -- C ABI of the MI355X (gfx950) chunkwise linear-sequence-modeling library.
 *
 * The library evaluates, for every (batch, head) pair independently, the
 * unified LSM recurrence of the paper (Eq. 5) with the rank-1 update of
 * Table 1 (BLA, Lightning Attn / RetNet, Mamba2, GLA / RWKV6 / HGRN2 rows)
 *
 *     M_t = diag(a_t) M_{t-1} + k_t^T v_t ,      o_t = q_t M_t ,
 *
 * in the chunkwise-parallel form of Algorithm 2 (intra-chunk masked scores +
 * inter-chunk product with the prefix of chunk states), generalised to a
 * decay, and its backward.  q_t, k_t are 1 x d_k rows, v_t, o_t are 1 x d_v
 * rows, M is d_k x d_v.  The decay is passed as log-decay g = log a <= 0.
 * The two delta-rule rows of the same table (DeltaNet, Gated DeltaNet), whose
 * transition is not diagonal, have entry points of their own further down
 * (lsm_delta_fwd, lsm_delta_bwd, lsm_delta_step).
 *
 * Readings of the paper fixed by this ABI: o_t sees token t itself; the mask
 * of Algorithm 2 is the multiplicative 0/1 lower triangle; there is no
 * normaliser, feature map or 1/sqrt(d) scale inside the library; a vector
 * decay acts on the key dimension (rows of M); the decay of token t hits
 * M_{t-1}, the token's own k_t^T v_t enters undecayed.
 *
 * All data pointers are DEVICE pointers (HIP), 16-byte aligned, to dense
 * row-major arrays.  The caller owns every buffer; the library allocates
 * nothing, keeps nothing between calls and never synchronises: all work is
 * enqueued on `stream` and outputs are valid once the stream reaches that
 * point.  Outputs are overwritten, never accumulated; inputs are not
 * modified; outputs must not alias inputs or each other.  Results are
 * bitwise reproducible from run to run (no atomics).  Calls may be made from
 * several threads at once (the only state kept is a per-device cache that is
 * written once); the benchmark aids of lsm_bench.h are the exception and say
 * so there.
 *
 * Every argument check happens before the first HIP call, so the error
 * returns below can be exercised on a host without a GPU.
 */
#ifndef LSM_H
#define LSM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Decay coefficient kinds (Table 1, "Parameter" column). */
typedef enum {
    LSM_DECAY_NONE   = 0, /* a = 1 (BLA);                      log_decay must be NULL          */
    LSM_DECAY_HEAD   = 1, /* fixed a per head (Lightning/RetNet);   log_decay [H]              */
    LSM_DECAY_SCALAR = 2, /* a_t scalar per token (Mamba2 style);   log_decay [B,H,T]          */
    LSM_DECAY_VECTOR = 3  /* a_t in R^{d_k} per token (GLA style);  log_decay [B,H,T,d_k]      */
} lsm_decay_kind;

/* Element type of q, k, v, o, d_o, dq, dk, dv.  States, decays and their gradients are fp32. */
typedef enum { LSM_DTYPE_F32 = 0, LSM_DTYPE_BF16 = 1 } lsm_dtype;

typedef enum {
    LSM_OK              =  0,
    LSM_ERR_NULL        = -1, /* a required pointer is NULL, or a forbidden one is not           */
    LSM_ERR_SHAPE       = -2, /* non-positive dimension, struct_size mismatch, size overflow     */
    LSM_ERR_UNSUPPORTED = -3, /* d_k, d_v not in {64,128,256}; chunk_size not in {16,32,64,128};
                                 unknown decay_kind / dtype                                      */
    LSM_ERR_ALIGN       = -4, /* a pointer is not 16-byte aligned                                */
    LSM_ERR_WORKSPACE   = -5, /* workspace NULL or smaller than the *_workspace_bytes() figure   */
    LSM_ERR_LAUNCH      = -6  /* HIP reported an error when the kernels were enqueued            */
} lsm_status;

/* Memory order of q, k, v, o, d_o, dq, dk, dv and of the per-token decays and their gradient. */
typedef enum {
    LSM_LAYOUT_BHTD = 0, /* [B,H,T,d]: head-major (per-token scalar decay [B,H,T])                        */
    LSM_LAYOUT_BTHD = 1  /* [B,T,H,d]: token-major, as a fused QKV projection leaves it (decay [B,T,H])    */
} lsm_layout;

/*
 * lsm_params.flags.
 * LSM_FLAG_SAVE_STATES: the states that the forward call computes anyway are kept for the backward
 * call instead of being computed again there (the usual trade of memory for recomputation in
 * training).  Set it in the params of BOTH calls.  Contract: the two calls get the same params, the
 * same q, k, v, log_decay and init_state, and the same workspace buffer, of at least
 * lsm_chunk_fwd_workspace_bytes(p) (with the flag set, both size queries return one figure that
 * covers both calls), and nothing else writes to that buffer between them; lsm_chunk_bwd then reads
 * what lsm_chunk_fwd left there and is wrong if the buffer was touched.  What is kept: for the scalar
 * decay kinds on the matrix-core kernels the state at the start of every segment of chunks (one
 * d_k x d_v fp32 matrix per segment; nothing when a sequence is a single segment), for the vector
 * kind the per-chunk states and decayed operands.  The flag is a permission: shapes served by kernels
 * that keep nothing recompute as usual (lsm_keeps_states tells).  Both calls take the decision from
 * the params alone, so they always agree.  LSM_FLAG_SAVE_ALWAYS (only together with
 * LSM_FLAG_SAVE_STATES) is accepted for compatibility and changes nothing.
 */
typedef enum { LSM_FLAG_SAVE_STATES = 1, LSM_FLAG_SAVE_ALWAYS = 2 } lsm_flags;

typedef struct {
    uint32_t struct_size; /* = sizeof(lsm_params) */
    int32_t  B, H, T;     /* batch, heads, tokens per sequence (any T >= 1; the last chunk may be ragged) */
    int32_t  d_k, d_v;    /* key / value head dimensions                                         */
    int32_t  chunk_size;  /* C: tokens per chunk of Algorithm 2 (size of the quadratic block)    */
    int32_t  decay_kind;  /* lsm_decay_kind                                                      */
    int32_t  dtype;       /* lsm_dtype                                                           */
    int32_t  layout;      /* lsm_layout                                                          */
    /*
     * Packed variable-length input (the paper's handling of batches of unequal sequences: one
     * continuous token axis, the state starting afresh at every sequence boundary).  n_seq = 0: B
     * sequences of T tokens each.  n_seq > 0: B must be 1, T is the total token count and
     * cu_seqlens (DEVICE pointer, n_seq + 1 ints, 16-byte aligned) holds the first token of each
     * sequence, cu_seqlens[0] = 0 <= ... <= cu_seqlens[n_seq] = T (content not checked).  Every
     * sequence is chunked on its own, so no chunk straddles a boundary; init_state, final_state and
     * their gradients are then [n_seq,H,d_k,d_v].  The result equals n_seq separate calls.
     */
    int32_t  n_seq;
    int32_t  flags;       /* bitwise OR of lsm_flags; 0 = none                                   */
    const int32_t* cu_seqlens;
} lsm_params;

/*
 * Forward (Algorithm 2 with decay; Eq. 5; Table 1).
 *   q, k        [B,H,T,d_k]  dtype          in      (shapes as written are for LSM_LAYOUT_BHTD; with
 *   v           [B,H,T,d_v]  dtype          in       LSM_LAYOUT_BTHD the H and T axes of q, k, v, o and of
 *   log_decay   per decay_kind, fp32, finite and <= 0 (not checked)      in      the per-token decays swap)
 *   init_state  NULL (= zeros) or [B,H,d_k,d_v] fp32: M_0                in      ([n_seq,H,d_k,d_v] for packed input,
 *   o           [B,H,T,d_v]  dtype          out                                   as are the other three states)
 *   final_state NULL (not wanted) or [B,H,d_k,d_v] fp32: M_T             out
 *   workspace   device scratch of at least lsm_chunk_fwd_workspace_bytes(p); contents undefined after the call
 *   stream      hipStream_t, NULL = the default stream
 * Returns an lsm_status.  On any error nothing has been enqueued, except for
 * LSM_ERR_LAUNCH, where earlier kernels of the call may have been.
 */
int lsm_chunk_fwd(const lsm_params* p,
                  const void* q, const void* k, const void* v,
                  const float* log_decay, const float* init_state,
                  void* o, float* final_state,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * lsm_chunk_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels and
 * results as lsm_chunk_fwd, minus the workspace: the scratch (segment entry states, decay tables, the
 * chunk table of a packed input) lives in a device array built into the library, LSM_NOALLOC_SCRATCH_BYTES
 * per GPU, held from the first call on that GPU until the process ends.  Parameter sets whose
 * lsm_chunk_fwd_workspace_bytes(p) exceeds that size are rejected with LSM_ERR_WORKSPACE before anything
 * is enqueued.  The call allocates and frees nothing.  All calls on one GPU share the one array, which
 * keeps the previous call's contents (nothing in it has to start at zero): calls that overlap on one GPU,
 * on different streams or from different threads, race - serialise them.  LSM_FLAG_SAVE_STATES has no
 * meaning here (there is no workspace to hand to lsm_chunk_bwd); leave flags at 0.
 */
#define LSM_NOALLOC_SCRATCH_BYTES (8u << 20)
int lsm_chunk_fwd_noalloc(const lsm_params* p,
                          const void* q, const void* k, const void* v,
                          const float* log_decay, const float* init_state,
                          void* o, float* final_state, void* stream);

/*
 * Forward of the two delta-rule rows of Table 1 under Eq. 5, chunkwise:
 *     M_t = alpha_t (I - beta_t k_t^T k_t) M_{t-1} + b_t k_t^T v_t ,    o_t = q_t M_t
 * DeltaNet:        alpha = 1 (log_alpha NULL, decay_kind LSM_DECAY_NONE), beta = the row's a_t, b = the row's b_t;
 * Gated DeltaNet:  alpha = the row's a_t (log_alpha = log a_t <= 0, decay_kind LSM_DECAY_SCALAR), beta NULL (= 1).
 *   q, k, v, init_state, o, final_state   as in lsm_chunk_fwd (both layouts)
 *   log_alpha, beta, b   fp32 per token, [B,H,T] ([B,T,H] with LSM_LAYOUT_BTHD); NULL = the constant 1        in
 *   workspace            at least lsm_delta_fwd_workspace_bytes(p); contents undefined after the call
 * Served for bf16 elements, d_k = d_v = 128, chunk_size 64 (packed variable-length input included, as for
 * lsm_chunk_fwd); everything else returns LSM_ERR_UNSUPPORTED (the workspace query then returns 0).  LSM_FLAG_SAVE_STATES (in the params of both calls, same
 * contract as for lsm_chunk_fwd / lsm_chunk_bwd: same inputs, same workspace of lsm_delta_fwd_workspace_bytes(p) =
 * lsm_delta_bwd_workspace_bytes(p) bytes, untouched in between): the forward call leaves the chunks' triangular
 * inverses and pseudo-values in the workspace and lsm_delta_bwd does not compute them again.  Keys are expected to have
 * at most unit length times sqrt(2 / beta) (the erase factor is then a contraction); nothing is checked.
 * With fewer than about 200 sequences each is cut into segments that run in parallel (at the price of a summary pass).
 */
size_t lsm_delta_fwd_workspace_bytes(const lsm_params* p);
int lsm_delta_fwd(const lsm_params* p,
                  const void* q, const void* k, const void* v,
                  const float* log_alpha, const float* beta, const float* b,
                  const float* init_state,
                  void* o, float* final_state,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * One recurrent step of the delta-rule rows (decoding), for every (b,h):
 *     state <- alpha (I - beta k^T k) state + b k^T v ,      o = q state .
 *   q, k [B,H,d_k], v, o [B,H,d_v] in dtype; log_alpha, beta, b: [B,H] fp32 or NULL (= 1; log_alpha exactly when
 *   decay_kind is LSM_DECAY_SCALAR); state [B,H,d_k,d_v] fp32, updated in place.
 * Both element types, d_k and d_v in {64,128,256}; p->T and p->chunk_size are not used (pass T = 1).  No workspace.
 * T calls from init_state give the o and final_state of lsm_delta_fwd over the same T tokens, up to rounding.
 */
int lsm_delta_step(const lsm_params* p,
                   const void* q, const void* k, const void* v,
                   const float* log_alpha, const float* beta, const float* b,
                   float* state, void* o, void* stream);

/*
 * Backward of lsm_delta_fwd for  L = <o, d_o> + <M_T, d_final_state>  (the adjoint of the recurrence above,
 * evaluated chunkwise; nothing saved by the forward call is needed).
 *   q, k, v, log_alpha, beta, b, init_state   as in lsm_delta_fwd                                   in
 *   d_o            like o;  d_final_state NULL (= zeros) or [B,H,d_k,d_v] fp32                       in
 *   dq, dk, dv     like q, k, v                                                                     out
 *   d_log_alpha, d_beta, d_b   fp32 per token like the parameter; required exactly where the parameter was given,
 *                  NULL where it was NULL                                                            out
 *   d_init_state   NULL (not wanted) or [B,H,d_k,d_v] fp32                                           out
 *   workspace      at least lsm_delta_bwd_workspace_bytes(p)
 * Same shapes served and same error behaviour as lsm_delta_fwd.
 */
size_t lsm_delta_bwd_workspace_bytes(const lsm_params* p);
int lsm_delta_bwd(const lsm_params* p,
                  const void* q, const void* k, const void* v,
                  const float* log_alpha, const float* beta, const float* b,
                  const float* init_state,
                  const void* d_o, const float* d_final_state,
                  void* dq, void* dk, void* dv,
                  float* d_log_alpha, float* d_beta, float* d_b, float* d_init_state,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of  L = <o, d_o> + <M_T, d_final_state>  (the paper states no
 * backward; it is the adjoint of the forward above, evaluated chunkwise with a
 * reverse scan over chunk-state gradients).  The forward's states that the
 * gradients need are recomputed from the inputs; nothing saved by the forward
 * call is needed (unless LSM_FLAG_SAVE_STATES is set, see lsm_flags).
 * Shapes outside the matrix-core family (lsm_kernel_path(p) == 0: fp32
 * elements, d_k other than 128, d_v = 64, chunk other than 64) run on plain
 * fp32 kernels that are correct to the fp32 tolerance and far slower; they are
 * meant for checks and odd shapes.  (d_v = 256 is in the family: the vector
 * kind scans each 128-wide value slice, the other kinds run one pass per slice
 * and keep no states between the two calls, whatever the flags say.)
 *   q,k,v,log_decay,init_state   as in the forward                         in
 *   d_o            [B,H,T,d_v] dtype                                       in
 *   d_final_state  NULL (= zeros) or [B,H,d_k,d_v] fp32                    in
 *   dq, dk         [B,H,T,d_k] dtype;  dv [B,H,T,d_v] dtype                out
 *   d_log_decay    shape of log_decay, fp32.  Must be NULL for LSM_DECAY_NONE;
 *                  for the other kinds NULL skips it                       out
 *   d_init_state   NULL (not wanted) or [B,H,d_k,d_v] fp32                 out
 */
int lsm_chunk_bwd(const lsm_params* p,
                  const void* q, const void* k, const void* v,
                  const float* log_decay, const float* init_state,
                  const void* d_o, const float* d_final_state,
                  void* dq, void* dk, void* dv,
                  float* d_log_decay, float* d_init_state,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * One recurrent step, the constant-memory form of the same recurrence used for decoding (Eq. 5 with the
 * rank-1 update of Table 1, one token):  for every (b,h)
 *     state <- diag(a) state + k^T v ,      o = q state .
 *   q, k        [B,H,d_k]  dtype          in
 *   v           [B,H,d_v]  dtype          in
 *   log_decay   NONE: NULL;  HEAD: [H];  SCALAR: [B,H];  VECTOR: [B,H,d_k];  fp32, <= 0      in
 *   state       [B,H,d_k,d_v] fp32, updated in place                                          in/out
 *   o           [B,H,d_v]  dtype          out
 * p->T and p->chunk_size are not used (they must still be valid; pass T = 1).  No workspace.  T calls of
 * lsm_step from init_state give the o and final_state of lsm_chunk_fwd over the same T tokens, up to rounding.
 */
int lsm_step(const lsm_params* p,
             const void* q, const void* k, const void* v, const float* log_decay,
             float* state, void* o, void* stream);

/* Scratch the calls above need, in bytes; 0 if *p is invalid.  Host-only, no HIP call. */
size_t lsm_chunk_fwd_workspace_bytes(const lsm_params* p);
size_t lsm_chunk_bwd_workspace_bytes(const lsm_params* p);

/*
 * Which kernel family a parameter set is routed to: 1 = bf16 MFMA kernels,
 * 0 = generic fp32-arithmetic kernels, negative = lsm_status of invalid params.
 * Host-only.  (Both families run on the GPU; there is no CPU fallback.)
 */
int lsm_kernel_path(const lsm_params* p);

/* 1 if, for these params, lsm_chunk_fwd keeps its chunk states for lsm_chunk_bwd (see lsm_flags), 0 if the
 * backward call recomputes them, a negative lsm_status for invalid params. */
int lsm_keeps_states(const lsm_params* p);

/* Static, NUL-terminated description of a status code. */
const char* lsm_status_string(int status);

/* ABI version, bumped when a signature or struct changes (2: layout and packed input in lsm_params; 3: flags; 4: workspace query of the benchmark aid; 5: lsm_chunk_fwd_noalloc). */
int lsm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LSM_H */
