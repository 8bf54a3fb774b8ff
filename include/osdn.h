/*
 * libosdn -- OSDN hot path on one AMD MI355X (gfx950): the chunkwise-parallel gated
 * delta-rule recurrence whose write-side key is rescaled per feature by an online
 * diagonal preconditioner, forward and backward.
 *
 * What is computed (paper: "OSDN: Improving Delta Rule with Provable Online
 * Preconditioning in Linear Attention"), per batch b and head h independently, for
 * t = 1..T, with S in R^{V x K}, d in R^K:
 *
 *   phase 1 (Algorithm 1; Eq. (dt_update), with retention Eq. (dt_update_apf)):
 *       k~_t = d_t (.) k_t
 *       s = k_t (.) k_t,  n = max(sum s, eps),  p = <d_t, s>,  b' = beta_t (or 1 if !beta_aware)
 *       d_{t+1} = clip( r_t d_t + eta b' (1 - b' p)/n * s , d_min, d_max )
 *   phase 2 (Eq. (equiv_update)/(recurrent_form), gated as in Appendix B.1):
 *       S_t = alpha_t S_{t-1} + beta_t (v_t - alpha_t S_{t-1} k_t) k~_t^T ,  alpha_t = exp(log_alpha_t)
 *       o_t = scale * S_t q_t
 *
 * The library evaluates phase 2 in the chunkwise WY/UT form (Appendix A.2, B.1) with
 * chunk length 64; results equal the recurrence up to floating-point reassociation.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; tensors are contiguous,
 *     row-major, in the stated layout.  Inputs are never written; outputs must not alias
 *     inputs or each other.  Optional pointers may be NULL where stated.
 *   - q, k, v, o, dO, dq, dk, dv, k_tilde have element type params->io_dtype (fp32 or
 *     bf16).  beta, log_alpha, retention, every d and every S (and their gradients) are
 *     always fp32: the recurrent state and the preconditioner are kept in fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return without synchronising.
 *   - Return value: OSDN_OK (0) or a negative osdn_status.  On an argument error nothing
 *     is launched.  osdn_strerror() gives a static description.
 *   - The library allocates no device memory: scratch comes from the caller's `workspace`
 *     (256-byte aligned, at least osdn_workspace_bytes()).  It reads no environment variables.
 *     Process-wide state: the optional profiling switch at the end of this file and, created on
 *     first use and kept until the process ends, one side stream with a few events per
 *     (device, caller stream): osdn_fwd / osdn_bwd run the preconditioner phase on it, forked
 *     from and joined back into `stream` with events, so that to the caller all work still is
 *     ordered as if enqueued on `stream` (also under stream capture: the side stream joins the
 *     capture and leaves it inside the call).  Calls on different streams share nothing; calls
 *     that share one stream must be issued one after the other, as any work on one stream.
 *     params->segments = 1 keeps everything on `stream`.
 *     With at most 32 (batch, head) chains of at least 64 chunks, osdn_fwd computes the
 *     preconditioner as a few sweeps over pieces of the sequence that run side by side, all on
 *     `stream` (same results to the tolerance of the sweeps, 1e-6 relative; params->p1_pieces = -1
 *     keeps the one sequential sweep per chain).
 *   - retention values are assumed >= 0 (they are sigmoid gates in the paper).  Wherever a
 *     signature says retention / dretention [B,T,H], params->retention_per_channel = 1 makes
 *     it [B,T,H,K]: one value per coordinate.  Likewise params->gate_per_channel = 1 makes
 *     log_alpha / dlog_alpha [B,T,H,K]: one state gate per key channel, S <- S Diag(alpha_t)
 *     (online-scaled KDA, appendix section on Kimi Delta Attention with online scaling).
 *   - Supported shapes: chunk == 64; any T >= 1 (osdn_fwd/osdn_bwd pad a ragged last chunk
 *     inside the workspace with tokens that change nothing; osdn_precond_update needs
 *     T % 64 == 0 only when d_ckpt is asked for; 1 <= T <= 64 for osdn_step); K in {64, 128}
 *     (K = 256 is not built: the [64 x K] operand tiles of the chain and backward kernels would
 *     no longer fit the 160 KB of LDS next to each other); V a multiple of 64 up to 512; B, H >= 1 with H * max(K, V) < 2^24 (the 64 token rows of
 *     a chunk are addressed with 32-bit byte offsets).  Anything else returns OSDN_ERR_SHAPE.
 */
#ifndef OSDN_H
#define OSDN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { OSDN_F32 = 0, OSDN_BF16 = 1 } osdn_dtype;

typedef enum {
    OSDN_OK = 0,
    OSDN_ERR_NULL = -1,       /* a required pointer is NULL */
    OSDN_ERR_SHAPE = -2,      /* unsupported B/T/H/K/V/chunk */
    OSDN_ERR_DTYPE = -3,      /* io_dtype is neither OSDN_F32 nor OSDN_BF16 */
    OSDN_ERR_WORKSPACE = -4,  /* workspace too small or not 256-byte aligned */
    OSDN_ERR_PARAM = -5,      /* eta < 0, eps <= 0, or a non-finite scalar */
    OSDN_ERR_LAUNCH = -6      /* the HIP runtime reported a launch error */
} osdn_status;

typedef struct {
    int32_t B, T, H, K, V, chunk;   /* chunk must be 64 */
    int32_t io_dtype;               /* osdn_dtype */
    float scale;                    /* multiplies q in the read-out (Listing 1: K^-0.5) */
    float eta;                      /* online step size of the d update (paper: 0.003) */
    float d_min, d_max;             /* box of the projection (paper: 0.5, 2.0); d_min > d_max => none */
    float eps;                      /* floor of the squared key norm (Listing 1: 1e-6) */
    int32_t beta_aware;             /* 1: beta enters the d update (default); 0: replaced by 1 there */
    int32_t retention_per_channel;  /* 0: retention is one gate per (token, head), [B,T,H] (Section 4.4);
                                       1: one per coordinate, [B,T,H,K], diag(r_t) in place of r_t I (the
                                       vector-retention extension stated with the proposition that APF is a
                                       piecewise-affine recurrence); dretention then has that shape too */
    int32_t gate_per_channel;       /* 0: log_alpha is one state gate per (token, head), [B,T,H];
                                       1: one per key channel, [B,T,H,K]: S <- S Diag(alpha_t), the
                                       online-scaled KDA recurrence (appendix section on Kimi Delta
                                       Attention with online scaling; its K x V state is the transpose
                                       of the [V,K] state kept here); dlog_alpha then has that shape
                                       too and log_alpha must not be NULL.  In the chunkwise entry
                                       points the cumulative log-decay of a channel inside a chunk
                                       of 64 tokens has to stay above about -80 */
    /* Scheduling knobs; 0 everywhere = the library decides (what the benchmarks use).  They change
       how the work is cut, not what is computed (p1_pieces: to the sweeps' tolerance, see above). */
    int32_t segments;               /* > 0: cut the sequence into this many segments of chunks for the
                                       two-stream pipeline of osdn_fwd / osdn_bwd (1: one stream) */
    int32_t p1_pieces;              /* > 0: osdn_fwd runs the preconditioner as sweeps over this many
                                       pieces per chain; -1: never (always the sequential sweep) */
    int32_t p1_piece_sweeps;        /* > 0: at most this many such sweeps (up to 13) before the sequential
                                       sweep finishes the chains that have not settled */
    int32_t p1_solved;              /* osdn_bwd: 1: the reverse sweep takes chunks in solved form (a 64 x 64
                                       triangular system per chunk, inverted for all chunks side by side):
                                       without retention the chunks in which no coordinate met the box, with
                                       one retention value per (token, head) every chunk; -1: never; 0: the
                                       library decides (only ever without retention) */
} osdn_params;

/* Bytes of scratch osdn_fwd needs (for_backward == 0) or osdn_fwd followed by osdn_bwd
 * needs (for_backward != 0).  Returns 0 if the parameters are invalid. */
size_t osdn_workspace_bytes(const osdn_params *p, int for_backward);

const char *osdn_strerror(int status);

/*
 * Phase 1 alone (Algorithm 1 / Eq. (dt_update_apf)); also the preconditioner half of a
 * streaming decode step (T may be 1).
 *   k         [B,T,H,K] io_dtype   keys (read side)
 *   beta      [B,T,H]   fp32
 *   retention [B,T,H]   fp32 or NULL (=> r = 1)
 *   d_in      [B,H,K]   fp32 or NULL (=> ones); not projected on entry
 *   k_tilde   [B,T,H,K] io_dtype   out: d_t (.) k_t, rounded once from fp32
 *   d_out     [B,H,K]   fp32       out: d after the last token
 *   d_ckpt    [B,H,T/64,K] fp32 or NULL   out: d at the start of every chunk (needs T % 64 == 0)
 */
int osdn_precond_update(const osdn_params *p, const void *k, const float *beta,
                        const float *retention, const float *d_in, void *k_tilde, float *d_out,
                        float *d_ckpt, void *stream);

/*
 * The same map as osdn_fwd in its recurrent form, for short inputs: the decode step of
 * Appendix K (state gate, rank-one write with the scaled key, read, then the preconditioner
 * update with its projection), token by token for 1 <= T <= 64 tokens in one launch, the state
 * in registers and fp32 throughout (k~ is not rounded to io_dtype here).  No workspace.
 *   q, k      [B,T,H,K] io_dtype ;  v [B,T,H,V] io_dtype
 *   beta      [B,T,H] fp32 ;  log_alpha, retention [B,T,H] fp32 or NULL
 *   d_in      [B,H,K] fp32 or NULL (=> ones) ;  S_in [B,H,V,K] fp32 or NULL (=> zeros)
 *   o         [B,T,H,V] io_dtype  out
 *   S_out     [B,H,V,K] fp32      out; MAY be the same buffer as S_in (updated in place)
 *   d_out     [B,H,K]   fp32      out; must NOT be d_in (OSDN_ERR_NULL if it is)
 * T > 64 returns OSDN_ERR_SHAPE (use osdn_fwd); params->chunk is still required to be 64.
 */
int osdn_step(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
              const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
              void *o, float *S_out, float *d_out, void *stream);

/*
 * Forward (both phases).
 *   q, k      [B,T,H,K] io_dtype ;  v [B,T,H,V] io_dtype
 *   beta      [B,T,H] fp32 ; log_alpha [B,T,H] fp32 (<= 0) or NULL (=> ungated, alpha = 1)
 *   retention, d_in as above ;  S_in [B,H,V,K] fp32 or NULL (=> zeros)
 *   o         [B,T,H,V] io_dtype  out
 *   S_out     [B,H,V,K] fp32      out: state after the last token
 *   d_out     [B,H,K]   fp32      out
 *   workspace: scratch; when osdn_bwd follows, pass the same buffer, untouched, to it.
 *     What only a backward pass reads (the chunks' (I + A)^-1 and intra-chunk scores) is written
 *     iff workspace_bytes >= osdn_workspace_bytes(p, 1); osdn_bwd rejects a smaller workspace, so a
 *     forward call that is to be followed by osdn_bwd must already be given the larger size.
 */
int osdn_fwd(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             void *o, float *S_out, float *d_out, void *workspace, size_t workspace_bytes,
             void *stream);

/*
 * osdn_fwd for callers that cannot allocate device memory and have no workspace to hand in
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * same computation with the scratch taken from a fixed device array that is part of the
 * library, OSDN_NOALLOC_MAX_WORKSPACE bytes, which every GPU the library is used on holds from
 * the moment the library is loaded until the process ends.  The call allocates nothing, creates
 * no stream or event, and runs entirely on `stream`; all other arguments are those of osdn_fwd.
 *   - Problems whose osdn_workspace_bytes(p, 0) exceeds OSDN_NOALLOC_MAX_WORKSPACE return
 *     OSDN_ERR_WORKSPACE and launch nothing; if the array's address cannot be obtained,
 *     OSDN_ERR_LAUNCH.
 *   - All calls on one GPU share that GPU's array: calls that may overlap in time (different
 *     streams, different threads) race on it and must be ordered by the caller.  Nothing in it
 *     has to start at zero (every buffer is written before it is read), so what the previous
 *     call left behind is harmless.
 *   - The scratch is not a workspace for osdn_bwd: use osdn_fwd with a caller workspace when a
 *     backward pass follows.
 */
#define OSDN_NOALLOC_MAX_WORKSPACE ((size_t)64 << 20)
int osdn_fwd_noalloc(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
                     const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
                     void *o, float *S_out, float *d_out, void *stream);

/*
 * Backward of osdn_fwd (Section 4.5: phase 2 yields dL/dk~; dL/dd_t = k_t (.) dL/dk~_t,
 * dL/dk_t += d_t (.) dL/dk~_t; reverse sweep through the projected affine d recurrence,
 * whose projection passes gradient where d_min <= unprojected value <= d_max).
 *   forward inputs exactly as given to osdn_fwd, and the workspace it filled
 *   dO        [B,T,H,V] io_dtype   gradient of o
 *   dS_out    [B,H,V,K] fp32 or NULL (=> 0)   gradient of S_out
 *   dd_out    [B,H,K]   fp32 or NULL (=> 0)   gradient of d_out
 *   dq, dk    [B,T,H,K] io_dtype out ; dv [B,T,H,V] io_dtype out
 *   dbeta     [B,T,H] fp32 out ; dlog_alpha [B,T,H] fp32 out (may be NULL iff log_alpha is)
 *   dretention [B,T,H] fp32 out (may be NULL iff retention is)
 *   dd_in     [B,H,K] fp32 out ; dS_in [B,H,V,K] fp32 out
 */
int osdn_bwd(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             const void *dO, const float *dS_out, const float *dd_out, void *dq, void *dk, void *dv,
             float *dbeta, float *dlog_alpha, float *dretention, float *dd_in, float *dS_in,
             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Packed sequences (the training set-up in the appendix on training and evaluation details,
 * paragraph on optimizer, batch and precision: one long token axis per device that holds
 * variable-length segments back to back, their boundaries in cu_seqlens, the recurrent state
 * reset at every boundary).  The _packed entry points are osdn_fwd / osdn_bwd for that input:
 *   params->B must be 1 and params->T the total number of tokens;
 *   cu_seqlens  HOST pointer to n_seqs + 1 ascending int32 token offsets, cu_seqlens[0] = 0,
 *               cu_seqlens[n_seqs] = T; sequence s is the tokens [cu_seqlens[s], cu_seqlens[s+1]);
 *               read before the call returns (it need not outlive the call); every sequence
 *               has at least one token, else OSDN_ERR_SHAPE;
 *   token tensors (q, k, v, beta, log_alpha, retention, o, dO and the token gradients) are
 *               [1,T,H,*] as before;
 *   carried tensors have one entry per sequence: d_in, d_out, dd_out, dd_in are [n_seqs,H,K];
 *               S_in, S_out, dS_out, dS_in are [n_seqs,H,V,K].  Every sequence starts from its own
 *               d_in / S_in entry (NULL => ones / zeros: the reset) and leaves its own final
 *               d and S; no state crosses a boundary.
 * Sequences need not be whole chunks: inside the workspace each sequence is moved to start on
 * a chunk boundary and padded with tokens that change nothing (no copies are made when every
 * length is a multiple of 64).  The sequential kernels run one chain per (sequence, head).
 * osdn_workspace_bytes_packed sizes the workspace for exactly this cu_seqlens (0 on invalid
 * arguments); osdn_bwd_packed takes the same cu_seqlens and the workspace osdn_fwd_packed filled.
 */
size_t osdn_workspace_bytes_packed(const osdn_params *p, const int32_t *cu_seqlens, int32_t n_seqs,
                                   int for_backward);

int osdn_fwd_packed(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
                    const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
                    void *o, float *S_out, float *d_out, const int32_t *cu_seqlens, int32_t n_seqs,
                    void *workspace, size_t workspace_bytes, void *stream);

int osdn_bwd_packed(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
                    const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
                    const void *dO, const float *dS_out, const float *dd_out, void *dq, void *dk, void *dv,
                    float *dbeta, float *dlog_alpha, float *dretention, float *dd_in, float *dS_in,
                    const int32_t *cu_seqlens, int32_t n_seqs, void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * Diagnostic query for tests: the decisions of the projection's derivative (Section 4.5,
 * reverse sweep through the projected affine recurrence) that osdn_bwd took, as it left them
 * in the workspace.  Returns the byte offset, inside a workspace of a plain (not packed) batch
 * that osdn_bwd has processed, of an array [B, H, ceil(T/64), K] of 64-bit words (low 32 bits
 * first): bit i of word (b, h, n, c) is set iff the unprojected update of coordinate c at
 * token 64 n + i landed inside the box [d_min, d_max], faces included.  Bits of tokens past T
 * are unspecified; with d_min > d_max (no projection) the array is not written.  Returns 0 for
 * invalid parameters.  Host-only: launches nothing.
 */
size_t osdn_debug_mask_offset(const osdn_params *p);

/*
 * Optional per-kernel timing (for benchmarks; off by default; not thread-safe -- this switch
 * and its event list are the only process-wide state of the library).  While enabled, every
 * kernel an entry point launches is bracketed by a pair of HIP events on the caller's stream.
 * osdn_profile_read() waits for the recorded events, returns for each kernel id the summed
 * duration in milliseconds and the number of launches since the previous read (arrays of
 * n >= osdn_profile_kernel_count() host elements), and forgets them.
 */
void osdn_profile_enable(int on);
int osdn_profile_kernel_count(void);
const char *osdn_profile_kernel_name(int id);
int osdn_profile_read(double *ms_sum, int *launches, int n);

#ifdef __cplusplus
}
#endif
#endif /* OSDN_H */
