// Argument blocks and launchers of the OSDN kernels (internal to the library).
#pragma once
#include "osdn_device.h"

namespace osdn {

// Every kernel works on the chunks [n0, n1) of the sequence (all of them in one launch, or a
// segment when the two phases are pipelined against each other); what a sequential kernel
// carries across a segment boundary (d, S, dS, the adjoint of d) goes through the same
// buffers that hold it at the ends of the sequence.
//
// Packed sequences (seq_chunks != null): the token axis holds n_seqs sequences one after the
// other, each starting on a chunk boundary; sequence s owns the chunks
// [seq_chunks[s], seq_chunks[s+1]).  The token tensors and per-chunk buffers then have one
// batch entry, the carried tensors (d, S and their adjoints) one entry per sequence, and the
// sequential kernels run one chain per (sequence, head).  A chain takes its start value from
// the *_first / *_last pointer when its sequence begins (ends, in the backward pass) inside
// [n0, n1), and from the carry buffer otherwise.
struct PrecondArgs {
    int B, T, H, K;
    int n0, n1;
    int n_seqs;               // 0: plain batch
    const int *seq_chunks;    // [n_seqs + 1] or null
    const float *d_first;     // packed sequences: d before the first token, [n_seqs,H,K] or null
    float eta, d_min, d_max, eps;
    int beta_aware;
    const void *k;            // [B,T,H,K] io
    const float *beta;        // [B,T,H]
    const float *retention;   // [B,T,H] ([B,T,H,K] with ret_vec) or null
    int ret_vec;              // one retention per coordinate
    const float *d_in;        // [B,H,K] or null
    void *k_tilde;            // [B,T,H,K] io
    float *d_out;             // [B,H,K]
    float *d_ckpt;            // [B,H,T/64,K] or null
    float *tok_scalars;       // [B,T,H,4] or null: per token (step, <d,k^2>, sum k^2, unused), kept for the backward
    // Sweeps over the whole sequence (pieces > 0, plain batches only): a chain is cut into
    // pieces of piece_chunks chunks, one workgroup per piece.  Sweep number `sweep` reads the
    // start values and piece maps x -> clip3(A x + B, L, H) that sweep - 1 left (two buffers
    // each, used in turn) and returns at once for a chain whose start values no longer move.
    int pieces, piece_chunks, sweep;
    float *piece_start;       // [2][B*H*pieces, K]
    float4 *piece_map;        // [2][B*H*pieces, K]  (A, B, L, H)
    int *settled;             // [B*H] or null: a chain whose entry is set is left alone
};

struct PrecondBwdArgs {
    int B, T, H, K;
    int n0, n1;
    int n_seqs;
    const int *seq_chunks;
    const float *dd_last;     // packed sequences: adjoint of the final d, [n_seqs,H,K] or null
    float eta, d_min, d_max, eps;
    int beta_aware;
    const void *k;
    const float *beta, *retention, *d_ckpt;     // retention [B,T,H], or [B,T,H,K] with ret_vec
    int ret_vec;
    float *tok_scalars;       // [B,T,H,4] from the forward sweep: (step, <d,k^2>, sum k^2, -); the chain
                              // kernel puts sigma_t into the fourth slot for the post kernel
    uint2 *masks;             // [B,H,T/64,K]: bit i = token i of the chunk stayed inside the box
    float *a_ckpt;            // [B,H,T/64,K]: adjoint of d at the right end of every chunk
    const void *dkt;          // [B,T,H,K] io: dL/dk~ from phase 2
    const void *dk_read;      // [B,T,H,K] io: read-side dL/dk from phase 2
    const float *dd_out;      // [B,H,K] or null
    void *dk;                 // [B,T,H,K] io
    float *dbeta;             // [B,T,H] in/out
    float *dretention;        // [B,T,H] ([B,T,H,K] with ret_vec) or null
    float *dd_in;             // [B,H,K]
    // chunks in solved form (no retention; null: never): per chunk, whether it qualifies (no
    // coordinate met the box), the inverse (I + U)^-1, rho0 and the chunk's sum of lambda
    int *lin_clean;           // [B,H,T/64]
    void *lin_M;              // [B,H,T/64,64,64] io
    float *lin_r0;            // [B,H,T/64,64]
    float *lin_t0;            // [B,H,T/64,K]
    unsigned char *lin_aux;   // [B,H,T/64,2048]: with a retention gate, the indicators and retention products of the chunk
};

// The recurrent step (decode): state in registers, 1..64 tokens per launch.
struct StepArgs {
    int B, T, H, K, V;
    float scale, eta, d_min, d_max, eps;
    int beta_aware;
    const void *q, *k, *v;            // [B,T,H,*] io
    const float *beta, *log_alpha, *retention;   // [B,T,H]; log_alpha, retention may be null;
    int ret_vec;                      // retention is [B,T,H,K]: one value per coordinate
    int gate_vec;                     // log_alpha is [B,T,H,K]: one state gate per key channel
    const float *d_in, *S_in;         // [B,H,K], [B,H,V,K]; may be null (ones / zeros)
    void *o;                          // [B,T,H,V] io
    float *S_out, *d_out;             // S_out may be S_in (a workgroup reads its rows before it writes them)
};

// Everything the chunkwise (phase 2) kernels need.  Per-chunk tiles live in the workspace
// in [B,H,N,rows,cols] order (one contiguous tile per chunk and head).
struct ChunkArgs {
    int B, T, H, K, V, N;
    int n0, n1;
    int n_seqs;
    const int *seq_chunks;
    const float *S_first;             // packed sequences: [n_seqs,H,V,K] or null
    const float *dS_last;             // packed sequences: adjoint of the final S, or null
    float scale;
    // caller tensors
    const void *q, *k, *v;            // [B,T,H,*] io
    const float *beta, *log_alpha;    // [B,T,H]; log_alpha may be null
    const float *S_in;                // [B,H,V,K] or null
    void *o;                          // [B,T,H,V] io
    float *S_out;                     // [B,H,V,K]
    // workspace (forward)
    void *kt;                         // [B,T,H,K] io      k~
    void *Tm;                         // [B,H,N,64,64] io  (I + A)^-1
    void *Wt;                         // [B,H,N,K,64] io   -W^T
    void *Ktr;                        // [B,H,N,K,64] io   (rho . K~)^T
    void *Ut;                         // [B,H,N,V,64] io   U^T
    void *Et;                         // [B,H,N,V,64] io   E transposed
    void *S_ckpt;                     // [B,H,N,V,K] io    state at the start of each chunk (null: not kept)
    void *Pm;                         // [B,H,N,64,64] io  P = tril(Gamma . Q K~^T), from output_fwd for the backward
                                      //                   chain (null: not kept; Tm may be null likewise)
    int narrow_slices;                // chain kernels: 16 rows of the state per workgroup instead of 32
    // one state gate per key channel (gate_vec: log_alpha is [B,T,H,K]; forward only): chunk_prep
    // folds the cumulative channel decays Gamma into the operands and leaves
    int gate_vec;
    void *Qg;                         // [B,T,H,K] io      Gamma . Q
    void *Kg;                         // [B,T,H,K] io      Gamma . K
    void *Kd;                         // [B,T,H,K] io      K~ / Gamma
    float *gamC;                      // [B,H,N,K] f32     decay of every channel over the whole chunk
    float *dgamC;                     // [B,H,N,K] f32     backward: dL/d(that decay)
    // backward
    const void *dO;                   // [B,T,H,V] io
    const float *dS_out;              // [B,H,V,K] or null
    void *dEt;                        // [B,H,N,V,64] io   dE transposed (complete)
    void *dS_ckpt;                    // [B,H,N,V,K] io    adjoint of the state at the END of each chunk
    float *dS_in;                     // [B,H,V,K]
    void *dq, *dv;                    // io
    void *dk_read, *dkt;              // [B,T,H,K] io: the two parts of dL/dk that phase 1 combines
    float *dbeta, *dlog_alpha;        // [B,T,H]; dlog_alpha may be null
};

int launch_precond_fwd(const PrecondArgs &a, bool bf16_io, hipStream_t st);
int launch_step(const StepArgs &a, bool bf16_io, hipStream_t st);
int launch_copy_rows(const void *src, int Ts, void *dst, int Td, int B, size_t row_bytes, uint32_t fill,
                     hipStream_t st);
int launch_upload_ints(const int *host, size_t count, int *dst, hipStream_t st);
int launch_move_chunk_rows(const void *src, void *dst, const int *chunk_row, const int *chunk_len, int n_chunks,
                           size_t row_bytes, bool to_padded, uint32_t fill, hipStream_t st);
int launch_precond_mask(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st);
// solved form with a retention gate per (token, head): which = 0 masks, inverse and indicators (forward
// data only), 1 rho0 and t0 (needs dL/dk~), 2 the chain; chunks [n0, n1)
int launch_precond_gen(const PrecondBwdArgs &a, bool bf16_io, int which, hipStream_t st);
int launch_precond_lin_bwd(const PrecondBwdArgs &a, bool bf16_io, bool m_part, hipStream_t st);
int launch_precond_chain(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st);
int launch_precond_post(const PrecondBwdArgs &a, bool bf16_io, hipStream_t st);
int launch_chunk_prep(const ChunkArgs &a, bool bf16_io, hipStream_t st);
int launch_state_fwd(const ChunkArgs &a, bool bf16_io, hipStream_t st);
int launch_output_fwd(const ChunkArgs &a, bool bf16_io, hipStream_t st);
int launch_bwd_chain(const ChunkArgs &a, bool bf16_io, hipStream_t st);
int launch_bwd_post(const ChunkArgs &a, bool bf16_io, hipStream_t st);

// Backward with one state gate per key channel: phase 2 runs on the folded operands
// (Gamma . Q, Gamma . K, K~ / Gamma) and leaves the gradients with respect to those; this
// kernel turns them, in place, into the gradients with respect to q, k (read side) and k~,
// and collects dL/dlog_alpha.
struct UnfoldArgs {
    int B, T, H, K, N;
    int n0, n1;
    const float *log_alpha;           // [B,T,H,K]
    const void *q, *k, *kt;           // [B,T,H,K] io: the unfolded operands
    void *dq, *dk_read, *dkt;         // [B,T,H,K] io: in: w.r.t. the folded operands; out: w.r.t. q, k, k~
    const float *gamC, *dgamC;        // [B,H,N,K]
    float *dlog_alpha;                // [B,T,H,K]
};
int launch_unfold(const UnfoldArgs &a, bool bf16_io, hipStream_t st);

}  // namespace osdn
