/*
 * kda.h -- C ABI of libkda: Kimi Delta Attention (KDA), forward and backward, on one MI355X.
 *
 * KDA is the gated delta rule of the paper's Section 3, Eq. (1):
 *
 *     S_t = (I - beta_t k_t k_t^T) Diag(alpha_t) S_{t-1} + beta_t k_t v_t^T,
 *     o_t = scale * S_t^T q_t,          alpha_t = exp(log_alpha_t) in (0,1]^dk
 *
 * with one dk x dv state S per (sequence, head).  Two entry points compute it:
 * kda_chunk_fwd with the chunkwise WY / UT-transform algorithm of Section 3.1
 * (prefill), kda_recurrent_step with one literal step of Eq. (1) (decode,
 * Section 6.3 "Inference strategy").
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers to contiguous row-major arrays,
 *     16-byte aligned.  The caller owns every buffer, including the workspace.
 *     The library allocates nothing, frees nothing, creates no stream or event
 *     and keeps no state between calls (beyond per-device caches of constant
 *     device attributes).
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = default stream): every kernel of a call is launched on that stream,
 *     no host synchronisation happens inside (kda_chunk_fwd_check, which exists to
 *     wait, aside), and a call may be captured into a graph.
 *   - Concurrency: calls may be issued from several host threads and on several
 *     streams at once, each with its own workspace (a workspace belongs to one call
 *     until that call has completed).  The bf16 prefill runs its per-chunk stage and
 *     its sequential stage as workgroups of ONE kernel: the sequential workgroups (one
 *     per (sequence, head), or a few for calls with few pairs and long sequences, each
 *     on half a compute unit, never more than half of the device's such places at a
 *     time) wait for the slots that the per-chunk workgroups behind them
 *     in the same grid produce.  The producers wait for nothing and are dispatched as
 *     soon as any half compute unit is free, so every wait ends; each wait is bounded
 *     all the same (about two seconds).  Should other work on the device starve the
 *     producers that long, the waiting workgroup gives up: the outputs it had still
 *     to write for that (sequence, head), to the end of the sequence (a call that scans
 *     ranges of a long sequence side by side: at least to the end of the range), and the
 *     final state if the stretch reaches it, are NaN, never stale data, and
 *     kda_chunk_fwd_check reports it.
 *   - Element offsets are 64-bit; tensors with more than 2^31 elements are fine.
 *   - Errors: a non-zero kda_status is returned and kda_last_error() holds a
 *     thread-local description.  For KDA_ERR_INVALID_ARG, KDA_ERR_UNSUPPORTED
 *     and KDA_ERR_WORKSPACE nothing has been launched.  No exception crosses
 *     the ABI.
 *   - log_alpha must be finite and <= 0 (alpha = 0 is not representable);
 *     alpha = 1 (log_alpha = 0) is allowed.  Values are never clamped.
 */
#ifndef KDA_H_
#define KDA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KDA_OK = 0,
    KDA_ERR_INVALID_ARG = 1,   /* null pointer, negative size, bad combination   */
    KDA_ERR_UNSUPPORTED = 2,   /* head dim / chunk / dtype outside the built set */
    KDA_ERR_WORKSPACE = 3,     /* workspace missing, misaligned or too small     */
    KDA_ERR_LAUNCH = 4         /* the HIP runtime refused a launch               */
} kda_status;

typedef enum { KDA_F32 = 0, KDA_BF16 = 1 } kda_dtype;

/*
 * Problem description.
 *   Fixed-length batch : cu_seqlens == NULL, num_seqs == batch, every batch row
 *                        is one sequence of `seqlen` tokens.
 *   Packed batch       : cu_seqlens != NULL, batch == 1, `seqlen` is the total
 *                        number of packed tokens, sequence n owns tokens
 *                        [cu_seqlens[n], cu_seqlens[n+1]).
 * Supported: dk == dv in {64, 128}, chunk == 64, in_dtype KDA_F32 or KDA_BF16
 * (bf16 inputs with head dim 64 are processed by the fp32 kernels: exact
 * widening, fp32 arithmetic, fp32 o).  out_dtype KDA_F32 always; KDA_BF16 with
 * in_dtype KDA_BF16 and head dim 128 (o is computed in fp32 and rounded to
 * nearest even once, when it is stored; states stay fp32).
 */
typedef struct {
    int32_t   batch;       /* B                                                  */
    int64_t   seqlen;      /* T per batch row, or total packed tokens            */
    int32_t   heads;       /* H                                                  */
    int32_t   dk, dv;      /* key / value head dimension                         */
    int32_t   chunk;       /* C of Section 3.1; must be 64                       */
    int32_t   num_seqs;    /* N                                                  */
    kda_dtype in_dtype;    /* q, k, v, log_alpha, beta all share it              */
    kda_dtype out_dtype;   /* dtype of o                                         */
    float     scale;       /* multiplies o; 1.0f gives Eq. (1), dk^-0.5 gives    */
                           /* the App. C listing                                 */
    int64_t   max_seqlen;  /* packed batches only: upper bound on the longest    */
                           /* sequence, 0 = unknown (seqlen is assumed)          */
} kda_dims;

/*
 * Workspace, in bytes, with which kda_chunk_fwd runs `dims` in a single
 * segment (fastest).  kda_chunk_fwd also accepts any workspace of at least
 * kda_chunk_fwd_min_workspace_size(dims) bytes and then walks the time axis
 * in several segments, carrying the state between them.  Both return 0 for an
 * unsupported or malformed `dims`, and for problems that need no workspace.
 * KDA_F32 inputs: the minimum is 0 (one sequential kernel per sequence, head and
 * 32 state columns); with kda_chunk_fwd_workspace_size(dims) bytes (per chunk and
 * head two 64 x 66 and three 64 x dk fp32 tiles) a parallel per-chunk kernel and a
 * matrix-core walk run instead, about sixteen times faster at 4 x 4096 tokens x 16
 * heads; anything in between runs the sequential kernel.
 */
size_t kda_chunk_fwd_workspace_size(const kda_dims *dims);
size_t kda_chunk_fwd_min_workspace_size(const kda_dims *dims);

/*
 * Chunkwise prefill (Section 3.1: chunk expansion, WY representation, UT
 * transform, chunk state update, inter/intra-chunk output; the decay products
 * follow the reading gamma^{i->r} = exp(G^r - G^i), G the inclusive running
 * sum of log_alpha inside a chunk).  Each sequence is cut into chunks of 64
 * tokens starting at its own first token; a shorter last chunk is legal.
 *
 *   q, k       [B,T,H,dk]      in_dtype
 *   v          [B,T,H,dv]      in_dtype
 *   log_alpha  [B,T,H,dk]      in_dtype, natural log of the per-channel decay
 *   beta       [B,T,H]         in_dtype
 *   h0         [N,H,dk,dv]     fp32 initial states, or NULL for zeros
 *   cu_seqlens [N+1]           int32, device memory, non-decreasing, starts at
 *                              0, last entry <= T; or NULL (fixed length)
 *   o          [B,T,H,dv]      out_dtype; rows of tokens owned by no sequence
 *                              are left untouched
 *   hT         [N,H,dk,dv]     fp32 final states (state after the last token of
 *                              each sequence; equals h0 for an empty sequence),
 *                              or NULL if not wanted.  May alias h0.
 *   workspace                  device scratch, 256-byte aligned (may be NULL
 *                              when the required size is 0)
 * o must not alias any input.  Arithmetic: KDA_F32 inputs are processed in fp32
 * throughout; KDA_BF16 inputs use fp16 matrix-core operands with fp32
 * accumulation, fp32 cumulative decay and an fp32 state.  Domain of the KDA_BF16
 * path: |k_t| <= 4 and entries of q within +-3.9 (the paper's q and k are
 * L2-normalised, Section 4), and states, values and pseudo-values small enough for
 * fp16 (below 65504 in magnitude).  bf16 inputs convert to fp16 exactly while their magnitude is
 * zero or within [2^-14, 65504]; smaller ones lose bits or flush, larger ones
 * become infinite.  Beyond the domain an fp16 operand overflows to infinity and
 * the affected outputs and states come back as Inf or NaN; kda_chunk_fwd_check
 * reports a key beyond the domain and a state that is not finite.
 */
kda_status kda_chunk_fwd(const kda_dims *dims,
                         const void *q, const void *k, const void *v,
                         const void *log_alpha, const void *beta,
                         const float *h0, const int32_t *cu_seqlens,
                         void *o, float *hT,
                         void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * kda_chunk_fwd for callers that cannot allocate device memory and have no workspace to bring: code
 * under graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is a
 * static device array inside the library, kda_static_scratch_size() bytes (64 MiB) per GPU that the
 * library runs on, held until the process ends.  Everything else (arguments, results, arithmetic) is
 * that of kda_chunk_fwd given a workspace of that size: long inputs are walked in time segments with
 * the state carried between them.  The call allocates nothing and frees nothing.  A call whose
 * smallest workspace (kda_chunk_fwd_min_workspace_size) exceeds the array is refused with
 * KDA_ERR_WORKSPACE and launches nothing: at dk = dv = 128 that is beyond about 190 (sequence, head)
 * pairs per call.  All calls on one GPU share that GPU's array, which keeps the last call's contents
 * (each call clears what it needs at zero itself): calls that overlap in time on one GPU, from any
 * stream or thread, race on it and must not be made.  kda_chunk_fwd_check does not apply.
 */
size_t kda_static_scratch_size(void);
kda_status kda_chunk_fwd_static_scratch(const kda_dims *dims,
                                        const void *q, const void *k, const void *v,
                                        const void *log_alpha, const void *beta,
                                        const float *h0, const int32_t *cu_seqlens,
                                        void *o, float *hT, void *hip_stream);

/*
 * Backward pass of kda_chunk_fwd: gradients of  sum(o . d_o) + sum(hT . d_hT)  with respect to
 * every input.  The paper motivates a training kernel (Section 3.1 compares the chunkwise form
 * with the general DPLR one for exactly that purpose) but derives no backward algorithm; what
 * is computed here is the chain rule applied to Eq. (1), organised chunk by chunk through the
 * quantities of Section 3.1 (A_kk, A_qk, the UT transform, the chunk state update), in fp32
 * throughout, every decay kept as a pairwise difference of cumulative log decays so that it
 * cannot overflow.
 *
 *   q, k, v, log_alpha, beta, h0, cu_seqlens   as for kda_chunk_fwd (in_dtype KDA_F32 or
 *                              KDA_BF16, dk == dv in {64, 128})
 *   d_o        [B,T,H,dv]      gradient of o in out_dtype, i.e. the dtype o had: fp32, or bf16
 *                              with bf16 inputs (rows of tokens owned by no sequence are not
 *                              read)
 *   d_hT       [N,H,dk,dv]     fp32 gradient of the final states, or NULL for zeros
 *   dq, dk, dlog_alpha [B,T,H,dk], dv [B,T,H,dv], dbeta [B,T,H]    fp32, written; rows of
 *                              tokens owned by no sequence are left untouched
 *   dh0        [N,H,dk,dv]     fp32 gradient of the initial states (equals d_hT for an empty
 *                              sequence), or NULL if not wanted
 *   workspace                  at least kda_chunk_bwd_workspace_size(dims) bytes, 256-byte
 *                              aligned: the state at the start of every chunk and the
 *                              gradient of the state at its end (2 * dk * dv floats per chunk
 *                              and head), three [tokens, H, dv] arrays and four C x C tiles
 *                              per chunk and head; it is not bounded by time segments
 * No gradient may alias an input or another gradient.  Sequences of more than 65535 * 64
 * tokens are KDA_ERR_UNSUPPORTED.  Everything runs on `hip_stream`.
 */
size_t kda_chunk_bwd_workspace_size(const kda_dims *dims);
kda_status kda_chunk_bwd(const kda_dims *dims,
                         const void *q, const void *k, const void *v,
                         const void *log_alpha, const void *beta,
                         const float *h0, const int32_t *cu_seqlens,
                         const void *d_o, const float *d_hT,
                         float *dq, float *dk, float *dv, float *dlog_alpha, float *dbeta,
                         float *dh0,
                         void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * Fused input prologue (Section 4, "Neural Parameterization").  With a kda_prologue the kernels
 * take the raw projections and apply, in fp32 and before anything else,
 *     q <- q / sqrt(sum_c q_c^2 + l2norm_eps),   k likewise            (L2Norm over dk)
 *     beta <- 1 / (1 + exp(-beta))                                       (Sigmoid)
 *     log_alpha[c] <- -a_scale[h] * log(1 + exp(gate[c] + dt_bias[h][c]))
 * The paper does not print its decay function f; this is the softplus form of the two models
 * it names as its pattern, with the constants exposed (a_scale = NULL means 1, dt_bias = NULL
 * means 0, which gives log_alpha = -softplus(gate)).  The short convolution, Swish and the
 * projections themselves stay with the caller.
 */
typedef struct {
    float        l2norm_eps;   /* >= 0                                            */
    const float *a_scale;      /* [H]     fp32, device memory, or NULL            */
    const float *dt_bias;      /* [H,dk]  fp32, device memory, or NULL            */
} kda_prologue;

/*
 * Fused output gate (Section 4): with a kda_epilogue the kernels replace each o (one vector of
 * dv values per token and head) by
 *     o <- Sigmoid(gate) * o / sqrt(mean_j o_j^2 + rms_eps) * norm_weight
 * in fp32 before they store it (`scale` is applied to o first; the prefill carries the factor
 * norm_weight * Sigmoid(gate) from its per-chunk stage to its sequential stage as fp16, the decode
 * kernel evaluates it in fp32).  The paper gives neither the epsilon nor the shape of the learned
 * RMSNorm weight: one vector of dv values shared by all heads is taken (NULL = ones).  The gate's
 * and the output's projections stay with the caller.
 */
typedef struct {
    float        rms_eps;      /* >= 0                                                       */
    const void  *gate;         /* gate logits, same shape and dtype as v ([..,H,dv]), device  */
    const float *norm_weight;  /* [dv] fp32, device memory, or NULL                           */
} kda_epilogue;

/*
 * Workspace sizes for kda_chunk_fwd_fused: as kda_chunk_fwd_workspace_size and
 * kda_chunk_fwd_min_workspace_size, plus, when `epilogue` is not NULL, room for the gate factors that
 * the per-chunk stage leaves for the sequential stage (16 KiB per chunk and head held at once).
 * With epilogue == NULL they equal the plain functions.  A fused call whose workspace is smaller
 * than the first figure still runs, in more segments.
 */
size_t kda_chunk_fwd_fused_workspace_size(const kda_dims *dims, const kda_epilogue *epilogue);
size_t kda_chunk_fwd_fused_min_workspace_size(const kda_dims *dims, const kda_epilogue *epilogue);

/*
 * kda_chunk_fwd with the fused stages: `prologue` (or NULL: q, k, gate = log_alpha and beta are
 * taken as kda_chunk_fwd takes them) and `epilogue` (or NULL: o is stored as it is).  Everything
 * else is as for kda_chunk_fwd.  Built for KDA_BF16 inputs with dk == dv == 128.
 */
kda_status kda_chunk_fwd_fused(const kda_dims *dims, const kda_prologue *prologue,
                               const kda_epilogue *epilogue,
                               const void *q_raw, const void *k_raw, const void *v,
                               const void *gate, const void *beta_logit,
                               const float *h0, const int32_t *cu_seqlens,
                               void *o, float *hT,
                               void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/*
 * kda_chunk_fwd for the scalar-gate special case of Eq. (1) (Section 2.2: alpha_t = a_t I, one
 * decay per token and head): log_alpha_head is [B,T,H] in in_dtype, everything else as for
 * kda_chunk_fwd.  The result equals kda_chunk_fwd on that decay repeated over the dk channels; the
 * per-chunk kernel is cheaper (the decay leaves the matrix-core operands and multiplies the fp32
 * tiles instead, so no range handling is needed whatever the decay).  Built for KDA_BF16 inputs with
 * dk == dv == 128; workspace sizes as for kda_chunk_fwd.
 */
kda_status kda_chunk_fwd_scalar_gate(const kda_dims *dims,
                                     const void *q, const void *k, const void *v,
                                     const void *log_alpha_head, const void *beta,
                                     const float *h0, const int32_t *cu_seqlens,
                                     void *o, float *hT,
                                     void *workspace, size_t workspace_bytes,
                                     void *hip_stream);

/*
 * Optional check after a bf16 kda_chunk_fwd: waits for `hip_stream` and reads
 * the status word that the call left in `workspace` (same dims, workspace and
 * size as that call).  The sequential workgroups of the prefill wait, for a
 * bounded time, for each workspace slot; if such a wait ever ran out, the call
 * has written NaN to o from that point of the (sequence, head) on (see the
 * conventions above) and this returns KDA_ERR_LAUNCH.  If a state of the call ended
 * up not finite (an fp16 operand overflowed) or a key was beyond the domain
 * stated at kda_chunk_fwd it returns KDA_ERR_INVALID_ARG.  KDA_OK otherwise (also for
 * calls that keep no status word: fp32 inputs).
 */
kda_status kda_chunk_fwd_check(const kda_dims *dims, const void *workspace, size_t workspace_bytes,
                               void *hip_stream);

/*
 * One decode step of Eq. (1) for N = dims->num_seqs sequences (Section 6.3):
 *     S <- Diag(alpha) S;  r = v - S^T k;  S <- S + beta k r^T;  o = scale S^T q.
 * dims->seqlen must be 1 and dims->batch == dims->num_seqs.
 *
 *   q, k, log_alpha [N,H,dk]   in_dtype
 *   v               [N,H,dv]   in_dtype
 *   beta            [N,H]      in_dtype
 *   S               [N,H,dk,dv] fp32, read and written IN PLACE
 *   o               [N,H,dv]   out_dtype
 * All arithmetic is fp32.  No workspace.
 */
kda_status kda_recurrent_step(const kda_dims *dims,
                              const void *q, const void *k, const void *v,
                              const void *log_alpha, const void *beta,
                              float *S, void *o, void *hip_stream);

/*
 * Decode over a state pool (serving-shaped variant of kda_recurrent_step, same
 * Eq. (1) and Section 6.3): sequence n works on the state S_pool[state_indices[n]]
 * and takes Tq = dims->seqlen new tokens (1 <= Tq <= 8) through it in order, e.g.
 * the draft tokens of a speculative-decoding verification step.  The state is read
 * once and written once per call, whatever Tq is.  dims->batch == dims->num_seqs = N.
 *
 *   q, k, log_alpha [N,Tq,H,dk]   in_dtype
 *   v               [N,Tq,H,dv]   in_dtype
 *   beta            [N,Tq,H]      in_dtype
 *   S_pool          [P,H,dk,dv]   fp32 pool of P states; only the addressed ones are
 *                                 read and written, in place
 *   state_indices   [N]           int32, device memory; entry n in [0,P) names the state
 *                                 of sequence n, a negative entry skips the sequence
 *                                 (its rows of o are left untouched); NULL = 0,1,..,N-1.
 *                                 Entries are not range-checked against P, and two
 *                                 sequences naming the same state race.
 *   o               [N,Tq,H,dv]   out_dtype; o of token t reads the state after token t
 * All arithmetic is fp32.  No workspace.
 */
kda_status kda_recurrent_steps_pooled(const kda_dims *dims,
                                      const void *q, const void *k, const void *v,
                                      const void *log_alpha, const void *beta,
                                      float *S_pool, const int32_t *state_indices,
                                      void *o, void *hip_stream);

/* kda_recurrent_steps_pooled with one decay per token and head: log_alpha_head is [N,Tq,H]. */
kda_status kda_recurrent_steps_pooled_scalar_gate(const kda_dims *dims,
                                                  const void *q, const void *k, const void *v,
                                                  const void *log_alpha_head, const void *beta,
                                                  float *S_pool, const int32_t *state_indices,
                                                  void *o, void *hip_stream);

/*
 * kda_recurrent_steps_pooled with the fused stages (either may be NULL; see kda_prologue and
 * kda_epilogue); q_raw, k_raw, gate [N,Tq,H,dk], beta_logit [N,Tq,H], epilogue->gate [N,Tq,H,dv].
 */
kda_status kda_recurrent_steps_fused(const kda_dims *dims, const kda_prologue *prologue,
                                     const kda_epilogue *epilogue,
                                     const void *q_raw, const void *k_raw, const void *v,
                                     const void *gate, const void *beta_logit,
                                     float *S_pool, const int32_t *state_indices,
                                     void *o, void *hip_stream);

/* Static description of a status code (never NULL). */
const char *kda_status_string(kda_status status);

/* Detail of the last error raised on the calling thread ("" if none). */
const char *kda_last_error(void);

/* Library version string, e.g. "kda-gfx950 0.1". */
const char *kda_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KDA_H_ */
