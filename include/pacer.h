/*
 * pacer.h -- C ABI of the MI355X (gfx950) hot path of Pacer adaptive speculative decoding
 * (Zhang et al., "Pacer: Blockwise Pre-verification for Speculative Decoding with Adaptive
 * Length").  One decoding step of the paper's Alg. 1 is four calls:
 *
 *     pacer_draft_step        x b      Eq. 3 / Eq. 6   one draft-model token
 *     pacer_preverify_block            Eq. 7 + the halting test of Alg. 1's inner loop
 *       ... repeated while the block passes ...
 *     pacer_verify                     Eq. 4           one target pass over the drafts
 *     pacer_accept_rollback            Eq. 5 + the verification part of Alg. 1
 *
 * Conventions
 *   - Every pointer named dev_* is DEVICE memory, everything else is HOST memory.
 *   - The library allocates no device memory.  Weights, KV caches, the workspace and every
 *     output buffer are owned by the caller and only BORROWED for the life of the context;
 *     the caller frees them after pacer_destroy.
 *   - All work is enqueued on the HIP stream given to pacer_create.  Hot calls do not
 *     synchronise with the host, except where a call says so.
 *   - Every call returns a status: 0 = PACER_OK, negative = error (arguments are validated
 *     on the host before anything is enqueued, so a failed call has no effect on device state).
 *     pacer_last_error gives a static, human readable string for the context's last failure.
 *   - A context is bound to one device and one stream and is not thread safe.
 *   - Token ids are int32.  Sequences are numbered 0..max_batch-1.
 *
 * Model: Llama-style decoder (pre-norm RMSNorm, rotate-half RoPE at absolute positions,
 * causal multi-head attention, SwiGLU).  The pre-verification layer M_B is one such layer of
 * the draft model's width over its own KV cache, a final RMSNorm and a 2-class head; its input
 * row j is  hidden_j + PosEmb[draft position]  (Sec. 3.2).  Prefix rows use PosEmb row 0.
 */
#ifndef PACER_H
#define PACER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PACER_OK 0
#define PACER_EINVAL (-1)     /* bad argument: null pointer, bad shape, bad sequence id, bad mode */
#define PACER_ESTATE (-2)     /* call out of order, tensor / cache / workspace not bound          */
#define PACER_EOVERFLOW (-3)  /* KV capacity (max_seq) or gamma_max would be exceeded             */
#define PACER_EHIP (-4)       /* the HIP runtime reported an error                                */
#define PACER_ENUMERIC (-5)   /* a token id outside the vocabulary was met on the device (pacer_prefill) */

#define PACER_F32 0
#define PACER_BF16 1

#define PACER_TARGET 0
#define PACER_DRAFT 1
#define PACER_PREVERIFY 2

#define PACER_GREEDY 0
#define PACER_SAMPLE 1

#define PACER_MAX_BATCH 16

/* tensor ids for pacer_bind; "layer" is ignored for the per-model tensors */
#define PACER_T_EMBED 0       /* [vocab][d]        model dtype, row major (TARGET, DRAFT)        */
#define PACER_T_FINAL_NORM 1  /* [d]               f32                                           */
#define PACER_T_HEAD 2        /* [vocab][d]        matrix (TARGET, DRAFT)                        */
#define PACER_T_ATTN_NORM 3   /* [d]               f32, per layer                                */
#define PACER_T_WQKV 4        /* [3d][d]           matrix, rows = Wq then Wk then Wv, per layer  */
#define PACER_T_WO 5          /* [d][d]            matrix, per layer                             */
#define PACER_T_FFN_NORM 6    /* [d]               f32, per layer                                */
#define PACER_T_WGU 7         /* [2*d_ffn][d]      matrix, rows = W_gate then W_up, per layer    */
#define PACER_T_WD 8          /* [d][d_ffn]        matrix, per layer                             */
#define PACER_T_POSEMB 9      /* [gamma_max+1][d]  f32, PREVERIFY only; row 0 must be zero       */
#define PACER_T_CLS 10        /* [2][d]            f32, PREVERIFY only: logits of reject/accept  */
#define PACER_T_COUNT 11
/*
 * "matrix" tensors are [out][in] (y = W x).  For a PACER_F32 model they are plain row-major
 * f32.  For a PACER_BF16 model they must be in the tiled layout written by pacer_pack_weight
 * (same byte count as the row-major bf16 matrix); out must be a multiple of 16 and in a
 * multiple of 32.
 */

typedef struct pacer_ctx pacer_ctx;

typedef struct {
  int32_t n_layers, d_model, n_heads, head_dim /* 64 or 128 */, d_ffn, vocab, max_seq;
  float rope_theta, rms_eps;
  int32_t dtype; /* PACER_F32 or PACER_BF16: type of the matrices and the embedding */
} pacer_model_cfg;

#define PACER_HALT_MEAN 0 /* stop if mean(alpha) <= t: the paper's criterion (Alg. 1)        */
#define PACER_HALT_ANY 1  /* stop if any alpha_j <= t   (stricter alternative of Sec. 5.2)   */
#define PACER_HALT_LAST 2 /* stop if the block's last alpha <= t   (Sec. 5.2)                */

/* Inputs of Alg. 1: block size b, initial threshold t, growth factor rho; gamma_max caps the
 * window (the paper's inner loop has no cap) and must be a multiple of block. */
typedef struct {
  int32_t block, gamma_max;
  float t0, rho;
  int32_t halting; /* PACER_HALT_* */
} pacer_pv_cfg;

/* ---- set-up (not hot) ---------------------------------------------------------------- */

/* Creates a context.  Touches no GPU.  The pre-verification layer has the draft's d_model,
 * n_heads, head_dim, d_ffn, dtype and max_seq.  hip_stream: a hipStream_t (may be 0). */
int32_t pacer_create(pacer_ctx** out, const pacer_model_cfg* target, const pacer_model_cfg* draft,
                     const pacer_pv_cfg* pv, int32_t max_batch, void* hip_stream);
void pacer_destroy(pacer_ctx* ctx);
const char* pacer_last_error(const pacer_ctx* ctx); /* ctx may be NULL: last failure of a context-free call on this thread */

/* Re-tiles a row-major bf16 matrix [n_out][n_in] (dev_src) into the layout the bf16 kernels
 * stream (dev_dst, same size, must not alias).  The packed copy holds each bf16 value as an IEEE
 * half float (what the matrix instructions multiply; exact for |w| >= 2^-17, smaller values round
 * to the nearest half subnormal).  The tiling depends on the role of the matrix:
 * tensor_id is the PACER_T_* id it will be bound as (WQKV, WO, WGU, WD or HEAD); head_dim is
 * needed for WQKV (rotation pairs of a head share a tile) and ignored otherwise.
 * Half floats end at 65504: a weight beyond that (or an inf / NaN in the source) becomes a non-finite
 * half.  dev_not_finite (device int32, may be NULL; the caller zeroes it) is incremented once per such
 * weight, so that the caller can refuse the model instead of decoding garbage.  The same range holds for
 * what the kernels store as half floats at run time: normalised activations times the norm gain, the
 * SwiGLU product and the K/V cache entries must stay below 65504 in magnitude.
 * Enqueued on hip_stream. */
int32_t pacer_pack_weight(void* dev_dst, const void* dev_src, int32_t n_out, int32_t n_in,
                          int32_t tensor_id, int32_t head_dim, int32_t* dev_not_finite, void* hip_stream);

/* Borrow one weight tensor.  nbytes must equal the tensor's size for the model's shape. */
int32_t pacer_bind(pacer_ctx* ctx, int32_t which, int32_t tensor_id, int32_t layer,
                   const void* dev_ptr, uint64_t nbytes);

/* KV cache of one model for all max_batch sequences, max_batch * n_layers * 2 * max_seq *
 * d_model elements: f32 for a PACER_F32 model ([seq][layer][K|V][position][d_model]), 2-byte
 * IEEE half floats for a PACER_BF16 model ([seq][layer] x { K, then V }, each stored per head in
 * the 1 KiB tile order the attention kernel's matrix instructions read: K as
 * [head][position/16][feature/32][64 lanes][8], V as [head][position/32][feature/16][64 lanes][8];
 * max_seq must be a multiple of 32).  The layout is the
 * library's own; contents need not be initialised: pacer_bind_kv clears the buffer (a memset
 * enqueued on the context's stream), because attention reads whole 32-position groups and the
 * slots past a sequence's end must hold finite values.  pacer_kv_bytes returns the exact size
 * pacer_bind_kv expects. */
uint64_t pacer_kv_bytes(const pacer_ctx* ctx, int32_t which);
int32_t pacer_bind_kv(pacer_ctx* ctx, int32_t which, void* dev_ptr, uint64_t nbytes);

/* Scratch memory for activations, draft logits, committed tokens, attention partials.
 * Must be 256-byte aligned and at least pacer_workspace_bytes large.  Binding it is the call
 * that first touches the GPU (it also allocates a few hundred bytes of pinned host memory
 * through which pacer_accept_rollback reports its results). */
uint64_t pacer_workspace_bytes(const pacer_ctx* ctx);
int32_t pacer_bind_workspace(pacer_ctx* ctx, void* dev_ptr, uint64_t nbytes);

/* Prompt ingestion (support; Alg. 1 takes the prefix as given).  Resets sequence `seq` to the
 * committed tokens dev_tokens[0..n-1], n >= 1, and fills the three caches for positions
 * 0..n-2 (M_B with prefix rows), 512 positions per pass through the weights.  The workspace
 * is sized for such a pass whatever max_batch is.
 * Token ids live on the device, so this call cannot refuse a bad one.  Instead no kernel ever
 * uses an id outside [0, vocab) as an index: the copy of the prompt, and every kernel that
 * chooses a token (an argmax over logits without a finite value has no winner), replaces such an
 * id by the nearest valid one and sets a word for the sequence in pinned host memory.  The
 * sequence's next pacer_wait_stop, pacer_get_state or pacer_begin_step then returns
 * PACER_ENUMERIC and the sequence takes no further step until it is prefilled again.  (A used
 * sequence's prefill waits for the stream first, so that no earlier kernel reports into the new
 * prompt's word.) */
int32_t pacer_prefill(pacer_ctx* ctx, int32_t seq, const int32_t* dev_tokens, int32_t n);

/* Debug / teacher forcing: replace the committed tokens of `seq` from position `from` on with
 * host_tokens[0..n-1] and set the committed length to from+n.  Valid only if all three caches
 * already hold correct rows for positions < from+n-1 (e.g. directly after a step whose first
 * from+n-1 positions agree).  Synchronises. */
int32_t pacer_force_commit(pacer_ctx* ctx, int32_t seq, int32_t from, const int32_t* host_tokens,
                           int32_t n);

/* ---- the hot path -------------------------------------------------------------------- */

/* Start of one outer iteration of Alg. 1 for `seq`: threshold <- t0, draft position <- 1,
 * no drafts.  Collects the sequence's previous pacer_accept_rollback first, as pacer_get_state does, if
 * that has not happened yet (this waits for its kernels). */
int32_t pacer_begin_step(pacer_ctx* ctx, int32_t seq);

/* Eq. 3 / Eq. 6: one draft-model forward per listed sequence on its newest token (the last
 * committed token, or the previous draft), appending to the draft KV cache.  Keeps the logits
 * q_i (f32 [vocab]) and the hidden state h_i (final-norm output, f32 [d]) in the workspace and
 * picks y_i = argmax (PACER_GREEDY; lowest id wins ties) or y_i ~ softmax (PACER_SAMPLE,
 * Gumbel-max on Philox-4x32-10 keyed by rng_seed; rng_ctr = index of the decoding step).
 * PACER_EOVERFLOW if the sequence already holds gamma_max drafts. */
int32_t pacer_draft_step(pacer_ctx* ctx, const int32_t* seqs, int32_t n_seqs, int32_t mode,
                         uint64_t rng_seed, uint64_t rng_ctr);

/* Eq. 7 and the halting test: runs M_B on the last `block` hidden states (+ their draft
 * position embeddings) of each listed sequence, appends to M_B's KV cache, writes
 * dev_alpha[n_seqs][block] (estimated acceptance rates), dev_stop[n_seqs] = (mean alpha <= t)
 * evaluated in f32, then multiplies the sequence's threshold by rho.  dev_alpha / dev_stop may
 * be read after synchronising the stream.  PACER_ESTATE unless exactly `block` new drafts
 * exist since the last call. */
int32_t pacer_preverify_block(pacer_ctx* ctx, const int32_t* seqs, int32_t n_seqs,
                              float* dev_alpha, int32_t* dev_stop);

/* Test tap: forces the stop flag of the NEXT pacer_preverify_block of `seq` (flag 1 = stop, 0 = go on; -1 takes a
 * pending force back).  The pre-verification kernel still computes and writes alpha, then writes the forced flag to
 * dev_stop and to the host-polled word instead of its own decision; the force is used up by that call.  Any stopping
 * rule that looks only at draft-side quantities leaves the output law unchanged (Sec. 2.2), so sweeping forced
 * patterns checks losslessness for every pre-verification decision. */
int32_t pacer_force_stop(pacer_ctx* ctx, int32_t seq, int32_t flag);

/* The stop flags of the last pacer_preverify_block of each listed sequence, as host values:
 * host_stop[n_seqs] (host array).  The kernel also writes each flag, tagged with the number of
 * the call, to pinned host memory; this call polls those words, which takes a few microseconds
 * after the kernel has finished where a stream synchronisation plus a device-to-host copy takes
 * tens.  It waits for that kernel only, not for the stream.  This is what decides whether
 * drafting goes on (Alg. 1, the stop test of the inner loop).  PACER_ESTATE if a listed sequence
 * has had no pre-verification call since its prefill. */
int32_t pacer_wait_stop(pacer_ctx* ctx, const int32_t* seqs, int32_t n_seqs, int32_t* host_stop);

/* The inner loop of Alg. 1 in one call, for sequences at the start of a step (after pacer_begin_step, no drafts
 * yet): rounds of `block` draft steps (Eq. 6) and one pre-verification call (Eq. 7) for the sequences still
 * drafting, until each has stopped (halting test, or a forced flag) or another block would exceed gamma_max.  It is
 * the same sequence of pacer_draft_step / pacer_preverify_block / pacer_wait_stop calls a caller would issue (same
 * kernels, same results); the loop runs inside the library so that between two rounds the host does nothing but
 * read the kernel-written flag words and enqueue.  mode, rng_seed, rng_ctr as in pacer_draft_step.  dev_alpha
 * [n_seqs][block] and dev_stop [n_seqs] are the outputs of the pre-verification calls (on return: of the last round,
 * for the sequences that took part in it, in list order).  host_gamma[n_seqs] (host array) receives the windows.
 * If a call inside the loop fails, its status is returned and the sequences keep the drafts made so far. */
int32_t pacer_draft_window(pacer_ctx* ctx, const int32_t* seqs, int32_t n_seqs, int32_t mode, uint64_t rng_seed,
                           uint64_t rng_ctr, float* dev_alpha, int32_t* dev_stop, int32_t* host_gamma);

/* Eq. 4: one target pass over [last committed token, y_1..y_gamma] of each listed sequence
 * against its KV cache (appending those rows).  gamma = number of drafts since
 * pacer_begin_step, or gamma_override[s] if gamma_override != NULL and >= 0 (host array; must
 * not exceed the number of drafts made).  Writes f32 logits to
 * dev_logits[n_seqs][gamma_max+1][vocab] (rows beyond gamma+1 are left untouched).
 * The call only enqueues kernels on the context's stream (no allocation, no memset, no host
 * wait) and writes the same cache and logits rows when repeated, so it may be recorded by a
 * stream capture and replayed; positions and row counts are those of the recorded call. */
int32_t pacer_verify(pacer_ctx* ctx, const int32_t* seqs, int32_t n_seqs,
                     const int32_t* gamma_override, float* dev_logits);

/* Eq. 5 and the rest of Alg. 1: with effective target logits  l_T + beta[s] * l_D  (beta:
 * host array [n_seqs]; 0 gives the paper's plain rule), PACER_GREEDY accepts the leading drafts
 * equal to the effective argmax and emits the argmax at the first mismatch (or of the bonus
 * row); PACER_SAMPLE accepts y_i while r_i <= p_i[y_i]/q_i[y_i], then samples from
 * norm(max(0, p - q)) at the first rejection or from p_{gamma+1}.  Extends M_B's cache over
 * positions that no pacer_preverify_block covered.  The call only enqueues (rows i < gamma: the
 * accept tests and the token at the first rejection) and returns; it does not wait for the verify
 * pass.  A sequence that accepted all gamma drafts still needs the draft forward on y_gamma (it
 * completes the draft cache and yields the draft logits of the bonus row) and the bonus row's
 * token: that part is enqueued by the call that collects the result (pacer_get_state, or the
 * sequence's next pacer_begin_step), which is where the host first learns n.  Appends
 * y_1..y_n and the new token to the committed tokens; all three caches then logically hold
 * committed_length-1 positions (rollback = shorter length, nothing is erased).
 * dev_logits: the buffer pacer_verify wrote.  dev_n_accepted[n_seqs], dev_next_token[n_seqs]
 * receive n and the new token (-1 until the bonus row has been evaluated); the same values reach
 * the host through pacer_get_state.  dev_logits, dev_n_accepted and dev_next_token must stay valid
 * until the result has been collected.  PACER_ESTATE if a listed sequence still has an uncollected
 * result. */
int32_t pacer_accept_rollback(pacer_ctx* ctx, const int32_t* seqs, int32_t n_seqs, int32_t mode,
                              const float* beta, uint64_t rng_seed, uint64_t rng_ctr,
                              const float* dev_logits, int32_t* dev_n_accepted,
                              int32_t* dev_next_token);

/* For callers that cannot allocate device memory and hold no context: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  The acceptance rule of pacer_accept_rollback for ONE sequence on
 * logits the caller holds, through the same kernels, with their scratch (per-row, per-vocabulary-chunk statistics,
 * token candidates and reject flags; 17 KiB) in a fixed array inside the library's device image instead of a
 * workspace.  Calls no hipMalloc / hipFree and no allocating routine; enqueues on hip_stream and returns.
 *   dev_target_logits [gamma+1][vocab] f32  row i = target logits after y_1..y_i (row gamma: the bonus row)
 *   dev_draft_logits  [gamma+1][vocab] f32  row i = draft logits q_{i+1}; row gamma is read only if bonus_row != 0
 *   dev_draft_tokens  [gamma] i32           y_1..y_gamma
 *   bonus_row         nonzero: if every draft is accepted the new token is taken from row gamma of both logits
 *                     buffers; zero: that case yields next token -1 and the caller evaluates the bonus row later
 *   beta, mode, rng_seed, rng_ctr, seq      as in pacer_accept_rollback (seq 0..PACER_MAX_BATCH-1 keys the random streams)
 *   dev_n_accepted[1], dev_next_token[1]    results (device memory, valid after the stream has passed the call);
 *                     next token 0x7fffffff: the logits that decide it held no finite value.  A draft token id
 *                     outside [0, vocab) is read as the nearest valid id (it never indexes past a logits row)
 * gamma may be 0..PACER_NOALLOC_MAX_GAMMA; a larger gamma is refused with PACER_EOVERFLOW.  Nothing but the two
 * results is written: no tokens are committed and no cache length changes.  The device that is current when the
 * call is made must be the one hip_stream belongs to; on the first call on a device the library looks up that
 * device's copy of the array.  All calls on one GPU share that GPU's array: calls whose kernels may overlap there
 * (different streams, or several threads) race and must be serialised by the caller; calls on one stream are
 * ordered.  The array keeps the previous call's contents; every word a call reads it has written itself before.
 * After a failure pacer_last_error(NULL) returns the message (per thread). */
#define PACER_NOALLOC_MAX_GAMMA 31
int32_t pacer_accept_noalloc(const float* dev_target_logits, const float* dev_draft_logits,
                             const int32_t* dev_draft_tokens, int32_t gamma, int32_t bonus_row, int32_t vocab,
                             int32_t mode, float beta, uint64_t rng_seed, uint64_t rng_ctr, int32_t seq,
                             int32_t* dev_n_accepted, int32_t* dev_next_token, void* hip_stream);

/* Waits for the sequence's pending pacer_accept_rollback, if any (by polling the pinned host
 * words its last kernel writes; it does not synchronise the stream), enqueues and awaits the bonus-row
 * part for sequences that accepted every draft, folds the result into the
 * host-side state and reports: gamma (drafts of the current/last step), len (committed tokens), t (current
 * threshold), n_accepted / next_token of the last finished step (-1 if none).  Any output
 * pointer may be NULL. */
int32_t pacer_get_state(pacer_ctx* ctx, int32_t seq, int32_t* gamma, int32_t* len, float* t,
                        int32_t* n_accepted, int32_t* next_token);

/* ---- test taps (not hot) ------------------------------------------------------------- */
#define PACER_PEEK_DRAFT_LOGITS 0 /* f32 [gamma_max+1][vocab]  row j = logits of draft forward j */
#define PACER_PEEK_DRAFT_HIDDEN 1 /* f32 [gamma_max+1][d_draft]                                   */
#define PACER_PEEK_DRAFT_TOKENS 2 /* i32 [gamma_max+1]                                            */
#define PACER_PEEK_TOKENS 3       /* i32 [max_seq] committed tokens                               */
/* Device pointer (inside the workspace) of a per-sequence buffer; valid while bound. */
int32_t pacer_peek(pacer_ctx* ctx, int32_t seq, int32_t what, void** dev_ptr, uint64_t* nbytes);

/* Host only, no context: how the weight-streaming GEMM of the target model would be launched for a
 * few-tile matrix (fewer than 512 output tiles of 16: the O and down projections) of n_out x n_in
 * weights on `rows` activation rows (1..32) with `operand_parts` f16 parts per activation (1 = hi,
 * 2 = hi + lo): output tiles per block and K slices across blocks (1 = K is not split; with more, the
 * blocks of a tile group add their partial tiles through the workspace).  PACER_EINVAL on a null
 * pointer or sizes outside those bounds. */
int32_t pacer_launch_plan(int32_t n_out, int32_t n_in, int32_t rows, int32_t operand_parts,
                          int32_t* tiles_per_block, int32_t* k_slices);

/* Number of kernels the context has enqueued since it was created (benchmarks: launches per call). */
int32_t pacer_launch_count(const pacer_ctx* ctx, int64_t* n_launches);

/* Benchmark support, no context: one kernel that reads dev_src[0..nbytes) once (16-byte loads, 256 blocks of 4
 * waves) and folds it into dev_sink (256 bytes of device memory, caller-zeroed or not).  Timed by the caller, it
 * gives the streaming-read rate a kernel reaches on this GPU when it does nothing but load: the practical ceiling
 * beside which the weight-streaming GEMMs' rates are reported.  dev_src must be 16-byte aligned.  repeat (1..100000)
 * launches of the same read are enqueued back to back: with a few KiB this measures what one more kernel in a
 * sequence of launches costs when it does next to nothing. */
int32_t pacer_stream_probe(const void* dev_src, uint64_t nbytes, int32_t repeat, void* dev_sink, void* hip_stream);

/* Kernel timing for benchmarks: while enabled, every launch of the target model's GEMM kernels
 * carries a pair of HIP events on the context's stream that receive the kernel's own begin and end
 * time stamps (up to 16384 launches between two reads; later ones run untimed).
 * pacer_profile_read synchronises and returns the number of timed launches, their summed duration
 * and the summed weight bytes they streamed, then clears the counters. */
int32_t pacer_profile_enable(pacer_ctx* ctx, int32_t on);
int32_t pacer_profile_read(pacer_ctx* ctx, int64_t* n_launches, double* total_ms,
                           double* weight_bytes);

#ifdef __cplusplus
}
#endif
#endif /* PACER_H */
