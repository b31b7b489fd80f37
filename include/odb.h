/* odb.h - C ABI of the MI355X (gfx950) block-decode / cache-refresh library.
 *
 * The library computes the model step of ODB-dLLM (arXiv 2511.21759):
 *   - odb_prefill: the full-sequence bidirectional forward that refreshes the
 *     K/V cache and yields a decoding attempt for every response position
 *     (Sec. 2.1 "DualCache" refresh; Sec. 4.1, first paragraph);
 *   - odb_block_step: the forward of S mutually invisible drafts of one
 *     response block against the cached K/V of every position outside the
 *     block, followed by the confidence-threshold acceptance
 *     (Sec. 3 Observation 3; Sec. 4.2 and Fig. 8 for the drafts);
 * and, built on those two, the paper's controllers: odb_predict_length (Sec. 4.1),
 * odb_accept_jump (Sec. 4.2.1) and its form for eight blocks, odb_speculative_jump,
 * odb_block_step_shared (Sec. 4.2.2) and the whole block-wise loop, odb_generate
 * (Sec. 2.1).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on the current HIP device,
 *     "host" pointers are ordinary host memory.  The caller owns every buffer
 *     it passes; the library owns models, caches and its internal scratch.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls with a stream argument are asynchronous on it unless they say
 *     otherwise (odb_generate is synchronous): outputs are valid once the caller
 *     has synchronised the stream.  Calls that use the same model must be issued
 *     on one stream at a time (they share scratch).
 *   - Every function returns ODB_OK (0) or a negative ODB_E_* code; a message
 *     for the last failure on the calling thread is kept in odb_last_error().
 *     Arguments are validated on the host before any kernel is launched, so an
 *     invalid call launches nothing.
 *   - There is no CPU fallback: without a usable gfx950 device calls fail with
 *     ODB_E_HIP.
 */
#ifndef ODB_H
#define ODB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ODB_OK 0
#define ODB_E_INVALID_ARG (-1)
#define ODB_E_NOMEM (-2)
#define ODB_E_HIP (-3)
#define ODB_E_UNSUPPORTED (-4)
#define ODB_E_NO_PROGRESS (-5)   /* odb_generate: a decode step left the block's MASK count unchanged */

typedef struct odb_model odb_model;
typedef struct odb_cache odb_cache;

/* Architecture of the masked-diffusion transformer.  The paper names the LLaDA
 * 8B models (Sec. 5.1) without listing the architecture; this library fixes
 * pre-norm residual blocks, RMSNorm, rotate-half RoPE on the full head
 * dimension, SwiGLU, an untied LM head and no biases.
 * Requirements: d_model = n_heads*head_dim; head_dim is 64 or 128; d_model and
 * d_ff are multiples of 256; vocab is a multiple of 16; 0 <= mask_id < vocab. */
typedef struct {
    int n_layers, d_model, n_heads, head_dim, d_ff, vocab;
    float rope_base; /* pair j of a head turns by pos * rope_base^(-2j/head_dim) */
    float rms_eps;
    int mask_id;     /* token id of [MASK] */
} odb_config;

/* Optional device allocator (e.g. backed by torch.empty(device="cuda")).
 * alloc returns a device pointer aligned to 256 B or NULL. */
typedef struct {
    void *(*alloc)(size_t bytes, void *user);
    void (*free)(void *dev_ptr, void *user);
    void *user;
} odb_allocator;

/* Tensor ids for odb_model_set_tensor / odb_model_get_tensor.  Logical shapes
 * are row-major [out, in]: EMBED and LM [vocab, d]; WQ WK WV WO [d, d]; WG WU
 * [d_ff, d]; WD [d, d_ff]; the gains G1 (before attention), G2 (before the
 * MLP) and GF (before the LM head) are [d].  `layer` is ignored for EMBED, LM
 * and GF. */
enum {
    ODB_T_EMBED = 0, ODB_T_WQ, ODB_T_WK, ODB_T_WV, ODB_T_WO, ODB_T_WG, ODB_T_WU,
    ODB_T_WD, ODB_T_LM, ODB_T_G1, ODB_T_G2, ODB_T_GF, ODB_T_COUNT
};

/* Creates a model and allocates its weights in HBM (private tiled layout).
 * allocator may be NULL (hipMalloc/hipFree are used).  Weights are
 * uninitialised until odb_model_init_random or odb_model_set_tensor. */
int odb_model_create(const odb_config *cfg, const odb_allocator *allocator,
                     odb_model **out);
void odb_model_destroy(odb_model *m);

/* Fills every weight with bf16_rne(float(std * x)), x ~ N(0,1) drawn by the
 * counter-based generator below from the element's logical flat index, and
 * sets all gains to 1.  Element i of tensor t at layer l uses
 *   key = SM(SM(seed) + (t << 32 | l)),   z = SplitMix64 output i of state key,
 *   u1 = (hi32(z)+0.5)/2^32, u2 = (lo32(z)+0.5)/2^32,
 *   x = sqrt(-2 ln u1) cos(2 pi u2)   evaluated in binary64,
 * where SM(s) is the first SplitMix64 output for state s.  Asynchronous on
 * `stream`. */
int odb_model_init_random(odb_model *m, uint64_t seed, double std, void *stream);

/* Replaces / reads back one tensor as bf16 bit patterns in logical row-major
 * order (host memory, n = number of elements, must match the shape).
 * Synchronous.  Inside the library the projection matrices are held as IEEE
 * binary16, which represents every bf16 value of magnitude 2^-16 .. 65504
 * exactly; smaller magnitudes are rounded to a multiple of 2^-24 (an absolute
 * error below 3e-8).  A projection matrix with an element beyond that range (or
 * a NaN) is rejected with ODB_E_UNSUPPORTED and the model is left unchanged; the
 * embedding table and the gains are kept as given (bf16 / float). */
int odb_model_set_tensor(odb_model *m, int tensor_id, int layer,
                         const uint16_t *host_bf16, size_t n);
int odb_model_get_tensor(const odb_model *m, int tensor_id, int layer,
                         uint16_t *host_bf16, size_t n);

/* K/V cache for `batch` sequences of up to max_len positions: post-RoPE K and
 * V, two bytes per element (binary16), for every layer, head and position
 * (Sec. 2.1). */
int odb_cache_create(odb_model *m, int batch, int max_len, odb_cache **out);
void odb_cache_destroy(odb_cache *c);
/* Current sequence length set by the last odb_prefill (0 before). */
int odb_cache_length(const odb_cache *c);
/* Cuts the cached sequences to new_len positions (ODB-dLLM Sec. 4.1: the response is
 * truncated at the predicted end): positions new_len .. length-1 stop being keys of later
 * decode steps; the K/V of the kept positions stay as the last odb_prefill wrote them.
 * Host-side bookkeeping only; takes effect for calls issued afterwards.  Errors:
 * ODB_E_INVALID_ARG for a NULL cache or new_len outside [1, current length]. */
int odb_cache_truncate(odb_cache *c, int new_len);

/* Cache refresh (Sec. 2.1; Sec. 4.1).  tokens: dev int32 [batch, L], ids in
 * [0, vocab).  Runs the bidirectional forward over all L positions of every
 * sequence (positions 0..L-1), stores post-RoPE K and V of all of them in the
 * cache (its length becomes L) and writes, for response positions i >=
 * resp_off, conf (dev float [batch, L-resp_off]) = probability of the greedy
 * token and argmax (dev int32, same shape) = greedy token id, lowest id on
 * ties.  1 <= L <= max_len, 0 <= resp_off < L. */
int odb_prefill(odb_model *m, odb_cache *c, const int32_t *tokens_dev, int L,
                int resp_off, float *conf_dev, int32_t *argmax_dev, void *stream);

/* Block-decode step (Sec. 3 Obs. 3; Sec. 4.2).  drafts: dev int32
 * [batch, S, b]: S versions of the block at positions block_off ..
 * block_off+b-1 (all drafts share these position ids).  Each draft's b rows
 * attend to the cached K/V of positions outside the block and to the draft's
 * own fresh K/V; the cache entries at the block's positions are ignored and
 * the cache is not modified.  Outputs, all dev [batch, S, b]: conf (float),
 * argmax (int32) and unmask (uint8): 1 iff the draft holds mask_id there and
 * (conf > tau or the position is the draft's most confident masked position,
 * lowest index on ties).  Requires a prefilled cache, 0 <= block_off,
 * block_off + b <= cache length, 1 <= b <= 256, 1 <= S. */
int odb_block_step(odb_model *m, const odb_cache *c, const int32_t *drafts_dev,
                   int block_off, int b, int S, float tau, float *conf_dev,
                   int32_t *argmax_dev, uint8_t *unmask_dev, void *stream);

/* Run-time switches of a model.
 *   ODB_OPT_KSPLIT_REDUCE (default 1): projections with few rows and a long K may run on the
 *     streaming kernel that splits K over four workgroups, which exchange their partial sums
 *     through device-scope stores and an arrival counter inside the one launch (the last
 *     workgroup to arrive adds them in slice order, so results do not depend on timing).
 *     0 routes those projections to the kernels that exchange nothing inside a launch (the
 *     plain streaming kernel, or the tile kernel with a separate reduction pass).
 * Errors: ODB_E_INVALID_ARG for a NULL model, an unknown option or a value outside its range. */
enum { ODB_OPT_KSPLIT_REDUCE = 0 };
int odb_set_option(odb_model *m, int option, int value);

/* Synchronises the device, reads the model's status word and clears it.  Returns ODB_OK, or
 *   ODB_E_UNSUPPORTED  an activation left the binary16 range since the last check.  Between the
 *       kernels activations travel as binary16: Q, K, V, the SwiGLU output and, because the
 *       RMSNorm is folded into its neighbours, the un-normalised residual stream times the
 *       norm's gain, h[i] * g[i].  All of them must stay within +-65504 (for h * g that is a
 *       bound on the residual stream of the model, about 3e3 times what the 8B-shaped synthetic
 *       weights reach); a value beyond is clamped and flagged, as is a NaN.  Outputs of the
 *       calls since the last check are then not to be trusted;
 *   ODB_E_INVALID_ARG  odb_block_step_shared met a block with more MASK positions than n_masked. */
int odb_model_status(odb_model *m);

/* odb_block_step for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and same results as odb_block_step, but every intermediate buffer lives in a fixed
 * area of ODB_STATIC_SCRATCH_BYTES bytes that is part of the loaded library (one per GPU,
 * held until the process ends); the call itself allocates and frees nothing.
 * A step whose rows need more than that area is rejected with ODB_E_UNSUPPORTED before
 * anything is launched (at the 8B shape of the paper's models, d = 4096, d_ff = 12288,
 * vocab = 126464, the area holds steps of up to 128 rows).  All models on one GPU share the
 * area and every call overwrites what the last one left there: calls on one GPU that overlap
 * in time, on whatever streams or models, race; issue them one after the other on one
 * stream.  Other errors as odb_block_step. */
#define ODB_STATIC_SCRATCH_BYTES (32u << 20)
int odb_block_step_static(odb_model *m, const odb_cache *c, const int32_t *drafts_dev,
                          int block_off, int b, int S, float tau, float *conf_dev,
                          int32_t *argmax_dev, uint8_t *unmask_dev, void *stream);

/* Test-only variants that materialise the logits (dev float, row-major
 * [batch, L-resp_off, vocab] resp. [batch, S, b, vocab]) through an unfused
 * store instead of the fused confidence/argmax reduction. */
int odb_prefill_logits(odb_model *m, odb_cache *c, const int32_t *tokens_dev,
                       int L, int resp_off, float *logits_dev, void *stream);
int odb_block_step_logits(odb_model *m, const odb_cache *c,
                          const int32_t *drafts_dev, int block_off, int b, int S,
                          float *logits_dev, void *stream);

/* Adaptive length prediction after a refresh (ODB-dLLM Sec. 4.1).  The refresh's
 * decoding attempt (the conf / argmax that odb_prefill wrote for response positions
 * resp_off .. L-1) is scanned per sequence for [EOS]: the response as currently
 * drafted holds tokens[p] where position p is decoded and argmax where it still holds
 * the model's MASK id; an attempted [EOS] counts only if its confidence exceeds
 * truncate_thr (strictly), a decoded one counts as it stands.  new_len_dev[b] = index
 * of the earliest such position + 1 (the [EOS] stays the last position of the
 * sequence), or L when there is none.  The paper prints neither the threshold nor the
 * [EOS] id: both are arguments.
 *   tokens_dev  device int32 [batch, L]          the tokens the refresh ran on
 *   conf_dev    device float [batch, L-resp_off] \ outputs of odb_prefill
 *   argmax_dev  device int32 [batch, L-resp_off] /
 *   new_len_dev device int32 [batch]             written
 * Asynchronous on `stream`; all buffers are the caller's.  Errors: ODB_E_INVALID_ARG
 * for NULL pointers, batch < 1, L < 1, resp_off outside [0, L), eos_id outside
 * [0, vocab) or equal to the MASK id. */
int odb_predict_length(const odb_model *m, const int32_t *tokens_dev, const float *conf_dev,
                       const int32_t *argmax_dev, int batch, int L, int resp_off, int eos_id,
                       float truncate_thr, int32_t *new_len_dev, void *stream);

/* Decode step in the decoded-share stage (ODB-dLLM Sec. 4.2.2, Fig. 8 caption).
 * drafts_dev [batch, S, b] as for odb_block_step, with S >= 2 and b <= 64; the drafts of a
 * sequence must agree with its block_0 (draft 0) wherever block_0 holds a decoded token.
 * block_0 is forwarded in full, exactly as odb_block_step does it.  A speculative block
 * s >= 1 is reduced to the positions that block_0 still has MASKed (position ids kept); at
 * every layer its rows attend to the cached K/V outside the block, to block_0's fresh K/V
 * of the decoded positions, and to their own fresh K/V - not to other speculative blocks,
 * not to block_0's rows at masked positions.  So the decoded tokens are computed once per
 * step and the step has b + (S-1) * n_masked rows per sequence (each of the two parts
 * padded to a multiple of 16) instead of S * b.
 *   n_masked    host value: upper bound of the MASK positions in block_0 of any sequence
 *               (sets the row count; a block with more raises an error that
 *               odb_model_status reports as ODB_E_INVALID_ARG, its outputs are then invalid)
 *   conf_dev, argmax_dev, unmask_dev [batch, S, b] as for odb_block_step; for s >= 1 the
 *               entries at decoded positions are not computed and read conf 0,
 *               argmax = the token held there, unmask 0
 * Asynchronous on `stream`; does not modify the cache.  Errors as odb_block_step, plus
 * ODB_E_INVALID_ARG for b > 64, S outside [2, 64], n_masked outside [0, b]. */
int odb_block_step_shared(odb_model *m, const odb_cache *c, const int32_t *drafts_dev,
                          int block_off, int b, int S, int n_masked, float tau,
                          float *conf_dev, int32_t *argmax_dev, uint8_t *unmask_dev, void *stream);

/* Test aid: rows of a decoded-share step (block_0 of every sequence, padded to 16, then
 * per sequence its speculative blocks one after the other, together padded to 16), or a
 * negative error code. */
int odb_block_step_shared_rows(int batch, int b, int S, int n_masked);
/* Test aid: the logits of every row of the decoded-share step, float [rows, vocab], and for
 * every row its index into [batch, S, b] (-1 for padding rows), int32 [rows]; both device
 * buffers of the caller. */
int odb_block_step_shared_logits(odb_model *m, const odb_cache *c, const int32_t *drafts_dev,
                                 int block_off, int b, int S, int n_masked, float *logits_dev,
                                 int32_t *rowout_dev, void *stream);

/* Accept-jump controller (ODB-dLLM Sec. 4.2.1): decides which of the four drafts of
 * the last block step is adopted and builds the drafts of the next one, on the device.
 * The step ran on drafts[.,0] = block_0 (the block as it stood), [.,1] = block_0 with
 * candidate B unmasked beforehand, [.,2] = with candidate D, [.,3] = with both
 * (cand_pos / cand_tok: position inside the block and speculated token of B and D;
 * position -1 = no such candidate, as in the first step of a block).  A candidate is
 * verified in a draft when that draft's step unmasks its position with exactly the
 * speculated token.  Both verified in block_0: block_3 is adopted.  Only one: the draft
 * that had it unmasked beforehand is taken, and block_3 instead if the other candidate is
 * verified there.  Neither: block_0.  Adopting a draft = its tokens plus every position
 * its own step unmasked (with that step's greedy token); that is new_drafts[.,0].  The
 * next candidates are the two most confident positions of the adopted draft that are
 * still MASK afterwards (lower index first on equal confidence; -1 / token 0 if fewer
 * remain), their tokens that draft's greedy tokens, and new_drafts[.,1..3] unmask them.
 *   drafts_dev, argmax_dev  device int32 [batch, 4, b]     inputs / outputs of odb_block_step
 *   conf_dev device float [batch, 4, b], unmask_dev device uint8 [batch, 4, b]
 *   cand_pos_dev, cand_tok_dev       device int32 [batch, 2]
 *   chosen_dev device int32 [batch] (0..3), new_drafts_dev device int32 [batch, 4, b],
 *   new_cand_pos_dev, new_cand_tok_dev device int32 [batch, 2]             written
 * Output buffers must not overlap input buffers.  Asynchronous on `stream`; all buffers
 * are the caller's.  Errors: ODB_E_INVALID_ARG for NULL pointers, batch < 1, b < 1. */
int odb_accept_jump(const odb_model *m, const int32_t *drafts_dev, const float *conf_dev,
                    const int32_t *argmax_dev, const uint8_t *unmask_dev,
                    const int32_t *cand_pos_dev, const int32_t *cand_tok_dev, int batch, int b,
                    int32_t *chosen_dev, int32_t *new_drafts_dev, int32_t *new_cand_pos_dev,
                    int32_t *new_cand_tok_dev, void *stream);

/* The jump rule over the S = 4 or 8 blocks of a step (ODB-dLLM Sec. 4.2.1, carried over to the
 * eight blocks of Sec. 4.2.2; the paper states the rule for the two candidates B and D only).
 * With the candidates ranked by confidence, block s holds the block with these candidates
 * unmasked beforehand: s = 0 none, 1 {B}, 2 {D}, 3 {B, D}, 4 {third}, 5 {B, D, third},
 * 6 {fourth}, 7 {all four}.  The walk starts at block_0.  At a block with candidate set X the
 * verified set is X plus every other candidate whose position this block's own step unmasks
 * with exactly the speculated token; the block whose set lies strictly above X inside the
 * verified set and holds the most candidates (the lowest number among equals) is visited
 * next, and the block at which no such block exists is adopted.  For S = 4 this is the rule
 * of odb_accept_jump.  The adopted block plus every position its own step unmasked is
 * new_drafts[.,0]; the n_next / 2 most confident positions still MASK there (lower index
 * first on equal confidence; -1 / token 0 where fewer remain, and in the entries behind
 * n_next / 2) are the next candidates and new_drafts[.,1 .. n_next) the blocks built on them.
 *   drafts_dev, argmax_dev  device int32 [batch, S, b]; conf_dev float, unmask_dev uint8, same shape
 *   cand_pos_dev, cand_tok_dev  device int32 [batch, 4] (the first S / 2 are read)
 *   chosen_dev device int32 [batch], new_drafts_dev device int32 [batch, n_next, b],
 *   new_cand_pos_dev, new_cand_tok_dev device int32 [batch, 4]                 written
 * Output buffers must not overlap input buffers.  Asynchronous on `stream`; all buffers are
 * the caller's.  Errors: ODB_E_INVALID_ARG for NULL pointers, batch < 1, b < 1, S or n_next
 * other than 4 and 8. */
int odb_speculative_jump(const odb_model *m, const int32_t *drafts_dev, const float *conf_dev,
                         const int32_t *argmax_dev, const uint8_t *unmask_dev,
                         const int32_t *cand_pos_dev, const int32_t *cand_tok_dev, int batch, int b,
                         int S, int n_next, int32_t *chosen_dev, int32_t *new_drafts_dev,
                         int32_t *new_cand_pos_dev, int32_t *new_cand_tok_dev, void *stream);

/* Block-wise generation of one response (ODB-dLLM Sec. 2.1, with the adaptive length
 * prediction of Sec. 4.1 and the jump-share decoding of Sec. 4.2 switched on by the
 * parameters).  The host loop is the library's; every decision is taken by kernels and the
 * host reads back sixteen 32-bit words per forward.
 *
 * The response starts as resp_len MASK tokens behind the prompt and is decoded block by
 * block, front to back.  A block cycle opens with a refresh (odb_prefill over the whole
 * sequence: the cache is rebuilt and every response position attempted).  Then
 *   1. if eos_id >= 0, the attempt is scanned as odb_predict_length does and the sequence
 *      is cut at once: dropped positions leave the token sequence and, as for
 *      odb_cache_truncate, stop being keys of this cycle's steps;
 *   2. the attempt at the current block goes through the acceptance rule of odb_block_step
 *      (MASK positions whose confidence exceeds tau, and always the most confident one), so
 *      the refresh is also the block's first decoding iteration;
 *   3. decode steps follow until the block holds no MASK.  n_drafts = 1: odb_block_step on
 *      the block alone.  n_drafts = 4: the four accept-jump drafts and odb_accept_jump (the
 *      first candidates are the two most confident positions the refresh left MASKed); once
 *      share_from positions of the block are decoded the step is odb_block_step_shared
 *      on the same four drafts.  n_drafts = 8 (needs share_from >= 0): as n_drafts = 4 until
 *      share_from positions are decoded, then odb_block_step_shared on eight blocks - the four
 *      most confident positions left MASKed are the candidates (Sec. 4.2.2: the third, the top
 *      three, the fourth and the top four join B, D and B + D) - and odb_speculative_jump;
 *      with row_budget > 0 a step of that stage whose eight blocks would come to more rows
 *      runs on the four accept-jump blocks instead.
 *      A step that leaves the block's MASK count unchanged (an untrained model may attempt
 *      the MASK token itself) ends the call with ODB_E_NO_PROGRESS rather than repeating for ever.
 * Generation ends when the next block would start at or behind the end of the sequence.
 * None of the parameter values is printed in the paper.
 *
 *   tokens_dev  device int32 [prompt_len + resp_len]; the caller fills the prompt, the call
 *               writes the MASKs and then the decoded tokens; positions behind the final
 *               length are left as they were when they were cut
 *   c           a cache for batch 1 with max_len >= prompt_len + resp_len; left holding the
 *               last refresh, cut to the final length
 *   stats       host, written (counts, lengths, host wall-clock of the two phases)
 *   events      host array of max_events records or NULL: one record per forward, in order
 *   event_tokens_dev  device int32 [max_events, prompt_len + resp_len] or NULL: the token
 *               sequence after every forward (test aid; costs one device copy per forward)
 * Synchronous: returns after the last forward has finished; the stream is synchronised
 * once per forward.  Working buffers come from the model's allocator and are released
 * before returning.  Errors: ODB_E_INVALID_ARG for NULL handles / tokens / params / stats,
 * prompt_len < 1, resp_len < 1, a cache of batch != 1 or too short, block_len outside
 * [1, 256] (or > 64 with share_from >= 0), n_drafts other than 1, 4 and 8 (or 8 with
 * share_from < 0), eos_id >= vocab or
 * equal to the MASK id; more than max_events forwards stop being recorded (stats.n_events
 * still counts them).  On an error of an inner call its code is returned and tokens_dev is
 * left partly decoded. */
enum { ODB_EV_REFRESH = 0, ODB_EV_STEP = 1, ODB_EV_STEP_SHARED = 2 };
typedef struct {
    int block_len;        /* positions per block (32 in the paper's runs) */
    int n_drafts;         /* 1: threshold decoding; 4: accept-jump (Sec. 4.2.1); 8: accept-jump, then
                             eight blocks in the decoded-share stage (Sec. 4.2.2) */
    float tau;            /* acceptance threshold */
    int eos_id;           /* < 0: no length prediction */
    float truncate_thr;   /* Sec. 4.1 */
    int share_from;       /* decoded positions of the block from which steps run in the
                             decoded-share stage (Sec. 4.2.2); < 0: never */
    int row_budget;       /* n_drafts = 8: a decoded-share step forwards eight blocks only if its
                             block_len + 7 * masked rows fit this budget, else the four accept-jump
                             blocks (Sec. 4.2: the step has to stay memory-bound; Sec. 4.2.2: the
                             shrinking blocks make room for the extra candidates); <= 0: always eight */
} odb_generate_params;
typedef struct {
    int kind;             /* ODB_EV_* */
    int length;           /* sequence length after the event */
    int block_off, block_len;   /* block_len 0: the cut fell into what was already decoded */
    int chosen;           /* adopted draft (0 for a refresh and for n_drafts = 1) */
    int n_masked;         /* MASK positions left in the block */
    int cand_pos[4], cand_tok[4];   /* the candidates handed to the next step, best first (-1 / 0:
                                       none; n_drafts < 8 uses two) */
} odb_generate_event;
typedef struct {
    int n_refresh, n_step, n_step_shared, final_len, n_events;
    long long refresh_positions;    /* sum of the refreshed lengths */
    long long step_rows;            /* rows forwarded by the steps (padding not counted) */
    double refresh_ms, step_ms, total_ms;   /* host wall-clock, each phase up to its read-back */
} odb_generate_stats;
int odb_generate(odb_model *m, odb_cache *c, int32_t *tokens_dev, int prompt_len, int resp_len,
                 const odb_generate_params *params, odb_generate_stats *stats,
                 odb_generate_event *events, int32_t *event_tokens_dev, int max_events,
                 void *stream);

/* Copies cached K (kv = 0, post-RoPE, logical channel order) or V (kv = 1) of
 * positions pos0 .. pos0+n-1 of one sequence and layer to host memory as
 * float [n, n_heads, head_dim].  Synchronous (device-wide). */
int odb_cache_read(const odb_cache *c, int layer, int kv, int batch_index,
                   int pos0, int n, float *host_f32);

/* Measurement aid.  Between odb_profile_begin and odb_profile_end every launch
 * of the kernel class `kernel_class` made by calls on this model is bracketed
 * by a pair of HIP events recorded on the launch stream (at most max_launches
 * pairs; further launches are not timed).  odb_profile_end synchronises the
 * device, returns the number of timed launches and the sum of their durations
 * in milliseconds, and releases the events.  A pair also spans the latency
 * from its first event to the start of the kernel, which a kernel trace does
 * not count: behind every pair a third event is recorded, and empty_pairs_ms
 * (may be NULL) receives the sum of the intervals between second and third
 * events - what a pair measures with nothing in between.  The events serialise
 * nothing but do cost a few microseconds each: do not time whole steps while
 * enabled. */
enum {
    ODB_K_GEMM_QKV = 0, ODB_K_ATTENTION, ODB_K_GEMM_O, ODB_K_GEMM_GATE_UP,
    ODB_K_GEMM_DOWN, ODB_K_GEMM_LM_HEAD, ODB_K_RMSNORM, ODB_K_COUNT
};
int odb_profile_begin(odb_model *m, int kernel_class, int max_launches);
int odb_profile_end(odb_model *m, int *n_launches, float *total_ms, float *empty_pairs_ms);

const char *odb_strerror(int code);
const char *odb_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ODB_H */
