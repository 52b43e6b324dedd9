/*
 * bild.h - C ABI of the MI355X (gfx950) Big Little Decoder library.
 *
 * The calls follow the paper's problem statement (Section 3.2) and Algorithm 1:
 * a small model drafts tokens autoregressively, a large model reviews a block
 * of drafts in one non-autoregressive pass.  Every numerical step runs in HIP
 * kernels on the device; the host side of this library only owns memory and
 * launches.  There is no CPU fallback.
 *
 * Conventions
 *   - every function returns BILD_OK (0) or a negative BILD_E* code; nothing
 *     throws or aborts across this boundary; on error the object passed in is
 *     left as it was;
 *   - pointers named host_* / src / out / draft are HOST memory owned by the
 *     caller and only read or written during the call;
 *   - all device memory is owned by the library behind the opaque handles;
 *   - a handle is not thread-safe; distinct states are independent but calls
 *     on states sharing one stream serialise on it;
 *   - a call that runs a decoder pass returns once the pass's results have
 *     reached the host; the stream may still be retiring that pass's last
 *     kernel, so work the caller adds must go through the same stream or
 *     wait for it (bild_encode and the bench/profile calls do wait for the stream);
 *   - token ids are int32 in [0, vocab).
 *
 * Sequence model held by a bild_state
 *   y[0..y_len)       the sequence so far: <s> (encoder-decoder pairs) or the
 *                     prompt (decoder-only pairs) followed by generated tokens
 *   draft_start       y[draft_start..y_len) are small-model drafts the large
 *                     model has not reviewed yet
 *   len_small/large   number of leading tokens of y each model has consumed
 *                     into its KV cache (cache row p holds K/V of y[p])
 * A pass of a model consumes rows y[len..y_len) at positions len.. and yields,
 * for each row, the distribution of the token that follows it.
 *
 * Environment (read when a bild_state is created)
 *   BILD_NO_GRAPH=1      launch every kernel of a pass directly instead of replaying a captured
 *                        HIP graph (needed under rocprofv3, which cannot follow graph launches)
 */
#ifndef BILD_H
#define BILD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BILD_OK      0
#define BILD_EINVAL (-1) /* bad argument (null pointer, size out of range, token id >= vocab, unsupported shape) */
#define BILD_ESTATE (-2) /* call not valid in the current state (e.g. step before encode, nothing to consume) */
#define BILD_ECAP   (-3) /* capacity exceeded (source longer than max_src, sequence longer than max_len, n > max rows) */
#define BILD_EHIP   (-4) /* a HIP runtime call failed */
#define BILD_ENOMEM (-5) /* host or device allocation failed */

#define BILD_ACT_RELU        0 /* relu(x W_in) W_out                       */
#define BILD_ACT_GATED_GELU  1 /* (gelu_tanh(x W_in) * (x W_up)) W_out     */
#define BILD_ACT_SWIGLU      2 /* (silu(x W_in) * (x W_up)) W_out          */
#define BILD_POS_SINUSOIDAL  0 /* PE added to the embedding                */
#define BILD_POS_ROPE        1 /* rotary on q and k, pairs (2i, 2i+1)      */
#define BILD_POS_RELATIVE    2 /* learned bias on self-attention scores by clamped key-query distance */
#define BILD_DT_F32          0
#define BILD_DT_BF16         1 /* weights and cached K/V stored as bf16    */

#define BILD_MAX_ROWS 32       /* most rows one decoder pass processes     */

/* Architecture of one network.  The paper fixes only layer counts and widths
 * (Table 2); the rest is this benchmark's model contract:
 *   x = embed_scale*E[(tok+tie_shift) mod vocab] (+ sinusoidal PE; relative-position
 *   models add nothing here and bias their self-attention scores instead); pre-RMSNorm
 *   sublayers x += f(norm(x)) in the order self-attn, cross-attn, FFN; scores
 *   scaled by 1/sqrt(d_head); logits = logit_scale * norm(x) E_out^T.
 * d_model, n_heads*d_head and d_ff must be multiples of 32. */
typedef struct bild_model_config {
    int32_t n_enc_layers;   /* 0: no encoder of its own                                     */
    int32_t n_dec_layers;
    int32_t d_model;
    int32_t n_heads;
    int32_t d_head;         /* 64 or 128 or any multiple of 8 up to 128                     */
    int32_t d_ff;
    int32_t act;            /* BILD_ACT_*                                                   */
    int32_t pos;            /* BILD_POS_*                                                   */
    int32_t vocab;
    int32_t tied_head;      /* 1: the LM head is the embedding matrix                       */
    int32_t dtype;          /* BILD_DT_*                                                    */
    int32_t cross_attn;     /* 1: decoder layers have a cross-attention sublayer            */
    int32_t bos;            /* first token of y for encoder-decoder pairs                   */
    int32_t tie_shift;      /* row offset of the embedding lookup, 0 = ordinary             */
    float   logit_scale;
    float   embed_scale;
    float   norm_eps;
    float   rope_base;
    int32_t rel_max_dist;   /* BILD_POS_RELATIVE: distances are clamped to [-rel_max_dist, rel_max_dist] */
} bild_model_config;

/* Counters of one bild_generate call (Table 4 reports fallback and rollback
 * rates; the paper does not define their denominators, so raw counts are given). */
typedef struct bild_stats {
    int32_t small_steps;        /* small-model passes                                  */
    int32_t large_calls;        /* large-model passes (= fallbacks of both kinds)      */
    int32_t rows_verified;      /* rows processed by large-model passes                */
    int32_t fallbacks_conf;     /* fallbacks because max p_S < alpha_FB                */
    int32_t fallbacks_forced;   /* fallbacks because n_max drafts were pending         */
    int32_t rollbacks;          /* reviews that rejected a draft                       */
    int32_t tokens_discarded;   /* drafts removed by rollbacks                         */
    int32_t n_generated;
} bild_stats;

typedef struct bild_model bild_model; /* one network's weights on the device, immutable            */
typedef struct bild_pair  bild_pair;  /* {small, large}; borrows both models                       */
typedef struct bild_state bild_state; /* one request: y, both KV caches, cross K/V, control block  */

/* Number of entries bild_model_create expects in host_tensors for this config. */
int bild_model_num_tensors(const bild_model_config* cfg);

/* Uploads one network.  host_tensors[i] are fp32 host arrays in this order
 * (entries that do not exist for the config are simply absent from the list):
 *   emb [vocab][d]; head [vocab][d] (only if !tied_head);
 *   enc_final_norm [d] (only if n_enc_layers > 0); dec_final_norm [d];
 *   (BILD_POS_RELATIVE only) enc_rel_bias (only if n_enc_layers > 0), dec_rel_bias: [n_heads][2*rel_max_dist+1],
 *     entry [h][r + rel_max_dist] is added to the self-attention score of head h for a key r positions after
 *     the query (r clamped to +-rel_max_dist); one table per stack, shared by its layers; kept in fp32;
 *   per encoder layer: ln1 [d], wq [d][I], wk [d][I], wv [d][I], wo [I][d], ln2 [d],
 *                      w_in [d][F], w_up [d][F] (gated only), w_out [F][d];
 *   per decoder layer: ln1, wq, wk, wv, wo, then (cross_attn only) lnc [d], cwq [d][I],
 *                      cwk [d][I], cwv [d][I], cwo [I][d], then ln2, w_in, w_up (gated only), w_out.
 * Matrices are row-major [inputs][outputs] (a layer computes x W); I = n_heads*d_head, F = d_ff.
 * For BILD_DT_BF16 values are rounded to bf16 (nearest even) on upload.  The
 * arrays are copied; the caller may free them on return. */
int bild_model_create(const bild_model_config* cfg, const float* const* host_tensors, int n_tensors,
                      bild_model** out);
int bild_model_destroy(bild_model* m);

/* Pairs two models (Section 3.5.1: the only requirement is a shared
 * vocabulary).  Fails with BILD_EINVAL if vocab sizes or cross_attn differ, or if the
 * small model has cross-attention but no encoder and its d_model differs from the
 * large one's (it then attends to the large model's encoder output, the early-exit
 * arrangement of Section 4.4).  The pair borrows the models: destroy it first. */
int bild_pair_create(bild_model* small_model, bild_model* large_model, bild_pair** out);

/* Early-exit pair (Section 4.4, "Early Exiting Strategy in the BiLD Framework"): the small model IS the
 * first k decoder layers of `large` followed by the large model's final norm and its LM head (the shared
 * prediction head), with a logit scale of its own.  No weights are copied.  A state of such a pair keeps
 * ONE K/V cache for those k layers and remembers the hidden state each consumed token left after layer k,
 * so a pass of the large model runs layers k..L-1 only; if the trunk has not yet consumed the rows a
 * large pass needs, the library runs it first.  Results equal those of bild_pair_create on a separately
 * uploaded copy of the first k layers up to summation order.  1 <= k < n_dec_layers, else BILD_EINVAL.
 * The pair borrows `large`: destroy the pair first. */
int bild_pair_create_early_exit(bild_model* large_model, int k, float small_logit_scale, bild_pair** out);
int bild_pair_destroy(bild_pair* p);

/* Allocates the per-request device state: room for max_src source/prompt tokens
 * and a sequence y of at most max_len tokens (including <s> or the prompt).
 * n_max: cap on consecutive small-model tokens (appendix: 10); 0 disables it.
 * hip_stream: a hipStream_t to launch on, or NULL for a stream the state creates. */
int bild_state_create(const bild_pair* p, int max_src, int max_len, int n_max, void* hip_stream,
                      bild_state** out);
int bild_state_destroy(bild_state* s);

/* Starts a request (Section 3.2: both models map the input x and the partial output y_1..n-1 to a distribution
 * over the next token; this call does the part of that map which depends on x alone, once per request).
 * Encoder-decoder pairs: runs the encoder(s) over src[0..n_src)
 * and fills every decoder layer's cross-attention K/V; y = [bos].  Decoder-only
 * pairs: y = src (the prompt) and both caches are prefilled with its first
 * n_src-1 tokens.  Requires 1 <= n_src <= max_src. */
int bild_encode(bild_state* s, const int32_t* src, int n_src);

/* One autoregressive pass of the small model (Algorithm 1, lines 3-6): consumes the
 * unconsumed tail of y, takes token = argmax p_S and
 *   fallback_flag = (max p_S < alpha_fb) or (n_max drafts already pending).
 * If the flag is 0 the token is appended to y as a draft; if 1 it is returned
 * for diagnostics only and y is unchanged.  BILD_ESTATE if nothing is unconsumed
 * (two steps in a row after a fallback), BILD_ECAP if y is full.
 * max_prob (nullable) receives max p_S. */
int bild_small_step(bild_state* s, float alpha_fb, int32_t* token, int32_t* fallback_flag, float* max_prob);

/* One non-autoregressive pass of the large model over the pending drafts
 * (Algorithm 1, lines 9-16; rollback policy of Section 3.4 with d = -ln p_L(draft)).
 * draft == NULL reviews the n = y_len - draft_start drafts pending in the state
 * (n is then ignored).  draft != NULL first replaces the pending block by
 * draft[0..n) (tests and stress runs drive arbitrary blocks this way; the small
 * cache is cut back to the reviewed prefix).  n + 1 <= BILD_MAX_ROWS.
 * On return rollback_pos = r in [0, n]: the first draft with -ln p_L > alpha_rb,
 * or n if none; out_tokens (capacity n+1) receives the r accepted drafts followed
 * by the large model's token for position r; *n_out = r + 1.  y and both caches
 * are committed accordingly.  nll (nullable, capacity n) receives -ln p_L of each draft. */
int bild_large_verify(bild_state* s, const int32_t* draft, int n, float alpha_rb, int32_t* out_tokens,
                      int32_t* n_out, int32_t* rollback_pos, float* nll);

/* Sampling variant (Appendix, "BiLD with Sampling"): with top_p in (0, 1] every token either model commits
 * is DRAWN from the nucleus of its distribution instead of being the argmax; the fallback and the rollback
 * tests are unchanged.  Nucleus: the smallest set of most likely tokens whose probability reaches top_p,
 * plus any token tied with its least likely member.  Draw: the members are walked in increasing token id and
 * the first whose running probability exceeds u * P(nucleus) is taken.  The uniform numbers are the caller's:
 * u_small[p] / u_large[p] in [0, 1) is used when the small / large model commits the token at position p of
 * the sequence (host arrays of n >= max_len floats, copied).  top_p <= 0 switches back to argmax (the arrays
 * may then be NULL).  BILD_EINVAL for top_p > 1, a missing array, n < max_len or a number outside [0, 1). */
int bild_set_sampling(bild_state* s, float top_p, const float* u_small, const float* u_large, int n);

/* Acceptance rule of the review (Section 4.2 and the appendix comparison with speculative decoding, Tables 3-4).
 * BILD_ACCEPT_THRESHOLD (the default) is the paper's rollback policy, Section 3.4: the first draft with
 * -ln p_L(draft) > alpha_RB is rolled back.  BILD_ACCEPT_REJECTION is the stochastic rule of the methods the paper
 * compares with; it needs the sampling variant (bild_set_sampling called first, else BILD_ESTATE): with p_S the nucleus
 * distribution the small model drew a draft x from and p_L the large model's nucleus distribution of the same position,
 * x is kept iff u_accept[position] * p_S(x) < p_L(x); the first refused draft is replaced by a draw (the large model's
 * uniform number of that position, ids walked in increasing order) from the normalised positive part of p_L - p_S, and
 * if none is refused the next token is drawn from p_L as usual; alpha_RB is ignored.  The fallback policy is unchanged
 * (alpha_FB = 0 with n_max = w gives the fixed window w of those methods).  u_accept: host array of n >= max_len
 * numbers in [0, 1), copied; may be NULL for BILD_ACCEPT_THRESHOLD.  The library then keeps the small model's logits
 * of every pending draft (32 x vocabulary floats of device memory).  BILD_EINVAL for an unknown rule, a missing or
 * short array or a number outside [0, 1). */
#define BILD_ACCEPT_THRESHOLD 0
#define BILD_ACCEPT_REJECTION 1
int bild_set_acceptance(bild_state* s, int rule, const float* u_accept, int n);

/* Lowers a cache length (Algorithm 1, the rollback step y <- y[:m] + [large model's token]; Section 3.4: the
 * predictions after the rolled-back position are discarded): which = 1 small, 2 large, 3 both; the cache(s) keep
 * their first pos rows (O(1): only a length changes).  BILD_EINVAL if pos exceeds
 * the current length of a selected cache.  y is not changed; a later pass simply
 * re-consumes the rows that were cut. */
int bild_kv_truncate(bild_state* s, int which, int pos);

/* Cuts the sequence to its first n_keep tokens (n_keep >= the initial length),
 * with draft_start and both caches cut to match, so that decoding continues
 * as if only that prefix had been generated. */
int bild_seq_truncate(bild_state* s, int n_keep);

/* Driver hook for tests and stress runs: overwrites y[first .. first+n) with
 * tokens (n may be 0), sets y_len = first + n and draft_start, and cuts both caches
 * back to the rows that are still valid (len_small <= first, len_large <=
 * min(first, draft_start - 1)); later passes re-consume what was cut.  Requires
 * initial length <= first <= y_len, initial length <= draft_start <= first + n,
 * first + n < max_len.  No model runs. */
int bild_force_tokens(bild_state* s, int first, const int32_t* tokens, int n, int draft_start);

/* Algorithm 1 end to end: encode(src), then small steps / large reviews until
 * max_new tokens exist or the last token equals eos (eos < 0: none).  out
 * (capacity max_new) receives the generated tokens without <s> / the prompt.
 * Equals the composition of the calls above.  src == NULL skips the encode step
 * and continues from the state as it is (max_new then counts all tokens after
 * the initial <s> / prompt); the same holds for bild_greedy. */
int bild_generate(bild_state* s, const int32_t* src, int n_src, float alpha_fb, float alpha_rb, int max_new,
                  int32_t eos, int32_t* out, int32_t* n_out, bild_stats* stats /* nullable */);

/* Vanilla inference with one model alone (which = 1 small, 2 large): greedy
 * autoregressive decoding, the baseline the paper normalises speedups to. */
int bild_greedy(bild_state* s, int which, const int32_t* src, int n_src, int max_new, int32_t eos,
                int32_t* out, int32_t* n_out);

/* The vocabulary sweep of a decoder pass as a call of its own (Section 3.2: each model maps its hidden state to
 * a distribution over the entire vocabulary; Sections 3.3 and 3.4 test max p and -ln p(draft) of it).  For each of
 * `rows` hidden rows (1..BILD_MAX_ROWS) the final RMSNorm of model m, its LM head and logit scale are applied and the
 * row's statistics are written: zmax = largest logit, lse = ln sum exp(logit), argmax (lowest id among equal
 * maxima) and z_target = logit of targets_dev[row] (NaN without targets or for an id outside the vocabulary), so
 * that max p = exp(zmax - lse) and -ln p(target) = lse - z_target.  Logits are never written to memory.
 * x_dev [rows][d_model] fp32 (16-byte aligned), targets_dev [rows] int32 (nullable) and out_dev [rows] are DEVICE
 * memory of the caller, read and written by kernels on hip_stream (NULL: the default stream).  The call allocates
 * a scratch buffer for its kernels' partial results and returns after the stream has finished with it. */
typedef struct bild_row_stats {
    float zmax;
    float lse;
    int32_t argmax;
    float z_target;
} bild_row_stats;
int bild_head_stats(const bild_model* m, const float* x_dev, int rows, const int32_t* targets_dev,
                    bild_row_stats* out_dev, void* hip_stream);
/* bild_head_stats for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same kernels, same results, but the scratch buffer is a
 * 4 MiB device array inside the library (one per GPU, held until the process ends), and the call neither allocates
 * nor frees anything and does not wait for the stream: it returns once its three kernels are enqueued on hip_stream.
 * Limit: the head's launch must not have more than 8191 workgroups (one 512-byte block of partial statistics each),
 * else BILD_ECAP; vocabularies up to 250112 at widths of 512 and 1024 are well inside it.  Every call on a GPU uses
 * that GPU's one array, which keeps the previous call's contents (the call clears what it reads before writing): calls
 * that overlap on one GPU - two streams, two threads - race; calls on one stream are ordered and safe. */
int bild_head_stats_static(const bild_model* m, const float* x_dev, int rows, const int32_t* targets_dev,
                           bild_row_stats* out_dev, void* hip_stream);

/* Introspection (host copies of the control block). */
int bild_get_lengths(bild_state* s, int32_t* y_len, int32_t* draft_start, int32_t* len_small, int32_t* len_large);
int bild_get_sequence(bild_state* s, int32_t* out, int cap, int32_t* n);

/* Test/debug: when enabled, each pass also writes its rows' full logits to a device
 * buffer that bild_debug_logits copies out ([rows][vocab] fp32, rows of the last pass
 * of model `which`).  Off by default: the product path never materialises logits. */
int bild_debug_enable_logits(bild_state* s, int enable);
int bild_debug_logits(bild_state* s, int which, int row, float* out_vocab);
/* Test/debug: copies cached self-attention keys (is_v = 0) or values (is_v = 1) of decoder layer `layer` of model
 * `which` for positions pos0 .. pos0+n-1 to out ([n][n_heads*d_head] fp32, host; bf16 storage is widened exactly).
 * Positions must lie below the model's consumed length.  BILD_EINVAL otherwise. */
int bild_debug_kv(bild_state* s, int which, int layer, int is_v, int pos0, int n, float* out);

const char* bild_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* BILD_H */
