/*
 * minions_verify.h: C ABI of the LLM verification step of aggregated speculative execution
 * (Minions, arXiv 2402.15678) for AMD MI355X (gfx950).
 *
 * One verification step is three calls on one HIP stream:
 *
 *   mn_mv_vote            tree-based weighted majority decision over the n SSM drafts of every
 *                         sequence (paper section 3.2, "Tree-based Weighted Majority Decision").
 *   mn_verify_forward     the LLM scores the pending token and the k_b voted tokens of every
 *                         sequence in one decoder forward against the existing paged KV cache and
 *                         takes the argmax per position (section 2.1; section 4, multi-token input
 *                         with an existing KV cache).
 *   mn_accept_and_commit  longest-prefix acceptance (the greedy case of section 2.1's rule) and
 *                         removal of the rejected tokens' KV entries (section 4).
 *
 * General rules
 *   - "dev" pointers are device (HBM) pointers, "host" pointers are host pointers.  The caller
 *     owns every buffer.  The library allocates no device memory, frees nothing of the caller's
 *     and keeps no reference to per-call buffers after the call returns.
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and performs no device synchronisation.
 *   - Every call returns an mn_status.  Problems the host can see (null pointer, bad shape,
 *     unsupported configuration, workspace too small) are reported before anything is launched.
 *     Problems only the device can see (a block table too short for a sequence, a block id out
 *     of range, a device spec_len that disagrees with the host copy) set bits in *dev_status
 *     (device int32, MN_DEV_* flags, OR-ed in; the caller zeroes it) and turn the affected
 *     sequence into a no-op: nothing of it is written to the cache, its outputs are -1 / 0.
 *   - Token ids are int32.  Padding value in voted/greedy/out_tokens is -1.
 *   - All matrices are [out][in] row-major: the contraction index is contiguous.
 */
#ifndef MINIONS_VERIFY_H
#define MINIONS_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mn_ctx mn_ctx; /* opaque; host memory only */

typedef enum {
  MN_OK = 0,
  MN_EINVAL = -1,       /* argument out of range */
  MN_ENULL = -2,        /* required pointer is NULL */
  MN_ESHAPE = -3,       /* shapes inconsistent with the model or with each other */
  MN_EUNSUPPORTED = -4, /* configuration not implemented (the message names it) */
  MN_ECAPACITY = -5,    /* host-visible capacity exceeded (e.g. max_ctx beyond the block table) */
  MN_EWORKSPACE = -6,   /* workspace smaller than mn_workspace_bytes() or misaligned */
  MN_EHIP = -7          /* a HIP call failed; mn_last_error() has the HIP error string */
} mn_status;

enum { MN_ARCH_OPT = 0, MN_ARCH_LLAMA = 1 };
enum { MN_DT_F32 = 0, MN_DT_BF16 = 1 };
enum { MN_VOTE_TREE = 0, MN_VOTE_COLUMN = 1 };
enum {
  MN_DEV_BLOCK_TABLE = 1, /* block table does not cover ctx_b + k_b + 1 tokens, or a block id is out of range */
  MN_DEV_SPEC_LEN = 2,    /* device spec_len differs from the host copy / exceeds k_max / is negative */
  MN_DEV_TOKEN = 4,       /* an input token id or position is outside the vocabulary / position table */
  MN_DEV_DRAFTS = 8,      /* mv_vote: spec_len outside [0, k_max] */
  MN_DEV_RANGE = 16,      /* bf16 models: a weight (mn_pack_weight) or an activation handed from one kernel to the next
                             lay outside the fp16 range +-65504 (or was not a number) and was saturated to the nearest
                             finite value.  Nothing is disabled: no infinity or NaN is produced, the call completes, but
                             the affected rows no longer follow the arithmetic stated at mn_verify_forward */
  MN_DEV_CTX = 32         /* ctx_b + k_b + 1 exceeds the max_ctx the host passed (the sequence is a no-op) */
};

/* Limits (checked; MN_EINVAL / MN_EUNSUPPORTED beyond them). */
#define MN_MAX_DRAFTS 64   /* n, SSMs per sequence */
#define MN_MAX_BATCH 4096  /* B */
#define MN_MAX_SPLIT_K 16

typedef struct {
  int arch;  /* MN_ARCH_OPT: LayerNorm, biases, ReLU FFN, learned absolute positions, n_kv_heads == n_heads.
                MN_ARCH_LLAMA: RMSNorm, no biases, SwiGLU FFN, rotary positions, grouped-query attention. */
  int dtype; /* storage type: MN_DT_F32 (matrices, embeddings and KV pages fp32) or MN_DT_BF16 (matrices and
                embeddings given as bf16; KV pages 16 bits per element too, in the fp16 encoding the library's
                products run in, see mn_kv).  Norm gains/shifts and biases are fp32 in both. */
  int n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int max_pos;     /* rows of pos_emb (OPT); upper bound on ctx_b + k_b + 1 in either arch */
  float norm_eps;  /* inside the square root of both norms */
  float rope_base; /* Llama: angle of pair (i, i + head_dim/2) at position p is p * base^(-2i/head_dim) */
} mn_model_desc;

/* Device pointers to the parameters.  The per-layer members are HOST arrays of n_layers device
 * pointers; mn_create copies the arrays (not the parameters).  Unused members are NULL.
 *   tok_emb [vocab][d]            pos_emb [max_pos][d] (OPT)       lm_head [vocab][d]
 *   final_norm_g/b [d]            (b: OPT only)
 *   ln1_g/ln1_b, ln2_g/ln2_b [d]  (b: OPT only)
 *   wqkv [(H + 2 Hkv) hd][d]      rows: all query heads, then all key heads, then all value heads
 *   bqkv [(H + 2 Hkv) hd] (OPT)   wo [d][H hd]    bo [d] (OPT)
 *   w1: OPT [F][d], Llama [2F][d] with rows [0,F) = gate and [F,2F) = up;  b1 [F] (OPT)
 *   w2 [d][F]                     b2 [d] (OPT)
 * Matrix layout.  fp32 models: row-major as written above.  bf16 models: the five matrices
 * (wqkv, wo, w1, w2, lm_head) must be in the library's packed streaming layout, produced from the
 * row-major matrix by mn_pack_weight (w1 of a Llama-style model with interleave_half = F); the
 * embedding tables stay row-major.
 */
typedef struct {
  const void *tok_emb, *pos_emb, *final_norm_g, *final_norm_b, *lm_head;
  const void *const *ln1_g, *const *ln1_b, *const *wqkv, *const *bqkv, *const *wo, *const *bo;
  const void *const *ln2_g, *const *ln2_b, *const *w1, *const *b1, *const *w2, *const *b2;
} mn_weights;

/* Paged KV cache (section 4: every cached token is addressed by a logical block id and an
 * offset).  Token p of sequence b is in physical block block_tables[b][p / block_size] at offset
 * p % block_size.  Per layer, fp32 in MN_DT_F32 models and IEEE fp16 in MN_DT_BF16 models (the cache is the
 * library's own state: it writes the rows and reads them back, and fp16 is what its matrix instructions multiply;
 * a bf16 value whose magnitude lies in [2^-14, 65504] is the same number in fp16, three mantissa bits to spare,
 * so a caller holding bf16 rows converts them without loss):
 *   K pages [num_blocks][n_kv_heads][head_dim/8][block_size][8]   (8 consecutive head-dim
 *                                                                  elements of one token together)
 *   V pages [num_blocks][n_kv_heads][head_dim][block_size]        (one head-dim element of the
 *                                                                  block's tokens together)
 * k_layers / v_layers are HOST arrays of n_layers device pointers, read at each call.
 * Rows at positions >= ctx_lens[b] are undefined; mn_verify_forward writes the k_b + 1 scored
 * tokens' rows there tentatively, only mn_accept_and_commit advances ctx_lens. */
typedef struct {
  void *const *k_layers;
  void *const *v_layers;
  int block_size;              /* tokens per block; the MFMA attention kernel needs 16 */
  int num_blocks;              /* physical blocks per layer */
  int max_blocks_per_seq;      /* row length of block_tables */
  const int32_t *block_tables; /* dev [B][max_blocks_per_seq] */
  int32_t *ctx_lens;           /* dev [B]; written only by mn_accept_and_commit */
} mn_kv;

/* ---- lifetime --------------------------------------------------------------------------- */

/* Validates the description, copies the pointer tables.  *out is NULL on failure; with out != NULL
 * a failed create leaves a message retrievable through mn_last_error(NULL). */
mn_status mn_create(mn_ctx **out, const mn_model_desc *desc, const mn_weights *weights);
void mn_destroy(mn_ctx *ctx);

/* Message of the last failed call on ctx (or of the last failed mn_create when ctx is NULL).
 * The string is owned by the library and valid until the next failing call on the same ctx. */
const char *mn_last_error(const mn_ctx *ctx);
const char *mn_status_str(mn_status s);

/* Bytes of device workspace mn_verify_forward needs for at most max_rows = sum_b (k_b + 1) scored
 * positions, B sequences and contexts up to max_ctx tokens (including the scored ones).
 * The workspace must be 256-byte aligned.  Returns 0 on invalid arguments. */
size_t mn_workspace_bytes(const mn_ctx *ctx, int B, int max_rows, int max_ctx);

/* ---- weight packing (bf16 models) ---------------------------------------------------------------
 * HBM streams near its peak only over long contiguous runs, so the projection kernel reads its
 * weights pre-tiled: blocks of 128 output columns x 128 inputs, 32 KB each, consecutive along k for
 * one column block, every 1 KB inside in the order the MFMA lanes consume it, every value re-encoded
 * from bf16 to the fp16 the MFMA multiplies (still two bytes; exact for magnitudes in [2^-14, 65504],
 * smaller ones truncated to the fp16 subnormal grid, an absolute error below 2^-24; larger ones, which
 * trained or initialised weights do not hold, are saturated to +-65280, the largest bf16 value fp16 can
 * hold, and reported).  Columns are padded with zeros to a multiple of 128.  The packed form is private to
 * this library version. */

/* Bytes of the packed form of an [N][K] bf16 matrix (K a multiple of 128).  0 on invalid arguments. */
size_t mn_packed_weight_bytes(int N, int K);

/* src dev [N][K] bf16 row-major -> dst dev packed (mn_packed_weight_bytes(N, K) bytes, 256-byte
 * aligned, not overlapping src).  interleave_half = 0 keeps the row order.  interleave_half = F > 0
 * (N must be 2F, F a multiple of 16) is for the gate||up matrix of a SwiGLU FFN: packed column tile
 * 2t holds gate rows [16t, 16t+16) and tile 2t+1 up rows F + [16t, 16t+16), which lets the
 * projection kernel apply silu(gate) * up in its epilogue.
 * dev_status (dev [1] int32, flags OR-ed in, or NULL): MN_DEV_RANGE when a weight was saturated. */
mn_status mn_pack_weight(const void *src, void *dst, int N, int K, int interleave_half, int32_t *dev_status,
                         void *stream);

/* ---- the verification step --------------------------------------------------------------- */

/* Majority vote (section 3.2).  For every sequence b the n drafts drafts[b][j][0..k_b) form a
 * token tree rooted at the last committed token; a node's weight is the fp32 sum, in ascending
 * draft order, of ssm_w[j] over the drafts passing through it; from the root the heaviest child
 * is taken at every level (ties: the child whose first supporting draft has the lowest index).
 * voted[b][0..k_b) is the chosen branch (positions >= k_b are set to -1) and voted_ssm[b] the
 * lowest-index draft equal to it (the paper's voted_SSM).
 * mode MN_VOTE_COLUMN votes every position over all n drafts without the prefix filter;
 * voted_ssm is then the lowest-index draft equal to the result, or -1 if there is none.
 *   drafts    dev [B][n][k_max] int32          spec_len  dev [B] int32, 0 <= k_b <= k_max
 *   ssm_w     dev [n] fp32                     voted     dev [B][k_max] int32 (out)
 *   voted_ssm dev [B] int32 (out)              dev_status dev [1] int32 (flags OR-ed in) or NULL
 * Limits: 1 <= n <= MN_MAX_DRAFTS, 0 <= k_max, 0 <= B <= MN_MAX_BATCH (B = 0 is a no-op).
 * ctx may be NULL (the vote does not depend on the model). */
mn_status mn_mv_vote(mn_ctx *ctx, const int32_t *drafts, const int32_t *spec_len, const float *ssm_w, int B, int n,
                     int k_max, int mode, int32_t *voted, int32_t *voted_ssm, int32_t *dev_status, void *stream);

/* Verification forward (sections 2.1 and 4).  Sequence b contributes q_b = k_b + 1 rows: input
 * tokens [last_tok[b], voted[b][0..k_b)] at positions ctx_b .. ctx_b + k_b.  Row j attends to
 * the cached tokens [0, ctx_b) and to rows 0..j of its own sequence (causal among the speculated
 * tokens).  The rows' K/V are written into the cache at their positions (tentatively, beyond
 * ctx_lens).  greedy[b][j] = lowest token id attaining the maximum logit of row j, j <= k_b;
 * entries j > k_b are set to -1.  With ctx_b = 0 this call is a prefill.
 *   last_tok   dev [B]            voted dev [B][k_max] (ignored where k_max == 0; may be NULL then)
 *   spec_len   dev [B]            h_spec_len HOST [B], the same values: they size the launch
 *   max_ctx    upper bound on ctx_b + k_b + 1 over the batch (sizes the attention launch)
 *   greedy     dev [B][k_max+1] (out)
 *   logits     dev [sum_b q_b][vocab] fp32 (out), rows packed in sequence order, or NULL
 *   workspace  dev, >= mn_workspace_bytes(ctx, B, sum_b q_b, max_ctx), 256-byte aligned
 * Arithmetic: fp32 residual stream, norm statistics, softmax and logits in both storage types.
 * With MN_DT_BF16 the weights are given as bf16 and re-encoded as fp16 by mn_pack_weight (same 16 bits
 * per parameter; exact for magnitudes in [2^-14, 65504], the range weights live in), cache entries
 * are fp16; the activations fed to the matrix products (norm outputs, queries, softmax
 * probabilities, attention outputs, FFN activations) are rounded to fp16 (round-to-nearest-even)
 * and the products run on the fp16 MFMA with fp32 accumulation.  New K/V rows are rounded to
 * fp16 when they are written to the cache, and the attention of the same call reads them from there, as
 * every later call does: scoring k + 1 positions in one pass multiplies exactly the numbers that k + 1
 * single-position calls multiply (section 2.1: the LLM scores the speculated tokens in parallel with the
 * outcome of scoring them one by one); what is left between the two is the order of the fp32 sums.
 * Range of the fp16 stages: every such activation (and every K/V row written to the cache) is saturated to
 * +-65504 instead of overflowing to infinity, and MN_DEV_RANGE is set in *dev_status when that happens
 * (with N(0, 0.02)-initialised or trained weights these values stay below 10^2).  Cache entries the caller
 * supplies must lie within +-65504 as well.
 * max_ctx is checked on the device against ctx_lens: a sequence with ctx_b + k_b + 1 > max_ctx sets MN_DEV_CTX
 * and becomes a no-op (the attention launch was sized for max_ctx keys). */
mn_status mn_verify_forward(mn_ctx *ctx, const int32_t *last_tok, const int32_t *voted, const int32_t *spec_len,
                            const int32_t *h_spec_len, int B, int k_max, int max_ctx, const mn_kv *kv,
                            int32_t *greedy, float *logits, void *workspace, size_t workspace_bytes,
                            int32_t *dev_status, void *stream);

/* Acceptance and commit (section 2.1, greedy case; section 4).  a_b = length of the longest prefix
 * of voted[b][0..k_b) equal to greedy[b][0..k_b).  The step emits the a_b + 1 tokens
 * greedy[b][0..a_b] (the last one corrects the first mismatch, or is the bonus token when
 * a_b == k_b).  The cache keeps the pending token and the a_b accepted drafts:
 * ctx_lens[b] += a_b + 1; the k_b - a_b rejected tokens' entries fall outside ctx_lens and are
 * thereby deleted (the accepted set is a prefix, so nothing moves).
 *   accepted_len dev [B] (out)            out_tokens dev [B][k_max+1] (out, padded with -1)
 *   n_out dev [B] (out) = a_b + 1         next_last_tok dev [B] (out) = greedy[b][a_b]
 *   blocks_in_use dev [B] (out) = ceil(ctx_lens[b] / block_size) after the commit
 * A sequence whose greedy[b][0] is -1 (made a no-op by mn_verify_forward) keeps its ctx_lens and
 * reports accepted_len = 0, n_out = 0, next_last_tok = -1.  ctx may be NULL. */
mn_status mn_accept_and_commit(mn_ctx *ctx, const int32_t *voted, const int32_t *greedy, const int32_t *spec_len,
                               int B, int k_max, mn_kv *kv, int32_t *accepted_len, int32_t *out_tokens,
                               int32_t *n_out, int32_t *next_last_tok, int32_t *blocks_in_use,
                               int32_t *dev_status, void *stream);

/* Stochastic verification (section 2.1, the general rule; the greedy tokens of mn_verify_forward are its
 * temperature -> 0 case).  With o_j = softmax(logits row of position j / temperature) and q_j the
 * drafting SSM's distribution at that position, the speculated token x = voted[b][j] survives when
 * q_j(x) <= o_j(x), and otherwise with probability o_j(x) / q_j(x); where it does not survive, a
 * replacement is drawn from max(0, o_j - q_j) renormalised (should that be zero everywhere, which only a
 * draft_probs row summing above 1 can cause: from o_j without the token x; should o_j have no other mass
 * either, x stays); at position k_b, after the last speculated token, a token is drawn from o_{k_b}.
 * The result is written in the layout of `greedy`: sampled[b][j] = voted[b][j] where the token
 * survived, the drawn token elsewhere, -1 beyond k_b.  A replacement never equals the token it
 * replaces, so mn_accept_and_commit(voted, sampled, ...) then yields exactly the rule's output: the
 * survivors before the first rejection plus the replacement (or the bonus token), and the cache commit.
 * Every position is decided independently of the others (entries after the first rejection are
 * computed and then ignored by the acceptance).
 *   logits      dev [M][vocab] fp32, rows packed as by mn_verify_forward (sequence b's k_b + 1 rows
 *               follow those of sequence b - 1); M = sum_b (spec_len[b] + 1)
 *   voted       dev [B][k_max]            draft_probs dev [B][k_max][vocab] fp32: q_j of the SSM whose
 *   spec_len    dev [B]                   draft was voted (used as given, not renormalised)
 *   greedy      dev [B][k_max+1] from mn_verify_forward: a sequence with greedy[b][0] == -1 (a no-op
 *               there) gets sampled[b][*] = -1 and stays a no-op in mn_accept_and_commit
 *   sampled     dev [B][k_max+1] (out)
 * Arithmetic is fp64.  Random numbers: Philox-4x32-10 with key = seed and counter = (b, j, step); the
 * first two output words give the 53-bit uniform number of the survival test (top 27 bits of word 0,
 * top 26 of word 1), the last two that of the draw, which takes the first token, in token order, whose
 * running sum of mass exceeds u times the total.  The same (seed, step, b, j) always gives the same
 * numbers: the caller advances `step` once per verification step.  The top byte of the counter's last
 * word (above the 56 bits of `step`) is 0 here and 1 + i for drafting SSM i (mn_draft_sample), so one seed
 * serves all of them without shared numbers.
 * Scores may be minus infinity (masked tokens: no mass); every row needs a finite maximum.
 * Errors: temperature must be positive and finite; step < 2^56; vocab <= 2^21; k_max <= 4096.  Rows that do not add
 * up to M set MN_DEV_SPEC_LEN in *dev_status and give -1.  ctx may be NULL. */
mn_status mn_verify_sample(mn_ctx *ctx, const float *logits, const int32_t *voted, const float *draft_probs,
                           const int32_t *spec_len, const int32_t *greedy, int B, int k_max, int M, int vocab,
                           double temperature, uint64_t seed, uint64_t step, int32_t *sampled, int32_t *dev_status,
                           void *stream);

/* The drafting side of the stochastic rule (section 2.1: the SSM predicts its tokens from its own
 * distribution q).  For each sequence b, q_b = softmax(logits[b] / temperature) is rounded to fp32 and,
 * when probs is given, written to probs[b * probs_stride + v]; the token is drawn from exactly those
 * fp32 values (inverse CDF in token order, as in mn_verify_sample) and written to
 * tokens[b * token_stride].  The strides (in elements) let the caller aim both at their final place:
 * tokens at drafts[b][ssm][t] of mn_mv_vote's input (stride n * k_max), probs at row [b][t] of a
 * [B][k_max][vocab] array (stride k_max * vocab) that mn_verify_sample reads for the SSM whose draft wins
 * the vote.
 *   logits dev [B][vocab] fp32: one row per sequence (an SSM's mn_verify_forward with spec_len = 0)
 * Random numbers: Philox-4x32-10, key = seed, counter = (b, t, step, consumer 1 + ssm); words 2, 3 give
 * the uniform number of the draw.  0 <= ssm < MN_MAX_DRAFTS, t >= 0, step < 2^56, temperature positive
 * and finite, vocab <= 2^21, token_stride >= 1, probs_stride >= vocab.  ctx may be NULL. */
mn_status mn_draft_sample(mn_ctx *ctx, const float *logits, int B, int vocab, double temperature, uint64_t seed,
                          uint64_t step, int ssm, int t, int32_t *tokens, long token_stride, float *probs,
                          long probs_stride, void *stream);

/* ---- after the step: closing the loop (sections 3.2 and 3.3) --------------------------------- */

/* Speculation quality metric and SSM weight update (section 3.2, equation ACR).  For every SSM i,
 * ACR_i = mean over the verified outputs b whose voted_ssm[b] == i of accepted_len[b] / spec_len[b]
 * (fp64, outputs taken in ascending b; outputs with spec_len[b] <= 0, or with n_out[b] <= 0 when n_out
 * is given, i.e. not verified by this step, are not in the set).  ssm_w[i] is multiplied (fp32) by
 * reward_factor when ACR_i > reward_threshold and by punish_factor when ACR_i < punish_threshold; an
 * SSM that won no vote keeps its weight and reports NaN.  The paper leaves the four constants to the
 * operator; they are arguments here.
 *   voted_ssm dev [B] (from mn_mv_vote)      accepted_len, n_out dev [B] (from mn_accept_and_commit;
 *   spec_len  dev [B]                         n_out may be NULL)
 *   ssm_w     dev [n] fp32, updated in place (the next mn_mv_vote reads it: no host round trip)
 *   acr       dev [n] fp64 (out) or NULL
 * 1 <= n <= MN_MAX_DRAFTS, 0 <= B <= MN_MAX_BATCH, factors > 0, punish_threshold <= reward_threshold.
 * ctx may be NULL. */
mn_status mn_acr_update(mn_ctx *ctx, const int32_t *voted_ssm, const int32_t *accepted_len, const int32_t *spec_len,
                        const int32_t *n_out, int B, int n, double reward_threshold, double punish_threshold,
                        float reward_factor, float punish_factor, float *ssm_w, double *acr, void *stream);

/* Adaptive speculation length selector (section 3.3).  Host-side state, no device work.  Every
 * verification step contributes one sample t_llm / vl (step time over the average number of tokens
 * a request gained from the step).  When decision_threshold samples have been collected since the
 * last change (the text's "greater than or equal"; the listing's strict comparison differs by one
 * sample), the least-squares line through (0, y_0) .. (m-1, y_{m-1}) is fitted: slope > 0 lowers s by
 * s_penalty, any other slope raises it by s_reward (the listing's else branch); s is clamped to
 * [s_min, s_max] and the samples are discarded.
 * mn_selector_create: 0 <= s_min <= s_init <= s_max, decision_threshold >= 2, s_penalty, s_reward >= 0.
 * mn_selector_observe: t_llm >= 0 and vl > 0, both finite (MN_EINVAL otherwise, nothing recorded);
 * *s_out (may be NULL) = the speculation length to use next; *slope_out (may be NULL) = the fitted slope
 * when this call triggered a decision, NaN otherwise.  The caller owns the object; calls on one object
 * must not overlap. */
typedef struct mn_selector mn_selector;
mn_status mn_selector_create(mn_selector **out, int s_init, int s_min, int s_max, int decision_threshold,
                             int s_penalty, int s_reward);
void mn_selector_destroy(mn_selector *sel);
mn_status mn_selector_observe(mn_selector *sel, double t_llm, double vl, int *s_out, double *slope_out);
int mn_selector_current(const mn_selector *sel);   /* -1 when sel is NULL */
long mn_selector_adjustments(const mn_selector *sel); /* decisions taken so far; -1 when sel is NULL */

/* ---- measuring sticks (no part of the method) ---------------------------------------------------
 * For callers who cannot bring their own microbenchmarks: what a plain streaming read and a dense fp16
 * MFMA loop sustain on the chip at hand, to read the roofline fractions against.  The caller times the
 * launches (events on `stream`).
 * mn_probe_stream_read: one pass over buf (dev, 16-byte aligned, >= 1 MiB; bytes / time = read rate).
 * mn_probe_mfma: every SIMD runs iters x 32 independent 16x16x32 fp16 MFMAs on two waves (1 <= iters <=
 * 2^22, else MN_EINVAL); *flop (HOST, may be NULL) receives the floating-point operations of the launch.
 * Every operand element is the constant 0.5: the rate of the matrix pipe at the boost clock.
 * mn_probe_mfma_data: the same loop on operands of random sign and mantissa (magnitudes in [0.5, 1)):
 * the rate the chip sustains once the multipliers toggle as they do on data and the power management
 * has settled the clock; a dense product is to be read against this one. */
mn_status mn_probe_stream_read(const void *buf, size_t bytes, void *stream);
mn_status mn_probe_mfma(int iters, double *flop, void *stream);
mn_status mn_probe_mfma_data(int iters, double *flop, void *stream);

/* ---- component entry points (the kernels mn_verify_forward is made of, at their own shapes) -- */

/* The projection GEMM of a bf16 model: out[m][n] = sum_k a[m][k] * w[n][k] (+ bias[n]).
 * a dev [M][K] fp16 (the activation type of bf16 models), w dev: the [N][K] bf16 matrix in packed
 * layout (mn_pack_weight with interleave_half = 0, which also re-encodes the values as fp16),
 * fp16 MFMA with fp32 accumulation, bias dev [N] fp32 or NULL, out dev [M][N]
 * fp32.  split_k in [0, MN_MAX_SPLIT_K]: 0 lets the library choose; with split_k > 1 `workspace`
 * (dev, >= split_k*M*N*4 bytes, 256-byte aligned) holds the partial sums, which are added in a
 * fixed order.  K must be a multiple of 128; M >= 0, N >= 1 arbitrary. */
mn_status mn_proj_gemm(mn_ctx *ctx, const void *a, const void *w, const float *bias, float *out, int M, int N, int K,
                       int split_k, void *workspace, size_t workspace_bytes, void *stream);

/* mn_proj_gemm for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc, and callers with no device memory to spare for a workspace.  Same operation, same
 * kernels and the same bits in `out` as mn_proj_gemm with the same arguments; the split-K partial sums go to a
 * buffer built into the library (MN_NOALLOC_SCRATCH_BYTES of device memory per GPU, a static array of the
 * library's device code which the runtime places when the first call on that GPU looks it up, and which
 * stays until the process ends) instead of a workspace.  The call allocates and
 * frees nothing, on the device or through any library, and clears nothing (every partial sum it reads it has
 * written itself).  a, w, bias, out, M, N, K, split_k as for mn_proj_gemm.
 * Errors: MN_ECAPACITY when split * M * N * 4 bytes exceed MN_NOALLOC_SCRATCH_BYTES (split = split_k, or the
 * library's choice when split_k == 0; nothing is launched; pass a smaller split_k or use mn_proj_gemm);
 * MN_EUNSUPPORTED on a device ordinal above 63; otherwise as mn_proj_gemm.
 * All calls on one GPU share that GPU's buffer, which keeps the previous call's contents: calls that overlap on
 * one GPU (different streams, or different host threads without ordering between their streams) race; calls on
 * one stream, or ordered by events, are safe. */
#define MN_NOALLOC_SCRATCH_BYTES (32u << 20)
mn_status mn_proj_gemm_noalloc(mn_ctx *ctx, const void *a, const void *w, const float *bias, float *out, int M, int N,
                               int K, int split_k, void *stream);

/* Multi-token paged attention of one layer (section 4) on caller-supplied queries.  Rows are
 * packed as in mn_verify_forward: sequence b has q_b = h_spec_len[b] + 1 query rows at positions
 * ctx_b .. ctx_b + q_b - 1, whose K/V must already be in the cache.
 *   q   dev [sum_b q_b][n_heads][head_dim]   fp32 in fp32 models, fp16 in bf16 models
 *   out dev [sum_b q_b][n_heads*head_dim]    same type as q
 *   layer selects kv->k_layers[layer] / v_layers[layer].
 * Uses the model's head counts and head_dim; workspace as for mn_verify_forward. */
mn_status mn_attention(mn_ctx *ctx, const void *q, const int32_t *spec_len, const int32_t *h_spec_len, int B,
                       int max_ctx, const mn_kv *kv, int layer, void *out, void *workspace, size_t workspace_bytes,
                       int32_t *dev_status, void *stream);

/* ---- timing taps (for benchmarks; off by default) --------------------------------------------- */

/* Kernel families of the step, as indexed in mn_profile_collect's arrays. */
enum {
  MN_PROF_PREPARE = 0, MN_PROF_NORM = 1, MN_PROF_GEMM = 2, MN_PROF_ROPE_APPEND = 3, MN_PROF_ATTENTION = 4,
  MN_PROF_ACT = 5, MN_PROF_ARGMAX = 6, MN_PROF_VOTE = 7, MN_PROF_ACCEPT = 8, MN_PROF_KINDS = 9
};

/* With on != 0 every later call on ctx brackets each kernel-family launch with a pair of HIP events
 * on the call's stream (host-side objects; no device memory is allocated).  The taps cost a few
 * microseconds of stream time per launch, so throughput is measured with them off. */
mn_status mn_profile_enable(mn_ctx *ctx, int on);

/* After the caller has synchronised the stream: ms[kind] = summed device time of the launches of
 * that family since the last collect, counts[kind] = number of launches.  Both arrays hold
 * MN_PROF_KINDS entries.  Resets the taps. */
mn_status mn_profile_collect(mn_ctx *ctx, double *ms, int *counts);

#ifdef __cplusplus
}
#endif
#endif /* MINIONS_VERIFY_H */
