/*
 * csd.h — C ABI of the MI355X (gfx950) verify path of Cascade Speculative Drafting.
 *
 * One verify step of the cascade is three calls:
 *   csd_bigram_draft   the statistical model at the bottom of both cascades drafts k tokens
 *                      (Max-Gram with a bigram fallback; Section 3.3, Appendix A);
 *   csd_verify_block   the reviewing model runs once over the whole drafted block against
 *                      its KV cache and yields one distribution per position (Section 2);
 *   csd_accept         speculative-sampling review: keep a prefix of the drafts, replace the
 *                      first rejected one, or append one extra token (Section 2), with
 *                      lenience and the greedy rule of Section 3.1.
 *
 * Conventions that hold for every call:
 *   - The return value is a status: CSD_OK, or a negative CSD_E* code.  Nothing throws, logs
 *     or synchronises the host with the device.
 *   - Every array argument is a DEVICE pointer owned by the caller and must stay valid until
 *     the stream has executed the work, unless the comment says "host".
 *   - `stream` is a hipStream_t passed as void*; all work is enqueued on it, in order.
 *   - Outputs are fully overwritten.  Inputs are never modified, except the KV cache.
 *   - After csd_model_create nothing allocates device memory; scratch lives in the model, so
 *     two calls that use the same model must not overlap (use one stream per model).
 *   - Arguments are validated on the host before anything is enqueued; on error nothing is
 *     enqueued.  Values that live on the device (token ids, lengths) cannot be validated by
 *     the host: kernels clamp their own accesses and out-of-range ids give -1 outputs
 *     (draft) or an all-zero embedding row (verify).
 */
#ifndef CSD_H
#define CSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CSD_OK       0
#define CSD_EINVAL  (-1)  /* a scalar argument is out of its domain                         */
#define CSD_ESHAPE  (-2)  /* a size exceeds what the model / kernel was created for         */
#define CSD_ENULL   (-3)  /* a required pointer is NULL                                     */
#define CSD_EHIP    (-4)  /* a HIP call failed; see csd_last_hip_error()                    */
#define CSD_EUNSUPPORTED (-5) /* configuration not implemented (e.g. arch > 1)              */

#define CSD_DTYPE_FP32 0
#define CSD_DTYPE_BF16 1
#define CSD_MODE_SAMPLE 0
#define CSD_MODE_GREEDY 1

/* Reviewing-model description (Section 5.1 names the families; the benchmark configurations give
 * the shapes).  arch 0 is the LLaMA-style decoder: RMSNorm, rotary embedding (half-split pairing,
 * K cached after rotation), causal attention scaled by 1/sqrt(head_dim), SwiGLU, no biases, untied
 * LM head.  arch 1 is the T5-style decoder: RMS layer norm, no rotary embedding, unscaled causal
 * self-attention with a bucketed relative-position bias (32 buckets, maximum distance 128, one
 * table for all layers), unmasked cross-attention over a fixed encoder output of enc_len rows, gated
 * tanh-GELU feed-forward, untied LM head. */
typedef struct csd_model_cfg {
    int32_t arch;        /* 0 or 1                                                          */
    int32_t dtype;       /* CSD_DTYPE_*: storage type of the matrices and of the KV cache;  */
                         /* norm gains, logits and probabilities are always fp32            */
    int32_t n_layers, d_model, n_heads, head_dim, d_ffn, vocab;
    int32_t max_batch;   /* most sequences per call                                         */
    int32_t max_seq;     /* rows per sequence in the KV cache                               */
    int32_t max_block;   /* most block rows m = k+1 per sequence per call                   */
    int32_t enc_len;     /* arch 1: rows of the encoder output per sequence (>= 1); arch 0: 0 */
    float   rms_eps, rope_theta;
} csd_model_cfg;

typedef struct csd_model csd_model;   /* opaque; owns its packed copy of the weights + scratch */

/* Library identification (host string, static storage). */
const char *csd_version(void);
/* hipError_t of the most recent failing HIP call made by this library on this thread's
 * behalf (0 if none). */
int32_t csd_last_hip_error(void);

/*
 * Build a model from caller-owned device tensors.  weight_ptrs is a HOST array of n_weights
 * device pointers in canonical order:
 *   embed[V][d], then per layer: attn_norm[d], wq[d][H*dh], wk, wv, wo[H*dh][d], ffn_norm[d],
 *   w_gate[d][F], w_up[d][F], w_down[F][d]; then final_norm[d], lm_head[d][V].
 * Matrices are row-major [in][out] in cfg->dtype; norm gains are fp32.  The weights are
 * copied (re-tiled for the MFMA kernels when dtype is bf16); the caller may free its tensors
 * once the stream has passed this call.  Allocates weights + scratch; this is the only
 * allocating call besides destroy.  n_weights must be 3 + 9*n_layers.  The packing kernels and the
 * clearing of the model's counters run on `stream`: later calls that use the model must be ordered behind
 * this one on the device (the same stream, or an event).
 * arch 1: per layer self_norm[d], wq, wk, wv, wo, cross_norm[d], cq[d][H*dh], ck, cv, co[H*dh][d],
 * ffn_norm[d], w0[d][F] (through the GELU), w1[d][F], w_out[F][d]; then final_norm[d], lm_head[d][V],
 * rel_bias[32][H] (fp32 whatever dtype is); n_weights must be 4 + 14*n_layers.
 */
int32_t csd_model_create(const csd_model_cfg *cfg, const void *const *weight_ptrs, int32_t n_weights,
                         void *stream, csd_model **out);
/* Frees everything the model owns.  The caller synchronises its streams first. */
int32_t csd_model_destroy(csd_model *model);

/* Size in bytes of the KV cache the caller must allocate (256-byte aligned) for
 * max_batch x max_seq rows.  The layout is private to the library; use csd_kv_write /
 * csd_kv_read to move rows in canonical form. */
size_t csd_kv_bytes(const csd_model *model);

/* arch 1, once per prompt (Section 5.1's encoder-decoder reviewers attend a fixed encoder output):
 * project enc_out (device, fp32 [B][enc_len][d_model], values taken as exact in the model dtype) to
 * the cross-attention keys and values of every layer and store them in the second part of the cache
 * `kv` (sequences 0..B-1).  Must precede the first csd_verify_block on that cache.
 * CSD_EUNSUPPORTED for arch 0. */
int32_t csd_cross_kv_init(csd_model *model, void *kv, const float *enc_out, int32_t B, void *stream);

/* Copy n rows [pos0, pos0+n) of sequence b, layer `layer` into / out of the cache.
 * K and V are fp32 [n][H*dh] (K as cached, i.e. after rotation); values are rounded to the
 * cache dtype on write (round-to-nearest-even).  These address the self-attention rows only. */
int32_t csd_kv_write(const csd_model *model, void *kv, int32_t layer, int32_t b, int32_t pos0, int32_t n,
                     const float *K, const float *V, void *stream);
int32_t csd_kv_read(const csd_model *model, const void *kv, int32_t layer, int32_t b, int32_t pos0, int32_t n,
                    float *K, float *V, void *stream);

/*
 * Fit the bigram fallback table of Max-Gram on a token stream (Section 3.3; one parameter per
 * vocabulary entry, Section 5.2): next_table[a] = the successor of a with the highest count;
 * equal counts: the pair whose last occurrence is latest.  Entries of tokens with no
 * successor in the stream keep the value the caller pre-filled.  n <= 8192.
 */
int32_t csd_bigram_fit(const int32_t *tokens, int32_t n, int32_t vocab, int32_t *next_table, void *stream);

/*
 * Max-Gram draft (Section 3.3, Appendix A).  ctx[B][ctx_stride] holds each sequence (prompt
 * + generation so far), ctx_len[B] its length (1 <= len <= ctx_stride).  For each sequence:
 * find the longest suffix that also ends at an earlier position e <= len-2 (the left-most e
 * among the longest; match length optionally capped by max_match > 0) and emit the k tokens
 * that follow e, reading on into the draft itself when the sequence ends.  If even the last
 * token never occurred before, chain next_table from it.  out_tokens[B][k];
 * out_match_len[B] (optional) receives the match length, 0 for the fallback.
 */
int32_t csd_bigram_draft(const int32_t *ctx, const int32_t *ctx_len, int32_t B, int32_t ctx_stride,
                         const int32_t *next_table, int32_t vocab, int32_t k, int32_t max_match,
                         int32_t *out_tokens, int32_t *out_match_len, void *stream);

/*
 * Max-Gram with a haystack of its own (Appendix A: the listing searches the encoder's ids for the longest
 * suffix of the decoder's ids; Section 3.3: "the initial input (or existing generation)").  For each sequence:
 * the longest suffix of needle[0 .. needle_len) that ends at some haystack position e (the left-most e among
 * the longest; length optionally capped by max_match > 0), then the tokens haystack[e+1 ..] while the haystack
 * lasts: out_n_copied[B] (optional) receives how many of the k tokens that is, which is exactly what Appendix A
 * returns (possibly none).  The remaining positions, and all k when even the needle's last token does not occur
 * in the haystack (out_match_len 0), chain next_table from the last token so far (the bigram fallback of
 * Section 3.3), so out_tokens[B][k] is always full.  haystack_len >= 0, 1 <= needle_len <= needle_stride.
 */
int32_t csd_maxgram_draft(const int32_t *haystack, const int32_t *haystack_len, int32_t haystack_stride,
                          const int32_t *needle, const int32_t *needle_len, int32_t needle_stride, int32_t B,
                          const int32_t *next_table, int32_t vocab, int32_t k, int32_t max_match,
                          int32_t *out_tokens, int32_t *out_match_len, int32_t *out_n_copied, void *stream);

/*
 * Review forward (Section 2: the reviewer scores all drafted positions in one run).
 * tokens[B][m]: row 0 is the last committed token of the sequence (not yet in the cache),
 * rows 1..m-1 are the drafts.  cache_len[B]: rows of the cache that are valid.  Row i sits at
 * position cache_len[b]+i, attends cache rows 0..cache_len[b]+i, and its K/V are written
 * there unconditionally; rows beyond what the caller later commits are simply overwritten
 * by the next block (no rollback needed after a rejection).
 * logits[B][m][V] fp32 (row i = distribution of the token after row i).  probs: optional
 * softmax(logits / temperature), temperature > 0 required when probs != NULL.
 * 1 <= B <= max_batch, 1 <= m <= max_block; cache_len[b]+m <= max_seq is the caller's duty.
 */
int32_t csd_verify_block(csd_model *model, void *kv, const int32_t *tokens, const int32_t *cache_len,
                         int32_t B, int32_t m, float temperature, float *logits, float *probs, void *stream);

/*
 * Speculative-sampling review of k drafts per sequence (Section 2; lenience and greedy rule:
 * Section 3.1).  p[B][k+1][V]: reviewer rows (row i scores draft i; row k is the extra
 * token); probabilities for CSD_MODE_SAMPLE; logits are enough for CSD_MODE_GREEDY with
 * lenience 1.  q[B][k][V]: draft distributions, or NULL when every draft was deterministic;
 * q_onehot[k] (optional, device) marks positions whose draft was deterministic (Max-Gram)
 * although q is given.  draft[B][k]; u_acc[B][k] and u_samp[B]: uniforms in [0,1).
 *   sample: keep draft i iff fl32(u_i*q_i(x_i)) < fl32(l*p_i(x_i)); at the first rejection
 *           draw from norm(max(0, l*p_i - q_i)) (all-zero: from p_i); no rejection: draw the
 *           extra token from row k.  Draws use an exact 40-bit fixed-point inverse CDF in
 *           increasing token id, so the result does not depend on reduction order.
 *   greedy: keep draft i iff it is the arg-max of row i (ties: smallest id) or, for l > 1
 *           (p must then hold probabilities), q_i(x_i) <= fl32(l*p_i(x_i)); emit the arg-max
 *           of the row after the kept drafts.
 * n_accepted[B] in [0,k]; next_token[B].  1 <= lenience <= 256; k >= 0; V >= 1.
 * A draft id outside [0, V) cannot be checked on the host (the drafts are on the device): the
 * kernel treats it as a rejection at that position and draws the replacement from p_i.
 * next_token is -1 for a row of p that is not a distribution (all weights zero).
 */
int32_t csd_accept(const float *p, const float *q, const uint8_t *q_onehot, const int32_t *draft,
                   const float *u_acc, const float *u_samp, int32_t B, int32_t k, int32_t V,
                   float lenience, int32_t mode, int32_t *n_accepted, int32_t *next_token, void *stream);

/*
 * csd_verify_block followed by csd_accept on the block's own rows, in one enqueue
 * (k = m-1 drafts = tokens[b][1..m-1]): the same decisions, bit for bit, as the two calls on the
 * probabilities csd_verify_block would write (Section 2: the review of a block is one run of the
 * reviewer followed by the accept rule).  logits and probs are optional outputs here: without probs
 * no probability is written anywhere (softmax, the tests of all rows and the draw run in one launch
 * behind the forward; vocabularies above 32768 or not a multiple of 4 take softmax and review as two).
 */
int32_t csd_verify_accept(csd_model *model, void *kv, const int32_t *tokens, const int32_t *cache_len,
                          int32_t B, int32_t m, float temperature,
                          const float *q, const uint8_t *q_onehot, const float *u_acc, const float *u_samp,
                          float lenience, int32_t mode, float *logits, float *probs,
                          int32_t *n_accepted, int32_t *next_token, void *stream);

/*
 * csd_verify_accept for callers that cannot allocate and do not want the call to touch memory that a
 * hipMalloc of this library returned for scratch: code under HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, same results, same kernels; the per-call scratch
 * (residual stream, GEMM input planes, split-K partial sums, attention partial states, probabilities) lives
 * in a static device array of CSD_STATIC_SCRATCH_BYTES per GPU instead of in the model, and the call makes
 * no hipMalloc / hipFree (nor does any other call after csd_model_create).
 *   CSD_ESHAPE        the model's scratch (it grows with max_batch * max_block and the widest matrix) does not
 *                     fit the static array.
 * Every call on a GPU shares that GPU's array, whatever the model or stream: calls that overlap on one GPU
 * race.  The call clears the few counters in it that must start at zero and overwrites everything else it reads.
 */
#define CSD_STATIC_SCRATCH_BYTES (8u << 20)
int32_t csd_verify_accept_static(csd_model *model, void *kv, const int32_t *tokens, const int32_t *cache_len,
                                 int32_t B, int32_t m, float temperature,
                                 const float *q, const uint8_t *q_onehot, const float *u_acc, const float *u_samp,
                                 float lenience, int32_t mode, float *logits, float *probs,
                                 int32_t *n_accepted, int32_t *next_token, void *stream);

/*
 * Device-resident control of the cascade (Algorithm 1; Sections 3.2, 3.4): the two calls below keep a sequence's
 * tokens (kept tokens followed by the drafts in flight), its lengths and the draft distributions on the device, so
 * that a whole multi-level step -- Max-Gram drafts, a draft model's reviews "until k_i tokens exist", the
 * horizontal cascade's tail, the target's review -- is a chain of enqueues with no host synchronisation.  Every
 * pointer in csd_review is a device pointer.
 */
typedef struct csd_review {
    int32_t *ctx;                  /* [B][ctx_stride] tokens: kept ++ drafts in flight; the reviewer's token is appended    */
    int32_t  ctx_stride;
    int32_t *ctx_len;              /* [B] in/out: tokens present (kept + in flight); out: kept + 1                           */
    int32_t *cache_len;            /* [B] in/out: rows of this reviewer's cache in use; out: position of its own token      */
    const int32_t *prefix_len;     /* [B] position of the first draft under review (>= cache_len + 1); < 0: skip sequence    */
    const float   *q_tab;          /* draft distributions by position, row (pos - q_base[b]) of [B][q_stride][V], or NULL   */
    const uint8_t *q_onehot_tab;   /* [B][q_stride] nonzero: the draft at that position was deterministic; or NULL           */
    const int32_t *q_base;         /* [B]                                                                                    */
    int32_t  q_stride;
    const float *u_acc_tab;        /* [B][ctx_stride] uniform of the acceptance test of the draft at a position              */
    const float *u_samp_tab;       /* [B][ctx_stride] uniform of the draw of a review whose first draft sits at a position   */
    float   *out_q_tab;            /* this reviewer's rows of the tokens it emits, for the level above: row (pos - out_base)  */
    uint8_t *out_onehot_tab;       /* ... and their flags (0 when sampling, 1 under the greedy rule); either may be NULL      */
    const int32_t *out_base;       /* [B]                                                                                    */
    int32_t  out_stride;
    int32_t *lower_cache_len[4];   /* cache lengths [B] of the levels below: clamped to the kept length                      */
    int32_t  n_lower;
    int32_t *n_accepted, *next_token;   /* [B] optional outputs (-1 for a skipped sequence)                                  */
    int32_t *status;               /* [B] out: 0 reviewed, 1 skipped on request, 2 skipped: the state does not fit the call   */
    const float *ext_rows;         /* NULL: run the model.  Else [B][m_max][V] reviewer rows given by the caller (block row i) */
} csd_review;

/*
 * One review.  Block of sequence b = ctx[b][cache_len[b] .. ctx_len[b]) (at most m_max rows, else status 2): rows the
 * reviewer has not cached yet, ending with the drafts ctx[b][prefix_len[b] .. ctx_len[b]).  The forward runs over
 * m_max rows per sequence (zero tokens as padding; their cache rows lie beyond the kept length), then accept /
 * resample as csd_accept does, with k = ctx_len - prefix_len drafts per sequence, draft distributions and uniforms
 * taken by position, then the commit: ctx[prefix + n] = the reviewer's token, ctx_len = prefix + n + 1, cache_len =
 * prefix + n, lower levels' cache lengths = min(theirs, prefix + n), the reviewer's rows of the n + 1 emitted tokens
 * into out_q_tab.  cache_len + m_max <= max_seq and ctx_len < ctx_stride are the caller's duty (the latter is
 * checked on the device: status 2).
 */
int32_t csd_review_ctx(csd_model *model, void *kv, const csd_review *r, int32_t B, int32_t m_max, float temperature,
                       float lenience, int32_t mode, void *stream);

/*
 * csd_bigram_draft that appends: for every sequence with gate == NULL or gate[b] >= 0, draft k tokens continuing
 * ctx[b][0 .. ctx_len[b]), write them at ctx_len[b], advance ctx_len[b] by k, and set q_onehot_tab[b][pos - q_base[b]]
 * = 1 for their positions (optional); other sequences are left alone.  ctx_len + k < ctx_stride is checked on the
 * device (such a sequence is left alone).
 */
int32_t csd_bigram_draft_append(int32_t *ctx, int32_t ctx_stride, int32_t *ctx_len, int32_t B, const int32_t *next_table,
                                int32_t vocab, int32_t k, int32_t max_match, const int32_t *gate, uint8_t *q_onehot_tab,
                                const int32_t *q_base, int32_t q_stride, void *stream);

/*
 * The loop condition of Algorithm 1 ("while fewer than k_i tokens exist") on the device: gate[b] = ctx_len[b] if
 * ctx_len[b] - loop_start[b] < need (loop_start NULL: always) and the enclosing step is active (parent_gate NULL or
 * parent_gate[b] >= 0), else -1.  The value doubles as the prefix_len of the step it gates: csd_bigram_draft_append and
 * csd_review_ctx skip sequences whose gate / prefix_len is negative.
 */
int32_t csd_cascade_gate(const int32_t *ctx_len, const int32_t *loop_start, int32_t need, const int32_t *parent_gate,
                         int32_t B, int32_t *gate, void *stream);

/*
 * Review forward over a tree of drafts (Section 5.1: the cascade combined with tree attention; Appendix B: the lead
 * node has eight children, the other nodes none).  tokens[B][m], parent[B][m] (device): row 0 is the last kept
 * token (parent -1, not read); parent[b][i] in [0, i) names the row that row i continues (a value outside that range
 * is read as 0).  A row's position is cache_len[b] + its distance from row 0; it attends the cached rows
 * [0, cache_len[b]), the rows above it in the tree and itself; its K/V are stored at cache row cache_len[b] + i.
 * So every root-to-node path is scored exactly as a plain block holding that path would be.  logits[B][m][V]
 * (and probs, as csd_verify_block).  m <= 64 and <= max_block; arch 0 only (CSD_EUNSUPPORTED otherwise).
 */
int32_t csd_verify_tree(csd_model *model, void *kv, const int32_t *tokens, const int32_t *parent,
                        const int32_t *cache_len, int32_t B, int32_t m, float temperature, float *logits, float *probs,
                        void *stream);

/*
 * Review of a tree of deterministic candidates (same passages; the accept rule of Section 2 for drafts whose
 * distribution is one-hot, taken one level of the tree at a time).  Walk down from row 0: take the reviewer's own
 * token for the position after the current row (mode CSD_MODE_SAMPLE: the fixed-point inverse-CDF draw of
 * csd_accept from row `current` of p with the walk's j-th uniform u[b][j]; CSD_MODE_GREEDY: the arg-max, ties to the
 * smallest id, and p may hold logits); if a child of the current row carries that token (the lowest such row), keep
 * it and continue from it, else the token is next_token[b] and the walk ends.  Every emitted token is the
 * reviewer's own, so the output law is the reviewer's whatever the tree holds.  p[B][m][V], tokens, parent as for
 * csd_verify_tree, u[B][m] (may be NULL in greedy mode).  Outputs: n_accepted[B], path[B][m] (the kept rows, the
 * first n_accepted entries), next_token[B] (-1 if a row of p is not a distribution).
 */
int32_t csd_tree_accept(const float *p, const int32_t *tokens, const int32_t *parent, const float *u, int32_t B,
                        int32_t m, int32_t V, int32_t mode, int32_t *n_accepted, int32_t *path, int32_t *next_token,
                        void *stream);

/*
 * After csd_verify_tree + csd_tree_accept: move the K/V of the kept rows path[b][0 .. n_accepted[b]) to cache rows
 * cache_len[b] + 1 .., where a plain block would have stored them; the caller then commits
 * cache_len[b] += 1 + n_accepted[b] as after a plain review.  path must be increasing with path[b][j] >= j + 1 (what
 * csd_tree_accept writes); an entry that is not cuts the move there.  All layers, one launch.
 */
int32_t csd_tree_commit(const csd_model *model, void *kv, const int32_t *cache_len, const int32_t *path,
                        const int32_t *n_accepted, int32_t B, int32_t m, void *stream);

/* Test hook: when trace != NULL the next verify calls also copy the residual stream of all
 * B*m rows after the embedding and after every layer to trace[(n_layers+1)][B*m][d] (fp32). */
int32_t csd_debug_set_trace(csd_model *model, float *trace);

/* Which forward csd_verify_block would run for B sequences of m rows: 0 = one kernel per operation with
 * split-K partial sums and epilogue kernels (any shape, both architectures), 1 = the forward whose GEMM
 * kernels own whole output tiles and hold their epilogues (bf16 models of either architecture, B*m <= 32 rows; the default
 * where it applies).  The environment variable CSD_PATH=multikernel at csd_model_create forces 0. */
int32_t csd_debug_path(const csd_model *model, int32_t B, int32_t m);

/* Test hook, host only (no device call): the launch plan of the GEMM that serves blocks of 33 to 144 rows, for an
 * N x K weight matrix (N a multiple of 16, K of 32) and a block of `rows` rows when the partial-sum buffer holds
 * max_splits planes of rows x N floats: *ct = 16-column tiles per workgroup, *S = K splits.  The plan comes as close
 * to one workgroup per compute unit (256) as ceil(N / 16 / ct) * S allows, S <= 8, the wider workgroup on a tie.
 * CSD_EINVAL for other shapes or rows outside [1, 144]. */
int32_t csd_debug_gemm_plan(int32_t N, int32_t K, int32_t rows, int32_t max_splits, int32_t *ct, int32_t *S);

/* Counter calibration for benchmarks: a plain streaming copy of `bytes` bytes (a multiple of 16; dst and
 * src are device pointers, 16-byte aligned, not overlapping), launched as kernel k_copy_calib, so that a
 * hardware counter's reading for exactly 2 x bytes of HBM traffic (one read, one write) can be taken
 * in the same profiler run as the kernels being measured. */
int32_t csd_debug_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Peaks measured on the box, for benchmarks (the roofline fractions are quoted against the published
 * peaks; these say what a plain kernel reaches).  csd_debug_read: a grid-stride streaming read of `bytes`
 * bytes (a multiple of 16, src 16-byte aligned; device) with 16-byte loads, 2048 workgroups; each
 * workgroup stores one word to sink (device, >= 2048 uint32) so that the loads are kept.  csd_debug_mfma:
 * 1024 workgroups of 4 waves, every wave issues `iters` x 8 independent 16x16x32 bf16 matrix instructions
 * on registers (no memory traffic), i.e. 4096 x iters x 8 x 16384 flops in all; sink as above.  Both are
 * asynchronous on `stream`; the caller times them. */
int32_t csd_debug_read(const void *src, size_t bytes, uint32_t *sink, void *stream);
int32_t csd_debug_mfma(int64_t iters, uint32_t *sink, void *stream);

/* Kernel timing hook for benchmarks.  While enabled, each verify call brackets every kernel
 * it launches with a pair of HIP events on the caller's stream (this perturbs the step, so
 * throughput is timed with the hook off).  After the caller has synchronised the stream,
 * csd_prof_read adds up the bracketed milliseconds and launch counts per kernel class since
 * the last reset: class 0 = weight-streaming GEMMs, 1 = attention, 2 = everything else. */
int32_t csd_prof_enable(csd_model *model, int32_t on);
int32_t csd_prof_read(csd_model *model, int32_t kernel_class, double *ms, int64_t *launches, int32_t reset);

#ifdef __cplusplus
}
#endif
#endif /* CSD_H */
