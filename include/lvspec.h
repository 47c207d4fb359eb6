/*
 * lvspec.h — C ABI of the MI355X (gfx950) verify-step hot path of LVSpec, the loosely
 * speculative decoding method for Video-LLMs ("See the Forest for the Trees: Loosely
 * Speculative Decoding via Visual-Semantic Guidance for Efficient Inference of Video LLMs").
 *
 * One decode step of the method: a draft model proposes K tokens, the target model processes
 * them in parallel (Eq. 1), a visual-relevance score is computed per draft token from
 * final-layer hidden states (Eq. 8), the lambda*K least relevant positions are loosened
 * (Eq. 9), every position gets a verdict (Eq. 10, with position-shift tolerance Eq. 11) and the
 * accepted length is the longest accepted prefix (Eq. 2).  This library implements the
 * data-parallel part of that step on one GPU:
 *
 *   lvspec_verify_attn        attention of the K (= gamma) draft rows over the target's long KV
 *                             cache, for one layer
 *   lvspec_visual_relevance   Eq. 8
 *   lvspec_loose_accept       lm_head logits of the gamma rows, greedy target tokens, softmax
 *                             top-k, Eq. 9, Eq. 10/11, Eq. 2
 *
 * Conventions for every entry point
 *   - returns LVSPEC_OK (0) or a negative lvspec_status; never throws, never aborts
 *   - all argument checking happens on the host before anything is launched
 *   - work is only ENQUEUED on `stream` (a hipStream_t passed as void*; NULL = default
 *     stream); no host synchronisation, no allocation, no host<->device copy inside
 *   - pointers marked DEVICE are device memory owned by the caller (valid until the enqueued
 *     work has finished); pointers marked HOST are read during the call only
 *   - bf16 tensors are raw 16-bit patterns; strides are in ELEMENTS; the innermost dimension
 *     is contiguous and every row start is 16-byte aligned
 *   - `workspace` is DEVICE scratch of at least lvspec_*_workspace() bytes, 256-byte aligned,
 *     private to the call until its work has finished
 *   - results are deterministic: no floating-point atomics, fixed reduction orders
 */
#ifndef LVSPEC_H_
#define LVSPEC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LVSPEC_VERSION 106          /* 0.1.6 */
#define LVSPEC_MAX_GAMMA 16         /* draft tokens of one chain */
#define LVSPEC_MAX_DRAFT_ROWS 32    /* draft rows per sequence and step (all chains of a tree) */
#define LVSPEC_MAX_BRANCHES 8       /* chains of a draft tree */
#define LVSPEC_MAX_TOPK 16
#define LVSPEC_MAX_TOPN 1024        /* N of the relevance metric */
#define LVSPEC_HEAD_DIM 128         /* only head dimension implemented */

typedef enum {
  LVSPEC_OK = 0,
  LVSPEC_EINVAL = -1,        /* NULL / out-of-range / inconsistent argument */
  LVSPEC_EUNSUPPORTED = -2,  /* legal but not implemented shape (e.g. head dim != 128) */
  LVSPEC_EWORKSPACE = -3,    /* workspace NULL, misaligned or smaller than required */
  LVSPEC_EHIP = -4,          /* a HIP call failed; see lvspec_last_hip_error() */
  LVSPEC_ESCRATCH = -5       /* lvspec_verify_attn_static: the shapes need more scratch than the
                                library's static device array holds */
} lvspec_status;

/* static string for a status code */
const char* lvspec_status_string(int status);
/* LVSPEC_VERSION the library was built from */
int lvspec_version(void);
/* raw hipError_t of the most recent LVSPEC_EHIP on this thread (0 if none) */
int lvspec_last_hip_error(void);

/* ---------------------------------------------------------------------------------------------
 * Verification attention (target forward of Eq. 1, one layer; the paper uses scaled-dot-product
 * attention).  For sequence b, draft row i (0 <= i < gamma) and query head h:
 *     visible keys = cache positions 0 .. kv_len[b]-1  plus draft positions kv_len[b]+j for the
 *                    j allowed by the draft mask (default: j <= i, causal chain)
 *     out[b,i,h,:] = softmax(scale * q[b,i,h,:] . K[b, h/(Hq/Hkv), visible, :]) @ V[...]
 * The draft tokens' own K/V rows must already be stored at cache rows kv_len[b] ..
 * kv_len[b]+gamma-1.  Optional extras from the same pass: the natural-log sum-exp of the scaled
 * scores, and the softmax mass that falls on the video-token span (a diagnostic; the accept
 * rule of the paper does not use it).
 * Draft trees (appendix on draft token trees): the rows of all chains are stored one after the
 * other, gamma counts them all, and draft_mask says which rows a row sees (for two independent
 * chains: a block-diagonal lower-triangular pattern).
 * ------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t B, gamma, Hq, Hkv, D;     /* D must be 128; Hq % Hkv == 0; 1 <= gamma <= 32 */
  const void* q;                    /* DEVICE bf16 [B, gamma, Hq, D] */
  int64_t q_sb, q_sg, q_sh;         /* strides of q: batch, draft row, head */
  const void* k;                    /* DEVICE bf16 [B, Hkv, cap, D] */
  const void* v;                    /* DEVICE bf16 [B, Hkv, cap, D] */
  int64_t kv_sb, kv_sh, kv_sl;      /* strides of k and v: batch, kv head, cache row */
  int64_t cap;                      /* cache rows allocated per (b, kv head) */
  const int32_t* kv_len;            /* DEVICE [B]; 0 <= kv_len[b], kv_len[b]+gamma <= cap; may be
                                       NULL when kv_len_host is given.  A value outside that
                                       range (a stale length) is clamped to [0, cap-gamma] by
                                       the kernel, so no read leaves the declared rows; host
                                       lengths outside it are LVSPEC_EINVAL */
  const int32_t* kv_len_host;       /* HOST [B] or NULL: the same lengths, known to the caller.
                                       For B <= 5 they travel in the launch arguments, which
                                       saves the kernel a dependent device read before its
                                       first K/V load; for B <= 32 they can stand in for a
                                       missing device array.  They are launch arguments: a
                                       captured graph replays the lengths it was captured
                                       with (pass NULL to have replays read kv_len) */
  int64_t max_kv_len;               /* HOST hint: upper bound of kv_len[] used to size the
                                       launch; 0 = cap - gamma */
  const int32_t* vis_begin;         /* DEVICE [B] or NULL: first cache row of the video span */
  const int32_t* vis_end;           /* DEVICE [B] or NULL: one past its last row */
  const uint32_t* draft_mask;       /* HOST [gamma] or NULL: bit j of draft_mask[i] set = row i
                                       sees draft row j (draft trees); NULL = causal chain */
  float scale;                      /* score scale; 0 = 1/sqrt(D) */
  void* out;                        /* DEVICE bf16 [B, gamma, Hq, D] */
  int64_t o_sb, o_sg, o_sh;         /* strides of out */
  float* lse;                       /* DEVICE fp32 [B, Hq, gamma] or NULL */
  float* vis_mass;                  /* DEVICE fp32 [B, Hq, gamma] or NULL (needs vis_begin/end) */
  void* workspace;                  /* DEVICE */
  size_t workspace_bytes;
} lvspec_attn_args;

/* bytes of workspace lvspec_verify_attn needs for these shapes; 0 if the arguments are invalid.
 * The three *_workspace queries and lvspec_describe_plan read only shape fields and touch no
 * device memory, but they ask the HIP runtime for the current device's compute-unit count
 * (which initialises the runtime; without a device the count of an MI355X, 256, is assumed).
 * Planning and launching may run concurrently from several host threads. */
size_t lvspec_verify_attn_workspace(const lvspec_attn_args* args);
int lvspec_verify_attn(const lvspec_attn_args* args, void* stream);

/* lvspec_verify_attn for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same results as lvspec_verify_attn; `workspace` and
 * `workspace_bytes` are ignored.  The split partials live in a static device array of
 * LVSPEC_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library
 * runs on holds its own copy until the process ends).  The call allocates nothing: no
 * hipMalloc / hipFree, no allocating library routine.  The first call on a device looks the
 * array's address up (one hipGetSymbolAddress, with that device current) and keeps it; make
 * that first call outside stream capture.
 * Errors: as lvspec_verify_attn, and LVSPEC_ESCRATCH when lvspec_verify_attn_workspace(args)
 * exceeds LVSPEC_STATIC_SCRATCH_BYTES (nothing is launched).
 * All calls on one GPU share the array, and it keeps the previous call's contents (every
 * partial is rewritten before it is read, nothing needs clearing): calls on the same GPU must
 * not overlap in time (different streams without ordering between them race); calls ordered
 * on one stream, or on different GPUs, are fine. */
#define LVSPEC_STATIC_SCRATCH_BYTES (16u << 20)
int lvspec_verify_attn_static(const lvspec_attn_args* args, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Visual relevance (Eq. 8): cosine similarity between each draft token's final-layer hidden
 * state and every video token's final-layer hidden state, then the mean of the top_n largest
 * similarities along the video axis.
 *     relevance[b,i] = mean of the min(top_n, l_v[b]) largest cos(h_d[b,i,:], h_v[b,j,:]),
 *     j < l_v[b]; norms are clamped below at 1e-8; l_v[b] == 0 gives 0.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t B, gamma, d, top_n;       /* d % 128 == 0; 1 <= gamma <= 32 (rows of all chains of a
                                       tree); 1 <= top_n <= LVSPEC_MAX_TOPN */
  const void* h_d;                  /* DEVICE bf16 [B, gamma, d] */
  int64_t hd_sb, hd_sg;
  const void* h_v;                  /* DEVICE bf16 [B, lv_max, d] */
  int64_t hv_sb, hv_sl;
  int64_t lv_max;                   /* rows allocated per sequence in h_v */
  const int32_t* l_v;               /* DEVICE [B]; 0 <= l_v[b] <= lv_max */
  const float* hv_inv_norm;         /* DEVICE fp32 [B, lv_max] or NULL: 1 / max(|h_v[b,j,:]|, 1e-8)
                                       as written by lvspec_hv_prepare.  Given: the values are
                                       used as they are and the pass computes dot products
                                       only; NULL: the norms are taken in the same pass */
  float* relevance;                 /* DEVICE fp32 [B, gamma] */
  void* workspace;                  /* DEVICE */
  size_t workspace_bytes;
} lvspec_rel_args;

size_t lvspec_visual_relevance_workspace(const lvspec_rel_args* args);
int lvspec_visual_relevance(const lvspec_rel_args* args, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Prefill-side preparation of the video hidden states (Eq. 7: H_V is extracted once during
 * prefill and kept for the whole generation; Eq. 8 normalises every similarity by the norms).
 * One pass over h_v writes, for every row,
 *     hv_inv_norm[b,j] = 1 / max(|h_v[b,j,:]|, 1e-8)          (fp32 accumulation)
 * for all lv_max rows of every sequence, to be passed to lvspec_visual_relevance at every
 * decode step.  Needs no workspace.  Errors: LVSPEC_EINVAL for NULL / misaligned pointers or bad
 * strides, LVSPEC_EUNSUPPORTED for d % 128 != 0 or more than 2^30 rows.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t B, d;                     /* d % 128 == 0 */
  const void* h_v;                  /* DEVICE bf16 [B, lv_max, d] */
  int64_t hv_sb, hv_sl;
  int64_t lv_max;                   /* rows per sequence, >= 0 */
  float* hv_inv_norm;               /* DEVICE out fp32 [B, lv_max] */
} lvspec_hv_args;

int lvspec_hv_prepare(const lvspec_hv_args* args, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Loose acceptance.  Per sequence b and draft position i:
 *     z[b,i,:]   = lm_head @ h_d[b,i,:]                               (Eq. 6)
 *     y[b,i]     = argmax_v z   (greedy target token; lowest id on exact ties)
 *     I'_b       = the n_loose positions with the lowest relevance (stable ascending order,
 *                  Eq. 9; n_loose = floor(lambda*gamma), see lvspec_n_loose)
 *     verdict    = EXACT if draft == y; else LOOSE if i in I'_b (and, only when
 *                  loose_topk_gate = g > 0, the draft id is among the row's g most probable
 *                  tokens; the paper's rule is g = 0); else SHIFT if y[b,i] equals some draft
 *                  id at a position k != i with |k - i| <= pst_window (Eq. 11; pst_window >=
 *                  gamma-1 is the paper's range, 0 switches it off); else REJECT
 *     accept_len = number of leading non-REJECT verdicts (Eq. 2)
 *     bonus_id   = y[b, accept_len] if accept_len < gamma, else -1
 * Bonus row (standard speculative decoding; Eq. 1 lists only the first gamma outputs of the
 * target's forward pass over [last committed token, drafts], which has gamma + 1 rows): with
 * bonus_row = 1 every chain brings gamma + 1 hidden rows, row i < gamma yields y[b,i] as above
 * and row gamma the token that follows the last draft, so that bonus_id = y[b, accept_len] is a
 * token also when every draft is accepted.  h_d, target_ids, topk_ids, topk_probs, logits and
 * entropy then have gamma + 1 rows per chain; draft_ids, relevance and verdict keep gamma.
 * Draft trees (appendix on draft token trees): with n_branches = n > 1 the B chains are the
 * branches of B/n sequences (chains s*n .. s*n+n-1 belong to sequence s); every chain is
 * verified on its own exactly as above (ranking and shift window local to the chain), and
 *     best_branch[s] = the branch with the largest accept_len (lowest index on ties).
 * Text-only loose rules (the entropy-gated methods of the paper's comparison: baselines
 * paragraph of the experiment setup; baseline-details appendix, window 4, thresholds 0.1 / 0.2):
 * with rule = LVSPEC_RULE_ENTROPY_GATE or LVSPEC_RULE_ENTROPY_WINDOW, Eq. 9-11 are replaced by
 *     verdict    = EXACT if draft == y; else GATED if the entropy (nats, binary32) of row i's
 *                  softmax exceeds entropy_threshold and, for ..._WINDOW with defer_window = w,
 *                  positions i+1 .. i+w are all draft positions of the chain (i + w <= gamma-1)
 *                  and match exactly; else REJECT
 * (a window that runs past the last draft is not confirmed; a position accepted only through
 * the gate does not count as a match; the bonus row is no window position).  relevance,
 * n_loose, pst_window and loose_topk_gate are then ignored and relevance may be NULL.
 * ------------------------------------------------------------------------------------------- */
enum { LVSPEC_REJECT = 0, LVSPEC_EXACT = 1, LVSPEC_LOOSE = 2, LVSPEC_SHIFT = 3, LVSPEC_GATED = 4 };
enum { LVSPEC_RULE_VISUAL = 0, LVSPEC_RULE_ENTROPY_GATE = 1, LVSPEC_RULE_ENTROPY_WINDOW = 2 };

typedef struct {
  int32_t B, gamma, d, V, topk;     /* B chains of gamma <= 16 tokens; d % 128 == 0;
                                       1 <= topk <= 16.  One pass over lm_head serves up to 64
                                       hidden rows; with more rows the chains are taken in
                                       groups of whole sequences, one pass each */
  const void* h_d;                  /* DEVICE bf16 [B, gamma + bonus_row, d] final hidden rows */
  int64_t hd_sb, hd_sg;
  const void* lm_head;              /* DEVICE bf16 [V, d] row-major, no bias */
  int64_t w_sv;                     /* row stride of lm_head (0 = d) */
  const int32_t* draft_ids;         /* DEVICE [B, gamma], each in [0, V) */
  const float* relevance;           /* DEVICE fp32 [B, gamma] (from lvspec_visual_relevance);
                                       may be NULL with an entropy rule */
  int32_t n_loose;                  /* 0 .. gamma */
  int32_t pst_window;               /* >= 0 */
  int32_t loose_topk_gate;          /* 0 .. topk */
  int32_t n_branches;               /* 0 or 1: every chain is a sequence; else 2 .. 8, divides B */
  int32_t bonus_row;                /* 0 or 1: hidden rows per chain = gamma + bonus_row */
  int32_t rule;                     /* LVSPEC_RULE_*: 0 = the paper's rule (Eq. 9-11) */
  float entropy_threshold;          /* entropy rules: gate threshold in nats, >= 0 */
  int32_t defer_window;             /* LVSPEC_RULE_ENTROPY_WINDOW: 0 .. LVSPEC_MAX_GAMMA */
  int32_t* target_ids;              /* DEVICE out [B, gamma + bonus_row] */
  int32_t* topk_ids;                /* DEVICE out [B, gamma + bonus_row, topk] or NULL */
  float* topk_probs;                /* DEVICE out [B, gamma + bonus_row, topk] or NULL */
  uint8_t* verdict;                 /* DEVICE out [B, gamma]: LVSPEC_REJECT .. LVSPEC_GATED */
  int32_t* accept_len;              /* DEVICE out [B] */
  int32_t* bonus_id;                /* DEVICE out [B] */
  int32_t* best_branch;             /* DEVICE out [B / n_branches] or NULL */
  float* logits;                    /* DEVICE out fp32 [B, gamma + bonus_row, V] or NULL */
  float* entropy;                   /* DEVICE out fp32 [B, gamma + bonus_row] or NULL: entropy (nats) of each
                                       row's softmax, from the same pass.  A diagnostic: the
                                       paper's rule does not use it (the text-only loose
                                       methods it compares against gate on it) */
  void* workspace;                  /* DEVICE */
  size_t workspace_bytes;
} lvspec_accept_args;

/* floor(lambda * gamma + 1e-6) clamped to [0, gamma]: the length of Eq. 9's slice */
int lvspec_n_loose(float lambda, int gamma);
size_t lvspec_loose_accept_workspace(const lvspec_accept_args* args);
int lvspec_loose_accept(const lvspec_accept_args* args, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Committing a verified step to the KV cache (the step after Eq. 2: the accepted draft tokens
 * join the history of Eq. 1; the paper leaves the bookkeeping to the implementation).
 * The draft rows of a step sit behind the cache, chain c's token i at cache row
 * kv_len[b] + c*chain_len + i (the layout lvspec_verify_attn reads).  For every sequence b
 *     kept       = best_branch[b]               (0 when n_branches <= 1 or best_branch == NULL)
 *     tau        = accept_len[b*n_branches + kept]
 *     new_len[b] = kv_len[b] + tau
 * and, when kept > 0, the K and V rows kv_len[b] + kept*chain_len + i move to rows kv_len[b] + i
 * for i < tau, in every layer and kv head (source and destination never overlap: tau <=
 * chain_len).  Rows at and behind new_len[b] are left as they are; rejecting drafts needs no
 * data movement.  The token to feed next is the caller's (bonus_id of lvspec_loose_accept).
 * Errors: LVSPEC_EINVAL for NULL / out-of-range arguments or new_len aliasing kv_len.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t B, Hkv, D;                /* D % 8 == 0 (16-byte chunks) */
  int32_t n_layers;                 /* layers served by this call (>= 1) */
  int32_t n_branches, chain_len;    /* n_branches in 1..8 (0 = 1), chain_len in 1..16,
                                       n_branches * chain_len <= LVSPEC_MAX_DRAFT_ROWS */
  void* k;                          /* DEVICE bf16 [n_layers][B, Hkv, cap, D], changed in place */
  void* v;
  int64_t kv_slayer;                /* elements between layers (unused when n_layers == 1) */
  int64_t kv_sb, kv_sh, kv_sl;      /* elements; kv_sl % 8 == 0, rows 16-byte aligned */
  int64_t cap;                      /* rows allocated per (sequence, head) */
  const int32_t* kv_len;            /* DEVICE [B] context length before the step;
                                       kv_len[b] + n_branches*chain_len <= cap (a sequence that
                                       violates this gets its length updated, no rows moved) */
  const int32_t* accept_len;        /* DEVICE [B * n_branches] */
  const int32_t* best_branch;       /* DEVICE [B] or NULL */
  int32_t* new_len;                 /* DEVICE out [B]; must not alias kv_len */
} lvspec_commit_args;

int lvspec_kv_commit(const lvspec_commit_args* args, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Diagnostics: how the three verify calls would be launched for the given shapes (no paper
 * passage behind this one: it reports the library's own launch planning, for tuning and tests).
 * Any of the argument pointers may be NULL; its fields of *out are then left untouched.  Only
 * shape fields are read (no device pointer is dereferenced, nothing is launched).
 * Returns the first planning error among the given arguments, else LVSPEC_OK.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t attn_rows_padded;      /* query rows per workgroup: 16, 32, 48 or 64 */
  int32_t attn_row_chunks;       /* workgroups that share one kv head's key range */
  int32_t attn_splits;           /* key-range splits per (sequence, kv head, row chunk) */
  int32_t rel_splits;            /* splits of the hidden dimension */
  int32_t rel_stage_bytes;       /* bytes of a video row per pipeline stage: 256 or 512 */
  int32_t rel_slices;            /* slices of the two-kernel Top-N; 0 = single-kernel selection */
  int32_t rel_slice_rows;        /* video rows per slice */
  int32_t acc_rows_per_task;     /* vocabulary rows per lm_head task: 64 or 128 */
  int32_t acc_chains_per_pass;   /* chains served by one pass over lm_head */
  int32_t acc_passes;            /* passes over lm_head */
} lvspec_plan_info;

int lvspec_describe_plan(const lvspec_attn_args* attn, const lvspec_rel_args* rel,
                         const lvspec_accept_args* accept, lvspec_plan_info* out);

#ifdef __cplusplus
}
#endif
#endif /* LVSPEC_H_ */
