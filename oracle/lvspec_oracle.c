/*
 * CPU oracle for the LVSpec verify-step hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow, obviously-correct statement of what the GPU library computes.
 * It is used by the tests, by the smoke check and by the benchmark's "cpu_baseline" leg, and by
 * nothing else.  It shares no code, header, table or helper with the HIP path.
 *
 * Everything is evaluated in IEEE double precision from the bf16 *bit patterns* of the inputs,
 * in the order the definitions are written, with no blocking, fusion or reordering.  OpenMP is
 * used only across independent output units (a query row, a vocabulary row, a visual row); the
 * arithmetic of any single output value is sequential and therefore independent of the thread
 * count.
 *
 * Sections (paper = "See the Forest for the Trees: Loosely Speculative Decoding via
 * Visual-Semantic Guidance for Efficient Inference of Video LLMs"):
 *   O1  lvo_verify_attn        target verification attention of the K draft rows   (Eq. 1; the
 *                              paper states scaled-dot-product attention in its implementation
 *                              details and gives no formula: the textbook definition is used)
 *   O2  lvo_visual_relevance   mean of the Top-N cosine similarities               (Eq. 8)
 *   O3  lvo_logits / lvo_softmax_topk   lm_head on the final hidden rows, greedy target token
 *                              (Eq. 6; "identical to the target model's generation")
 *   O4  lvo_loosened_set       index set of the lambda*K lowest relevance scores    (Eq. 9)
 *   O5  lvo_verdicts           per-position verdict incl. position-shift tolerance  (Eq. 10, 11)
 *                              and accepted length by longest-accepted-prefix       (Eq. 2)
 *   O6  lvo_select_branch      draft trees: the chain with the longest accepted length is kept
 *                              (appendix on draft token trees)
 *   O7  (kv_commit in lvspec_oracle.py, numpy) the KV cache after the step: the accepted tokens
 *                              of the kept chain join the history of Eq. 1
 *
 * Pins: every function here is pinned by tests marked "not gpu" (closed forms, brute force,
 * library routines it reduces to in special cases, hand-derived cases of Eq. 9-11 and of the
 * two-branch tree, the strict
 * acceptance bound of Prop. 2.2).  The paper prints no worked numeric example of a whole verify
 * step, so the end-to-end composition (O1..O5 chained) is "parity unpinned" against the paper;
 * each stage is pinned on its own.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int lvo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void lvo_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/* bf16 is the upper half of an IEEE binary32: widen exactly. */
static double bf16_bits_to_double(uint16_t bits) {
  uint32_t u = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* ------------------------------------------------------------------------------------------
 * O1  verification attention (Eq. 1: the K draft tokens are appended to the history and the
 * target model processes them in parallel; inside every layer that is causal attention of the
 * K new rows over [cached prefix, drafts]).
 *
 * Layouts (dense, last dim contiguous):
 *   q   [B, gamma, Hq, D]  bf16 bits        k, v  [B, Hkv, cap, D]  bf16 bits
 *   kv_len[b] = L_b cached positions; the draft rows' own K/V sit at L_b .. L_b+gamma-1.
 * Row i of sequence b sees positions 0..L_b-1 and the draft positions j for which
 * draft_mask[i] has bit j set; draft_mask == NULL means causal (j <= i).  A tree of drafts is
 * expressed with an ancestor mask (appendix "Exploration on Draft Token Trees").
 * Grouped-query mapping: query head h reads kv head h / (Hq / Hkv).
 * vis_begin/vis_end (may be NULL): half-open span of cache positions; vis_mass is the softmax
 * probability that falls on it (a diagnostic, not part of the paper's accept rule).
 * One (b, i, h) unit; out[D], *lse, *vis_mass.
 * ------------------------------------------------------------------------------------------ */
static void attn_one_row(int gamma, int Hq, int Hkv, int D, int64_t cap,
                         const uint16_t* q, const uint16_t* k, const uint16_t* v,
                         const int32_t* kv_len, const int32_t* vis_begin, const int32_t* vis_end,
                         const uint32_t* draft_mask, double scale,
                         int b, int i, int h, double* out, double* lse, double* vis_mass) {
  const int G = Hq / Hkv;
  const int kvh = h / G;
  const int64_t L = kv_len[b];
  const int64_t n_pos = L + gamma;
  const uint16_t* qrow = q + (((int64_t)b * gamma + i) * Hq + h) * D;
  const uint16_t* kbase = k + ((int64_t)b * Hkv + kvh) * cap * D;
  const uint16_t* vbase = v + ((int64_t)b * Hkv + kvh) * cap * D;
  double* s = (double*)malloc(sizeof(double) * (size_t)n_pos);
  unsigned char* vis = (unsigned char*)malloc((size_t)n_pos);
  double m = -INFINITY;
  for (int64_t j = 0; j < n_pos; ++j) {
    int visible;
    if (j < L) {
      visible = 1;
    } else {
      int dj = (int)(j - L);
      visible = draft_mask ? (int)((draft_mask[i] >> dj) & 1u) : (dj <= i);
    }
    vis[j] = (unsigned char)visible;
    if (!visible) continue;
    double dot = 0.0;
    for (int t = 0; t < D; ++t)
      dot += bf16_bits_to_double(qrow[t]) * bf16_bits_to_double(kbase[j * D + t]);
    s[j] = scale * dot;
    if (s[j] > m) m = s[j];
  }
  double denom = 0.0;
  for (int64_t j = 0; j < n_pos; ++j)
    if (vis[j]) denom += exp(s[j] - m);
  for (int t = 0; t < D; ++t) out[t] = 0.0;
  double mass = 0.0;
  for (int64_t j = 0; j < n_pos; ++j) {
    if (!vis[j]) continue;
    double p = exp(s[j] - m) / denom;
    for (int t = 0; t < D; ++t) out[t] += p * bf16_bits_to_double(vbase[j * D + t]);
    if (vis_begin && vis_end && j >= vis_begin[b] && j < vis_end[b]) mass += p;
  }
  *lse = m + log(denom);
  *vis_mass = mass;
  free(s);
  free(vis);
}

/* All rows.  out [B, gamma, Hq, D], lse and vis_mass [B, Hq, gamma] (doubles). */
void lvo_verify_attn(int B, int gamma, int Hq, int Hkv, int D, int64_t cap,
                     const uint16_t* q, const uint16_t* k, const uint16_t* v,
                     const int32_t* kv_len, const int32_t* vis_begin, const int32_t* vis_end,
                     const uint32_t* draft_mask, double scale,
                     double* out, double* lse, double* vis_mass) {
  const int64_t units = (int64_t)B * gamma * Hq;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t u = 0; u < units; ++u) {
    int h = (int)(u % Hq);
    int i = (int)((u / Hq) % gamma);
    int b = (int)(u / ((int64_t)Hq * gamma));
    double l, vm;
    attn_one_row(gamma, Hq, Hkv, D, cap, q, k, v, kv_len, vis_begin, vis_end, draft_mask, scale,
                 b, i, h, out + (((int64_t)b * gamma + i) * Hq + h) * D, &l, &vm);
    lse[((int64_t)b * Hq + h) * gamma + i] = l;
    vis_mass[((int64_t)b * Hq + h) * gamma + i] = vm;
  }
}

/* A chosen subset of rows: sel holds n_sel triples (b, i, h); out [n_sel, D], lse/vis_mass
 * [n_sel].  Same per-row routine as above; used to spot-check full-size problems. */
void lvo_verify_attn_rows(int gamma, int Hq, int Hkv, int D, int64_t cap,
                          const uint16_t* q, const uint16_t* k, const uint16_t* v,
                          const int32_t* kv_len, const int32_t* vis_begin,
                          const int32_t* vis_end, const uint32_t* draft_mask, double scale,
                          int n_sel, const int32_t* sel,
                          double* out, double* lse, double* vis_mass) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < n_sel; ++s) {
    attn_one_row(gamma, Hq, Hkv, D, cap, q, k, v, kv_len, vis_begin, vis_end, draft_mask, scale,
                 sel[3 * s], sel[3 * s + 1], sel[3 * s + 2], out + (int64_t)s * D, lse + s,
                 vis_mass + s);
  }
}

/* ------------------------------------------------------------------------------------------
 * O2  visual relevance (Eq. 8): cosine similarity between every draft hidden row and every
 * visual hidden row, then the mean of the N largest similarities along the visual axis.
 *   h_d [B, gamma, d] bf16 bits, h_v [B, lv_max, d] bf16 bits, l_v[b] valid visual rows.
 *   relevance [B, gamma] doubles; cos_out (may be NULL) [B, gamma, lv_max] doubles.
 * Readings where the paper is silent: each norm is clamped below at 1e-8; the effective N is
 * min(top_n, l_v); l_v == 0 gives relevance 0.
 * ------------------------------------------------------------------------------------------ */
static int cmp_desc(const void* a, const void* b) {
  double x = *(const double*)a, y = *(const double*)b;
  return (x < y) - (x > y);
}

void lvo_visual_relevance(int B, int gamma, int d, int top_n,
                          const uint16_t* h_d, const uint16_t* h_v, const int32_t* l_v,
                          int64_t lv_max, double* relevance, double* cos_out) {
  for (int b = 0; b < B; ++b) {
    const int64_t lv = l_v[b];
    for (int i = 0; i < gamma; ++i) {
      const uint16_t* hd = h_d + ((int64_t)b * gamma + i) * d;
      double* c = (double*)malloc(sizeof(double) * (size_t)(lv > 0 ? lv : 1));
      double nd2 = 0.0;
      for (int t = 0; t < d; ++t) {
        double x = bf16_bits_to_double(hd[t]);
        nd2 += x * x;
      }
      double nd = sqrt(nd2);
      if (nd < 1e-8) nd = 1e-8;
#pragma omp parallel for schedule(static)
      for (int64_t j = 0; j < lv; ++j) {
        const uint16_t* hv = h_v + ((int64_t)b * lv_max + j) * d;
        double dot = 0.0, nv2 = 0.0;
        for (int t = 0; t < d; ++t) {
          double x = bf16_bits_to_double(hd[t]);
          double y = bf16_bits_to_double(hv[t]);
          dot += x * y;
          nv2 += y * y;
        }
        double nv = sqrt(nv2);
        if (nv < 1e-8) nv = 1e-8;
        c[j] = dot / (nd * nv);
      }
      if (cos_out)
        for (int64_t j = 0; j < lv; ++j) cos_out[((int64_t)b * gamma + i) * lv_max + j] = c[j];
      int64_t n_eff = top_n < lv ? top_n : lv;
      double acc = 0.0;
      if (n_eff > 0) {
        qsort(c, (size_t)lv, sizeof(double), cmp_desc);
        for (int64_t n = 0; n < n_eff; ++n) acc += c[n];
        acc /= (double)n_eff;
      }
      relevance[(int64_t)b * gamma + i] = acc;
      free(c);
    }
  }
}

/* ------------------------------------------------------------------------------------------
 * O2p  the prefill-side part of Eq. 7/8: H_V is produced once at prefill and kept for the whole
 * generation, so everything in Eq. 8 that depends on H_V alone can be kept with it.  That is
 * the norm of each visual row; stored as its inverse, r_j = 1 / max(|h_v[j]|, 1e-8) (the same
 * floor as in O2).
 *   h_v [B, lv_max, d] bf16 bits; inv_norm [B, lv_max] doubles (all lv_max rows).
 * ------------------------------------------------------------------------------------------ */
void lvo_hv_inv_norm(int B, int64_t lv_max, int d, const uint16_t* h_v, double* inv_norm) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < (int64_t)B * lv_max; ++r) {
    const uint16_t* hv = h_v + r * d;
    double n2 = 0.0;
    for (int t = 0; t < d; ++t) {
      double y = bf16_bits_to_double(hv[t]);
      n2 += y * y;
    }
    double nv = sqrt(n2);
    if (nv < 1e-8) nv = 1e-8;
    inv_norm[r] = 1.0 / nv;
  }
}

/* Eq. 8 with the visual rows' inverse norms given (binary32, the type the library keeps them
 * in): cos_ij = <hd_i, hv_j> * r_j / max(|hd_i|, 1e-8); Top-N mean as in O2.  With r_j from
 * lvo_hv_inv_norm this is O2 up to the rounding of r_j. */
void lvo_visual_relevance_prepared(int B, int gamma, int d, int top_n, const uint16_t* h_d,
                                   const uint16_t* h_v, const float* inv_norm,
                                   const int32_t* l_v, int64_t lv_max, double* relevance,
                                   double* cos_out) {
  for (int b = 0; b < B; ++b) {
    const int64_t lv = l_v[b];
    for (int i = 0; i < gamma; ++i) {
      const uint16_t* hd = h_d + ((int64_t)b * gamma + i) * d;
      double* c = (double*)malloc(sizeof(double) * (size_t)(lv > 0 ? lv : 1));
      double nd2 = 0.0;
      for (int t = 0; t < d; ++t) {
        double x = bf16_bits_to_double(hd[t]);
        nd2 += x * x;
      }
      double nd = sqrt(nd2);
      if (nd < 1e-8) nd = 1e-8;
#pragma omp parallel for schedule(static)
      for (int64_t j = 0; j < lv; ++j) {
        const uint16_t* hv = h_v + ((int64_t)b * lv_max + j) * d;
        double dot = 0.0;
        for (int t = 0; t < d; ++t) dot += bf16_bits_to_double(hd[t]) * bf16_bits_to_double(hv[t]);
        c[j] = dot * (double)inv_norm[(int64_t)b * lv_max + j] / nd;
      }
      if (cos_out)
        for (int64_t j = 0; j < lv; ++j) cos_out[((int64_t)b * gamma + i) * lv_max + j] = c[j];
      int64_t n_eff = top_n < lv ? top_n : lv;
      double acc = 0.0;
      if (n_eff > 0) {
        qsort(c, (size_t)lv, sizeof(double), cmp_desc);
        for (int64_t n = 0; n < n_eff; ++n) acc += c[n];
        acc /= (double)n_eff;
      }
      relevance[(int64_t)b * gamma + i] = acc;
      free(c);
    }
  }
}

/* ------------------------------------------------------------------------------------------
 * O3  target logits (Eq. 6: the model is lm_head applied to the final-layer hidden states).
 *   h [rows, d] bf16 bits, w [V, d] bf16 bits (row-major, no bias), z [rows, V] doubles.
 * ------------------------------------------------------------------------------------------ */
void lvo_logits(int64_t rows, int d, int64_t V, const uint16_t* h, const uint16_t* w, double* z) {
#pragma omp parallel for schedule(static)
  for (int64_t vv = 0; vv < V; ++vv) {
    const uint16_t* wr = w + vv * d;
    for (int64_t r = 0; r < rows; ++r) {
      const uint16_t* hr = h + r * d;
      double dot = 0.0;
      for (int t = 0; t < d; ++t) dot += bf16_bits_to_double(hr[t]) * bf16_bits_to_double(wr[t]);
      z[r * V + vv] = dot;
    }
  }
}

/* Logits of chosen vocabulary rows only: vsel [n_v]; z [rows, n_v]. */
void lvo_logits_cols(int64_t rows, int d, const uint16_t* h, const uint16_t* w, int n_v,
                     const int64_t* vsel, double* z) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < n_v; ++c) {
    const uint16_t* wr = w + vsel[c] * d;
    for (int64_t r = 0; r < rows; ++r) {
      const uint16_t* hr = h + r * d;
      double dot = 0.0;
      for (int t = 0; t < d; ++t) dot += bf16_bits_to_double(hr[t]) * bf16_bits_to_double(wr[t]);
      z[r * n_v + c] = dot;
    }
  }
}

/* One row of logits -> greedy target token, softmax statistics and the k most probable tokens.
 * The target token is the argmax ("the target model's generation" under greedy decoding).
 * Integer decisions (argmax, top-k order) are taken on the logits rounded to binary32, the
 * precision in which the GPU path holds its logits; ties go to the lowest token id.
 * Outputs: *y argmax id; *lse = ln sum exp z; topk_ids/topk_probs [k] ordered by (value desc,
 * id asc); *margin = (z_(1) - z_(2)) / max_v |z_v|  (how safely the argmax is decided;
 * +inf for V == 1); *entropy = -sum p ln p. */
void lvo_softmax_topk(int64_t V, const double* z, int k, int32_t* y, double* lse,
                      int32_t* topk_ids, double* topk_probs, double* margin, double* entropy) {
  double m = -INFINITY, amax = 0.0;
  for (int64_t vv = 0; vv < V; ++vv) {
    if (z[vv] > m) m = z[vv];
    if (fabs(z[vv]) > amax) amax = fabs(z[vv]);
  }
  double denom = 0.0;
  for (int64_t vv = 0; vv < V; ++vv) denom += exp(z[vv] - m);
  double ent = 0.0;
  for (int64_t vv = 0; vv < V; ++vv) {
    double p = exp(z[vv] - m) / denom;
    if (p > 0.0) ent -= p * log(p);
  }
  *lse = m + log(denom);
  *entropy = ent;
  /* selection by repeated scan: k passes, each picks the best not yet taken */
  unsigned char* taken = (unsigned char*)calloc((size_t)V, 1);
  for (int n = 0; n < k; ++n) {
    int64_t best = -1;
    float bestv = 0.0f;
    for (int64_t vv = 0; vv < V; ++vv) {
      if (taken[vv]) continue;
      float zf = (float)z[vv];
      if (best < 0 || zf > bestv) {
        best = vv;
        bestv = zf;
      }
    }
    if (best < 0) {
      topk_ids[n] = -1;
      topk_probs[n] = 0.0;
      continue;
    }
    taken[best] = 1;
    topk_ids[n] = (int32_t)best;
    topk_probs[n] = exp(z[best] - m) / denom;
  }
  free(taken);
  *y = topk_ids[0];
  if (V >= 2) {
    double z1 = -INFINITY, z2 = -INFINITY;
    for (int64_t vv = 0; vv < V; ++vv) {
      if (z[vv] > z1) {
        z2 = z1;
        z1 = z[vv];
      } else if (z[vv] > z2) {
        z2 = z[vv];
      }
    }
    *margin = (z1 - z2) / (amax > 0.0 ? amax : 1.0);
  } else {
    *margin = INFINITY;
  }
}

/* ------------------------------------------------------------------------------------------
 * O4  loosened index set (Eq. 9): ascending argsort of the step's relevance scores, first
 * n_loose entries.  n_loose = floor(lambda * K) (slice semantics; lambda = 0.7, K = 10 gives 7,
 * i.e. visual density rho = 0.3 as the paper states).  Equal scores keep index order (stable).
 *   a [gamma] binary32 (the type the library passes relevance in), mask [gamma] 0/1,
 *   order [gamma] the full ascending argsort.
 * ------------------------------------------------------------------------------------------ */
int lvo_n_loose(double lambda, int gamma) {
  int n = (int)floor(lambda * (double)gamma + 1e-6);
  if (n < 0) n = 0;
  if (n > gamma) n = gamma;
  return n;
}

void lvo_loosened_set(int gamma, const float* a, int n_loose, uint8_t* mask, int32_t* order) {
  for (int i = 0; i < gamma; ++i) order[i] = i;
  /* insertion sort: stable, ascending */
  for (int i = 1; i < gamma; ++i) {
    int32_t cur = order[i];
    int j = i - 1;
    while (j >= 0 && a[order[j]] > a[cur]) {
      order[j + 1] = order[j];
      --j;
    }
    order[j + 1] = cur;
  }
  for (int i = 0; i < gamma; ++i) mask[i] = 0;
  for (int n = 0; n < n_loose && n < gamma; ++n) mask[order[n]] = 1;
}

/* ------------------------------------------------------------------------------------------
 * O5  verdicts (Eq. 10 and its position-shift-tolerant form Eq. 11) and accepted length
 * (Eq. 2, longest accepted prefix).
 * For position i, first rule that fires:
 *   1 EXACT   draft[i] == target[i]
 *   2 LOOSE   i is in the loosened set (and, only when gate_ok != NULL, gate_ok[i] != 0; the
 *             paper's rule has no gate)
 *   3 PST     the target's token target[i] occurs among the drafts at some k != i with
 *             |k - i| <= pst_window   (pst_window >= gamma-1 is the paper's whole-draft range;
 *             0 switches the mechanism off)
 *   0 REJECT  otherwise
 * tau = number of leading non-REJECT verdicts.
 * target holds n_target >= gamma tokens: the target's token at each draft position and, with
 * n_target = gamma + 1, the token it generates after the last draft (the forward pass over
 * [last committed token, drafts] yields gamma + 1 rows; Eq. 1 lists the first gamma).  The
 * step's extra token (standard speculative decoding; the paper does not spell it out) is
 * bonus = target[tau] if tau < n_target else -1.
 * ------------------------------------------------------------------------------------------ */
void lvo_verdicts(int gamma, int n_target, const int32_t* draft, const int32_t* target,
                  const uint8_t* loose, const uint8_t* gate_ok, int pst_window, uint8_t* verdict,
                  int32_t* tau, int32_t* bonus) {
  for (int i = 0; i < gamma; ++i) {
    uint8_t vd = 0;
    if (draft[i] == target[i]) {
      vd = 1;
    } else if (loose[i] && (!gate_ok || gate_ok[i])) {
      vd = 2;
    } else if (pst_window > 0) {
      for (int k = 0; k < gamma; ++k) {
        int dist = k > i ? k - i : i - k;
        if (k != i && dist <= pst_window && draft[k] == target[i]) {
          vd = 3;
          break;
        }
      }
    }
    verdict[i] = vd;
  }
  int t = 0;
  while (t < gamma && verdict[t] != 0) ++t;
  *tau = t;
  *bonus = t < n_target ? target[t] : -1;
}

/* ------------------------------------------------------------------------------------------
 * O5e  the text-only loose rules the paper compares against (baselines paragraph of the
 * experiment setup; baseline-details appendix: window 4, entropy thresholds 0.1 and 0.2): an
 * entropy gate, alone or with a deferred window.  A mismatched draft token is accepted when the
 * entropy of the target's distribution at its position exceeds the threshold and every token of
 * the following window matches.
 * For position i, first rule that fires:
 *   1 EXACT   draft[i] == target[i]
 *   4 GATED   entropy[i] > threshold, and (window > 0) the positions i+1 .. i+window are all
 *             draft positions (i + window <= gamma - 1) and draft[k] == target[k] at each.
 *             Reading where the paper is silent: a window that runs past the last draft cannot
 *             be confirmed in this step, so the mismatch is not accepted; a position that is
 *             itself only accepted through the gate does not count as a match; the row after
 *             the last draft has no draft token and is not a window position.
 *   0 REJECT  otherwise
 * window == 0 is the gate alone.  entropy is binary32 (nats), the type the library holds it in,
 * and the comparison is made in that type.  tau and bonus as in O5.
 * ------------------------------------------------------------------------------------------ */
void lvo_verdicts_entropy(int gamma, int n_target, const int32_t* draft, const int32_t* target,
                          const float* entropy, float threshold, int window, uint8_t* verdict,
                          int32_t* tau, int32_t* bonus) {
  for (int i = 0; i < gamma; ++i) {
    uint8_t vd = 0;
    if (draft[i] == target[i]) {
      vd = 1;
    } else if (entropy[i] > threshold) {
      int confirmed = (i + window <= gamma - 1);
      for (int k = i + 1; confirmed && k <= i + window; ++k)
        if (draft[k] != target[k]) confirmed = 0;
      if (confirmed) vd = 4;
    }
    verdict[i] = vd;
  }
  int t = 0;
  while (t < gamma && verdict[t] != 0) ++t;
  *tau = t;
  *bonus = t < n_target ? target[t] : -1;
}

/* ------------------------------------------------------------------------------------------
 * O6  draft trees (appendix "Exploration on Draft Token Trees"): a static tree of n_branches
 * chains that share only the committed context; every chain is verified loosely on its own
 * (O4 and O5 per chain, ranking and shift window local to the chain) and the chain with the
 * longest accepted length is kept.  The paper does not say which chain wins a tie: the lowest
 * branch index does here.
 *   tau [n_branches] accepted lengths of one sequence's chains; returns the kept branch.
 * ------------------------------------------------------------------------------------------ */
int32_t lvo_select_branch(int n_branches, const int32_t* tau) {
  int32_t best = 0;
  for (int a = 1; a < n_branches; ++a)
    if (tau[a] > tau[best]) best = a;
  return best;
}
