// Small kernels that finish the two streamed contractions.  They run one or a few workgroups of
// 16 waves on a chip of 256 CUs, so what they cost is latency and instruction count, not
// bandwidth: loads are issued together and never consumed right behind their issue, loops over
// per-thread slots are branch-free, and selections run as wave-wide maxima over the DPP network.
//
// rel_finalize:    cosines from the split dot products / squared norms, then the mean of the
//                  Top-N largest cosines per draft row (paper Eq. 8).  The N-th largest value
//                  is found exactly (duplicates count by value) and the sum is taken in fixed
//                  point, so the result does not depend on thread scheduling.
// accept_finalize: merges the per-vocabulary-block (max, sum exp, top-k candidates) into the
//                  greedy target token and the k most probable tokens per draft row
//                  (optionally the row's softmax entropy).
// accept_decide:   one wave per chain, one lane per draft position: the paper's Eq. 9
//                  (loosened set), Eq. 10/11 (verdicts incl. position-shift tolerance) and
//                  Eq. 2 (accepted length = longest accepted prefix); the chains of a draft
//                  tree share a workgroup, which then keeps the longest one.
#include "lvspec_dev.h"
#include "lvspec_kernels.h"

namespace lvspec {

namespace {

constexpr int kFinThreads = 1024;
constexpr int kMaxBranches = 8;   // chains of a draft tree (one wave each)

constexpr int kCandCap = 4096;       // candidates kept in LDS for the exact selection

struct SelectScratch {
  uint32_t hist[kFinThreads / 64][256];   // one histogram per wave: 16x less contention
  uint32_t wave_tot[4];
  uint32_t prefix, remaining;
};

// Exact n-th largest of `count` keys (key_at(idx), idx < count), 1 <= n <= count, by a 4-pass
// most-significant-digit radix select.  Returns the key; *need_eq = how many keys equal to it
// belong to the n largest.  All threads of the block must call it.
template <class KeyAt>
LVS_DEV uint32_t radix_select(int count, int n, KeyAt key_at, SelectScratch& sc,
                              uint32_t* need_eq) {
  const int tid = threadIdx.x;
  if (tid == 0) {
    sc.prefix = 0;
    sc.remaining = (uint32_t)n;
  }
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int t = tid; t < (kFinThreads / 64) * 256; t += kFinThreads) (&sc.hist[0][0])[t] = 0;
    __syncthreads();
    const uint32_t prefix = sc.prefix;
    const uint32_t rem = sc.remaining;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int idx = tid; idx < count; idx += kFinThreads) {
      const uint32_t k = key_at(idx);
      if ((k & hi_mask) == prefix) atomicAdd(&sc.hist[tid >> 6][(k >> shift) & 0xffu], 1u);
    }
    __syncthreads();
    // suffix sums S[t] = sum_{u >= t} hist[u]; the selected digit is the t with
    // S[t] >= rem > S[t+1]
    uint32_t own = 0, suf = 0;
    if (tid < 256) {
#pragma unroll
      for (int w = 0; w < kFinThreads / 64; ++w) own += sc.hist[w][tid];
      suf = own;
      const int lane = tid & 63;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t o = __shfl_down(suf, off, 64);
        if (lane + off < 64) suf += o;
      }
      if (lane == 0) sc.wave_tot[tid >> 6] = suf;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = (tid >> 6) + 1; w < 4; ++w) suf += sc.wave_tot[w];
      if (suf >= rem && suf - own < rem) {
        sc.prefix = prefix | ((uint32_t)tid << shift);
        sc.remaining = rem - (suf - own);   // copies of the selected digit still needed
      }
    }
    __syncthreads();
  }
  const uint32_t key = sc.prefix;
  *need_eq = sc.remaining;
  __syncthreads();   // the scratch may be reused by the next call
  return key;
}

// Cosines of the rows j = jr + 1024 * u + tid, u < U, from the split partial sums.  Written for
// instruction count (16 waves share four SIMDs here): the row index is clamped instead of
// predicated, every split pointer is uniform (scalar base + one 32-bit lane offset per row), all
// loads of the round are issued before the first is used, splits past n_ds re-read split 0 with
// weight 0, and the cosine is dot * rsqrt(max(|v|^2, 1e-16)) / |h_d| (rsqrt of the clamped
// square = 1 / max(|v|, 1e-8)).  Writes the cosines to cosb and returns the largest key.
// pre: nbase holds the rows' prepared inverse norms (one plane, nstep = 0) instead of squared
// norms per split (planes nstep apart).
template <int U, int NS>
LVS_DEV uint32_t cos_round(int jr, int tid, int lv, int n_ds, const float* dbase,
                           const float* nbase, int64_t dstep, int64_t nstep, bool pre,
                           float inv_nd, float* cosb) {
  float dv[U][NS], nv[U][NS];
  uint32_t off[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int j = jr + u * kFinThreads + tid;
    off[u] = (uint32_t)(j < lv ? j : lv - 1) * 4u;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const int sc = s < n_ds ? s : 0;                                     // uniform
      const char* dp = reinterpret_cast<const char*>(dbase + sc * dstep);   // uniform
      const char* np = reinterpret_cast<const char*>(nbase + sc * nstep);   // uniform
      dv[u][s] = *reinterpret_cast<const float*>(dp + off[u]);
      nv[u][s] = *reinterpret_cast<const float*>(np + off[u]);
    }
  }
  uint32_t mk = 0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int j = jr + u * kFinThreads + tid;
    float dot = dv[u][0], n2 = nv[u][0];
#pragma unroll
    for (int s = 1; s < NS; ++s) {
      const float ws = s < n_ds ? 1.f : 0.f;                               // uniform
      dot = __builtin_fmaf(dv[u][s], ws, dot);
      n2 = __builtin_fmaf(nv[u][s], pre ? 0.f : ws, n2);
    }
    const float c = dot * (pre ? n2 : __builtin_amdgcn_rsqf(fmaxf(n2, 1e-16f))) * inv_nd;
    if (j < lv) *reinterpret_cast<float*>(reinterpret_cast<char*>(cosb) + off[u]) = c;
    mk = max(mk, j < lv ? order_key(c) : 0u);
  }
  return mk;
}

constexpr float kFixScale = 1099511627776.0f;   // 2^40: cosines as 64-bit fixed point

constexpr int kSmallN = 16;          // Top-N sizes served by the shuffle-based selection
constexpr int kSmallCand = 256;      // candidates wave 0 can hold (4 per lane)

// One round of "largest remaining key" over NK keys per lane: returns the key (0 = none
// left), counts its copies and retires them.  Wave-uniform result.
template <int NK>
LVS_DEV uint32_t take_largest(uint32_t (&k)[NK], int& copies) {
  uint32_t best = k[0];
#pragma unroll
  for (int j = 1; j < NK; ++j) best = max(best, k[j]);
  const uint32_t w = wave_max_u32(best);
  copies = 0;
#pragma unroll
  for (int j = 0; j < NK; ++j) {
    copies += __popcll(__ballot(k[j] == w));
    k[j] = k[j] == w ? 0u : k[j];
  }
  return w;
}

// SMALL: top_n <= kSmallN.  The two selections (the bound from the per-thread maxima, then the
// exact Top-N among the candidates) are then done by wave-wide maxima over the DPP network, a
// handful of instructions per round and five barriers in the whole kernel, instead of two
// 4-pass radix selects (about 36 barriers of 16 waves).  Rows with more than kSmallCand
// candidates (many values at the bound) continue on the general path.
template <bool SMALL>
__global__ __launch_bounds__(kFinThreads) void rel_finalize_kernel(const RelFinalizeArgs p) {
  __shared__ float red[16];
  __shared__ SelectScratch sc;
  __shared__ uint32_t tmax[kFinThreads];
  __shared__ float cand[kCandCap];
  __shared__ int cand_count;
  __shared__ long long fix_part[kFinThreads / 64];
  __shared__ uint32_t sm_top[4][kSmallN];
  __shared__ uint32_t sm_t0;
  const int i = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LVS_TRACE_BEGIN;
  LVS_TRACE(0);
  int lv = p.l_v[b];
  if (lv > p.lv_max) lv = (int)p.lv_max;
  float* rel_out = p.relevance + (int64_t)b * p.gamma + i;
  if (lv <= 0) {
    if (tid == 0) *rel_out = 0.f;
    return;
  }
  // |h_d row|^2 (rows are 16-byte aligned and d is a multiple of 128: eight elements per load)
  const uint16_t* hd = p.h_d + (int64_t)b * p.hd_sb + (int64_t)i * p.hd_sg;
  float part = 0.f;
  for (int t = tid * 8; t < p.d; t += kFinThreads * 8) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(hd + t);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __builtin_bit_cast(float, w[e] << 16);
      const float hi = __builtin_bit_cast(float, w[e] & 0xffff0000u);
      part = __builtin_fmaf(lo, lo, part);
      part = __builtin_fmaf(hi, hi, part);
    }
  }
  part = wave_sum(part);
  if (lane == 0) red[wave] = part;
  __syncthreads();
  float nd2 = 0.f;
#pragma unroll
  for (int w = 0; w < kFinThreads / 64; ++w) nd2 += red[w];
  const float inv_nd = 1.0f / fmaxf(sqrtf(nd2), 1e-8f);
  LVS_TRACE(1);
  float* cosb = p.cosbuf + ((int64_t)b * p.gamma + i) * p.ld;
  const float* dbase = p.dots + (((int64_t)b * p.n_ds) * p.gamma + i) * p.ld;
  const bool pre = p.inv_norm != nullptr;
  const float* nbase = pre ? p.inv_norm + (int64_t)b * p.lv_max
                           : p.nv2 + ((int64_t)b * p.n_ds) * p.ld;
  const int64_t nstep = pre ? 0 : p.ld;
  const int64_t dstep = (int64_t)p.gamma * p.ld;
  const int n_eff = p.top_n < lv ? p.top_n : lv;

  // ---- pass 1: cosines to the workspace (split partial sums added in split order), largest
  // value of every thread kept
  uint32_t mk = 0;
  if (p.n_ds == 1) {
    for (int jr = 0; jr < lv; jr += 16 * kFinThreads)
      mk = max(mk, cos_round<16, 1>(jr, tid, lv, 1, dbase, nbase, dstep, nstep, pre, inv_nd, cosb));
  } else if (p.n_ds == 2) {
    for (int jr = 0; jr < lv; jr += 8 * kFinThreads)
      mk = max(mk, cos_round<8, 2>(jr, tid, lv, 2, dbase, nbase, dstep, nstep, pre, inv_nd, cosb));
  } else {
    for (int jr = 0; jr < lv; jr += 2 * kFinThreads)
      mk = max(mk, cos_round<2, 8>(jr, tid, lv, p.n_ds, dbase, nbase, dstep, nstep, pre, inv_nd, cosb));
  }
  LVS_TRACE(2);
  // ---- lower bound of the answer: the n-th largest of the per-thread maxima.  At least n
  // values are >= it, so only values >= it can be among the n largest.
  uint32_t need_eq;
  uint32_t t0key;
  if (tid == 0) cand_count = 0;
  if constexpr (SMALL) {
    // the thread maxima go through LDS to waves 0..3 (four per lane, one wave per SIMD), each
    // of which lists the n_eff largest of its 256 (copies included) ...
    tmax[tid] = mk;
    __syncthreads();
    if (wave < 4) {
      uint32_t k4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) k4[j] = tmax[wave * 256 + 64 * j + lane];
      int got = 0;
      while (got < n_eff) {
        int copies;
        const uint32_t w = take_largest(k4, copies);
        if (w == 0u) break;
        if (lane < copies && got + lane < n_eff) sm_top[wave][got + lane] = w;
        got += copies;
      }
      if (lane < kSmallN && lane >= got) sm_top[wave][lane] = 0u;
    }
    __syncthreads();
    // ... and wave 0 takes the n_eff-th largest of the four lists
    if (wave == 0) {
      uint32_t cur = (lane & (kSmallN - 1)) < n_eff ? sm_top[lane / kSmallN][lane & (kSmallN - 1)]
                                                    : 0u;
      uint32_t t0 = 0u;
      for (int got = 0; got < n_eff;) {
        const uint32_t w = wave_max_u32(cur);
        if (w == 0u) break;
        got += __popcll(__ballot(cur == w));
        cur = cur == w ? 0u : cur;
        t0 = w;
      }
      if (lane == 0) sm_t0 = t0;
    }
    __syncthreads();
    t0key = sm_t0;
  } else {
    tmax[tid] = mk;
    __syncthreads();
    t0key = radix_select(kFinThreads, n_eff, [&](int idx) { return tmax[idx]; }, sc, &need_eq);
  }
  LVS_TRACE(3);
  // ---- pass 2: every thread re-reads the cosines it wrote and keeps those >= the bound in
  // LDS (in no particular order: they are only counted, compared and summed exactly)
  for (int jr = 0; jr < lv; jr += 16 * kFinThreads) {
    float c[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int j = jr + u * kFinThreads + tid;
      c[u] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(cosb) +
                                             (uint32_t)(j < lv ? j : lv - 1) * 4u);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int j = jr + u * kFinThreads + tid;
      if (j < lv && order_key(c[u]) >= t0key) {
        const int slot = atomicAdd(&cand_count, 1);
        if (slot < kCandCap) cand[slot] = c[u];
      }
    }
  }
  __syncthreads();
  LVS_TRACE(4);
  const int total = cand_count;
  if constexpr (SMALL) {
    if (total <= kSmallCand) {
      // exact Top-N among the candidates by wave 0: largest first, copies counted by value;
      // the sum is taken in 2^-40 fixed point like on the general path, so both give the same
      // bits
      if (wave != 0) return;
      uint32_t k4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int idx = lane + 64 * j;
        k4[j] = idx < total ? order_key(cand[idx]) : 0u;
      }
      long long tot = 0;
      for (int got = 0; got < n_eff;) {
        int copies;
        const uint32_t w = take_largest(k4, copies);
        if (w == 0u) break;
        const int take = copies < n_eff - got ? copies : n_eff - got;
        tot += (long long)take * (long long)(key_value(w) * kFixScale);
        got += copies;
      }
      if (lane == 0) *rel_out = (float)((double)tot / (double)kFixScale / (double)n_eff);
      LVS_TRACE(5);
      LVS_TRACE_END;
      return;
    }
  }
  uint32_t tkey;
  long long fix = 0;     // sum of the values above the n-th largest, exact in 2^-40 units
  if (total <= kCandCap) {
    tkey = radix_select(total, n_eff, [&](int idx) { return order_key(cand[idx]); }, sc, &need_eq);
    for (int idx = tid; idx < total; idx += kFinThreads)
      if (order_key(cand[idx]) > tkey) fix += (long long)(cand[idx] * kFixScale);
  } else {
    // (many equal values at the bound) select over the whole row in the workspace
    tkey = radix_select(lv, n_eff, [&](int idx) { return order_key(cosb[idx]); }, sc, &need_eq);
    for (int j = tid; j < lv; j += kFinThreads) {
      const float c = cosb[j];
      if (order_key(c) > tkey) fix += (long long)(c * kFixScale);
    }
  }
  // integer addition is associative: any reduction order gives the same bits
#pragma unroll
  for (int sft = 1; sft < 64; sft <<= 1) fix += __shfl_xor(fix, sft, 64);
  if ((tid & 63) == 0) fix_part[tid >> 6] = fix;
  __syncthreads();
  if (tid == 0) {
    long long tot = 0;
    for (int w = 0; w < kFinThreads / 64; ++w) tot += fix_part[w];
    tot += (long long)need_eq * (long long)(key_value(tkey) * kFixScale);
    *rel_out = (float)((double)tot / (double)kFixScale / (double)n_eff);
  }
}

// ------------------------------------------------------------------------------------------
constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / 64;
constexpr int kCandRegs = 20;     // candidates a thread can keep in registers (V = 152064, k = 16)

// (value desc, id asc) order, written without short-circuit branches
LVS_DEV bool better(float v, int id, float bv, int bid) {
  return (v > bv) | ((v == bv) & (id < bid));
}

// Merge of the per-vocabulary-block statistics and top-k candidates of one logits column when
// all candidates fit in registers (kCandRegs per thread: any k at V = 152064).  Every wave
// first selects the k best of its own candidates with k wave-wide maxima over the DPP network
// (no LDS, no barrier), then wave 0 selects the k best of the 16 x k survivors the same way:
// two barriers in the whole kernel.  SLOTS = candidates per thread, a compile-time bound so that
// the loops over them carry no branches (a taken branch costs about as much as five vector
// instructions, and there would be two per slot and round).
template <int SLOTS>
__global__ __launch_bounds__(kAccThreads) void accept_finalize_kernel(const AcceptFinalizeArgs p) {
  __shared__ float red_max[kAccWaves], red_sum[kAccWaves], red_sz[kAccWaves];
  __shared__ uint64_t sm_keys[kAccWaves * 16];
  const int i = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = b * p.rows + i;
  const int n_cand = p.n_tasks * p.topk;
  LVS_TRACE_BEGIN;
  LVS_TRACE(0);

  // candidates of this thread (requested first: they are not needed before the rounds below)
  float cv[SLOTS];
  int ci[SLOTS];
#pragma unroll
  for (int u = 0; u < SLOTS; ++u) {
    const int c = tid + u * kAccThreads;
    const int cc = c < n_cand ? c : n_cand - 1;
    const int t = (int)fast_div((uint32_t)cc, p.div_topk);
    const int e = cc - t * p.topk;
    const int64_t off = ((int64_t)t * p.n_cols + col) * p.topk + e;
    ci[u] = p.cand_idx[off];     // (no use of the loaded values here: a select on them
    cv[u] = p.cand_val[off];     // would make every slot wait for its own load)
  }
  LVS_TRACE(1);
  // global max and denominator over the vocabulary blocks
  constexpr int kStatRegs = 2;
  float smax[kStatRegs], ssum[kStatRegs];
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < kStatRegs; ++u) {
    const int t = tid + u * kAccThreads;
    smax[u] = -INFINITY;
    ssum[u] = 0.f;
    if (t < p.n_tasks) {
      const float* st = p.stats + ((int64_t)t * p.n_cols + col) * 2;
      smax[u] = st[0];
      ssum[u] = st[1];
    }
  }
#pragma unroll
  for (int u = 0; u < kStatRegs; ++u) mx = fmaxf(mx, smax[u]);
  for (int t = tid + kStatRegs * kAccThreads; t < p.n_tasks; t += kAccThreads)
    mx = fmaxf(mx, p.stats[((int64_t)t * p.n_cols + col) * 2]);
  mx = wave_max(mx);
  if (lane == 0) red_max[wave] = mx;
  LVS_TRACE(5);

  // ---- the k best candidates of this wave ---------------------------------------------------
  uint64_t key[SLOTS];
#pragma unroll
  for (int u = 0; u < SLOTS; ++u)   // slots past the end hold a clamped copy
    key[u] = tid + u * kAccThreads < n_cand ? cand_key(cv[u], ci[u]) : 0ull;
  uint64_t mine = 0;     // lane r keeps the wave's r-th best
  for (int r = 0; r < p.topk; ++r) {
    uint64_t best = 0;
#pragma unroll
    for (int u = 0; u < SLOTS; ++u) best = key[u] > best ? key[u] : best;
    const uint64_t w = wave_max_u64(best);
#pragma unroll
    for (int u = 0; u < SLOTS; ++u) key[u] = key[u] == w ? 0ull : key[u];
    mine = lane == r ? w : mine;
  }
  if (lane < p.topk) sm_keys[wave * 16 + lane] = mine;
  LVS_TRACE(6);
  __syncthreads();
  LVS_TRACE(2);
  mx = wave_max(lane < kAccWaves ? red_max[lane] : -INFINITY);
  float se = 0.f;
#pragma unroll
  for (int u = 0; u < kStatRegs; ++u) se += ssum[u] * __expf(smax[u] - mx);
  for (int t = tid + kStatRegs * kAccThreads; t < p.n_tasks; t += kAccThreads) {
    const float* st = p.stats + ((int64_t)t * p.n_cols + col) * 2;
    se += st[1] * __expf(st[0] - mx);
  }
  se = wave_sum(se);
  if (lane == 0) red_sum[wave] = se;
  if (p.entropy != nullptr) {   // same rescaling for the blocks' sum exp(z - max) * z
    float sz = 0.f;
    for (int t = tid; t < p.n_tasks; t += kAccThreads) {
      const int64_t rec = (int64_t)t * p.n_cols + col;
      sz += p.stats_z[rec] * __expf(p.stats[rec * 2] - mx);
    }
    sz = wave_sum(sz);
    if (lane == 0) red_sz[wave] = sz;
  }
  __syncthreads();
  LVS_TRACE(3);
  if (wave != 0) return;

  // ---- wave 0: the k best of the 16 x k survivors, denominators, results --------------------
  se = wave_sum(lane < kAccWaves ? red_sum[lane] : 0.f);
  if (p.entropy != nullptr) {
    // H = -sum p ln p with p = exp(z - max) / se:  ln se + max - (sum exp(z - max) z) / se
    const float sz = wave_sum(lane < kAccWaves ? red_sz[lane] : 0.f);
    if (lane == 0) p.entropy[col] = __logf(se) + mx - sz / se;
  }
  uint64_t k4[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int idx = lane + 64 * j;          // wave idx / 16, rank idx % 16
    k4[j] = (idx & 15) < p.topk ? sm_keys[idx] : 0ull;
  }
  mine = 0;
  for (int r = 0; r < p.topk; ++r) {
    uint64_t best = k4[0] > k4[1] ? k4[0] : k4[1];
    const uint64_t b2 = k4[2] > k4[3] ? k4[2] : k4[3];
    best = best > b2 ? best : b2;
    const uint64_t w = wave_max_u64(best);
#pragma unroll
    for (int j = 0; j < 4; ++j) k4[j] = k4[j] == w ? 0ull : k4[j];
    mine = lane == r ? w : mine;
  }
  if (lane < p.topk) {
    const bool none = mine == 0ull;
    const float win_v = key_value((uint32_t)(mine >> 32));
    const int out_id = none ? -1 : 0x7fffffff - (int)(uint32_t)mine;
    const float prob = none ? 0.f : __expf(win_v - mx) / se;
    if (lane == 0) p.target_ids[col] = out_id;
    p.ws_topk_ids[col * 16 + lane] = out_id;
    if (p.topk_ids) p.topk_ids[(int64_t)col * p.topk + lane] = out_id;
    if (p.topk_probs) p.topk_probs[(int64_t)col * p.topk + lane] = prob;
  }
  LVS_TRACE(4);
  LVS_TRACE_END;
}

// The same merge for candidate counts beyond the register budget: every round re-reads the
// candidates from memory.
__global__ __launch_bounds__(kAccThreads) void accept_finalize_general_kernel(
    const AcceptFinalizeArgs p) {
  __shared__ float redf[2][kAccWaves];
  __shared__ int redi[2][kAccWaves];
  const int i = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = b * p.rows + i;
  const int n_cand = p.n_tasks * p.topk;
  const bool in_regs = n_cand <= kCandRegs * kAccThreads;
  LVS_TRACE_BEGIN;
  LVS_TRACE(0);

  // candidates of this thread (requested first: they are not needed before the rounds below)
  float cv[kCandRegs];
  int ci[kCandRegs];
  if (in_regs) {
#pragma unroll
    for (int u = 0; u < kCandRegs; ++u) {
      const int c = tid + u * kAccThreads;
      cv[u] = -INFINITY;
      ci[u] = -1;
      if (c < n_cand) {
        const int t = c / p.topk;
        const int e = c - t * p.topk;
        const int64_t off = ((int64_t)t * p.n_cols + col) * p.topk + e;
        ci[u] = p.cand_idx[off];
        cv[u] = p.cand_val[off];
      }
    }
  }

  LVS_TRACE(1);
  // global max and denominator over the vocabulary blocks (each block's pair loaded once)
  constexpr int kStatRegs = 2;
  float smax[kStatRegs], ssum[kStatRegs];
  float mx = -INFINITY;
#pragma unroll
  for (int u = 0; u < kStatRegs; ++u) {
    const int t = tid + u * kAccThreads;
    smax[u] = -INFINITY;
    ssum[u] = 0.f;
    if (t < p.n_tasks) {
      const float* st = p.stats + ((int64_t)t * p.n_cols + col) * 2;
      smax[u] = st[0];
      ssum[u] = st[1];
    }
  }
#pragma unroll
  for (int u = 0; u < kStatRegs; ++u) mx = fmaxf(mx, smax[u]);
  for (int t = tid + kStatRegs * kAccThreads; t < p.n_tasks; t += kAccThreads)
    mx = fmaxf(mx, p.stats[((int64_t)t * p.n_cols + col) * 2]);
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
  if (lane == 0) redf[0][wave] = mx;
  __syncthreads();
  mx = redf[0][0];
  for (int w = 1; w < kAccWaves; ++w) mx = fmaxf(mx, redf[0][w]);
  LVS_TRACE(2);
  float se = 0.f;
#pragma unroll
  for (int u = 0; u < kStatRegs; ++u) se += ssum[u] * __expf(smax[u] - mx);
  for (int t = tid + kStatRegs * kAccThreads; t < p.n_tasks; t += kAccThreads) {
    const float* st = p.stats + ((int64_t)t * p.n_cols + col) * 2;
    se += st[1] * __expf(st[0] - mx);
  }
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) se += __shfl_xor(se, s, 64);
  if (lane == 0) redf[1][wave] = se;
  __syncthreads();
  se = 0.f;
  for (int w = 0; w < kAccWaves; ++w) se += redf[1][w];
  __syncthreads();
  if (p.entropy != nullptr) {   // see accept_finalize_kernel
    float sz = 0.f;
    for (int t = tid; t < p.n_tasks; t += kAccThreads) {
      const int64_t rec = (int64_t)t * p.n_cols + col;
      sz += p.stats_z[rec] * __expf(p.stats[rec * 2] - mx);
    }
    sz = wave_sum(sz);
    if (lane == 0) redf[1][wave] = sz;
    __syncthreads();
    sz = 0.f;
    for (int w = 0; w < kAccWaves; ++w) sz += redf[1][w];
    if (tid == 0) p.entropy[col] = __logf(se) + mx - sz / se;
    __syncthreads();
  }

  LVS_TRACE(3);
  // k rounds: best candidate strictly after the previous winner in (value desc, id asc) order
  float pv = INFINITY, win_v = -INFINITY;
  int pid = -1, win_i = -1;
  for (int r = 0; r < p.topk; ++r) {
    float bv = -INFINITY;
    int bid = 0x7fffffff;
    if (in_regs) {
#pragma unroll
      for (int u = 0; u < kCandRegs; ++u) {
        const bool after_prev = (cv[u] < pv) | ((cv[u] == pv) & (ci[u] > pid));
        const bool take = (ci[u] >= 0) & after_prev & better(cv[u], ci[u], bv, bid);
        bv = take ? cv[u] : bv;
        bid = take ? ci[u] : bid;
      }
    } else {
      for (int c = tid; c < n_cand; c += kAccThreads) {
        const int t = c / p.topk;
        const int e = c - t * p.topk;
        const int64_t off = ((int64_t)t * p.n_cols + col) * p.topk + e;
        const int id = p.cand_idx[off];
        const float v = p.cand_val[off];
        const bool after_prev = v < pv || (v == pv && id > pid);
        if (id >= 0 && after_prev && better(v, id, bv, bid)) {
          bv = v;
          bid = id;
        }
      }
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const float ov = __shfl_xor(bv, s, 64);
      const int oi = __shfl_xor(bid, s, 64);
      const bool take = better(ov, oi, bv, bid);
      bv = take ? ov : bv;
      bid = take ? oi : bid;
    }
    const int buf = r & 1;
    if (lane == 0) {
      redf[buf][wave] = bv;
      redi[buf][wave] = bid;
    }
    __syncthreads();
    pv = redf[buf][0];
    pid = redi[buf][0];
#pragma unroll
    for (int w = 1; w < kAccWaves; ++w) {
      const float ov = redf[buf][w];
      const int oi = redi[buf][w];
      const bool take = better(ov, oi, pv, pid);
      pv = take ? ov : pv;
      pid = take ? oi : pid;
    }
    if (tid == r) {   // thread r keeps the winner of round r; results are stored after the loop
      win_v = pv;     // (a store inside the loop would be waited for at every barrier)
      win_i = pid;
    }
  }
  if (tid < p.topk) {
    const int out_id = win_v == -INFINITY ? -1 : win_i;
    const float prob = win_v == -INFINITY ? 0.f : __expf(win_v - mx) / se;
    if (tid == 0) p.target_ids[col] = out_id;
    p.ws_topk_ids[col * 16 + tid] = out_id;
    if (p.topk_ids) p.topk_ids[(int64_t)col * p.topk + tid] = out_id;
    if (p.topk_probs) p.topk_probs[(int64_t)col * p.topk + tid] = prob;
  }
  LVS_TRACE(4);
  LVS_TRACE_END;
}

// One workgroup per sequence, one wave per chain of its draft tree (a plain chain draft is a
// tree with one branch), one lane per draft position: loosened set (Eq. 9), verdicts (Eq. 10 /
// 11), accepted length (Eq. 2) per chain, then the chain with the longest accepted length
// (appendix on draft token trees).  Everything a position needs from the others comes through
// v_readlane in a loop over the positions, so there is no serial single-lane code and no LDS
// traffic.  Runs after accept_finalize_kernel in stream order, so the target tokens are visible
// without any in-kernel fence.
__global__ __launch_bounds__(64 * kMaxBranches) void accept_decide_kernel(
    const AcceptFinalizeArgs p) {
  __shared__ int sh_tau[kMaxBranches];
  const int seq = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int br = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // branch of this wave
  const int b = seq * p.n_branches + br;                             // chain index
  const int g = p.gamma;
  const bool on = lane < g;
  const int idx = b * g + (on ? lane : 0);                 // draft position of this lane
  const int row = b * p.rows + (lane < p.rows ? lane : 0);  // hidden row of this lane
  const int dk = p.draft_ids[idx];
  const int yk = p.target_ids[row];
  unsigned char vd = 0;
  if (p.rule == 0) {
    const float ak = p.relevance[idx];
    int gate_ok = 1;
    if (p.gate > 0) {
      gate_ok = 0;
      for (int e = 0; e < p.gate; ++e) gate_ok |= (p.ws_topk_ids[row * 16 + e] == dk);
    }
    // position of this lane in the stable ascending order of the relevance scores (Eq. 9: the
    // n_loose first are loosened), and whether its target token occurs among the other drafts
    // within the shift window (Eq. 11)
    int rank = 0;
    bool shifted = false;
    for (int j = 0; j < g; ++j) {
      const float aj = __builtin_bit_cast(
          float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, ak), j));
      const int dj = __builtin_amdgcn_readlane(dk, j);
      rank += ((aj < ak) | ((aj == ak) & (j < lane))) ? 1 : 0;
      const int dist = j > lane ? j - lane : lane - j;
      shifted |= (j != lane) & (dist <= p.pst_window) & (dj == yk);
    }
    if (dk == yk) {
      vd = 1;
    } else if (rank < p.n_loose && gate_ok) {
      vd = 2;
    } else if (p.pst_window > 0 && shifted) {
      vd = 3;
    }
  } else {
    // Entropy-gated rules of the text-only loose methods the paper compares against: a
    // mismatch passes when its row's entropy exceeds the threshold and (rule 2) the w
    // positions behind it are all draft positions that match exactly.  The row entropies were
    // written by accept_finalize_kernel earlier in stream order.
    const float hk = p.ent_rows[row];
    const unsigned long long exact = __ballot(on && dk == yk);
    const int w = p.rule == 2 ? p.defer_window : 0;
    const unsigned long long need = ((1ull << w) - 1ull) << (on ? lane + 1 : 0);   // < 2^33
    const bool confirmed = (lane + w <= g - 1) && ((exact & need) == need);
    if (dk == yk) {
      vd = 1;
    } else if (hk > p.ent_threshold && confirmed) {
      vd = 4;
    }
  }
  if (on) p.verdict[idx] = vd;
  const unsigned long long rejected = __ballot(on && vd == 0);
  const int tau = rejected ? __ffsll((long long)rejected) - 1 : g;   // first rejected position
  // the target's token at the first rejected position, or the one after the last draft when
  // the chain brought that row
  const int bonus = __builtin_amdgcn_readlane(yk, tau < p.rows ? tau : 0);
  if (lane == 0) {
    p.accept_len[b] = tau;
    p.bonus_id[b] = tau < p.rows ? bonus : -1;
    sh_tau[br] = tau;
  }
  __syncthreads();
  if (threadIdx.x == 0 && p.best_branch != nullptr) {
    int best = 0;
    for (int a = 1; a < p.n_branches; ++a)
      if (sh_tau[a] > sh_tau[best]) best = a;
    p.best_branch[seq] = best;
  }
}

// ------------------------------------------------------------------------------------------
// Two-kernel Top-N for N <= 16 and up to 65536 video rows: the row is cut into slices of 1024
// video tokens, one small workgroup per (slice, draft row) keeps the slice's N largest scores
// (rel_cand_kernel, hundreds of workgroups spread over the chip), and one workgroup per draft
// row takes the N largest of the slices' lists (rel_merge_kernel).  The single-workgroup kernel
// above does all of a row's work on one CU, which at 63488 video rows is 54 us of mostly
// serial latency.
//
// Scores are ranked as s = dot * rsqrt(max(|v|^2, 1e-16)); the cosine is s / |h_d| with
// |h_d| > 0 constant over the row, so the order is the same, and the merge kernel applies the
// factor to the N winners (the same floating-point operations, in the same order, as the
// single-kernel path: both give the same bits).
template <int NS, bool MULTI>
__global__ __launch_bounds__(256) void rel_cand_kernel(const RelFinalizeArgs p) {
  __shared__ uint32_t sm_top[4][kRelSmallN];
  const int part = blockIdx.x;
  const int i = blockIdx.y;
  const int b = blockIdx.z;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int lv = p.l_v[b];
  if (lv > p.lv_max) lv = (int)p.lv_max;
  const int n = p.top_n;
  uint32_t* out = p.cand_keys + (((int64_t)b * p.gamma + i) * p.n_parts + part) * kRelSmallN;
  const int j0 = part * p.slice_rows;
  if (j0 >= lv) {   // slice past the sequence's video tokens: an empty list
    if (tid < kRelSmallN) out[tid] = 0u;
    return;
  }
  const float* dbase = p.dots + (((int64_t)b * p.n_ds) * p.gamma + i) * p.ld;
  const bool pre = p.inv_norm != nullptr;   // prepared inverse norms instead of squared norms
  const float* nbase = pre ? p.inv_norm + (int64_t)b * p.lv_max
                           : p.nv2 + ((int64_t)b * p.n_ds) * p.ld;
  const int64_t nstep = pre ? 0 : p.ld;
  const int64_t dstep = (int64_t)p.gamma * p.ld;
  // The slice is taken 1024 rows (four per thread) at a time; MULTI: slices of several such
  // chunks (more than 65536 video rows), each wave carrying its list of the n largest so far
  // (one entry per lane) into the selection of the next chunk.
  constexpr int NK = MULTI ? 5 : 4;
  const int jend = j0 + p.slice_rows < lv ? j0 + p.slice_rows : lv;
  for (int jc = j0; jc < jend; jc += kRelSliceRows) {
    float dv[4][NS], nv[4][NS];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = jc + u * 256 + tid;
      const uint32_t off = (uint32_t)(j < lv ? j : lv - 1) * 4u;
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const int sc = s < p.n_ds ? s : 0;
        dv[u][s] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(dbase + sc * dstep) + off);
        nv[u][s] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(nbase + sc * nstep) + off);
      }
    }
    uint32_t k[NK];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float dot = dv[u][0], n2 = nv[u][0];
#pragma unroll
      for (int s = 1; s < NS; ++s) {
        const float ws = s < p.n_ds ? 1.f : 0.f;
        dot = __builtin_fmaf(dv[u][s], ws, dot);
        n2 = __builtin_fmaf(nv[u][s], pre ? 0.f : ws, n2);
      }
      const float sc = dot * (pre ? n2 : __builtin_amdgcn_rsqf(fmaxf(n2, 1e-16f)));
      k[u] = jc + u * 256 + tid < jend ? order_key(sc) : 0u;
    }
    if constexpr (MULTI) k[4] = (jc > j0 && lane < n) ? sm_top[wave][lane] : 0u;
    // the n largest of this wave's scores so far (copies included) ...
    int got = 0;
    while (got < n) {
      int copies;
      const uint32_t w = take_largest(k, copies);
      if (w == 0u) break;
      if (lane < copies && got + lane < n) sm_top[wave][got + lane] = w;
      got += copies;
    }
    if (lane < kRelSmallN && lane >= got) sm_top[wave][lane] = 0u;
    if constexpr (!MULTI) break;
  }
  __syncthreads();
  if (wave != 0) return;
  // ... and of the four waves' lists
  uint32_t cur = (lane & (kRelSmallN - 1)) < n ? sm_top[lane / kRelSmallN][lane & (kRelSmallN - 1)]
                                               : 0u;
  int got = 0;
  while (got < n) {
    const uint32_t w = wave_max_u32(cur);
    if (w == 0u) break;
    const int copies = __popcll(__ballot(cur == w));
    if (lane < copies && got + lane < n) out[got + lane] = w;
    cur = cur == w ? 0u : cur;
    got += copies;
  }
  if (lane < kRelSmallN && lane >= (got < n ? got : n)) out[lane] = 0u;
}

__global__ __launch_bounds__(256) void rel_merge_kernel(const RelFinalizeArgs p) {
  __shared__ float red[4];
  __shared__ uint32_t sm_top[4][kRelSmallN];
  const int i = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int lv = p.l_v[b];
  if (lv > p.lv_max) lv = (int)p.lv_max;
  float* rel_out = p.relevance + (int64_t)b * p.gamma + i;
  if (lv <= 0) {
    if (tid == 0) *rel_out = 0.f;
    return;
  }
  const int n_eff = p.top_n < lv ? p.top_n : lv;
  // the slices' lists: n_parts * 16 keys, four per thread (n_parts <= 64)
  const uint32_t* keys = p.cand_keys + ((int64_t)b * p.gamma + i) * p.n_parts * kRelSmallN;
  const int total = p.n_parts * kRelSmallN;
  uint32_t k4[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int idx = u * 256 + tid;
    k4[u] = keys[idx < total ? idx : total - 1];
  }
  // |h_d row| while the keys are on their way
  const uint16_t* hd = p.h_d + (int64_t)b * p.hd_sb + (int64_t)i * p.hd_sg;
  float part = 0.f;
  for (int t = tid * 8; t < p.d; t += 256 * 8) {
    const u32x4 w = *reinterpret_cast<const u32x4*>(hd + t);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __builtin_bit_cast(float, w[e] << 16);
      const float hi = __builtin_bit_cast(float, w[e] & 0xffff0000u);
      part = __builtin_fmaf(lo, lo, part);
      part = __builtin_fmaf(hi, hi, part);
    }
  }
  part = wave_sum(part);
  if (lane == 0) red[wave] = part;
#pragma unroll
  for (int u = 0; u < 4; ++u) k4[u] = u * 256 + tid < total ? k4[u] : 0u;
  int got = 0;
  while (got < n_eff) {
    int copies;
    const uint32_t w = take_largest(k4, copies);
    if (w == 0u) break;
    if (lane < copies && got + lane < n_eff) sm_top[wave][got + lane] = w;
    got += copies;
  }
  if (lane < kRelSmallN && lane >= got) sm_top[wave][lane] = 0u;
  __syncthreads();
  if (wave != 0) return;
  const float inv_nd = 1.0f / fmaxf(sqrtf(((red[0] + red[1]) + red[2]) + red[3]), 1e-8f);
  uint32_t cur = (lane & (kRelSmallN - 1)) < n_eff
                     ? sm_top[lane / kRelSmallN][lane & (kRelSmallN - 1)]
                     : 0u;
  long long tot = 0;
  got = 0;
  while (got < n_eff) {
    const uint32_t w = wave_max_u32(cur);
    if (w == 0u) break;
    const int copies = __popcll(__ballot(cur == w));
    const int take = copies < n_eff - got ? copies : n_eff - got;
    tot += (long long)take * (long long)(key_value(w) * inv_nd * kFixScale);
    cur = cur == w ? 0u : cur;
    got += copies;
  }
  if (lane == 0) *rel_out = (float)((double)tot / (double)kFixScale / (double)n_eff);
}

}  // namespace

hipError_t launch_rel_finalize(const RelFinalizeArgs& a, hipStream_t stream) {
  static_assert(kRelSmallN == kSmallN, "same small-N bound on both paths");
  if (a.top_n <= kRelSmallN && a.n_parts >= 1 && a.n_parts <= kRelMaxParts &&
      a.slice_rows >= kRelSliceRows && a.slice_rows % kRelSliceRows == 0) {
    const dim3 grid(a.n_parts, a.gamma, a.B);
    const bool multi = a.slice_rows > kRelSliceRows;
    if (a.n_ds == 1) {
      if (multi) hipLaunchKernelGGL((rel_cand_kernel<1, true>), grid, dim3(256), 0, stream, a);
      else hipLaunchKernelGGL((rel_cand_kernel<1, false>), grid, dim3(256), 0, stream, a);
    } else if (a.n_ds == 2) {
      if (multi) hipLaunchKernelGGL((rel_cand_kernel<2, true>), grid, dim3(256), 0, stream, a);
      else hipLaunchKernelGGL((rel_cand_kernel<2, false>), grid, dim3(256), 0, stream, a);
    } else {
      if (multi) hipLaunchKernelGGL((rel_cand_kernel<8, true>), grid, dim3(256), 0, stream, a);
      else hipLaunchKernelGGL((rel_cand_kernel<8, false>), grid, dim3(256), 0, stream, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rel_merge_kernel, dim3(a.gamma, a.B), dim3(256), 0, stream, a);
    return hipGetLastError();
  }
  if (a.top_n <= kSmallN)
    hipLaunchKernelGGL(rel_finalize_kernel<true>, dim3(a.gamma, a.B), dim3(kFinThreads), 0, stream,
                       a);
  else
    hipLaunchKernelGGL(rel_finalize_kernel<false>, dim3(a.gamma, a.B), dim3(kFinThreads), 0,
                       stream, a);
  return hipGetLastError();
}

hipError_t launch_accept_finalize(const AcceptFinalizeArgs& a, hipStream_t stream) {
  static_assert(kCandRegs * kAccThreads == kAcceptRegCandidates, "planner and merge kernel agree");
  const int64_t n_cand = (int64_t)a.n_tasks * a.topk;
  const dim3 grid(a.rows, a.B);
  if (n_cand <= 5 * kAccThreads)
    hipLaunchKernelGGL(accept_finalize_kernel<5>, grid, dim3(kAccThreads), 0, stream, a);
  else if (n_cand <= 10 * kAccThreads)
    hipLaunchKernelGGL(accept_finalize_kernel<10>, grid, dim3(kAccThreads), 0, stream, a);
  else if (n_cand <= (int64_t)kCandRegs * kAccThreads)
    hipLaunchKernelGGL(accept_finalize_kernel<kCandRegs>, grid, dim3(kAccThreads), 0, stream, a);
  else
    hipLaunchKernelGGL(accept_finalize_general_kernel, grid, dim3(kAccThreads), 0,
                       stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(accept_decide_kernel, dim3(a.B / a.n_branches), dim3(64 * a.n_branches), 0,
                     stream, a);
  return hipGetLastError();
}

}  // namespace lvspec
