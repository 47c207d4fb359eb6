// Small latency-bound kernels that finish the two streamed contractions.
//
// rel_finalize:    cosines from the split dot products / squared norms, then the mean of the
//                  Top-N largest cosines per draft row (paper Eq. 8).  The N-th largest value
//                  is found exactly with a 4-pass radix select over order-preserving integer
//                  keys, so duplicates count by value and the result does not depend on
//                  thread scheduling.
// accept_finalize: merges the per-vocabulary-block (max, sum exp, top-k candidates) into the
//                  greedy target token and the k most probable tokens per draft row; the last
//                  workgroup of a sequence then applies the paper's Eq. 9 (loosened set),
//                  Eq. 10/11 (verdicts incl. position-shift tolerance) and Eq. 2 (accepted
//                  length = longest accepted prefix).
#include "lvspec_dev.h"
#include "lvspec_kernels.h"

namespace lvspec {

namespace {

constexpr int kFinThreads = 1024;

LVS_DEV uint32_t order_key(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

LVS_DEV float key_value(uint32_t k) {
  const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __builtin_bit_cast(float, u);
}

// deterministic block sum: lanes butterfly, then waves in index order
LVS_DEV float block_sum(float x, float* scratch) {
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) x += __shfl_xor(x, s, 64);
  const int wave = threadIdx.x >> 6;
  const int nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[wave] = x;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < nw; ++w) t += scratch[w];
  return t;
}

__global__ __launch_bounds__(kFinThreads) void rel_finalize_kernel(const RelFinalizeArgs p) {
  __shared__ float red[16];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sel_prefix, sel_remaining;
  const int i = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  int lv = p.l_v[b];
  if (lv > p.lv_max) lv = (int)p.lv_max;
  float* rel_out = p.relevance + (int64_t)b * p.gamma + i;
  if (lv <= 0) {
    if (tid == 0) *rel_out = 0.f;
    return;
  }
  // |h_d row|^2
  const uint16_t* hd = p.h_d + (int64_t)b * p.hd_sb + (int64_t)i * p.hd_sg;
  float part = 0.f;
  for (int t = tid; t < p.d; t += kFinThreads) {
    const float x = __builtin_bit_cast(float, (uint32_t)hd[t] << 16);
    part = __builtin_fmaf(x, x, part);
  }
  const float nd = fmaxf(sqrtf(block_sum(part, red)), 1e-8f);
  // cosines
  float* cosb = p.cosbuf + ((int64_t)b * p.gamma + i) * p.ld;
  for (int j = tid; j < lv; j += kFinThreads) {
    float dot = 0.f, n2 = 0.f;
    for (int s = 0; s < p.n_ds; ++s) {
      dot += p.dots[(((int64_t)b * p.n_ds + s) * p.gamma + i) * p.ld + j];
      n2 += p.nv2[((int64_t)b * p.n_ds + s) * p.ld + j];
    }
    const float nv = fmaxf(sqrtf(n2), 1e-8f);
    cosb[j] = dot / (nd * nv);
  }
  // radix select of the n_eff-th largest key (each thread re-reads only what it wrote)
  const int n_eff = p.top_n < lv ? p.top_n : lv;
  if (tid == 0) {
    sel_prefix = 0;
    sel_remaining = (uint32_t)n_eff;
  }
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    const uint32_t prefix = sel_prefix;
    const uint32_t hi_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int j = tid; j < lv; j += kFinThreads) {
      const uint32_t k = order_key(cosb[j]);
      if ((k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & 0xffu], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t rem = sel_remaining;
      int dgt = 255;
      for (; dgt > 0; --dgt) {
        const uint32_t cnt = hist[dgt];
        if (cnt >= rem) break;
        rem -= cnt;
      }
      sel_prefix = prefix | ((uint32_t)dgt << shift);
      sel_remaining = rem;   // copies of the selected digit still needed
    }
    __syncthreads();
  }
  const uint32_t tkey = sel_prefix;          // exact key of the n_eff-th largest value
  const uint32_t need_eq = sel_remaining;    // how many values equal to it belong to the top
  float s = 0.f;
  for (int j = tid; j < lv; j += kFinThreads) {
    const float c = cosb[j];
    if (order_key(c) > tkey) s += c;
  }
  const float total = block_sum(s, red) + (float)need_eq * key_value(tkey);
  if (tid == 0) *rel_out = total / (float)n_eff;
}

// ------------------------------------------------------------------------------------------
constexpr int kAccThreads = 256;

struct Best {
  float v;
  int id;
};

LVS_DEV bool better(float v, int id, float bv, int bid) {
  return v > bv || (v == bv && id < bid);
}

__global__ __launch_bounds__(kAccThreads) void accept_finalize_kernel(const AcceptFinalizeArgs p) {
  __shared__ float redf[8];
  __shared__ int redi[8];
  __shared__ float bc_v;
  __shared__ int bc_i;
  __shared__ int is_last;
  const int i = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int col = b * p.gamma + i;

  // global max and denominator
  float mx = -INFINITY;
  for (int t = tid; t < p.n_tasks; t += kAccThreads)
    mx = fmaxf(mx, p.stats[((int64_t)t * p.n_cols + col) * 2]);
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) mx = fmaxf(mx, __shfl_xor(mx, s, 64));
  if (lane == 0) redf[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(redf[0], redf[1]), fmaxf(redf[2], redf[3]));
  __syncthreads();
  float se = 0.f;
  for (int t = tid; t < p.n_tasks; t += kAccThreads) {
    const float* st = p.stats + ((int64_t)t * p.n_cols + col) * 2;
    se += st[1] * __expf(st[0] - mx);
  }
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) se += __shfl_xor(se, s, 64);
  if (lane == 0) redf[4 + wave] = se;
  __syncthreads();
  se = ((redf[4] + redf[5]) + redf[6]) + redf[7];

  // k rounds: best candidate strictly after the previous winner in (value desc, id asc) order
  float pv = INFINITY;
  int pid = -1;
  const int n_cand = p.n_tasks * p.topk;
  for (int r = 0; r < p.topk; ++r) {
    float bv = -INFINITY;
    int bid = 0x7fffffff;
    for (int c = tid; c < n_cand; c += kAccThreads) {
      const int t = c / p.topk;
      const int e = c - t * p.topk;
      const int64_t off = ((int64_t)t * p.n_cols + col) * p.topk + e;
      const int id = p.cand_idx[off];
      if (id < 0) continue;
      const float v = p.cand_val[off];
      const bool after_prev = v < pv || (v == pv && id > pid);
      if (after_prev && better(v, id, bv, bid)) {
        bv = v;
        bid = id;
      }
    }
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const float ov = __shfl_xor(bv, s, 64);
      const int oi = __shfl_xor(bid, s, 64);
      if (better(ov, oi, bv, bid)) {
        bv = ov;
        bid = oi;
      }
    }
    __syncthreads();
    if (lane == 0) {
      redf[wave] = bv;
      redi[wave] = bid;
    }
    __syncthreads();
    if (tid == 0) {
      float fv = redf[0];
      int fi = redi[0];
      for (int w = 1; w < 4; ++w)
        if (better(redf[w], redi[w], fv, fi)) {
          fv = redf[w];
          fi = redi[w];
        }
      bc_v = fv;
      bc_i = fi;
    }
    __syncthreads();
    pv = bc_v;
    pid = bc_i;
    if (tid == 0) {
      const int out_id = pv == -INFINITY ? -1 : pid;
      const float prob = pv == -INFINITY ? 0.f : __expf(pv - mx) / se;
      if (r == 0) p.target_ids[col] = out_id;
      p.ws_topk_ids[col * 16 + r] = out_id;
      if (p.topk_ids) p.topk_ids[(int64_t)col * p.topk + r] = out_id;
      if (p.topk_probs) p.topk_probs[(int64_t)col * p.topk + r] = prob;
    }
  }

  // ---- the last workgroup of sequence b decides ------------------------------------------
  if (tid == 0) {
    __threadfence();
    const int old = atomicAdd(&p.counters[b], 1);
    is_last = (old == p.gamma - 1);
  }
  __syncthreads();
  if (!is_last || tid != 0) return;
  __threadfence();
  const int g = p.gamma;
  int y[16], dft[16], order[16];
  float a[16];
  unsigned char loose[16];
  for (int k = 0; k < g; ++k) {
    y[k] = __hip_atomic_load(&p.target_ids[b * g + k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    dft[k] = p.draft_ids[b * g + k];
    a[k] = p.relevance[b * g + k];
    order[k] = k;
    loose[k] = 0;
  }
  // stable ascending insertion sort of the relevance scores (Eq. 9)
  for (int k = 1; k < g; ++k) {
    const int cur = order[k];
    int j = k - 1;
    while (j >= 0 && a[order[j]] > a[cur]) {
      order[j + 1] = order[j];
      --j;
    }
    order[j + 1] = cur;
  }
  for (int n = 0; n < p.n_loose && n < g; ++n) loose[order[n]] = 1;
  int tau = g;
  bool open = true;
  for (int k = 0; k < g; ++k) {
    unsigned char vd = 0;
    if (dft[k] == y[k]) {
      vd = 1;
    } else {
      bool gate_ok = true;
      if (p.gate > 0) {
        gate_ok = false;
        for (int e = 0; e < p.gate; ++e) {
          const int id = __hip_atomic_load(&p.ws_topk_ids[(b * g + k) * 16 + e], __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
          gate_ok |= (id == dft[k]);
        }
      }
      if (loose[k] && gate_ok) {
        vd = 2;
      } else if (p.pst_window > 0) {
        for (int m = 0; m < g; ++m) {
          const int dist = m > k ? m - k : k - m;
          if (m != k && dist <= p.pst_window && dft[m] == y[k]) {
            vd = 3;
            break;
          }
        }
      }
    }
    p.verdict[b * g + k] = vd;
    if (vd == 0 && open) {
      tau = k;
      open = false;
    }
  }
  p.accept_len[b] = tau;
  p.bonus_id[b] = tau < g ? y[tau] : -1;
  p.counters[b] = 0;
}

}  // namespace

hipError_t launch_rel_finalize(const RelFinalizeArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(rel_finalize_kernel, dim3(a.gamma, a.B), dim3(kFinThreads), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_accept_finalize(const AcceptFinalizeArgs& a, hipStream_t stream) {
  hipLaunchKernelGGL(accept_finalize_kernel, dim3(a.gamma, a.B), dim3(kAccThreads), 0, stream, a);
  return hipGetLastError();
}

}  // namespace lvspec
