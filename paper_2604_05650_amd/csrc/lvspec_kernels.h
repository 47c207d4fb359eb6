// Host-visible launch interface between the C ABI (api.hip) and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace lvspec {

// Raises a kernel's dynamic-LDS limit once per device.  The HIP call is idempotent, so threads
// that race on a first launch may both make it; the per-device flag only saves later calls
// (devices past the table always make the call).
struct LdsLimitOnce {
  std::atomic<int> done[64] = {};
  hipError_t ensure(const void* kernel, size_t bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && tracked) done[dev].store(1, std::memory_order_release);
    return e;
  }
};

// Exact unsigned division by a launch-time constant without a divide: for 0 <= x < 2^27,
// x / d == (x * mul) >> shift with shift = 27 + ceil(log2 d), mul = ceil(2^shift / d) < 2^32
// (Granlund-Montgomery).  On the GPU a uniform x / d compiles to ~30 vector instructions even
// when both operands sit in scalar registers; this form is three scalar ones.
struct FastDiv {
  uint32_t mul, shift;
};
inline FastDiv make_fast_div(uint32_t d) {
  uint32_t l = 0;
  while ((1u << l) < d) ++l;
  FastDiv f;
  f.shift = 27 + l;
  f.mul = (uint32_t)((((uint64_t)1 << f.shift) + d - 1) / d);
  return f;
}
__host__ __device__ inline uint32_t fast_div(uint32_t x, FastDiv f) {
  return (uint32_t)(((uint64_t)x * f.mul) >> f.shift);
}

// ---------------------------------------------------------------- verification attention
struct AttnKernelArgs {
  // -- first 192 bytes: everything the kernels need before their first loads, so that the start
  //    of a kernel fetches its arguments as one batch of wide scalar loads
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* kv_len;
  int64_t q_sb, q_sg, q_sh;
  int64_t kv_sb, kv_sh, kv_sl;
  int gamma, Hq, Hkv;
  int G;         // Hq / Hkv
  int R;         // query rows per kv head = G * gamma, ordered r = i * G + (h % G)
  int rpad;      // rows per row chunk: 16, 32, 48 or 64
  int xcd_map;   // 1: units (B * n_rc * Hkv) are a multiple of 8 and mapped one XCD each
  int n_rc;      // row chunks = ceil(R / rpad)
  int n_split;   // key-range splits
  int len_mode;  // where kv_len[b] comes from: 0 device read, 1 len_hot[b] (B <= 5), 2 len_host[b]
  float* ws;     // partials [B*Hkv][n_rc][n_split][rpad * 131]
  FastDiv div_split, div_rpad, div_hkv, div_rc, div_g;   // by n_split, rpad, Hkv, n_rc, G
  int len_hot[5];            // host-known lengths inside the lines the prologue fetches anyway
  int lmax;                  // cap - gamma: a length read from device memory is clamped to [0, lmax]
  int len_host[32];          // host-known lengths of up to 32 sequences (a further line)
  // -- used later
  float scale_log2e;
  int B;
  int variant;   // kernel variant, 0 = default for rpad (development knob; host side only)
  const int32_t* vis_begin;   // nullptr = no span
  const int32_t* vis_end;
  uint16_t* out;
  int64_t o_sb, o_sg, o_sh;
  float* lse;
  float* vis_mass;
  uint32_t draft_mask[32];
};
static_assert(offsetof(AttnKernelArgs, len_host) == 192, "prologue arguments fill three 64-byte lines");

hipError_t launch_attn(const AttnKernelArgs& a, hipStream_t stream);

// ---------------------------------------------------------------- streamed skinny GEMM
// C[r][c] = sum_t A[r][t] * X[c][t]: A is a tall bf16 matrix streamed once from HBM (video
// hidden states or lm_head), X a handful of bf16 rows (draft hidden states).
struct GemmKernelArgs {
  const uint8_t* a;          // A base
  int64_t a_sb;              // bytes between batches of A (relevance) / 0
  int64_t a_sr;              // bytes between rows of A
  const int32_t* n_rows_dev; // [B] valid rows per batch (relevance) or nullptr
  int n_rows;                // rows (lm_head) / allocated rows per batch (relevance)
  const uint8_t* x;          // X base; column (xb, xi) at x + xb * x_sb + xi * x_sg
  int64_t x_sb, x_sg;        // bytes
  int row_bytes;             // bytes of a row one pipeline stage covers: 256 or 512
  int gamma;                 // columns per batch
  int n_cols;                // relevance: gamma; lm_head: B * gamma
  int B;                     // batches of A (relevance) / 1
  int rows_per_block;        // rows of A per workgroup task (64 or 128)
  int n_rb;                  // row blocks per batch
  int n_ds;                  // splits of the contraction dimension
  int kc;                    // 128-element chunks per split
  int n_tasks;               // B * n_rb * n_ds
  // relevance outputs
  float* dots;               // [B][n_ds][gamma][ld]
  float* nv2;                // [B][n_ds][ld]
  int64_t ld;
  // lm_head outputs
  float* stats;
  float* stats_z;            // optional [n_tasks][n_cols]: sum exp(z - max) * z per block (entropy)              // [n_tasks][n_cols][2]  (max, sum exp(z - max))
  float* cand_val;           // [n_tasks][n_cols][topk]
  int32_t* cand_idx;         // [n_tasks][n_cols][topk]
  int topk;
  float* logits;             // optional [n_cols][n_rows]
};

hipError_t launch_rel_gemm(const GemmKernelArgs& a, int num_cu, hipStream_t stream);
hipError_t launch_lmh_gemm(const GemmKernelArgs& a, int num_cu, hipStream_t stream);
int rel_rows_per_block(int big);   // 64, or 128 rows when there are plenty of row blocks
// vocabulary rows per task: 64 or 128
int lmh_rows_per_block(int n_cols, int64_t row_pitch_bytes, int64_t n_rows, int topk);
// candidates per column (row blocks x top-k) that accept_finalize_kernel keeps in registers
constexpr int kAcceptRegCandidates = 20 * 1024;

// ---------------------------------------------------------------- relevance finalize
struct RelFinalizeArgs {
  const uint16_t* h_d;
  int64_t hd_sb, hd_sg;      // elements
  int d, gamma, B, top_n, n_ds;
  const int32_t* l_v;
  int64_t lv_max;
  const float* dots;
  const float* nv2;
  const float* inv_norm;     // optional [B][lv_max]: prepared 1 / max(|h_v row|, 1e-8); then nv2 is unused
  int64_t ld;
  float* cosbuf;             // [B][gamma][ld]
  uint32_t* cand_keys;       // [B][gamma][n_parts][16]: per-slice candidates (two-kernel path)
  int n_parts;               // slices of slice_rows video rows; 0 = single-kernel path only
  int slice_rows;            // a multiple of kRelSliceRows
  float* relevance;          // [B][gamma]
};
constexpr int kRelSliceRows = 1024;   // video rows the candidate kernel takes at a time (four per thread)
constexpr int kRelMaxParts = 64;      // slices the merge kernel can take
constexpr int kRelMaxChunks = 16;     // 1024-row chunks per slice at most (lv_max <= 1048576)
constexpr int kRelSmallN = 16;        // Top-N sizes served by the two-kernel path
hipError_t launch_rel_finalize(const RelFinalizeArgs& a, hipStream_t stream);

// ---------------------------------------------------------------- prefill-side H_V preparation
struct HvPrepareArgs {
  const uint8_t* h_v;
  int64_t sb, sl;            // bytes between sequences / rows
  int64_t n_rows;            // rows per sequence
  int B, d;
  float* inv_norm;           // [B][n_rows]
};
hipError_t launch_hv_prepare(const HvPrepareArgs& a, hipStream_t stream);

// ---------------------------------------------------------------- accept finalize
struct AcceptFinalizeArgs {
  int B, gamma, V, topk, n_tasks, n_cols;
  int rows;                  // hidden rows per chain: gamma, or gamma + 1 with a bonus row
  FastDiv div_topk;
  const float* stats;
  const float* stats_z;      // optional, see GemmKernelArgs
  float* entropy;            // optional [B*rows]
  const float* cand_val;
  const int32_t* cand_idx;
  const int32_t* draft_ids;
  const float* relevance;
  int n_loose, pst_window, gate;
  int rule;                  // 0 the paper's rule; 1 entropy gate; 2 entropy gate + deferred window
  float ent_threshold;
  int defer_window;
  const float* ent_rows;     // [B*rows] entropies the entropy rules read (entropy, or scratch)
  int n_branches;            // chains per sequence (>= 1)
  int32_t* best_branch;      // optional, [B / n_branches]
  int32_t* target_ids;
  int32_t* topk_ids;         // optional
  float* topk_probs;         // optional
  int32_t* ws_topk_ids;      // [B*rows][16]
  uint8_t* verdict;
  int32_t* accept_len;
  int32_t* bonus_id;
};
hipError_t launch_accept_finalize(const AcceptFinalizeArgs& a, hipStream_t stream);

// ---------------------------------------------------------------- KV commit
struct CommitKernelArgs {
  uint8_t* k;
  uint8_t* v;
  int64_t slayer, sb, sh, sl;   // bytes
  int B, Hkv, n_layers, n_branches, chain_len;
  int chunks;                   // 16-byte chunks per row (D / 8)
  int64_t cap;                  // rows allocated per (sequence, head)
  const int32_t* kv_len;
  const int32_t* accept_len;
  const int32_t* best_branch;   // optional
  int32_t* new_len;
};
hipError_t launch_kv_commit(const CommitKernelArgs& a, hipStream_t stream);

}  // namespace lvspec
