// C ABI of the library: argument validation, launch planning (all on the host, no device access)
// and kernel launches on the caller's stream.
#include <hip/hip_runtime.h>

#include <atomic>

#include "../../include/lvspec.h"
#include "lvspec_kernels.h"

// Scratch of lvspec_verify_attn_static: part of the code object, one copy per GPU.  In host code
// the array's name is only a handle for the symbol lookup, never a device address: everything
// below works with the pointer that hipGetSymbolAddress returned for the current device.
static __device__ __align__(256) unsigned char scratch[LVSPEC_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  return LVSPEC_EHIP;
}

// compute units of the current device; 256 (MI355X) when no device can be queried.  Cached per
// device; the query is idempotent, so racing first calls store the same value.
int num_compute_units() {
  static std::atomic<int> cached[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return 256;
  }
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked) {
    const int c = cached[dev].load(std::memory_order_relaxed);
    if (c > 0) return c;
  }
  int n = 0;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) {
    if (tracked) cached[dev].store(n, std::memory_order_relaxed);
    return n;
  }
  (void)hipGetLastError();
  return 256;
}

size_t round_up(size_t x, size_t m) { return (x + m - 1) / m * m; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool stride_ok(int64_t s) { return s >= 0 && (s % 8) == 0; }

// ------------------------------------------------------------------------------ attention
struct AttnPlan {
  int G, R, rpad, n_rc, n_split;
  size_t ws_bytes;
};

int plan_attn(const lvspec_attn_args* a, AttnPlan* pl) {
  if (a == nullptr) return LVSPEC_EINVAL;
  if (a->B < 1 || a->gamma < 1 || a->gamma > LVSPEC_MAX_DRAFT_ROWS || a->Hq < 1 || a->Hkv < 1 ||
      a->D < 1)
    return LVSPEC_EINVAL;
  if (a->Hq % a->Hkv != 0) return LVSPEC_EINVAL;
  if (a->D != LVSPEC_HEAD_DIM) return LVSPEC_EUNSUPPORTED;
  if (a->cap < a->gamma || a->max_kv_len < 0 || a->max_kv_len + a->gamma > a->cap)
    return LVSPEC_EINVAL;
  if (a->cap > (int64_t)1 << 30) return LVSPEC_EUNSUPPORTED;
  if (!(a->scale >= 0.f) || a->scale > 1.0e6f) return LVSPEC_EINVAL;
  const int64_t lmax = a->max_kv_len > 0 ? a->max_kv_len : a->cap - a->gamma;
  pl->G = a->Hq / a->Hkv;
  pl->R = pl->G * a->gamma;
  pl->n_rc = (pl->R + 63) / 64;
  const int per_chunk = (pl->R + pl->n_rc - 1) / pl->n_rc;
  pl->rpad = per_chunk <= 16 ? 16 : per_chunk <= 32 ? 32 : per_chunk <= 48 ? 48 : 64;
  const int64_t units = (int64_t)a->B * a->Hkv * pl->n_rc;
  // block ids and row indices stay below 2^27, the range of the kernels' multiply-shift division
  if (units * 64 > (int64_t)1 << 27 || a->Hq > 65536) return LVSPEC_EUNSUPPORTED;
  const int64_t n_tiles = (lmax + a->gamma + 31) / 32;
  int64_t ns = num_compute_units() / units;
  const int64_t cap_split = (n_tiles + 3) / 4;
  if (ns > cap_split) ns = cap_split;
  if (ns > 256) ns = 256;
  if (ns < 1) ns = 1;
  pl->n_split = (int)ns;
  pl->ws_bytes = (size_t)units * (size_t)ns * (size_t)pl->rpad * 131 * sizeof(float);
  return LVSPEC_OK;
}

int check_attn_pointers(const lvspec_attn_args* a) {
  if (!a->q || !a->k || !a->v || !a->out) return LVSPEC_EINVAL;
  if (!a->kv_len && !(a->kv_len_host && a->B <= 32)) return LVSPEC_EINVAL;
  if (a->kv_len_host != nullptr) {
    const int64_t lmax = a->max_kv_len > 0 ? a->max_kv_len : a->cap - a->gamma;
    for (int b = 0; b < a->B; ++b)
      if (a->kv_len_host[b] < 0 || a->kv_len_host[b] > lmax) return LVSPEC_EINVAL;
  }
  if (!aligned16(a->q) || !aligned16(a->k) || !aligned16(a->v) || !aligned16(a->out))
    return LVSPEC_EINVAL;
  if (!stride_ok(a->q_sb) || !stride_ok(a->q_sg) || !stride_ok(a->q_sh) || !stride_ok(a->kv_sb) ||
      !stride_ok(a->kv_sh) || !stride_ok(a->kv_sl) || !stride_ok(a->o_sb) || !stride_ok(a->o_sg) ||
      !stride_ok(a->o_sh))
    return LVSPEC_EINVAL;
  if (a->kv_sl < a->D || a->q_sh < a->D || a->o_sh < a->D) return LVSPEC_EINVAL;
  if ((a->vis_begin == nullptr) != (a->vis_end == nullptr)) return LVSPEC_EINVAL;
  if (a->vis_mass != nullptr && a->vis_begin == nullptr) return LVSPEC_EINVAL;
  if (a->draft_mask != nullptr) {
    for (int i = 0; i < a->gamma; ++i) {
      if (!((a->draft_mask[i] >> i) & 1u)) return LVSPEC_EINVAL;   // a row always sees itself
      if (a->gamma < 32 && (a->draft_mask[i] >> a->gamma) != 0u) return LVSPEC_EINVAL;
    }
  }
  return LVSPEC_OK;
}

// ------------------------------------------------------------------------------ relevance
struct RelPlan {
  int rows, n_rb, n_ds, kc, row_bytes;
  int64_t ld;
  size_t off_nv2, off_cos, off_keys, ws_bytes;
  int n_parts, slice_rows;
};

int plan_rel(const lvspec_rel_args* a, RelPlan* pl) {
  if (a == nullptr) return LVSPEC_EINVAL;
  if (a->B < 1 || a->gamma < 1 || a->gamma > LVSPEC_MAX_DRAFT_ROWS || a->d < 1 ||
      a->top_n < 1 || a->top_n > LVSPEC_MAX_TOPN || a->lv_max < 0)
    return LVSPEC_EINVAL;
  if (a->d % 128 != 0) return LVSPEC_EUNSUPPORTED;
  if (a->lv_max > (int64_t)1 << 30) return LVSPEC_EUNSUPPORTED;
  // Stages of 64 rows x 512 bytes when the shape allows (up to 16 draft rows, d a multiple of
  // 256): longer contiguous row segments stream measurably faster from HBM than 256-byte ones.
  // Otherwise 256-byte stages: 128-row tasks (bigger stages, fewer barriers per byte) once they
  // fill the persistent workgroups without splitting the hidden dimension, 64-row tasks else.
  const int64_t wg_slots = 2 * (int64_t)num_compute_units();
  pl->row_bytes = (a->gamma <= 16 && a->d % 256 == 0) ? 512 : 256;
  const int big = (pl->row_bytes == 256 &&
                   (int64_t)a->B * ((a->lv_max + 127) / 128) >= wg_slots) ? 1 : 0;
  const int rows = lvspec::rel_rows_per_block(big);
  pl->rows = rows;
  pl->n_rb = (int)((a->lv_max + rows - 1) / rows);
  if (pl->n_rb < 1) pl->n_rb = 1;
  // task indices (row blocks x up to 8 splits x sequences) stay in 32-bit range, and the
  // sequence index is a grid dimension of the finalize kernels
  if (a->B > 65535 || (int64_t)a->B * pl->n_rb * 8 > (int64_t)1 << 30) return LVSPEC_EUNSUPPORTED;
  const int nchunks = a->d * 2 / pl->row_bytes;
  // Split the hidden dimension when the row blocks alone leave most of the persistent
  // workgroups (two per CU) without a task.  A split is not free: shorter tasks, partial results
  // per split and their sum in the finalize kernels cost about 9 % of the streaming rate per
  // doubling (measured at equal fill: 6.2 TB/s unsplit against 5.7 and 5.5 TB/s in two and four
  // splits on 4 GB of hidden states), so the fill of the last round is weighed against that;
  // among near-equal scores the fewest splits win.  At most 8 splits, at least 2 chunks each.
  const int64_t slots = 2 * (int64_t)num_compute_units();
  int best = 1;
  double best_score = 0.0;
  for (int ds = 1; ds <= nchunks && ds <= 8; ++ds) {
    if (nchunks % ds != 0) continue;
    if (nchunks / ds < 2 && ds != 1) break;
    const int64_t tasks = (int64_t)a->B * pl->n_rb * ds;
    const int64_t rounds = (tasks + slots - 1) / slots;
    const double fill = (double)tasks / (double)(rounds * slots);
    const double score = fill / (1.0 + 0.1 * __builtin_log2((double)ds));
    if (score > best_score + 0.03) {
      best = ds;
      best_score = score;
    }
  }
  pl->n_ds = best;
  pl->kc = nchunks / best;
  pl->ld = (int64_t)round_up((size_t)(a->lv_max > 0 ? a->lv_max : 1), 128);
  const size_t f = sizeof(float);
  const size_t dots = round_up((size_t)a->B * pl->n_ds * a->gamma * pl->ld * f, 256);
  const size_t nv2 = round_up((size_t)a->B * pl->n_ds * pl->ld * f, 256);
  const size_t cosb = round_up((size_t)a->B * a->gamma * pl->ld * f, 256);
  // slices of the two-kernel Top-N (small N): at most kRelMaxParts slices of as few 1024-row
  // chunks as that allows; n_parts = 0: not used (large N, or more than a million video rows)
  const int64_t per_slice = (int64_t)lvspec::kRelSliceRows * lvspec::kRelMaxParts;
  int64_t chunks = (a->lv_max + per_slice - 1) / per_slice;
  if (chunks < 1) chunks = 1;
  pl->slice_rows = (int)(chunks * lvspec::kRelSliceRows);
  const int64_t parts = (a->lv_max + pl->slice_rows - 1) / pl->slice_rows;
  pl->n_parts = (a->top_n <= lvspec::kRelSmallN && parts >= 1 && parts <= lvspec::kRelMaxParts &&
                 chunks <= lvspec::kRelMaxChunks)
                    ? (int)parts : 0;
  const size_t keys = round_up((size_t)a->B * a->gamma * (size_t)pl->n_parts *
                               lvspec::kRelSmallN * sizeof(uint32_t), 256);
  pl->off_nv2 = dots;
  pl->off_cos = dots + nv2;
  pl->off_keys = dots + nv2 + cosb;
  pl->ws_bytes = dots + nv2 + cosb + keys;
  return LVSPEC_OK;
}

// ------------------------------------------------------------------------------ accept
struct AccPlan {
  int n_tasks, n_cols;     // n_cols: columns of one (full) pass
  int rows_per_block;      // vocabulary rows per task
  int group;               // chains per pass (a multiple of the branches per sequence)
  size_t off_cval, off_cidx, off_cnt, off_topk, off_sz, off_ent, ws_bytes;
};

int plan_acc(const lvspec_accept_args* a, AccPlan* pl) {
  if (a == nullptr) return LVSPEC_EINVAL;
  if (a->B < 1 || a->gamma < 1 || a->gamma > LVSPEC_MAX_GAMMA || a->d < 1 || a->V < 1 ||
      a->topk < 1 || a->topk > LVSPEC_MAX_TOPK)
    return LVSPEC_EINVAL;
  if (a->n_loose < 0 || a->n_loose > a->gamma || a->pst_window < 0 || a->loose_topk_gate < 0 ||
      a->loose_topk_gate > a->topk)
    return LVSPEC_EINVAL;
  if (a->n_branches < 0 || a->n_branches > LVSPEC_MAX_BRANCHES ||
      (a->n_branches > 1 && a->B % a->n_branches != 0))
    return LVSPEC_EINVAL;
  if (a->bonus_row != 0 && a->bonus_row != 1) return LVSPEC_EINVAL;
  if (a->rule < LVSPEC_RULE_VISUAL || a->rule > LVSPEC_RULE_ENTROPY_WINDOW) return LVSPEC_EINVAL;
  if (a->rule != LVSPEC_RULE_VISUAL &&
      (!(a->entropy_threshold >= 0.f) || a->defer_window < 0 || a->defer_window > LVSPEC_MAX_GAMMA))
    return LVSPEC_EINVAL;
  if (a->d % 128 != 0) return LVSPEC_EUNSUPPORTED;
  // one pass of the lm_head stream serves at most kMaxCols hidden rows; more chains take
  // several passes (whole sequences per pass: the branches of a tree stay together)
  constexpr int kMaxCols = 64;
  const int nbr = a->n_branches > 1 ? a->n_branches : 1;
  const int rpc = a->gamma + a->bonus_row;   // hidden rows per chain
  if (nbr * rpc > kMaxCols || a->B > 4096) return LVSPEC_EUNSUPPORTED;
  // Fewest passes first; among equal pass counts the smallest group whose columns fit the
  // narrower (faster) kernel variants.
  const int gmax = (kMaxCols / rpc) / nbr * nbr;
  const int passes = (a->B + gmax - 1) / gmax;
  pl->group = ((a->B + passes - 1) / passes + nbr - 1) / nbr * nbr;
  if (pl->group > a->B) pl->group = a->B;
  pl->n_cols = pl->group * rpc;
  const int rows = lvspec::lmh_rows_per_block(pl->n_cols, (a->w_sv > 0 ? a->w_sv : a->d) * 2, a->V,
                                                a->topk);
  pl->rows_per_block = rows;
  pl->n_tasks = (a->V + rows - 1) / rows;
  const size_t rec = (size_t)pl->n_tasks * pl->n_cols;
  const size_t stats = round_up(rec * 2 * sizeof(float), 256);
  const size_t cval = round_up(rec * a->topk * sizeof(float), 256);
  const size_t cidx = round_up(rec * a->topk * sizeof(int32_t), 256);
  const size_t cnt = round_up((size_t)a->B * sizeof(int32_t), 256);
  const size_t topk = round_up((size_t)pl->n_cols * 16 * sizeof(int32_t), 256);
  pl->off_cval = stats;
  pl->off_cidx = stats + cval;
  pl->off_cnt = stats + cval + cidx;
  pl->off_topk = stats + cval + cidx + cnt;
  pl->off_sz = stats + cval + cidx + cnt + topk;
  pl->off_ent = pl->off_sz + round_up(rec * sizeof(float), 256);
  // row entropies of one pass, for the entropy rules when the caller asks for no entropy output
  pl->ws_bytes = pl->off_ent + round_up((size_t)pl->n_cols * sizeof(float), 256);
  return LVSPEC_OK;
}

int enqueue_attn(const lvspec_attn_args* a, const AttnPlan& pl, void* workspace, void* stream);

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  static std::atomic<void*> cached[64] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  const bool tracked = dev >= 0 && dev < 64;
  void* ptr = tracked ? cached[dev].load(std::memory_order_acquire) : nullptr;
  if (ptr == nullptr) {
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (ptr == nullptr) return hip_fail(hipErrorInvalidSymbol);
    if (tracked) cached[dev].store(ptr, std::memory_order_release);   // same value from any thread
  }
  *out = ptr;
  return LVSPEC_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
  if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || have < need)
    return LVSPEC_EWORKSPACE;
  return LVSPEC_OK;
}

}  // namespace

extern "C" {

const char* lvspec_status_string(int status) {
  switch (status) {
    case LVSPEC_OK: return "ok";
    case LVSPEC_EINVAL: return "invalid argument";
    case LVSPEC_EUNSUPPORTED: return "unsupported shape";
    case LVSPEC_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LVSPEC_EHIP: return "HIP error";
    case LVSPEC_ESCRATCH: return "static scratch too small for these shapes";
    default: return "unknown status";
  }
}

int lvspec_version(void) { return LVSPEC_VERSION; }
int lvspec_last_hip_error(void) { return g_last_hip_error; }

int lvspec_n_loose(float lambda, int gamma) {
  if (gamma < 0) return 0;
  int n = (int)__builtin_floor((double)lambda * (double)gamma + 1e-6);
  if (n < 0) n = 0;
  if (n > gamma) n = gamma;
  return n;
}

size_t lvspec_verify_attn_workspace(const lvspec_attn_args* args) {
  AttnPlan pl;
  return plan_attn(args, &pl) == LVSPEC_OK ? pl.ws_bytes : 0;
}

int lvspec_verify_attn(const lvspec_attn_args* a, void* stream) {
  AttnPlan pl;
  int rc = plan_attn(a, &pl);
  if (rc != LVSPEC_OK) return rc;
  rc = check_attn_pointers(a);
  if (rc != LVSPEC_OK) return rc;
  rc = check_ws(a->workspace, a->workspace_bytes, pl.ws_bytes);
  if (rc != LVSPEC_OK) return rc;
  return enqueue_attn(a, pl, a->workspace, stream);
}

int lvspec_verify_attn_static(const lvspec_attn_args* a, void* stream) {
  AttnPlan pl;
  int rc = plan_attn(a, &pl);
  if (rc != LVSPEC_OK) return rc;
  rc = check_attn_pointers(a);
  if (rc != LVSPEC_OK) return rc;
  if (pl.ws_bytes > (size_t)LVSPEC_STATIC_SCRATCH_BYTES) return LVSPEC_ESCRATCH;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != LVSPEC_OK) return rc;
  return enqueue_attn(a, pl, ws, stream);
}

}  // extern "C"

namespace {

int enqueue_attn(const lvspec_attn_args* a, const AttnPlan& pl, void* workspace, void* stream) {
  lvspec::AttnKernelArgs k{};
  k.q = static_cast<const uint16_t*>(a->q);
  k.q_sb = a->q_sb; k.q_sg = a->q_sg; k.q_sh = a->q_sh;
  k.k = static_cast<const uint16_t*>(a->k);
  k.v = static_cast<const uint16_t*>(a->v);
  k.kv_sb = a->kv_sb; k.kv_sh = a->kv_sh; k.kv_sl = a->kv_sl;
  k.kv_len = a->kv_len;
  // lengths known to the host travel in the launch arguments: up to 6 in the lines the kernel's
  // prologue fetches anyway; a longer table only when there is no device array to read
  k.len_mode = (a->kv_len_host != nullptr && a->B <= 5) ? 1
               : (a->kv_len == nullptr && a->kv_len_host != nullptr && a->B <= 32) ? 2 : 0;
  for (int b = 0; b < 5; ++b)
    k.len_hot[b] = (k.len_mode == 1 && b < a->B) ? a->kv_len_host[b] : 0;
  for (int b = 0; b < 32; ++b)
    k.len_host[b] = (k.len_mode == 2 && b < a->B) ? a->kv_len_host[b] : 0;
  k.lmax = (int)(a->cap - a->gamma);
  k.vis_begin = a->vis_begin;
  k.vis_end = a->vis_end;
  k.B = a->B; k.gamma = a->gamma; k.Hq = a->Hq; k.Hkv = a->Hkv;
  k.G = pl.G; k.R = pl.R; k.rpad = pl.rpad; k.n_rc = pl.n_rc; k.n_split = pl.n_split;
  k.div_split = lvspec::make_fast_div((uint32_t)pl.n_split);
  k.div_rpad = lvspec::make_fast_div((uint32_t)pl.rpad);
  k.div_hkv = lvspec::make_fast_div((uint32_t)a->Hkv);
  k.div_rc = lvspec::make_fast_div((uint32_t)pl.n_rc);
  k.div_g = lvspec::make_fast_div((uint32_t)pl.G);
  const float scale = a->scale > 0.f ? a->scale : 1.0f / __builtin_sqrtf((float)a->D);
  k.xcd_map = ((int64_t)a->B * pl.n_rc * a->Hkv) % 8 == 0 ? 1 : 0;
  k.scale_log2e = scale * 1.4426950408889634f;
  k.ws = static_cast<float*>(workspace);
  for (int i = 0; i < 32; ++i)
    k.draft_mask[i] = a->draft_mask ? (i < a->gamma ? a->draft_mask[i] : 0u)
                                    : (0xffffffffu >> (31 - i));
  k.out = static_cast<uint16_t*>(a->out);
  k.o_sb = a->o_sb; k.o_sg = a->o_sg; k.o_sh = a->o_sh;
  k.lse = a->lse;
  k.vis_mass = a->vis_mass;
  hipError_t e = lvspec::launch_attn(k, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LVSPEC_OK : hip_fail(e);
}

}  // namespace

extern "C" {

size_t lvspec_visual_relevance_workspace(const lvspec_rel_args* args) {
  RelPlan pl;
  return plan_rel(args, &pl) == LVSPEC_OK ? pl.ws_bytes : 0;
}

int lvspec_visual_relevance(const lvspec_rel_args* a, void* stream) {
  RelPlan pl;
  int rc = plan_rel(a, &pl);
  if (rc != LVSPEC_OK) return rc;
  if (!a->h_d || !a->l_v || !a->relevance || (a->lv_max > 0 && !a->h_v)) return LVSPEC_EINVAL;
  if (!aligned16(a->h_d) || !aligned16(a->h_v)) return LVSPEC_EINVAL;
  if (!stride_ok(a->hd_sb) || !stride_ok(a->hd_sg) || !stride_ok(a->hv_sb) ||
      !stride_ok(a->hv_sl) || a->hd_sg < a->d || a->hv_sl < a->d)
    return LVSPEC_EINVAL;
  rc = check_ws(a->workspace, a->workspace_bytes, pl.ws_bytes);
  if (rc != LVSPEC_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* ws = static_cast<uint8_t*>(a->workspace);
  float* dots = reinterpret_cast<float*>(ws);
  float* nv2 = reinterpret_cast<float*>(ws + pl.off_nv2);
  float* cosb = reinterpret_cast<float*>(ws + pl.off_cos);
  if (a->lv_max > 0) {
    lvspec::GemmKernelArgs g{};
    g.a = static_cast<const uint8_t*>(a->h_v);
    g.a_sb = a->hv_sb * 2;
    g.a_sr = a->hv_sl * 2;
    g.n_rows_dev = a->l_v;
    g.n_rows = (int)a->lv_max;
    g.x = static_cast<const uint8_t*>(a->h_d);
    g.x_sb = a->hd_sb * 2;
    g.x_sg = a->hd_sg * 2;
    g.gamma = a->gamma;
    g.n_cols = a->gamma;
    g.B = a->B;
    g.rows_per_block = pl.rows;
    g.row_bytes = pl.row_bytes;
    g.n_rb = pl.n_rb;
    g.n_ds = pl.n_ds;
    g.kc = pl.kc;
    g.n_tasks = a->B * pl.n_rb * pl.n_ds;
    g.dots = dots;
    g.nv2 = a->hv_inv_norm ? nullptr : nv2;   // prepared norms: dot products only
    g.ld = pl.ld;
    hipError_t e = lvspec::launch_rel_gemm(g, num_compute_units(), st);
    if (e != hipSuccess) return hip_fail(e);
  }
  lvspec::RelFinalizeArgs f{};
  f.h_d = static_cast<const uint16_t*>(a->h_d);
  f.hd_sb = a->hd_sb; f.hd_sg = a->hd_sg;
  f.d = a->d; f.gamma = a->gamma; f.B = a->B; f.top_n = a->top_n; f.n_ds = pl.n_ds;
  f.l_v = a->l_v;
  f.lv_max = a->lv_max;
  f.dots = dots; f.nv2 = nv2; f.ld = pl.ld; f.cosbuf = cosb;
  f.inv_norm = a->hv_inv_norm;
  f.cand_keys = reinterpret_cast<uint32_t*>(ws + pl.off_keys);
  f.n_parts = pl.n_parts;
  f.slice_rows = pl.slice_rows;
  f.relevance = a->relevance;
  hipError_t e = lvspec::launch_rel_finalize(f, st);
  return e == hipSuccess ? LVSPEC_OK : hip_fail(e);
}

int lvspec_hv_prepare(const lvspec_hv_args* a, void* stream) {
  if (a == nullptr) return LVSPEC_EINVAL;
  if (a->B < 1 || a->B > 65535 || a->d < 1 || a->lv_max < 0) return LVSPEC_EINVAL;
  if (a->d % 128 != 0 || a->lv_max > (int64_t)1 << 30) return LVSPEC_EUNSUPPORTED;
  if (!a->hv_inv_norm || (a->lv_max > 0 && !a->h_v)) return LVSPEC_EINVAL;
  if (!aligned16(a->h_v) || !stride_ok(a->hv_sb) || !stride_ok(a->hv_sl) || a->hv_sl < a->d)
    return LVSPEC_EINVAL;
  if (a->lv_max == 0) return LVSPEC_OK;
  lvspec::HvPrepareArgs k{};
  k.h_v = static_cast<const uint8_t*>(a->h_v);
  k.sb = a->hv_sb * 2; k.sl = a->hv_sl * 2;
  k.n_rows = a->lv_max; k.B = a->B; k.d = a->d;
  k.inv_norm = a->hv_inv_norm;
  hipError_t e = lvspec::launch_hv_prepare(k, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LVSPEC_OK : hip_fail(e);
}

size_t lvspec_loose_accept_workspace(const lvspec_accept_args* args) {
  AccPlan pl;
  return plan_acc(args, &pl) == LVSPEC_OK ? pl.ws_bytes : 0;
}

int lvspec_loose_accept(const lvspec_accept_args* a, void* stream) {
  AccPlan pl;
  int rc = plan_acc(a, &pl);
  if (rc != LVSPEC_OK) return rc;
  if (!a->h_d || !a->lm_head || !a->draft_ids || !a->target_ids || !a->verdict ||
      !a->accept_len || !a->bonus_id)
    return LVSPEC_EINVAL;
  if (a->rule == LVSPEC_RULE_VISUAL && !a->relevance) return LVSPEC_EINVAL;
  if (!aligned16(a->h_d) || !aligned16(a->lm_head)) return LVSPEC_EINVAL;
  const int64_t w_sv = a->w_sv > 0 ? a->w_sv : a->d;
  if (!stride_ok(a->hd_sb) || !stride_ok(a->hd_sg) || !stride_ok(w_sv) || a->hd_sg < a->d ||
      w_sv < a->d)
    return LVSPEC_EINVAL;
  rc = check_ws(a->workspace, a->workspace_bytes, pl.ws_bytes);
  if (rc != LVSPEC_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* ws = static_cast<uint8_t*>(a->workspace);
  const int nbr = a->n_branches > 1 ? a->n_branches : 1;
  const int rpc = a->gamma + a->bonus_row;                         // hidden rows per chain
  for (int b0 = 0; b0 < a->B; b0 += pl.group) {
    const int nb = a->B - b0 < pl.group ? a->B - b0 : pl.group;   // chains of this pass
    const int n_cols = nb * rpc;
    const int64_t c0 = (int64_t)b0 * rpc;                          // first hidden row of this pass
    const int64_t t0 = (int64_t)b0 * a->gamma;                     // first draft token of this pass
    lvspec::GemmKernelArgs g{};
    g.a = static_cast<const uint8_t*>(a->lm_head);
    g.a_sb = 0;
    g.a_sr = w_sv * 2;
    g.n_rows_dev = nullptr;
    g.n_rows = a->V;
    g.x = static_cast<const uint8_t*>(a->h_d) + (int64_t)b0 * a->hd_sb * 2;
    g.x_sb = a->hd_sb * 2;
    g.x_sg = a->hd_sg * 2;
    g.gamma = rpc;
    g.n_cols = n_cols;
    g.B = 1;
    g.rows_per_block = pl.rows_per_block;
    g.n_rb = pl.n_tasks;
    g.n_ds = 1;
    g.kc = a->d / 128;
    g.row_bytes = 256;
    g.n_tasks = pl.n_tasks;
    g.stats = reinterpret_cast<float*>(ws);
    g.cand_val = reinterpret_cast<float*>(ws + pl.off_cval);
    g.cand_idx = reinterpret_cast<int32_t*>(ws + pl.off_cidx);
    // the entropy rules read the row entropies: into the caller's array, else into scratch
    float* ent = a->entropy ? a->entropy + c0
                 : a->rule != LVSPEC_RULE_VISUAL ? reinterpret_cast<float*>(ws + pl.off_ent)
                                                 : nullptr;
    g.stats_z = ent ? reinterpret_cast<float*>(ws + pl.off_sz) : nullptr;
    g.topk = a->topk;
    g.logits = a->logits ? a->logits + c0 * a->V : nullptr;
    hipError_t e = lvspec::launch_lmh_gemm(g, num_compute_units(), st);
    if (e != hipSuccess) return hip_fail(e);
    lvspec::AcceptFinalizeArgs f{};
    f.B = nb; f.gamma = a->gamma; f.rows = rpc; f.V = a->V; f.topk = a->topk;
    f.n_tasks = pl.n_tasks; f.n_cols = n_cols;
    f.div_topk = lvspec::make_fast_div((uint32_t)a->topk);
    f.stats = g.stats; f.cand_val = g.cand_val; f.cand_idx = g.cand_idx;
    f.stats_z = g.stats_z;
    f.entropy = ent;
    f.ent_rows = ent;
    f.rule = a->rule; f.ent_threshold = a->entropy_threshold; f.defer_window = a->defer_window;
    f.draft_ids = a->draft_ids + t0;
    f.relevance = a->relevance ? a->relevance + t0 : nullptr;
    f.n_loose = a->n_loose; f.pst_window = a->pst_window; f.gate = a->loose_topk_gate;
    f.n_branches = nbr;
    f.best_branch = a->best_branch ? a->best_branch + b0 / nbr : nullptr;
    f.target_ids = a->target_ids + c0;
    f.topk_ids = a->topk_ids ? a->topk_ids + c0 * a->topk : nullptr;
    f.topk_probs = a->topk_probs ? a->topk_probs + c0 * a->topk : nullptr;
    f.ws_topk_ids = reinterpret_cast<int32_t*>(ws + pl.off_topk);
    f.verdict = a->verdict + t0;
    f.accept_len = a->accept_len + b0;
    f.bonus_id = a->bonus_id + b0;
    e = lvspec::launch_accept_finalize(f, st);
    if (e != hipSuccess) return hip_fail(e);
  }
  return LVSPEC_OK;
}

int lvspec_kv_commit(const lvspec_commit_args* a, void* stream) {
  if (a == nullptr) return LVSPEC_EINVAL;
  const int nbr = a->n_branches > 1 ? a->n_branches : 1;
  if (a->B < 1 || a->B > 65535 || a->Hkv < 1 || a->D < 8 || a->D % 8 != 0 || a->n_layers < 1 ||
      a->n_layers > 65535 || a->n_branches < 0 || a->n_branches > LVSPEC_MAX_BRANCHES ||
      a->chain_len < 1 || a->chain_len > LVSPEC_MAX_GAMMA ||
      nbr * a->chain_len > LVSPEC_MAX_DRAFT_ROWS || a->cap < nbr * a->chain_len)
    return LVSPEC_EINVAL;
  if (!a->k || !a->v || !a->kv_len || !a->accept_len || !a->new_len ||
      a->new_len == a->kv_len)
    return LVSPEC_EINVAL;
  if (!aligned16(a->k) || !aligned16(a->v)) return LVSPEC_EINVAL;
  if (!stride_ok(a->kv_sb) || !stride_ok(a->kv_sh) || !stride_ok(a->kv_sl) || a->kv_sl < a->D ||
      (a->n_layers > 1 && (!stride_ok(a->kv_slayer) || a->kv_slayer < 1)))
    return LVSPEC_EINVAL;
  if ((int64_t)2 * a->Hkv * a->chain_len * (a->D / 8) > ((int64_t)1 << 30))
    return LVSPEC_EUNSUPPORTED;
  lvspec::CommitKernelArgs c{};
  c.k = static_cast<uint8_t*>(a->k);
  c.v = static_cast<uint8_t*>(a->v);
  c.slayer = a->n_layers > 1 ? a->kv_slayer * 2 : 0;
  c.sb = a->kv_sb * 2; c.sh = a->kv_sh * 2; c.sl = a->kv_sl * 2;
  c.B = a->B; c.Hkv = a->Hkv; c.n_layers = a->n_layers;
  c.n_branches = nbr; c.chain_len = a->chain_len;
  c.chunks = a->D / 8;
  c.cap = a->cap;
  c.kv_len = a->kv_len; c.accept_len = a->accept_len;
  c.best_branch = nbr > 1 ? a->best_branch : nullptr;
  c.new_len = a->new_len;
  hipError_t e = lvspec::launch_kv_commit(c, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? LVSPEC_OK : hip_fail(e);
}

int lvspec_describe_plan(const lvspec_attn_args* attn, const lvspec_rel_args* rel,
                         const lvspec_accept_args* accept, lvspec_plan_info* out) {
  if (out == nullptr) return LVSPEC_EINVAL;
  int first = LVSPEC_OK;
  if (attn != nullptr) {
    AttnPlan pl;
    const int rc = plan_attn(attn, &pl);
    if (rc == LVSPEC_OK) {
      out->attn_rows_padded = pl.rpad;
      out->attn_row_chunks = pl.n_rc;
      out->attn_splits = pl.n_split;
    } else if (first == LVSPEC_OK) {
      first = rc;
    }
  }
  if (rel != nullptr) {
    RelPlan pl;
    const int rc = plan_rel(rel, &pl);
    if (rc == LVSPEC_OK) {
      out->rel_splits = pl.n_ds;
      out->rel_stage_bytes = pl.row_bytes;
      out->rel_slices = pl.n_parts;
      out->rel_slice_rows = pl.slice_rows;
    } else if (first == LVSPEC_OK) {
      first = rc;
    }
  }
  if (accept != nullptr) {
    AccPlan pl;
    const int rc = plan_acc(accept, &pl);
    if (rc == LVSPEC_OK) {
      out->acc_rows_per_task = pl.rows_per_block;
      out->acc_chains_per_pass = pl.group;
      out->acc_passes = (accept->B + pl.group - 1) / pl.group;
    } else if (first == LVSPEC_OK) {
      first = rc;
    }
  }
  return first;
}

}  // extern "C"
