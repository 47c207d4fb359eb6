// KV-cache commit after a verified step: the accepted prefix of the kept chain moves to the
// front of the draft area (only when a chain other than the first one of a draft tree is kept),
// and the sequence lengths advance by the accepted length (Eq. 2).  Pure data movement: 16-byte
// chunks, one thread each.
#include "lvspec_dev.h"
#include "lvspec_kernels.h"

namespace lvspec {

namespace {

// grid: x = row-chunk items of one (layer, sequence), y = sequence, z = layer.
// item = ((tensor * Hkv + head) * chain_len + i) * chunks + c
__global__ __launch_bounds__(256) void kv_commit_kernel(const CommitKernelArgs p) {
  const int b = blockIdx.y;
  const int layer = blockIdx.z;
  // values from device memory are clamped to the ranges the addressing below relies on
  int kept = (p.best_branch != nullptr && p.n_branches > 1) ? p.best_branch[b] : 0;
  kept = kept < 0 ? 0 : (kept >= p.n_branches ? p.n_branches - 1 : kept);
  int tau = p.accept_len[b * p.n_branches + kept];
  tau = tau < 0 ? 0 : (tau > p.chain_len ? p.chain_len : tau);
  const int len = p.kv_len[b];
  if (layer == 0 && blockIdx.x == 0 && threadIdx.x == 0) p.new_len[b] = len + tau;
  // a length that does not leave room for the draft rows is the caller's error: move nothing
  if (kept == 0 || len < 0 || (int64_t)len + (int64_t)p.n_branches * p.chain_len > p.cap) return;
  const int item = blockIdx.x * 256 + threadIdx.x;
  const int c = item % p.chunks;
  int t = item / p.chunks;
  const int i = t % p.chain_len;
  t /= p.chain_len;
  const int head = t % p.Hkv;
  const int tensor = t / p.Hkv;
  if (tensor >= 2 || i >= tau) return;
  uint8_t* base = (tensor == 0 ? p.k : p.v) + (int64_t)layer * p.slayer + (int64_t)b * p.sb +
                  (int64_t)head * p.sh;
  const int64_t src = (int64_t)(len + kept * p.chain_len + i) * p.sl + (int64_t)c * 16;
  const int64_t dst = (int64_t)(len + i) * p.sl + (int64_t)c * 16;
  *reinterpret_cast<u32x4*>(base + dst) = *reinterpret_cast<const u32x4*>(base + src);
}

}  // namespace

hipError_t launch_kv_commit(const CommitKernelArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)2 * a.Hkv * a.chain_len * a.chunks;
  const dim3 grid((unsigned)((items + 255) / 256), (unsigned)a.B, (unsigned)a.n_layers);
  hipLaunchKernelGGL(kv_commit_kernel, grid, dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace lvspec
