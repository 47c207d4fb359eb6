// Prefill-side preparation of the video hidden states for the relevance metric (paper Eq. 7:
// H_V is extracted once at prefill and kept for the whole generation; Eq. 8 divides every dot
// product by the row's norm).  One pass over H_V writes r_j = 1 / max(|h_v[j]|, 1e-8) per row;
// the per-step relevance pass then needs no norm arithmetic at all.
//
// HBM-bound streaming read (2 bytes per element, one fp32 out per row).  One wave per row: lane
// l reads the 16-byte chunks l, l + 64, ... of the row (coalesced, non-temporal: the data is not
// needed again soon), squares and adds in a fixed order, and the 64 partial sums are combined
// over the DPP lane network, so the result does not depend on scheduling.  Four rows per
// workgroup; the grid covers all rows of all sequences.
#include "lvspec_dev.h"
#include "lvspec_kernels.h"

namespace lvspec {

namespace {

constexpr int kPrepWaves = 4;

__global__ __launch_bounds__(64 * kPrepWaves) void hv_prepare_kernel(const HvPrepareArgs p) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t row = (int64_t)blockIdx.x * kPrepWaves + wave;
  const int b = blockIdx.y;
  if (row >= p.n_rows) return;
  const uint8_t* src = p.h_v + (int64_t)b * p.sb + row * p.sl;
  const int chunks = p.d / 8;   // 16-byte chunks of the row (d is a multiple of 8)
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  int c = lane;
  // four independent loads in flight per lane, then the tail
  for (; c + 192 < chunks; c += 256) {
    u32x4 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      w[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + c + 64 * u);
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float lo = __builtin_bit_cast(float, w[u][e] << 16);
        const float hi = __builtin_bit_cast(float, w[u][e] & 0xffff0000u);
        acc[u] = __builtin_fmaf(lo, lo, acc[u]);
        acc[u] = __builtin_fmaf(hi, hi, acc[u]);
      }
  }
  for (; c < chunks; c += 64) {
    const u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src) + c);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float lo = __builtin_bit_cast(float, w[e] << 16);
      const float hi = __builtin_bit_cast(float, w[e] & 0xffff0000u);
      acc[0] = __builtin_fmaf(lo, lo, acc[0]);
      acc[0] = __builtin_fmaf(hi, hi, acc[0]);
    }
  }
  const float n2 = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
  if (lane == 0) p.inv_norm[(int64_t)b * p.n_rows + row] = 1.0f / fmaxf(sqrtf(n2), 1e-8f);
}

}  // namespace

hipError_t launch_hv_prepare(const HvPrepareArgs& a, hipStream_t stream) {
  const dim3 grid((unsigned)((a.n_rows + kPrepWaves - 1) / kPrepWaves), (unsigned)a.B);
  hipLaunchKernelGGL(hv_prepare_kernel, grid, dim3(64 * kPrepWaves), 0, stream, a);
  return hipGetLastError();
}

}  // namespace lvspec
