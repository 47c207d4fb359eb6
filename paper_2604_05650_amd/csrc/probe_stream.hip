// Measurement aid, not part of the library: how fast can a kernel of the split kernel's launch
// shape merely READ a cold buffer of the size of one layer's KV cache with the same copy path
// (16-byte direct-to-LDS copies, non-temporal, per-wave ring in LDS)?  The verify-attention
// kernel cannot be faster than this; the numbers bound what its fixed costs (launch, ramp-up of
// the memory pipeline, drain) leave of the 8 TB/s peak at a given size.
//
// Launches run back to back on one stream over distinct buffers (more than the 256 MB
// last-level cache in total), timed with HIP events around the whole series, as bench.py times
// the attention stack.  Usage: probe_stream [MiB per launch ...]   (default 16 32 64 128 256)
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                   \
  do {                                                                          \
    hipError_t e_ = (x);                                                        \
    if (e_ != hipSuccess) {                                                     \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
      std::exit(1);                                                             \
    }                                                                           \
  } while (0)

namespace {

constexpr int kStep = 8192;   // bytes a wave moves per ring slot: eight 1 KiB copy instructions

__device__ __forceinline__ void copy16(const void* g, uint32_t lds) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)g,
      (__attribute__((address_space(3))) void*)(uintptr_t)__builtin_amdgcn_readfirstlane(lds), 16,
      0, 2 /* non-temporal */);
}

// Every wave streams its contiguous share of the buffer through a private ring of DEPTH slots and
// reads one word of every slot back from LDS, so that no copy can be dropped.  The host checks
// that the share is a whole number of slots.
template <int DEPTH>
__global__ void read_kernel(const uint8_t* __restrict__ p, long bytes_per_wave, uint32_t* sink) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long wid = (long)blockIdx.x * (blockDim.x >> 6) + wave;
  const uint8_t* base = p + wid * bytes_per_wave + lane * 16;
  const uint32_t ring =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem + wave * DEPTH * kStep;
  const int n = (int)(bytes_per_wave / kStep);
  uint32_t acc = 0;
  auto issue = [&](int i) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      copy16(base + (long)i * kStep + j * 1024, ring + (i % DEPTH) * kStep + j * 1024);
  };
  for (int i = 0; i < DEPTH && i < n; ++i) issue(i);
  for (int i = 0; i < n; ++i) {
    if (n - i >= DEPTH)
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"((DEPTH - 1) * 8 > 63 ? 63 : (DEPTH - 1) * 8)
                   : "memory");
    else
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    uint32_t v;
    const uint32_t a = ring + (i % DEPTH) * kStep + lane * 16;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    acc ^= v;
    if (i + DEPTH < n) issue(i + DEPTH);
  }
  if (acc == 0x12345678u) sink[0] = 1;   // never true for the fill pattern; keeps the reads alive
}

template <int DEPTH>
void run(const char* name, int wgs, int threads, const uint8_t* buf, size_t bytes, int nbuf,
         uint32_t* sink) {
  const int waves = wgs * (threads / 64);
  if (bytes % ((size_t)waves * kStep) != 0) {
    std::printf("  %-38s skipped (size not a multiple of %d waves x 8 KiB)\n", name, waves);
    return;
  }
  const long per_wave = (long)(bytes / waves);
  const size_t lds = (size_t)(threads / 64) * DEPTH * kStep;
  CK(hipFuncSetAttribute((const void*)&read_kernel<DEPTH>,
                         hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  for (int r = 0; r < nbuf; ++r)   // warm-up pass over all buffers
    read_kernel<DEPTH><<<wgs, threads, lds>>>(buf + (size_t)r * bytes, per_wave, sink);
  CK(hipDeviceSynchronize());
  const int reps = 3 * nbuf;
  CK(hipEventRecord(e0, 0));
  for (int r = 0; r < reps; ++r)
    read_kernel<DEPTH><<<wgs, threads, lds>>>(buf + (size_t)(r % nbuf) * bytes, per_wave, sink);
  CK(hipEventRecord(e1, 0));
  CK(hipEventSynchronize(e1));
  CK(hipGetLastError());
  float ms = 0.f;
  CK(hipEventElapsedTime(&ms, e0, e1));
  const double us = ms * 1e3 / reps;
  std::printf("  %-38s %4d workgroups x %4d threads: %7.2f us per launch, %6.2f TB/s\n", name, wgs,
              threads, us, (double)bytes / us / 1e6);
  CK(hipEventDestroy(e0));
  CK(hipEventDestroy(e1));
}

}  // namespace

int main(int argc, char** argv) {
  std::vector<int> sizes;
  for (int i = 1; i < argc; ++i) sizes.push_back(std::atoi(argv[i]));
  if (sizes.empty()) sizes = {16, 32, 64, 128, 256};
  uint32_t* sink = nullptr;
  CK(hipMalloc(&sink, 4));
  for (int mib : sizes) {
    if (mib < 16 || mib > 2048 || mib % 16 != 0) {
      std::printf("size %d MiB skipped (multiples of 16 MiB between 16 and 2048)\n", mib);
      continue;
    }
    const size_t bytes = (size_t)mib << 20;
    int nbuf = (int)(((size_t)1536 << 20) / bytes);   // 1.5 GB of distinct buffers
    if (nbuf < 4) nbuf = 4;
    uint8_t* buf = nullptr;
    CK(hipMalloc(&buf, bytes * nbuf));
    CK(hipMemset(buf, 1, bytes * nbuf));
    CK(hipDeviceSynchronize());
    std::printf("%d MiB per launch, %d distinct buffers:\n", mib, nbuf);
    run<2>("8 waves, 2-slot rings (split kernel)", 256, 512, buf, bytes, nbuf, sink);
    run<4>("4 waves, 4-slot rings", 256, 256, buf, bytes, nbuf, sink);
    run<2>("4 waves, 2-slot rings, 2 per CU", 512, 256, buf, bytes, nbuf, sink);
    run<1>("16 waves, 1-slot rings", 256, 1024, buf, bytes, nbuf, sink);
    CK(hipFree(buf));
  }
  CK(hipFree(sink));
  return 0;
}
