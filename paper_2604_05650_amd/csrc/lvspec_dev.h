// Device-side building blocks shared by the gfx950 kernels: vector types, direct-to-LDS loads,
// LDS reads whose completion is waited for by hand, bf16 MFMA wrappers, cross-lane helpers.
//
// Memory pipeline used by every streaming kernel here
// ---------------------------------------------------
// Rows of 128 bf16 (256 bytes) are the unit.  A wave copies rows from HBM straight into LDS with
// global_load_lds_dwordx4 (no VGPR staging): one instruction moves four rows (64 lanes x 16 B),
// sixteen consecutive lanes cover one 256-byte row, so the HBM side is fully coalesced.  Inside
// LDS the sixteen 16-byte chunks of row r are stored at chunk position (c ^ key(r)), key(r) = r & 15
// in the GEMM kernels (the attention kernel, which also reads tiles row-wise, flips one more bit);
// an MFMA operand read, where sixteen lanes hold sixteen different rows at the same logical
// chunk, then touches sixteen different bank groups.  The permutation is applied on the *global* side of the
// copy (each lane fetches the chunk that belongs at its LDS position), which costs nothing.
//
// The compiler cannot see which LDS bytes such a copy writes and would wait for *all*
// outstanding copies before any LDS read.  LDS reads of streamed tiles are therefore written as
// inline assembly together with the exact s_waitcnt they need; copies complete in issue order,
// so "vmcnt(n)" means "everything except the youngest n copy instructions has landed".
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace lvspec {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowBytes = 256;   // 128 bf16
constexpr int kWave = 64;

#define LVS_DEV __device__ __forceinline__

// Optional in-kernel timeline hook for development builds; expands to nothing in the library.
#ifndef LVS_TRACE
#define LVS_TRACE(id)
#define LVS_TRACE_BEGIN
#define LVS_TRACE_END
#endif
#ifndef LVS_TRACE2          // same, for the second kernel of an entry point
#define LVS_TRACE2(id)
#define LVS_TRACE2_BEGIN
#define LVS_TRACE2_END
#endif

// 32-bit LDS byte address of a __shared__ object
LVS_DEV uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// Cache policy of a copy.  Data that is read exactly once (K/V tiles, video hidden states,
// lm_head rows) is fetched with the non-temporal hint: measured on MI355X, a pure streaming read
// sustains about 15 % more HBM bandwidth with it than without.  Small operands that every
// workgroup re-reads keep the default policy so they stay in L2.
constexpr int kCopyDefault = 0;
constexpr int kCopyStream = 2;   // "nt" bit of the gfx94x/gfx950 cache-policy field

// One direct-to-LDS copy instruction: lane l fetches 16 bytes from gptr (per lane) and the wave
// writes 1 KiB to lds_base + l*16.  lds_base must be wave-uniform.
template <int POLICY = kCopyStream>
LVS_DEV void dma16(const void* gptr, uint32_t lds_base) {
  __builtin_amdgcn_global_load_lds(
      (const __attribute__((address_space(1))) void*)gptr,
      (__attribute__((address_space(3))) void*)(uintptr_t)__builtin_amdgcn_readfirstlane(lds_base),
      16, 0, POLICY);
}

// Wait until at most N copy instructions of this wave are outstanding, then read eight 16-byte
// values from LDS: r[j] from a[j & 3] + (j >> 2) * OFF, and wait for them.
template <int N, int OFF>
LVS_DEV void lds_read8_after(u32x4 (&r)[8], const uint32_t (&a)[4]) {
  asm volatile(
      "s_waitcnt vmcnt(%12)\n\t"
      "ds_read_b128 %0, %8\n\t"
      "ds_read_b128 %1, %9\n\t"
      "ds_read_b128 %2, %10\n\t"
      "ds_read_b128 %3, %11\n\t"
      "ds_read_b128 %4, %8 offset:%13\n\t"
      "ds_read_b128 %5, %9 offset:%13\n\t"
      "ds_read_b128 %6, %10 offset:%13\n\t"
      "ds_read_b128 %7, %11 offset:%13\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]),
        "=&v"(r[6]), "=&v"(r[7])
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "n"(N), "n"(OFF)
      : "memory");
}

// Four 16-byte LDS reads from a[0..3], no copy wait.
LVS_DEV void lds_read4(u32x4 (&r)[4], const uint32_t (&a)[4]) {
  asm volatile(
      "ds_read_b128 %0, %4\n\t"
      "ds_read_b128 %1, %5\n\t"
      "ds_read_b128 %2, %6\n\t"
      "ds_read_b128 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
      : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3])
      : "memory");
}

template <int N>
LVS_DEV void wait_copies() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// D[m][n] += sum_k A[m][k] * B[k][n], 16x16 output, 32-deep, bf16 in, fp32 accumulate.
// Operand layout (lane l): A holds row m = l % 16, k = 8*(l/16) .. +7; B holds column n = l % 16,
// same k; D holds column n = l % 16, rows m = 4*(l/16) .. +3.
LVS_DEV f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// pack two fp32 into one dword of two bf16 (round to nearest even), lo = a, hi = b
LVS_DEV uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 t = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, t);
}

LVS_DEV float xor_shuffle(float x, int mask) { return __shfl_xor(x, mask, 64); }

LVS_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Order-preserving map from fp32 to unsigned integers (larger float = larger key) and back.
LVS_DEV uint32_t order_key(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

LVS_DEV float key_value(uint32_t k) {
  const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __builtin_bit_cast(float, u);
}

// A (value, token id) candidate as one 64-bit key, larger = better in (value descending, id
// ascending) order; 0 = no candidate.  Ids are unique within a column, so equal keys are the
// same candidate.
LVS_DEV uint64_t cand_key(float v, int id) {
  return id < 0 ? 0ull : (((uint64_t)order_key(v) << 32) | (uint32_t)(0x7fffffff - id));
}

// Wave-wide reductions through the DPP lane network (no LDS traffic): two quad permutes, two
// row mirrors, then the row broadcasts of the gfx9 family; lane 63 ends up with the result,
// which is handed back through scalar registers (so the result is wave-uniform).  `ident` is
// the operation's identity; the order of the combination is fixed, so sums are reproducible.
template <int CTRL, int ROW_MASK>
LVS_DEV uint32_t dpp_move(uint32_t ident, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)ident, (int)v, CTRL, ROW_MASK, 0xf, false);
}

template <class Op>
LVS_DEV float wave_reduce(float x, float ident, Op op) {
  const uint32_t id = __builtin_bit_cast(uint32_t, ident);
  auto f = [](uint32_t u) { return __builtin_bit_cast(float, u); };
  auto u = [](float v) { return __builtin_bit_cast(uint32_t, v); };
  x = op(x, f(dpp_move<0xB1, 0xf>(id, u(x))));    // quad_perm [1,0,3,2]
  x = op(x, f(dpp_move<0x4E, 0xf>(id, u(x))));    // quad_perm [2,3,0,1]
  x = op(x, f(dpp_move<0x141, 0xf>(id, u(x))));   // row_half_mirror
  x = op(x, f(dpp_move<0x140, 0xf>(id, u(x))));   // row_mirror
  x = op(x, f(dpp_move<0x142, 0xa>(id, u(x))));   // row_bcast:15 into rows 1 and 3
  x = op(x, f(dpp_move<0x143, 0xc>(id, u(x))));   // row_bcast:31 into rows 2 and 3
  return f((uint32_t)__builtin_amdgcn_readlane((int)u(x), 63));
}

LVS_DEV float wave_max(float x) {
  return wave_reduce(x, -INFINITY, [](float a, float b) { return fmaxf(a, b); });
}

LVS_DEV float wave_sum(float x) {
  return wave_reduce(x, 0.f, [](float a, float b) { return a + b; });
}

// maximum of a 32-bit unsigned key over the wave (identity 0), same network
LVS_DEV uint32_t wave_max_u32(uint32_t x) {
  x = max(x, dpp_move<0xB1, 0xf>(0u, x));
  x = max(x, dpp_move<0x4E, 0xf>(0u, x));
  x = max(x, dpp_move<0x141, 0xf>(0u, x));
  x = max(x, dpp_move<0x140, 0xf>(0u, x));
  x = max(x, dpp_move<0x142, 0xa>(0u, x));
  x = max(x, dpp_move<0x143, 0xc>(0u, x));
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// maximum of a 64-bit unsigned key over the wave (identity 0), same network
LVS_DEV uint64_t wave_max_u64(uint64_t x) {
  auto step = [&](auto ctrl, auto row_mask) {
    const uint32_t lo = dpp_move<decltype(ctrl)::value, decltype(row_mask)::value>(0u, (uint32_t)x);
    const uint32_t hi =
        dpp_move<decltype(ctrl)::value, decltype(row_mask)::value>(0u, (uint32_t)(x >> 32));
    const uint64_t o = ((uint64_t)hi << 32) | lo;
    x = o > x ? o : x;
  };
  using std::integral_constant;
  step(integral_constant<int, 0xB1>{}, integral_constant<int, 0xf>{});
  step(integral_constant<int, 0x4E>{}, integral_constant<int, 0xf>{});
  step(integral_constant<int, 0x141>{}, integral_constant<int, 0xf>{});
  step(integral_constant<int, 0x140>{}, integral_constant<int, 0xf>{});
  step(integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{});
  step(integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{});
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, 63);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), 63);
  return ((uint64_t)hi << 32) | lo;
}

}  // namespace lvspec
