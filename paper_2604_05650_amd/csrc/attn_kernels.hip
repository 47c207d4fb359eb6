// Verification attention for gfx950: the gamma draft rows of every query head attend over the
// target's long KV cache (the target forward of the paper's Eq. 1, one layer; scaled-dot-product
// attention per its implementation details).
//
// Kernel 1 (split):   one workgroup per (key-range split, kv head, sequence, row chunk), laid out
//   on a 1-D grid so that all workgroups of a kv head land on one XCD; 4 * RS waves.
//   All G*gamma query rows that share one kv head are processed together (G = Hq/Hkv), so every
//   K/V byte is read from HBM exactly once (more than 64 rows take several row chunks).  The key
//   range of the workgroup is cut into tiles of 32 keys; stream s takes tiles s, s+4, ... and
//   moves them through its own two-slot LDS ring with direct-to-LDS copies (one or two tiles
//   beyond a multiple of four go through extra slots instead of a round of their own).
//   Per tile:  S^T[key][row] = K Q^T  by 16x16x32 bf16 MFMA (keys are the M side, so a lane owns
//   one query row and four keys per block);  online softmax in base 2 with a lazily updated
//   running maximum;  O^T[dv][row] += V^T P^T  by MFMA, the V operand being transposed on the fly
//   with byte permutes from 16-byte row reads.  The softmax mass on the video-token span is
//   accumulated from the same probabilities.  Draft rows see each other through a per-row bit
//   mask (causal chain by default, ancestor masks for draft trees).
//   The four streams merge their (max, sum, O) through LDS in a fixed order and the workgroup
//   writes one fp32 partial per split.
// Kernel 2 (combine): log-sum-exp merge of the split partials in split order, bf16 output.
#include "lvspec_dev.h"
#include "lvspec_kernels.h"

namespace lvspec {

namespace {

constexpr int kTileKeys = 32;
constexpr int kTileBytes = kTileKeys * kRowBytes;   // 8 KiB per K or V tile
constexpr int kSlotBytes = 2 * kTileBytes;          // K tile + V tile
constexpr int kRingBytesPerWave = 2 * kSlotBytes;   // two slots
constexpr float kNegBig = -1.0e30f;
constexpr int kORowStride = 132;                    // floats per row in the merge buffer (pad)
constexpr int kMaxExtraTiles = 2;                   // extra-tile slots of a workgroup
constexpr int kExtraTileAfterRound = 0;             // an extra tile is taken behind this round

// A K or V tile is 32 rows of 256 bytes in LDS; the 16-byte chunk c of row r sits at position
// c ^ tile_swz(r).  The LDS serves a 16-byte-per-lane read of a wave in four passes of 16 lanes
// (64 banks of 4 bytes), and the passes are not lanes 0-15, 16-31, ...: counters on in-bounds
// probe reads show lanes {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31} and the same two sets + 32.
// With r & 15 alone as the key, the K operand reads (lane -> row n16, chunk 4*ks + g4) are free
// of conflicts but the V reads (lane -> row 4*g4 + i, chunk n16) put rows i and 4 + i of one pass
// on the same banks and take twice as long; flipping bit 3 of the key in rows with bit 2 set
// separates them and keeps the K reads conflict-free.
LVS_DEV constexpr int tile_swz(int r) { return (r & 15) ^ ((r & 4) << 1); }

// issue the eight copy instructions of one 32-row tile; row index clamped to last_row
LVS_DEV void issue_tile(const uint8_t* __restrict__ base, int64_t row_stride_bytes, int tile,
                        int last_row, uint32_t lds_tile, int g4, const uint32_t (&coff)[4]) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    int row = tile * kTileKeys + 4 * j + g4;
    row = row < last_row ? row : last_row;
    dma16(base + (int64_t)row * row_stride_bytes + coff[j & 3], lds_tile + j * 1024);
  }
}

// The same copies from per-lane row pointers computed once per kernel (rowp[j] points at the
// chunk this lane fetches for copy instruction j of tile 0): one 64-bit add per instruction.
// Valid for every tile whose 32 rows all exist, i.e. all but the last tile of a sequence.
template <int N>
LVS_DEV void issue_rows(const uint8_t* const (&rowp)[N], int64_t tile_off, uint32_t lds_tile,
                        int j0) {
#pragma unroll
  for (int jj = 0; jj < N; ++jj) dma16(rowp[jj] + tile_off, lds_tile + (j0 + jj) * 1024);
}

template <int NB>
struct WaveState {
  f32x4 acc[8][NB];   // O^T: [dv block][row block]
  float m[NB];        // running max of scaled scores (log2 units), same in the 4 lanes of a row
  float l[NB];        // this lane's share of the denominator
  float lvis[NB];     // this lane's share of the mass on the video span
};

// S^T[key][row] = K Q^T for one 32-key tile: kop[kb*4 + ks] is the K operand of key block kb and
// 32-wide slice ks of the head dimension.
template <int NB>
LVS_DEV void tile_scores(f32x4 (&s)[2][NB], const u32x4 (&kop)[8], const u32x4 (&qreg)[NB][4]) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) z = mfma16(kop[kb * 4 + ks], qreg[nb][ks], z);
      s[kb][nb] = z;
    }
}

// Visibility for tiles that reach past the cached prefix: draft key j is visible to a row iff
// bit j of the row's mask is set; keys past the last draft row are never visible.
template <int NB>
LVS_DEV void tile_mask(f32x4 (&s)[2][NB], int key0, int L, const uint32_t (&rowmask)[NB], int g4) {
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // rowmask has no bit at or above gamma (<= 32), so draft index j in [gamma, 32) reads 0
        const int j = key0 + kb * 16 + 4 * g4 + i - L;
        const int jc = j < 0 ? 0 : (j > 31 ? 31 : j);
        const uint32_t bit = (rowmask[nb] >> jc) & 1u;
        const bool vis = (j < 0) | ((j < 32) & (bit != 0u));
        s[kb][nb][i] = vis ? s[kb][nb][i] : -INFINITY;
      }
}

// Online softmax in base 2 with a lazily updated running maximum; returns the probabilities as
// the bf16 B operand of the PV product and accumulates the denominators.
template <int NB>
LVS_DEV void tile_softmax(WaveState<NB>& st, const f32x4 (&s)[2][NB], u32x4 (&pop)[NB], int key0,
                          float c, int vis_b, int vis_e, int g4) {
  bool grow = false;
  float tmax[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float t = fmaxf(fmaxf(s[0][nb][0], s[0][nb][1]), fmaxf(s[0][nb][2], s[0][nb][3]));
    t = fmaxf(t, fmaxf(fmaxf(s[1][nb][0], s[1][nb][1]), fmaxf(s[1][nb][2], s[1][nb][3])));
    tmax[nb] = t * c;
    grow |= tmax[nb] > st.m[nb];
  }
  if (__any(grow)) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float x = fmaxf(st.m[nb], tmax[nb]);
      x = fmaxf(x, xor_shuffle(x, 16));
      x = fmaxf(x, xor_shuffle(x, 32));
      const float alpha = fast_exp2(st.m[nb] - x);
      st.m[nb] = x;
      st.l[nb] *= alpha;
      st.lvis[nb] *= alpha;
#pragma unroll
      for (int mb = 0; mb < 8; ++mb) st.acc[mb][nb] *= alpha;
    }
  }
  const bool vis_any = (key0 < vis_e) && (key0 + kTileKeys > vis_b);
  const bool vis_all = (key0 >= vis_b) && (key0 + kTileKeys <= vis_e);
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float p[8];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        p[kb * 4 + i] = fast_exp2(__builtin_fmaf(s[kb][nb][i], c, -st.m[nb]));
    const float tsum = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
    st.l[nb] += tsum;
    if (vis_all) {
      st.lvis[nb] += tsum;
    } else if (vis_any) {
      float vs = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int key = key0 + (e >> 2) * 16 + 4 * g4 + (e & 3);
        vs += (key >= vis_b && key < vis_e) ? p[e] : 0.f;
      }
      st.lvis[nb] += vs;
    }
    pop[nb] = u32x4{pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]),
                    pack_bf16(p[6], p[7])};
  }
}

// O^T += V^T P^T.  vraw[half*4 + i] holds key half*16 + 4*g4 + i, channels 8*n16 .. +7; byte
// permutes gather, for each of the 8 channels, the 8 keys of this lane into one A operand.
template <int NB>
LVS_DEV void tile_pv(WaveState<NB>& st, const u32x4 (&vraw)[8], const u32x4 (&pop)[NB]) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    u32x4 lo, hi;
#pragma unroll
    for (int d2 = 0; d2 < 4; ++d2) {
      lo[d2] = __builtin_amdgcn_perm(vraw[2 * d2 + 1][w], vraw[2 * d2][w], 0x05040100u);
      hi[d2] = __builtin_amdgcn_perm(vraw[2 * d2 + 1][w], vraw[2 * d2][w], 0x07060302u);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      st.acc[2 * w][nb] = mfma16(lo, pop[nb], st.acc[2 * w][nb]);
      st.acc[2 * w + 1][nb] = mfma16(hi, pop[nb], st.acc[2 * w + 1][nb]);
    }
  }
}

// One tile of a wave-private stream.  WK / WV: copy instructions that may stay outstanding when
// the K / V tile is read.
// refill_k / refill_v are called as soon as the K / V part of the slot has been read (they issue
// the copies of a later tile into it, or do nothing).
template <int NB, int WK, int WV, class RefillK, class RefillV>
LVS_DEV void process_tile(WaveState<NB>& st, const u32x4 (&qreg)[NB][4], uint32_t lds_slot,
                          const uint32_t (&kaddr)[4], const uint32_t (&vaddr)[4], int tile,
                          int L, const uint32_t (&rowmask)[NB], float c, int vis_b, int vis_e,
                          int g4, RefillK&& refill_k, RefillV&& refill_v) {
  f32x4 s[2][NB];
  {
    uint32_t a[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) a[ks] = lds_slot + kaddr[ks];
    u32x4 kop[8];   // [kb*4 + ks]
    lds_read8_after<WK, 16 * kRowBytes>(kop, a);
    refill_k();
    tile_scores<NB>(s, kop, qreg);
  }
  const int key0 = tile * kTileKeys;
  if (key0 + kTileKeys > L) tile_mask<NB>(s, key0, L, rowmask, g4);
  u32x4 pop[NB];
  tile_softmax<NB>(st, s, pop, key0, c, vis_b, vis_e, g4);
  {
    uint32_t a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = lds_slot + kTileBytes + vaddr[i];
    u32x4 vraw[8];
    lds_read8_after<WV, 16 * kRowBytes>(vraw, a);
    refill_v();
    tile_pv<NB>(st, vraw, pop);
  }
}

// Block id -> (item, unit), unit = (sequence, row chunk, kv head), `per_unit` items per unit.
// Workgroups are handed to the 8 XCDs round-robin by linear id and every XCD has its own L2.
// When the number of units is a multiple of 8, all items of a unit are placed on one XCD (the
// split workgroups of a kv head, and later the combine workgroups of its rows), so that the
// partial results written by the first kernel are read back from the same L2 by the second.
LVS_DEV void decode_block(int xcd_map, int id, FastDiv div_per_unit, int per_unit, int& item,
                          int& unit) {
  if (xcd_map) {
    const int xcd = id & 7;
    const int j = id >> 3;
    const int u_local = (int)fast_div((uint32_t)j, div_per_unit);
    item = j - u_local * per_unit;
    unit = u_local * 8 + xcd;
  } else {
    unit = (int)fast_div((uint32_t)id, div_per_unit);
    item = id - unit * per_unit;
  }
}

// copy this wave's share (8 / CW instructions) of one 32-row tile that CW waves load together
template <int CW>
LVS_DEV void issue_part(const uint8_t* __restrict__ base, int64_t row_stride_bytes, int tile,
                        int last_row, uint32_t lds_tile, int rh, int n16, int g4) {
  constexpr int IPH = 8 / CW;
  // This path runs once per sequence (its last, possibly ragged tile).  The lane coordinates
  // are made opaque here so that none of its per-lane address arithmetic is hoisted out of the
  // caller's tile loop, where it would occupy registers through every round (16 fewer in the
  // 32-row variant).
  asm volatile("" : "+v"(n16), "+v"(g4));
#pragma unroll
  for (int jj = 0; jj < IPH; ++jj) {
    const int j = rh * IPH + jj;
    int row = tile * kTileKeys + 4 * j + g4;
    row = row < last_row ? row : last_row;
    const uint32_t off = (uint32_t)((n16 ^ tile_swz(4 * j + g4)) << 4);
    dma16(base + (int64_t)row * row_stride_bytes + off, lds_tile + j * 1024);
  }
}

// RS = 1: four waves, each streaming its own tiles through a private ring and holding all
//         16*NBW query rows (no barrier in the main loop).
// RS > 1: 4*RS waves; the RS waves of a stream share one ring and one copy of every K/V tile,
//         each holding its own 16*NBW of the 16*NBW*RS query rows.  This keeps the per-wave
//         register footprint and dependent instruction chains short when many query rows share
//         a kv head, and puts RS waves on every SIMD so that their MFMA, exp and LDS phases
//         overlap.  The waves of the workgroup meet at two barriers per tile round.
// RS = 3: as RS = 2 (the first two waves of a stream issue its copies) plus a third wave per
//         stream that only computes: 48 query rows, for row counts between 33 and 48.
//
// Fast start.  All waves of all workgroups read the same few lines of the argument buffer when
// the kernel starts, and that read is slow (in-kernel timestamps: the first wave has its
// arguments 0.9 us after entry, the median wave after 2.5 us, the last after 4 us), so the
// memory pipeline fills late.  For one sequence whose length the host knows (fast = 1: the
// common decode case), everything the first tile copies depend on travels in thirteen leading
// scalar arguments, which qualify for kernel-argument
// preloading into scalar registers by the command processor (the file is built with
// -amdgpu-kernarg-preload-count; without that service the compatibility prologue loads them):
//   k0, v0, kv_sh0, kv_sl0   cache pointers and strides (elements)
//   n_split0, split_mul0     key-range splits and their multiply-shift divisor
//   Hkv0, hkv_mul0           kv heads and their multiply-shift divisor
//   packed0                  bits 0-7 shift of the split divisor, bit 8 xcd_map, bits 16-21 gamma,
//                            bits 24-30 shift of the head divisor, bit 31 fast
//   len0                     kv_len[0]
// The structure behind them is then first needed for the query rows, behind the first copies.
// In every other case (fast = 0) the kernel starts from the structure as before.
template <int RS, int NBW>
__global__ __launch_bounds__(256 * RS, 1) void attn_split_kernel(
    const uint16_t* k0, const uint16_t* v0, int64_t kv_sh0, int kv_sl0, int n_split0,
    uint32_t split_mul0, int Hkv0, uint32_t hkv_mul0, uint32_t packed0, int len0,
    const AttnKernelArgs p) {
  extern __shared__ __align__(16) uint8_t smem[];
  constexpr int NB = NBW;
  constexpr int RPAD = 16 * NBW * RS;
  constexpr int NT = 256 * RS;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int stream = wave & 3;
  const int rh = wave >> 2;
  const int n16 = lane & 15;
  const int g4 = lane >> 4;
  LVS_TRACE_BEGIN;
  LVS_TRACE(0);
  int split, unit, kvh, b, rc, L, gamma, n_split;
  FastDiv div_split;
  const uint8_t* kbase;
  const uint8_t* vbase;
  int64_t rsb;
  if (packed0 >> 31) {
    gamma = (int)((packed0 >> 16) & 63u);
    n_split = n_split0;
    div_split = FastDiv{split_mul0, packed0 & 255u};
    decode_block((int)((packed0 >> 8) & 1u), blockIdx.x, div_split, n_split, split, unit);
    // one sequence: unit = row chunk * Hkv + kv head
    rc = (int)fast_div((uint32_t)unit, FastDiv{hkv_mul0, (packed0 >> 24) & 127u});
    kvh = unit - rc * Hkv0;
    b = 0;
    L = len0;
    rsb = (int64_t)kv_sl0 * 2;
    kbase = reinterpret_cast<const uint8_t*>(k0) + (int64_t)kvh * kv_sh0 * 2;
    vbase = reinterpret_cast<const uint8_t*>(v0) + (int64_t)kvh * kv_sh0 * 2;
  } else {
    // Everything the first tile copies need comes from the block id and the launch arguments
    // in straight-line code.  One statement that needs all of them in scalar registers: the
    // compiler otherwise fetches each argument right before its first use, which turns the
    // start of the kernel into a chain of dependent scalar-memory round trips.
    asm volatile("" ::"s"(p.k), "s"(p.v), "s"(p.kv_len), "s"(p.kv_sb), "s"(p.kv_sh), "s"(p.kv_sl),
                 "s"(p.gamma), "s"(p.Hkv), "s"(p.xcd_map), "s"(p.n_rc), "s"(p.n_split),
                 "s"(p.len_mode), "s"(p.div_split.mul), "s"(p.div_split.shift),
                 "s"(p.div_hkv.mul), "s"(p.div_hkv.shift), "s"(p.div_rc.mul),
                 "s"(p.div_rc.shift));
    gamma = p.gamma;
    n_split = p.n_split;
    div_split = p.div_split;
    decode_block(p.xcd_map, blockIdx.x, div_split, n_split, split, unit);
    const int z = (int)fast_div((uint32_t)unit, p.div_hkv);
    kvh = unit - z * p.Hkv;
    b = (int)fast_div((uint32_t)z, p.div_rc);
    rc = z - b * p.n_rc;
    // The sequence length, uniform over the workgroup.  Host-known lengths of small batches sit
    // in the argument lines fetched above (a scalar-cache hit); a larger host table is a
    // further line of the argument buffer, which nobody has touched yet (a trip to memory,
    // slower than the device read below, which usually hits in L2: it is used only without a
    // device array).  The device read goes through a scalar register inside its branch, so the
    // wait for it stays there.
    if (p.len_mode == 1) {
      L = p.len_hot[b < 5 ? b : 0];
    } else if (p.len_mode == 2) {
      L = p.len_host[b & 31];
    } else {
      // a length from device memory is not the host's to check: a stale or oversized value is
      // clamped so that no copy reaches past the rows the caller declared (cap)
      L = __builtin_amdgcn_readfirstlane(p.kv_len[b]);
      L = L < 0 ? 0 : (L > p.lmax ? p.lmax : L);
    }
    rsb = p.kv_sl * 2;
    kbase = reinterpret_cast<const uint8_t*>(p.k) +
            ((int64_t)b * p.kv_sb + (int64_t)kvh * p.kv_sh) * 2;
    vbase = reinterpret_cast<const uint8_t*>(p.v) +
            ((int64_t)b * p.kv_sb + (int64_t)kvh * p.kv_sh) * 2;
  }
  const int n_keys = L + gamma;
  const int n_tiles = (n_keys + kTileKeys - 1) / kTileKeys;
  // balanced contiguous tile ranges: the first (n_tiles % n_split) splits get one tile more
  const int t_base = (int)fast_div((uint32_t)n_tiles, div_split);
  const int t_rem = n_tiles - t_base * n_split;
  const int t_begin = split * t_base + (split < t_rem ? split : t_rem);
  const int t_end = t_begin + t_base + (split < t_rem ? 1 : 0);
  // A workgroup whose tile count is 4q + 1 or 4q + 2 would run q + 1 rounds, the last with one
  // or two of its four streams: that round is pure latency (its data arrived long before) and,
  // when most workgroups have 4q tiles, it is what the whole launch ends on (the 32B shape with
  // 16384 cached keys and 5 draft keys: 513 tiles per kv head over 32 workgroups; 0.6 us of a
  // 15 us kernel, and as much for 514 or 515 tiles).  Such a workgroup instead keeps its last
  // one or two tiles in extra LDS slots, requested ahead of everything else, and streams 0 and 1
  // take them right behind their first regular tile, early in the kernel, where a late stream
  // costs its workgroup nothing at the end.  Taking them behind the second tile measures the
  // same, behind the third loses the gain.  The assignment is a fixed function of the shape, so
  // results stay repeatable.
  int n_x = 0;
  if constexpr (kMaxExtraTiles > 0) {
    const int t_all = t_end - t_begin;
    const int e = t_all & 3;
    n_x = e >= 1 && e <= kMaxExtraTiles && t_all >= 3 * 4 ? e : 0;
  }
  const int t_main_end = t_end - n_x;
  const bool has_x = stream < n_x;
  const int x_tile = t_main_end + stream;
  const int first = t_begin + stream;
  const int my_n = first < t_main_end ? (t_main_end - first + 3) >> 2 : 0;
  LVS_TRACE(1);

  uint32_t coff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) coff[i] = (uint32_t)((n16 ^ tile_swz(4 * i + g4)) << 4);
  const uint32_t ring = lds_addr(smem) + stream * kRingBytesPerWave;
  const int last_row = n_keys - 1;
  constexpr int CW = RS == 3 ? 2 : RS;  // waves of a stream that issue its copies
  constexpr int IPH = 8 / CW;           // copy instructions of such a wave per K or V tile
  const bool copier = rh < CW;
  const int j0 = copier ? rh * IPH : 0;
  const uint8_t* krow[IPH];
#pragma unroll
  for (int jj = 0; jj < IPH; ++jj) {
    const int j = j0 + jj;
    krow[jj] = kbase + (int64_t)(4 * j + g4) * rsb + ((n16 ^ tile_swz(4 * j + g4)) << 4);
  }
  const int64_t v_minus_k = vbase - kbase;
  const int64_t tile_step = (int64_t)kTileKeys * rsb;
  // copies of K (which = 0) or V (which = 1) tile t into lds_tile; the last tile of the sequence
  // may be ragged and takes the clamping path
  auto copy_tile = [&](int which, int t, uint32_t lds_tile) {
    if (RS == 3 && !copier) return;     // the waits below then find nothing outstanding
    if (t != n_tiles - 1) {
      issue_rows<IPH>(krow, (int64_t)t * tile_step + (which ? v_minus_k : 0), lds_tile, j0);
    } else if constexpr (RS == 1) {
      issue_tile(which ? vbase : kbase, rsb, t, last_row, lds_tile, g4, coff);
    } else {
      issue_part<CW>(which ? vbase : kbase, rsb, t, last_row, lds_tile, rh, n16, g4);
    }
  };

  // First copies.  Only what the first tile needs leaves here; the rest of the two ring slots is
  // requested further down, behind the set-up code.  Measured at the 32B/72B shapes: with every
  // wave of the chip asking for both slots at once, everybody's first tile lands later and the
  // call takes 0.3-1.0 us longer (the memory system is already saturated by the first tiles; an
  // explicit delay on top of the set-up code only loses again).  The 32-row two-wave variant
  // keeps V0 up front (17.5 against 17.8 us), the others do better with K0 alone.
  constexpr bool kV0Early = RS <= 2 && NBW == 1;
  const uint32_t x_slot = lds_addr(smem) + 4 * kRingBytesPerWave + stream * kSlotBytes;
  if (has_x) {   // older than every other copy of the wave: any later wait covers them
    copy_tile(0, x_tile, x_slot);
    copy_tile(1, x_tile, x_slot + kTileBytes);
  }
  if (my_n > 0) {
    copy_tile(0, first, ring);
    if (kV0Early) copy_tile(1, first, ring + kTileBytes);
  }
  LVS_TRACE(2);
  // LDS addresses of the MFMA operand reads (not needed to issue copies: computed behind them)
  uint32_t kaddr[4], vaddr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 4 * g4 + i;
    kaddr[i] = n16 * kRowBytes + (((4 * i + g4) ^ tile_swz(n16)) << 4);   // chunk 4*ks+g4, ks = i
    vaddr[i] = r * kRowBytes + ((n16 ^ tile_swz(r)) << 4);
  }
  // ---- query operand: rows of this wave, B-operand layout (branch-free: rows past R read a
  // valid row and are zeroed).  Requested behind the first tile copies: every instruction ahead
  // of those delays the whole stream.  Loads return in order, so the rows arrive after these
  // copies; their first use below waits for all of them, and from then on the copy counters of
  // the loop see tile copies only.
  asm volatile("" ::"s"(p.q), "s"(p.q_sb), "s"(p.q_sg), "s"(p.q_sh), "s"(p.G), "s"(p.R),
               "s"(p.Hkv), "s"(p.div_g.mul), "s"(p.div_g.shift));   // one batch, see above
  const int bh = b * p.Hkv + kvh;
  u32x4 qreg[NB][4];
  int draft_row[NB];      // draft row of this lane's query row, -1 past the last row
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int r = rc * RPAD + (rh * NBW + nb) * 16 + n16;
    const bool valid = r < p.R;
    const int rcl = valid ? r : p.R - 1;
    const int i = (int)fast_div((uint32_t)rcl, p.div_g);
    const int gq = rcl - i * p.G;
    draft_row[nb] = valid ? i : -1;
    const uint16_t* qp = p.q + (int64_t)b * p.q_sb + (int64_t)i * p.q_sg +
                         (int64_t)(kvh * p.G + gq) * p.q_sh;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      qreg[nb][ks] = *reinterpret_cast<const u32x4*>(qp + (4 * ks + g4) * 8);
  }
  LVS_TRACE(3);

  WaveState<NB> st;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    st.m[nb] = kNegBig;
    st.l[nb] = 0.f;
    st.lvis[nb] = 0.f;
#pragma unroll
    for (int mb = 0; mb < 8; ++mb) st.acc[mb][nb] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const float c = p.scale_log2e;
  int vis_b = 0, vis_e = 0;
  if (p.vis_begin != nullptr) {   // not needed before the first softmax: keep it off the start
    vis_b = p.vis_begin[b];
    vis_e = p.vis_end[b];
  }
  // Visibility masks of this lane's rows among the draft rows: only the tiles that reach past
  // the cached prefix use them, so the mask words are fetched here, behind the first tile
  // copies, in branch-free code.
  uint32_t rowmask[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    uint32_t mk = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) mk = (draft_row[nb] == j) ? p.draft_mask[j] : mk;
    rowmask[nb] = mk & (0xffffffffu >> (32 - gamma));
  }
  // First use of the query rows (rows past the last one become zero): the wait for them sits
  // here, behind the first tile copies, so their latency overlaps with the copies' instead of
  // preceding it, and the loop below starts without a pending register load.
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qreg[nb][ks] = draft_row[nb] >= 0 ? qreg[nb][ks] : u32x4{0u, 0u, 0u, 0u};
      asm volatile("" : "+v"(qreg[nb][ks]));
    }

  // the rest of the first requests: RS = 1 fills both slots (K0 V0 K1 V1), the shared rings
  // start with K0 V0 K1 (V1 follows K0's arrival, see the loop)
  if (my_n > 0 && !kV0Early) copy_tile(1, first, ring + kTileBytes);
  if (my_n > 1) {
    copy_tile(0, first + 4, ring + kSlotBytes);
    if constexpr (RS == 1) copy_tile(1, first + 4, ring + kSlotBytes + kTileBytes);
  }
  if constexpr (RS == 1) {
    if (my_n > 0) {
      int it = 0;
      auto nothing = [] {};
      if (n_x > 0) {
        // three or more tiles per stream: the first one in the steady-state form, then the extra
        // tile of this stream (its copies are older than K(0), which has just been read)
        process_tile<NB, 24, 24>(st, qreg, ring, kaddr, vaddr, first, L, rowmask, c, vis_b, vis_e, g4,
                                 [&] { copy_tile(0, first + 8, ring); },
                                 [&] { copy_tile(1, first + 8, ring + kTileBytes); });
        if (has_x)
          process_tile<NB, 63, 63>(st, qreg, x_slot, kaddr, vaddr, x_tile, L, rowmask, c, vis_b,
                                   vis_e, g4, nothing, nothing);
        it = 1;
      }
      // steady state: two tiles in flight behind the one being consumed
      for (; it + 2 < my_n; ++it) {
        const int tile = first + 4 * it;
        const uint32_t slot = ring + (it & 1) * kSlotBytes;
        process_tile<NB, 24, 24>(st, qreg, slot, kaddr, vaddr, tile, L, rowmask, c, vis_b, vis_e,
                                 g4, [&] { copy_tile(0, tile + 8, slot); },
                                 [&] { copy_tile(1, tile + 8, slot + kTileBytes); });
        LVS_TRACE(4);
      }
      if (it + 1 < my_n) {   // second to last: K(t) V(t) K(t+1) V(t+1) outstanding at most
        process_tile<NB, 24, 16>(st, qreg, ring + (it & 1) * kSlotBytes, kaddr, vaddr,
                                 first + 4 * it, L, rowmask, c, vis_b, vis_e, g4, nothing,
                                 nothing);
        LVS_TRACE(4);
        ++it;
      }
      // last: only K(t) V(t) outstanding
      process_tile<NB, 8, 0>(st, qreg, ring + (it & 1) * kSlotBytes, kaddr, vaddr, first + 4 * it,
                             L, rowmask, c, vis_b, vis_e, g4, nothing, nothing);
    }
  } else {
    // every wave of the workgroup runs the same number of rounds (streams differ by one tile)
    const int max_n = (t_main_end - t_begin + 3) >> 2;
    auto round = [&](int it) {
      const bool active = it < my_n;
      const bool has1 = it + 1 < my_n;
      const bool has2 = it + 2 < my_n;
      const uint32_t slot = ring + (it & 1) * kSlotBytes;
      const int tile = first + 4 * it;
      const int key0 = tile * kTileKeys;
      // K(it): younger copies of this wave are V(it) and, if there is a next tile, K(it+1)
      if (active) {
        if (has1) wait_copies<2 * IPH>(); else wait_copies<IPH>();
      }
      __builtin_amdgcn_s_barrier();   // all shares of K(it) landed; V slot of it-1 is free
      if (has1) copy_tile(1, tile + 4, ring + ((it + 1) & 1) * kSlotBytes + kTileBytes);
      u32x4 pop[NB];
      if (active) {
        f32x4 s[2][NB];
        uint32_t a[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) a[ks] = slot + kaddr[ks];
        u32x4 kop[8];
        lds_read8_after<63, 16 * kRowBytes>(kop, a);
        tile_scores<NB>(s, kop, qreg);
        if (key0 + kTileKeys > L) tile_mask<NB>(s, key0, L, rowmask, g4);
        tile_softmax<NB>(st, s, pop, key0, c, vis_b, vis_e, g4);
        // V(it): younger copies are K(it+1) and V(it+1) when there is a next tile
        if (has1) wait_copies<2 * IPH>(); else wait_copies<0>();
      }
      __builtin_amdgcn_s_barrier();   // all shares of V(it) landed; K slot of it is free
      if (has2) copy_tile(0, tile + 8, slot);
      if (active) {
        uint32_t a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = slot + kTileBytes + vaddr[i];
        u32x4 vraw[8];
        lds_read8_after<63, 16 * kRowBytes>(vraw, a);
        tile_pv<NB>(st, vraw, pop);
      }
      LVS_TRACE(4);
    };
    // The extra tile of a stream is taken between two rounds, outside the loops, so that the
    // rounds themselves stay free of the extra branch.  Its copies are older than K(0), whose
    // arrival every wave of the stream has waited for before the first barrier of round 0.
    int it = 0;
    for (; it < max_n && it <= kExtraTileAfterRound; ++it) round(it);
    if (has_x) {
      const int xkey0 = x_tile * kTileKeys;
      f32x4 s[2][NB];
      u32x4 pop[NB];
      uint32_t a[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) a[ks] = x_slot + kaddr[ks];
      u32x4 kop[8];
      lds_read8_after<63, 16 * kRowBytes>(kop, a);
      tile_scores<NB>(s, kop, qreg);
      if (xkey0 + kTileKeys > L) tile_mask<NB>(s, xkey0, L, rowmask, g4);
      tile_softmax<NB>(st, s, pop, xkey0, c, vis_b, vis_e, g4);
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = x_slot + kTileBytes + vaddr[i];
      u32x4 vraw[8];
      lds_read8_after<63, 16 * kRowBytes>(vraw, a);
      tile_pv<NB>(st, vraw, pop);
    }
    for (; it < max_n; ++it) round(it);
  }

  LVS_TRACE(5);
  // ---- reduce the per-lane sums over the four lanes of a row --------------------------------
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    st.l[nb] += xor_shuffle(st.l[nb], 16);
    st.l[nb] += xor_shuffle(st.l[nb], 32);
    st.lvis[nb] += xor_shuffle(st.lvis[nb], 16);
    st.lvis[nb] += xor_shuffle(st.lvis[nb], 32);
  }

  // ---- merge the four streams through LDS (fixed order) -------------------------------------
  // Every wave stores its state unscaled; the readers take the common maximum of the four
  // streams and rescale while they add (one barrier less than exchanging the maxima first).
  __syncthreads();   // every wave has left the rings
  LVS_TRACE(6);
  float* sm_m = reinterpret_cast<float*>(smem);            // [4][RPAD]
  float* sm_l = sm_m + 4 * RPAD;                           // [4][RPAD]
  float* sm_v = sm_l + 4 * RPAD;                           // [4][RPAD]
  float* sm_o = sm_v + 4 * RPAD;                           // [4][RPAD][kORowStride]
  const int row0 = rh * 16 * NBW;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int row = row0 + nb * 16 + n16;
    if (g4 == 0) {
      sm_m[stream * RPAD + row] = st.m[nb];
      sm_l[stream * RPAD + row] = st.l[nb];
      sm_v[stream * RPAD + row] = st.lvis[nb];
    }
    float* orow = sm_o + ((size_t)stream * RPAD + row) * kORowStride + 32 * g4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f32x4 lo = {st.acc[0][nb][i], st.acc[1][nb][i], st.acc[2][nb][i], st.acc[3][nb][i]};
      f32x4 hi = {st.acc[4][nb][i], st.acc[5][nb][i], st.acc[6][nb][i], st.acc[7][nb][i]};
      *reinterpret_cast<f32x4*>(orow + 8 * i) = lo;
      *reinterpret_cast<f32x4*>(orow + 8 * i + 4) = hi;
    }
  }
  __syncthreads();
  LVS_TRACE(7);
  float* part = p.ws + (((size_t)bh * p.n_rc + rc) * n_split + split) * (size_t)(RPAD * 131);
  // only the rows that exist are written (the combine kernel reads no others)
  const int rows_here = p.R - rc * RPAD < RPAD ? p.R - rc * RPAD : RPAD;
  for (int row = threadIdx.x; row < rows_here; row += NT) {
    const float m0 = sm_m[row], m1 = sm_m[RPAD + row], m2 = sm_m[2 * RPAD + row],
                m3 = sm_m[3 * RPAD + row];
    const float mm = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
    const float f0 = fast_exp2(m0 - mm), f1 = fast_exp2(m1 - mm), f2 = fast_exp2(m2 - mm),
                f3 = fast_exp2(m3 - mm);
    part[row] = mm;
    part[RPAD + row] = ((sm_l[row] * f0 + sm_l[RPAD + row] * f1) + sm_l[2 * RPAD + row] * f2) +
                       sm_l[3 * RPAD + row] * f3;
    part[2 * RPAD + row] = ((sm_v[row] * f0 + sm_v[RPAD + row] * f1) + sm_v[2 * RPAD + row] * f2) +
                           sm_v[3 * RPAD + row] * f3;
  }
  float* po = part + 3 * RPAD;
  for (int idx = threadIdx.x; idx < rows_here * 32; idx += NT) {
    const int row = idx >> 5;
    const int c4 = (idx & 31) * 4;
    const float m0 = sm_m[row], m1 = sm_m[RPAD + row], m2 = sm_m[2 * RPAD + row],
                m3 = sm_m[3 * RPAD + row];
    const float mm = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
    const float f0 = fast_exp2(m0 - mm), f1 = fast_exp2(m1 - mm), f2 = fast_exp2(m2 - mm),
                f3 = fast_exp2(m3 - mm);
    const float* src = sm_o + (size_t)row * kORowStride + c4;
    const size_t ws = (size_t)RPAD * kORowStride;
    f32x4 a0 = *reinterpret_cast<const f32x4*>(src);
    f32x4 a1 = *reinterpret_cast<const f32x4*>(src + ws);
    f32x4 a2 = *reinterpret_cast<const f32x4*>(src + 2 * ws);
    f32x4 a3 = *reinterpret_cast<const f32x4*>(src + 3 * ws);
    const f32x4 o4 = ((a0 * f0 + a1 * f1) + a2 * f2) + a3 * f3;
    // written through (agent scope) as it is produced: nothing of the partials is left dirty for
    // the write-back at the end of the kernel, which the combine launch waits for
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(po + (size_t)row * 128 + c4), "v"(o4)
                 : "memory");
  }
  LVS_TRACE(8);
  LVS_TRACE_END;
}

// One workgroup of 128 * kSG threads per (unit, row slot), i.e. per output row (b, i, h).  Wave w
// owns output channels 64*(w&1) .. +63 and every kSG-th split starting at w>>1.  The kernel is a
// chain of latencies (launch, arguments, partials, store), so its instruction count matters:
// everything that is uniform over the workgroup (row decode, split addresses, weights) is kept
// in scalar registers, the per-split statistics are reduced inside each wave by shuffles (no
// LDS round, no barrier before the partial outputs are consumed), and all loads of a thread are
// issued before the first is used.  Sums run in a fixed order.
constexpr int kMaxSplits = 256;

// kChunks: 64-split chunks covered, 1 (n_split <= 64) or kMaxSplits / 64.  kSG: split groups =
// wave pairs of the workgroup (2 for up to 32 splits, where four groups would only add clamped
// duplicate loads and waves to dispatch; 4 beyond).
//
// The fourteen leading scalar arguments are all that the partial loads depend on.  They are
// plain kernel arguments (not fields of the argument structure) so that they qualify for
// kernel-argument preloading into scalar registers by the command processor (the file is built
// with -amdgpu-kernarg-preload-count): the row decode then does not wait for a first, cold
// read of the argument buffer.  Where preloading is not available the kernel's compatibility
// prologue loads them as usual.  The structure behind them serves the output stage.
template <int kChunks, int kSG>
__global__ __launch_bounds__(128 * kSG) void attn_combine_kernel(
    const float* ws, int rpad, int xcd_map, int Hkv, int n_rc, int R, int n_split,
    uint32_t rpad_mul, uint32_t rpad_shift, uint32_t hkv_mul, uint32_t hkv_shift, uint32_t rc_mul,
    uint32_t rc_shift, const AttnKernelArgs p) {
  __shared__ float sm_o[kSG][128];
  LVS_TRACE2_BEGIN;
  LVS_TRACE2(0);
  LVS_TRACE2(5);
  const int RPAD = rpad;
  // divisions by launch constants are multiply-shifts, so the whole decode and the address
  // arithmetic below stay in scalar registers
  int rr, unit;
  decode_block(xcd_map, blockIdx.x, FastDiv{rpad_mul, rpad_shift}, RPAD, rr, unit);
  const int z = (int)fast_div((uint32_t)unit, FastDiv{hkv_mul, hkv_shift});
  const int kvh = unit - z * Hkv;
  const int b = (int)fast_div((uint32_t)z, FastDiv{rc_mul, rc_shift});
  const int rc = z - b * n_rc;
  const int r = rc * RPAD + rr;          // query row of this kv head: r = i * G + (h % G)
  if (r >= R) return;
  const int bh = b * Hkv + kvh;
  const int ns = n_split;
  const uint32_t stride = (uint32_t)RPAD * 131u;           // floats per partial record
  const float* base = ws + ((size_t)bh * n_rc + rc) * ns * stride;   // uniform
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sg = wave >> 1;
  const int dv = (wave & 1) * 64 + lane;
  LVS_TRACE2(6);

  // statistics of split 64*c + lane (every wave keeps its own copy)
  float ms[kChunks], ls[kChunks], vs[kChunks];
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    ms[c] = kNegBig;
    ls[c] = 0.f;
    vs[c] = 0.f;
    if (c * 64 < ns) {
      const int sidx = c * 64 + lane;
      const uint32_t off = (uint32_t)(sidx < ns ? sidx : ns - 1) * stride + (uint32_t)rr;
      ms[c] = base[off];
      ls[c] = base[off + RPAD];
      vs[c] = base[off + 2 * RPAD];
    }
  }
  // partial outputs of the first 64 splits, requested before the statistics are used
  const uint32_t dv_bytes = (uint32_t)dv * 4u;
  const float* orow = base + 3 * RPAD + (size_t)rr * 128;                  // uniform
  auto load_vals = [&](float (&vals)[16], int c0) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int sidx = c0 + sg + kSG * u;
      const float* pu = orow + (size_t)(sidx < ns ? sidx : ns - 1) * stride;   // uniform
      vals[u] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pu) + dv_bytes);
    }
  };
  float vals[16];
  load_vals(vals, 0);
  // keep the statistics' first use behind these loads: waiting for the (older) statistics then
  // leaves the partial outputs in flight
  __builtin_amdgcn_sched_barrier(0);
  LVS_TRACE2(1);
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    const bool on = c * 64 + lane < ns;     // lanes past the last split hold a clamped copy
    ms[c] = on ? ms[c] : kNegBig;
    ls[c] = on ? ls[c] : 0.f;
    vs[c] = on ? vs[c] : 0.f;
  }

  float mm = ms[0];
#pragma unroll
  for (int c = 1; c < kChunks; ++c) mm = fmaxf(mm, ms[c]);
  mm = wave_max(mm);
  float f[kChunks];
  float l = 0.f, lv = 0.f;
#pragma unroll
  for (int c = 0; c < kChunks; ++c) {
    f[c] = fast_exp2(ms[c] - mm);       // 0 for lanes past the last split
    l += ls[c] * f[c];
    lv += vs[c] * f[c];
  }
  l = wave_sum(l);
  lv = wave_sum(lv);
  LVS_TRACE2(2);

  // weight of split sidx (uniform): lane sidx % 64 of chunk sidx / 64
  auto weight = [&](int sidx) {
    float w = 0.f;
#pragma unroll
    for (int c = 0; c < kChunks; ++c)
      if ((sidx >> 6) == c)
        w = __builtin_bit_cast(
            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, f[c]), sidx & 63));
    return sidx < ns ? w : 0.f;
  };
  float o = 0.f;
  for (int c0 = 0; c0 < ns; c0 += 16 * kSG) {
    if (c0 > 0) load_vals(vals, c0);
#pragma unroll
    for (int u = 0; u < 16; ++u) o += vals[u] * weight(c0 + sg + kSG * u);
  }
  sm_o[sg][dv] = o;
  LVS_TRACE2(3);
  __syncthreads();
  if (sg == 0) {
    const int i = (int)fast_div((uint32_t)r, p.div_g);
    const int h = kvh * p.G + (r - i * p.G);
    float tot = sm_o[0][dv];
#pragma unroll
    for (int k = 1; k < kSG; ++k) tot += sm_o[k][dv];
    const float inv = 1.0f / l;
    uint16_t* op = p.out + (int64_t)b * p.o_sb + (int64_t)i * p.o_sg + (int64_t)h * p.o_sh;
    const __bf16 ob = (__bf16)(tot * inv);
    op[dv] = __builtin_bit_cast(uint16_t, ob);
    if (dv == 0) {
      const size_t idx = ((size_t)b * p.Hq + h) * p.gamma + i;
      if (p.lse) p.lse[idx] = (mm + log2f(l)) * 0.69314718055994530942f;
      if (p.vis_mass) p.vis_mass[idx] = lv * inv;
    }
  }
  LVS_TRACE2(4);
  LVS_TRACE2_END;
}

}  // namespace

// extra: whether some workgroup of the launch can hold more than 4q tiles with q >= 3 (only
// those use the extra-tile slots behind the rings)
static size_t split_lds_bytes(int rpad, bool extra) {
  const size_t ring = 4 * (size_t)kRingBytesPerWave + (extra ? kMaxExtraTiles * (size_t)kSlotBytes : 0);
  const size_t merge = (3 * 4 * (size_t)rpad + 4 * (size_t)rpad * kORowStride) * sizeof(float);
  return ring > merge ? ring : merge;
}

template <int RS, int NBW>
static hipError_t launch_split(const AttnKernelArgs& a, hipStream_t stream) {
  // no sequence longer than lmax + gamma keys: the most tiles a workgroup can get
  const int64_t max_tiles = ((int64_t)a.lmax + a.gamma + kTileKeys - 1) / kTileKeys;
  const bool extra = (max_tiles + a.n_split - 1) / a.n_split > 3 * 4;
  const size_t lds = split_lds_bytes(16 * NBW * RS, extra);
  static LdsLimitOnce lds_limit;
  hipError_t e = lds_limit.ensure(reinterpret_cast<const void*>(&attn_split_kernel<RS, NBW>),
                                  split_lds_bytes(16 * NBW * RS, true));
  if (e != hipSuccess) return e;
  dim3 grid(a.n_split * a.Hkv * a.B * a.n_rc);
  // fast start: one sequence with a host-known length (see the kernel)
  const bool fast = a.B == 1 && a.len_mode == 1 && a.kv_sl < ((int64_t)1 << 31) &&
                    a.div_split.shift < 256u && a.div_hkv.shift < 128u;
  const uint32_t packed = (a.div_split.shift & 255u) | ((a.xcd_map ? 1u : 0u) << 8) |
                          ((uint32_t)a.gamma << 16) | ((a.div_hkv.shift & 127u) << 24) |
                          ((fast ? 1u : 0u) << 31);
  hipLaunchKernelGGL((attn_split_kernel<RS, NBW>), grid, dim3(256 * RS), lds, stream, a.k, a.v,
                     a.kv_sh, (int)a.kv_sl, a.n_split, a.div_split.mul, a.Hkv, a.div_hkv.mul,
                     packed, a.len_hot[0], a);
  return hipGetLastError();
}

// variant = 10 * RS + NBW; 0 picks the default for the row-chunk size
hipError_t launch_attn(const AttnKernelArgs& a, hipStream_t stream) {
  int variant = a.variant;
  if (variant == 0) variant = a.rpad == 16 ? 11 : a.rpad == 32 ? 21 : a.rpad == 48 ? 31 : 22;
  hipError_t e;
  switch (variant) {
    case 11: if (a.rpad != 16) return hipErrorInvalidValue; e = launch_split<1, 1>(a, stream); break;
    case 12: if (a.rpad != 32) return hipErrorInvalidValue; e = launch_split<1, 2>(a, stream); break;
    case 21: if (a.rpad != 32) return hipErrorInvalidValue; e = launch_split<2, 1>(a, stream); break;
    case 31: if (a.rpad != 48) return hipErrorInvalidValue; e = launch_split<3, 1>(a, stream); break;
    case 14: if (a.rpad != 64) return hipErrorInvalidValue; e = launch_split<1, 4>(a, stream); break;
    case 22: if (a.rpad != 64) return hipErrorInvalidValue; e = launch_split<2, 2>(a, stream); break;
    case 41: if (a.rpad != 64) return hipErrorInvalidValue; e = launch_split<4, 1>(a, stream); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  const dim3 cgrid(a.B * a.n_rc * a.Hkv * a.rpad);
#define LVS_COMBINE_ARGS                                                                        \
  a.ws, a.rpad, a.xcd_map, a.Hkv, a.n_rc, a.R, a.n_split, a.div_rpad.mul, a.div_rpad.shift,     \
      a.div_hkv.mul, a.div_hkv.shift, a.div_rc.mul, a.div_rc.shift, a
  if (a.n_split <= 32)
    hipLaunchKernelGGL((attn_combine_kernel<1, 2>), cgrid, dim3(256), 0, stream, LVS_COMBINE_ARGS);
  else if (a.n_split <= 64)
    hipLaunchKernelGGL((attn_combine_kernel<1, 4>), cgrid, dim3(512), 0, stream, LVS_COMBINE_ARGS);
  else
    hipLaunchKernelGGL((attn_combine_kernel<kMaxSplits / 64, 4>), cgrid, dim3(512), 0, stream,
                       LVS_COMBINE_ARGS);
#undef LVS_COMBINE_ARGS
  return hipGetLastError();
}

}  // namespace lvspec
