// Streamed skinny GEMM for gfx950: C[r][c] = sum_t A[r][t] X[c][t] with A a tall bf16 matrix read
// exactly once from HBM and X at most 64 bf16 rows.  Two users:
//   relevance (paper Eq. 8):  A = video hidden states H_V [l_v, d], X = draft hidden states
//       H_D [gamma, d]; the kernel emits raw dot products and squared row norms per split of d;
//       a finalize kernel turns them into cosines and the mean of the Top-N.
//   lm_head (paper Eq. 6):    A = lm_head [V, d], X = the B*gamma final hidden rows; the
//       epilogue reduces each block of vocabulary rows to (max, sum exp, top-k candidates) per
//       column, so the gamma x V logits never have to be re-read (they are written only on
//       request).
//
// Structure: persistent workgroups (two per CU, 4 waves each).  A workgroup walks its tasks (row
// block x split of d) as one uninterrupted sequence of stages; a stage is a slice of d of RB
// bytes per row (RB = 256 or 512: 128 or 256 elements).  Every wave copies its own 16*MB rows of
// A plus a share of the X slice straight into LDS (a ring of as many slots as fit into half of
// the CU's LDS: two to four), then all waves meet at one barrier per stage and feed 16x16x32
// bf16 MFMAs from LDS.  The ring keeps running across task boundaries, so there is no pipeline
// bubble between tasks.  Squared norms of the A rows come from the diagonal of A A^T on the
// same MFMA operands.
//
// Instances <MODE, MB, NBX, RB>: 64*MB rows of A per task, 16*NBX columns of X.
//   relevance: <1,1,512> (up to 16 draft rows, d % 256 == 0); otherwise <1|2, 1|2, 256>
//   lm_head:   <1,1,256> or <2,1,256> up to 16 columns, <1,2,256> or <2,2,256> up to 32,
//              <1,3,256> up to 48, <1,4,256> up to 64 (a last,
//              narrower pass over a group of chains keeps the task size of the full passes)
#include "lvspec_dev.h"
#include "lvspec_kernels.h"

namespace lvspec {

namespace {

constexpr int MODE_REL = 0;    // relevance, squared row norms of A taken in the same pass
constexpr int MODE_LMH = 1;
constexpr int MODE_RELP = 2;   // relevance with the rows' inverse norms prepared by the caller
constexpr bool is_rel(int mode) { return mode != MODE_LMH; }
constexpr float kLog2e = 1.4426950408889634f;

template <int MB, int NBX, int RB>
struct Geo {
  static_assert(RB == 256 || RB == 512, "row bytes per stage");
  static constexpr int kKSteps = RB / 64;                  // 32-deep MFMA steps per stage
  static constexpr int kRowsPerInstr = 1024 / RB;          // rows one copy instruction covers
  static constexpr int kLanesPerRow = RB / 16;
  static constexpr int kAInstr = 16 * MB / kRowsPerInstr;  // A copy instructions per wave
  static constexpr int kXInstr = 16 * NBX / kRowsPerInstr / 4;   // X copy instructions per wave
  static constexpr int kInstrPerStage = kAInstr + kXInstr;
  static constexpr int kAWave = MB * 16 * RB;              // bytes of A per wave per stage
  static constexpr int kA = 4 * kAWave;
  static constexpr int kX = NBX * 16 * RB;
  static constexpr int kStage = kA + kX;
  // Two workgroups share a CU (80 KiB of LDS each): while one waits at its stage barrier or for
  // LDS, the other one issues copies and MFMAs.  Each gets as many ring slots as fit (at most
  // 8); the epilogue tile reuses the slot that has just been consumed.
  static constexpr int kWgPerCu = 2;
  static constexpr int kFit = (160 * 1024 / kWgPerCu) / kStage;
  static constexpr int kStages = kFit > 8 ? 8 : kFit;
  static constexpr int kRing = kStages * kStage;
  static constexpr int kRowsWg = 64 * MB;
  static constexpr int kZtStride = kRowsWg + 4;            // floats per column in the epilogue tile
  static constexpr int kZt = 16 * NBX * kZtStride * 4;     // bytes
};

struct Cursor {
  int task;   // global task index (strided by gridDim.x)
  int kc;     // chunk within the task
  int cb;     // batch whose row count is cached in cn (-1: none); consecutive tasks of a
  int cn;     // workgroup mostly share the batch, so the device read happens once per batch
};

template <int MODE>
LVS_DEV void decode_task(const GemmKernelArgs& p, int task, int& b, int& rb, int& ds) {
  if (is_rel(MODE)) {
    ds = task % p.n_ds;
    const int t2 = task / p.n_ds;
    rb = t2 % p.n_rb;
    b = t2 / p.n_rb;
  } else {
    ds = 0;
    rb = task;
    b = 0;
  }
}

template <int MODE>
LVS_DEV int rows_of(const GemmKernelArgs& p, Cursor& c, int b) {
  if (is_rel(MODE)) {
    if (b != c.cb) {
      const int n = __builtin_amdgcn_readfirstlane(p.n_rows_dev[b]);
      c.cb = b;
      c.cn = n < p.n_rows ? n : p.n_rows;
    }
    return c.cn;
  }
  return p.n_rows;
}

// skip tasks whose row block lies beyond the valid rows of their batch
template <int MODE, int ROWS_WG>
LVS_DEV void settle(const GemmKernelArgs& p, Cursor& c) {
  if (is_rel(MODE)) {
    while (c.task < p.n_tasks) {
      int b, rb, ds;
      decode_task<MODE>(p, c.task, b, rb, ds);
      if (rb * ROWS_WG < rows_of<MODE>(p, c, b)) break;
      c.task += gridDim.x;
    }
  }
}

template <int MODE, int ROWS_WG>
LVS_DEV void advance(const GemmKernelArgs& p, Cursor& c) {
  if (++c.kc == p.kc) {
    c.kc = 0;
    c.task += gridDim.x;
    settle<MODE, ROWS_WG>(p, c);
  }
}

// Per-lane source pointers of the task the issue cursor is in: computed once per task, so that a
// stage costs one 64-bit add per copy instruction instead of a multiply-add chain.
//
// Copy geometry: one instruction moves 1 KiB = kRowsPerInstr rows x RB bytes; lane l handles
// row (l / kLanesPerRow) of the instruction at LDS chunk position cpos = l % kLanesPerRow and
// fetches the global chunk cpos ^ (row & 15) of the stage's RB-byte row segment (the XOR stays
// inside a 256-byte half, so MFMA operand reads of 16 rows at one logical chunk hit 16
// different bank groups).
template <int MB, int NBX, int RB>
struct IssuePtrs {
  const uint8_t* arow[Geo<MB, NBX, RB>::kAInstr];   // A row of copy instruction j at the task's first column
  const uint8_t* xcol[Geo<MB, NBX, RB>::kXInstr];   // X row of copy instruction k
  int rot;                                          // task mod chunks per task: first chunk read
};

template <int MODE, int MB, int NBX, int RB>
LVS_DEV void setup_task(const GemmKernelArgs& p, Cursor& c, IssuePtrs<MB, NBX, RB>& ip,
                        int wave, int lane) {
  using G = Geo<MB, NBX, RB>;
  if (c.task >= p.n_tasks) return;
  int b, rb, ds;
  decode_task<MODE>(p, c.task, b, rb, ds);
  const int n_rows = rows_of<MODE>(p, c, b);
  ip.rot = c.task % p.kc;
  const int rsub = lane / G::kLanesPerRow;
  const int cpos = lane % G::kLanesPerRow;
  const int64_t col_byte = (int64_t)ds * p.kc * RB;
  const uint8_t* abase = p.a + (int64_t)b * p.a_sb + col_byte;
  const int row0 = rb * G::kRowsWg + wave * 16 * MB;
#pragma unroll
  for (int j = 0; j < G::kAInstr; ++j) {
    const int rl = G::kRowsPerInstr * j + rsub;      // row within the wave's tile
    int row = row0 + rl;
    row = row < n_rows ? row : n_rows - 1;
    ip.arow[j] = abase + (int64_t)row * p.a_sr + ((cpos ^ (rl & 15)) << 4);
  }
#pragma unroll
  for (int k = 0; k < G::kXInstr; ++k) {
    const int jx = 4 * k + wave;
    const int cl = G::kRowsPerInstr * jx + rsub;     // LDS row of this lane in the X tile
    const int col = cl < p.n_cols ? cl : p.n_cols - 1;
    int xb, xi;
    if (is_rel(MODE)) {
      xb = b;
      xi = col;
    } else {
      xb = col / p.gamma;
      xi = col - xb * p.gamma;
    }
    ip.xcol[k] = p.x + (int64_t)xb * p.x_sb + (int64_t)xi * p.x_sg + col_byte +
                 ((cpos ^ (cl & 15)) << 4);
  }
}

// Stage kc of a task reads column chunk (kc + task) mod n_chunks of its slice: the workgroups
// walk the hidden dimension from different starting points, so at any moment their row
// segments spread over all HBM channels (with a power-of-two row pitch, e.g. d = 8192, all
// rows of a column chunk fall into the same few channels).  The order is a fixed function of
// the task, so results stay reproducible.
template <int MB, int NBX, int RB>
LVS_DEV void issue_stage(const IssuePtrs<MB, NBX, RB>& ip, int kc, int n_chunks, uint32_t slot,
                         int wave) {
  using G = Geo<MB, NBX, RB>;
  int chunk = kc + ip.rot;
  chunk = chunk >= n_chunks ? chunk - n_chunks : chunk;
  const int64_t off = (int64_t)chunk * RB;
#pragma unroll
  for (int j = 0; j < G::kAInstr; ++j) dma16(ip.arow[j] + off, slot + wave * G::kAWave + j * 1024);
#pragma unroll
  for (int k = 0; k < G::kXInstr; ++k)
    dma16<kCopyDefault>(ip.xcol[k] + off, slot + G::kA + (4 * k + wave) * 1024);
}

// advance the issue cursor; recompute the source pointers when it enters a new task
template <int MODE, int MB, int NBX, int RB>
LVS_DEV void advance_issue(const GemmKernelArgs& p, Cursor& c, IssuePtrs<MB, NBX, RB>& ip,
                           int wave, int lane) {
  using G = Geo<MB, NBX, RB>;
  if (++c.kc == p.kc) {
    c.kc = 0;
    c.task += gridDim.x;
    settle<MODE, G::kRowsWg>(p, c);
    setup_task<MODE, MB, NBX, RB>(p, c, ip, wave, lane);
  }
}

// wait until at most `ahead` whole stages (IPS copy instructions each) of this wave are still
// outstanding; ahead is uniform and in [0, MAXA]
template <int IPS, int MAXA>
LVS_DEV void wait_stages(int ahead) {
  if constexpr (MAXA <= 0) {
    wait_copies<0>();
  } else {
    if (ahead >= MAXA) {
      wait_copies<(IPS * MAXA > 63 ? 63 : IPS * MAXA)>();
    } else {
      wait_stages<IPS, MAXA - 1>(ahead);
    }
  }
}

template <int MODE, int MB, int NBX, int RB>
__global__ __launch_bounds__(256, 2) void gemm_stream_kernel(const GemmKernelArgs p) {
  using G = Geo<MB, NBX, RB>;
  extern __shared__ __align__(16) uint8_t smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n16 = lane & 15;
  const int g4 = lane >> 4;
  const uint32_t ring = lds_addr(smem);

  // operand chunk 4*ks + g4 of row n16, for ks = 0..3; steps 4..7 (RB = 512) sit 256 bytes on
  uint32_t oaddr[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) oaddr[i] = n16 * RB + (((4 * i + g4) ^ n16) << 4);

  f32x4 acc[MB][NBX];
  f32x4 accn[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    accn[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nx = 0; nx < NBX; ++nx) acc[mb][nx] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  Cursor cc{(int)blockIdx.x, 0, -1, 0};   // compute cursor
  settle<MODE, G::kRowsWg>(p, cc);
  Cursor ic = cc;                  // issue cursor
  IssuePtrs<MB, NBX, RB> ip;
  setup_task<MODE, MB, NBX, RB>(p, ic, ip, wave, lane);
  int ahead = -1;                  // stages issued beyond the one about to be consumed
  wait_copies<0>();
#pragma unroll
  for (int s = 0; s < G::kStages - 1; ++s) {
    if (ic.task < p.n_tasks) {
      issue_stage<MB, NBX, RB>(ip, ic.kc, p.kc, ring + s * G::kStage, wave);
      advance_issue<MODE, MB, NBX, RB>(p, ic, ip, wave, lane);
      ++ahead;
    }
  }

  int slot_c = 0;    // ring slot of the stage being consumed
  while (cc.task < p.n_tasks) {
    const uint32_t slot = ring + slot_c * G::kStage;
    // epilogue tile: the slot being consumed is free from the last operand read of this
    // iteration until the next iteration's barrier
    float* zt = reinterpret_cast<float*>(smem + slot_c * G::kStage);
    wait_stages<G::kInstrPerStage, G::kStages - 2>(ahead);
    __builtin_amdgcn_s_barrier();
    // refill the slot consumed in the previous iteration (it + kStages - 1 lands there)
    if (ic.task < p.n_tasks) {
      const int slot_i = slot_c == 0 ? G::kStages - 1 : slot_c - 1;
      issue_stage<MB, NBX, RB>(ip, ic.kc, p.kc, ring + slot_i * G::kStage, wave);
      advance_issue<MODE, MB, NBX, RB>(p, ic, ip, wave, lane);
    } else {
      ahead -= 1;
    }
    // ---- operands from LDS, four 32-deep steps at a time -------------------------------------
#pragma unroll
    for (int half = 0; half < G::kKSteps / 4; ++half) {
      u32x4 aop[MB][4];
      u32x4 xop[NBX][4];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        uint32_t a[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          a[ks] = slot + wave * G::kAWave + mb * 16 * RB + half * 256 + oaddr[ks];
        lds_read4(aop[mb], a);
      }
#pragma unroll
      for (int nx = 0; nx < NBX; ++nx) {
        uint32_t a[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
          a[ks] = slot + G::kA + nx * 16 * RB + half * 256 + oaddr[ks];
        lds_read4(xop[nx], a);
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
          for (int nx = 0; nx < NBX; ++nx)
            acc[mb][nx] = mfma16(aop[mb][ks], xop[nx][ks], acc[mb][nx]);
          if (MODE == MODE_REL) accn[mb] = mfma16(aop[mb][ks], aop[mb][ks], accn[mb]);
        }
      }
    }
    // ---- end of a task: epilogue -----------------------------------------------------------
    if (cc.kc == p.kc - 1) {
      int b, rb, ds;
      decode_task<MODE>(p, cc.task, b, rb, ds);
      const int row0 = rb * G::kRowsWg;
      if (is_rel(MODE)) {
        // acc[mb][nx][i] = dot(A row row0 + wave*16*MB + 16*mb + 4*g4 + i, X column 16*nx + n16)
#pragma unroll
        for (int nx = 0; nx < NBX; ++nx) {
          const int col = 16 * nx + n16;
          if (col < p.gamma) {
            float* dp = p.dots + (((int64_t)b * p.n_ds + ds) * p.gamma + col) * p.ld + row0 +
                        wave * 16 * MB + 4 * g4;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) *reinterpret_cast<f32x4*>(dp + 16 * mb) = acc[mb][nx];
          }
        }
        // squared norms sit on the diagonal of A A^T: lane (n16, g4 == n16/4), element n16 % 4
        if (MODE == MODE_REL && g4 == (n16 >> 2)) {
          float* np = p.nv2 + ((int64_t)b * p.n_ds + ds) * p.ld + row0 + wave * 16 * MB + n16;
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) {
            const int e = n16 & 3;
            const float v = e == 0 ? accn[mb][0] : e == 1 ? accn[mb][1] : e == 2 ? accn[mb][2]
                                                                                 : accn[mb][3];
            np[16 * mb] = v;
          }
        }
      } else {
        const int n_rows = p.n_rows;
        // the tile overlays the slot just consumed: every wave must be done reading operands
        __builtin_amdgcn_s_barrier();
        // logits tile to LDS as [column][row]
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int nx = 0; nx < NBX; ++nx)
            *reinterpret_cast<f32x4*>(zt + (16 * nx + n16) * G::kZtStride + wave * 16 * MB +
                                      16 * mb + 4 * g4) = acc[mb][nx];
        __syncthreads();
        if (p.logits != nullptr) {
          for (int idx = threadIdx.x; idx < p.n_cols * G::kRowsWg; idx += 256) {
            const int col = idx / G::kRowsWg;
            const int r = idx - col * G::kRowsWg;
            if (row0 + r < n_rows)
              p.logits[(int64_t)col * n_rows + row0 + r] = zt[col * G::kZtStride + r];
          }
        }
        // per column: block maximum, sum of exponentials and the k best (value, id) pairs, by
        // wave-wide reductions over the DPP lane network (lane l holds rows l and l + 64)
        for (int col = wave; col < p.n_cols; col += 4) {
          float v[MB];
          uint64_t key[MB];
          float mx = -INFINITY;
#pragma unroll
          for (int j = 0; j < MB; ++j) {
            const int r = lane + 64 * j;
            const bool on = row0 + r < n_rows;
            v[j] = on ? zt[col * G::kZtStride + r] : -INFINITY;
            key[j] = (on && v[j] != -INFINITY) ? cand_key(v[j], row0 + r) : 0ull;
            mx = fmaxf(mx, v[j]);
          }
          mx = wave_max(mx);
          float se = 0.f;
#pragma unroll
          for (int j = 0; j < MB; ++j) se += fast_exp2((v[j] - mx) * kLog2e);
          se = wave_sum(se);
          const int64_t rec = (int64_t)cc.task * p.n_cols + col;
          if (lane == 0) {
            p.stats[rec * 2] = mx;
            p.stats[rec * 2 + 1] = se;
          }
          if (p.stats_z != nullptr) {   // sum exp(z - max) * z, for the row entropy
            float sz = 0.f;
#pragma unroll
            for (int j = 0; j < MB; ++j)
              sz += v[j] == -INFINITY ? 0.f : fast_exp2((v[j] - mx) * kLog2e) * v[j];
            sz = wave_sum(sz);
            if (lane == 0) p.stats_z[rec] = sz;
          }
          uint64_t mine = 0;   // lane r keeps the r-th best
          for (int r = 0; r < p.topk; ++r) {
            uint64_t best = key[0];
#pragma unroll
            for (int j = 1; j < MB; ++j) best = key[j] > best ? key[j] : best;
            const uint64_t w = wave_max_u64(best);
#pragma unroll
            for (int j = 0; j < MB; ++j) key[j] = key[j] == w ? 0ull : key[j];
            mine = lane == r ? w : mine;
          }
          if (lane < p.topk) {
            p.cand_val[rec * p.topk + lane] =
                mine ? key_value((uint32_t)(mine >> 32)) : -INFINITY;
            p.cand_idx[rec * p.topk + lane] = mine ? 0x7fffffff - (int)(uint32_t)mine : -1;
          }
        }
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        accn[mb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nx = 0; nx < NBX; ++nx) acc[mb][nx] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
    advance<MODE, G::kRowsWg>(p, cc);
    slot_c = slot_c + 1 == G::kStages ? 0 : slot_c + 1;
  }
}

template <int MODE, int MB, int NBX, int RB>
hipError_t launch_gemm(const GemmKernelArgs& a, int num_cu, hipStream_t stream) {
  using G = Geo<MB, NBX, RB>;
  static_assert(G::kZt <= G::kStage, "epilogue tile must fit in one ring slot");
  static_assert(G::kStages >= 2, "ring too small");
  static_assert(G::kInstrPerStage * (G::kStages - 2) <= 63, "copy counter range");
  const size_t lds = (size_t)G::kRing;
  static LdsLimitOnce lds_limit;
  hipError_t e = lds_limit.ensure(
      reinterpret_cast<const void*>(&gemm_stream_kernel<MODE, MB, NBX, RB>), lds);
  if (e != hipSuccess) return e;
  // As many workgroups as fit at once, then trimmed so that every workgroup walks the same
  // number of tasks (1188 tasks on 512 slots: 396 workgroups x 3 instead of 164 doing a third
  // task while 348 sit idle).  The kernel is bandwidth-bound, so a few idle CUs cost nothing.
  const int slots = num_cu * G::kWgPerCu;
  int grid = a.n_tasks < slots ? a.n_tasks : slots;
  if (grid < 1) grid = 1;
  const int rounds = (a.n_tasks + grid - 1) / grid;
  if (rounds > 0) grid = (a.n_tasks + rounds - 1) / rounds;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL((gemm_stream_kernel<MODE, MB, NBX, RB>), dim3(grid), dim3(256), lds, stream,
                     a);
  return hipGetLastError();
}

}  // namespace

int rel_rows_per_block(int big) { return big ? Geo<2, 1, 256>::kRowsWg : Geo<1, 1, 256>::kRowsWg; }
int lmh_rows_per_block(int n_cols, int64_t row_pitch_bytes, int64_t n_rows, int topk) {
  if (n_cols > 32) return Geo<1, 4, 256>::kRowsWg;
  // twice the row blocks are twice the top-k candidates: stay within what the merge kernel
  // keeps in registers (V = 152064: k <= 8)
  const int64_t blocks64 = (n_rows + Geo<1, 1, 256>::kRowsWg - 1) / Geo<1, 1, 256>::kRowsWg;
  if (blocks64 * topk > kAcceptRegCandidates) return Geo<2, 1, 256>::kRowsWg;
  // Up to 32 columns: 64-row tasks with a three- or four-slot ring stream 2-4 % faster than
  // 128-row tasks with two slots (d = 2048 .. 7168), except at row pitches that are multiples
  // of 8 KiB (d = 4096, 8192), where the 64 segments of a stage fall into too few HBM channels
  // (d = 4096, five columns: 5.6 against 6.4 TB/s).
  return row_pitch_bytes % 8192 == 0 ? Geo<2, 1, 256>::kRowsWg : Geo<1, 1, 256>::kRowsWg;
}

template <int MODE>
static hipError_t launch_rel_mode(const GemmKernelArgs& a, int num_cu, hipStream_t stream) {
  if (a.row_bytes == 512) return launch_gemm<MODE, 1, 1, 512>(a, num_cu, stream);
  const bool big = a.rows_per_block == Geo<2, 1, 256>::kRowsWg;
  if (a.n_cols <= 16)
    return big ? launch_gemm<MODE, 2, 1, 256>(a, num_cu, stream)
               : launch_gemm<MODE, 1, 1, 256>(a, num_cu, stream);
  return big ? launch_gemm<MODE, 2, 2, 256>(a, num_cu, stream)
             : launch_gemm<MODE, 1, 2, 256>(a, num_cu, stream);
}

// nv2 == nullptr: the caller prepared the rows' inverse norms, the pass takes dot products only
hipError_t launch_rel_gemm(const GemmKernelArgs& a, int num_cu, hipStream_t stream) {
  return a.nv2 != nullptr ? launch_rel_mode<MODE_REL>(a, num_cu, stream)
                          : launch_rel_mode<MODE_RELP>(a, num_cu, stream);
}

hipError_t launch_lmh_gemm(const GemmKernelArgs& a, int num_cu, hipStream_t stream) {
  // The task size is the planner's (it sized the partial results by it): 64-row tasks for
  // 33..64 columns (the wider X slice then still leaves two ring slots for each of the two
  // workgroups of a CU) and, unless the row pitch speaks against it, for up to 16 columns;
  // 128-row tasks otherwise.
  if (a.rows_per_block == Geo<1, 1, 256>::kRowsWg) {
    if (a.n_cols <= 16) return launch_gemm<MODE_LMH, 1, 1, 256>(a, num_cu, stream);
    if (a.n_cols <= 32) return launch_gemm<MODE_LMH, 1, 2, 256>(a, num_cu, stream);
    if (a.n_cols <= 48) return launch_gemm<MODE_LMH, 1, 3, 256>(a, num_cu, stream);
    if (a.n_cols <= 64) return launch_gemm<MODE_LMH, 1, 4, 256>(a, num_cu, stream);
    return hipErrorInvalidValue;
  }
  if (a.n_cols <= 16) return launch_gemm<MODE_LMH, 2, 1, 256>(a, num_cu, stream);
  if (a.n_cols <= 32) return launch_gemm<MODE_LMH, 2, 2, 256>(a, num_cu, stream);
  return hipErrorInvalidValue;
}

}  // namespace lvspec
