// Steps 2 and 3 of Section 5 in one kernel, for layers with m = 2 and few input channels (the 5x5
// layer of Section 6: 48 channels per group): the per-position products never leave the CU.
//
// Section 5 gives each core its own images through all three steps and remarks that this lets steps
// 2 and 3 run fused, out of cache.  The same decomposition here: a workgroup owns one block of 64
// tiles and 64 rows of W_F (output channels) for ALL positions.  Per position it stages the
// C x 64 panel V[p][:, block] and its own rows' weights in LDS, every wave multiplies its four rows
// as in the stand-alone product kernel (quarter waves, four tiles per lane), and the result - the
// lane's four values of M[p][k][.] - is folded straight into the lane's m x m output accumulators,
//     Y[a][b] += A^T[a][i] * A^T[b][j] * M[(i,j)]     (p = i*t + j),
// column factor first (compile-time j), row factor once per i.  With m = 2 that is 16 accumulators
// per lane; M (t^2/m^2 = 9 times the output for F(2x2,5x5)) is never written or read.
//
// Memory pipeline: the panel and the weights of a position form one package; a thread carries its
// 16-byte pieces of the next D packages in registers (D = t, or t/2 for the wider panels), so D
// packages per workgroup are in flight while one is computed, and writes the oldest to the LDS
// buffer that is not being read (two buffers, one barrier per position).  All vector-memory
// loads of the loop are package loads in program order, so waiting for the oldest never waits for
// a younger one; the weights are read from LDS, not from memory, for the same reason.
#pragma once
#include "swconv_kernels.hpp"

namespace swconv {

// Where the m x m outputs of a tile go (host-built, one entry per tile of the padded tile range).
struct OutTile {
  uint32_t n;      // image
  uint32_t pix;    // (ty*m)*Wo + tx*m: offset of the tile's first pixel inside an output plane
  uint32_t valid;  // rows (low 16 bits) and columns (high 16 bits) of the tile inside Ho x Wo; 0 = padding tile
  uint32_t pad;
};

constexpr int kFusedWaves = 16;                          // waves per workgroup: one slice (4 rows) each
constexpr int kFusedRows = kFusedWaves * kSliceRows;     // rows of W_F per workgroup
constexpr int kFusedMaxBatches = 2;                      // 16-step weight batches per slice and position
constexpr int kFusedMaxPieces = 2;                       // 16-byte panel pieces per thread: C <= 128

// A^T[a][i] of F(2, R): row 0 = (1, ..., 1, 0), row 1 = (0, 1, -1, -1) or (0, 1, -1, 2, -2, 1).
template <int R>
__device__ __forceinline__ float at_coef(int a, int i) {
  if (a == 0) return i < R ? 1.0f : 0.0f;
  if constexpr (R == 3)
    return i == 0 ? 0.0f : i == 1 ? 1.0f : -1.0f;
  else
    return i == 0 ? 0.0f : i == 1 ? 1.0f : i == 2 ? -1.0f : i == 3 ? 2.0f : i == 4 ? -2.0f : 1.0f;
}

__device__ __forceinline__ void acc_add(Acc4& y, const Acc4& x) {
  y.a0 += x.a0; y.a1 += x.a1; y.a2 += x.a2; y.a3 += x.a3;
}
__device__ __forceinline__ void acc_fma(Acc4& y, float c, const Acc4& x) {
  y.a0 = fmaf(c, x.a0, y.a0); y.a1 = fmaf(c, x.a1, y.a1); y.a2 = fmaf(c, x.a2, y.a2); y.a3 = fmaf(c, x.a3, y.a3);
}

// Weight packages: wpk[p][kc][b][wave] = one 512-byte batch in the stream layout of the product
// kernel ([q][s] -> (row byte offset in the panel, weight) of row kc*64 + wave*4 + q, step 16 b + s),
// rows in their natural order.  lens[p][kc*16 + wave] = steps of that slice (a multiple of 4, at
// most 16 B).  Grid: n_wgs = tile blocks * KC workgroups of 1024 threads;
// LDS: 2 * (C * 256 + 16 * B * 512) + 1024 bytes.
template <int R, int PP>
__global__ __launch_bounds__(kFusedWaves * 64) void product_output_kernel(
    const float* __restrict__ V, float* __restrict__ out, const uint32_t* __restrict__ wpk, uint32_t wpk_bytes,
    const uint8_t* __restrict__ lens, const OutTile* __restrict__ otiles, int C, int K, int Tp, int KC, int B,
    int n_wgs, uint32_t v_bytes, uint32_t plane, int Wo, uint32_t out_image_stride, uint32_t out_bytes) {
  constexpr int t = R + 1, P = t * t, NW = kFusedWaves, NT = NW * 64, TB = kTileBlock;
  constexpr int D = PP == 1 ? t : t / 2;  // packages in flight; divides t, so a package's slot is known from j
  static_assert(t % D == 0 && t % 2 == 0 && P <= 64, "slot and buffer of a package follow from j; one lane per position");
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  constexpr uint32_t kParked = 0xfffffff0u;  // past the end of every buffer: reads 0, touches no memory
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int quarter = lane >> 4;
  const uint32_t lane_sub = (uint32_t)(lane & 15) * 16u;
  const int vid = xcd_contiguous_id(blockIdx.x, n_wgs);  // the KC workgroups of a tile block are neighbours on one XCD
  const int tb = vid / KC, kc = vid - tb * KC;
  const uint32_t panel_bytes = (uint32_t)C * TB * 4u, w_bytes = (uint32_t)NW * B * 512u;
  const uint32_t buf_floats = (panel_bytes + w_bytes) / 4u;
  const __amdgpu_buffer_rsrc_t vr = make_rsrc(V, v_bytes), wr = make_rsrc(wpk, wpk_bytes);

  // the lane's view of the slice lengths: lane l holds the length at position l
  const int spp = KC * NW;
  const int lens_v = lane < P ? (int)lens[(size_t)lane * spp + kc * NW + wave] : 0;

  uint32_t voff[PP];
#pragma unroll
  for (int u = 0; u < PP; ++u) {
    const int idx = threadIdx.x + u * NT;
    voff[u] = idx < C * (TB / 4) ? ((uint32_t)(idx / (TB / 4)) * Tp + (idx % (TB / 4)) * 4) * 4u : kParked;
  }
  const uint32_t woff = threadIdx.x * 16u < w_bytes ? threadIdx.x * 16u : kParked;

  u32x4_t ring_v[D][PP], ring_w[D];
  auto issue = [&](u32x4_t (&pv)[PP], u32x4_t& pw, int p) {  // package p -> registers; nothing is read for p >= P
    const bool live = p < P;
    const uint32_t vs = live ? ((uint32_t)p * C * Tp + (uint32_t)tb * TB) * 4u : 0u;
    const uint32_t ws = live ? ((uint32_t)p * KC + kc) * w_bytes : 0u;
#pragma unroll
    for (int u = 0; u < PP; ++u)
      pv[u] = __builtin_amdgcn_raw_buffer_load_b128(vr, (int)(live ? voff[u] : kParked), (int)vs, 0);
    pw = __builtin_amdgcn_raw_buffer_load_b128(wr, (int)(live ? woff : kParked), (int)ws, 0);
  };
  // registers -> LDS buffer `half`.  Threads without a piece write their (zero) registers to a
  // spare 16 bytes per lane behind the buffers: with unconditional writes the compiler cannot move a
  // load into a branch next to its use, where it would have to be waited for at once.
  float* const spare = lds + (size_t)2 * buf_floats + lane * 4;
  auto write = [&](const u32x4_t (&pv)[PP], const u32x4_t& pw, int half) {
    float* buf = lds + (size_t)half * buf_floats;
#pragma unroll
    for (int u = 0; u < PP; ++u) {
      const int idx = threadIdx.x + u * NT;
      *reinterpret_cast<u32x4_t*>(idx < C * (TB / 4) ? buf + idx * 4 : spare) = pv[u];
    }
    *reinterpret_cast<u32x4_t*>(threadIdx.x * 16u < w_bytes ? buf + panel_bytes / 4u + threadIdx.x * 4 : spare) = pw;
  };

  // the packages go out in order (the waits below count on it)
#pragma unroll
  for (int s = 0; s < D; ++s) {
    issue(ring_v[s], ring_w[s], s);
    __builtin_amdgcn_sched_barrier(0);
  }
  write(ring_v[0], ring_w[0], 0);
  __builtin_amdgcn_sched_barrier(0);
  issue(ring_v[0], ring_w[0], D);
  __builtin_amdgcn_sched_barrier(0);

  Acc4 y00 = {0.0f, 0.0f, 0.0f, 0.0f}, y01 = y00, y10 = y00, y11 = y00;  // Y[a][b] of the lane's four tiles
  for (int i = 0; i < t; ++i) {
    Acc4 r0 = {0.0f, 0.0f, 0.0f, 0.0f}, r1 = r0;  // sum_j A^T[b][j] M[(i,j)], b = 0, 1
#pragma unroll
    for (int j = 0; j < t; ++j) {
      const int p = i * t + j;
      // package p is in buffer j % 2 (t is even); every wave is done with the other buffer
      __syncthreads();
      write(ring_v[(j + 1) % D], ring_w[(j + 1) % D], (j + 1) & 1);   // package p + 1
      issue(ring_v[(j + 1) % D], ring_w[(j + 1) % D], p + 1 + D);
      const int len = __builtin_amdgcn_readlane(lens_v, p);
      Acc4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
      if (len > 0) {
        const float* panel = lds + (size_t)(j & 1) * buf_floats;
        const char* wb = reinterpret_cast<const char*>(panel) + panel_bytes + wave * 512 + lane * 8;
        for (int b = 0, rem = len; rem > 0; ++b, rem -= kBatchSteps) {
          const u32x2_t batch = *reinterpret_cast<const u32x2_t*>(wb + b * (NW * 512));
          quarter_batch(panel, lane_sub, batch, rem, acc);
        }
      }
      const float c0 = at_coef<R>(0, j), c1 = at_coef<R>(1, j);  // constants after unrolling
      if (c0 != 0.0f) acc_add(r0, acc);                          // A^T[0][j] is 0 or 1
      if (c1 != 0.0f) acc_fma(r1, c1, acc);
    }
    const float a0 = at_coef<R>(0, i), a1 = at_coef<R>(1, i);
    acc_fma(y00, a0, r0);
    acc_fma(y01, a0, r1);
    acc_fma(y10, a1, r0);
    acc_fma(y11, a1, r1);
  }

  // Epilogue.  The four OutTile entries of the lane are fetched together; the stores go through a
  // descriptor over the whole output tensor, so a lane with nothing to store (padding row or tile,
  // pixel outside Ho x Wo) parks its offset past the end instead of branching.  A pair of
  // horizontally adjacent pixels is one 8-byte store.
  const int k = kc * kFusedRows + wave * kSliceRows + quarter;
  const __amdgpu_buffer_rsrc_t orr = make_rsrc(out, out_bytes);
  const u32x4_t* ot = reinterpret_cast<const u32x4_t*>(otiles + (size_t)tb * TB + (lane & 15) * 4);
  const u32x4_t o0 = ot[0], o1 = ot[1], o2 = ot[2], o3 = ot[3];  // (n, pix, valid, -)
  const uint32_t krow = k < K ? (uint32_t)k * plane : 0u;
  auto store_tile = [&](const u32x4_t& o, float v00, float v01, float v10, float v11) {
    const int rows = k < K ? (int)(o.z & 0xffffu) : 0, cols = (int)(o.z >> 16);
    const uint32_t at = (o.x * (uint32_t)out_image_stride + krow + o.y) * 4u;
    const uint32_t pair = cols > 1 ? at : kParked, single = cols == 1 ? at : kParked;
    buffer_store_f32x2<SWCONV_AUX_OUT>(orr, rows > 0 ? pair : kParked, 0u, v00, v01);
    buffer_store_f32<SWCONV_AUX_OUT>(orr, rows > 0 ? single : kParked, 0u, v00);
    const uint32_t below = (uint32_t)Wo * 4u;  // added to live offsets only: a parked one must not wrap around
    buffer_store_f32x2<SWCONV_AUX_OUT>(orr, rows > 1 && cols > 1 ? at + below : kParked, 0u, v10, v11);
    buffer_store_f32<SWCONV_AUX_OUT>(orr, rows > 1 && cols == 1 ? at + below : kParked, 0u, v10);
  };
  store_tile(o0, y00.a0, y01.a0, y10.a0, y11.a0);
  store_tile(o1, y00.a1, y01.a1, y10.a1, y11.a1);
  store_tile(o2, y00.a2, y01.a2, y10.a2, y11.a2);
  store_tile(o3, y00.a3, y01.a3, y10.a3, y11.a3);
}

// ---------------------------------------------------------------------------------------------
// Steps 2 and 3 in one kernel for F(4x4,3x3) (t = 6, P = 36, 16 outputs per tile and row).
//
// Same decomposition as above - a workgroup of 16 waves owns one 64-tile block and 64 rows of W_F
// through all 36 positions, a wave four rows, a lane one row and four tiles - with the memory side
// rebuilt around the register file: the lane's 4 x 16 output accumulators and the 16 row sums take
// 80 of the 128 vector registers a wave has at 16 waves per CU.
//   - The C x 64 panel of a position goes from memory straight into LDS (16-byte direct loads:
//     the 64 lanes of a load fill 1024 consecutive bytes of LDS = four panel rows), two panel
//     buffers, one barrier per position: the panel of position p + 1 arrives while p is computed.
//     The two buffers are two separate arrays, which is what lets the compiler see that work on
//     one never has to wait for a direct load into the other.
//   - The weights do not pass through LDS: a lane fetches its own (row offset, weight) pairs, 16
//     steps per load.  Two sets of two batch registers in turn: while a position runs on one set,
//     the other receives the first two batches of the next position, a whole position ahead.
//   - Inner loop: the steps of a slice run as one rolling pipeline - the panel read of step s + 4
//     is issued right after the multiply-adds of step s, so a wave always has four LDS reads in
//     flight.  With the waves of a workgroup re-aligned by the barrier of every position, reads
//     issued group by group would leave LDS idle while all waves multiply and the vector ALU idle
//     while all wait.  A unit of the pipeline is two batches (32 steps), written in assembly
//     with fixed registers for the four reads in flight, and left after the slice's last group of
//     four steps.
//   - The fold Y += A^T[.][i] (x) sum_j A^T[.][j] M[(i,j)] runs per position on the lane's four
//     values (column factor) and once per row of positions (row factor).
//   - Epilogue: the 4 x 4 outputs go through LDS (the panels are done with) into the layout of the
//     output rows, one row of W_F at a time per wave, and leave as whole rows with lane-contiguous
//     stores, as in the stand-alone output transform.
// M (36 floats per output tile and row; 16 are stored) never exists in memory.
//
// Requires C % 4 == 0 (a direct load covers four whole rows), C <= 256 (the two panel arrays) and
// an output staging area of at most 2048 floats per wave.  G = ceil(C / 64) direct loads per wave
// and panel; a wave with fewer row groups than G repeats the panel's first group.
// Weight packages: wpk[p][kc][b][wave], B batches per slice and position (B even: whole units);
// lens[p][kc*16 + wave] = steps of the slice (a multiple of 4).

constexpr int kFused4MaxBatches = 14;  // steps of a slice must fit the 8-bit length table
constexpr int kFused4MaxC = 256;       // rows of a panel array
constexpr int kFused4MaxOutArea = kFused4MaxC * kTileBlock / (kFusedWaves / 2);  // floats per wave: eight waves per array

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// The rolling unit of the inner loop (unit_rolling_hi: its reads in flight live in v[112:127]) is
// defined in swconv_kernels.hpp.

// Row a of A^T of F(4,3) at column i: (1, p, p^2, p^3) for the points p = 0, 1, -1, 2, -2 and
// (0, 0, 0, 1) for the point at infinity (i = 5).
__device__ __forceinline__ void at_column(int i, float (&c)[4]) {
  const float pt = i == 1 ? 1.0f : i == 2 ? -1.0f : i == 3 ? 2.0f : i == 4 ? -2.0f : 0.0f;
  c[0] = i < 5 ? 1.0f : 0.0f;
  c[1] = pt;
  c[2] = pt * pt;
  c[3] = pt * pt * pt + (i == 5 ? 1.0f : 0.0f);
}

template <int R, int G>
__global__ __launch_bounds__(kFusedWaves * 64) void product_output4_kernel(
    const float* __restrict__ V, float* __restrict__ out, const uint32_t* __restrict__ wpk, uint32_t wpk_bytes,
    const uint8_t* __restrict__ lens, const TileInfo* __restrict__ tiles, const BlockImage* __restrict__ blocks,
    int KC, int B, int n_wgs, const Geometry g) {
  static_assert(R == 3, "F(4x4,3x3)");
  constexpr int t = R + 3, P = t * t, NW = kFusedWaves, TB = kTileBlock;
  static_assert(P <= 64 && P % 2 == 0, "one lane per position holds the slice length; positions run in pairs");
  static_assert(G >= 1 && (G - 1) * NW * 4 < kFused4MaxC, "G direct loads per wave cover up to 64 G rows");
  __shared__ __attribute__((aligned(1024))) float panel_even[kFused4MaxC * TB];  // panels of the even positions
  __shared__ __attribute__((aligned(1024))) float panel_odd[kFused4MaxC * TB];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int quarter = lane >> 4;
  const uint32_t lane_sub = (uint32_t)(lane & 15) * 16u;
  const int vid = xcd_contiguous_id(blockIdx.x, n_wgs);  // the KC workgroups of a tile block are neighbours on one XCD
  const int tb = vid / KC, kc = vid - tb * KC;
  const int C = g.C, Tp = g.Tp;
  const __amdgpu_buffer_rsrc_t wr = make_rsrc(wpk, wpk_bytes), vr = make_rsrc(V, g.v_bytes);

  // the lane's view of its wave's slice lengths: lane l holds the length at position l
  const int spp = KC * NW;
  const int lens_v = lane < P ? (int)lens[(size_t)lane * spp + kc * NW + wave] : 0;

  // Panel loads: load u of wave w moves the row group 16 u + w (rows 4 (16 u + w) .. + 3), or group
  // 0 again where the panel has no such group; lane l fetches piece l % 16 of row l / 16 of them.
  const uint32_t voff = ((uint32_t)(lane >> 4) * (uint32_t)Tp) * 4u + lane_sub;
  int group_of[G];
#pragma unroll
  for (int u = 0; u < G; ++u) group_of[u] = u * NW + wave < C / 4 ? u * NW + wave : 0;
  auto fetch_panel = [&](int p, float* dst) {
    const uint32_t soff = ((uint32_t)p * C * Tp + (uint32_t)tb * TB) * 4u;
#pragma unroll
    for (int u = 0; u < G; ++u)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(vr, (lds_ptr_t)(dst + group_of[u] * 256), 16, (int)voff,
                                               (int)(soff + (uint32_t)group_of[u] * (uint32_t)Tp * 16u), 0, 0);
  };

  // weight batches of this wave: position p, batch b at ((p KC + kc) B + b) * NW * 512 + wave * 512
  const uint32_t lane8 = (uint32_t)lane * 8u;
  const uint32_t pos_bytes = (uint32_t)KC * B * NW * 512u;
  const uint32_t w0 = ((uint32_t)kc * B * NW + wave) * 512u;
  constexpr uint32_t kBatchStride = NW * 512u;
  auto load_batch = [&](uint32_t byte_off) -> u32x2_t {
    return __builtin_amdgcn_raw_buffer_load_b64(wr, (int)lane8, (int)byte_off, 0);  // past the end: reads 0
  };

  Acc4 y[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) y[a][b] = Acc4{0.0f, 0.0f, 0.0f, 0.0f};
  Acc4 r0 = {0.0f, 0.0f, 0.0f, 0.0f}, r1 = r0, r2 = r0, r3 = r0;  // sum_j A^T[b][j] M[(i,j)], b = 0 .. 3

  // One position: its panel is in `panel`, its first two weight batches in (c0, c1); meanwhile the
  // panel of the next position goes into `other` and its first batches into (n0, n1).
  auto position = [&](int p, const float* panel, float* other, u32x2_t& c0, u32x2_t& c1, u32x2_t& n0, u32x2_t& n1) {
    // every wave has finished position p - 1 (which read the array that is filled next) and has
    // waited for its share of panel p
    __syncthreads();
    const uint32_t cur = (uint32_t)p * pos_bytes + w0;
    const uint32_t nxt = p + 1 < P ? cur + pos_bytes : 0xffff0000u;  // parked past the end after the last position
    if (p + 1 < P) fetch_panel(p + 1, other);
    n0 = load_batch(nxt);
    n1 = load_batch(nxt + kBatchStride);
    // an empty slice runs one group of steps on all-zero pairs: no branch around the pipeline
    const int len = max(__builtin_amdgcn_readlane(lens_v, p), kStepGroup);
    const int units = (len + kUnitSteps - 1) / kUnitSteps;
    const uint32_t lane_base = (uint32_t)(uintptr_t)(lds_ptr_t)panel + lane_sub;
    Acc4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    unit_rolling_hi(lane_base, c0, c1, min(len, kUnitSteps), acc);
    for (int u = 1; u < units; ++u) {  // a slice of more than 32 steps: further batches, fetched as they are needed
      const u32x2_t e0 = load_batch(cur + (uint32_t)(2 * u) * kBatchStride);
      const u32x2_t e1 = load_batch(cur + (uint32_t)(2 * u + 1) * kBatchStride);
      unit_rolling_hi(lane_base, e0, e1, min(len - u * kUnitSteps, kUnitSteps), acc);
    }
    // column j of A^T
    const int j = p % t;
    float cc[4];
    at_column(j, cc);
    acc_fma(r0, cc[0], acc);
    acc_fma(r1, cc[1], acc);
    acc_fma(r2, cc[2], acc);
    acc_fma(r3, cc[3], acc);
    if (j == t - 1) {  // row i of positions is complete: Y[a][b] += A^T[a][i] * r_b
      float rc[4];
      at_column(p / t, rc);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        acc_fma(y[a][0], rc[a], r0);
        acc_fma(y[a][1], rc[a], r1);
        acc_fma(y[a][2], rc[a], r2);
        acc_fma(y[a][3], rc[a], r3);
      }
      r0 = r1 = r2 = r3 = Acc4{0.0f, 0.0f, 0.0f, 0.0f};
    }
    // this wave's share of panel p + 1 is in LDS and the next batches are in their registers (both
    // were asked for a whole position ago)
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
  };

  fetch_panel(0, panel_even);
  u32x2_t ca0 = load_batch(w0), ca1 = load_batch(w0 + kBatchStride), cb0 = {0u, 0u}, cb1 = {0u, 0u};
  __builtin_amdgcn_s_waitcnt(0x0f70);
  for (int p = 0; p < P; p += 2) {
    position(p, panel_even, panel_odd, ca0, ca1, cb0, cb1);
    position(p + 1, panel_odd, panel_even, cb0, cb1, ca0, ca1);
  }

  // Epilogue.  Every wave has an LDS area laid out like the output rows its tile block covers (the
  // tables of the stand-alone output transform say where a tile's pixels go and which runs of whole
  // rows the block has in each image), eight waves per panel array.  Row by row of W_F: the 16
  // lanes of the row's quarter drop their 4 x 4 outputs there, then all 64 lanes write the runs out
  // with lane-contiguous stores.  LDS executes a wave's operations in order, so inside a wave no
  // barrier is needed.
  __syncthreads();  // every wave is done with the panels
  float* my = (wave < NW / 2 ? panel_even : panel_odd) + (size_t)(wave % (NW / 2)) * g.out_area;
  const TileInfo* ti = tiles + (size_t)tb * TB + (lane & 15) * 4;
  const TileInfo ti0 = ti[0], ti1 = ti[1], ti2 = ti[2], ti3 = ti[3];
  const BlockImage* bi = blocks + (size_t)tb * g.slots;
  const size_t plane = (size_t)g.Ho * g.Wo;
  for (int q = 0; q < kSliceRows; ++q) {
    const int k = kc * kFusedRows + wave * kSliceRows + q;  // wave-uniform
    if (k >= g.K) break;
    if (quarter == q) {
      auto drop = [&](const TileInfo& tile, auto pick) {
        const int y0 = (int16_t)(tile.yx0 & 0xffff), x0 = tile.yx0 >> 16;
        // rows / columns of the tile inside the output (<= 0 for a padding tile, whose y0 is -32768)
        const int rows = y0 == -32768 ? 0 : g.Ho - (y0 + g.pad), cols = g.Wo - (x0 + g.pad);
        float* px = my + tile.out_org;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
          for (int b = 0; b < 4; ++b)
            if (a < rows && b < cols) px[a * g.Wo + b] = pick(y[a][b]);
      };
      drop(ti0, [](const Acc4& v) { return v.a0; });
      drop(ti1, [](const Acc4& v) { return v.a1; });
      drop(ti2, [](const Acc4& v) { return v.a2; });
      drop(ti3, [](const Acc4& v) { return v.a3; });
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the drops are in LDS before any lane reads them
    for (int sidx = 0; sidx < g.slots; ++sidx) {
      const BlockImage b = bi[sidx];
      if (b.n < 0) continue;
      const float* src = my + b.out_off;
      float* dst = out + (size_t)b.n * g.out_image_stride + k * plane + b.out_elem0;
      // stores past the part's end are dropped by the descriptor: no lane predicate
      const __amdgpu_buffer_rsrc_t orr = make_rsrc(dst, (uint32_t)b.out_span * 4u);
      if (b.whole) {
        for (int e0 = 0; e0 < b.out_span; e0 += 64)
          buffer_store_f32<SWCONV_AUX_OUT>(orr, lane * 4u, e0 * 4u, src[e0 + lane]);
      } else {
        const int row_first = b.out_elem0 / g.Wo;  // wave-uniform
        for (int e0 = 0; e0 < b.out_span; e0 += 64) {
          const int e = e0 + lane;
          const int ry = (int)__umulhi((uint32_t)e, g.wo_magic), x = e - ry * g.Wo;
          const int tl = ((row_first + ry) >> g.m_shift) * g.tw + (x >> g.m_shift);
          const bool mine = tl >= b.t_lo && tl <= b.t_hi;  // a pixel of a tile of this block
          buffer_store_f32<SWCONV_AUX_OUT>(orr, mine ? lane * 4u : 0xfffffff0u, e0 * 4u, src[e]);
        }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the reads are done before the next row's drops
  }
}

}  // namespace swconv
