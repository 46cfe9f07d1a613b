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

}  // namespace swconv
