// HIP kernels of the sparse Winograd forward pass (Section 5's three steps) for gfx950.
//
// Layouts in device memory (all fp32):
//   in   [N][C][H][W]            caller's NCHW tensor
//   V    [P][C][Tp]              transformed input, position-major, tiles fastest (Section 5:
//                                "the fastest moving dimension is tiles"); Tp = T rounded up to
//                                the tile-block size, the pad columns hold zeros
//   M    [P][K][Tp]              per-position products
//   out  [N][K][Ho][Wo]
// Lanes of a wavefront map to consecutive tiles tau everywhere, so every V/M access of a wave
// is one contiguous 256-byte (or 512-byte) segment.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "winograd_transforms.hpp"

namespace swconv {

struct Geometry {
  int N, C, H, W, K, pad;
  int Ho, Wo, th, tw, tpi;  // tpi = th*tw tiles per image
  int T;                    // N*tpi
  int Tp;                   // padded tile count (row pitch of V and M)
};

// One slice = four rows of one position's sparse matrix, rows sorted by length.
struct Slice {
  uint32_t slot0;  // first slot of the slice in the packed stream (8 dwords per slot)
  int32_t len;     // slots in the slice = length of its longest row
  int32_t row0;    // index of its first row in the sorted-row table (P * Kp entries)
  int32_t p;       // position
};

// One workgroup's share of the sparse product: a tile block of one position and a strided
// subset of that position's slices.
struct WorkItem {
  int32_t p;
  int32_t tau_block;
  int32_t slice_begin;  // first slice taken
  int32_t slice_end;    // one past the position's last slice
  int32_t stride;       // distance between slices taken
};

constexpr int kSliceRows = 4;
constexpr int kXcds = 8;

// Workgroup ids are dealt round-robin to the 8 XCDs; remap them so that each XCD gets one
// contiguous range of virtual ids (neighbours in the work list then share an L2).
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nblocks) {
  const int per = nblocks / kXcds, rem = nblocks % kXcds;
  const int xcd = bid % kXcds, local = bid / kXcds;
  return xcd * per + (xcd < rem ? xcd : rem) + local;
}

__device__ __forceinline__ void decode_tile(const Geometry& g, int tau, int& n, int& ty, int& tx) {
  n = tau / g.tpi;
  const int rem = tau - n * g.tpi;
  ty = rem / g.tw;
  tx = rem - ty * g.tw;
}

// ---------------------------------------------------------------------------------------------
// Step 1: gather phi + V = B^T d B.  One lane per (channel, tile); block = 4 channels x 64 tiles.
template <int M>
__global__ __launch_bounds__(256) void input_transform_kernel(const float* __restrict__ in, float* __restrict__ V,
                                                              const Geometry g) {
  constexpr int t = Wino<M>::t;
  const int lane = threadIdx.x & 63;
  const int c = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int tau = blockIdx.x * 64 + lane;
  if (c >= g.C) return;
  float d[t][t];
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) d[i][j] = 0.0f;
  if (tau < g.T) {
    int n, ty, tx;
    decode_tile(g, tau, n, ty, tx);
    const float* plane = in + ((size_t)n * g.C + c) * g.H * g.W;
    const int y0 = ty * M - g.pad, x0 = tx * M - g.pad;
#pragma unroll
    for (int i = 0; i < t; ++i) {
      const int y = y0 + i;
#pragma unroll
      for (int j = 0; j < t; ++j) {
        const int x = x0 + j;
        if (y >= 0 && y < g.H && x >= 0 && x < g.W) d[i][j] = plane[y * g.W + x];
      }
    }
  }
  float v[t][t];
  input_transform<M>(d, v);
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) V[((size_t)(i * t + j) * g.C + c) * g.Tp + tau] = v[i][j];
}

// ---------------------------------------------------------------------------------------------
// Step 2: M[p] = W_F[p] * V[p] on the plain fp32 ALUs.
// A workgroup stages the C x TB panel V[p][:, tau_block] in LDS once; each wave then walks its
// slices: per slot it fetches four (column, weight) pairs with wave-uniform (scalar) loads,
// reads the four panel rows at lane-consecutive addresses and does four FMAs into four
// register accumulators (one per row of the slice).  TPL tiles per lane, TB = 64 * TPL.
template <int TPL, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) void spmm_kernel(const float* __restrict__ V, float* __restrict__ Mbuf,
                                                           const uint32_t* __restrict__ stream,
                                                           const Slice* __restrict__ slices,
                                                           const int32_t* __restrict__ sorted_rows,
                                                           const WorkItem* __restrict__ items, int n_items, int C,
                                                           int K, int Tp) {
  constexpr int TB = 64 * TPL;
  extern __shared__ float panel[];  // [C][TB]
  const int vid = xcd_contiguous_id(blockIdx.x, n_items);
  const WorkItem it = items[vid];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tau0 = it.tau_block * TB;

  {  // stage the panel: rows of TB floats, 16 bytes per lane
    const float* src = V + ((size_t)it.p * C) * Tp + tau0;
    constexpr int V4_PER_ROW = TB / 4;
    const int total = C * V4_PER_ROW;
    for (int idx = threadIdx.x; idx < total; idx += NWAVES * 64) {
      const int row = idx / V4_PER_ROW, q = idx - row * V4_PER_ROW;
      const float4 x = *reinterpret_cast<const float4*>(src + (size_t)row * Tp + q * 4);
      *reinterpret_cast<float4*>(panel + row * TB + q * 4) = x;
    }
  }
  __syncthreads();

  const float* lane_panel = panel + lane * TPL;
  for (int s = it.slice_begin + wave * it.stride; s < it.slice_end; s += NWAVES * it.stride) {
    const Slice sl = slices[s];
    const uint32_t* sp = stream + (size_t)sl.slot0 * 8;
    float acc[kSliceRows][TPL];
#pragma unroll
    for (int r = 0; r < kSliceRows; ++r)
#pragma unroll
      for (int e = 0; e < TPL; ++e) acc[r][e] = 0.0f;
    for (int slot = 0; slot < sl.len; ++slot) {
      uint32_t cw[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) cw[e] = sp[slot * 8 + e];
#pragma unroll
      for (int r = 0; r < kSliceRows; ++r) {
        const float w = __uint_as_float(cw[4 + r]);
        const float* vrow = lane_panel + cw[r] * TB;
#pragma unroll
        for (int e = 0; e < TPL; ++e) acc[r][e] = fmaf(w, vrow[e], acc[r][e]);
      }
    }
#pragma unroll
    for (int r = 0; r < kSliceRows; ++r) {
      const int k = sorted_rows[sl.row0 + r];
      if (k >= 0) {
        float* dst = Mbuf + ((size_t)it.p * K + k) * Tp + tau0 + lane * TPL;
#pragma unroll
        for (int e = 0; e < TPL; ++e) dst[e] = acc[r][e];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Step 3: Y = A^T z A + scatter psi.  One lane per (output channel, tile); block = 4 k x 64 tiles.
template <int M>
__global__ __launch_bounds__(256) void output_transform_kernel(const float* __restrict__ Mbuf,
                                                               float* __restrict__ out, const Geometry g) {
  constexpr int t = Wino<M>::t;
  const int lane = threadIdx.x & 63;
  const int k = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int tau = blockIdx.x * 64 + lane;
  if (k >= g.K || tau >= g.T) return;
  float z[t][t];
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) z[i][j] = Mbuf[((size_t)(i * t + j) * g.K + k) * g.Tp + tau];
  float y[M][M];
  output_transform<M>(z, y);
  int n, ty, tx;
  decode_tile(g, tau, n, ty, tx);
  float* plane = out + ((size_t)n * g.K + k) * g.Ho * g.Wo;
#pragma unroll
  for (int a = 0; a < M; ++a) {
    const int yy = ty * M + a;
#pragma unroll
    for (int b = 0; b < M; ++b) {
      const int xx = tx * M + b;
      if (yy < g.Ho && xx < g.Wo) plane[yy * g.Wo + xx] = y[a][b];
    }
  }
}

}  // namespace swconv
