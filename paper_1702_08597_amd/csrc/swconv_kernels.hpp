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
  // LDS staging of the transforms: a block of 64 consecutive tiles touches at most `slots` images,
  // and in each of them a run of at most `in_span` input / `out_span` output floats (whole rows)
  int slots, in_span, out_span;
};

// The part of image n that a block of 64 consecutive tiles [tau0, last] covers.
struct ImagePart {
  int t_lo, t_hi;    // first / last tile of the block inside image n (image-local tile index)
  int ty_lo, ty_hi;  // tile rows they span
};

__device__ __forceinline__ ImagePart image_part(const Geometry& g, int n, int tau0, int last) {
  ImagePart ip;
  const int base = n * g.tpi;
  ip.t_lo = max(tau0, base) - base;
  ip.t_hi = min(last, base + g.tpi - 1) - base;
  ip.ty_lo = ip.t_lo / g.tw;
  ip.ty_hi = ip.t_hi / g.tw;
  return ip;
}

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
// Step 1: gather phi + V = B^T d B.  A wave owns one channel and 64 consecutive tiles: it copies
// the input rows those tiles touch into its private LDS area with lane-contiguous (coalesced)
// loads - each pixel is read from memory once although up to (t/m)^2 tiles use it - then every
// lane gathers its t x t tile from LDS (zero outside the image), transforms it in registers and
// stores one value per position: 64 lanes -> 256 contiguous bytes of V[p][c][.].
// Block = 4 waves = 4 channels of the same tile block.
template <int M>
__global__ __launch_bounds__(256) void input_transform_kernel(const float* __restrict__ in, float* __restrict__ V,
                                                              const Geometry g) {
  constexpr int t = Wino<M>::t;
  extern __shared__ float stage[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.y * 4 + wave;
  const int tau0 = blockIdx.x * 64;
  const int last = min(tau0 + 63, g.T - 1);
  const int n_first = tau0 / g.tpi, n_last = last / g.tpi;
  float* my = stage + wave * g.slots * g.in_span;
  if (c < g.C) {
    for (int n = n_first; n <= n_last; ++n) {
      const ImagePart ip = image_part(g, n, tau0, last);
      const int y_lo = max(0, ip.ty_lo * M - g.pad), y_hi = min(g.H, ip.ty_hi * M - g.pad + t);
      const int span = (y_hi - y_lo) * g.W;
      const float* src = in + (((size_t)n * g.C + c) * g.H + y_lo) * g.W;
      float* dst = my + (n - n_first) * g.in_span;
      for (int e = lane; e < span; e += 64) dst[e] = src[e];
    }
  }
  __syncthreads();
  if (c >= g.C) return;
  const int tau = tau0 + lane;
  float d[t][t];
  {
    // every lane reads t*t LDS words at clamped (always valid) addresses and zeroes what lies
    // outside the image or belongs to a padding tile: selects, no divergent branches
    const bool live = tau < g.T;
    int n, ty, tx;
    decode_tile(g, live ? tau : tau0, n, ty, tx);
    const ImagePart ip = image_part(g, n, tau0, last);
    const int y_lo = max(0, ip.ty_lo * M - g.pad);
    const float* img = my + (n - n_first) * g.in_span - y_lo * g.W;
    const int y0 = ty * M - g.pad, x0 = tx * M - g.pad;
    int xo[t];
    bool xok[t];
#pragma unroll
    for (int j = 0; j < t; ++j) {
      const int x = x0 + j;
      xok[j] = live && x >= 0 && x < g.W;
      xo[j] = min(max(x, 0), g.W - 1);
    }
#pragma unroll
    for (int i = 0; i < t; ++i) {
      const int y = y0 + i;
      const bool yok = y >= 0 && y < g.H;
      const float* row = img + min(max(y, y_lo), g.H - 1) * g.W;
#pragma unroll
      for (int j = 0; j < t; ++j) {
        const float val = row[xo[j]];
        d[i][j] = (yok && xok[j]) ? val : 0.0f;
      }
    }
  }
  float v[t][t];
  input_transform<M>(d, v);
  float* dst = V + (size_t)c * g.Tp + tau;
  const size_t pstride = (size_t)g.C * g.Tp;
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) dst[(i * t + j) * pstride] = v[i][j];
}

// ---------------------------------------------------------------------------------------------
// Step 2: M[p] = W_F[p] * V[p] on the plain fp32 ALUs.
// A workgroup stages the C x TB panel V[p][:, tau_block] in LDS once (all its loads in flight
// before the first LDS write); each wave then walks its slices.  A slice's stream is a sequence
// of slots, each holding one (column, weight) pair for each of the slice's four rows; slices are
// padded to an even number of slots.  Per batch of eight slots the wave fetches 64 dwords with
// wave-uniform (scalar) loads, reads the 32 panel rows at lane-consecutive addresses and does
// 32 FMAs per tile into four register accumulators (one per row).  TPL tiles per lane,
// TB = 64 * TPL.
constexpr int kSlotUnroll = 2;   // slice lengths are multiples of this many slots
constexpr int kBatchSlots = 8;   // slots fetched per scalar-memory round trip

template <int TPL, int NWAVES>
__global__ __launch_bounds__(NWAVES * 64) void spmm_kernel(const float* __restrict__ V, float* __restrict__ Mbuf,
                                                           const uint32_t* __restrict__ stream,
                                                           const Slice* __restrict__ slices,
                                                           const int32_t* __restrict__ sorted_rows,
                                                           const WorkItem* __restrict__ items, int n_items, int C,
                                                           int K, int Tp) {
  constexpr int TB = 64 * TPL;
  constexpr int NT = NWAVES * 64;
  extern __shared__ float panel[];  // [C][TB]
  const int vid = xcd_contiguous_id(blockIdx.x, n_items);
  const WorkItem it = items[vid];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tau0 = it.tau_block * TB;

  {  // stage the panel: rows of TB floats, 16 bytes per lane, 4 loads in flight per lane
    const float* src = V + ((size_t)it.p * C) * Tp + tau0;
    constexpr int V4_PER_ROW = TB / 4;
    constexpr int U = 4;
    const int total = C * V4_PER_ROW;
    int base = threadIdx.x;
    for (; base + (U - 1) * NT < total; base += NT * U) {  // full batches, no bounds checks
      float4 buf[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int idx = base + u * NT;
        const int row = idx / V4_PER_ROW, q = idx - row * V4_PER_ROW;
        buf[u] = *reinterpret_cast<const float4*>(src + (size_t)row * Tp + q * 4);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) *reinterpret_cast<float4*>(panel + (base + u * NT) * 4) = buf[u];
    }
    for (; base < total; base += NT) {
      const int row = base / V4_PER_ROW, q = base - row * V4_PER_ROW;
      *reinterpret_cast<float4*>(panel + base * 4) = *reinterpret_cast<const float4*>(src + (size_t)row * Tp + q * 4);
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
    // one batch = kBatchSlots slots = 64 dwords fetched with four back-to-back scalar loads, so
    // the scalar-memory latency is paid once per 32 (column, weight) pairs; the stream carries
    // one spare batch at its end, so the fetch of a short last batch stays in bounds
    for (int remaining = sl.len; remaining > 0; remaining -= kBatchSlots, sp += 8 * kBatchSlots) {
      // four 64-byte wave-uniform loads issued back to back; the empty asm statements pin all
      // of them in scalar registers here, so the compiler cannot sink each load next to its
      // (conditional) use and pay the scalar-memory latency four times
      typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
      static_assert(kBatchSlots == 8, "batch = four 16-dword fetches");
      u32x16 q0 = *reinterpret_cast<const u32x16*>(sp);
      u32x16 q1 = *reinterpret_cast<const u32x16*>(sp + 16);
      u32x16 q2 = *reinterpret_cast<const u32x16*>(sp + 32);
      u32x16 q3 = *reinterpret_cast<const u32x16*>(sp + 48);
      asm volatile("" : "+s"(q0), "+s"(q1), "+s"(q2), "+s"(q3));
      uint32_t cw[8 * kBatchSlots];
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        cw[e] = q0[e];
        cw[16 + e] = q1[e];
        cw[32 + e] = q2[e];
        cw[48 + e] = q3[e];
      }
#pragma unroll
      for (int u = 0; u < kBatchSlots; u += kSlotUnroll) {
        if (u < remaining) {  // wave-uniform
#pragma unroll
          for (int uu = u; uu < u + kSlotUnroll; ++uu)
#pragma unroll
            for (int r = 0; r < kSliceRows; ++r) {
              const float w = __uint_as_float(cw[uu * 8 + 4 + r]);
              const float* vrow = lane_panel + cw[uu * 8 + r] * TB;
#pragma unroll
              for (int e = 0; e < TPL; ++e) acc[r][e] = fmaf(w, vrow[e], acc[r][e]);
            }
        }
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
// Step 3: Y = A^T z A + scatter psi.  A wave owns one output channel and 64 consecutive tiles:
// each lane reads its t*t values of M (256 contiguous bytes per wave and position), transforms
// them in registers and drops its m x m outputs into the wave's LDS area laid out like the output
// rows; the wave then writes those rows out with lane-contiguous stores (whole image planes when
// the block covers whole images).  Pixels of tiles that belong to a neighbouring block are
// skipped.  Block = 4 waves = 4 output channels of the same tile block.
template <int M>
__global__ __launch_bounds__(256) void output_transform_kernel(const float* __restrict__ Mbuf,
                                                               float* __restrict__ out, const Geometry g) {
  constexpr int t = Wino<M>::t;
  extern __shared__ float stage[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int k = blockIdx.y * 4 + wave;
  const int tau0 = blockIdx.x * 64;
  if (tau0 >= g.T) return;  // whole block is padding (uniform for the block)
  const int last = min(tau0 + 63, g.T - 1);
  const int n_first = tau0 / g.tpi, n_last = last / g.tpi;
  const int tau = tau0 + lane;
  float* my = stage + wave * g.slots * g.out_span;
  if (k < g.K && tau < g.T) {
    const float* msrc = Mbuf + (size_t)k * g.Tp + tau;
    const size_t pstride = (size_t)g.K * g.Tp;
    float z[t][t];
#pragma unroll
    for (int i = 0; i < t; ++i)
#pragma unroll
      for (int j = 0; j < t; ++j) z[i][j] = msrc[(i * t + j) * pstride];
    float y[M][M];
    output_transform<M>(z, y);
    int n, ty, tx;
    decode_tile(g, tau, n, ty, tx);
    const ImagePart ip = image_part(g, n, tau0, last);
    float* img = my + (n - n_first) * g.out_span - ip.ty_lo * M * g.Wo;
#pragma unroll
    for (int a = 0; a < M; ++a) {
      const int yy = ty * M + a;
#pragma unroll
      for (int b = 0; b < M; ++b) {
        const int xx = tx * M + b;
        if (yy < g.Ho && xx < g.Wo) img[yy * g.Wo + xx] = y[a][b];
      }
    }
  }
  __syncthreads();
  if (k >= g.K) return;
  for (int n = n_first; n <= n_last; ++n) {
    const ImagePart ip = image_part(g, n, tau0, last);
    const int y_lo = ip.ty_lo * M, y_hi = min(g.Ho, (ip.ty_hi + 1) * M);
    const int span = (y_hi - y_lo) * g.Wo;
    const float* src = my + (n - n_first) * g.out_span;
    float* dst = out + (((size_t)n * g.K + k) * g.Ho + y_lo) * g.Wo;
    const bool whole_rows = (ip.t_lo % g.tw == 0) && ((ip.t_hi + 1) % g.tw == 0);
    if (whole_rows) {
      for (int e = lane; e < span; e += 64) dst[e] = src[e];
    } else {
      for (int e = lane; e < span; e += 64) {
        const int ry = e / g.Wo, x = e - ry * g.Wo;
        const int tl = ((y_lo + ry) / M) * g.tw + x / M;
        if (tl >= ip.t_lo && tl <= ip.t_hi) dst[e] = src[e];
      }
    }
  }
}

}  // namespace swconv
