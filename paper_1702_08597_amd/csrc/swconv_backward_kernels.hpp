// HIP kernels of the backward pass of the Winograd layer (Section 3, Eq. 5 and Eq. 6) for gfx950.
//
//   dZ  [P][K][Tp]   dL/dZ = A dL/dO~ A^T            (Eq. 5, first line)   - held in the M workspace
//   dW               dL/dW_F(k,c,p) = sum_tau dZ[p][k][tau] V[p][c][tau] at the stored entries (Eq. 5)
//   dV  [P][C][Tp]   dL/dI_F[p] = W_F[p]^T dZ[p]     (Eq. 6, first line): the sparse product kernel of the
//                    forward pass, run on the packed transpose of W_F
//   dI~ [P][C][Tp]   dL/dI~ = B dL/dI_F B^T          (Eq. 6, second line), one t x t patch per (c, tile),
//                    stored position-major like V
//   dI  [N][C][H][W] every pixel sums the patch entries phi maps to it (Eq. 6, third line)
//
// Layouts, tile order and the index tables are those of the forward kernels.
#pragma once
#include "swconv_kernels.hpp"

namespace swconv {

// ---------------------------------------------------------------------------------------------
// Eq. 5, first line.  A wave owns one output channel and 64 consecutive tiles: it copies the rows
// of dL/dO its tiles own into its LDS area with lane-contiguous loads (the staging layout of the
// output transform, read instead of written), every lane gathers its m x m tile - zero where the
// tile reaches past H_o x W_o: those outputs were dropped by psi and carry no gradient -
// transforms it in registers and stores one value per position.
template <int M, int R>
__global__ __launch_bounds__(256) void output_grad_transform_kernel(const float* __restrict__ dout,
                                                                    float* __restrict__ dZ,
                                                                    const TileInfo* __restrict__ tiles,
                                                                    const BlockImage* __restrict__ blocks,
                                                                    const Geometry g) {
  constexpr int t = Wino<M, R>::t;
  extern __shared__ float stage[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int k = blockIdx.y * 4 + wave;
  const int tau0 = blockIdx.x * 64;
  float* my = stage + wave * g.out_area;
  const BlockImage* bi = blocks + (size_t)blockIdx.x * g.slots;
  const size_t plane = (size_t)g.Ho * g.Wo;
  if (k < g.K) {
    for (int sidx = 0; sidx < g.slots; ++sidx) {
      const BlockImage b = bi[sidx];
      if (b.n < 0) continue;
      // loads past the part's end return 0 (descriptor), so the padded tail of the run is zero
      const __amdgpu_buffer_rsrc_t src = make_rsrc(dout + (size_t)b.n * g.out_image_stride + k * plane + b.out_elem0,
                                                   (uint32_t)b.out_span * 4u);
      float* dst = my + b.out_off + lane;
      constexpr int EL = 4;  // loads per lane in flight
      for (int e0 = 0; e0 < b.out_span; e0 += 64 * EL) {
        float buf[EL];
#pragma unroll
        for (int u = 0; u < EL; ++u)
          if (e0 + u * 64 < b.out_span) buf[u] = buffer_load_f32(src, (lane + u * 64) * 4u, e0 * 4u);
#pragma unroll
        for (int u = 0; u < EL; ++u)
          if (e0 + u * 64 < b.out_span) dst[e0 + u * 64] = buf[u];
      }
    }
  }
  __syncthreads();
  if (k >= g.K) return;
  float gr[M][M];
  {
    const TileInfo ti = tiles[tau0 + lane];
    const int y0 = (int16_t)(ti.yx0 & 0xffff), x0 = ti.yx0 >> 16;
    // rows / columns of the tile inside the output (<= 0 for a padding tile, whose y0 is -32768)
    const int rows = y0 == -32768 ? 0 : g.Ho - (y0 + g.pad), cols = g.Wo - (x0 + g.pad);
    const float* px = my + ti.out_org;
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; ++b) {
        const bool inside = a < rows && b < cols;
        const float v = px[inside ? a * g.Wo + b : 0];  // a staged address in any case (a padding tile reads offset 0)
        gr[a][b] = inside ? v : 0.0f;
      }
  }
  float z[t][t];
  output_grad_transform<M, R>(gr, z);
  const __amdgpu_buffer_rsrc_t zr = make_rsrc(dZ, g.m_bytes);
  const uint32_t pstride = (uint32_t)g.K * (uint32_t)g.Tp * 4u;
  uint32_t soff = ((uint32_t)k * g.Tp + tau0) * 4u;
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) {
      buffer_store_f32<SWCONV_AUX_M>(zr, lane * 4u, soff, z[i][j]);
      soff += pstride;
      asm volatile("" : "+s"(soff));
    }
}

// ---------------------------------------------------------------------------------------------
// Eq. 6, second line.  A wave owns one input channel and 64 consecutive tiles: each lane reads the
// t*t values dL/dI_F(c, tau, :, :) (256 contiguous bytes per wave and position), applies B . B^T in
// registers and stores the t x t patch dL/dI~(c, tau, :, :), again one value per position.
template <int M, int R>
__global__ __launch_bounds__(256) void input_grad_patch_kernel(const float* __restrict__ dV,
                                                               float* __restrict__ patches, const Geometry g) {
  constexpr int t = Wino<M, R>::t;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.y * 4 + wave;
  const int tau0 = blockIdx.x * 64;
  if (c >= g.C || tau0 >= g.T) return;
  const __amdgpu_buffer_rsrc_t src = make_rsrc(dV, g.v_bytes), dst = make_rsrc(patches, g.v_bytes);
  const uint32_t row0 = ((uint32_t)c * g.Tp + tau0) * 4u;
  const uint32_t pstride = (uint32_t)g.C * (uint32_t)g.Tp * 4u;
  float f[t][t], d[t][t];
  uint32_t soff = row0;
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) {
      f[i][j] = buffer_load_f32(src, lane * 4u, soff);
      soff += pstride;
      asm volatile("" : "+s"(soff));
    }
  input_grad_transform<M, R>(f, d);
  soff = row0;
#pragma unroll
  for (int a = 0; a < t; ++a)
#pragma unroll
    for (int b = 0; b < t; ++b) {
      buffer_store_f32<SWCONV_AUX_V>(dst, lane * 4u, soff, d[a][b]);
      soff += pstride;
      asm volatile("" : "+s"(soff));
    }
}

// ---------------------------------------------------------------------------------------------
// Eq. 6, third line, as a gather.  The input plane is cut into m x m cells aligned with the tile
// stride: cell (qy, qx) holds the pixels y = qy*m - pad + ry, x = qx*m - pad + rx.  Every pixel of a
// cell receives from the same tiles (qy - dy, qx - dx), dy, dx in 0 .. (t-1)/m (one tile back for
// the 3x3 filters, two for F(2x2,5x5)), the patch entry (ry + m*dy, rx + m*dx) where that lies
// inside the t x t patch.  A
// thread owns one cell of one (n, c) plane and lanes run over consecutive cells, i.e. consecutive
// tiles, so every patch load of a wave is a contiguous run of one position plane and each patch
// entry is read exactly once; each pixel is written once, its sum taken in ascending tile order.
// Threads run over all cells of all (n, c) planes.
template <int M, int R>
__global__ __launch_bounds__(256) void input_grad_gather_kernel(const float* __restrict__ patches,
                                                                float* __restrict__ din, const Geometry g) {
  constexpr int t = Wino<M, R>::t;
  constexpr int back = (t - 1) / M;  // tiles before its own that still cover a cell, per dimension
  const int cells_y = (g.H - 1 + g.pad) / M + 1, cells_x = (g.W - 1 + g.pad) / M + 1;
  const int cells = cells_y * cells_x;
  const uint32_t idx = blockIdx.x * 256u + threadIdx.x;  // (n, c) plane major, cells of a plane consecutive
  if (idx >= (uint32_t)g.N * g.C * cells) return;
  const int nc = idx / cells, cell = idx - nc * cells;
  const int n = nc / g.C, c = nc - n * g.C;
  const int qy = cell / cells_x, qx = cell - qy * cells_x;
  const __amdgpu_buffer_rsrc_t src = make_rsrc(patches, g.v_bytes);
  const uint32_t pstride = (uint32_t)g.C * (uint32_t)g.Tp;  // floats between positions
  float acc[M][M];
#pragma unroll
  for (int ry = 0; ry < M; ++ry)
#pragma unroll
    for (int rx = 0; rx < M; ++rx) acc[ry][rx] = 0.0f;
  // tiles in ascending order: (qy-back, qx-back), ..., (qy, qx)
#pragma unroll
  for (int dy = back; dy >= 0; --dy) {
    const int ty = qy - dy;
#pragma unroll
    for (int dx = back; dx >= 0; --dx) {
      const int tx = qx - dx;
      if (ty < 0 || ty >= g.th || tx < 0 || tx >= g.tw) continue;
      const uint32_t base = ((uint32_t)c * g.Tp + (uint32_t)(n * g.th + ty) * g.tw + tx) * 4u;
#pragma unroll
      for (int ry = 0; ry < M; ++ry)
#pragma unroll
        for (int rx = 0; rx < M; ++rx) {
          const int a = ry + M * dy, b = rx + M * dx;  // compile-time after unrolling
          if (a < t && b < t) acc[ry][rx] += buffer_load_f32(src, base + (uint32_t)(a * t + b) * pstride * 4u, 0);
        }
    }
  }
  float* plane = din + (size_t)n * g.in_image_stride + (size_t)c * g.H * g.W;
#pragma unroll
  for (int ry = 0; ry < M; ++ry) {
    const int y = qy * M - g.pad + ry;
    if (y < 0 || y >= g.H) continue;
#pragma unroll
    for (int rx = 0; rx < M; ++rx) {
      const int x = qx * M - g.pad + rx;
      if (x >= 0 && x < g.W) plane[y * g.W + x] = acc[ry][rx];
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Eq. 6, second and third line in one kernel, for images whose planes fit LDS: no patch buffer.
// A wave owns one input channel and a group of G whole images (G = 64 / tiles per image, at least
// 1), whose planes it keeps in LDS.  In passes of 64 consecutive tiles every lane reads the t*t
// values dL/dI_F(c, tau, :, :), applies B . B^T in registers and adds its t x t patch into the
// plane.  Patches of tiles closer than t pixels overlap, so the additions run in (back+1)^2
// phases, phase (ty mod (back+1), tx mod (back+1)): the tiles of one phase are disjoint, LDS
// executes a wave's operations in order, and every pixel therefore receives its terms in a fixed
// order.  Then the wave writes its planes with lane-contiguous stores.  Block = 4 waves = 4
// channels of the same image group.
struct GradTile {
  int32_t org;  // float offset of pixel (0, 0) of the tile's image inside the wave's LDS area
  int32_t yx0;  // as TileInfo::yx0; y0 = x0 = -32768 for tiles past the last image
};

template <int M, int R>
__global__ __launch_bounds__(256) void input_grad_kernel(const float* __restrict__ dV, float* __restrict__ din,
                                                         const GradTile* __restrict__ gtiles, int images_per_group,
                                                         const Geometry g) {
  constexpr int t = Wino<M, R>::t;
  constexpr int back = (t - 1) / M, PH = back + 1;
  extern __shared__ float stage[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.y * 4 + wave;
  if (c >= g.C) return;  // no barrier in this kernel: waves are independent
  const int n0 = blockIdx.x * images_per_group;
  const int n_img = min(images_per_group, g.N - n0);
  const int plane = g.H * g.W;
  const int area = images_per_group * plane;
  const int area_padded = (area + 63) / 64 * 64;  // the wave's planes, then one spare float per lane
  float* my = stage + (size_t)wave * (area_padded + 64);
  for (int e = lane; e < area; e += 64) my[e] = 0.0f;
  const __amdgpu_buffer_rsrc_t src = make_rsrc(dV, g.v_bytes);
  const uint32_t pstride = (uint32_t)g.C * (uint32_t)g.Tp * 4u;
  const int tau0 = n0 * g.tpi, tau_end = tau0 + n_img * g.tpi;
  for (int base = tau0; base < tau_end; base += 64) {
    const int tau = base + lane;
    const bool live = tau < tau_end;
    // lanes past the group's last tile are parked past the end of the buffer: they read zeros
    const uint32_t voff = live ? ((uint32_t)c * g.Tp + (uint32_t)tau) * 4u : 0xfffffff0u;
    float f[t][t], d[t][t];
    uint32_t soff = 0;
#pragma unroll
    for (int i = 0; i < t; ++i)
#pragma unroll
      for (int j = 0; j < t; ++j) {
        f[i][j] = buffer_load_f32(src, voff, soff);
        soff += pstride;
        asm volatile("" : "+s"(soff));
      }
    const GradTile gt = gtiles[live ? tau : tau0];
    input_grad_transform<M, R>(f, d);
    const int y0 = (int16_t)(gt.yx0 & 0xffff), x0 = gt.yx0 >> 16;
    const int ty = (y0 + g.pad) >> g.m_shift, tx = (x0 + g.pad) >> g.m_shift;
    const int phase = live ? (ty % PH) * PH + tx % PH : -1;
    // LDS index of every patch entry; entries outside the image go to a spare float of the lane
    const int spare = area_padded + lane;
    const int org = gt.org + y0 * g.W + x0;
    int at[t][t];
#pragma unroll
    for (int a = 0; a < t; ++a) {
      const bool yok = y0 + a >= 0 && y0 + a < g.H;
#pragma unroll
      for (int b = 0; b < t; ++b) at[a][b] = (yok && x0 + b >= 0 && x0 + b < g.W) ? org + a * g.W + b : spare;
    }
#pragma unroll
    for (int ph = 0; ph < PH * PH; ++ph) {
      if (ph == 0 && base == tau0) {
        // first phase of the first pass: the planes still hold zeros, so the patch is stored as it is
        if (phase == 0) {
#pragma unroll
          for (int a = 0; a < t; ++a)
#pragma unroll
            for (int b = 0; b < t; ++b) my[at[a][b]] = d[a][b];
        }
      } else if (phase == ph) {
        // plain read-add-write (an LDS float atomic costs about 38 clocks per instruction here):
        // the lanes of a phase touch disjoint pixels, and a lane's own entries are distinct
        float cur[t][t];
#pragma unroll
        for (int a = 0; a < t; ++a)
#pragma unroll
          for (int b = 0; b < t; ++b) cur[a][b] = my[at[a][b]];
#pragma unroll
        for (int a = 0; a < t; ++a)
#pragma unroll
          for (int b = 0; b < t; ++b) my[at[a][b]] = cur[a][b] + d[a][b];
      }
      // the next phase adds to what this one wrote: keep the compiler from moving LDS accesses across
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }
  for (int i = 0; i < n_img; ++i) {
    const float* from = my + (size_t)i * plane;
    const __amdgpu_buffer_rsrc_t dst =
        make_rsrc(din + (size_t)(n0 + i) * g.in_image_stride + (size_t)c * plane, (uint32_t)plane * 4u);
    for (int e0 = 0; e0 < plane; e0 += 64)  // lanes past the plane's end read their wave's padding and store nothing
      buffer_store_f32<SWCONV_AUX_OUT>(dst, lane * 4u, e0 * 4u, from[min(e0 + lane, plane - 1)]);
  }
}

// ---------------------------------------------------------------------------------------------
// Eq. 5, second line, last step: the per-tile-block partial sums of every stream entry (written by
// the sparse kernel in sampled mode) are added over the tile blocks, in ascending order, and go to
// the entry's place in the caller's CSR order; padding entries (index -1) are skipped.
__global__ __launch_bounds__(256) void weight_grad_reduce_kernel(const float* __restrict__ partial, int n_tau_blocks,
                                                                 uint32_t partial_stride,
                                                                 const int32_t* __restrict__ entry_index,
                                                                 uint32_t n_entries, float* __restrict__ dvals) {
  const uint32_t e = blockIdx.x * 256u + threadIdx.x;
  if (e >= n_entries) return;
  const int32_t q = entry_index[e];
  if (q < 0) return;
  // eight loads in flight, added in ascending order of the tile block
  float sum = 0.0f;
  int tb = 0;
  for (; tb + 8 <= n_tau_blocks; tb += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = partial[(size_t)(tb + u) * partial_stride + e];
#pragma unroll
    for (int u = 0; u < 8; ++u) sum += v[u];
  }
  for (; tb < n_tau_blocks; ++tb) sum += partial[(size_t)tb * partial_stride + e];
  dvals[q] = sum;
}

}  // namespace swconv
