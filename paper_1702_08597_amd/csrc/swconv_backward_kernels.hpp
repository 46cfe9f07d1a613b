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
template <int M>
__global__ __launch_bounds__(256) void output_grad_transform_kernel(const float* __restrict__ dout,
                                                                    float* __restrict__ dZ,
                                                                    const TileInfo* __restrict__ tiles,
                                                                    const BlockImage* __restrict__ blocks,
                                                                    const Geometry g) {
  constexpr int t = Wino<M>::t;
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
      const __amdgpu_buffer_rsrc_t src = make_rsrc(dout + ((size_t)b.n * g.K + k) * plane + b.out_elem0,
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
  output_grad_transform<M>(gr, z);
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
template <int M>
__global__ __launch_bounds__(256) void input_grad_patch_kernel(const float* __restrict__ dV,
                                                               float* __restrict__ patches, const Geometry g) {
  constexpr int t = Wino<M>::t;
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
  input_grad_transform<M>(f, d);
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
// Eq. 6, third line, as a gather: a thread owns one input pixel (n, c, y, x) and adds the entries
// of the at most 2 x 2 patches that phi maps to it, tiles in ascending order, so every pixel is
// written once and the sum has a fixed order.  (t - m = r - 1 < m for the supported F(m, 3), so a
// pixel lies in at most two tiles per dimension.)  Grid: x = pixel chunks of a plane, y = (n, c).
template <int M>
__global__ __launch_bounds__(256) void input_grad_gather_kernel(const float* __restrict__ patches,
                                                                float* __restrict__ din, const Geometry g) {
  constexpr int t = Wino<M>::t;
  static_assert(t - M < M || M == 2, "two tiles per dimension");
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= g.H * g.W) return;
  const int nc = blockIdx.y, n = nc / g.C, c = nc - n * g.C;
  const int y = e / g.W, x = e - y * g.W;
  const int qy = (y + g.pad) / M, ry = (y + g.pad) - qy * M;
  const int qx = (x + g.pad) / M, rx = (x + g.pad) - qx * M;
  const __amdgpu_buffer_rsrc_t src = make_rsrc(patches, g.v_bytes);
  const uint32_t pstride = (uint32_t)g.C * (uint32_t)g.Tp;  // floats between positions
  float sum = 0.0f;
  // tiles ty = qy - dy with patch row a = ry + M * dy < t, ascending ty first
  constexpr int kBack = (t - 1) / M;  // how many tiles back a pixel can reach: 1 for F(4,3) and F(2,3)
#pragma unroll
  for (int dy = kBack; dy >= 0; --dy) {
    const int ty = qy - dy, a = ry + M * dy;
    if (ty < 0 || ty >= g.th || a >= t) continue;
#pragma unroll
    for (int dx = kBack; dx >= 0; --dx) {
      const int tx = qx - dx, b = rx + M * dx;
      if (tx < 0 || tx >= g.tw || b >= t) continue;
      const uint32_t tau = (uint32_t)(n * g.th + ty) * g.tw + tx;
      sum += buffer_load_f32(src, (((uint32_t)(a * t + b) * pstride) + (uint32_t)c * g.Tp + tau) * 4u, 0);
    }
  }
  din[((size_t)nc * g.H + y) * g.W + x] = sum;
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
  float sum = 0.0f;
  for (int tb = 0; tb < n_tau_blocks; ++tb) sum += partial[(size_t)tb * partial_stride + e];
  dvals[q] = sum;
}

}  // namespace swconv
