// Dense comparison path for step 2: M[p] = W_F[p] * V[p] with a dense W_F, as a batched fp32
// GEMM on the MFMA units (v_mfma_f32_32x32x2_f32).  This is the 0 %-sparsity baseline the sparse
// product is compared with; the paper itself only projects a dense Winograd (Section 6.2).
//
//   WT  [P][C][Kq]   dense weights, transposed on the host so that output channels are fastest;
//                    Kq = K rounded up to 128, zero padded
//   V   [P][C][Tp]   Tp is a multiple of 128
//   M   [P][K][Tp]
// Workgroup = 4 waves, 128 (k) x 128 (tiles) of M[p]; each wave owns 64 x 64 = 2 x 2 MFMA blocks.
// The C dimension is walked 16 channels at a time through LDS with a register prefetch of the
// next chunk.
#pragma once
#include <hip/hip_runtime.h>

namespace swconv {

constexpr int kDenseTileM = 128;  // output channels per workgroup
constexpr int kDenseTileN = 128;  // tiles per workgroup
constexpr int kDenseKc = 16;      // channels per LDS chunk

typedef float floatx16 __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void dense_position_gemm_kernel(const float* __restrict__ WT,
                                                                  const float* __restrict__ V,
                                                                  float* __restrict__ Mbuf, int K, int Kq, int C,
                                                                  int Tp) {
  __shared__ float As[kDenseKc][kDenseTileM];
  __shared__ float Bs[kDenseKc][kDenseTileN];
  const int p = blockIdx.z;
  const int k0 = blockIdx.y * kDenseTileM, n0 = blockIdx.x * kDenseTileN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
  const float* Wp = WT + (size_t)p * C * Kq + k0;
  const float* Vp = V + (size_t)p * C * Tp + n0;

  floatx16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

  float4 ra[2], rb[2];
  auto load_chunk = [&](int c0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + i * 256, row = idx >> 5, col = (idx & 31) * 4;
      const int c = c0 + row;
      if (c < C) {
        ra[i] = *reinterpret_cast<const float4*>(Wp + (size_t)c * Kq + col);
        rb[i] = *reinterpret_cast<const float4*>(Vp + (size_t)c * Tp + col);
      } else {
        ra[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        rb[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };

  load_chunk(0);
  for (int c0 = 0; c0 < C; c0 += kDenseKc) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + i * 256, row = idx >> 5, col = (idx & 31) * 4;
      *reinterpret_cast<float4*>(&As[row][col]) = ra[i];
      *reinterpret_cast<float4*>(&Bs[row][col]) = rb[i];
    }
    __syncthreads();
    if (c0 + kDenseKc < C) load_chunk(c0 + kDenseKc);
#pragma unroll
    for (int kk = 0; kk < kDenseKc; kk += 2) {
      const int kr = kk + (lane >> 5), col = lane & 31;
      float a[2], b[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) a[mi] = As[kr][wm + mi * 32 + col];
#pragma unroll
      for (int ni = 0; ni < 2; ++ni) b[ni] = Bs[kr][wn + ni * 32 + col];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    }
    __syncthreads();
  }

  // D layout of the 32x32 MFMA: register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32.
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = k0 + wm + mi * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int col = n0 + wn + ni * 32 + (lane & 31);
        if (row < K) Mbuf[((size_t)p * K + row) * Tp + col] = acc[mi][ni][v];
      }
}

}  // namespace swconv
