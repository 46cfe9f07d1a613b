// Device-side Winograd transform constants and the two small matrix sandwiches
//   V = B^T d B   (input transform, step 1 of Section 5 / Eq. 4)
//   Y = A^T z A   (output transform, step 3)
// for F(2x2,3x3) and F(4x4,3x3).  The paper does not print A and B (Section 3, after Eq. 3,
// defers to Lavin & Gray); these are the standard minimal-filtering matrices for the points
// {0,1,-1,inf} and {0,1,-1,2,-2,inf}.
//
// The 1-D transforms are written out by hand (shared sub-expressions, no multiplications by
// 0 or +-1); the 2-D sandwich applies them to columns, then to rows.
#pragma once
#include <hip/hip_runtime.h>

namespace swconv {

template <int M>
struct Wino;
template <>
struct Wino<2> {
  static constexpr int m = 2, t = 4;
};
template <>
struct Wino<4> {
  static constexpr int m = 4, t = 6;
};

// r = B^T x for one column (or row) of a tile.
//   F(2,3): B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]
//   F(4,3): B^T = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0; 0 2 -1 -2 1 0; 0 4 0 -5 0 1]
template <int M>
__device__ __forceinline__ void bt_apply(const float (&x)[Wino<M>::t], float (&r)[Wino<M>::t]);

template <>
__device__ __forceinline__ void bt_apply<2>(const float (&x)[4], float (&r)[4]) {
  r[0] = x[0] - x[2];
  r[1] = x[1] + x[2];
  r[2] = x[2] - x[1];
  r[3] = x[1] - x[3];
}

template <>
__device__ __forceinline__ void bt_apply<4>(const float (&x)[6], float (&r)[6]) {
  const float a = x[4] - 4.0f * x[2];  // -4 x2 + x4
  const float b = x[3] - 4.0f * x[1];  // -4 x1 + x3
  const float c = x[4] - x[2];         // -x2 + x4
  const float d = 2.0f * (x[3] - x[1]);  // -2 x1 + 2 x3
  r[0] = fmaf(4.0f, x[0], fmaf(-5.0f, x[2], x[4]));
  r[1] = a + b;
  r[2] = a - b;
  r[3] = c + d;
  r[4] = c - d;
  r[5] = fmaf(4.0f, x[1], fmaf(-5.0f, x[3], x[5]));
}

// y = A^T z for one column (or row).
//   F(2,3): A^T = [1 1 1 0; 0 1 -1 -1]
//   F(4,3): A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]
template <int M>
__device__ __forceinline__ void at_apply(const float (&z)[Wino<M>::t], float (&y)[M]);

template <>
__device__ __forceinline__ void at_apply<2>(const float (&z)[4], float (&y)[2]) {
  y[0] = z[0] + z[1] + z[2];
  y[1] = z[1] - z[2] - z[3];
}

template <>
__device__ __forceinline__ void at_apply<4>(const float (&z)[6], float (&y)[4]) {
  const float s12 = z[1] + z[2], d12 = z[1] - z[2];
  const float s34 = z[3] + z[4], d34 = z[3] - z[4];
  y[0] = z[0] + s12 + s34;
  y[1] = fmaf(2.0f, d34, d12);
  y[2] = fmaf(4.0f, s34, s12);
  y[3] = fmaf(8.0f, d34, d12) + z[5];
}

// v = B^T d B  (t x t): columns first, then rows.
template <int M>
__device__ __forceinline__ void input_transform(const float (&d)[Wino<M>::t][Wino<M>::t],
                                                float (&v)[Wino<M>::t][Wino<M>::t]) {
  constexpr int t = Wino<M>::t;
  float tmp[t][t];  // B^T d
#pragma unroll
  for (int j = 0; j < t; ++j) {
    float col[t], res[t];
#pragma unroll
    for (int a = 0; a < t; ++a) col[a] = d[a][j];
    bt_apply<M>(col, res);
#pragma unroll
    for (int i = 0; i < t; ++i) tmp[i][j] = res[i];
  }
#pragma unroll
  for (int i = 0; i < t; ++i) bt_apply<M>(tmp[i], v[i]);  // (tmp B)[i][j] = sum_b tmp[i][b] B^T[j][b]
}

// y = A^T z A  (m x m).
template <int M>
__device__ __forceinline__ void output_transform(const float (&z)[Wino<M>::t][Wino<M>::t],
                                                 float (&y)[M][M]) {
  constexpr int t = Wino<M>::t;
  float tmp[M][t];  // A^T z
#pragma unroll
  for (int j = 0; j < t; ++j) {
    float col[t], res[M];
#pragma unroll
    for (int i = 0; i < t; ++i) col[i] = z[i][j];
    at_apply<M>(col, res);
#pragma unroll
    for (int a = 0; a < M; ++a) tmp[a][j] = res[a];
  }
#pragma unroll
  for (int a = 0; a < M; ++a) at_apply<M>(tmp[a], y[a]);
}

}  // namespace swconv
