// Device-side Winograd transform constants and the two small matrix sandwiches
//   V = B^T d B   (input transform, step 1 of Section 5 / Eq. 4)
//   Y = A^T z A   (output transform, step 3)
// for F(2x2,3x3) and F(4x4,3x3).  The paper does not print A and B (Section 3, after Eq. 3,
// defers to Lavin & Gray); these are the standard minimal-filtering matrices for the points
// {0,1,-1,inf} and {0,1,-1,2,-2,inf}.
//
// All loops are fully unrolled over constexpr tables, so zero coefficients cost nothing and
// +-1 coefficients become plain adds/subtracts.
#pragma once
#include <hip/hip_runtime.h>

namespace swconv {

template <int M>
struct Wino;

template <>
struct Wino<2> {
  static constexpr int m = 2, t = 4;
  static constexpr float BT[4][4] = {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}};
  static constexpr float AT[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
};

template <>
struct Wino<4> {
  static constexpr int m = 4, t = 6;
  static constexpr float BT[6][6] = {{4, 0, -5, 0, 1, 0},  {0, -4, -4, 1, 1, 0}, {0, 4, -4, -1, 1, 0},
                                     {0, -2, -1, 2, 1, 0}, {0, 2, -1, -2, 1, 0}, {0, 4, 0, -5, 0, 1}};
  static constexpr float AT[4][6] = {
      {1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};
};

// s (+)= coef * x with the trivial coefficients folded at compile time.
template <bool First>
__device__ __forceinline__ float axpy_c(float s, float coef, float x) {
  if (coef == 1.0f) return First ? x : s + x;
  if (coef == -1.0f) return First ? -x : s - x;
  return First ? coef * x : fmaf(coef, x, s);
}

// out[i] = sum_a Mat[i][a] * in[a]   for one column/row vector, Mat is ROWS x COLS constexpr.
template <int ROWS, int COLS, typename MatT>
__device__ __forceinline__ void matvec_c(const MatT& Mat, const float (&in)[COLS], float (&out)[ROWS]) {
#pragma unroll
  for (int i = 0; i < ROWS; ++i) {
    float s = 0.0f;
    bool first = true;
#pragma unroll
    for (int a = 0; a < COLS; ++a) {
      const float coef = Mat[i][a];
      if (coef != 0.0f) {
        s = first ? axpy_c<true>(s, coef, in[a]) : axpy_c<false>(s, coef, in[a]);
        first = false;
      }
    }
    out[i] = s;
  }
}

// v = B^T d B  (t x t).
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
    matvec_c<t, t>(Wino<M>::BT, col, res);
#pragma unroll
    for (int i = 0; i < t; ++i) tmp[i][j] = res[i];
  }
#pragma unroll
  for (int i = 0; i < t; ++i) {
    float res[t];
    matvec_c<t, t>(Wino<M>::BT, tmp[i], res);  // (tmp B)[i][j] = sum_b tmp[i][b] BT[j][b]
#pragma unroll
    for (int j = 0; j < t; ++j) v[i][j] = res[j];
  }
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
    matvec_c<M, t>(Wino<M>::AT, col, res);
#pragma unroll
    for (int a = 0; a < M; ++a) tmp[a][j] = res[a];
  }
#pragma unroll
  for (int a = 0; a < M; ++a) {
    float res[M];
    matvec_c<M, t>(Wino<M>::AT, tmp[a], res);
#pragma unroll
    for (int b = 0; b < M; ++b) y[a][b] = res[b];
  }
}

}  // namespace swconv
