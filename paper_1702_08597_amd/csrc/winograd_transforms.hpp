// Device-side Winograd transform constants and the two small matrix sandwiches
//   V = B^T d B   (input transform, step 1 of Section 5 / Eq. 4)
//   Y = A^T z A   (output transform, step 3)
//   Z' = A g A^T, D = B f B^T   (their transposes, backward pass: Eq. 5 first line, Eq. 6 second line)
// for F(2x2,3x3), F(4x4,3x3) and F(2x2,5x5).  The paper does not print A and B (Section 3, after
// Eq. 3, defers to Lavin & Gray); these are the standard minimal-filtering matrices for the points
// {0,1,-1,inf} and {0,1,-1,2,-2,inf}.  F(2,5) (the 5x5 layers of Section 6) has t = 6 like F(4,3) and
// is built on the same six points, so it shares B^T with F(4,3); its A^T keeps the first two rows of
// the F(4,3) one, with the point at infinity entering the row of the highest output power.
// F(4,5), t = 8, is the same Toom-Cook construction on {0,1,-1,2,-2,1/2,-1/2,inf}: row i of B^T holds
// the coefficients of prod_{k != i} (x - p_k) (last row: of prod_k (x - p_k)), A^T[a][i] = p_i^a; all
// entries are dyadic rationals.
//
// The 1-D transforms are written out by hand (shared sub-expressions, no multiplications by
// 0 or +-1); the 2-D sandwich applies them to columns, then to rows.
#pragma once
#include <hip/hip_runtime.h>

namespace swconv {

template <int M, int R>
struct Wino {
  static_assert((M == 2 && R == 3) || (M == 4 && R == 3) || (M == 2 && R == 5) || (M == 4 && R == 5),
                "F(m x m, r x r) not built");
  static constexpr int m = M, r = R, t = M + R - 1;
};

// r = B^T x for one column (or row) of a tile.
//   F(2,3): B^T = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]
//   F(4,3): B^T = [4 0 -5 0 1 0; 0 -4 -4 1 1 0; 0 4 -4 -1 1 0; 0 -2 -1 2 1 0; 0 2 -1 -2 1 0; 0 4 0 -5 0 1]
// (selected by t: B^T depends on the interpolation points only)
template <int T>
__device__ __forceinline__ void bt_apply(const float (&x)[T], float (&r)[T]);

template <>
__device__ __forceinline__ void bt_apply<4>(const float (&x)[4], float (&r)[4]) {
  r[0] = x[0] - x[2];
  r[1] = x[1] + x[2];
  r[2] = x[2] - x[1];
  r[3] = x[1] - x[3];
}

template <>
__device__ __forceinline__ void bt_apply<6>(const float (&x)[6], float (&r)[6]) {
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

//   t = 8:  B^T = [-1 0 21/4 0 -21/4 0 1 0; 0 1 1 -17/4 -17/4 1 1 0; 0 -1 1 17/4 -17/4 -1 1 0;
//                  0 1/2 1/4 -5/2 -5/4 2 1 0; 0 -1/2 1/4 5/2 -5/4 -2 1 0; 0 2 4 -5/2 -5 1/2 1 0;
//                  0 -2 4 5/2 -5 -1/2 1 0; 0 -1 0 21/4 0 -21/4 0 1]
// rows 1..6 come in pairs that share their even-index part and differ in the sign of the odd one
template <>
__device__ __forceinline__ void bt_apply<8>(const float (&x)[8], float (&r)[8]) {
  const float e12 = fmaf(-4.25f, x[4], x[2]) + x[6], o12 = fmaf(-4.25f, x[3], x[1]) + x[5];
  const float e34 = fmaf(0.25f, x[2], fmaf(-1.25f, x[4], x[6])), o34 = fmaf(0.5f, x[1], fmaf(-2.5f, x[3], 2.0f * x[5]));
  const float e56 = fmaf(4.0f, x[2], fmaf(-5.0f, x[4], x[6])), o56 = fmaf(2.0f, x[1], fmaf(-2.5f, x[3], 0.5f * x[5]));
  r[0] = fmaf(5.25f, x[2] - x[4], x[6] - x[0]);
  r[1] = e12 + o12;
  r[2] = e12 - o12;
  r[3] = e34 + o34;
  r[4] = e34 - o34;
  r[5] = e56 + o56;
  r[6] = e56 - o56;
  r[7] = fmaf(5.25f, x[3] - x[5], x[7] - x[1]);
}

// y = A^T z for one column (or row).
//   F(2,3): A^T = [1 1 1 0; 0 1 -1 -1]
//   F(4,3): A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 0; 0 1 1 4 4 0; 0 1 -1 8 -8 1]
//   F(2,5): A^T = [1 1 1 1 1 0; 0 1 -1 2 -2 1]
template <int M, int R>
__device__ __forceinline__ void at_apply(const float (&z)[M + R - 1], float (&y)[M]);

template <>
__device__ __forceinline__ void at_apply<2, 3>(const float (&z)[4], float (&y)[2]) {
  y[0] = z[0] + z[1] + z[2];
  y[1] = z[1] - z[2] - z[3];
}

template <>
__device__ __forceinline__ void at_apply<4, 3>(const float (&z)[6], float (&y)[4]) {
  const float s12 = z[1] + z[2], d12 = z[1] - z[2];
  const float s34 = z[3] + z[4], d34 = z[3] - z[4];
  y[0] = z[0] + s12 + s34;
  y[1] = fmaf(2.0f, d34, d12);
  y[2] = fmaf(4.0f, s34, s12);
  y[3] = fmaf(8.0f, d34, d12) + z[5];
}

template <>
__device__ __forceinline__ void at_apply<2, 5>(const float (&z)[6], float (&y)[2]) {
  const float s12 = z[1] + z[2], d12 = z[1] - z[2];
  const float s34 = z[3] + z[4], d34 = z[3] - z[4];
  y[0] = z[0] + s12 + s34;
  y[1] = fmaf(2.0f, d34, d12) + z[5];
}

//   F(4,5): A^T = [1 1 1 1 1 1 1 0; 0 1 -1 2 -2 1/2 -1/2 0; 0 1 1 4 4 1/4 1/4 0; 0 1 -1 8 -8 1/8 -1/8 1]
template <>
__device__ __forceinline__ void at_apply<4, 5>(const float (&z)[8], float (&y)[4]) {
  const float s12 = z[1] + z[2], d12 = z[1] - z[2];
  const float s34 = z[3] + z[4], d34 = z[3] - z[4];
  const float s56 = z[5] + z[6], d56 = z[5] - z[6];
  y[0] = z[0] + s12 + s34 + s56;
  y[1] = fmaf(2.0f, d34, fmaf(0.5f, d56, d12));
  y[2] = fmaf(4.0f, s34, fmaf(0.25f, s56, s12));
  y[3] = fmaf(8.0f, d34, fmaf(0.125f, d56, d12)) + z[7];
}

// v = B^T d B  (t x t): columns first, then rows.
template <int M, int R>
__device__ __forceinline__ void input_transform(const float (&d)[M + R - 1][M + R - 1],
                                                float (&v)[M + R - 1][M + R - 1]) {
  constexpr int t = Wino<M, R>::t;
  float tmp[t][t];  // B^T d
#pragma unroll
  for (int j = 0; j < t; ++j) {
    float col[t], res[t];
#pragma unroll
    for (int a = 0; a < t; ++a) col[a] = d[a][j];
    bt_apply<t>(col, res);
#pragma unroll
    for (int i = 0; i < t; ++i) tmp[i][j] = res[i];
  }
#pragma unroll
  for (int i = 0; i < t; ++i) bt_apply<t>(tmp[i], v[i]);  // (tmp B)[i][j] = sum_b tmp[i][b] B^T[j][b]
}

// y = A^T z A  (m x m).
template <int M, int R>
__device__ __forceinline__ void output_transform(const float (&z)[M + R - 1][M + R - 1], float (&y)[M][M]) {
  constexpr int t = Wino<M, R>::t;
  float tmp[M][t];  // A^T z
#pragma unroll
  for (int j = 0; j < t; ++j) {
    float col[t], res[M];
#pragma unroll
    for (int i = 0; i < t; ++i) col[i] = z[i][j];
    at_apply<M, R>(col, res);
#pragma unroll
    for (int a = 0; a < M; ++a) tmp[a][j] = res[a];
  }
#pragma unroll
  for (int a = 0; a < M; ++a) at_apply<M, R>(tmp[a], y[a]);
}

// ---- backward pass (Eq. 5, Eq. 6): the transposed 1-D transforms ----

// z = A g for one column (or row) of an m x m tile of dL/dO~:  z_i = sum_a A^T[a][i] g_a.
template <int M, int R>
__device__ __forceinline__ void a_apply(const float (&g)[M], float (&z)[M + R - 1]);

template <>
__device__ __forceinline__ void a_apply<2, 3>(const float (&g)[2], float (&z)[4]) {
  z[0] = g[0];
  z[1] = g[0] + g[1];
  z[2] = g[0] - g[1];
  z[3] = -g[1];
}

template <>
__device__ __forceinline__ void a_apply<2, 5>(const float (&g)[2], float (&z)[6]) {
  const float h = 2.0f * g[1];
  z[0] = g[0];
  z[1] = g[0] + g[1];
  z[2] = g[0] - g[1];
  z[3] = g[0] + h;
  z[4] = g[0] - h;
  z[5] = g[1];
}

template <>
__device__ __forceinline__ void a_apply<4, 5>(const float (&g)[4], float (&z)[8]) {
  const float e1 = g[0] + g[2], o1 = g[1] + g[3];
  const float e2 = fmaf(4.0f, g[2], g[0]), o2 = fmaf(8.0f, g[3], 2.0f * g[1]);
  const float e5 = fmaf(0.25f, g[2], g[0]), o5 = fmaf(0.125f, g[3], 0.5f * g[1]);
  z[0] = g[0];
  z[1] = e1 + o1;
  z[2] = e1 - o1;
  z[3] = e2 + o2;
  z[4] = e2 - o2;
  z[5] = e5 + o5;
  z[6] = e5 - o5;
  z[7] = g[3];
}

template <>
__device__ __forceinline__ void a_apply<4, 3>(const float (&g)[4], float (&z)[6]) {
  const float e = g[0] + g[2], o = g[1] + g[3];                            // even / odd sums
  const float e4 = fmaf(4.0f, g[2], g[0]), o4 = fmaf(8.0f, g[3], 2.0f * g[1]);  // g0 + 4 g2, 2 g1 + 8 g3
  z[0] = g[0];
  z[1] = e + o;
  z[2] = e - o;
  z[3] = e4 + o4;
  z[4] = e4 - o4;
  z[5] = g[3];
}

// d = B f for one column (or row) of a t x t tile of dL/dI_F:  d_a = sum_i B^T[i][a] f_i.
template <int T>
__device__ __forceinline__ void b_apply(const float (&f)[T], float (&d)[T]);

template <>
__device__ __forceinline__ void b_apply<4>(const float (&f)[4], float (&d)[4]) {
  d[0] = f[0];
  d[1] = f[1] - f[2] + f[3];
  d[2] = f[1] + f[2] - f[0];
  d[3] = -f[3];
}

template <>
__device__ __forceinline__ void b_apply<6>(const float (&f)[6], float (&d)[6]) {
  const float s12 = f[1] + f[2], d12 = f[1] - f[2];
  const float s34 = f[3] + f[4], d34 = f[3] - f[4];
  d[0] = 4.0f * f[0];
  d[1] = fmaf(-4.0f, d12, fmaf(-2.0f, d34, 4.0f * f[5]));
  d[2] = fmaf(-5.0f, f[0], fmaf(-4.0f, s12, -s34));
  d[3] = fmaf(2.0f, d34, fmaf(-5.0f, f[5], d12));
  d[4] = f[0] + s12 + s34;
  d[5] = f[5];
}

template <>
__device__ __forceinline__ void b_apply<8>(const float (&f)[8], float (&d)[8]) {
  const float s12 = f[1] + f[2], d12 = f[1] - f[2];
  const float s34 = f[3] + f[4], d34 = f[3] - f[4];
  const float s56 = f[5] + f[6], d56 = f[5] - f[6];
  d[0] = -f[0];
  d[1] = fmaf(0.5f, d34, fmaf(2.0f, d56, d12)) - f[7];
  d[2] = fmaf(5.25f, f[0], fmaf(0.25f, s34, fmaf(4.0f, s56, s12)));
  d[3] = fmaf(-4.25f, d12, fmaf(-2.5f, d34 + d56, 5.25f * f[7]));
  d[4] = fmaf(-5.25f, f[0], fmaf(-4.25f, s12, fmaf(-1.25f, s34, -5.0f * s56)));
  d[5] = fmaf(2.0f, d34, fmaf(0.5f, d56, fmaf(-5.25f, f[7], d12)));
  d[6] = f[0] + s12 + s34 + s56;
  d[7] = f[7];
}

// z = A g A^T  (t x t from m x m): columns first, then rows.
template <int M, int R>
__device__ __forceinline__ void output_grad_transform(const float (&g)[M][M], float (&z)[M + R - 1][M + R - 1]) {
  constexpr int t = Wino<M, R>::t;
  float tmp[t][M];  // A g
#pragma unroll
  for (int b = 0; b < M; ++b) {
    float col[M], res[t];
#pragma unroll
    for (int a = 0; a < M; ++a) col[a] = g[a][b];
    a_apply<M, R>(col, res);
#pragma unroll
    for (int i = 0; i < t; ++i) tmp[i][b] = res[i];
  }
#pragma unroll
  for (int i = 0; i < t; ++i) a_apply<M, R>(tmp[i], z[i]);
}

// d = B f B^T  (t x t).
template <int M, int R>
__device__ __forceinline__ void input_grad_transform(const float (&f)[M + R - 1][M + R - 1],
                                                     float (&d)[M + R - 1][M + R - 1]) {
  constexpr int t = Wino<M, R>::t;
  float tmp[t][t];  // B f
#pragma unroll
  for (int j = 0; j < t; ++j) {
    float col[t], res[t];
#pragma unroll
    for (int i = 0; i < t; ++i) col[i] = f[i][j];
    b_apply<t>(col, res);
#pragma unroll
    for (int a = 0; a < t; ++a) tmp[a][j] = res[a];
  }
#pragma unroll
  for (int a = 0; a < t; ++a) b_apply<t>(tmp[a], d[a]);
}

}  // namespace swconv
