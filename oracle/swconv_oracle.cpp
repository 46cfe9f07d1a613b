// CPU oracle for the sparse Winograd-layer forward pass.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
// GPU library is checked against.  It shares no code, header, table or helper
// with the HIP path and must never be linked, imported or called by it.
// Only the test-suite, the smoke check and the benchmark's CPU-baseline leg
// may use it.
//
// What it computes (all citations are to the paper, arxiv 1702.08597):
//   * Section 3, Eq. 4  - the Winograd layer  O = f(I; W_F)  with W_F a free
//     K x C x t x t parameter tensor, t = m + r - 1, read per position as in
//     the remark after Eq. 4's intermediate variables:  Z(:,:,i,j) =
//     W_F(:,:,i,j) * I_F(:,:,i,j)  (a K x C by C x T matrix product for each of
//     the t*t positions; Section 5 names it the second step).
//   * Section 3, Eq. 1  - brute-force direct convolution (cross-correlation,
//     the CNN convention), with optional zero padding, as an independent
//     definition the layer must reduce to when W_F = G w G^T (Eq. 3).
//   * Section 3, Eq. 3  - the helper W_F = G w G^T.
//
//   * Section 3, Eq. 5 and Eq. 6 - the backward pass of the layer: from dL/dO to
//     dL/dZ = A dL/dO~ A^T, dL/dW_F(:,:,i,j) = dL/dZ(:,:,i,j) I_F(:,:,i,j)^T (read at
//     the stored entries of the pruned W_F), dL/dI_F(:,:,i,j) = W_F(:,:,i,j)^T
//     dL/dZ(:,:,i,j), dL/dI~ = B dL/dI_F B^T and the overlap-add through phi.
//
//   * Section 4.2, Eq. 8 and Eq. 9 - one pruning step on the stored entries of W_F:
//     w <- T_{eps,beta}(w - eta (dL/dw + lambda sign w)), T(w) = 0 if |w| (|dL/dw| + beta) < eps,
//     followed by dropping the zeroed entries from the CSR pattern.
//
// Every pin that ties these functions to the paper lives in tests/ (brute
// force on tiny inputs, zero weights, linearity, single non-zero closed form,
// the overlapped-tiling example of Section 3, permutation invariances).
// No function in this file is "parity unpinned".
//
// Readings where the paper is silent (kept identical in the GPU library's
// documentation):
//   * A, B, G are the standard minimal-filtering matrices for interpolation
//     points {0, 1, -1, inf} (F(2,3)), {0, 1, -1, 2, -2, inf} (F(4,3), F(2,5)) and, with 1/2 and -1/2
//     added, F(4,5);
//     Section 3 only says the F(2x2,3x3) ones have entries 0, +-1, +-1/2.
//   * position index p = i*t + j, i = row of the transformed tile.
//   * tile index tau = (n*th + ty)*tw + tx, th = ceil(H_o/m), tw = ceil(W_o/m);
//     the input is virtually zero-extended for padding and for a ragged last
//     tile (footnote to the divisibility assumption in Section 3); outputs
//     outside H_o x W_o are computed and dropped.
//
// Two instantiations of the same plain loops: double (parity ground truth) and
// float (the timed CPU baseline).  OpenMP over independent outer iterations
// only; no blocking, fusion or reordering.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

constexpr int kMaxT = 8;  // largest transformed tile: F(4,5)

struct WinogradMatrices {
  int m, r, t;
  double AT[4][kMaxT];      // m x t   (A^T)
  double BT[kMaxT][kMaxT];  // t x t   (B^T)
  double G[kMaxT][5];       // t x r
};

bool winograd_matrices(int m, int r, WinogradMatrices* w) {
  std::memset(w, 0, sizeof(*w));
  w->m = m;
  w->r = r;
  w->t = m + r - 1;
  if (m == 2 && r == 3) {
    const double BT[4][4] = {{1, 0, -1, 0}, {0, 1, 1, 0}, {0, -1, 1, 0}, {0, 1, 0, -1}};
    const double G[4][3] = {{1, 0, 0}, {0.5, 0.5, 0.5}, {0.5, -0.5, 0.5}, {0, 0, 1}};
    const double AT[2][4] = {{1, 1, 1, 0}, {0, 1, -1, -1}};
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 4; ++j) w->BT[i][j] = BT[i][j];
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 3; ++j) w->G[i][j] = G[i][j];
    for (int i = 0; i < 2; ++i)
      for (int j = 0; j < 4; ++j) w->AT[i][j] = AT[i][j];
    return true;
  }
  if (m == 4 && r == 3) {
    const double BT[6][6] = {{4, 0, -5, 0, 1, 0},  {0, -4, -4, 1, 1, 0}, {0, 4, -4, -1, 1, 0},
                             {0, -2, -1, 2, 1, 0}, {0, 2, -1, -2, 1, 0}, {0, 4, 0, -5, 0, 1}};
    const double G[6][3] = {{1.0 / 4, 0, 0},
                            {-1.0 / 6, -1.0 / 6, -1.0 / 6},
                            {-1.0 / 6, 1.0 / 6, -1.0 / 6},
                            {1.0 / 24, 1.0 / 12, 1.0 / 6},
                            {1.0 / 24, -1.0 / 12, 1.0 / 6},
                            {0, 0, 1}};
    const double AT[4][6] = {
        {1, 1, 1, 1, 1, 0}, {0, 1, -1, 2, -2, 0}, {0, 1, 1, 4, 4, 0}, {0, 1, -1, 8, -8, 1}};
    for (int i = 0; i < 6; ++i)
      for (int j = 0; j < 6; ++j) w->BT[i][j] = BT[i][j];
    for (int i = 0; i < 6; ++i)
      for (int j = 0; j < 3; ++j) w->G[i][j] = G[i][j];
    for (int i = 0; i < 4; ++i)
      for (int j = 0; j < 6; ++j) w->AT[i][j] = AT[i][j];
    return true;
  }
  if (m == 2 && r == 5) {
    // Same six interpolation points as F(4,3), {0, 1, -1, 2, -2, inf}: B^T depends on the points
    // only and is the F(4,3) one; A^T[a][i] = p_i^a and G[i][j] = c_i p_i^j with the F(4,3)
    // scalings c = (1/4, -1/6, -1/6, 1/24, 1/24), the point at infinity taking the last row of
    // A^T and the highest filter coefficient.  (The paper names 5x5 layers, Section 6, without
    // printing matrices; this is the construction its reference for the 3x3 ones uses.)
    const double p[5] = {0, 1, -1, 2, -2};
    const double c[5] = {1.0 / 4, -1.0 / 6, -1.0 / 6, 1.0 / 24, 1.0 / 24};
    const double BT[6][6] = {{4, 0, -5, 0, 1, 0},  {0, -4, -4, 1, 1, 0}, {0, 4, -4, -1, 1, 0},
                             {0, -2, -1, 2, 1, 0}, {0, 2, -1, -2, 1, 0}, {0, 4, 0, -5, 0, 1}};
    for (int i = 0; i < 6; ++i)
      for (int j = 0; j < 6; ++j) w->BT[i][j] = BT[i][j];
    for (int i = 0; i < 5; ++i) {
      double pw = 1;
      for (int j = 0; j < 5; ++j) {
        w->G[i][j] = c[i] * pw;
        if (j < 2) w->AT[j][i] = pw;
        pw *= p[i];
      }
    }
    w->G[5][4] = 1;
    w->AT[1][5] = 1;
    return true;
  }
  if (m == 4 && r == 5) {
    // F(4,5), t = 8: the Toom-Cook construction on the points {0, 1, -1, 2, -2, 1/2, -1/2, inf}.
    // Row i of B^T holds the coefficients (ascending powers) of prod_{k != i} (x - p_k), the row of
    // the point at infinity those of prod_k (x - p_k); A^T[a][i] = p_i^a with the point at infinity
    // in the row of the highest power; G[i][j] = p_i^j / prod_{k != i} (p_i - p_k), last row e_4.
    // All entries of A^T and B^T are dyadic rationals, exact in binary floating point.
    const double BT[8][8] = {{-1, 0, 5.25, 0, -5.25, 0, 1, 0},
                             {0, 1, 1, -4.25, -4.25, 1, 1, 0},
                             {0, -1, 1, 4.25, -4.25, -1, 1, 0},
                             {0, 0.5, 0.25, -2.5, -1.25, 2, 1, 0},
                             {0, -0.5, 0.25, 2.5, -1.25, -2, 1, 0},
                             {0, 2, 4, -2.5, -5, 0.5, 1, 0},
                             {0, -2, 4, 2.5, -5, -0.5, 1, 0},
                             {0, -1, 0, 5.25, 0, -5.25, 0, 1}};
    const double p[7] = {0, 1, -1, 2, -2, 0.5, -0.5};
    for (int i = 0; i < 8; ++i)
      for (int j = 0; j < 8; ++j) w->BT[i][j] = BT[i][j];
    for (int i = 0; i < 7; ++i) {
      double norm = 1;
      for (int k = 0; k < 7; ++k)
        if (k != i) norm *= p[i] - p[k];
      double pw = 1;
      for (int j = 0; j < 5; ++j) {
        w->G[i][j] = pw / norm;
        if (j < 4) w->AT[j][i] = pw;
        pw *= p[i];
      }
    }
    w->G[7][4] = 1;
    w->AT[3][7] = 1;
    return true;
  }
  return false;
}

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Eq. 4, evaluated in the order the paper lists its three steps (Section 5).
template <typename real>
int winograd_layer_forward(int N, int C, int H, int W, int K, int m, int r, int pad,
                           const real* in, const int32_t* rowptr, const int32_t* colidx,
                           const real* vals, real* V_out, real* M_out, real* out) {
  WinogradMatrices wm;
  if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || pad < 0) return 1;
  if (!winograd_matrices(m, r, &wm)) return 2;
  const int t = wm.t, P = t * t;
  const int Ho = H + 2 * pad - r + 1, Wo = W + 2 * pad - r + 1;
  if (Ho < 1 || Wo < 1) return 1;
  const int th = ceil_div(Ho, m), tw = ceil_div(Wo, m);
  const int64_t T = (int64_t)N * th * tw;

  std::vector<real> V_own, M_own;
  real* V = V_out;
  real* M = M_out;
  if (!V) {
    V_own.resize((size_t)P * C * T);
    V = V_own.data();
  }
  if (!M) {
    M_own.resize((size_t)P * K * T);
    M = M_own.data();
  }

  // Step 1: gather phi and input transform  I_F(c,tau,:,:) = B^T I~(c,tau,:,:) B.
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int c = 0; c < C; ++c) {
      for (int ty = 0; ty < th; ++ty) {
        for (int tx = 0; tx < tw; ++tx) {
          const int64_t tau = ((int64_t)n * th + ty) * tw + tx;
          real d[kMaxT][kMaxT], Btd[kMaxT][kMaxT];
          for (int i = 0; i < t; ++i) {
            for (int j = 0; j < t; ++j) {
              const int y = ty * m + i - pad, x = tx * m + j - pad;
              d[i][j] = (y >= 0 && y < H && x >= 0 && x < W)
                            ? in[(((int64_t)n * C + c) * H + y) * W + x]
                            : (real)0;
            }
          }
          for (int i = 0; i < t; ++i) {
            for (int j = 0; j < t; ++j) {
              real s = 0;
              for (int a = 0; a < t; ++a) s += (real)wm.BT[i][a] * d[a][j];
              Btd[i][j] = s;
            }
          }
          for (int i = 0; i < t; ++i) {
            for (int j = 0; j < t; ++j) {
              real s = 0;
              for (int b = 0; b < t; ++b) s += Btd[i][b] * (real)wm.BT[j][b];
              V[((int64_t)(i * t + j) * C + c) * T + tau] = s;
            }
          }
        }
      }
    }
  }

  // Step 2: for every position p, Z(:,:,p) = W_F(:,:,p) * I_F(:,:,p), W_F in CSR.
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
  for (int p = 0; p < P; ++p) {
    for (int k = 0; k < K; ++k) {
      const int64_t row = (int64_t)p * K + k;
      real* Mrow = M + row * T;
      for (int64_t tau = 0; tau < T; ++tau) Mrow[tau] = 0;
      for (int32_t q = rowptr[row]; q < rowptr[row + 1]; ++q) {
        const real w = vals[q];
        const real* Vrow = V + ((int64_t)p * C + colidx[q]) * T;
        for (int64_t tau = 0; tau < T; ++tau) Mrow[tau] += w * Vrow[tau];
      }
    }
  }

  // Step 3: O~(k,tau,:,:) = A^T Z(k,tau,:,:) A, then the scatter psi.
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int k = 0; k < K; ++k) {
      for (int ty = 0; ty < th; ++ty) {
        for (int tx = 0; tx < tw; ++tx) {
          const int64_t tau = ((int64_t)n * th + ty) * tw + tx;
          real z[kMaxT][kMaxT], Atz[4][kMaxT];
          for (int i = 0; i < t; ++i)
            for (int j = 0; j < t; ++j) z[i][j] = M[((int64_t)(i * t + j) * K + k) * T + tau];
          for (int a = 0; a < m; ++a) {
            for (int j = 0; j < t; ++j) {
              real s = 0;
              for (int i = 0; i < t; ++i) s += (real)wm.AT[a][i] * z[i][j];
              Atz[a][j] = s;
            }
          }
          for (int a = 0; a < m; ++a) {
            for (int b = 0; b < m; ++b) {
              real s = 0;
              for (int j = 0; j < t; ++j) s += Atz[a][j] * (real)wm.AT[b][j];
              const int y = ty * m + a, x = tx * m + b;
              if (y < Ho && x < Wo) out[(((int64_t)n * K + k) * Ho + y) * Wo + x] = s;
            }
          }
        }
      }
    }
  }
  return 0;
}

// Eq. 5 and Eq. 6, in the paper's order.  dout: [N][K][Ho][Wo].  Outputs (each optional):
// dZ [P][K][T], dV [P][C][T] (dL/dI_F), dvals [nnz] (dL/dW_F at the stored entries, CSR
// order), din [N][C][H][W].
template <typename real>
int winograd_layer_backward(int N, int C, int H, int W, int K, int m, int r, int pad, const real* in,
                            const int32_t* rowptr, const int32_t* colidx, const real* vals,
                            const real* dout, real* dZ_out, real* dV_out, real* dvals, real* din) {
  WinogradMatrices wm;
  if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || pad < 0) return 1;
  if (!winograd_matrices(m, r, &wm)) return 2;
  const int t = wm.t, P = t * t;
  const int Ho = H + 2 * pad - r + 1, Wo = W + 2 * pad - r + 1;
  if (Ho < 1 || Wo < 1) return 1;
  const int th = ceil_div(Ho, m), tw = ceil_div(Wo, m);
  const int64_t T = (int64_t)N * th * tw;

  std::vector<real> V((size_t)P * C * T), dZ_own, dV_own;
  real* dZ = dZ_out;
  real* dV = dV_out;
  if (!dZ) {
    dZ_own.resize((size_t)P * K * T);
    dZ = dZ_own.data();
  }
  if (!dV) {
    dV_own.resize((size_t)P * C * T);
    dV = dV_own.data();
  }

  // I_F = B^T I~ B, as in the forward pass (Eq. 5 needs it).
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int c = 0; c < C; ++c) {
      for (int ty = 0; ty < th; ++ty) {
        for (int tx = 0; tx < tw; ++tx) {
          const int64_t tau = ((int64_t)n * th + ty) * tw + tx;
          real d[kMaxT][kMaxT], Btd[kMaxT][kMaxT];
          for (int i = 0; i < t; ++i)
            for (int j = 0; j < t; ++j) {
              const int y = ty * m + i - pad, x = tx * m + j - pad;
              d[i][j] = (y >= 0 && y < H && x >= 0 && x < W) ? in[(((int64_t)n * C + c) * H + y) * W + x] : (real)0;
            }
          for (int i = 0; i < t; ++i)
            for (int j = 0; j < t; ++j) {
              real s = 0;
              for (int a = 0; a < t; ++a) s += (real)wm.BT[i][a] * d[a][j];
              Btd[i][j] = s;
            }
          for (int i = 0; i < t; ++i)
            for (int j = 0; j < t; ++j) {
              real s = 0;
              for (int b = 0; b < t; ++b) s += Btd[i][b] * (real)wm.BT[j][b];
              V[((int64_t)(i * t + j) * C + c) * T + tau] = s;
            }
        }
      }
    }
  }

  // Eq. 5, first line: dL/dZ(k,tau,:,:) = A dL/dO~(k,tau,:,:) A^T, where dL/dO~ is dL/dO read
  // through psi^-1 (zero where the tile reaches past H_o x W_o: those outputs were dropped).
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int k = 0; k < K; ++k) {
      for (int ty = 0; ty < th; ++ty) {
        for (int tx = 0; tx < tw; ++tx) {
          const int64_t tau = ((int64_t)n * th + ty) * tw + tx;
          real g[4][4], Ag[kMaxT][4];
          for (int a = 0; a < m; ++a)
            for (int b = 0; b < m; ++b) {
              const int y = ty * m + a, x = tx * m + b;
              g[a][b] = (y < Ho && x < Wo) ? dout[(((int64_t)n * K + k) * Ho + y) * Wo + x] : (real)0;
            }
          for (int i = 0; i < t; ++i)
            for (int b = 0; b < m; ++b) {
              real s = 0;
              for (int a = 0; a < m; ++a) s += (real)wm.AT[a][i] * g[a][b];  // A = (A^T)^T
              Ag[i][b] = s;
            }
          for (int i = 0; i < t; ++i)
            for (int j = 0; j < t; ++j) {
              real s = 0;
              for (int b = 0; b < m; ++b) s += Ag[i][b] * (real)wm.AT[b][j];
              dZ[((int64_t)(i * t + j) * K + k) * T + tau] = s;
            }
        }
      }
    }
  }

  // Eq. 5, second line, at the stored entries: dL/dW_F(k,c,p) = sum_tau dL/dZ(k,tau,p) I_F(c,tau,p).
  if (dvals) {
#pragma omp parallel for collapse(2) schedule(dynamic, 8)
    for (int p = 0; p < P; ++p) {
      for (int k = 0; k < K; ++k) {
        const int64_t row = (int64_t)p * K + k;
        const real* Zrow = dZ + row * T;
        for (int32_t q = rowptr[row]; q < rowptr[row + 1]; ++q) {
          const real* Vrow = V.data() + ((int64_t)p * C + colidx[q]) * T;
          real s = 0;
          for (int64_t tau = 0; tau < T; ++tau) s += Zrow[tau] * Vrow[tau];
          dvals[q] = s;
        }
      }
    }
  }

  // Eq. 6, first line: dL/dI_F(:,:,p) = W_F(:,:,p)^T dL/dZ(:,:,p).
#pragma omp parallel for schedule(dynamic, 1)
  for (int p = 0; p < P; ++p) {
    real* dVp = dV + (int64_t)p * C * T;
    for (int64_t e = 0; e < (int64_t)C * T; ++e) dVp[e] = 0;
    for (int k = 0; k < K; ++k) {
      const int64_t row = (int64_t)p * K + k;
      const real* Zrow = dZ + row * T;
      for (int32_t q = rowptr[row]; q < rowptr[row + 1]; ++q) {
        const real w = vals[q];
        real* dVrow = dVp + (int64_t)colidx[q] * T;
        for (int64_t tau = 0; tau < T; ++tau) dVrow[tau] += w * Zrow[tau];
      }
    }
  }

  // Eq. 6, second and third line: dL/dI~ = B dL/dI_F B^T, summed over every (tau, i', j') that phi
  // maps to the same input pixel.
  if (din) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
      for (int c = 0; c < C; ++c) {
        real* plane = din + ((int64_t)n * C + c) * H * W;
        for (int e = 0; e < H * W; ++e) plane[e] = 0;
        for (int ty = 0; ty < th; ++ty) {
          for (int tx = 0; tx < tw; ++tx) {
            const int64_t tau = ((int64_t)n * th + ty) * tw + tx;
            real f[kMaxT][kMaxT], Bf[kMaxT][kMaxT];
            for (int i = 0; i < t; ++i)
              for (int j = 0; j < t; ++j) f[i][j] = dV[((int64_t)(i * t + j) * C + c) * T + tau];
            for (int a = 0; a < t; ++a)
              for (int j = 0; j < t; ++j) {
                real s = 0;
                for (int i = 0; i < t; ++i) s += (real)wm.BT[i][a] * f[i][j];  // B = (B^T)^T
                Bf[a][j] = s;
              }
            for (int a = 0; a < t; ++a)
              for (int b = 0; b < t; ++b) {
                real s = 0;
                for (int j = 0; j < t; ++j) s += Bf[a][j] * (real)wm.BT[j][b];
                const int y = ty * m + a - pad, x = tx * m + b - pad;
                if (y >= 0 && y < H && x >= 0 && x < W) plane[y * W + x] += s;
              }
          }
        }
      }
    }
  }
  return 0;
}

// Eq. 9 with the L1 penalty of Eq. 7 (its subgradient lambda * sign(w), sign(0) = 0), then the
// thresholding function of Eq. 8 applied to the updated value with the magnitude of the same
// gradient dL/dw(theta^(k)).  One rounding per operation in `real`: the sum g + lambda*sign(w),
// one fused multiply-add for w - eta * (.), the sum |g| + beta, the product with |w'|.
//   updated [nnz]: w' where kept, 0 where thresholded (the pattern of the input)
//   rowptr_out [rows+1], colidx_out / vals_out: the kept entries only (capacity nnz); returns their count
template <typename real>
int64_t prune_step(int64_t rows, const int32_t* rowptr, const int32_t* colidx, const real* vals, const real* grad,
                   real eta, real lambda, real eps, real beta, real* updated, int32_t* rowptr_out,
                   int32_t* colidx_out, real* vals_out) {
  int64_t kept = 0;
  rowptr_out[0] = 0;
  for (int64_t row = 0; row < rows; ++row) {
    for (int32_t q = rowptr[row]; q < rowptr[row + 1]; ++q) {
      const real w = vals[q], g = grad[q];
      const real sgn = w > 0 ? (real)1 : (w < 0 ? (real)-1 : (real)0);
      const real step = g + lambda * sgn;
      const real wn = std::fma(-eta, step, w);
      const bool drop = std::fabs(wn) * (std::fabs(g) + beta) < eps;
      if (updated) updated[q] = drop ? (real)0 : wn;
      if (!drop) {
        colidx_out[kept] = colidx[q];
        vals_out[kept] = wn;
        ++kept;
      }
    }
    rowptr_out[row + 1] = (int32_t)kept;
  }
  return kept;
}

}  // namespace

extern "C" {

int64_t oracle_prune_step_f32(int64_t rows, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                              const float* grad, float eta, float lambda, float eps, float beta, float* updated,
                              int32_t* rowptr_out, int32_t* colidx_out, float* vals_out) {
  return prune_step<float>(rows, rowptr, colidx, vals, grad, eta, lambda, eps, beta, updated, rowptr_out, colidx_out,
                           vals_out);
}
int64_t oracle_prune_step_f64(int64_t rows, const int32_t* rowptr, const int32_t* colidx, const double* vals,
                              const double* grad, double eta, double lambda, double eps, double beta, double* updated,
                              int32_t* rowptr_out, int32_t* colidx_out, double* vals_out) {
  return prune_step<double>(rows, rowptr, colidx, vals, grad, eta, lambda, eps, beta, updated, rowptr_out, colidx_out,
                            vals_out);
}


// Eq. 5 and Eq. 6 in double / float.  dZ, dV, dvals, din may each be NULL.
int oracle_backward_f64(int N, int C, int H, int W, int K, int m, int r, int pad, const double* in,
                        const int32_t* rowptr, const int32_t* colidx, const double* vals, const double* dout,
                        double* dZ, double* dV, double* dvals, double* din) {
  return winograd_layer_backward<double>(N, C, H, W, K, m, r, pad, in, rowptr, colidx, vals, dout, dZ, dV, dvals,
                                         din);
}
int oracle_backward_f32(int N, int C, int H, int W, int K, int m, int r, int pad, const float* in,
                        const int32_t* rowptr, const int32_t* colidx, const float* vals, const float* dout,
                        float* dZ, float* dV, float* dvals, float* din) {
  return winograd_layer_backward<float>(N, C, H, W, K, m, r, pad, in, rowptr, colidx, vals, dout, dZ, dV, dvals,
                                        din);
}


// A^T (m x t), B^T (t x t), G (t x r), row-major, into caller buffers.
int oracle_winograd_matrices(int m, int r, double* AT, double* BT, double* G) {
  WinogradMatrices wm;
  if (!winograd_matrices(m, r, &wm)) return 2;
  for (int a = 0; a < wm.m; ++a)
    for (int j = 0; j < wm.t; ++j) AT[a * wm.t + j] = wm.AT[a][j];
  for (int i = 0; i < wm.t; ++i)
    for (int j = 0; j < wm.t; ++j) BT[i * wm.t + j] = wm.BT[i][j];
  for (int i = 0; i < wm.t; ++i)
    for (int j = 0; j < wm.r; ++j) G[i * wm.r + j] = wm.G[i][j];
  return 0;
}

// Eq. 4 in double.  in: [N][C][H][W]; CSR rows are (p,k) -> p*K+k, global
// offsets; V (optional): [P][C][T]; M (optional): [P][K][T]; out: [N][K][Ho][Wo].
int oracle_forward_f64(int N, int C, int H, int W, int K, int m, int r, int pad, const double* in,
                       const int32_t* rowptr, const int32_t* colidx, const double* vals, double* V,
                       double* M, double* out) {
  return winograd_layer_forward<double>(N, C, H, W, K, m, r, pad, in, rowptr, colidx, vals, V, M,
                                        out);
}

// Same loops in float: the CPU baseline that gets timed.
int oracle_forward_f32(int N, int C, int H, int W, int K, int m, int r, int pad, const float* in,
                       const int32_t* rowptr, const int32_t* colidx, const float* vals, float* V,
                       float* M, float* out) {
  return winograd_layer_forward<float>(N, C, H, W, K, m, r, pad, in, rowptr, colidx, vals, V, M,
                                       out);
}

// Eq. 1 with zero padding, cross-correlation:
//   O[n][k][y][x] = sum_c sum_{u,v<r} w[k][c][u][v] * I[n][c][y+u-pad][x+v-pad].
int oracle_direct_conv_f64(int N, int C, int H, int W, int K, int r, int pad, const double* in,
                           const double* w, double* out) {
  const int Ho = H + 2 * pad - r + 1, Wo = W + 2 * pad - r + 1;
  if (N < 1 || C < 1 || K < 1 || Ho < 1 || Wo < 1 || pad < 0) return 1;
  for (int n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k)
      for (int y = 0; y < Ho; ++y)
        for (int x = 0; x < Wo; ++x) {
          double s = 0;
          for (int c = 0; c < C; ++c)
            for (int u = 0; u < r; ++u)
              for (int v = 0; v < r; ++v) {
                const int yy = y + u - pad, xx = x + v - pad;
                if (yy >= 0 && yy < H && xx >= 0 && xx < W)
                  s += w[(((int64_t)k * C + c) * r + u) * r + v] *
                       in[(((int64_t)n * C + c) * H + yy) * W + xx];
              }
          out[(((int64_t)n * K + k) * Ho + y) * Wo + x] = s;
        }
  return 0;
}

// Eq. 3's weight transform: wf[p][k][c] = (G w[k][c] G^T)[i][j], p = i*t + j.
int oracle_wf_from_spatial_f64(int K, int C, int m, int r, const double* w, double* wf) {
  WinogradMatrices wm;
  if (!winograd_matrices(m, r, &wm)) return 2;
  const int t = wm.t;
  for (int k = 0; k < K; ++k)
    for (int c = 0; c < C; ++c) {
      const double* g = w + ((int64_t)k * C + c) * r * r;
      double Gg[kMaxT][5];
      for (int i = 0; i < t; ++i)
        for (int v = 0; v < r; ++v) {
          double s = 0;
          for (int u = 0; u < r; ++u) s += wm.G[i][u] * g[u * r + v];
          Gg[i][v] = s;
        }
      for (int i = 0; i < t; ++i)
        for (int j = 0; j < t; ++j) {
          double s = 0;
          for (int v = 0; v < r; ++v) s += Gg[i][v] * wm.G[j][v];
          wf[((int64_t)(i * t + j) * K + k) * C + c] = s;
        }
    }
  return 0;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

}  // extern "C"
