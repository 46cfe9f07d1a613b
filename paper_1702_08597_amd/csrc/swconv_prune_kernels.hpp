// HIP kernels of one pruning step on the stored entries of W_F (Section 4.2, Eq. 8 and Eq. 9):
//   w' = w - eta (dL/dw + lambda sign w)                (SGD step on L + lambda |w|_1, Eq. 9 with Eq. 7)
//   T(w') = 0 if |w'| (|dL/dw| + beta) < eps, else w'   (Eq. 8, gradient taken at the point of the step)
// and the new per-position CSR without the entries T zeroed.  Arithmetic in fp32, one rounding per
// operation: g + lambda*sign(w), one fused multiply-add for w', |g| + beta, the product with |w'|.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace swconv {

__device__ __forceinline__ float pruned_value(float w, float g, float eta, float lambda, float eps, float beta,
                                              bool* drop) {
  const float sgn = w > 0.0f ? 1.0f : (w < 0.0f ? -1.0f : 0.0f);
  const float step = __fadd_rn(g, __fmul_rn(lambda, sgn));
  const float wn = __fmaf_rn(-eta, step, w);
  *drop = __fmul_rn(fabsf(wn), __fadd_rn(fabsf(g), beta)) < eps;
  return wn;
}

// One thread per CSR row: updates the row's values (0 where dropped) and counts what it keeps;
// the count goes to rowptr_out[row + 1] (rowptr_out[0] = 0).
__global__ __launch_bounds__(256) void prune_update_kernel(int64_t rows, const int32_t* __restrict__ rowptr,
                                                           const float* __restrict__ vals,
                                                           const float* __restrict__ grad, float eta, float lambda,
                                                           float eps, float beta, float* __restrict__ updated,
                                                           int32_t* __restrict__ rowptr_out) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row == 0) rowptr_out[0] = 0;
  if (row >= rows) return;
  int kept = 0;
  for (int32_t q = rowptr[row]; q < rowptr[row + 1]; ++q) {
    bool drop;
    const float wn = pruned_value(vals[q], grad[q], eta, lambda, eps, beta, &drop);
    updated[q] = drop ? 0.0f : wn;
    kept += drop ? 0 : 1;
  }
  rowptr_out[row + 1] = kept;
}

// Inclusive scan of rowptr_out[1 .. rows] in place, one workgroup of 1024 threads walking the array
// in chunks of 1024 with a running carry.
__global__ __launch_bounds__(1024) void prune_scan_kernel(int64_t rows, int32_t* __restrict__ rowptr_out) {
  __shared__ int32_t part[1024];
  int32_t carry = 0;
  for (int64_t base = 0; base < rows; base += 1024) {
    const int64_t i = base + threadIdx.x;
    const int32_t v = i < rows ? rowptr_out[i + 1] : 0;
    part[threadIdx.x] = v;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan of the chunk
      const int32_t add = (int)threadIdx.x >= off ? part[threadIdx.x - off] : 0;
      __syncthreads();
      part[threadIdx.x] += add;
      __syncthreads();
    }
    if (i < rows) rowptr_out[i + 1] = carry + part[threadIdx.x];
    carry += part[1023];
    __syncthreads();
  }
}

// One thread per row: copies the kept entries (in their order) to the compacted arrays.  An entry is
// kept exactly when prune_update_kernel kept it: the decision is taken again from the same inputs.
__global__ __launch_bounds__(256) void prune_compact_kernel(int64_t rows, const int32_t* __restrict__ rowptr,
                                                            const int32_t* __restrict__ colidx,
                                                            const float* __restrict__ vals,
                                                            const float* __restrict__ grad, float eta, float lambda,
                                                            float eps, float beta,
                                                            const int32_t* __restrict__ rowptr_out,
                                                            int32_t* __restrict__ colidx_out,
                                                            float* __restrict__ vals_out) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row >= rows) return;
  int32_t dst = rowptr_out[row];
  for (int32_t q = rowptr[row]; q < rowptr[row + 1]; ++q) {
    bool drop;
    const float wn = pruned_value(vals[q], grad[q], eta, lambda, eps, beta, &drop);
    if (!drop) {
      colidx_out[dst] = colidx[q];
      vals_out[dst] = wn;
      ++dst;
    }
  }
}

// Fine-tuning with the sparsity pattern fixed (Section 4.3): only the values of W_F change.  Every
// (offset, weight) pair of a packed stream takes its weight from the caller's CSR value array
// through the pair's index into that array; padding pairs (index -1) keep +0.0f.
__global__ __launch_bounds__(256) void refresh_values_kernel(uint32_t* __restrict__ pairs,
                                                             const int32_t* __restrict__ index, uint32_t n_pairs,
                                                             const float* __restrict__ vals) {
  const uint32_t e = blockIdx.x * 256u + threadIdx.x;
  if (e >= n_pairs) return;
  const int32_t q = index[e];
  if (q >= 0) pairs[2 * (size_t)e + 1] = __float_as_uint(vals[q]);
}

}  // namespace swconv
