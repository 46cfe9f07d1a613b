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
// is one contiguous 256-byte segment.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "winograd_transforms.hpp"

// Cache policy of the row stores of V, M and the output (buffer-instruction aux bits: 1 = sc0,
// 16 = sc1): write-through.  A kernel's output (19-28 MB on the AlexNet-sized layers) otherwise stays
// dirty in the 32 MB of L2 and is written back when the kernel ends, after the compute instead of
// under it; measured 38.8 -> 35.4 us per forward on the N=32 conv3 layer.
#ifndef SWCONV_AUX_V
#define SWCONV_AUX_V 17
#endif
#ifndef SWCONV_AUX_M
#define SWCONV_AUX_M 17
#endif
#ifndef SWCONV_AUX_OUT
#define SWCONV_AUX_OUT 17
#endif

namespace swconv {

struct Geometry {
  int N, C, H, W, K, pad;
  int Ho, Wo, th, tw, tpi;  // tpi = th*tw tiles per image
  int T;                    // N*tpi
  int Tp;                   // padded tile count (row pitch of V and M)
  // LDS staging of the transforms: a block of 64 consecutive tiles touches at most `slots` images,
  // and in each of them a run of whole rows; the runs of a block lie one behind the other in the
  // wave's staging area, each rounded up to a multiple of 64 floats; `in_area` / `out_area` =
  // floats of the largest such area over all blocks
  int slots, in_area, out_area;
  uint32_t v_bytes, m_bytes;  // sizes of the V and M workspaces (both below 4 GiB)
  uint32_t wo_magic;          // ceil(2^32 / Wo): e / Wo == umulhi(e, wo_magic) for every staged element index
  int m_shift;                // log2(m)
  // floats between consecutive images of the input (and dL/dI) and of the output (and dL/dO):
  // C*H*W and K*Ho*Wo for dense tensors, larger when the layer works on a channel group of them
  int64_t in_image_stride, out_image_stride;
};

// V and M are addressed through buffer descriptors: address = base + scalar byte offset (the
// row, wave-uniform) + vector byte offset (the lane), so a row access costs no vector address
// arithmetic.  An access whose vector + scalar offset reaches past `bytes` is dropped by the
// hardware (loads return 0); on gfx950 the scalar offset takes part in that check (measured).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buffer_load_f32(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}
template <int AUX>
__device__ __forceinline__ void buffer_store_f32(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff, float x) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, x), r, (int)voff, (int)soff, AUX);
}
typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
template <int AUX>
__device__ __forceinline__ void buffer_store_f32x2(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff, float x,
                                                   float y) {
  u32x2_t d = {__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y)};
  __builtin_amdgcn_raw_buffer_store_b64(d, r, (int)voff, (int)soff, AUX);
}

// Host-built index tables of the transform kernels (no integer division on the device).
// Per tile (Tp entries; padding tiles have y0 = x0 = -32768 so that every pixel reads as zero):
struct TileInfo {
  int32_t in_org;   // staging-area float offset such that input pixel (y,x) sits at in_org + y*W + x
  int32_t yx0;      // first input row y0 = ty*m - pad (low 16 bits, signed) and column x0 (high 16 bits)
  int32_t ylim;     // first (low 16) and last (high 16) staged input row of the tile's image part
  int32_t out_org;  // staging-area float offset of the tile's first output pixel
};
// Per block of 64 consecutive tiles and image slot (Tp/64 * slots entries): the part of one
// image the block covers.  n < 0 marks an unused slot.
struct BlockImage {
  int32_t n;          // image
  int32_t in_elem0;   // first staged input element inside a channel plane (a whole row start)
  int32_t in_span;    // staged input elements (whole rows)
  int32_t out_elem0;  // first output element of the part inside an output plane (a whole row start)
  int32_t out_span;   // output elements of the part (whole rows)
  int32_t t_lo, t_hi; // first / last tile of the block inside the image (image-local tile index)
  int32_t whole;      // 1 when the part consists of whole tile rows (every pixel of the span is owned)
  int32_t in_off;     // float offset of the part's staged input inside the wave's staging area
  int32_t out_off;    // float offset of the part's output rows inside the wave's staging area
};

// One slice = kSliceRows rows of one position's sparse matrix, rows sorted by length.  32 bytes,
// so a wave fetches a whole descriptor with one scalar load.
struct Slice {
  uint32_t batch0;  // first 512-byte batch of the slice in the packed stream
  int32_t len;      // steps in the slice (one (row offset, weight) pair per row each), a multiple of kStepGroup
  int32_t row0;     // index of its first row in the host's sorted-row table (P * Kp entries)
  int32_t p;        // position
  int32_t k[4];     // output channel of each row, -1 = padding row
};

// One unit of the schedule: a contiguous run of slices of one position, for one tile block.
struct WorkItem {
  int32_t p;
  int32_t tau_block;
  int32_t slice_begin;  // first slice
  int32_t slice_end;    // one past the last slice
};

// What a persistent workgroup needs to start, in one 32-byte scalar load: its range of work
// items and the first of them.
struct RangeHeader {
  int32_t item_begin, item_end;  // indices into the work-item list; never empty for a launched workgroup
  WorkItem first;                // = items[item_begin]
  int32_t pad[2];
};

constexpr int kSliceRows = 4;    // rows per slice = quarters of a wave
constexpr int kTileBlock = 64;   // tiles per panel row: 16 lanes of a quarter x 4 tiles
constexpr int kBatchSteps = 16;  // steps per 512-byte stream batch (one per lane of a quarter)
constexpr int kStepGroup = 4;    // steps issued together; a slice's length is a multiple of it
constexpr int kPanelPieces = 10; // 16-byte panel pieces a thread holds in registers
constexpr int kMaxItemSlices = 256;  // slices per work item: their descriptors are staged in LDS, two 16-byte
                                     // pieces each, one piece per thread of the smallest workgroup (512 threads)
constexpr int kMinItemSlices = 8;    // the least the LDS left over by a large panel must hold
constexpr int kXcds = 8;

// Workgroup ids are dealt round-robin to the 8 XCDs; remap them so that each XCD gets one
// contiguous range of virtual ids (neighbours in the work list then share an L2).
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nblocks) {
  const int per = nblocks / kXcds, rem = nblocks % kXcds;
  const int xcd = bid % kXcds, local = bid / kXcds;
  return xcd * per + (xcd < rem ? xcd : rem) + local;
}

// ---------------------------------------------------------------------------------------------
// Step 1: gather phi + V = B^T d B.  A wave owns one channel and 64 consecutive tiles: it copies
// the input rows those tiles touch into its private LDS area with lane-contiguous (coalesced)
// loads - each pixel is read from memory once although up to (t/m)^2 tiles use it; the loads of
// up to four images are all in flight before the first LDS write - then every lane gathers its
// t x t tile from LDS (clamped addresses, all reads issued back to back, then selects zero what
// lies outside the image), transforms it in registers and stores one value per position:
// 64 lanes -> 256 contiguous bytes of V[p][c][.], addressed as wave-uniform row + lane.
// Block = 4 waves = 4 channels of the same tile block.
template <int M, int R>
__global__ __launch_bounds__(256) void input_transform_kernel(const float* __restrict__ in, float* __restrict__ V,
                                                              const TileInfo* __restrict__ tiles,
                                                              const BlockImage* __restrict__ blocks,
                                                              const Geometry g) {
  constexpr int t = Wino<M, R>::t;
  extern __shared__ float stage[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.y * 4 + wave;
  const int tau0 = blockIdx.x * 64;
  float* my = stage + wave * g.in_area;
  const BlockImage* bi = blocks + (size_t)blockIdx.x * g.slots;
  const size_t plane = (size_t)g.H * g.W;
  const TileInfo ti = tiles[tau0 + lane];  // asked for first: it arrives while the rows are staged
  if (c < g.C) {
    // Each image part is read through its own buffer descriptor (base = first staged element,
    // size = the part's bytes): lanes past the end read zeros, so loads and LDS writes need no
    // lane predicates; every part's run is padded to a multiple of 64 floats to take the zero tail.
    constexpr int IG = 4, EL = 4;  // images x loads per lane in flight
    for (int s0 = 0; s0 < g.slots; s0 += IG) {
      __amdgpu_buffer_rsrc_t src[IG];
      float* dst[IG];
      int span[IG], max_span = 0;
#pragma unroll
      for (int i = 0; i < IG; ++i) {
        const int sidx = min(s0 + i, g.slots - 1);
        const BlockImage b = bi[sidx];
        const bool used = s0 + i < g.slots && b.n >= 0;
        span[i] = used ? b.in_span : 0;
        src[i] = make_rsrc(in + (size_t)max(b.n, 0) * g.in_image_stride + c * plane + b.in_elem0, (uint32_t)span[i] * 4u);
        dst[i] = my + b.in_off + lane;
        max_span = max(max_span, span[i]);
      }
      for (int e0 = 0; e0 < max_span; e0 += 64 * EL) {
        float buf[IG][EL];
#pragma unroll
        for (int i = 0; i < IG; ++i)
#pragma unroll
          for (int u = 0; u < EL; ++u)
            if (e0 + u * 64 < span[i]) buf[i][u] = buffer_load_f32(src[i], (lane + u * 64) * 4u, e0 * 4u);
#pragma unroll
        for (int i = 0; i < IG; ++i)
#pragma unroll
          for (int u = 0; u < EL; ++u)
            if (e0 + u * 64 < span[i]) dst[i][e0 + u * 64] = buf[i][u];
      }
    }
  }
  __syncthreads();
  if (c >= g.C) return;
  float d[t][t];
  {
    const int y0 = (int16_t)(ti.yx0 & 0xffff), x0 = ti.yx0 >> 16;
    const int y_lo = ti.ylim & 0xffff, y_last = ti.ylim >> 16;
    const float* img = my + ti.in_org;
    int xo[t];
    bool xok[t];
#pragma unroll
    for (int j = 0; j < t; ++j) {
      const int x = x0 + j;
      xok[j] = x >= 0 && x < g.W;
      xo[j] = min(max(x, 0), g.W - 1);
    }
#pragma unroll
    for (int i = 0; i < t; ++i) {
      const float* row = img + min(max(y0 + i, y_lo), y_last) * g.W;  // a staged row in any case
#pragma unroll
      for (int j = 0; j < t; ++j) d[i][j] = row[xo[j]];
    }
    // all t*t reads are issued above; pinning the values here keeps the compiler from turning
    // the selects below into one guarded (and serialised) read each
#pragma unroll
    for (int i = 0; i < t; ++i) {
      if constexpr (t == 8)
        asm volatile("" : "+v"(d[i][0]), "+v"(d[i][1]), "+v"(d[i][2]), "+v"(d[i][3]), "+v"(d[i][4]), "+v"(d[i][5]),
                          "+v"(d[i][6]), "+v"(d[i][7]));
      else if constexpr (t == 6)
        asm volatile("" : "+v"(d[i][0]), "+v"(d[i][1]), "+v"(d[i][2]), "+v"(d[i][3]), "+v"(d[i][4]), "+v"(d[i][5]));
      else
        asm volatile("" : "+v"(d[i][0]), "+v"(d[i][1]), "+v"(d[i][2]), "+v"(d[i][3]));
    }
#pragma unroll
    for (int i = 0; i < t; ++i) {
      const int y = y0 + i;
      const bool yok = y >= 0 && y < g.H;
#pragma unroll
      for (int j = 0; j < t; ++j) d[i][j] = (yok && xok[j]) ? d[i][j] : 0.0f;
    }
  }
  float v[t][t];
  input_transform<M, R>(d, v);
  const __amdgpu_buffer_rsrc_t vr = make_rsrc(V, g.v_bytes);
  const uint32_t row0 = ((uint32_t)c * g.Tp + tau0) * 4u;        // wave-uniform byte offset, position 0
  const uint32_t pstride = (uint32_t)g.C * (uint32_t)g.Tp * 4u;  // bytes between positions
  uint32_t soff = row0;  // one scalar add per store
#pragma unroll
  for (int i = 0; i < t; ++i)
#pragma unroll
    for (int j = 0; j < t; ++j) {
      buffer_store_f32<SWCONV_AUX_V>(vr, lane * 4u, soff, v[i][j]);
      soff += pstride;
      asm volatile("" : "+s"(soff));
    }
}

// ---------------------------------------------------------------------------------------------
// Step 2: M[p] = W_F[p] * V[p] on the plain fp32 ALUs.
//
// Persistent workgroups: the host cuts the sequence of all (position, tile block, slice) units
// into one contiguous, equal-cost range per workgroup; range r is run by the workgroup whose id
// maps to r under xcd_contiguous_id, so neighbouring ranges - which share panels and weights -
// share an XCD's L2.  A range is a short list of work items (runs of slices of one panel).  For an
// item the workgroup stages the C x 64 panel V[p][:, tau_block] in LDS, then the waves draw the
// item's slices from a shared counter, longest first.
//
// Lanes <-> tiles (Section 5: vectorise over tiles), four tiles per lane and four rows per wave:
// a slice has four rows and each quarter of a wave (16 lanes) works on one of them.  Lane (q, s)
// owns row q and the tiles 4s .. 4s+3 of the 64-tile block, so one 16-byte LDS read per lane
// feeds four FMAs, and one address addition serves four non-zeros x 64 tiles: 5 vector-ALU
// instructions per 256 tile-FMAs.  That matters because the vector ALU (one wave instruction per
// SIMD per 4 clocks) and LDS (a 16-byte-per-lane read per 4.8 clocks per CU, whether the quarters
// read one row or four different ones) are both close to saturated by this loop.
// The (row offset, weight) pairs differ between the quarters, so they travel through vector
// memory, 16 steps per load: lane (q, s) fetches the pair of row q, step 16 b + s, and at step i
// every lane of a quarter takes the pair from lane i of its quarter with a DPP row broadcast,
// folded into the address addition and into the FMAs.
//
// Stream layout: per slice, batches of 512 bytes; batch b holds [q][s] -> (offset, weight) of row
// q, step 16 b + s; rows shorter than the slice are padded with (0, +0.0f).  A slice's length is
// a multiple of kStepGroup steps.  Panel rows are 64 tiles = 256 bytes.

template <int I>
__device__ __forceinline__ uint32_t quarter_bcast(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x150 + I, 0xf, 0xf, true);  // row_newbcast:I
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned u32x4v_t __attribute__((ext_vector_type(4)));

// The four accumulators of a lane (its four tiles); separate scalars, so that the inline-asm FMAs
// update them in place.
struct Acc4 {
  float a0, a1, a2, a3;
};

// acc += w * x with w taken from lane I of the lane's quarter.  The broadcast rides on the FMAs
// themselves (DPP operand); the compiler would spend a separate move on it.  `bw` is only ever
// written by a memory load, and FIRST puts two wait states in front, so the rule "two wait states
// between a vector-ALU write of a register and a DPP read of it" holds whatever precedes the group.
template <int I, bool FIRST>
__device__ __forceinline__ void quarter_fma(Acc4& acc, uint32_t bw, const f32x4_t& x) {
#define SWCONV_QFMA(N)                                                                         \
  "v_fmac_f32_dpp %0, %4, %5 row_newbcast:" #N " row_mask:0xf bank_mask:0xf\n"                 \
  "v_fmac_f32_dpp %1, %4, %6 row_newbcast:" #N " row_mask:0xf bank_mask:0xf\n"                 \
  "v_fmac_f32_dpp %2, %4, %7 row_newbcast:" #N " row_mask:0xf bank_mask:0xf\n"                 \
  "v_fmac_f32_dpp %3, %4, %8 row_newbcast:" #N " row_mask:0xf bank_mask:0xf"
#define SWCONV_QFMA_CASE(N)                                                                    \
  if constexpr (I == N) {                                                                      \
    if constexpr (FIRST)                                                                       \
      asm("s_nop 1\n" SWCONV_QFMA(N)                                                           \
          : "+v"(acc.a0), "+v"(acc.a1), "+v"(acc.a2), "+v"(acc.a3)                             \
          : "v"(bw), "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]));                              \
    else                                                                                       \
      asm(SWCONV_QFMA(N)                                                                       \
          : "+v"(acc.a0), "+v"(acc.a1), "+v"(acc.a2), "+v"(acc.a3)                             \
          : "v"(bw), "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]));                              \
  }
  SWCONV_QFMA_CASE(0) SWCONV_QFMA_CASE(1) SWCONV_QFMA_CASE(2) SWCONV_QFMA_CASE(3)
  SWCONV_QFMA_CASE(4) SWCONV_QFMA_CASE(5) SWCONV_QFMA_CASE(6) SWCONV_QFMA_CASE(7)
  SWCONV_QFMA_CASE(8) SWCONV_QFMA_CASE(9) SWCONV_QFMA_CASE(10) SWCONV_QFMA_CASE(11)
  SWCONV_QFMA_CASE(12) SWCONV_QFMA_CASE(13) SWCONV_QFMA_CASE(14) SWCONV_QFMA_CASE(15)
#undef SWCONV_QFMA_CASE
#undef SWCONV_QFMA
}

// The four panel reads of steps G*kStepGroup .. +kStepGroup-1 of the batch whose row offsets are in
// boff, issued back to back.
struct Group4 {
  f32x4_t x0, x1, x2, x3;
};
template <int G>
__device__ __forceinline__ Group4 quarter_reads(const float* panel, uint32_t lane_sub, uint32_t boff) {
  constexpr int I0 = G * kStepGroup;
  static_assert(kStepGroup == 4, "four steps per group");
  const char* base = reinterpret_cast<const char*>(panel);
  Group4 g;
  g.x0 = *reinterpret_cast<const f32x4_t*>(base + (quarter_bcast<I0 + 0>(boff) + lane_sub));
  g.x1 = *reinterpret_cast<const f32x4_t*>(base + (quarter_bcast<I0 + 1>(boff) + lane_sub));
  g.x2 = *reinterpret_cast<const f32x4_t*>(base + (quarter_bcast<I0 + 2>(boff) + lane_sub));
  g.x3 = *reinterpret_cast<const f32x4_t*>(base + (quarter_bcast<I0 + 3>(boff) + lane_sub));
  return g;
}

// Steps G*kStepGroup .. +kStepGroup-1 of the batch held in (boff, bw): the reads, then the FMAs as
// the data arrives.
template <int G>
__device__ __forceinline__ void quarter_group(const float* panel, uint32_t lane_sub, uint32_t boff, uint32_t bw,
                                              Acc4& acc) {
  constexpr int I0 = G * kStepGroup;
  const Group4 g = quarter_reads<G>(panel, lane_sub, boff);
  quarter_fma<I0 + 0, true>(acc, bw, g.x0);
  quarter_fma<I0 + 1, false>(acc, bw, g.x1);
  quarter_fma<I0 + 2, false>(acc, bw, g.x2);
  quarter_fma<I0 + 3, false>(acc, bw, g.x3);
}

// The first `steps` (a positive multiple of kStepGroup, wave-uniform) steps of one batch.
__device__ __forceinline__ void quarter_batch(const float* panel, uint32_t lane_sub, const u32x2_t& b, int steps,
                                              Acc4& acc) {
  quarter_group<0>(panel, lane_sub, b.x, b.y, acc);
  if (steps > 1 * kStepGroup) quarter_group<1>(panel, lane_sub, b.x, b.y, acc);
  if (steps > 2 * kStepGroup) quarter_group<2>(panel, lane_sub, b.x, b.y, acc);
  if (steps > 3 * kStepGroup) quarter_group<3>(panel, lane_sub, b.x, b.y, acc);
}

// The rolling unit of the inner loop (see swconv_rolling_unit.inc): the same steps as quarter_batch over
// two batches, as one pipeline with four reads always in flight, in assembly with the sixteen registers
// of those reads fixed: v[112:127], the top of the 128 registers of the fused F(4x4,3x3) kernel, whose
// other registers are full of accumulators.  (In the stand-alone product kernel below the compiler's
// group-by-group code is as fast: there memory, not the inner loop, sets the pace.)
constexpr int kUnitSteps = 2 * kBatchSteps;
#define SWCONV_UNIT_NAME unit_rolling_hi
#define SWCONV_XR0 112
#define SWCONV_XR1 113
#define SWCONV_XR2 114
#define SWCONV_XR3 115
#define SWCONV_XR4 116
#define SWCONV_XR5 117
#define SWCONV_XR6 118
#define SWCONV_XR7 119
#define SWCONV_XR8 120
#define SWCONV_XR9 121
#define SWCONV_XR10 122
#define SWCONV_XR11 123
#define SWCONV_XR12 124
#define SWCONV_XR13 125
#define SWCONV_XR14 126
#define SWCONV_XR15 127
#include "swconv_rolling_unit.inc"
#undef SWCONV_UNIT_NAME
#undef SWCONV_XR0
#undef SWCONV_XR1
#undef SWCONV_XR2
#undef SWCONV_XR3
#undef SWCONV_XR4
#undef SWCONV_XR5
#undef SWCONV_XR6
#undef SWCONV_XR7
#undef SWCONV_XR8
#undef SWCONV_XR9
#undef SWCONV_XR10
#undef SWCONV_XR11
#undef SWCONV_XR12
#undef SWCONV_XR13
#undef SWCONV_XR14
#undef SWCONV_XR15

// ---- sampled mode (backward pass, Eq. 5 second line): dL/dW_F at the stored entries ----
// The same walk over the packed W_F, but instead of accumulating w * x into the row, every stored
// entry (k, c) gets the dot product of dL/dZ[p][k][.] with the panel row of c over the 64 tiles of
// the block: the lane multiplies its four tiles, the 16 lanes of the quarter are summed with DPP
// exchanges, and lane i of the quarter ends up with the sum of step i, so that after a batch every
// lane holds the partial sum of "its" stream entry and the wave stores 256 contiguous bytes.

// x + (the value of `send` in the lane given by the DPP control): one v_add_f32 with a DPP operand.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x, float send) {
  return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, send), CTRL, 0xf, 0xf, true));
}

// Steps G*kStepGroup .. +kStepGroup-1: the lane's share (its four tiles) of each step's dot product.
template <int G>
__device__ __forceinline__ void sampled_group(const float* panel, uint32_t lane_sub, uint32_t boff, const f32x4_t& z,
                                              float (&d)[kBatchSteps]) {
  constexpr int I0 = G * kStepGroup;
  const Group4 g = quarter_reads<G>(panel, lane_sub, boff);
  const f32x4_t* x[4] = {&g.x0, &g.x1, &g.x2, &g.x3};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const f32x4_t& v = *x[i];
    float p = z[0] * v[0];
    p = fmaf(z[1], v[1], p);
    p = fmaf(z[2], v[2], p);
    d[I0 + i] = fmaf(z[3], v[3], p);
  }
}

// The first `steps` steps of one batch; returns, in lane (q, i), the partial sum of row q, step i
// (0 for steps that were not run).  Every lane first collects its share of all 16 steps; the 16
// lanes of a quarter then add them up in a transposing butterfly: in the stage with partner
// lane ^ 15 (then ^ 7, ^ 3, ^ 1: the DPP mirror and quad patterns) a lane keeps the half of its
// values whose step has the lane's own bit 3 (2, 1, 0) and adds the partner's values for that
// half, so 8 + 4 + 2 + 1 additions leave the total of step i in lane i - against four additions
// per step for a reduction step by step.
__device__ __forceinline__ float sampled_batch(const float* panel, uint32_t lane_sub, const u32x2_t& b, int steps,
                                               const f32x4_t& z, int lane_in_quarter) {
  float d[kBatchSteps];
#pragma unroll
  for (int i = 0; i < kBatchSteps; ++i) d[i] = 0.0f;
  sampled_group<0>(panel, lane_sub, b.x, z, d);
  if (steps > 1 * kStepGroup) sampled_group<1>(panel, lane_sub, b.x, z, d);
  if (steps > 2 * kStepGroup) sampled_group<2>(panel, lane_sub, b.x, z, d);
  if (steps > 3 * kStepGroup) sampled_group<3>(panel, lane_sub, b.x, z, d);
  const bool b3 = lane_in_quarter & 8, b2 = lane_in_quarter & 4, b1 = lane_in_quarter & 2, b0 = lane_in_quarter & 1;
  float e[8], f[4], g[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) e[i] = dpp_add<0x140>(b3 ? d[i + 8] : d[i], b3 ? d[i] : d[i + 8]);  // row_mirror: lane ^ 15
#pragma unroll
  for (int i = 0; i < 4; ++i) f[i] = dpp_add<0x141>(b2 ? e[i + 4] : e[i], b2 ? e[i] : e[i + 4]);  // row_half_mirror: lane ^ 7
#pragma unroll
  for (int i = 0; i < 2; ++i) g[i] = dpp_add<0x1B>(b1 ? f[i + 2] : f[i], b1 ? f[i] : f[i + 2]);   // quad_perm [3,2,1,0]: lane ^ 3
  return dpp_add<0xB1>(b0 ? g[1] : g[0], b0 ? g[0] : g[1]);                                      // quad_perm [1,0,3,2]: lane ^ 1
}

// SAMPLED = false: Mbuf[p] = A[p] * V[p] (forward step 2; backward Eq. 6 first line on the packed
// transpose).  SAMPLED = true: Mbuf is read (dL/dZ), and partial[tau_block][stream entry] gets the
// entry's dot product over that tile block (Eq. 5 second line; `partial_stride` entries per block).
template <int NWAVES, bool SAMPLED>
__global__ __launch_bounds__(NWAVES * 64, NWAVES == 12 ? 6 : 4) void spmm_kernel(
    const float* __restrict__ V, float* __restrict__ Mbuf, const uint32_t* __restrict__ stream, uint32_t stream_bytes,
    const Slice* __restrict__ slices, int n_slices, const WorkItem* __restrict__ items,
    const RangeHeader* __restrict__ ranges, int n_wgs, int C, int K, int Tp, uint32_t m_bytes, uint32_t v_bytes,
    float* __restrict__ partial, uint32_t partial_stride) {
  constexpr int NT = NWAVES * 64;
  constexpr int TB = kTileBlock;
  typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
  // LDS: the panel [C][64] at offset 0 of the workgroup, the slice counter (64 bytes), then the
  // descriptors of the item's slices
  extern __shared__ float panel[];
  int* next_slice = reinterpret_cast<int*>(panel + (size_t)C * TB);
  u32x4_t* desc = reinterpret_cast<u32x4_t*>(panel + (size_t)C * TB + 16);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const RangeHeader hdr = ranges[xcd_contiguous_id(blockIdx.x, n_wgs)];
  const int quarter = lane >> 4;
  const uint32_t lane_sub = (uint32_t)(lane & 15) * 16u;  // byte offset of the lane's four tiles in a row
  const __amdgpu_buffer_rsrc_t mr = make_rsrc(Mbuf, m_bytes);
  const __amdgpu_buffer_rsrc_t sr = make_rsrc(stream, stream_bytes);
  const __amdgpu_buffer_rsrc_t dr = make_rsrc(slices, (uint32_t)n_slices * (uint32_t)sizeof(Slice));
  const uint32_t lane8 = (uint32_t)lane * 8u;

  // Panel staging: thread i moves the 16-byte pieces i, i + NT, ... of a panel; their offsets
  // inside a panel are the same for every item, so they are computed once.  The next item's panel
  // travels through registers.  Vector-memory results come back in issue order and the stream
  // batches use the same path, so a wave asks for the next panel only after its last slice of the
  // item: a wait on a batch never has a panel load in front of it.  (Surplus pieces are parked
  // past the end of the buffer and read 0 without touching memory.)  The descriptors of the item's
  // slices (32 bytes each, at most kMaxItemSlices) are staged the same way, one 16-byte piece per
  // thread: drawing a slice then costs an LDS atomic and an LDS read, and no scalar-memory load -
  // which shares its counter with the LDS reads of the inner loop - is in flight while it runs.
  constexpr int v4_per_row = TB / 4;
  const int total = C * v4_per_row;
  const __amdgpu_buffer_rsrc_t vr = make_rsrc(V, v_bytes);
  uint32_t voff[kPanelPieces];
#pragma unroll
  for (int u = 0; u < kPanelPieces; ++u) {
    const int idx = threadIdx.x + u * NT;
    const int row = idx / v4_per_row, q = idx % v4_per_row;
    voff[u] = idx < total ? ((uint32_t)row * Tp + q * 4) * 4u : 0xfffffff0u;
  }
  u32x4_t piece[kPanelPieces], desc_piece;
  auto load_batch = [&](uint32_t byte_off) -> u32x2_t {
    return __builtin_amdgcn_raw_buffer_load_b64(sr, (int)lane8, (int)byte_off, 0);  // past the end: reads 0
  };

  // A slice as the loop holds it: stream position and length in scalar registers, the output
  // channel of the lane's quarter in a vector register (-1 = padding row).
  struct Cur {
    uint32_t base;  // byte offset of the slice's first batch
    int len;        // steps
    int k;          // per lane
  };
  auto quarter_k = [&](int k0, int k1, int k2, int k3) {
    return quarter == 0 ? k0 : quarter == 1 ? k1 : quarter == 2 ? k2 : k3;
  };

  // Start of an item, issued as early as the item is known (for the first one: right after the
  // range header; for the others: after the wave's last slice of the item before): the panel
  // pieces and the descriptor piece, then the wave's first slice descriptor and its first two
  // batches, which arrive right behind the panel, so the first slice starts without another
  // memory round trip.
  Cur cur;
  u32x2_t b0 = {0u, 0u}, b1 = {0u, 0u};
  // sampled mode: the lane's four tiles of the dL/dZ row of its quarter (zeros for a padding row)
  f32x4_t z_cur = {0.0f, 0.0f, 0.0f, 0.0f};
  auto row_offset = [&](int p, int tau0, int k) -> uint32_t {  // quarters of padding rows are parked beyond the buffer
    return k >= 0 ? (((uint32_t)p * K + (uint32_t)k) * Tp + tau0) * 4u + lane_sub : 0xfffffff0u;
  };
  auto load_z = [&](int p, int tau0, int k) -> f32x4_t {
    return __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(mr, (int)row_offset(p, tau0, k), 0, 0));
  };
  auto start_item = [&](const WorkItem& w) {
    const uint32_t soff = ((uint32_t)w.p * C * Tp + (uint32_t)w.tau_block * TB) * 4u;
#pragma unroll
    for (int u = 0; u < kPanelPieces; ++u)
      piece[u] = __builtin_amdgcn_raw_buffer_load_b128(vr, (int)voff[u], (int)soff, 0);
    const int n_desc_pieces = 2 * (w.slice_end - w.slice_begin);
    desc_piece = __builtin_amdgcn_raw_buffer_load_b128(
        dr, (int)((int)threadIdx.x < n_desc_pieces ? threadIdx.x * 16u : 0xfffffff0u),
        (int)((uint32_t)w.slice_begin * (uint32_t)sizeof(Slice)), 0);
    const Slice sl = slices[min(w.slice_begin + wave, n_slices - 1)];  // clamped: unconditional, in bounds
    cur.base = sl.batch0 * 512u;
    cur.len = sl.len;
    cur.k = quarter_k(sl.k[0], sl.k[1], sl.k[2], sl.k[3]);
    b0 = load_batch(cur.base);
    b1 = load_batch(cur.base + 512u);
    if constexpr (SAMPLED) z_cur = load_z(w.p, w.tau_block * TB, cur.k);
  };

  WorkItem it = hdr.first;
  start_item(it);
  for (int item = hdr.item_begin;; ++item) {
    const int tau0 = it.tau_block * TB;
    const int n_item_slices = it.slice_end - it.slice_begin;
    // sampled mode: this tile block's row of the partial-sum buffer, one float per stream entry
    const __amdgpu_buffer_rsrc_t pr =
        make_rsrc(SAMPLED ? partial + (size_t)it.tau_block * partial_stride : nullptr, SAMPLED ? partial_stride * 4u : 0u);
    const bool has_next = item + 1 < hdr.item_end;
    const WorkItem it_next = items[has_next ? item + 1 : item];
    if (item != hdr.item_begin) __syncthreads();  // every wave is done with the previous panel and descriptors
#pragma unroll
    for (int u = 0; u < kPanelPieces; ++u) {
      const int idx = threadIdx.x + u * NT;
      if (idx < total) *reinterpret_cast<u32x4_t*>(panel + idx * 4) = piece[u];
    }
    if ((int)threadIdx.x < 2 * n_item_slices) desc[threadIdx.x] = desc_piece;
    if (threadIdx.x == 0) *next_slice = NWAVES;  // item-local index of the first slice to be drawn
    __syncthreads();

    // Waves take slices dynamically, longest first: the first one by wave number, every further
    // one from a counter in LDS.  The next slice is drawn before the current one is computed.
    if (wave < n_item_slices) {
      while (true) {
        int drawn = 0;
        if (lane == 0) drawn = __hip_atomic_fetch_add(next_slice, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const int i_next = __builtin_amdgcn_readfirstlane(drawn);
        const bool more = i_next < n_item_slices;
        const int i_desc = min(i_next, n_item_slices - 1);  // clamped: the read stays inside the staged part
        const u32x4_t d_head = desc[2 * i_desc], d_k = desc[2 * i_desc + 1];  // all lanes read the same 32 bytes
        Acc4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        // Two batch registers in turn: batch j of a slice sits in register j % 2.  A register is
        // refilled right after its batch is consumed, unconditionally, with the batch two ahead -
        // or, when the slice has no such batch, with batch 0 / 1 of the NEXT slice (parked past
        // the end of the stream when there is none: reads 0, touches no memory).  So the batches
        // of a slice are always on their way one or two batches of work before they are needed,
        // and no wait in the loop ever has more than one younger load in front of it.
        Cur nxt;
        nxt.base = more ? (uint32_t)__builtin_amdgcn_readfirstlane((int)d_head.x) * 512u : 0xfffff000u;
        nxt.len = __builtin_amdgcn_readfirstlane((int)d_head.y);
        nxt.k = quarter_k((int)d_k.x, (int)d_k.y, (int)d_k.z, (int)d_k.w);
        const int batches = (cur.len + kBatchSteps - 1) / kBatchSteps;
        f32x4_t z_next = {0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (SAMPLED) z_next = load_z(it.p, tau0, more ? nxt.k : -1);
        for (int j = 0, remaining = cur.len; j < batches; j += 2, remaining -= 2 * kBatchSteps) {
          if constexpr (SAMPLED) {
            const float r0 = sampled_batch(panel, lane_sub, b0, remaining, z_cur, lane & 15);
            buffer_store_f32<SWCONV_AUX_M>(pr, lane * 4u, cur.base / 2u + (uint32_t)j * 256u, r0);
          } else {
            quarter_batch(panel, lane_sub, b0, remaining, acc);
          }
          b0 = load_batch(j + 2 < batches ? cur.base + (uint32_t)(j + 2) * 512u : nxt.base);
          if (j + 1 < batches) {
            if constexpr (SAMPLED) {
              const float r1 = sampled_batch(panel, lane_sub, b1, remaining - kBatchSteps, z_cur, lane & 15);
              buffer_store_f32<SWCONV_AUX_M>(pr, lane * 4u, cur.base / 2u + (uint32_t)(j + 1) * 256u, r1);
            } else {
              quarter_batch(panel, lane_sub, b1, remaining - kBatchSteps, acc);
            }
          }
          b1 = load_batch(j + 3 < batches ? cur.base + (uint32_t)(j + 3) * 512u : nxt.base + 512u);
        }
        if (batches == 0) {  // an all-empty slice consumed nothing: fetch the next slice's batches here
          b0 = load_batch(nxt.base);
          b1 = load_batch(nxt.base + 512u);
        }
        if constexpr (!SAMPLED) {
          const u32x4v_t result = {__float_as_uint(acc.a0), __float_as_uint(acc.a1), __float_as_uint(acc.a2),
                                   __float_as_uint(acc.a3)};
          __builtin_amdgcn_raw_buffer_store_b128(result, mr, (int)row_offset(it.p, tau0, cur.k), 0, SWCONV_AUX_M);
        }
        if (!more) break;
        cur = nxt;
        z_cur = z_next;
      }
    }
    if (!has_next) break;
    it = it_next;
    start_item(it);
  }
}

// ---------------------------------------------------------------------------------------------
// Step 3: Y = A^T z A + scatter psi.  A wave owns one output channel and 64 consecutive tiles:
// each lane reads its t*t values of M (256 contiguous bytes per wave and position), transforms
// them in registers and drops its m x m outputs into the wave's LDS area laid out like the output
// rows; the wave then writes those rows out with lane-contiguous stores (whole image planes when
// the block covers whole images).  Pixels of tiles that belong to a neighbouring block are
// skipped.  Block = 4 waves = 4 output channels of the same tile block.
template <int M, int R>
__global__ __launch_bounds__(256) void output_transform_kernel(const float* __restrict__ Mbuf,
                                                               float* __restrict__ out,
                                                               const TileInfo* __restrict__ tiles,
                                                               const BlockImage* __restrict__ blocks,
                                                               const Geometry g) {
  constexpr int t = Wino<M, R>::t;
  extern __shared__ float stage[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int k = blockIdx.y * 4 + wave;
  const int tau0 = blockIdx.x * 64;
  if (tau0 >= g.T) return;  // whole block is padding (uniform for the block)
  float* my = stage + wave * g.out_area;
  const TileInfo ti = tiles[tau0 + lane];  // asked for before the t*t loads below, used after them
  if (k < g.K) {
    const __amdgpu_buffer_rsrc_t mr = make_rsrc(Mbuf, g.m_bytes);
    const uint32_t row0 = ((uint32_t)k * g.Tp + tau0) * 4u;        // wave-uniform byte offset, position 0
    const uint32_t pstride = (uint32_t)g.K * (uint32_t)g.Tp * 4u;  // bytes between positions
    float z[t][t];
    uint32_t soff = row0;  // one scalar add per load
#pragma unroll
    for (int i = 0; i < t; ++i)
#pragma unroll
      for (int j = 0; j < t; ++j) {
        z[i][j] = buffer_load_f32(mr, lane * 4u, soff);
        soff += pstride;
        asm volatile("" : "+s"(soff));
      }
    float y[M][M];
    output_transform<M, R>(z, y);
    const int y0 = (int16_t)(ti.yx0 & 0xffff), x0 = ti.yx0 >> 16;
    // rows / columns of the tile inside the output (<= 0 for a padding tile, whose y0 is -32768)
    const int rows = y0 == -32768 ? 0 : g.Ho - (y0 + g.pad), cols = g.Wo - (x0 + g.pad);
    float* px = my + ti.out_org;
#pragma unroll
    for (int a = 0; a < M; ++a)
#pragma unroll
      for (int b = 0; b < M; ++b)
        if (a < rows && b < cols) px[a * g.Wo + b] = y[a][b];
  }
  __syncthreads();
  if (k >= g.K) return;
  const BlockImage* bi = blocks + (size_t)blockIdx.x * g.slots;
  const size_t plane = (size_t)g.Ho * g.Wo;
  for (int sidx = 0; sidx < g.slots; ++sidx) {
    const BlockImage b = bi[sidx];
    if (b.n < 0) continue;
    const float* src = my + b.out_off;
    float* dst = out + (size_t)b.n * g.out_image_stride + k * plane + b.out_elem0;
    // stores past the part's end are dropped by the descriptor: no lane predicate
    const __amdgpu_buffer_rsrc_t orr = make_rsrc(dst, (uint32_t)b.out_span * 4u);
    if (b.whole) {
      for (int e0 = 0; e0 < b.out_span; e0 += 64)
        buffer_store_f32<SWCONV_AUX_OUT>(orr, lane * 4u, e0 * 4u, src[e0 + lane]);
    } else {
      const int row_first = b.out_elem0 / g.Wo;  // wave-uniform
      for (int e0 = 0; e0 < b.out_span; e0 += 64) {
        const int e = e0 + lane;
        const int ry = (int)__umulhi((uint32_t)e, g.wo_magic), x = e - ry * g.Wo;
        const int tl = ((row_first + ry) >> g.m_shift) * g.tw + (x >> g.m_shift);
        const bool mine = tl >= b.t_lo && tl <= b.t_hi;  // a pixel of a tile of this block
        buffer_store_f32<SWCONV_AUX_OUT>(orr, mine ? lane * 4u : 0xfffffff0u, e0 * 4u, src[e]);
      }
    }
  }
}

}  // namespace swconv
