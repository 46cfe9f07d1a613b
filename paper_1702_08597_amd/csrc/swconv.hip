// Host side of libswconv: plan, CSR validation and re-packing, work-list construction, launches.
// Implements the C ABI declared in include/swconv.h.
#include "../../include/swconv.h"

#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <atomic>
#include <mutex>
#include <numeric>
#include <thread>
#include <type_traits>
#include <vector>

#include "swconv_backward_kernels.hpp"
#include "swconv_dense_mfma.hpp"
#include "swconv_fused_kernels.hpp"
#include "swconv_kernels.hpp"
#include "swconv_prune_kernels.hpp"

using namespace swconv;

namespace {

constexpr int kMaxLdsBytes = 160 * 1024;
constexpr int kSpmmLdsExtra = 64;    // the sparse product's slice counter sits behind the panel, then the slice descriptors

int env_int(const char* name, int dflt) {
  const char* s = std::getenv(name);
  if (!s || !*s) return dflt;
  char* end = nullptr;
  long v = std::strtol(s, &end, 10);
  return (end && *end == 0) ? (int)v : dflt;
}

// Host threads for the re-packing of the weights (a plan's set_weights is a few milliseconds of
// host work on a pruned AlexNet layer; a training loop that prunes every step calls it every step).
int host_threads() {
  const int hw = (int)std::thread::hardware_concurrency();
  return std::max(1, std::min(16, env_int("SWCONV_HOST_THREADS", hw > 0 ? hw : 1)));
}

// f(i) for every i in [0, n), the indices handed out by a shared counter to up to host_threads()
// threads (the caller's included).  f must not throw.  Threads that cannot be started are done without.
template <typename F>
void parallel_for(int n, F&& f) {
  const int nt = std::min(n, host_threads());
  std::atomic<int> next{0};
  auto work = [&]() {
    for (int i = next.fetch_add(1, std::memory_order_relaxed); i < n; i = next.fetch_add(1, std::memory_order_relaxed)) f(i);
  };
  std::vector<std::thread> helpers;
  try {
    helpers.reserve((size_t)std::max(0, nt - 1));
    for (int t = 1; t < nt; ++t) helpers.emplace_back(work);
  } catch (...) {
  }
  work();
  for (std::thread& t : helpers) t.join();
}

#define HIP_TRY(expr)                         \
  do {                                        \
    hipError_t e_ = (expr);                   \
    if (e_ != hipSuccess) {                   \
      (void)hipGetLastError();                \
      return e_ == hipErrorOutOfMemory ? SWCONV_ENOMEM : SWCONV_EHIP; \
    }                                         \
  } while (0)

// Copy h to the device.  With `cap` (the bytes *dptr holds, kept by the caller) the allocation is kept
// while it is large enough: a weight update then costs copies only.  The caller makes sure no kernel
// still reads the old contents.
template <typename T>
int upload(T** dptr, const std::vector<T>& h, size_t* cap = nullptr) {
  const size_t bytes = std::max<size_t>(h.size(), 1) * sizeof(T);
  if (cap && *dptr && *cap >= bytes) {
    if (!h.empty()) HIP_TRY(hipMemcpy(*dptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return SWCONV_OK;
  }
  if (*dptr) {
    (void)hipFree(*dptr);
    *dptr = nullptr;
  }
  if (cap) *cap = 0;
  HIP_TRY(hipMalloc((void**)dptr, bytes));
  if (cap) *cap = bytes;
  if (!h.empty()) HIP_TRY(hipMemcpy(*dptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
  return SWCONV_OK;
}

}  // namespace

// One position-wise sparse operand of the sparse product kernel in its packed form: P matrices of
// `rows` x `cols`; the kernel stages panels of `cols` channels and produces `rows` output rows.
// The forward pass packs W_F (rows = K, cols = C); the backward pass also packs its transpose.
struct PackedMatrix {
  int rows = 0, cols = 0;
  int rows_padded = 0;                // rows rounded up to a multiple of the slice height
  int waves = 8;                      // waves per workgroup
  int item_cap = kMaxItemSlices;      // most slices a work item may have (their descriptors are staged in LDS)
  int n_wgs = 512;                    // persistent workgroups the device can hold at once
  int cus = 256;                      // compute units of the device
  int n_wgs_used = 0;                 // workgroups the current schedule uses
  bool packed = false, on_device = false;
  int64_t nnz = 0, padded_nnz = 0, max_item = 0;
  std::vector<uint32_t> stream;       // 512-byte batches of (row offset, weight) pairs
  std::vector<Slice> slices;          // P * rows_padded / kSliceRows
  std::vector<int32_t> sorted_rows;   // P * rows_padded: original row of each sorted row, -1 = padding
  std::vector<int32_t> sorted_len;    // P * rows_padded: stored entries of each sorted row
  std::vector<WorkItem> items;        // in range order
  std::vector<int32_t> wg_begin;      // n_wgs_used + 1 offsets into items, one range per workgroup
  std::vector<RangeHeader> ranges;    // the same, as the kernel reads it
  std::vector<int32_t> entry_index;   // per stream entry: its index in the caller's CSR arrays, -1 = padding
  uint32_t* d_stream = nullptr;
  Slice* d_slices = nullptr;
  WorkItem* d_items = nullptr;
  RangeHeader* d_ranges = nullptr;
  size_t cap_stream = 0, cap_slices = 0, cap_items = 0, cap_ranges = 0;  // bytes of the four allocations
};

// W_F packed for the fused product + output transform kernel (m = 2, few input channels): rows in
// their natural order, 64 per workgroup, one package of 16-step batches per position.
struct FusedProduct {
  int out_tile = 0;       // m of the kernel that would run: 2 (product_output_kernel) or 4 (product_output4_kernel)
  int mode = 1;           // SWCONV_FUSE_OUTPUT: 0 never, 1 where it pays (m = 2), 2 wherever a kernel can run
  bool wanted = true;     // m = 2: always; m = 4: only when asked for through SWCONV_FUSE_OUTPUT=2
  bool eligible = false;  // the layer shape allows the kernel
  bool ready = false;     // the current weights fit its format and are on the device
  int KC = 0;             // row chunks of kFusedRows
  int B = 0;              // batches per slice and position (the longest row decides)
  std::vector<uint32_t> wpk;
  std::vector<int32_t> value_index;  // per pair of wpk: index into the caller's value array, -1 = padding
  std::vector<uint8_t> lens;
  std::vector<OutTile> otiles;
  uint32_t* d_wpk = nullptr;
  uint8_t* d_lens = nullptr;
  OutTile* d_otiles = nullptr;
  int32_t* d_value_index = nullptr;
  size_t cap_wpk = 0, cap_lens = 0, cap_value_index = 0;
};

struct swconv_plan {
  Geometry g{};
  int m = 0, r = 0, t = 0, P = 0;
  int Kq = 0;    // K rounded up to the dense GEMM's row tile
  int n_tau_blocks = 0;

  PackedMatrix fw;  // W_F: K rows, panels of C channels (forward)
  PackedMatrix bt;  // W_F^T: C rows, panels of K channels (backward, Eq. 6 first line); packed on first use
  FusedProduct fz;  // W_F again, for the kernel that runs steps 2 and 3 together
  bool m_current = false;  // the M workspace holds the products of the last forward pass
  bool bt_supported = false, bt_current = false;

  // host-built index tables of the transform kernels
  std::vector<TileInfo> tiles;        // Tp
  std::vector<BlockImage> blocks;     // Tp/64 * slots
  TileInfo* d_tiles = nullptr;
  BlockImage* d_blocks = nullptr;

  // device
  bool on_device = false, dense_on_device = false, ran_forward = false;
  float *dV = nullptr, *dM = nullptr;
  float* dD = nullptr;        // backward pass: dL/dI_F, [P][C][Tp]
  // Eq. 6's last two lines as one kernel when G whole image planes per wave fit LDS
  int grad_images_per_group = 0;  // 0: the patch + gather kernels run instead
  std::vector<GradTile> gtiles;   // Tp
  GradTile* d_gtiles = nullptr;
  float* d_partial = nullptr; // backward pass: [tile blocks][stream entries of W_F] partial dot products
  size_t partial_floats = 0;
  int32_t* d_entry_index = nullptr;
  size_t cap_entry_index = 0;
  bool index_current = false;
  // swconv_update_values: the device streams hold newer values than the host copies
  bool host_values_stale = false;
  std::vector<int32_t> bt_value_index;  // per pair of the packed W_F^T: index into the caller's value array
  int32_t* d_bt_value_index = nullptr;
  size_t cap_bt_value_index = 0;
  bool ran_backward = false;
  float* d_wdense = nullptr;  // [P][C][Kq]
};

// Scratch of swconv_forward_noalloc: the V and M workspaces of one forward pass, for callers that
// cannot allocate.  One copy per GPU the library runs on, held until the process ends.  In host code
// the array's name only stands for the symbol: the memory is reached through the per-device address
// that static_scratch() asks the runtime for, never through the name.
constexpr size_t kStaticScratchBytes = SWCONV_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_of_device[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up once per device).
int static_scratch(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return SWCONV_EUNSUPPORTED;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_of_device[dev]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return SWCONV_EHIP;
    scratch_of_device[dev] = ptr;
  }
  *out = scratch_of_device[dev];
  return SWCONV_OK;
}

// The two intermediates of a forward pass: the plan's own buffers, or parts of the static scratch.
struct Workspace {
  float* V;
  float* M;
};

int ensure_workspace(swconv_plan* pl) {
  if (pl->on_device) return SWCONV_OK;
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (ndev < 1) return SWCONV_EHIP;
  const size_t vbytes = (size_t)pl->P * pl->g.C * pl->g.Tp * sizeof(float);
  const size_t mbytes = (size_t)pl->P * pl->g.K * pl->g.Tp * sizeof(float);
  // a call that failed half way left its buffers in the plan: take them up again
  if (!pl->dV) HIP_TRY(hipMalloc((void**)&pl->dV, vbytes));
  if (!pl->dM) HIP_TRY(hipMalloc((void**)&pl->dM, mbytes));
  HIP_TRY(hipMemset(pl->dV, 0, vbytes));
  HIP_TRY(hipMemset(pl->dM, 0, mbytes));
  int rc;
  if ((rc = upload(&pl->d_tiles, pl->tiles))) return rc;
  if ((rc = upload(&pl->d_blocks, pl->blocks))) return rc;
  // set-up time: look up this device's static scratch now, so that swconv_forward_noalloc finds it known
  void* unused = nullptr;
  (void)static_scratch(&unused);
  pl->on_device = true;
  return SWCONV_OK;
}

// Where a kernel goes: the stream and, for swconv_profile_forward, a pair of events that take the
// kernel's own start and end time stamps (no extra packets on the stream).
struct LaunchTarget {
  hipStream_t stream;
  hipEvent_t start, stop;
};

template <typename... Params, typename... Args>
int launch_kernel(void (*kern)(Params...), dim3 grid, dim3 block, size_t lds, const LaunchTarget& to, Args... args) {
  if (to.start || to.stop)
    hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)lds, to.stream, to.start, to.stop, 0u, Params(args)...);
  else
    hipLaunchKernelGGL(kern, grid, block, lds, to.stream, Params(args)...);
  HIP_TRY(hipGetLastError());
  return SWCONV_OK;
}

// Calls f(integral_constant<M>, integral_constant<R>) for the plan's F(m x m, r x r).
template <typename F>
int dispatch_mr(const swconv_plan* pl, F&& f) {
  using std::integral_constant;
  if (pl->r == 5)
    return pl->m == 2 ? f(integral_constant<int, 2>{}, integral_constant<int, 5>{})
                      : f(integral_constant<int, 4>{}, integral_constant<int, 5>{});
  return pl->m == 2 ? f(integral_constant<int, 2>{}, integral_constant<int, 3>{})
                    : f(integral_constant<int, 4>{}, integral_constant<int, 3>{});
}

template <int M, int R>
int launch_input_transform(const swconv_plan* pl, const LaunchTarget& to, const float* in, float* V) {
  dim3 grid(pl->g.Tp / 64, (pl->g.C + 3) / 4);
  const size_t lds = (size_t)4 * pl->g.in_area * sizeof(float);
  auto kern = input_transform_kernel<M, R>;
  static bool attr_set = false;
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
    attr_set = true;
  }
  return launch_kernel(kern, grid, dim3(256), lds, to, in, V, pl->d_tiles, pl->d_blocks, pl->g);
}

template <int M, int R>
int launch_output_transform(const swconv_plan* pl, const LaunchTarget& to, const float* Mbuf, float* out) {
  dim3 grid(pl->g.Tp / 64, (pl->g.K + 3) / 4);
  const size_t lds = (size_t)4 * pl->g.out_area * sizeof(float);
  auto kern = output_transform_kernel<M, R>;
  static bool attr_set = false;
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
    attr_set = true;
  }
  return launch_kernel(kern, grid, dim3(256), lds, to, Mbuf, out, pl->d_tiles, pl->d_blocks, pl->g);
}

// Y[p] = A[p] * X[p] for the packed operand `pm`: X has pm.cols rows of Tp tiles per position and
// x_bytes in all, Y gets pm.rows rows per position.  With `partial` set (sampled mode): Y is read
// and partial[tile block][stream entry] receives the entry's dot product over the block.
template <int NW, bool SAMPLED>
int launch_spmm_t(const swconv_plan* pl, const PackedMatrix& pm, const LaunchTarget& to, const float* X,
                  uint32_t x_bytes, float* Y, uint32_t y_bytes, float* partial) {
  if (pm.n_wgs_used == 0) return SWCONV_OK;
  const size_t lds = (size_t)pm.cols * kTileBlock * sizeof(float) + kSpmmLdsExtra + (size_t)pm.item_cap * sizeof(Slice);
  auto kern = spmm_kernel<NW, SAMPLED>;
  static bool attr_set = false;
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
    attr_set = true;
  }
  return launch_kernel(kern, dim3(pm.n_wgs_used), dim3(NW * 64), lds, to, X, Y, pm.d_stream,
                       (uint32_t)(pm.stream.size() * sizeof(uint32_t)), pm.d_slices, (int)pm.slices.size(),
                       pm.d_items, pm.d_ranges, pm.n_wgs_used, pm.cols, pm.rows, pl->g.Tp, y_bytes, x_bytes, partial,
                       (uint32_t)(pm.stream.size() / 2));
}

template <bool SAMPLED>
int launch_spmm_mode(const swconv_plan* pl, const PackedMatrix& pm, const LaunchTarget& to, const float* X,
                     uint32_t x_bytes, float* Y, uint32_t y_bytes, float* partial) {
  if (pm.waves == 12) return launch_spmm_t<12, SAMPLED>(pl, pm, to, X, x_bytes, Y, y_bytes, partial);
  return pm.waves == 16 ? launch_spmm_t<16, SAMPLED>(pl, pm, to, X, x_bytes, Y, y_bytes, partial)
                        : launch_spmm_t<8, SAMPLED>(pl, pm, to, X, x_bytes, Y, y_bytes, partial);
}

int launch_spmm(const swconv_plan* pl, const PackedMatrix& pm, const LaunchTarget& to, const float* X,
                uint32_t x_bytes, float* Y, uint32_t y_bytes) {
  return launch_spmm_mode<false>(pl, pm, to, X, x_bytes, Y, y_bytes, nullptr);
}

template <int R, int PP>
int launch_product_output_t(const swconv_plan* pl, const LaunchTarget& to, const float* V, float* out) {
  const FusedProduct& fz = pl->fz;
  const Geometry& g = pl->g;
  const size_t lds = (size_t)2 * ((size_t)g.C * kTileBlock * sizeof(float) + (size_t)kFusedWaves * fz.B * 512) + 1024;
  auto kern = product_output_kernel<R, PP>;
  static bool attr_set = false;
  if (!attr_set) {
    HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
    attr_set = true;
  }
  const int n_wgs = pl->n_tau_blocks * fz.KC;
  return launch_kernel(kern, dim3(n_wgs), dim3(kFusedWaves * 64), lds, to, V, out,
                       (const uint32_t*)fz.d_wpk, (uint32_t)(fz.wpk.size() * sizeof(uint32_t)),
                       (const uint8_t*)fz.d_lens, (const OutTile*)fz.d_otiles, g.C, g.K, g.Tp, fz.KC, fz.B, n_wgs,
                       g.v_bytes, (uint32_t)(g.Ho * g.Wo), g.Wo, (uint32_t)g.out_image_stride,
                       (uint32_t)((int64_t)g.N * g.out_image_stride * (int64_t)sizeof(float)));
}

int launch_product_output(const swconv_plan* pl, const LaunchTarget& to, const float* V, float* out) {
  const bool one_piece = pl->g.C * (kTileBlock / 4) <= kFusedWaves * 64;
  if (pl->r == 3)
    return one_piece ? launch_product_output_t<3, 1>(pl, to, V, out) : launch_product_output_t<3, 2>(pl, to, V, out);
  return one_piece ? launch_product_output_t<5, 1>(pl, to, V, out) : launch_product_output_t<5, 2>(pl, to, V, out);
}

template <int G>
int launch_product_output4_t(const swconv_plan* pl, const LaunchTarget& to, const float* V, float* out) {
  const FusedProduct& fz = pl->fz;
  const int n_wgs = pl->n_tau_blocks * fz.KC;
  return launch_kernel(product_output4_kernel<3, G>, dim3(n_wgs), dim3(kFusedWaves * 64), 0, to, V, out,
                       (const uint32_t*)fz.d_wpk, (uint32_t)(fz.wpk.size() * sizeof(uint32_t)),
                       (const uint8_t*)fz.d_lens, (const TileInfo*)pl->d_tiles, (const BlockImage*)pl->d_blocks, fz.KC,
                       fz.B, n_wgs, pl->g);
}

int launch_product_output4(const swconv_plan* pl, const LaunchTarget& to, const float* V, float* out) {
  switch ((pl->g.C + 63) / 64) {  // direct loads per wave and panel
    case 1: return launch_product_output4_t<1>(pl, to, V, out);
    case 2: return launch_product_output4_t<2>(pl, to, V, out);
    case 3: return launch_product_output4_t<3>(pl, to, V, out);
    default: return launch_product_output4_t<4>(pl, to, V, out);
  }
}

// The forward pass is three kernels, or two where steps 2 and 3 run fused.
bool fused_runs(const swconv_plan* pl) {
  // its output stores use 32-bit byte offsets from the output pointer
  return pl->fz.ready && pl->fz.wanted &&
         (int64_t)pl->g.N * pl->g.out_image_stride * (int64_t)sizeof(float) < ((int64_t)1 << 32) - 256;
}
bool forward_stage_runs(const swconv_plan* pl, int stage) { return stage < 2 || !fused_runs(pl); }

int launch_stage(const swconv_plan* pl, const LaunchTarget& to, int stage, const float* in, float* out,
                 const Workspace& ws) {
  if (stage == 1 && fused_runs(pl))
    return pl->fz.out_tile == 4 ? launch_product_output4(pl, to, ws.V, out) : launch_product_output(pl, to, ws.V, out);
  switch (stage) {
    case 0:
      return dispatch_mr(pl, [&](auto M, auto R) { return launch_input_transform<M(), R()>(pl, to, in, ws.V); });
    case 1: return launch_spmm(pl, pl->fw, to, ws.V, pl->g.v_bytes, ws.M, pl->g.m_bytes);
    default:
      return dispatch_mr(pl, [&](auto M, auto R) { return launch_output_transform<M(), R()>(pl, to, ws.M, out); });
  }
}
int launch_stage(const swconv_plan* pl, const LaunchTarget& to, int stage, const float* in, float* out) {
  return launch_stage(pl, to, stage, in, out, Workspace{pl->dV, pl->dM});
}

// Index tables of the two transform kernels: where each tile and each (tile block, image) part
// sits in the image and in a wave's LDS staging area.
void build_transform_tables(swconv_plan* pl) {
  Geometry& g = pl->g;
  g.in_area = g.out_area = 64;
  const int m = pl->m, t = pl->t, nblk = g.Tp / 64;
  TileInfo pad_tile;
  pad_tile.in_org = 0;
  pad_tile.yx0 = (int32_t)0x80008000u;  // y0 = x0 = -32768: nothing is inside the image
  pad_tile.ylim = 0;
  pad_tile.out_org = 0;
  pl->tiles.assign((size_t)g.Tp, pad_tile);
  BlockImage unused{};
  unused.n = -1;
  pl->blocks.assign((size_t)nblk * g.slots, unused);
  for (int b = 0; b < nblk; ++b) {
    const int tau0 = b * 64;
    if (tau0 >= g.T) continue;
    const int last = std::min(tau0 + 63, g.T - 1);
    const int n_first = tau0 / g.tpi, n_last = last / g.tpi;
    int in_off = 0, out_off = 0;
    for (int n = n_first; n <= n_last; ++n) {
      const int slot = n - n_first, base = n * g.tpi;
      const int t_lo = std::max(tau0, base) - base, t_hi = std::min(last, base + g.tpi - 1) - base;
      const int ty_lo = t_lo / g.tw, ty_hi = t_hi / g.tw;
      const int y_lo = std::max(0, ty_lo * m - g.pad), y_hi = std::min(g.H, ty_hi * m - g.pad + t);
      const int oy_lo = ty_lo * m, oy_hi = std::min(g.Ho, (ty_hi + 1) * m);
      BlockImage& bi = pl->blocks[(size_t)b * g.slots + slot];
      bi.n = n;
      bi.in_elem0 = y_lo * g.W;
      bi.in_span = (y_hi - y_lo) * g.W;
      bi.out_elem0 = oy_lo * g.Wo;
      bi.out_span = (oy_hi - oy_lo) * g.Wo;
      bi.t_lo = t_lo;
      bi.t_hi = t_hi;
      bi.whole = (t_lo % g.tw == 0) && ((t_hi + 1) % g.tw == 0);
      bi.in_off = in_off;
      bi.out_off = out_off;
      in_off += (bi.in_span + 63) / 64 * 64;
      out_off += (bi.out_span + 63) / 64 * 64;
      g.in_area = std::max(g.in_area, in_off);
      g.out_area = std::max(g.out_area, out_off);
      for (int tl = t_lo; tl <= t_hi; ++tl) {
        const int ty = tl / g.tw, tx = tl % g.tw;
        const int y0 = ty * m - g.pad, x0 = tx * m - g.pad;
        TileInfo& ti = pl->tiles[(size_t)base + tl];
        ti.in_org = bi.in_off - y_lo * g.W;
        ti.yx0 = (int32_t)(((uint32_t)y0 & 0xffffu) | ((uint32_t)x0 << 16));
        ti.ylim = (int32_t)((uint32_t)y_lo | ((uint32_t)(y_hi - 1) << 16));
        ti.out_org = bi.out_off + (ty * m - oy_lo) * g.Wo + tx * m;
        if (!pl->fz.otiles.empty()) {
          OutTile& ot = pl->fz.otiles[(size_t)base + tl];
          ot.n = (uint32_t)n;
          ot.pix = (uint32_t)(ty * m * g.Wo + tx * m);
          ot.valid = (uint32_t)std::min(m, g.Ho - ty * m) | ((uint32_t)std::min(m, g.Wo - tx * m) << 16);
        }
      }
    }
  }
}

// Packs W_F for the fused kernel: rows in natural order; slice s of position p = rows 4s .. 4s+3,
// workgroup chunk kc = slices 16 kc .. 16 kc + 15.  Not ready (and the three-kernel path runs) when
// a row is longer than the kernel's batches hold.
void pack_fused(swconv_plan* pl, const int32_t* rowptr, const int32_t* colidx, const float* vals) {
  FusedProduct& fz = pl->fz;
  fz.ready = false;
  if (!fz.eligible) return;
  const int P = pl->P, K = pl->g.K;
  const bool units = fz.out_tile == 4;  // F(4x4,3x3): whole units of two batches
  int32_t longest = 0;
  for (int64_t i = 0; i < (int64_t)P * K; ++i) longest = std::max(longest, rowptr[i + 1] - rowptr[i]);
  fz.KC = (K + kFusedRows - 1) / kFusedRows;
  fz.B = std::max(1, (longest + kBatchSteps - 1) / kBatchSteps);
  if (units) fz.B = (fz.B + 1) / 2 * 2;
  if (fz.B > (units ? kFused4MaxBatches : kFusedMaxBatches)) return;
  const int spp = fz.KC * kFusedWaves;
  const size_t dwords = (size_t)P * fz.KC * fz.B * kFusedWaves * 128;
  if (dwords * 4 >= ((size_t)1 << 32) - 4096) return;
  fz.wpk.assign(dwords, 0u);
  fz.value_index.assign(dwords / 2, -1);
  fz.lens.assign((size_t)P * spp, 0);
  const uint32_t row_bytes = (uint32_t)kTileBlock * sizeof(float);
  // steps of every slice: its longest row, rounded up to whole groups of steps
  for (int p = 0; p < P; ++p)
    for (int k = 0; k < K; ++k) {
      const int32_t len = rowptr[(int64_t)p * K + k + 1] - rowptr[(int64_t)p * K + k];
      uint8_t& steps = fz.lens[(size_t)p * spp + k / kSliceRows];
      steps = std::max<uint8_t>(steps, (uint8_t)((len + kStepGroup - 1) / kStepGroup * kStepGroup));
    }
  for (int p = 0; p < P; ++p)
    for (int k = 0; k < K; ++k) {
      const int sl = k / kSliceRows, q = k % kSliceRows, kc = sl / kFusedWaves, w = sl % kFusedWaves;
      const int32_t q0 = rowptr[(int64_t)p * K + k], len = rowptr[(int64_t)p * K + k + 1] - q0;
      for (int32_t e = 0; e < len; ++e) {
        const size_t batch = (((size_t)p * fz.KC + kc) * fz.B + e / kBatchSteps) * kFusedWaves + w;
        uint32_t* entry = &fz.wpk[batch * 128 + ((size_t)q * kBatchSteps + e % kBatchSteps) * 2];
        entry[0] = (uint32_t)colidx[q0 + e] * row_bytes;
        std::memcpy(&entry[1], &vals[q0 + e], sizeof(float));
        fz.value_index[(size_t)(entry - fz.wpk.data()) / 2] = q0 + e;
      }
    }
  fz.ready = true;
}

int upload_fused(swconv_plan* pl) {
  FusedProduct& fz = pl->fz;
  if (!fz.ready) return SWCONV_OK;
  fz.ready = false;
  int rc;
  if ((rc = upload(&fz.d_wpk, fz.wpk, &fz.cap_wpk))) return rc;
  if ((rc = upload(&fz.d_lens, fz.lens, &fz.cap_lens))) return rc;
  if ((rc = upload(&fz.d_value_index, fz.value_index, &fz.cap_value_index))) return rc;
  if (!fz.d_otiles && !fz.otiles.empty() && (rc = upload(&fz.d_otiles, fz.otiles))) return rc;
  HIP_TRY(hipDeviceSynchronize());
  fz.ready = true;
  return SWCONV_OK;
}

// Validate the caller's CSR; returns SWCONV_OK or SWCONV_EINVAL.
int validate_csr(const swconv_plan* pl, const int32_t* rowptr, const int32_t* colidx, const float* vals) {
  const int64_t rows = (int64_t)pl->P * pl->g.K;
  if (!rowptr || rowptr[0] != 0) return SWCONV_EINVAL;
  for (int64_t i = 0; i < rows; ++i)
    if (rowptr[i + 1] < rowptr[i]) return SWCONV_EINVAL;
  const int64_t nnz = rowptr[rows];
  if (nnz > 0 && (!colidx || !vals)) return SWCONV_EINVAL;
  const int C = pl->g.C;
  constexpr int64_t kChunk = 1024;  // rows per unit of work
  std::atomic<bool> bad{false};
  parallel_for((int)((rows + kChunk - 1) / kChunk), [&](int chunk) {
    const int64_t end = std::min(rows, (int64_t)(chunk + 1) * kChunk);
    for (int64_t i = (int64_t)chunk * kChunk; i < end; ++i) {
      if (rowptr[i + 1] - rowptr[i] > C) bad.store(true, std::memory_order_relaxed);
      int32_t prev = -1;
      for (int32_t q = rowptr[i]; q < rowptr[i + 1]; ++q) {
        const int32_t c = colidx[q];
        if (c <= prev || c >= C) bad.store(true, std::memory_order_relaxed);
        prev = c;
      }
    }
  });
  return bad.load() ? SWCONV_EINVAL : SWCONV_OK;
}

// Static schedule of the sparse product.  The units (position, tile block, slice), in that order,
// form one sequence; it is cut into one contiguous range per persistent workgroup such that every
// range costs about the same: a slice costs its stream length plus a fixed overhead, and entering
// a new panel costs one panel load.  The smallest feasible cost per
// range is found by bisection.  A range touches at most a few panels, consecutive ranges share
// panels and weights (and, through xcd_contiguous_id, an XCD's L2), and the split adapts by
// itself to positions of very different density.
void build_schedule(PackedMatrix* pm, int P, int ntb) {
  const int spp = pm->rows_padded / kSliceRows;
  // Costs in units of the time a workgroup spends on one step of a slice (four 16-byte LDS reads
  // per wave quarter-row, 16 FMAs per lane).  Fitted on MI355X over uniform and skewed patterns: a
  // slice costs about 32 steps on top of its own (draw, descriptor, first batches, row store),
  // staging a panel about 20 steps per KiB.
  const int64_t slice_ovh = env_int("SWCONV_SPMM_SLICE_COST", 32);
  const int64_t panel_kib = ((int64_t)pm->cols * kTileBlock * (int64_t)sizeof(float) + 1023) / 1024;
  const int64_t panel_cost = (int64_t)env_int("SWCONV_SPMM_PANEL_COST_PER_KIB", 20) * panel_kib;
  const int wgs_max = std::max(1, pm->n_wgs);

  // Workgroups are dispatched in id order, one per CU first: where a CU holds two, the one that
  // arrived second gets the issue slots the first one leaves (the oldest wave wins) and then runs on
  // alone with half the waves.  It therefore gets a smaller range: `second_share` percent of the
  // first one's budget.  A range's workgroup follows from xcd_contiguous_id for `n_launch` workgroups.
  const int64_t second_share = std::min(100, std::max(10, env_int("SWCONV_SPMM_SECOND_SHARE", 70)));
  const int64_t floor_budget = panel_cost + [&] {
    int64_t b = 0;
    for (const Slice& sl : pm->slices) b = std::max<int64_t>(b, sl.len + slice_ovh);
    return b;
  }();
  int n_launch = wgs_max;
  auto range_budget = [&](int64_t budget, int r) -> int64_t {
    if (second_share == 100) return budget;
    const int per = n_launch / kXcds, rem = n_launch % kXcds;
    // ranges of XCD x start at x * per + min(x, rem)
    int xcd = per > 0 ? std::min(kXcds - 1, r / std::max(1, per)) : 0;
    while (xcd > 0 && r < xcd * per + std::min(xcd, rem)) --xcd;
    const int local = r - (xcd * per + std::min(xcd, rem));
    const bool second = local * kXcds + xcd >= pm->cus;
    return second ? std::max(floor_budget, budget * second_share / 100) : budget;
  };

  std::vector<int64_t> cost_before(pm->slices.size() + 1, 0);
  for (size_t i = 0; i < pm->slices.size(); ++i) cost_before[i + 1] = cost_before[i] + pm->slices[i].len + slice_ovh;

  auto cut = [&](int64_t base_budget, std::vector<WorkItem>* items, std::vector<int32_t>* begin) -> int {
    int wgs = 0;
    int64_t acc = 0;
    int64_t budget = range_budget(base_budget, 0);
    bool open_wg = false;
    if (items) { items->clear(); begin->assign(1, 0); }
    auto close_wg = [&]() {
      if (!open_wg) return;
      ++wgs;
      if (begin) begin->push_back((int32_t)items->size());
      open_wg = false;
      acc = 0;
      budget = range_budget(base_budget, wgs);
    };
    for (int p = 0; p < P; ++p)
      for (int tb = 0; tb < ntb; ++tb) {
        int s = p * spp;
        const int s_end = s + spp;
        while (s < s_end) {
          // a new item in the current workgroup: pay the panel, then take slices while they fit
          if (open_wg && acc + panel_cost + pm->slices[s].len + slice_ovh > budget) close_wg();
          open_wg = true;
          acc += panel_cost;
          const int s0 = s;
          // the first slice in any case, then as many as the budget holds (prefix sums of the slice
          // costs: `cost_before[i]` = cost of all slices before slice i), at most item_cap and the position's
          const int limit = std::min(s_end, s0 + pm->item_cap);
          const int64_t room = cost_before[s0] + (budget - acc);
          s = (int)(std::upper_bound(cost_before.begin() + s0 + 1, cost_before.begin() + limit + 1, room) -
                    cost_before.begin()) - 1;
          s = std::max(s, s0 + 1);
          acc += cost_before[s] - cost_before[s0];
          if (items) items->push_back(WorkItem{p, tb, s0, s});
          if (s < s_end && s - s0 < pm->item_cap) close_wg();  // the budget, not the item cap, ended the item
        }
      }
    close_wg();
    return wgs;
  };

  int64_t total = 0, biggest = 0;
  for (const Slice& sl : pm->slices) {
    total += sl.len + slice_ovh;
    biggest = std::max<int64_t>(biggest, sl.len + slice_ovh);
  }
  total *= ntb;
  int64_t lo = panel_cost + biggest, hi = std::max(lo, total + (int64_t)P * ntb * panel_cost);
  for (int round = 0; round < 4; ++round) {
    int64_t l = lo, h = hi;
    while (l < h) {  // smallest budget that needs no more than wgs_max workgroups
      const int64_t mid = l + (h - l) / 2;
      if (cut(mid, nullptr, nullptr) <= wgs_max) h = mid; else l = mid + 1;
    }
    pm->n_wgs_used = cut(l, &pm->items, &pm->wg_begin);
    if (second_share == 100 || pm->n_wgs_used == n_launch) break;
    n_launch = pm->n_wgs_used;  // the id -> range map depends on the number launched: once more with that
  }
  pm->ranges.assign((size_t)pm->n_wgs_used, RangeHeader{});
  for (int b = 0; b < pm->n_wgs_used; ++b) {
    RangeHeader& h = pm->ranges[b];
    h.item_begin = pm->wg_begin[b];
    h.item_end = pm->wg_begin[b + 1];
    h.first = pm->items[h.item_begin];
  }
  pm->max_item = 0;
  for (int b = 0; b < pm->n_wgs_used; ++b) {
    int64_t steps = 0;
    for (int i = pm->wg_begin[b]; i < pm->wg_begin[b + 1]; ++i)
      for (int sidx = pm->items[i].slice_begin; sidx < pm->items[i].slice_end; ++sidx) steps += pm->slices[sidx].len;
    pm->max_item = std::max(pm->max_item, steps * kSliceRows);
  }
}

// Dword index of the (offset, weight) pair of row q, step e of a slice whose first 512-byte batch
// is `batch0`: lane (q, e % 16) of batch e / 16.
inline size_t stream_entry(uint32_t batch0, int q, int32_t e) {
  return ((size_t)batch0 + (size_t)(e / kBatchSteps)) * 128 + ((size_t)q * kBatchSteps + (size_t)(e % kBatchSteps)) * 2;
}

// Shape-dependent launch parameters of a packed operand with `rows` x `cols` matrices; false when
// the panel of `cols` channels (256 bytes each), the slice counter and the descriptors of at least
// kMinItemSlices slices do not fit LDS.
bool configure_packed(PackedMatrix* pm, int rows, int cols) {
  pm->rows = rows;
  pm->cols = cols;
  pm->rows_padded = (rows + kSliceRows - 1) / kSliceRows * kSliceRows;
  const int64_t panel_bytes = (int64_t)cols * kTileBlock * (int64_t)sizeof(float);
  const int64_t desc_room = (kMaxLdsBytes - kSpmmLdsExtra - panel_bytes) / (int64_t)sizeof(Slice);
  if (desc_room < kMinItemSlices) return false;
  pm->item_cap = (int)std::min<int64_t>(std::min<int64_t>(kMaxItemSlices, desc_room), pm->rows_padded / kSliceRows);
  // two workgroups of 12 waves per CU while two panels fit LDS (six waves per SIMD hide the LDS and
  // draw latencies better than four), else one of 16
  const int64_t wg_lds = panel_bytes + kSpmmLdsExtra + (int64_t)pm->item_cap * (int64_t)sizeof(Slice);
  const int dflt_waves = wg_lds * 2 > kMaxLdsBytes ? 16 : 12;
  pm->waves = env_int("SWCONV_SPMM_WAVES", dflt_waves);
  if (pm->waves != 8 && pm->waves != 12 && pm->waves != 16) pm->waves = dflt_waves;
  // a thread stages at most kPanelPieces 16-byte pieces of a panel
  if (panel_bytes > (int64_t)kPanelPieces * pm->waves * 64 * 16) pm->waves = 16;
  return true;
}

// Persistent workgroups the device holds at once: as many per CU as the operand's LDS allows - but
// one per CU when that would leave a workgroup fewer than 16 of the `units` (position, tile block,
// slice) on average: every workgroup stages a whole panel for its share, and on the single-image
// layer 256 workgroups measured 5.4 us against 6.4 us for 512.
void size_grid(PackedMatrix* pm, int64_t units) {
  int cus = 256, ndev = 0, dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0 && hipGetDevice(&dev) == hipSuccess &&
      hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
    cus = prop.multiProcessorCount;
  else
    (void)hipGetLastError();
  const size_t wg_lds = (size_t)pm->cols * kTileBlock * sizeof(float) + kSpmmLdsExtra + (size_t)pm->item_cap * sizeof(Slice);
  int per_cu = std::max<int>(1, std::min<int>(32 / pm->waves, (int)(kMaxLdsBytes / wg_lds)));
  if (units < (int64_t)16 * cus * per_cu) per_cu = 1;
  pm->cus = cus;
  pm->n_wgs = std::max(1, env_int("SWCONV_SPMM_WGS", cus * per_cu));
}

// Re-pack P row-major CSR matrices (rows (p, row) -> p * rows + row, global offsets) into the sliced
// layout and build the schedule.
void pack_matrix(PackedMatrix* pm, int P, int ntb, const int32_t* rowptr, const int32_t* colidx, const float* vals) {
  const int R = pm->rows, Rp = pm->rows_padded;
  const int slices_per_pos = Rp / kSliceRows;
  pm->nnz = rowptr[(int64_t)P * R];
  pm->sorted_rows.assign((size_t)P * Rp, -1);
  pm->sorted_len.assign((size_t)P * Rp, 0);
  pm->slices.assign((size_t)P * slices_per_pos, Slice{});

  // per position (in parallel): rows sorted by length, four to a slice
  std::vector<int32_t> order_all((size_t)P * R);
  parallel_for(P, [&](int p) {
    const int32_t* rp = rowptr + (int64_t)p * R;
    int32_t* order = order_all.data() + (size_t)p * R;
    std::iota(order, order + R, 0);
    std::stable_sort(order, order + R, [&](int32_t a, int32_t b) { return rp[a + 1] - rp[a] > rp[b + 1] - rp[b]; });
    for (int i = 0; i < R; ++i) {
      pm->sorted_rows[(size_t)p * Rp + i] = order[i];
      pm->sorted_len[(size_t)p * Rp + i] = rp[order[i] + 1] - rp[order[i]];
    }
    for (int s = 0; s < slices_per_pos; ++s) {
      Slice& sl = pm->slices[(size_t)p * slices_per_pos + s];
      sl.p = p;
      sl.row0 = p * Rp + s * kSliceRows;
      for (int r = 0; r < kSliceRows; ++r) sl.k[r] = pm->sorted_rows[sl.row0 + r];
      // rows are sorted: the first is the longest; whole groups of steps
      sl.len = (pm->sorted_len[sl.row0] + kStepGroup - 1) / kStepGroup * kStepGroup;
    }
  });
  // where each slice's batches start in the stream
  uint64_t cursor = 0;  // 512-byte batches
  pm->padded_nnz = 0;
  for (Slice& sl : pm->slices) {
    sl.batch0 = (uint32_t)cursor;
    cursor += (sl.len + kBatchSteps - 1) / kBatchSteps;
    pm->padded_nnz += (int64_t)sl.len * kSliceRows;
  }
  // an entry is (byte offset of the panel row of its column, weight); padding = row 0, weight +0.0f.
  // The kernel addresses the stream with 32-bit byte offsets and fetches up to two batches past a
  // slice's end: two spare batches keep even those inside the allocation.
  const uint64_t spare0 = cursor;
  cursor += 2;
  if (cursor * 512 >= ((uint64_t)1 << 32) - 4096) throw std::bad_alloc();
  const uint32_t row_bytes = (uint32_t)kTileBlock * sizeof(float);
  pm->stream.resize((size_t)cursor * 128);
  pm->entry_index.resize((size_t)cursor * 64);
  std::fill(pm->stream.begin() + (size_t)spare0 * 128, pm->stream.end(), 0u);
  std::fill(pm->entry_index.begin() + (size_t)spare0 * 64, pm->entry_index.end(), -1);
  // per position (in parallel): every pair of every batch of its slices is written once, entry or padding
  parallel_for(P, [&](int p) {
    const int32_t* rp = rowptr + (int64_t)p * R;
    for (int s = 0; s < slices_per_pos; ++s) {
      const Slice& sl = pm->slices[(size_t)p * slices_per_pos + s];
      const int batches = (sl.len + kBatchSteps - 1) / kBatchSteps;
      for (int r = 0; r < kSliceRows; ++r) {
        const int row = pm->sorted_rows[sl.row0 + r];
        const int32_t q0 = row < 0 ? 0 : rp[row], len = row < 0 ? 0 : rp[row + 1] - rp[row];
        for (int b = 0; b < batches; ++b) {
          const size_t first = stream_entry(sl.batch0, r, b * kBatchSteps);  // the row's 16 pairs of a batch are contiguous
          uint32_t* entry = &pm->stream[first];
          int32_t* index = &pm->entry_index[first / 2];
          for (int i = 0; i < kBatchSteps; ++i) {
            const int32_t e = b * kBatchSteps + i;
            if (e < len) {
              entry[2 * i] = (uint32_t)colidx[q0 + e] * row_bytes;
              std::memcpy(&entry[2 * i + 1], &vals[q0 + e], sizeof(float));
              index[i] = q0 + e;
            } else {
              entry[2 * i] = 0u;
              entry[2 * i + 1] = 0u;
              index[i] = -1;
            }
          }
        }
      }
    }
  });
  build_schedule(pm, P, ntb);
  pm->packed = true;
}

// The inverse of pack_matrix: back to CSR, padding dropped, rows in their original order.
void unpack_matrix(const PackedMatrix& pm, int P, int32_t* rowptr, int32_t* colidx, float* vals) {
  const int R = pm.rows, Rp = pm.rows_padded;
  rowptr[0] = 0;
  std::vector<int32_t> len((size_t)P * R, 0);
  for (int p = 0; p < P; ++p)
    for (int i = 0; i < Rp; ++i) {
      const int row = pm.sorted_rows[(size_t)p * Rp + i];
      if (row >= 0) len[(size_t)p * R + row] = pm.sorted_len[(size_t)p * Rp + i];
    }
  for (int64_t i = 0; i < (int64_t)P * R; ++i) rowptr[i + 1] = rowptr[i] + len[i];
  for (const Slice& sl : pm.slices)
    for (int r = 0; r < kSliceRows; ++r) {
      const int row = pm.sorted_rows[sl.row0 + r];
      if (row < 0) continue;
      const int32_t q0 = rowptr[(int64_t)sl.p * R + row];
      for (int32_t e = 0; e < pm.sorted_len[sl.row0 + r]; ++e) {
        const uint32_t* entry = &pm.stream[stream_entry(sl.batch0, r, e)];
        colidx[q0 + e] = (int32_t)(entry[0] / ((uint32_t)kTileBlock * sizeof(float)));
        std::memcpy(&vals[q0 + e], &entry[1], sizeof(float));
      }
    }
}

int upload_packed(PackedMatrix* pm) {
  int rc;
  pm->on_device = false;
  HIP_TRY(hipDeviceSynchronize());  // a pass still in flight may read the buffers that are overwritten below
  if ((rc = upload(&pm->d_stream, pm->stream, &pm->cap_stream))) return rc;
  if ((rc = upload(&pm->d_slices, pm->slices, &pm->cap_slices))) return rc;
  if ((rc = upload(&pm->d_items, pm->items, &pm->cap_items))) return rc;
  if ((rc = upload(&pm->d_ranges, pm->ranges, &pm->cap_ranges))) return rc;
  HIP_TRY(hipDeviceSynchronize());
  pm->on_device = true;
  return SWCONV_OK;
}

void free_packed(PackedMatrix* pm) {
  void* bufs[] = {pm->d_stream, pm->d_slices, pm->d_items, pm->d_ranges};
  for (void* b : bufs)
    if (b) (void)hipFree(b);
  pm->d_stream = nullptr;
  pm->d_slices = nullptr;
  pm->d_items = nullptr;
  pm->d_ranges = nullptr;
  pm->cap_stream = pm->cap_slices = pm->cap_items = pm->cap_ranges = 0;
  pm->on_device = false;
}

// True when the schedule of `pm` is a partition of its (position, tile block, slice) units.
bool schedule_is_partition(const PackedMatrix& pm, int P, int ntb) {
  const int spp = pm.rows_padded / kSliceRows;
  std::vector<uint8_t> seen((size_t)P * ntb * spp, 0);
  if ((int)pm.wg_begin.size() != pm.n_wgs_used + 1 || pm.wg_begin[0] != 0 ||
      pm.wg_begin.back() != (int32_t)pm.items.size() || pm.n_wgs_used > std::max(1, pm.n_wgs))
    return false;
  for (int b = 0; b < pm.n_wgs_used; ++b)
    if (pm.wg_begin[b + 1] <= pm.wg_begin[b]) return false;  // no idle workgroup is launched
  for (const WorkItem& w : pm.items) {
    if (w.p < 0 || w.p >= P || w.tau_block < 0 || w.tau_block >= ntb) return false;
    if (w.slice_begin < w.p * spp || w.slice_end > (w.p + 1) * spp || w.slice_begin >= w.slice_end) return false;
    if (w.slice_end - w.slice_begin > pm.item_cap) return false;  // descriptors must fit their LDS area
    for (int sidx = w.slice_begin; sidx < w.slice_end; ++sidx) {
      uint8_t& f = seen[((size_t)w.p * ntb + w.tau_block) * spp + (sidx - w.p * spp)];
      if (f) return false;
      f = 1;
    }
  }
  for (uint8_t f : seen)
    if (!f) return false;
  return true;
}

int copy_padded_to_host(const float* dsrc, float* hdst, size_t rows, int T, int Tp) {
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy2D(hdst, (size_t)T * sizeof(float), dsrc, (size_t)Tp * sizeof(float), (size_t)T * sizeof(float),
                      rows, hipMemcpyDeviceToHost));
  return SWCONV_OK;
}

// After swconv_update_values the device stream of W_F holds the current values: fetch it before
// the host copy is read (transposition for the backward pass, export).
int refresh_host_values(swconv_plan* pl) {
  if (!pl->host_values_stale) return SWCONV_OK;
  HIP_TRY(hipDeviceSynchronize());
  HIP_TRY(hipMemcpy(pl->fw.stream.data(), pl->fw.d_stream, pl->fw.stream.size() * sizeof(uint32_t), hipMemcpyDeviceToHost));
  pl->host_values_stale = false;
  return SWCONV_OK;
}

// Packs W_F^T (per position: C rows of (k, weight) entries, k ascending) from the packed W_F and
// allocates the dL/dI_F workspace.  Host work; done by the first backward pass after set_weights.
int prepare_backward(swconv_plan* pl) {
  if (!pl->bt_supported) return SWCONV_EUNSUPPORTED;
  if (pl->bt_current && pl->bt.on_device && pl->dD) return SWCONV_OK;
  const int P = pl->P, K = pl->g.K, C = pl->g.C;
  try {
    const int64_t nnz = pl->fw.nnz;
    std::vector<int32_t> rp((size_t)P * K + 1), ci((size_t)nnz), trp((size_t)P * C + 1, 0), tci((size_t)nnz);
    std::vector<float> va((size_t)nnz), tva((size_t)nnz);
    std::vector<int32_t> t_to_orig((size_t)nnz);  // entry of the transposed CSR -> entry of the caller's CSR
    int rc0 = refresh_host_values(pl);
    if (rc0) return rc0;
    unpack_matrix(pl->fw, P, rp.data(), ci.data(), va.data());
    for (int p = 0; p < P; ++p)
      for (int32_t q = rp[(size_t)p * K]; q < rp[(size_t)(p + 1) * K]; ++q) ++trp[(size_t)p * C + ci[q] + 1];
    for (size_t i = 0; i < (size_t)P * C; ++i) trp[i + 1] += trp[i];
    std::vector<int32_t> fill(trp.begin(), trp.end() - 1);
    for (int p = 0; p < P; ++p)
      for (int k = 0; k < K; ++k)  // k ascending, so every transposed row gets its columns in ascending order
        for (int32_t q = rp[(size_t)p * K + k]; q < rp[(size_t)p * K + k + 1]; ++q) {
          const int32_t dst = fill[(size_t)p * C + ci[q]]++;
          tci[dst] = k;
          tva[dst] = va[q];
          t_to_orig[dst] = q;
        }
    size_grid(&pl->bt, (int64_t)P * pl->n_tau_blocks * (pl->bt.rows_padded / kSliceRows));
    pack_matrix(&pl->bt, P, pl->n_tau_blocks, trp.data(), tci.data(), tva.data());
    pl->bt_value_index.assign(pl->bt.entry_index.size(), -1);
    for (size_t e = 0; e < pl->bt.entry_index.size(); ++e)
      if (pl->bt.entry_index[e] >= 0) pl->bt_value_index[e] = t_to_orig[(size_t)pl->bt.entry_index[e]];
  } catch (const std::bad_alloc&) {
    pl->bt.packed = false;
    return SWCONV_ENOMEM;
  }
  int rc = upload_packed(&pl->bt);
  if (rc) return rc;
  if ((rc = upload(&pl->d_bt_value_index, pl->bt_value_index, &pl->cap_bt_value_index))) return rc;
  if (!pl->dD) {
    HIP_TRY(hipMalloc((void**)&pl->dD, pl->g.v_bytes));
    HIP_TRY(hipMemset(pl->dD, 0, pl->g.v_bytes));
  }
  if (pl->grad_images_per_group > 0 && !pl->d_gtiles && (rc = upload(&pl->d_gtiles, pl->gtiles))) return rc;
  pl->bt_current = true;
  return SWCONV_OK;
}

// Device copies the weight gradient needs: the stream-entry -> CSR index map and the partial-sum buffer.
int prepare_weight_grad(swconv_plan* pl) {
  const size_t need = (size_t)pl->n_tau_blocks * (pl->fw.stream.size() / 2);
  if (need * sizeof(float) >= ((size_t)1 << 40)) return SWCONV_EUNSUPPORTED;
  if (pl->partial_floats < need) {
    if (pl->d_partial) (void)hipFree(pl->d_partial);
    pl->d_partial = nullptr;
    pl->partial_floats = 0;
    HIP_TRY(hipMalloc((void**)&pl->d_partial, std::max<size_t>(need, 1) * sizeof(float)));
    pl->partial_floats = need;
  }
  if (!pl->index_current) {
    HIP_TRY(hipDeviceSynchronize());  // an earlier backward pass may still read the index
    int rc = upload(&pl->d_entry_index, pl->fw.entry_index, &pl->cap_entry_index);
    if (rc) return rc;
    HIP_TRY(hipDeviceSynchronize());
    pl->index_current = true;
  }
  return SWCONV_OK;
}

template <int M, int R>
int launch_backward_transforms(swconv_plan* pl, const LaunchTarget& to, int which, const float* dout,
                                      float* din) {
  const Geometry& g = pl->g;
  if (which == 0) {  // dL/dZ = A dL/dO~ A^T into the M workspace
    auto kern = output_grad_transform_kernel<M, R>;
    static bool attr_set = false;
    if (!attr_set) {
      HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
      attr_set = true;
    }
    return launch_kernel(kern, dim3(g.Tp / 64, (g.K + 3) / 4), dim3(256), (size_t)4 * g.out_area * sizeof(float), to,
                         dout, pl->dM, pl->d_tiles, pl->d_blocks, g);
  }
  if (which == 1 && pl->grad_images_per_group > 0) {  // both remaining steps at once, planes in LDS
    const int G = pl->grad_images_per_group;
    const size_t lds = (size_t)4 * (((size_t)G * g.H * g.W + 63) / 64 * 64 + 64) * sizeof(float);
    auto kern = input_grad_kernel<M, R>;
    static bool attr_set = false;
    if (!attr_set) {
      HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes));
      attr_set = true;
    }
    return launch_kernel(kern, dim3((g.N + G - 1) / G, (g.C + 3) / 4), dim3(256), lds, to, (const float*)pl->dD, din,
                         (const GradTile*)pl->d_gtiles, G, g);
  }
  if (which == 1)  // dL/dI~ = B dL/dI_F B^T, from the dL/dI_F workspace into the V workspace
    return launch_kernel(input_grad_patch_kernel<M, R>, dim3(g.Tp / 64, (g.C + 3) / 4), dim3(256), 0, to, pl->dD, pl->dV,
                         g);
  const int cells = ((g.H - 1 + g.pad) / M + 1) * ((g.W - 1 + g.pad) / M + 1);
  const int64_t threads = (int64_t)g.N * g.C * cells;
  return launch_kernel(input_grad_gather_kernel<M, R>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, to, pl->dV,
                       din, g);
}

// The kernels of the backward pass, in launch order.
//   0  dL/dZ = A dL/dO~ A^T                      (Eq. 5, first line)      -> M workspace
//   1  I_F = B^T I~ B again (forward step 1)                              -> V workspace   } only for
//   2  per stored entry and tile block: <dL/dZ row, I_F row>              -> partial sums  } dL/dW_F
//   3  sum over the tile blocks, CSR order        (Eq. 5, second line)    -> dvals         }
//   4  dL/dI_F[p] = W_F[p]^T dL/dZ[p]             (Eq. 6, first line)     -> dL/dI_F workspace
//   5  dL/dI~ = B dL/dI_F B^T                     (Eq. 6, second line)    -> V workspace   } only for
//   6  every pixel gathers its patch entries      (Eq. 6, third line)     -> din           } dL/dI
constexpr int kBackwardStages = 7;

bool backward_stage_runs(const swconv_plan* pl, int stage, const float* in, const float* din, const float* dvals) {
  if (stage == 1 && !in) return false;  // I_F of the last forward pass is still in the V workspace
  if (stage >= 1 && stage <= 3) return dvals != nullptr && pl->fw.nnz > 0;
  if (stage == 6 && pl->grad_images_per_group > 0) return false;  // stage 5 did both
  if (stage >= 5) return din != nullptr;
  return true;
}

int backward_ready(swconv_plan* pl, const float* in_dev, const float* dout_dev, const float* dvals_dev) {
  if (!pl || !dout_dev) return SWCONV_EINVAL;
  if (!pl->fw.on_device) return SWCONV_ESTATE;
  if (!in_dev && dvals_dev && !pl->ran_forward) return SWCONV_ESTATE;  // no I_F to reuse
  if ((int64_t)pl->g.N * pl->g.C * (pl->g.H + pl->m) * (pl->g.W + pl->m) >= ((int64_t)1 << 31)) return SWCONV_EUNSUPPORTED;  // 32-bit cell index of the gather
  int rc = prepare_backward(pl);
  if (rc) return rc;
  return dvals_dev ? prepare_weight_grad(pl) : SWCONV_OK;
}

int launch_backward_stage(swconv_plan* pl, const LaunchTarget& to, int stage, const float* in_dev,
                          const float* dout_dev, float* din_dev, float* dvals_dev) {
  if (!backward_stage_runs(pl, stage, in_dev, din_dev, dvals_dev)) return SWCONV_OK;
  switch (stage) {
    case 0:
      return dispatch_mr(pl, [&](auto M, auto R) {
        return launch_backward_transforms<M(), R()>(pl, to, 0, dout_dev, nullptr);
      });
    case 1: return launch_stage(pl, to, 0, in_dev, nullptr);
    case 2:
      return launch_spmm_mode<true>(pl, pl->fw, to, pl->dV, pl->g.v_bytes, pl->dM, pl->g.m_bytes, pl->d_partial);
    case 3: {
      const uint32_t n_entries = (uint32_t)(pl->fw.stream.size() / 2);
      return launch_kernel(weight_grad_reduce_kernel, dim3((n_entries + 255) / 256), dim3(256), 0, to,
                           (const float*)pl->d_partial, pl->n_tau_blocks, n_entries,
                           (const int32_t*)pl->d_entry_index, n_entries, dvals_dev);
    }
    case 4: return launch_spmm(pl, pl->bt, to, pl->dM, pl->g.m_bytes, pl->dD, pl->g.v_bytes);
    default:
      return dispatch_mr(pl, [&](auto M, auto R) {
        return launch_backward_transforms<M(), R()>(pl, to, stage - 4, nullptr, din_dev);
      });
  }
}

}  // namespace

extern "C" {

const char* swconv_status_string(int status) {
  switch (status) {
    case SWCONV_OK: return "SWCONV_OK";
    case SWCONV_EINVAL: return "SWCONV_EINVAL: invalid argument";
    case SWCONV_EUNSUPPORTED: return "SWCONV_EUNSUPPORTED: unsupported configuration";
    case SWCONV_ENOMEM: return "SWCONV_ENOMEM: out of memory";
    case SWCONV_EHIP: return "SWCONV_EHIP: HIP runtime error";
    case SWCONV_ESTATE: return "SWCONV_ESTATE: weights not set or no forward pass yet";
    default: return "unknown swconv status";
  }
}

int swconv_plan_create(swconv_plan** out, int N, int C, int H, int W, int K, int m, int r, int pad) {
  if (!out) return SWCONV_EINVAL;
  if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || pad < 0 || m < 1 || r < 1) return SWCONV_EINVAL;
  if (!((m == 2 || m == 4) && (r == 3 || r == 5))) return SWCONV_EUNSUPPORTED;
  const int64_t Ho = (int64_t)H + 2 * pad - r + 1, Wo = (int64_t)W + 2 * pad - r + 1;
  if (Ho < 1 || Wo < 1) return SWCONV_EINVAL;
  const int t = m + r - 1, P = t * t;
  const int64_t th = (Ho + m - 1) / m, tw = (Wo + m - 1) / m;
  const int64_t T = (int64_t)N * th * tw;
  const int64_t lim = (int64_t)1 << 31;
  // every flat index the kernels form in 32 bits, and the CSR offsets, must fit int32
  if (T + 256 >= lim || (int64_t)P * K * C >= lim || (int64_t)H * W >= lim || Ho * Wo >= lim ||
      (int64_t)N * C * H * W >= ((int64_t)1 << 40) || (int64_t)P * (K + 4) >= lim)
    return SWCONV_EINVAL;

  swconv_plan* pl = new (std::nothrow) swconv_plan();
  if (!pl) return SWCONV_ENOMEM;
  if (!configure_packed(&pl->fw, K, C)) {  // the C x 64 panel of the sparse product must fit LDS
    delete pl;
    return SWCONV_EUNSUPPORTED;
  }
  pl->bt_supported = configure_packed(&pl->bt, C, K);  // the backward pass stages K x 64 panels of dL/dZ
  pl->m = m;
  pl->r = r;
  pl->t = t;
  pl->P = P;
  Geometry& g = pl->g;
  g.N = N; g.C = C; g.H = H; g.W = W; g.K = K; g.pad = pad;
  g.Ho = (int)Ho; g.Wo = (int)Wo; g.th = (int)th; g.tw = (int)tw; g.tpi = (int)(th * tw);
  g.T = (int)T;
  // row pitch of V and M: whole 64-tile blocks (transforms, sparse product) and a multiple of 128
  // for the dense comparison GEMM
  g.Tp = (int)((T + 127) / 128 * 128);
  // V and M are addressed with 32-bit byte offsets (buffer descriptors)
  if ((int64_t)P * std::max(C, K) * g.Tp * (int64_t)sizeof(float) >= ((int64_t)1 << 32) - 256) {
    delete pl;
    return SWCONV_EUNSUPPORTED;
  }
  g.v_bytes = (uint32_t)((int64_t)P * C * g.Tp * (int64_t)sizeof(float));
  g.m_bytes = (uint32_t)((int64_t)P * K * g.Tp * (int64_t)sizeof(float));
  // a block of 64 consecutive tiles touches at most this many images
  g.slots = (int)std::min<int64_t>(N, (64 + g.tpi - 2) / g.tpi + 1);
  pl->n_tau_blocks = (g.T + kTileBlock - 1) / kTileBlock;
  if (H >= 32768 || W >= 32768) {  // 16-bit fields of the tile table
    delete pl;
    return SWCONV_EUNSUPPORTED;
  }
  g.wo_magic = (uint32_t)((((uint64_t)1 << 32) + g.Wo - 1) / g.Wo);
  g.m_shift = m == 4 ? 2 : 1;
  g.in_image_stride = (int64_t)C * H * W;
  g.out_image_stride = (int64_t)K * Ho * Wo;
  // steps 2 and 3 in one kernel: m = 2 (16 output accumulators per lane) and a panel of at most
  // kFusedMaxPieces 16-byte pieces per thread
  // or F(4x4,3x3) with two C x 64 panels in LDS and whole groups of four panel rows
  const int fuse_mode = env_int("SWCONV_FUSE_OUTPUT", 1);
  pl->fz.out_tile = m;
  pl->fz.mode = fuse_mode;
  if (m == 2)
    pl->fz.eligible = C * (kTileBlock / 4) <= kFusedMaxPieces * kFusedWaves * 64 && fuse_mode != 0;
  else
    pl->fz.eligible = r == 3 && C % 4 == 0 && C <= kFused4MaxC && fuse_mode != 0;  // and its staging area, see below
  try {
    if (pl->fz.eligible && m == 2) pl->fz.otiles.assign((size_t)g.Tp, OutTile{0, 0u, 0u, 0u});
    build_transform_tables(pl);
  } catch (const std::bad_alloc&) {
    delete pl;
    return SWCONV_ENOMEM;
  }
  if (m == 4 && g.out_area > kFused4MaxOutArea) pl->fz.eligible = false;  // output rows of a tile block: staged per wave
  // backward pass, Eq. 6 second and third line in one kernel: G = 64 / (tiles per image) whole
  // images per wave (at least one), if four waves' planes fit LDS
  {
    const int G = (int)std::min<int64_t>(N, std::max<int64_t>(1, 64 / g.tpi));
    const int64_t wave_floats = ((int64_t)G * H * W + 63) / 64 * 64 + 64;
    // (with patches reaching two tiles back, F(2x2,5x5), its nine phases measured slower than the two kernels;
    // with 8 x 8 patches, F(4x4,5x5), patch, transform and LDS indices together overflow the 256 vector registers)
    if (4 * wave_floats * (int64_t)sizeof(float) <= kMaxLdsBytes && (t - 1) / m == 1 && t <= 6 &&
        env_int("SWCONV_FUSE_INPUT_GRAD", 1) != 0) {
      try {
        GradTile none;
        none.org = 0;
        none.yx0 = (int32_t)0x80008000u;
        pl->gtiles.assign((size_t)g.Tp, none);
        for (int64_t tau = 0; tau < T; ++tau) {
          const int n = (int)(tau / g.tpi), tl = (int)(tau % g.tpi), ty = tl / g.tw, tx = tl % g.tw;
          const int y0 = ty * m - pad, x0 = tx * m - pad;
          pl->gtiles[(size_t)tau].org = (n % G) * H * W;
          pl->gtiles[(size_t)tau].yx0 = (int32_t)(((uint32_t)y0 & 0xffffu) | ((uint32_t)x0 << 16));
        }
        pl->grad_images_per_group = G;
      } catch (const std::bad_alloc&) {
        delete pl;
        return SWCONV_ENOMEM;
      }
    }
  }
  // LDS staging areas of the transform kernels (four waves per workgroup)
  if ((int64_t)4 * std::max(g.in_area, g.out_area) * (int64_t)sizeof(float) > kMaxLdsBytes) {
    delete pl;
    return SWCONV_EUNSUPPORTED;
  }
  *out = pl;
  return SWCONV_OK;
}

int swconv_plan_set_image_strides(swconv_plan* pl, int64_t in_stride, int64_t out_stride) {
  if (!pl) return SWCONV_EINVAL;
  const Geometry& g = pl->g;
  const int64_t in_min = (int64_t)g.C * g.H * g.W, out_min = (int64_t)g.K * g.Ho * g.Wo;
  if (in_stride == 0) in_stride = in_min;
  if (out_stride == 0) out_stride = out_min;
  // the last image must still be addressable with the 40-bit bound plan_create checks
  if (in_stride < in_min || out_stride < out_min || in_stride > ((int64_t)1 << 40) / g.N ||
      out_stride > ((int64_t)1 << 40) / g.N)
    return SWCONV_EINVAL;
  pl->g.in_image_stride = in_stride;
  pl->g.out_image_stride = out_stride;
  return SWCONV_OK;
}

void swconv_plan_destroy(swconv_plan* pl) {
  if (!pl) return;
  void* bufs[] = {pl->dV, pl->dM, pl->dD, pl->d_partial, pl->d_entry_index, pl->d_wdense, pl->d_tiles, pl->d_blocks};
  for (void* b : bufs)
    if (b) (void)hipFree(b);
  free_packed(&pl->fw);
  free_packed(&pl->bt);
  void* fused[] = {pl->fz.d_wpk, pl->fz.d_lens, pl->fz.d_otiles, pl->d_gtiles, pl->fz.d_value_index, pl->d_bt_value_index};
  for (void* b : fused)
    if (b) (void)hipFree(b);
  delete pl;
}

int swconv_set_weights(swconv_plan* pl, const int32_t* rowptr, const int32_t* colidx, const float* vals) {
  if (!pl) return SWCONV_EINVAL;
  int rc = validate_csr(pl, rowptr, colidx, vals);
  if (rc) return rc;
  size_grid(&pl->fw, (int64_t)pl->P * pl->n_tau_blocks * (pl->fw.rows_padded / kSliceRows));
  pl->bt_current = false;
  pl->index_current = false;
  pl->host_values_stale = false;
  pl->fz.ready = false;
  // what the workspaces hold belongs to the old weights: the products are stale, and a backward pass
  // must not pair I_F of an earlier pass with the new pattern without a forward pass in between
  pl->m_current = false;
  pl->ran_forward = false;
  try {
    pack_matrix(&pl->fw, pl->P, pl->n_tau_blocks, rowptr, colidx, vals);
    pack_fused(pl, rowptr, colidx, vals);
    // The F(4x4,3x3) kernel runs only where asked for (SWCONV_FUSE_OUTPUT=2): with 64 + 16 accumulators per
    // lane it holds 16 waves per CU, its vector ALU stays at about two thirds busy between the barriers of
    // the 36 positions, and on the 56 x 56 layer it measured 217 us against 188 us for the two kernels.
    pl->fz.wanted = pl->fz.out_tile == 2 || pl->fz.mode == 2;
  } catch (const std::bad_alloc&) {
    pl->fw.packed = false;
    pl->fw.on_device = false;
    pl->fz.ready = false;
    return SWCONV_ENOMEM;
  }
  if ((rc = ensure_workspace(pl))) return rc;
  if ((rc = upload_packed(&pl->fw))) return rc;
  return upload_fused(pl);
}

int swconv_forward(swconv_plan* pl, void* hip_stream, const float* in_dev, float* out_dev) {
  if (!pl || !in_dev || !out_dev) return SWCONV_EINVAL;
  if (!pl->fw.on_device) return SWCONV_ESTATE;
  const LaunchTarget to{(hipStream_t)hip_stream, nullptr, nullptr};
  for (int stage = 0; stage < 3; ++stage) {
    if (!forward_stage_runs(pl, stage)) continue;
    int rc = launch_stage(pl, to, stage, in_dev, out_dev);
    if (rc) return rc;
  }
  pl->ran_forward = true;
  pl->m_current = !fused_runs(pl);
  return SWCONV_OK;
}

int swconv_forward_noalloc(swconv_plan* pl, void* hip_stream, const float* in_dev, float* out_dev) {
  if (!pl || !in_dev || !out_dev) return SWCONV_EINVAL;
  if (!pl->fw.on_device) return SWCONV_ESTATE;
  // V, then M behind it on a 256-byte boundary
  const size_t m_at = ((size_t)pl->g.v_bytes + 255) / 256 * 256;
  if (m_at + (size_t)pl->g.m_bytes > kStaticScratchBytes) return SWCONV_EUNSUPPORTED;
  void* base = nullptr;
  int rc = static_scratch(&base);
  if (rc) return rc;
  const Workspace ws{reinterpret_cast<float*>(base), reinterpret_cast<float*>(static_cast<unsigned char*>(base) + m_at)};
  const LaunchTarget to{(hipStream_t)hip_stream, nullptr, nullptr};
  // Nothing in the scratch has to start at zero: step 1 writes every column of V the later steps
  // read (the pad columns included), step 2 every row of M that step 3 reads.
  for (int stage = 0; stage < 3; ++stage) {
    if (!forward_stage_runs(pl, stage)) continue;
    if ((rc = launch_stage(pl, to, stage, in_dev, out_dev, ws))) return rc;
  }
  // the plan's own workspaces hold nothing of this pass
  pl->ran_forward = false;
  pl->m_current = false;
  return SWCONV_OK;
}

int swconv_profile_forward(swconv_plan* pl, void* hip_stream, const float* in_dev, float* out_dev, int iters,
                           float* stage_ms) {
  if (!pl || !in_dev || !out_dev || !stage_ms || iters < 1) return SWCONV_EINVAL;
  if (!pl->fw.on_device) return SWCONV_ESTATE;
  hipStream_t st = (hipStream_t)hip_stream;
  // one (start, stop) pair per kernel launch; the events take the kernel's own time stamps
  std::vector<hipEvent_t> ev((size_t)iters * 6, nullptr);
  int rc = SWCONV_OK;
  for (auto& e : ev)
    if (hipEventCreate(&e) != hipSuccess) rc = SWCONV_EHIP;
  for (int it = 0; it < iters && !rc; ++it)
    for (int stage = 0; stage < 3 && !rc; ++stage) {
      if (!forward_stage_runs(pl, stage)) continue;
      hipEvent_t* e = &ev[((size_t)it * 3 + stage) * 2];
      rc = launch_stage(pl, LaunchTarget{st, e[0], e[1]}, stage, in_dev, out_dev);
    }
  if (hipStreamSynchronize(st) != hipSuccess) rc = rc ? rc : SWCONV_EHIP;
  if (!rc) {
    double sum[3] = {0, 0, 0};
    for (int it = 0; it < iters && !rc; ++it)
      for (int stage = 0; stage < 3; ++stage) {
        if (!forward_stage_runs(pl, stage)) continue;
        hipEvent_t* e = &ev[((size_t)it * 3 + stage) * 2];
        float ms = 0;
        if (hipEventElapsedTime(&ms, e[0], e[1]) != hipSuccess) {
          rc = SWCONV_EHIP;
          break;
        }
        sum[stage] += ms;
      }
    if (!rc)
      for (int stage = 0; stage < 3; ++stage) stage_ms[stage] = (float)(sum[stage] / iters);
    pl->ran_forward = true;
    pl->m_current = !fused_runs(pl);
  }
  for (auto& e : ev)
    if (e) (void)hipEventDestroy(e);
  if (rc) (void)hipGetLastError();
  return rc;
}

int swconv_backward(swconv_plan* pl, void* hip_stream, const float* in_dev, const float* dout_dev, float* din_dev,
                    float* dvals_dev) {
  int rc = backward_ready(pl, in_dev, dout_dev, dvals_dev);
  if (rc) return rc;
  for (int stage = 0; stage < kBackwardStages; ++stage)
    if ((rc = launch_backward_stage(pl, LaunchTarget{(hipStream_t)hip_stream, nullptr, nullptr}, stage, in_dev,
                                    dout_dev, din_dev, dvals_dev)))
      return rc;
  pl->ran_forward = false;  // the V workspace no longer holds I_F
  pl->ran_backward = true;
  return SWCONV_OK;
}

int swconv_profile_backward(swconv_plan* pl, void* hip_stream, const float* in_dev, const float* dout_dev,
                            float* din_dev, float* dvals_dev, int iters, float* stage_ms) {
  if (!stage_ms || iters < 1) return SWCONV_EINVAL;
  int rc = backward_ready(pl, in_dev, dout_dev, dvals_dev);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  // one (start, stop) pair per kernel launch; the events take the kernel's own time stamps
  std::vector<hipEvent_t> ev((size_t)iters * kBackwardStages * 2, nullptr);
  for (auto& e : ev)
    if (hipEventCreate(&e) != hipSuccess) rc = SWCONV_EHIP;
  for (int it = 0; it < iters && !rc; ++it)
    for (int stage = 0; stage < kBackwardStages && !rc; ++stage) {
      hipEvent_t* e = &ev[((size_t)it * kBackwardStages + stage) * 2];
      rc = launch_backward_stage(pl, LaunchTarget{st, e[0], e[1]}, stage, in_dev, dout_dev, din_dev, dvals_dev);
    }
  if (hipStreamSynchronize(st) != hipSuccess) rc = rc ? rc : SWCONV_EHIP;
  if (!rc) {
    for (int stage = 0; stage < kBackwardStages; ++stage) {
      double sum = 0;
      if (backward_stage_runs(pl, stage, in_dev, din_dev, dvals_dev))
        for (int it = 0; it < iters && !rc; ++it) {
          hipEvent_t* e = &ev[((size_t)it * kBackwardStages + stage) * 2];
          float ms = 0;
          if (hipEventElapsedTime(&ms, e[0], e[1]) != hipSuccess) rc = SWCONV_EHIP;
          sum += ms;
        }
      stage_ms[stage] = (float)(sum / iters);
    }
    pl->ran_forward = false;
    pl->ran_backward = true;
  }
  for (auto& e : ev)
    if (e) (void)hipEventDestroy(e);
  if (rc) (void)hipGetLastError();
  return rc;
}

int swconv_debug_copy_dZ(swconv_plan* pl, float* dZ_host) {
  if (!pl || !dZ_host) return SWCONV_EINVAL;
  if (!pl->ran_backward) return SWCONV_ESTATE;
  return copy_padded_to_host(pl->dM, dZ_host, (size_t)pl->P * pl->g.K, pl->g.T, pl->g.Tp);
}

int swconv_debug_copy_dV(swconv_plan* pl, float* dV_host) {
  if (!pl || !dV_host) return SWCONV_EINVAL;
  if (!pl->ran_backward) return SWCONV_ESTATE;
  return copy_padded_to_host(pl->dD, dV_host, (size_t)pl->P * pl->g.C, pl->g.T, pl->g.Tp);
}

int swconv_prune_step(int64_t rows, const int32_t* rowptr_dev, const int32_t* colidx_dev, const float* vals_dev,
                      const float* grad_dev, float eta, float lambda, float eps, float beta, void* hip_stream,
                      float* updated_dev, int32_t* rowptr_out_dev, int32_t* colidx_out_dev, float* vals_out_dev) {
  if (rows < 1 || rows >= ((int64_t)1 << 31) - 256 || !rowptr_dev || !updated_dev || !rowptr_out_dev ||
      !colidx_out_dev || !vals_out_dev)
    return SWCONV_EINVAL;
  if (!(eta >= 0.0f) || !(lambda >= 0.0f) || !(eps >= 0.0f) || !(beta >= 0.0f)) return SWCONV_EINVAL;
  const LaunchTarget to{(hipStream_t)hip_stream, nullptr, nullptr};
  const dim3 grid((unsigned)((rows + 255) / 256));
  int rc;
  if ((rc = launch_kernel(prune_update_kernel, grid, dim3(256), 0, to, rows, rowptr_dev, vals_dev, grad_dev, eta, lambda,
                          eps, beta, updated_dev, rowptr_out_dev)))
    return rc;
  if ((rc = launch_kernel(prune_scan_kernel, dim3(1), dim3(1024), 0, to, rows, rowptr_out_dev))) return rc;
  return launch_kernel(prune_compact_kernel, grid, dim3(256), 0, to, rows, rowptr_dev, colidx_dev, vals_dev, grad_dev,
                       eta, lambda, eps, beta, (const int32_t*)rowptr_out_dev, colidx_out_dev, vals_out_dev);
}

int swconv_set_weights_device(swconv_plan* pl, void* hip_stream, const int32_t* rowptr_dev, const int32_t* colidx_dev,
                              const float* vals_dev) {
  if (!pl || !rowptr_dev) return SWCONV_EINVAL;
  const size_t rows = (size_t)pl->P * pl->g.K;
  try {
    std::vector<int32_t> rp(rows + 1);
    if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess ||
        hipMemcpy(rp.data(), rowptr_dev, rp.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess) {
      (void)hipGetLastError();
      return SWCONV_EHIP;
    }
    const int64_t nnz = rp[rows];
    if (rp[0] != 0 || nnz < 0 || nnz > (int64_t)rows * pl->g.C) return SWCONV_EINVAL;
    if (nnz > 0 && (!colidx_dev || !vals_dev)) return SWCONV_EINVAL;
    std::vector<int32_t> ci((size_t)nnz);
    std::vector<float> va((size_t)nnz);
    if (nnz > 0 && (hipMemcpy(ci.data(), colidx_dev, ci.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
                    hipMemcpy(va.data(), vals_dev, va.size() * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess)) {
      (void)hipGetLastError();
      return SWCONV_EHIP;
    }
    return swconv_set_weights(pl, rp.data(), ci.data(), va.data());
  } catch (const std::bad_alloc&) {
    return SWCONV_ENOMEM;
  }
}

int swconv_update_values(swconv_plan* pl, void* hip_stream, const float* vals_dev) {
  if (!pl) return SWCONV_EINVAL;
  if (!pl->fw.on_device) return SWCONV_ESTATE;
  if (pl->fw.nnz == 0) return SWCONV_OK;
  if (!vals_dev) return SWCONV_EINVAL;
  int rc;
  if (!pl->index_current) {  // the pair -> CSR index map of W_F (also used by the weight gradient)
    HIP_TRY(hipDeviceSynchronize());
    if ((rc = upload(&pl->d_entry_index, pl->fw.entry_index, &pl->cap_entry_index))) return rc;
    pl->index_current = true;
  }
  const LaunchTarget to{(hipStream_t)hip_stream, nullptr, nullptr};
  auto refresh = [&](uint32_t* pairs, const int32_t* index, size_t n_pairs) {
    return launch_kernel(refresh_values_kernel, dim3((unsigned)((n_pairs + 255) / 256)), dim3(256), 0, to, pairs, index,
                         (uint32_t)n_pairs, vals_dev);
  };
  if ((rc = refresh(pl->fw.d_stream, pl->d_entry_index, pl->fw.stream.size() / 2))) return rc;
  if (pl->fz.ready && (rc = refresh(pl->fz.d_wpk, pl->fz.d_value_index, pl->fz.wpk.size() / 2))) return rc;
  if (pl->bt_current && pl->bt.on_device &&
      (rc = refresh(pl->bt.d_stream, pl->d_bt_value_index, pl->bt.stream.size() / 2)))
    return rc;
  pl->host_values_stale = true;
  return SWCONV_OK;
}

int swconv_debug_copy_V(swconv_plan* pl, float* V_host) {
  if (!pl || !V_host) return SWCONV_EINVAL;
  if (!pl->ran_forward) return SWCONV_ESTATE;
  return copy_padded_to_host(pl->dV, V_host, (size_t)pl->P * pl->g.C, pl->g.T, pl->g.Tp);
}

int swconv_debug_copy_M(swconv_plan* pl, float* M_host) {
  if (!pl || !M_host) return SWCONV_EINVAL;
  if (!pl->ran_forward) return SWCONV_ESTATE;
  if (!pl->m_current) {  // the fused kernel kept the products on chip: run step 2 alone on the V of that pass
    HIP_TRY(hipDeviceSynchronize());
    int rc = launch_spmm(pl, pl->fw, LaunchTarget{nullptr, nullptr, nullptr}, pl->dV, pl->g.v_bytes, pl->dM, pl->g.m_bytes);
    if (rc) return rc;
    pl->m_current = true;
  }
  return copy_padded_to_host(pl->dM, M_host, (size_t)pl->P * pl->g.K, pl->g.T, pl->g.Tp);
}

int swconv_debug_export_weights(swconv_plan* pl, int32_t* rowptr, int32_t* colidx, float* vals) {
  if (!pl || !rowptr) return SWCONV_EINVAL;
  if (!pl->fw.packed) return SWCONV_ESTATE;
  if (pl->fw.nnz > 0 && (!colidx || !vals)) return SWCONV_EINVAL;
  int rc = refresh_host_values(pl);
  if (rc) return rc;
  unpack_matrix(pl->fw, pl->P, rowptr, colidx, vals);
  return SWCONV_OK;
}

int swconv_debug_check_schedule(const swconv_plan* pl) {
  if (!pl) return SWCONV_EINVAL;
  if (!pl->fw.packed) return SWCONV_ESTATE;
  return schedule_is_partition(pl->fw, pl->P, pl->n_tau_blocks) ? SWCONV_OK : SWCONV_EINVAL;
}

int swconv_plan_sizes(const swconv_plan* pl, int* P, int64_t* T, int* Ho, int* Wo) {
  if (!pl) return SWCONV_EINVAL;
  if (P) *P = pl->P;
  if (T) *T = pl->g.T;
  if (Ho) *Ho = pl->g.Ho;
  if (Wo) *Wo = pl->g.Wo;
  return SWCONV_OK;
}

int swconv_plan_weight_stats(const swconv_plan* pl, int64_t* nnz, int64_t* padded_nnz, int* work_items,
                             int64_t* max_item) {
  if (!pl) return SWCONV_EINVAL;
  if (!pl->fw.packed) return SWCONV_ESTATE;
  if (nnz) *nnz = pl->fw.nnz;
  if (padded_nnz) *padded_nnz = pl->fw.padded_nnz;
  if (work_items) *work_items = (int)pl->fw.items.size();
  if (max_item) *max_item = pl->fw.max_item;
  return SWCONV_OK;
}

int swconv_set_weights_dense(swconv_plan* pl, const float* wf) {
  if (!pl || !wf) return SWCONV_EINVAL;
  int rc = ensure_workspace(pl);
  if (rc) return rc;
  pl->dense_on_device = false;
  // transpose to [P][C][Kq], output channels fastest, zero padded to the GEMM's row tile
  const int P = pl->P, K = pl->g.K, C = pl->g.C;
  const int Kq = (K + kDenseTileM - 1) / kDenseTileM * kDenseTileM;
  std::vector<float> wt;
  try {
    wt.assign((size_t)P * C * Kq, 0.0f);
  } catch (const std::bad_alloc&) {
    return SWCONV_ENOMEM;
  }
  for (int p = 0; p < P; ++p)
    for (int k = 0; k < K; ++k)
      for (int c = 0; c < C; ++c) wt[((size_t)p * C + c) * Kq + k] = wf[((size_t)p * K + k) * C + c];
  if ((rc = upload(&pl->d_wdense, wt))) return rc;
  pl->Kq = Kq;
  pl->dense_on_device = true;
  return SWCONV_OK;
}

int swconv_forward_dense(swconv_plan* pl, void* hip_stream, const float* in_dev, float* out_dev) {
  if (!pl || !in_dev || !out_dev) return SWCONV_EINVAL;
  if (!pl->dense_on_device) return SWCONV_ESTATE;
  hipStream_t st = (hipStream_t)hip_stream;
  const LaunchTarget to{st, nullptr, nullptr};
  int rc = launch_stage(pl, to, 0, in_dev, out_dev);
  if (rc) return rc;
  {
    const Geometry& g = pl->g;
    dim3 grid((g.Tp + kDenseTileN - 1) / kDenseTileN, (g.K + kDenseTileM - 1) / kDenseTileM, pl->P);
    hipLaunchKernelGGL(dense_position_gemm_kernel, grid, dim3(256), 0, st, pl->d_wdense, pl->dV, pl->dM, g.K,
                       pl->Kq, g.C, g.Tp);
    HIP_TRY(hipGetLastError());
  }
  rc = launch_stage(pl, to, 2, in_dev, out_dev);
  if (rc) return rc;
  pl->ran_forward = true;
  pl->m_current = true;
  return SWCONV_OK;
}

}  // extern "C"
