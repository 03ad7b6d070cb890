// C ABI of the Adam-mini step library (include/adam_mini.h): argument checks,
// device work tables, kernel dispatch.  All arithmetic is in am_kernels.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/adam_mini.h"
#include "am_kernels.h"
#include "am_layout.h"

// Work tables, partial sums and step scales of adam_mini_step_static: one array per GPU, part of the
// library's code object, so that entry point never allocates.  Every GPU the library runs on holds its
// own copy from the moment the code object is loaded until the process ends.
static __device__ __align__(256) unsigned char scratch[ADAM_MINI_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_hip_error;
std::mutex g_tuning_mutex;
AmTuning g_tuning;

int hip_fail(hipError_t e, const char* what) {
  g_hip_error = std::string(what) + ": " + hipGetErrorString(e);
  (void)hipGetLastError();  // clear the sticky per-thread error
  return e == hipErrorOutOfMemory ? ADAM_MINI_OUT_OF_MEMORY : ADAM_MINI_HIP_ERROR;
}

#define AM_HIP(call)                                   \
  do {                                                 \
    hipError_t e_ = (call);                            \
    if (e_ != hipSuccess) return hip_fail(e_, #call);  \
  } while (0)

// RAII: make the layout's device current for the duration of a call.
struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  int enter(int device) {
    AM_HIP(hipGetDevice(&prev));
    if (prev != device) {
      AM_HIP(hipSetDevice(device));
      switched = true;
    }
    return ADAM_MINI_OK;
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

}  // namespace

// Device memory a step works in besides the caller's tensors.
struct AmDeviceMem {
  AmSeg* segs = nullptr;       // all buckets' segments, concatenated
  uint32_t* keys = nullptr;    // [3 * n_segs]: item_first of every segment, then lblock_first, then the item_first
                               // of the second work-item numbering (column-block update pass)
  float* partials = nullptr;   // LARGE: one float per chunk; STRIDED: [row chunks][columns] per tensor
  float* scales = nullptr;     // LARGE: one step scale per large block; STRIDED: one per column
  AmScalars* scalars = nullptr;  // the step's scalars of adam_mini_step_device_hparams
};

// The pointer lists a segment table currently holds.
struct AmPointerCache {
  bool valid = false;
  std::vector<const void*> p, g, m;
  bool same(void* const* params, const void* const* grads, void* const* exp_avg, size_t n) const {
    return valid && std::memcmp(p.data(), params, n * sizeof(void*)) == 0 &&
           std::memcmp(g.data(), grads, n * sizeof(void*)) == 0 &&
           std::memcmp(m.data(), exp_avg, n * sizeof(void*)) == 0;
  }
  void keep(void* const* params, const void* const* grads, void* const* exp_avg, size_t n) {
    std::memcpy(p.data(), params, n * sizeof(void*));
    std::memcpy(g.data(), grads, n * sizeof(void*));
    std::memcpy(m.data(), exp_avg, n * sizeof(void*));
    valid = true;
  }
};

struct adam_mini_layout {
  AmHostLayout host;
  int device = -1;
  uint64_t uid = 0;                // never reused, unlike the handle's address
  size_t lds_per_cu = 160 * 1024;  // read from the device by the first call that launches
  bool lds_per_cu_known = false;
  // device state, created by the first call that needs it
  bool device_ready = false;
  AmDeviceMem mem;                 // the layout's own allocations
  AmPointerCache cache;            // pointer lists held by mem.segs
  AmPointerCache static_cache;     // pointer lists this layout last wrote into the static scratch
  std::vector<unsigned char> static_image;  // host staging of those tables (so that entry point allocates no host memory either)
  // optional per-bucket timing: events[(step * n_buckets + bucket) * 2 + {0,1}]
  std::vector<hipEvent_t> events;
  uint32_t profile_capacity = 0;   // steps the pool can hold
  uint32_t profile_used = 0;       // steps recorded since the last read
  std::vector<double> bucket_ms;
  std::vector<uint64_t> bucket_launches;
};

namespace {

// ---------------------------------------------------------------------------
// kernel dispatch: the variant lists must match am_layout.cpp
// ---------------------------------------------------------------------------
#define AM_ROW_VARIANTS(X)                                                                              \
  X(16, 1) X(16, 2) X(16, 4)                                                                            \
  X(64, 1) X(64, 2) X(64, 4) X(64, 8) X(64, 16)                                                         \
  X(256, 1) X(256, 2) X(256, 3) X(256, 4) X(256, 6) X(256, 8) X(256, 12) X(256, 16)                     \
  X(512, 1) X(512, 2) X(512, 3) X(512, 4) X(512, 6) X(512, 8)                                           \
  X(1024, 1) X(1024, 2) X(1024, 3) X(1024, 4) X(1024, 6)
#define AM_LARGE_VARIANTS(X) X(256, 1) X(256, 2) X(256, 4) X(256, 8) X(256, 16)
#define AM_EW_VARIANTS(X) X(256, 1) X(256, 2) X(256, 4) X(256, 8)

// Does the instantiation exist?  (Register-heavy combinations are never chosen by the layout builder
// and are compiled out.)
constexpr bool am_row_ok(int vec, int lanes, int upt) {
  return upt * vec * 3 + 34 <= (lanes >= 1024 ? 128 : 256);
}

// Dynamic LDS bytes that leave room for exactly `cap` workgroups per CU (0 = no cap).  The kernels
// never touch this allocation: it only bounds how many workgroups, and so how many bytes in flight,
// a compute unit holds at once.
constexpr size_t kLdsPerCuMax = 160 * 1024;  // gfx950; the running device's figure is read at first use
size_t lds_for_cap(int64_t cap, size_t lds_per_cu) {
  if (cap <= 0) return 0;
  if (cap > 32) cap = 32;
  return lds_per_cu / (size_t)cap - kCapSlackBytes;  // the slack is for the kernel's own static LDS
}

// Kernels launched with more than 64 KB of dynamic LDS need the attribute raised once per device.
template <typename K>
int allow_big_lds(K kernel, size_t lds_per_cu) {
  struct Done { const void* kernel; int device; };
  static thread_local Done done[512];
  static thread_local int n_done = 0;
  const void* key = (const void*)kernel;
  int device = 0;
  AM_HIP(hipGetDevice(&device));
  for (int i = 0; i < n_done; ++i)
    if (done[i].kernel == key && done[i].device == device) return ADAM_MINI_OK;
  AM_HIP(hipFuncSetAttribute(key, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(lds_per_cu - kCapSlackBytes)));
  if (n_done < 512) done[n_done++] = Done{key, device};
  return ADAM_MINI_OK;
}

// What every launch of one call shares.
struct AmCtx {
  const AmTuning& t;
  hipStream_t stream;
  size_t lds_per_cu;
  AmDeviceMem mem;
};

uint32_t grid_for(uint64_t groups, const AmTuning& t) {
  uint64_t g = groups;
  if (t.grid_cap > 0 && g > (uint64_t)t.grid_cap) g = (uint64_t)t.grid_cap;
  if (g > 0x7fffffffull) g = 0x7fffffffull;
  return (uint32_t)g;
}

#define AM_TAB tab.segs, tab.item_keys, tab.lblock_keys, tab.n_segs, tab.xcd_code

// Launch one kernel with an optional occupancy cap (see lds_for_cap).
template <typename K, typename... Args>
int launch_capped(K kernel, uint32_t grid, uint32_t block, int64_t cap, const AmCtx& cx, Args... args) {
  const size_t lds = lds_for_cap(cap, cx.lds_per_cu);
  if (lds > 0) {
    const int rc = allow_big_lds(kernel, cx.lds_per_cu);
    if (rc != ADAM_MINI_OK) return rc;
  }
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), lds, cx.stream, args...);
  return ADAM_MINI_OK;
}

// Resident-workgroup cap of a row bucket: explicit, or derived from the bytes a workgroup loads.
int64_t row_cap(const AmBucket& bk, int teams, size_t grad_bytes, const AmTuning& t) {
  if (t.row_wg_per_cu > 0) return t.row_wg_per_cu;
  if (t.row_inflight_kb <= 0) return 0;
  uint64_t units = 0;
  for (const AmSeg& s : bk.segs)
    if (s.units_per_block > units) units = s.units_per_block;
  const uint64_t wg_bytes = units * (uint64_t)bk.var.vec * (8 + grad_bytes) * (uint64_t)teams;
  if (wg_bytes <= 24 * 1024) return 0;  // small workgroups: the wave-slot limit of a CU is cap enough
  int64_t cap = (int64_t)(((uint64_t)t.row_inflight_kb * 1024 + wg_bytes - 1) / (wg_bytes ? wg_bytes : 1));
  if (cap < 2) cap = 2;
  return cap > 16 ? 0 : cap;  // beyond 16 the hardware's own limits bind first
}

template <typename G, int VEC>
int launch_row(const AmBucket& bk, const AmTable& tab, float* v, const AmScalarsArg& sc, const AmCtx& cx) {
  const AmVariant& var = bk.var;
  const uint32_t n_items = (uint32_t)bk.n_items;
#define X(L, U)                                                                                       \
  if constexpr (am_row_ok(VEC, L, U)) {                                                               \
    if (var.lanes == L && var.upt == U) {                                                             \
      constexpr int WG = AmRowGeom<L>::WG, TEAMS = AmRowGeom<L>::TEAMS;                               \
      const uint32_t grid = grid_for((bk.n_items + TEAMS - 1) / TEAMS, cx.t);                         \
      return launch_capped(am_row_kernel<G, VEC, L, U>, grid, WG, row_cap(bk, TEAMS, sizeof(G), cx.t), cx, \
                           AM_TAB, n_items, (uint32_t)(cx.t.row_blocked != 0), v, sc);                \
    }                                                                                                 \
  }
  AM_ROW_VARIANTS(X)
#undef X
  return ADAM_MINI_INVALID_ARG;
}

template <int VEC>
int launch_row_ids(const AmBucket& bk, const AmTable& tab, uint32_t tensor, uint64_t* ids, const AmCtx& cx) {
  const AmVariant& var = bk.var;
  const uint32_t n_items = (uint32_t)bk.n_items;
#define X(L, U)                                                                                       \
  if (var.lanes == L && var.upt == U) {                                                               \
    constexpr int WG = AmRowGeom<L>::WG, TEAMS = AmRowGeom<L>::TEAMS;                                 \
    const uint32_t grid = grid_for((bk.n_items + TEAMS - 1) / TEAMS, cx.t);                           \
    hipLaunchKernelGGL((am_row_ids<VEC, L, U>), dim3(grid), dim3(WG), 0, cx.stream, AM_TAB, n_items,  \
                       (uint32_t)(cx.t.row_blocked != 0), tensor, ids);                               \
    return ADAM_MINI_OK;                                                                              \
  }
  AM_ROW_VARIANTS(X)
#undef X
  return ADAM_MINI_INVALID_ARG;
}

template <typename G, int VEC>
int launch_row_lds(const AmBucket& bk, const AmTable& tab, float* v, const AmScalarsArg& sc, const AmCtx& cx) {
  if constexpr (VEC == 1) {
    return ADAM_MINI_INVALID_ARG;  // the layout builder never stages scalar-unit blocks
  } else {
    const uint32_t n_items = (uint32_t)bk.n_items;
    const uint32_t grid = grid_for(bk.n_items, cx.t);
    const size_t lds = (size_t)((bk.lds_bytes + 15) & ~15ull);
    if (lds > cx.lds_per_cu - kCapSlackBytes) return ADAM_MINI_INVALID_ARG;
    const int rc = allow_big_lds(am_row_lds_kernel<G, VEC>, cx.lds_per_cu);
    if (rc != ADAM_MINI_OK) return rc;
    hipLaunchKernelGGL((am_row_lds_kernel<G, VEC>), dim3(grid), dim3(kLdsRowThreads), lds, cx.stream, AM_TAB,
                       n_items, v, sc);
    return ADAM_MINI_OK;
  }
}

template <int VEC>
int launch_row_lds_ids(const AmBucket& bk, const AmTable& tab, uint32_t tensor, uint64_t* ids, const AmCtx& cx) {
  const uint32_t n_items = (uint32_t)bk.n_items;
  const uint32_t grid = grid_for(bk.n_items, cx.t);
  hipLaunchKernelGGL((am_row_lds_ids<VEC>), dim3(grid), dim3(kLdsRowThreads), 0, cx.stream, AM_TAB, n_items, tensor,
                     ids);
  return ADAM_MINI_OK;
}

// Two units of a row per lane exist for bf16 gradients in 4-element units only.
template <typename G, int VEC, int CPL>
constexpr bool am_strided_ok() {
  return CPL == 1 || (sizeof(G) == 2 && VEC == 4);
}

// A table whose item keys are the bucket's second numbering (the column-block update pass's tiles).
AmTable second_numbering(const AmTable& tab, const uint32_t* keys_base, uint64_t n_segs_total, const AmBucket& bk) {
  AmTable t2 = tab;
  t2.item_keys = keys_base + 2 * n_segs_total + bk.table_offset;
  return t2;
}

template <typename G, int VEC, int CPL>
int launch_strided_cpl(const AmBucket& bk, const AmTable& tab, const AmTable& tab2, float* v, const AmScalarsArg& sc,
                       const AmCtx& cx) {
  if constexpr (!am_strided_ok<G, VEC, CPL>()) {
    return ADAM_MINI_INVALID_ARG;
  } else {
    const uint32_t n_items = (uint32_t)bk.n_items;
    const uint32_t n_cols = (uint32_t)bk.n_lblocks;
    const uint32_t rows = (uint32_t)bk.var.upt;
    const uint32_t grid = grid_for(bk.n_items, cx.t);
    const uint32_t fgrid = grid_for((bk.n_lblocks + 255) / 256, cx.t);
    hipLaunchKernelGGL((am_strided_partial<G, VEC, CPL>), dim3(grid), dim3(kStridedThreads), 0, cx.stream, AM_TAB,
                       n_items, rows, cx.mem.partials);
    hipLaunchKernelGGL(am_strided_finalize, dim3(fgrid), dim3(256), 0, cx.stream, AM_TAB, n_cols, rows,
                       (const float*)cx.mem.partials, v, cx.mem.scales, sc);
    const uint32_t n_items2 = (uint32_t)bk.n_items2;
    return launch_capped(am_strided_update<G, VEC>, grid_for(bk.n_items2, cx.t), kStridedThreads,
                         cx.t.strided_wg_per_cu, cx, tab2.segs, tab2.item_keys, tab2.lblock_keys, tab2.n_segs,
                         tab2.xcd_code, n_items2, (const float*)cx.mem.scales, sc);
  }
}

template <typename G, int VEC>
int launch_strided(const AmBucket& bk, const AmTable& tab, const AmTable& tab2, float* v, const AmScalarsArg& sc,
                   const AmCtx& cx) {
  if (bk.var.upt <= 0) return ADAM_MINI_INVALID_ARG;
  if (bk.var.aux == 2) return launch_strided_cpl<G, VEC, 2>(bk, tab, tab2, v, sc, cx);
  return launch_strided_cpl<G, VEC, 1>(bk, tab, tab2, v, sc, cx);
}

template <int VEC>
int launch_strided_ids(const AmBucket& bk, const AmTable& tab2, uint32_t tensor, uint64_t* ids, const AmCtx& cx) {
  const uint32_t n_items2 = (uint32_t)bk.n_items2;
  hipLaunchKernelGGL((am_strided_ids<VEC>), dim3(grid_for(bk.n_items2, cx.t)), dim3(kStridedThreads), 0, cx.stream,
                     tab2.segs, tab2.item_keys, tab2.lblock_keys, tab2.n_segs, tab2.xcd_code, n_items2, tensor, ids);
  return ADAM_MINI_OK;
}

template <typename G, int VEC>
int launch_large(const AmBucket& bk, const AmTable& tab, float* v, const AmScalarsArg& sc, const AmCtx& cx) {
  const AmVariant& var = bk.var;
  float* partials = cx.mem.partials;
  float* scales = cx.mem.scales;
  const uint32_t keep_g = cx.t.large_keep_g != 0;  // ordinary cached gradient loads instead of streaming ones
  // blocks of very many chunks: a workgroup instead of a wavefront sums each block's partials
  const bool wide = cx.t.large_wide_chunks > 0 && bk.max_chunks >= (uint64_t)cx.t.large_wide_chunks;
#define X(L, U)                                                                                           \
  if constexpr (VEC * U <= 64) { /* larger chunks are never chosen: they would not fit the registers */   \
    if (var.lanes == L && var.upt == U) {                                                                 \
      for (const AmSlice& sl : bk.slices) {                                                               \
        const uint32_t grid = grid_for(sl.n_items, cx.t);                                                 \
        const uint32_t fgrid = grid_for((sl.n_lblocks + 3) / 4, cx.t);                                    \
        const uint32_t pgrid = grid_for((sl.n_items + 3) / 4, cx.t);                                      \
        if (bk.alt_reducer)                                                                               \
          hipLaunchKernelGGL((am_large_partial<G, VEC, L, U, true>), dim3(pgrid), dim3(256), 0,           \
                             cx.stream, AM_TAB, sl.item_first, sl.n_items, keep_g, partials);             \
        else                                                                                              \
          hipLaunchKernelGGL((am_large_partial<G, VEC, L, U, false>), dim3(pgrid), dim3(256), 0,          \
                             cx.stream, AM_TAB, sl.item_first, sl.n_items, keep_g, partials);             \
        if (wide)                                                                                         \
          hipLaunchKernelGGL(am_large_finalize_wide, dim3(grid_for(sl.n_lblocks, cx.t)),                  \
                             dim3(kWideFinalizeThreads), 0, cx.stream, AM_TAB, sl.lblock_first,           \
                             sl.n_lblocks, (const float*)partials, v, scales, sc);                        \
        else                                                                                              \
          hipLaunchKernelGGL(am_large_finalize, dim3(fgrid), dim3(256), 0, cx.stream, AM_TAB,             \
                             sl.lblock_first, sl.n_lblocks, (const float*)partials, v, scales, sc);       \
        const int rc = launch_capped(am_large_update<G, VEC, L, U>, grid, L, cx.t.stream_wg_per_cu, cx,   \
                                     AM_TAB, sl.item_first, sl.n_items, keep_g, (const float*)scales, sc); \
        if (rc != ADAM_MINI_OK) return rc;                                                                \
      }                                                                                                   \
      return ADAM_MINI_OK;                                                                                \
    }                                                                                                     \
  }
  AM_LARGE_VARIANTS(X)
#undef X
  return ADAM_MINI_INVALID_ARG;
}

template <int VEC>
int launch_large_ids(const AmBucket& bk, const AmTable& tab, uint32_t tensor, uint64_t* ids, const AmCtx& cx) {
  const AmVariant& var = bk.var;
  const uint32_t n_items = (uint32_t)bk.n_items;
  const uint32_t grid = grid_for(bk.n_items, cx.t);
#define X(L, U)                                                                                      \
  if (var.lanes == L && var.upt == U) {                                                              \
    hipLaunchKernelGGL((am_large_ids<VEC, L, U>), dim3(grid), dim3(L), 0, cx.stream, AM_TAB, n_items, \
                       tensor, ids);                                                                 \
    return ADAM_MINI_OK;                                                                             \
  }
  AM_LARGE_VARIANTS(X)
#undef X
  return ADAM_MINI_INVALID_ARG;
}

template <typename G, int VEC>
int launch_elementwise(const AmBucket& bk, const AmTable& tab, float* v, const AmScalarsArg& sc, const AmCtx& cx) {
  const AmVariant& var = bk.var;
  const uint32_t n_items = (uint32_t)bk.n_items;
  const uint32_t grid = grid_for(bk.n_items, cx.t);
#define X(L, U)                                                                                       \
  if (var.lanes == L && var.upt == U)                                                                 \
    return launch_capped(am_elementwise<G, VEC, L, U>, grid, L, cx.t.ew_wg_per_cu, cx, AM_TAB,        \
                         n_items, v, sc);
  AM_EW_VARIANTS(X)
#undef X
  return ADAM_MINI_INVALID_ARG;
}

template <int VEC>
int launch_elementwise_ids(const AmBucket& bk, const AmTable& tab, uint32_t tensor, uint64_t* ids,
                           const AmCtx& cx) {
  const AmVariant& var = bk.var;
  const uint32_t n_items = (uint32_t)bk.n_items;
  const uint32_t grid = grid_for(bk.n_items, cx.t);
#define X(L, U)                                                                                          \
  if (var.lanes == L && var.upt == U) {                                                                  \
    hipLaunchKernelGGL((am_elementwise_ids<VEC, L, U>), dim3(grid), dim3(L), 0, cx.stream, AM_TAB,       \
                       n_items, tensor, ids);                                                            \
    return ADAM_MINI_OK;                                                                                 \
  }
  AM_EW_VARIANTS(X)
#undef X
  return ADAM_MINI_INVALID_ARG;
}

template <typename G, int VEC>
int launch_fused(const AmBucket& bk, const AmTable& tab, float* v, const AmScalarsArg& sc, const AmCtx& cx) {
  if constexpr (VEC != 4) {
    return ADAM_MINI_INVALID_ARG;  // the layout builder fuses lists of whole 4-element units only
  } else {
    const uint32_t n_items = (uint32_t)bk.n_items;
    hipLaunchKernelGGL((am_fused_kernel<G, VEC>), dim3(grid_for(bk.n_items, cx.t)), dim3(kFusedThreads), 0, cx.stream,
                       AM_TAB, n_items, v, sc);
    return ADAM_MINI_OK;
  }
}

template <int VEC>
int launch_fused_ids(const AmBucket& bk, const AmTable& tab, uint32_t tensor, uint64_t* ids, const AmCtx& cx) {
  if constexpr (VEC != 4) {
    return ADAM_MINI_INVALID_ARG;
  } else {
    const uint32_t n_items = (uint32_t)bk.n_items;
    hipLaunchKernelGGL((am_fused_ids<VEC>), dim3(grid_for(bk.n_items, cx.t)), dim3(kFusedThreads), 0, cx.stream,
                       AM_TAB, n_items, tensor, ids);
    return ADAM_MINI_OK;
  }
}

// Dispatch on (gradient type, vec) -> template arguments.
template <typename G_, int VEC_>
struct AmTag {
  using G = G_;
  static constexpr int VEC = VEC_;
};

template <typename F>
int dispatch_grad(int grad_dtype, int vec, F f) {
  if (grad_dtype == ADAM_MINI_GRAD_F32) {
    if (vec == 4) return f(AmTag<float, 4>{});
    if (vec == 1) return f(AmTag<float, 1>{});
  } else {
    if (vec == 4) return f(AmTag<am_bf16, 4>{});
    if (vec == 8) return f(AmTag<am_bf16, 8>{});
    if (vec == 1) return f(AmTag<am_bf16, 1>{});
  }
  return ADAM_MINI_INVALID_ARG;
}

template <typename F>
int dispatch_vec(int vec, F f) {
  if (vec == 4) return f(AmTag<void, 4>{});
  if (vec == 8) return f(AmTag<void, 8>{});
  if (vec == 1) return f(AmTag<void, 1>{});
  return ADAM_MINI_INVALID_ARG;
}

uint32_t floor_log2(int64_t x) {
  uint32_t r = 0;
  while ((int64_t(1) << (r + 1)) <= x) ++r;
  return r;
}

AmTable bucket_table(const adam_mini_layout* L, const AmDeviceMem& mem, const AmBucket& bk) {
  AmTable tab;
  tab.segs = mem.segs + bk.table_offset;
  tab.item_keys = mem.keys + bk.table_offset;
  tab.lblock_keys = mem.keys + L->host.n_segs + bk.table_offset;
  tab.n_segs = (uint32_t)bk.segs.size();
  const AmTuning& t = L->host.tuning;
  const int fam = bk.var.family;
  const int64_t chunk = (fam == AM_FAM_ROW || fam == AM_FAM_ROW_LDS) ? t.xcd_chunk
                        : fam == AM_FAM_STRIDED                      ? t.xcd_chunk_strided
                                                                     : t.xcd_chunk_stream;
  tab.xcd_code = 32;  // identity
  if (chunk > 0 && t.xcd_count > 1 && fam != AM_FAM_FUSED) tab.xcd_code = floor_log2(chunk) | (floor_log2(t.xcd_count) << 8);
  return tab;
}

int launch_bucket_step(const adam_mini_layout* L, const AmBucket& bk, float* v, const AmScalarsArg& sc,
                       const AmCtx& cx) {
  const AmTable tab = bucket_table(L, cx.mem, bk);
  return dispatch_grad(L->host.grad_dtype, bk.var.vec, [&](auto tag) {
    using T = decltype(tag);
    switch (bk.var.family) {
      case AM_FAM_ROW:
        return launch_row<typename T::G, T::VEC>(bk, tab, v, sc, cx);
      case AM_FAM_ROW_LDS:
        return launch_row_lds<typename T::G, T::VEC>(bk, tab, v, sc, cx);
      case AM_FAM_STRIDED:
        return launch_strided<typename T::G, T::VEC>(bk, tab, second_numbering(tab, cx.mem.keys, L->host.n_segs, bk), v,
                                                     sc, cx);
      case AM_FAM_LARGE:
        return launch_large<typename T::G, T::VEC>(bk, tab, v, sc, cx);
      case AM_FAM_ELEMENTWISE:
        return launch_elementwise<typename T::G, T::VEC>(bk, tab, v, sc, cx);
      case AM_FAM_FUSED:
        return launch_fused<typename T::G, T::VEC>(bk, tab, v, sc, cx);
      default:
        return (int)ADAM_MINI_INVALID_ARG;
    }
  });
}

int launch_bucket_ids(const adam_mini_layout* L, const AmBucket& bk, uint32_t tensor, uint64_t* ids,
                      const AmCtx& cx) {
  const AmTable tab = bucket_table(L, cx.mem, bk);
  return dispatch_vec(bk.var.vec, [&](auto tag) {
    constexpr int VEC = decltype(tag)::VEC;
    switch (bk.var.family) {
      case AM_FAM_ROW:
        return launch_row_ids<VEC>(bk, tab, tensor, ids, cx);
      case AM_FAM_ROW_LDS:
        return launch_row_lds_ids<VEC>(bk, tab, tensor, ids, cx);
      case AM_FAM_STRIDED:
        return launch_strided_ids<VEC>(bk, second_numbering(tab, cx.mem.keys, L->host.n_segs, bk), tensor, ids, cx);
      case AM_FAM_LARGE:
        return launch_large_ids<VEC>(bk, tab, tensor, ids, cx);
      case AM_FAM_ELEMENTWISE:
        return launch_elementwise_ids<VEC>(bk, tab, tensor, ids, cx);
      case AM_FAM_FUSED:
        return launch_fused_ids<VEC>(bk, tab, tensor, ids, cx);
      default:
        return (int)ADAM_MINI_INVALID_ARG;
    }
  });
}

// ---------------------------------------------------------------------------
// device tables
// ---------------------------------------------------------------------------
size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Byte layout of the work tables inside one allocation (or inside the static scratch).
struct AmTableBytes {
  size_t segs = 0, keys = 0, partials = 0, scales = 0, scalars = 0, total = 0;  // offsets, then the size
};

AmTableBytes table_bytes(const AmHostLayout& h) {
  AmTableBytes b;
  b.segs = 0;
  b.keys = round_up(h.n_segs * sizeof(AmSeg), 256);
  b.partials = b.keys + round_up(3 * h.n_segs * sizeof(uint32_t), 256);
  b.scales = b.partials + round_up(h.n_partials * sizeof(float), 256);
  b.scalars = b.scales + round_up(h.n_lblocks * sizeof(float), 256);
  b.total = b.scalars + 256;  // one AmScalars: the step's scalars when the hyper-parameters live on the device
  return b;
}

AmDeviceMem carve(unsigned char* base, const AmTableBytes& b) {
  AmDeviceMem m;
  m.segs = reinterpret_cast<AmSeg*>(base + b.segs);
  m.keys = reinterpret_cast<uint32_t*>(base + b.keys);
  m.partials = reinterpret_cast<float*>(base + b.partials);
  m.scales = reinterpret_cast<float*>(base + b.scales);
  m.scalars = reinterpret_cast<AmScalars*>(base + b.scalars);
  return m;
}

// Host image of the segment and key tables ([0, b.partials) of the byte layout) with the given pointer
// lists (null lists: pointers stay null, which is enough for the id kernels).
void table_image(const adam_mini_layout* L, const AmTableBytes& b, void* const* params, const void* const* grads,
                 void* const* exp_avg, std::vector<unsigned char>& img) {
  img.assign(b.partials, 0);  // no reallocation when the vector already has this size
  AmSeg* segs = reinterpret_cast<AmSeg*>(img.data() + b.segs);
  uint32_t* keys = reinterpret_cast<uint32_t*>(img.data() + b.keys);
  const size_t n = L->host.n_segs;
  for (const AmBucket& bk : L->host.buckets)
    for (size_t i = 0; i < bk.segs.size(); ++i) {
      AmSeg s = bk.segs[i];
      if (params) {
        s.p = (float*)params[s.tensor];
        s.g = grads[s.tensor];
        s.m = (float*)exp_avg[s.tensor];
      }
      segs[bk.table_offset + i] = s;
      keys[bk.table_offset + i] = s.item_first;
      keys[n + bk.table_offset + i] = s.lblock_first;
      keys[2 * n + bk.table_offset + i] = i < bk.item2_first.size() ? bk.item2_first[i] : 0u;
    }
}

void free_device_state(adam_mini_layout* L) {
  if (L->mem.segs) (void)hipFree(L->mem.segs);  // one allocation: the other pointers lie inside it
  L->mem = AmDeviceMem();
  L->device_ready = false;
  L->cache.valid = false;
}

// LDS of a compute unit, from the device (gfx950: 160 KB).
int query_device(adam_mini_layout* L) {
  int lds = 0;
  AM_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, L->device));
  if (lds >= 64 * 1024 && (size_t)lds <= kLdsPerCuMax) L->lds_per_cu = (size_t)lds;
  return ADAM_MINI_OK;
}

int allocate_device_state(adam_mini_layout* L) {
  const AmTableBytes b = table_bytes(L->host);
  unsigned char* base = nullptr;
  AM_HIP(hipMalloc((void**)&base, b.total));
  L->mem = carve(base, b);
  // the tables without data pointers; a step fills those in with am_write_pointers
  std::vector<unsigned char> img;
  table_image(L, b, nullptr, nullptr, nullptr, img);
  AM_HIP(hipMemcpy(base, img.data(), img.size(), hipMemcpyHostToDevice));
  const int rc = query_device(L);
  if (rc == ADAM_MINI_OK) L->lds_per_cu_known = true;
  return rc;
}

// Device tables and scratch, created by the first call that needs them.  On failure nothing is kept.
int ensure_device_state(adam_mini_layout* L) {
  if (L->device_ready) return ADAM_MINI_OK;
  int rc;
  try {
    rc = allocate_device_state(L);
  } catch (const std::bad_alloc&) {
    rc = ADAM_MINI_OUT_OF_MEMORY;
  }
  if (rc != ADAM_MINI_OK) {
    free_device_state(L);
    return rc;
  }
  L->device_ready = true;
  return ADAM_MINI_OK;
}

// New pointer lists for the layout's own segment table: sent as kernel arguments, kPointersPerLaunch
// segments per launch, in stream order before the step's kernels.  No copy, no wait.
int write_pointers(adam_mini_layout* L, void* const* params, const void* const* grads, void* const* exp_avg,
                   hipStream_t stream) {
  AmPointerBatch batch;
  uint32_t first = 0, n = 0;
  const uint32_t total = (uint32_t)L->host.n_segs;
  for (const AmBucket& bk : L->host.buckets)
    for (size_t i = 0; i < bk.segs.size(); ++i) {
      const uint32_t k = bk.segs[i].tensor;
      batch.t[n++] = AmPointerTriple{(float*)params[k], grads[k], (float*)exp_avg[k]};
      if (n == (uint32_t)kPointersPerLaunch || first + n == total) {
        hipLaunchKernelGGL(am_write_pointers, dim3(1), dim3(256), 0, stream, L->mem.segs, first, n, batch);
        first += n;
        n = 0;
      }
    }
  AM_HIP(hipGetLastError());
  return ADAM_MINI_OK;
}

// A byte image into device memory as kernel arguments, kWordsPerLaunch 16-byte words per launch.
int write_image(unsigned char* dst, const std::vector<unsigned char>& img, hipStream_t stream) {
  AmWords payload;
  const size_t words = img.size() / 16;  // images are padded to 256 bytes
  for (size_t w0 = 0; w0 < words; w0 += kWordsPerLaunch) {
    const size_t n = words - w0 < (size_t)kWordsPerLaunch ? words - w0 : (size_t)kWordsPerLaunch;
    std::memcpy(payload.w, img.data() + w0 * 16, n * 16);
    hipLaunchKernelGGL(am_write_words, dim3(1), dim3(256), 0, stream, reinterpret_cast<am_u32x4*>(dst) + w0,
                       (uint32_t)n, payload);
  }
  AM_HIP(hipGetLastError());
  return ADAM_MINI_OK;
}

bool finite_f(float x) { return std::isfinite(x); }

// Everything adam_mini_step checks before it touches a device.
int validate_step(const adam_mini_layout* layout, void* const* params, const void* const* grads,
                  void* const* exp_avg, const float* v_dev, const adam_mini_hparams* hp) {
  if (!layout || !params || !grads || !exp_avg || !v_dev || !hp) return ADAM_MINI_INVALID_ARG;
  if (hp->step == 0) return ADAM_MINI_INVALID_ARG;
  if (!finite_f(hp->lr) || !finite_f(hp->weight_decay) || !finite_f(hp->eps) || hp->eps < 0.0f)
    return ADAM_MINI_INVALID_ARG;
  if (!(hp->beta1 >= 0.0f && hp->beta1 < 1.0f) || !(hp->beta2 >= 0.0f && hp->beta2 < 1.0f))
    return ADAM_MINI_INVALID_ARG;
  const size_t n = layout->host.tensors.size();
  for (size_t k = 0; k < n; ++k)
    if (!params[k] || !grads[k] || !exp_avg[k]) return ADAM_MINI_INVALID_ARG;
  if (((uintptr_t)v_dev & 15u) != 0) return ADAM_MINI_MISALIGNED;
  for (size_t k = 0; k < n; ++k)
    if ((((uintptr_t)params[k] | (uintptr_t)grads[k] | (uintptr_t)exp_avg[k]) & 15u) != 0) return ADAM_MINI_MISALIGNED;
  if (layout->device < 0) return ADAM_MINI_NO_DEVICE;
  return ADAM_MINI_OK;
}

// Step scalars in double, rounded once.
AmScalars step_scalars(const adam_mini_hparams* hp) {
  const double b1 = hp->beta1, b2 = hp->beta2, t = (double)hp->step;
  const double bc1 = 1.0 - std::pow(b1, t), bc2 = 1.0 - std::pow(b2, t);
  AmScalars sc;
  sc.beta1 = hp->beta1;
  sc.omb1 = (float)(1.0 - b1);
  sc.beta2 = hp->beta2;
  sc.omb2 = (float)(1.0 - b2);
  sc.eps = hp->eps;
  sc.bc2 = (float)bc2;
  sc.step_size = (float)((double)hp->lr / bc1);
  sc.lr_wd = (float)((double)hp->lr * (double)hp->weight_decay);
  return sc;
}

// The launches of one step, with the tables and scratch of `mem`.
int launch_step(adam_mini_layout* layout, const AmDeviceMem& mem, float* v_dev, const AmScalarsArg& sc,
                hipStream_t stream) {
  const AmCtx cx{layout->host.tuning, stream, layout->lds_per_cu, mem};
  const size_t nb = layout->host.buckets.size();
  const bool timed = layout->profile_used < layout->profile_capacity;
  for (size_t b = 0; b < nb; ++b) {
    hipEvent_t* ev = timed ? &layout->events[((size_t)layout->profile_used * nb + b) * 2] : nullptr;
    if (ev) AM_HIP(hipEventRecord(ev[0], stream));
    const int rc = launch_bucket_step(layout, layout->host.buckets[b], v_dev, sc, cx);
    if (rc != ADAM_MINI_OK) return rc;
    if (ev) AM_HIP(hipEventRecord(ev[1], stream));
  }
  if (timed) layout->profile_used++;
  AM_HIP(hipGetLastError());
  return ADAM_MINI_OK;
}

// ---------------------------------------------------------------------------
// static scratch of adam_mini_step_static: one array per GPU, in the library's code object
// ---------------------------------------------------------------------------
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU (each holds its own copy)
uint64_t g_scratch_owner[kMaxDevices];       // uid of the layout whose tables the GPU's array holds (0: none)
uint64_t g_next_uid = 1;

// Device address of this GPU's copy of the array.  In host code the array's NAME is only a handle for
// this lookup, never an address a kernel could use.  The device must be current.
int scratch_address(int device, unsigned char** out) {
  if (device < 0 || device >= kMaxDevices) return ADAM_MINI_INVALID_ARG;
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    AM_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return ADAM_MINI_HIP_ERROR;
    g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return ADAM_MINI_OK;
}

}  // namespace

// ===========================================================================
// exported functions
// ===========================================================================
extern "C" {

int adam_mini_set_option(const char* key, int64_t value) {
  if (!key) return ADAM_MINI_INVALID_ARG;
  std::lock_guard<std::mutex> lock(g_tuning_mutex);
  const std::string k(key);
  if (k == "reset") { g_tuning = AmTuning(); return ADAM_MINI_OK; }
  if (value < 0) return ADAM_MINI_INVALID_ARG;
  if (k == "bf16_vec") { if (value != 4 && value != 8) return ADAM_MINI_INVALID_ARG; g_tuning.bf16_vec = value; }
  else if (k == "subwave_max_units") g_tuning.subwave_max_units = value;
  else if (k == "wave_max_units") g_tuning.wave_max_units = value;
  else if (k == "team_max_lanes") g_tuning.team_max_lanes = value;
  else if (k == "max_upt") g_tuning.max_upt = value;
  else if (k == "row_max_units") g_tuning.row_max_units = value;
  else if (k == "lds_max_bytes") {
    if (value > (int64_t)(kLdsPerCuMax - kCapSlackBytes)) return ADAM_MINI_INVALID_ARG;
    g_tuning.lds_max_bytes = value;
  }
  else if (k == "cu_count") g_tuning.cu_count = value;
  else if (k == "large_chunk_upt") g_tuning.large_chunk_upt = value;
  else if (k == "ew_upt") g_tuning.ew_upt = value;
  else if (k == "grid_cap") g_tuning.grid_cap = value;
  else if (k == "row_wg_per_cu") g_tuning.row_wg_per_cu = value;
  else if (k == "row_inflight_kb") g_tuning.row_inflight_kb = value;
  else if (k == "row_blocked") g_tuning.row_blocked = value;
  else if (k == "stream_wg_per_cu") g_tuning.stream_wg_per_cu = value;
  else if (k == "strided_wg_per_cu") g_tuning.strided_wg_per_cu = value;
  else if (k == "ew_wg_per_cu") g_tuning.ew_wg_per_cu = value;
  else if (k == "fuse_max_params") g_tuning.fuse_max_params = value;
  else if (k == "fuse_target_items") { if (value < 1) return ADAM_MINI_INVALID_ARG; g_tuning.fuse_target_items = value; }
  else if (k == "large_slice_mb") g_tuning.large_slice_mb = value;
  else if (k == "large_keep_g") g_tuning.large_keep_g = value;
  else if (k == "large_wide_chunks") g_tuning.large_wide_chunks = value;
  else if (k == "strided_rows") {
    if (value < 4 || value > 65536 || value % 4 != 0) return ADAM_MINI_INVALID_ARG;
    g_tuning.strided_rows = value;
  }
  else if (k == "xcd_count") {
    if (value < 1 || value > 64 || (value & (value - 1)) != 0) return ADAM_MINI_INVALID_ARG;
    g_tuning.xcd_count = value;
  }
  else if (k == "xcd_chunk" || k == "xcd_chunk_stream" || k == "xcd_chunk_strided") {
    if (value > (int64_t(1) << 20) || (value & (value - 1)) != 0) return ADAM_MINI_INVALID_ARG;
    (k == "xcd_chunk" ? g_tuning.xcd_chunk : k == "xcd_chunk_stream" ? g_tuning.xcd_chunk_stream
                                                                      : g_tuning.xcd_chunk_strided) = value;
  }
  else return ADAM_MINI_INVALID_ARG;
  return ADAM_MINI_OK;
}

int adam_mini_init_layout(const adam_mini_tensor_desc* descs, uint32_t n_tensors, int grad_dtype, int device,
                          adam_mini_layout** out) {
  if (!out) return ADAM_MINI_INVALID_ARG;
  *out = nullptr;
  if (!descs || n_tensors == 0 || device < -1) return ADAM_MINI_INVALID_ARG;
  adam_mini_layout* L = new (std::nothrow) adam_mini_layout();
  if (!L) return ADAM_MINI_OUT_OF_MEMORY;
  AmTuning tuning;
  {
    std::lock_guard<std::mutex> lock(g_tuning_mutex);
    tuning = g_tuning;
  }
  int rc;
  try {
    rc = am_build_layout(descs, n_tensors, grad_dtype, tuning, &L->host);
    if (rc == ADAM_MINI_OK) {
      for (AmPointerCache* c : {&L->cache, &L->static_cache}) {
        c->p.assign(n_tensors, nullptr);
        c->g.assign(n_tensors, nullptr);
        c->m.assign(n_tensors, nullptr);
      }
      const AmTableBytes b = table_bytes(L->host);
      if (b.total <= (size_t)ADAM_MINI_STATIC_SCRATCH_BYTES) L->static_image.assign(b.partials, 0);
    }
  } catch (const std::bad_alloc&) {
    rc = ADAM_MINI_OUT_OF_MEMORY;
  }
  if (rc != ADAM_MINI_OK) {
    delete L;
    return rc;
  }
  L->device = device;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    L->uid = g_next_uid++;
  }
  *out = L;
  return ADAM_MINI_OK;
}

uint64_t adam_mini_num_blocks(const adam_mini_layout* layout) { return layout ? layout->host.num_blocks : 0; }

uint32_t adam_mini_num_tensors(const adam_mini_layout* layout) {
  return layout ? (uint32_t)layout->host.tensors.size() : 0;
}

int adam_mini_export_layout(const adam_mini_layout* layout, uint64_t* v_offset, uint32_t* path_kind) {
  if (!layout) return ADAM_MINI_INVALID_ARG;
  const auto& ts = layout->host.tensors;
  if (v_offset) {
    for (size_t k = 0; k < ts.size(); ++k) v_offset[k] = ts[k].v_first;
    v_offset[ts.size()] = layout->host.num_blocks;
  }
  if (path_kind) {
    for (size_t k = 0; k < ts.size(); ++k) path_kind[k] = (uint32_t)am_path_kind(layout->host.buckets[ts[k].bucket].var);
  }
  return ADAM_MINI_OK;
}

int adam_mini_block_id(const adam_mini_layout* layout, uint32_t tensor, uint64_t elem, uint64_t* out) {
  if (!layout || !out || tensor >= layout->host.tensors.size()) return ADAM_MINI_INVALID_ARG;
  const AmTensorInfo& ti = layout->host.tensors[tensor];
  if (elem >= ti.numel) return ADAM_MINI_INVALID_ARG;
  *out = ti.strided ? ti.v_first + elem % ti.n_blocks : ti.v_first + elem / ti.block_numel;
  return ADAM_MINI_OK;
}

int adam_mini_write_block_ids(adam_mini_layout* layout, uint32_t tensor, uint64_t* ids_dev, void* hip_stream) {
  if (!layout || !ids_dev || tensor >= layout->host.tensors.size()) return ADAM_MINI_INVALID_ARG;
  if (layout->device < 0) return ADAM_MINI_NO_DEVICE;
  if (((uintptr_t)ids_dev & 7u) != 0) return ADAM_MINI_MISALIGNED;
  hipStream_t stream = (hipStream_t)hip_stream;
  DeviceGuard guard;
  int rc = guard.enter(layout->device);
  if (rc != ADAM_MINI_OK) return rc;
  rc = ensure_device_state(layout);
  if (rc != ADAM_MINI_OK) return rc;
  // the id kernels read the tables created above and no data pointer
  const AmBucket& bk = layout->host.buckets[layout->host.tensors[tensor].bucket];
  const AmCtx cx{layout->host.tuning, stream, layout->lds_per_cu, layout->mem};
  rc = launch_bucket_ids(layout, bk, tensor, ids_dev, cx);
  if (rc != ADAM_MINI_OK) return rc;
  AM_HIP(hipGetLastError());
  return ADAM_MINI_OK;
}

int adam_mini_step(adam_mini_layout* layout, void* const* params, const void* const* grads, void* const* exp_avg,
                   float* v_dev, const adam_mini_hparams* hp, void* hip_stream) {
  int rc = validate_step(layout, params, grads, exp_avg, v_dev, hp);
  if (rc != ADAM_MINI_OK) return rc;
  hipStream_t stream = (hipStream_t)hip_stream;
  DeviceGuard guard;
  rc = guard.enter(layout->device);
  if (rc != ADAM_MINI_OK) return rc;
  rc = ensure_device_state(layout);
  if (rc != ADAM_MINI_OK) return rc;
  const size_t n = layout->host.tensors.size();
  if (!layout->cache.same(params, grads, exp_avg, n)) {
    layout->cache.valid = false;
    rc = write_pointers(layout, params, grads, exp_avg, stream);
    if (rc != ADAM_MINI_OK) return rc;
    layout->cache.keep(params, grads, exp_avg, n);
  }
  return launch_step(layout, layout->mem, v_dev, AmScalarsArg{step_scalars(hp), nullptr}, stream);
}

int adam_mini_step_device_hparams(adam_mini_layout* layout, void* const* params, const void* const* grads,
                                  void* const* exp_avg, float* v_dev, adam_mini_hparams* hp_dev, uint32_t flags,
                                  void* hip_stream) {
  // host-side checks as for adam_mini_step, with stand-in hyper-parameters: the real ones cannot be read here
  if (!hp_dev || (flags & ~(uint32_t)ADAM_MINI_STEP_ADVANCE) != 0) return ADAM_MINI_INVALID_ARG;
  if (((uintptr_t)hp_dev & 7u) != 0) return ADAM_MINI_MISALIGNED;
  const adam_mini_hparams stand_in{1e-3f, 0.9f, 0.95f, 1e-8f, 0.0f, 1};
  int rc = validate_step(layout, params, grads, exp_avg, v_dev, &stand_in);
  if (rc != ADAM_MINI_OK) return rc;
  hipStream_t stream = (hipStream_t)hip_stream;
  DeviceGuard guard;
  rc = guard.enter(layout->device);
  if (rc != ADAM_MINI_OK) return rc;
  rc = ensure_device_state(layout);
  if (rc != ADAM_MINI_OK) return rc;
  const size_t n = layout->host.tensors.size();
  if (!layout->cache.same(params, grads, exp_avg, n)) {
    layout->cache.valid = false;
    rc = write_pointers(layout, params, grads, exp_avg, stream);
    if (rc != ADAM_MINI_OK) return rc;
    layout->cache.keep(params, grads, exp_avg, n);
  }
  static_assert(sizeof(AmDeviceHparams) == sizeof(adam_mini_hparams), "device view of adam_mini_hparams");
  hipLaunchKernelGGL(am_prepare_scalars, dim3(1), dim3(64), 0, stream, reinterpret_cast<AmDeviceHparams*>(hp_dev),
                     (uint32_t)((flags & ADAM_MINI_STEP_ADVANCE) != 0), layout->mem.scalars);
  return launch_step(layout, layout->mem, v_dev, AmScalarsArg{AmScalars{}, layout->mem.scalars}, stream);
}

int adam_mini_step_static(adam_mini_layout* layout, void* const* params, const void* const* grads,
                          void* const* exp_avg, float* v_dev, const adam_mini_hparams* hp, void* hip_stream) {
  int rc = validate_step(layout, params, grads, exp_avg, v_dev, hp);
  if (rc != ADAM_MINI_OK) return rc;
  const AmTableBytes b = table_bytes(layout->host);
  if (b.total > (size_t)ADAM_MINI_STATIC_SCRATCH_BYTES) return ADAM_MINI_TOO_LARGE;
  if (layout->device >= kMaxDevices) return ADAM_MINI_INVALID_ARG;
  hipStream_t stream = (hipStream_t)hip_stream;
  DeviceGuard guard;
  rc = guard.enter(layout->device);
  if (rc != ADAM_MINI_OK) return rc;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  unsigned char* base = nullptr;
  rc = scratch_address(layout->device, &base);  // first call on this GPU: looks the array's device address up
  if (rc != ADAM_MINI_OK) return rc;
  if (layout->lds_per_cu_known == false) {
    rc = query_device(layout);
    if (rc != ADAM_MINI_OK) return rc;
    layout->lds_per_cu_known = true;
  }
  const AmDeviceMem mem = carve(base, b);
  const size_t n = layout->host.tensors.size();
  // The array is shared by every layout stepped this way on the GPU and keeps what the last call left:
  // unless that call was this layout's, with these pointers, the tables are written again (as kernel
  // arguments, in stream order).  Partial sums and step scales need no clearing: every one a step reads
  // was written earlier in the same step.
  if (g_scratch_owner[layout->device] != layout->uid || !layout->static_cache.same(params, grads, exp_avg, n)) {
    g_scratch_owner[layout->device] = 0;
    layout->static_cache.valid = false;
    table_image(layout, b, params, grads, exp_avg, layout->static_image);  // sized by adam_mini_init_layout
    rc = write_image(base, layout->static_image, stream);
    if (rc != ADAM_MINI_OK) return rc;
    layout->static_cache.keep(params, grads, exp_avg, n);
    g_scratch_owner[layout->device] = layout->uid;
  }
  return launch_step(layout, mem, v_dev, AmScalarsArg{step_scalars(hp), nullptr}, stream);
}

uint32_t adam_mini_num_buckets(const adam_mini_layout* layout) {
  return layout ? (uint32_t)layout->host.buckets.size() : 0;
}

int adam_mini_profile_enable(adam_mini_layout* layout, uint32_t max_steps) {
  if (!layout) return ADAM_MINI_INVALID_ARG;
  if (layout->device < 0) return ADAM_MINI_NO_DEVICE;
  if (max_steps > 4096) return ADAM_MINI_INVALID_ARG;
  DeviceGuard guard;
  int rc = guard.enter(layout->device);
  if (rc != ADAM_MINI_OK) return rc;
  for (hipEvent_t e : layout->events) (void)hipEventDestroy(e);
  layout->events.clear();
  layout->profile_capacity = 0;
  layout->profile_used = 0;
  const size_t nb = layout->host.buckets.size();
  layout->bucket_ms.assign(nb, 0.0);
  layout->bucket_launches.assign(nb, 0);
  if (max_steps == 0) return ADAM_MINI_OK;
  try {
    layout->events.reserve((size_t)max_steps * nb * 2);
  } catch (const std::bad_alloc&) {
    return ADAM_MINI_OUT_OF_MEMORY;
  }
  for (size_t i = 0; i < (size_t)max_steps * nb * 2; ++i) {
    hipEvent_t e;
    AM_HIP(hipEventCreate(&e));
    layout->events.push_back(e);
  }
  layout->profile_capacity = max_steps;
  return ADAM_MINI_OK;
}

int adam_mini_profile_read(adam_mini_layout* layout, adam_mini_bucket_info* out, uint32_t capacity) {
  if (!layout || (!out && capacity > 0)) return ADAM_MINI_INVALID_ARG;
  const size_t nb = layout->host.buckets.size();
  if (layout->profile_used > 0) {
    DeviceGuard guard;
    int rc = guard.enter(layout->device);
    if (rc != ADAM_MINI_OK) return rc;
    for (uint32_t s = 0; s < layout->profile_used; ++s) {
      for (size_t b = 0; b < nb; ++b) {
        hipEvent_t* ev = &layout->events[((size_t)s * nb + b) * 2];
        AM_HIP(hipEventSynchronize(ev[1]));
        float ms = 0.0f;
        AM_HIP(hipEventElapsedTime(&ms, ev[0], ev[1]));
        layout->bucket_ms[b] += (double)ms;
        layout->bucket_launches[b] += 1;
      }
    }
    layout->profile_used = 0;
  }
  const char* gname = layout->host.grad_dtype == ADAM_MINI_GRAD_BF16 ? "am_bf16" : "float";
  for (size_t b = 0; b < nb && b < capacity; ++b) {
    const AmBucket& bk = layout->host.buckets[b];
    adam_mini_bucket_info& o = out[b];
    std::memset(&o, 0, sizeof o);
    o.family = am_path_kind(bk.var);
    o.vec = bk.var.vec;
    o.lanes = bk.var.lanes;
    o.upt = bk.var.upt;
    o.n_tensors = (uint32_t)bk.segs.size();
    o.n_kernels = bk.var.family == AM_FAM_STRIDED ? 3u : 1u;
    if (bk.var.family == AM_FAM_LARGE) o.n_kernels = 3u * (uint32_t)bk.slices.size();
    o.n_items = bk.n_items;
    for (const AmSeg& s : bk.segs) {
      const AmTensorInfo& ti = layout->host.tensors[s.tensor];
      o.numel += ti.numel;
      o.n_blocks += ti.n_blocks;
    }
    if (b < layout->bucket_ms.size()) {
      o.total_ms = layout->bucket_ms[b];
      o.timed_launches = layout->bucket_launches[b];
    }
    const char* kname = bk.var.family == AM_FAM_ROW ? "am_row_kernel"
                        : bk.var.family == AM_FAM_LARGE ? "am_large_update"
                        : bk.var.family == AM_FAM_ROW_LDS ? "am_row_lds_kernel" : "am_elementwise";
    if (bk.var.family == AM_FAM_FUSED)
      std::snprintf(o.kernel, sizeof o.kernel, "am_fused_kernel<%s, %d>", gname, bk.var.vec);
    else if (bk.var.family == AM_FAM_STRIDED)
      std::snprintf(o.kernel, sizeof o.kernel, "am_strided_update<%s, %d> after am_strided_partial<%s, %d, %d>", gname,
                    bk.var.vec, gname, bk.var.vec, bk.var.aux);
    else if (bk.var.family == AM_FAM_ROW_LDS)
      std::snprintf(o.kernel, sizeof o.kernel, "%s<%s, %d>", kname, gname, bk.var.vec);
    else
      std::snprintf(o.kernel, sizeof o.kernel, "%s<%s, %d, %d, %d>", kname, gname, bk.var.vec, bk.var.lanes, bk.var.upt);
  }
  if (layout->profile_capacity > 0) {  // totals are "since the last read"
    layout->bucket_ms.assign(nb, 0.0);
    layout->bucket_launches.assign(nb, 0);
  }
  return ADAM_MINI_OK;
}

void adam_mini_destroy_layout(adam_mini_layout* layout) {
  if (!layout) return;
  if (layout->device_ready) {
    DeviceGuard guard;
    if (guard.enter(layout->device) == ADAM_MINI_OK) {
      free_device_state(layout);
    }
  }
  if (!layout->events.empty()) {
    DeviceGuard guard;
    if (guard.enter(layout->device) == ADAM_MINI_OK)
      for (hipEvent_t e : layout->events) (void)hipEventDestroy(e);
  }
  delete layout;
}

const char* adam_mini_strerror(int status) {
  switch (status) {
    case ADAM_MINI_OK: return "ok";
    case ADAM_MINI_INVALID_ARG: return "invalid argument";
    case ADAM_MINI_MISALIGNED: return "device pointer is not 16-byte aligned";
    case ADAM_MINI_OUT_OF_MEMORY: return "out of memory";
    case ADAM_MINI_HIP_ERROR: return "HIP runtime error";
    case ADAM_MINI_NO_DEVICE: return "layout was built without a device";
    case ADAM_MINI_TOO_LARGE: return "layout needs more work memory than the static scratch holds";
    default: return "unknown status";
  }
}

const char* adam_mini_last_hip_error(void) { return g_hip_error.c_str(); }

}  // extern "C"
