// gfx950 kernels of the Adam-mini step (Algorithm 1, Section 2.3 of the paper).
//
//   am_row_kernel        one block per team of LANES threads, whole block in registers:
//                        loads g, m, p once, reduces sum(g^2), updates v, m, p.  Teams of 16
//                        or 64 threads are packed several to a 256-thread workgroup.
//   am_row_lds_kernel    one block per 1024-thread workgroup, gradient staged in LDS (blocks too big
//                        for the registers of one workgroup, up to ~150 KB of gradient)
//   am_large_partial     blocks too big for one workgroup: per-chunk sum(g^2)
//   am_large_finalize    per block: fixed-order sum of its chunk partials, v update, step scale
//   am_large_update      per chunk: m and p update with the block's step scale
//   am_strided_*         blocks that are the columns of the stored matrix (weight kept transposed)
//   am_elementwise       block_numel == 1 (AdamW-equivalent): dense v, per-element sqrt / divide
//   am_*_ids             the same work-item -> element walks, writing v indices instead
//
// A lane works on units of VEC consecutive elements: VEC = 4 means one 128-bit load / store of m
// and p and one 128-bit (fp32) or 64-bit (bf16) gradient load per unit, consecutive lanes owning
// consecutive units; VEC = 8 (bf16 only, optional) is a 128-bit gradient load beside two 128-bit
// words of m and p; VEC = 1 is the scalar fallback for block sizes that are not whole units.
#ifndef AM_KERNELS_H_
#define AM_KERNELS_H_

#include "am_device.h"

// A bucket's tables as kernel parameters.  They are separate restrict-qualified pointers (not a
// struct) so the compiler knows they are read-only and keeps the table walk on scalar loads.
#define AM_TABLE_PARAMS                                                                       \
  const AmSeg* __restrict__ segs, const uint32_t* __restrict__ item_keys,                     \
      const uint32_t* __restrict__ lblock_keys, uint32_t n_segs
#define AM_TABLE_ARGS segs, item_keys, lblock_keys, n_segs
// What every work-item kernel takes: the tables and the XCD swizzle of its workgroup passes.
#define AM_KERNEL_PARAMS AM_TABLE_PARAMS, uint32_t xcd_code

// Workgroup pass -> group of work items.  The hardware deals consecutive workgroups round-robin to
// the XCDs (8 when the device is one partition), each with an L2 of its own, so with the identity
// map the dies interleave at the grain of single work items over the whole address range.  The
// swizzle hands each die runs of 2^shift consecutive groups instead: passes b, b+X, b+2X, ... (all
// on die b % X) walk one run, and the X runs of a span of X * 2^shift groups go to the X dies.  It is
// a bijection on [0, n_groups): whole spans are permuted, the ragged tail keeps the identity.
// `xcd_code` = shift | log2(X) << 8; shift >= 32 switches it off.  Only the order in which blocks are
// visited changes, never a block's arithmetic.
__device__ __forceinline__ uint32_t am_xcd_swizzle(uint32_t b, uint32_t n_groups, uint32_t xcd_code) {
  const uint32_t shift = xcd_code & 0xffu, dies_log2 = xcd_code >> 8;
  if (shift >= 32) return b;
  const uint32_t span_shift = shift + dies_log2;
  if (b >= (n_groups >> span_shift) << span_shift) return b;
  const uint32_t die = b & ((1u << dies_log2) - 1u), j = b >> dies_log2;
  return ((((j >> shift) << dies_log2) + die) << shift) + (j & ((1u << shift) - 1u));
}

// Resident-workgroup caps are set by reserving dynamic LDS that the kernels never touch: cap
// workgroups fit a compute unit when each reserves (LDS per CU) / cap - kCapSlackBytes.  The slack
// is what a capped kernel may declare as static LDS of its own.
constexpr int kCapSlackBytes = 1024;

// ===========================================================================
// table writers: small host tables travel to the device as kernel ARGUMENTS, so an update of the
// work tables is an ordinary launch on the step's stream: no staging buffer, no copy, no wait.
// ===========================================================================
constexpr int kWordsPerLaunch = 224;  // 16-byte words per am_write_words launch (3584 of the 4096 argument bytes)
struct AmWords {
  am_u32x4 w[kWordsPerLaunch];
};
__global__ __launch_bounds__(256) void am_write_words(am_u32x4* __restrict__ dst, uint32_t n, AmWords payload) {
  if (threadIdx.x < n) dst[threadIdx.x] = payload.w[threadIdx.x];
}

constexpr int kPointersPerLaunch = 144;  // segments per am_write_pointers launch (24 bytes each)
struct AmPointerTriple {
  float* p;
  const void* g;
  float* m;
};
struct AmPointerBatch {
  AmPointerTriple t[kPointersPerLaunch];
};
// Fills in the data pointers of segments [first, first + n) of the concatenated segment table.
__global__ __launch_bounds__(256) void am_write_pointers(AmSeg* __restrict__ segs, uint32_t first, uint32_t n,
                                                         AmPointerBatch batch) {
  if (threadIdx.x < n) {
    AmSeg* s = segs + first + threadIdx.x;
    s->p = batch.t[threadIdx.x].p;
    s->g = batch.t[threadIdx.x].g;
    s->m = batch.t[threadIdx.x].m;
  }
}

// ===========================================================================
// hyper-parameters that live on the device: one thread turns them into the step's scalars, in double
// like the host does for an ordinary step, optionally advancing the step counter first (so that a
// captured graph of  prepare + step  replays as the NEXT step each time).  Layout of `hp`: the public
// adam_mini_hparams { float lr, beta1, beta2, eps, weight_decay; uint64_t step; }.
// ===========================================================================
struct AmDeviceHparams {
  float lr, beta1, beta2, eps, weight_decay;
  unsigned long long step;
};

__global__ __launch_bounds__(64) void am_prepare_scalars(AmDeviceHparams* __restrict__ hp, uint32_t advance,
                                                         AmScalars* __restrict__ out) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  unsigned long long t = hp->step;
  if (advance) {
    t += 1;
    hp->step = t;
  }
  const double b1 = hp->beta1, b2 = hp->beta2;
  const double bc1 = 1.0 - pow(b1, (double)t), bc2 = 1.0 - pow(b2, (double)t);
  AmScalars sc;
  sc.beta1 = hp->beta1;
  sc.omb1 = (float)(1.0 - b1);
  sc.beta2 = hp->beta2;
  sc.omb2 = (float)(1.0 - b2);
  sc.eps = hp->eps;
  sc.bc2 = (float)bc2;
  sc.step_size = (float)((double)hp->lr / bc1);
  sc.lr_wd = (float)((double)hp->lr * (double)hp->weight_decay);
  *out = sc;
}

// ===========================================================================
// ROW family
// ===========================================================================
template <int LANES>
struct AmRowGeom {
  static constexpr int WG = LANES < 256 ? 256 : LANES;  // threads per workgroup
  static constexpr int TEAMS = WG / LANES;              // blocks per workgroup pass
  static constexpr int WAVES = LANES / 64;              // wavefronts per team (0 for 16-lane teams)
};

// What a team needs to know about its work item.
struct AmRowItem {
  const AmSeg* seg;
  uint32_t block;  // block index inside the tensor
  uint64_t elem0;  // first element of the block inside the tensor
  bool active;
};

template <int LANES>
__device__ __forceinline__ AmRowItem am_row_decode(AM_TABLE_PARAMS, uint32_t n_items, uint32_t first_item) {
  const uint32_t team = threadIdx.x / LANES;
  uint32_t item = first_item + team;
  AmRowItem it;
  it.active = item < n_items;
  if (!it.active) item = n_items - 1;  // keep the lookup in range; loads and stores are masked
  uint32_t s;
  if constexpr (LANES >= 64) {
    // a team of whole wavefronts shares its item: keep the table walk on the scalar unit
    item = __builtin_amdgcn_readfirstlane(item);
    s = am_find_seg(item_keys, n_segs, item);
  } else {
    // several teams per wavefront: walk the table once for the workgroup's first item (scalar);
    // only teams that fall past that tensor's last item repeat the walk with their own item
    const uint32_t lead = first_item < n_items ? first_item : n_items - 1;
    s = am_find_seg(item_keys, n_segs, lead);
    const uint32_t next_key = s + 1 < n_segs ? item_keys[s + 1] : 0xffffffffu;
    if (item >= next_key) s = am_find_seg(item_keys, n_segs, item);
  }
  it.seg = segs + s;
  it.block = item - item_keys[s];
  it.elem0 = (uint64_t)it.block * it.seg->block_numel;
  return it;
}

// Unit index handled by a team lane at unroll step k.  Strided: step k of the whole team covers one
// contiguous run of LANES units.  Blocked: each wavefront owns UPT*64 consecutive units, step k
// covering 64 of them, so a wavefront's accesses stay inside one contiguous span of the block.
template <int LANES, int UPT>
__device__ __forceinline__ uint64_t am_row_unit(int k, uint32_t blocked) {
  const uint32_t lane = threadIdx.x % LANES;
  if (LANES >= 64 && blocked) return (uint64_t)((lane >> 6) * UPT + k) * 64 + (lane & 63);
  return (uint64_t)lane + (uint64_t)k * LANES;
}

template <typename G, int VEC, int LANES, int UPT>
__global__ __launch_bounds__(AmRowGeom<LANES>::WG) void am_row_kernel(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                      uint32_t blocked, float* __restrict__ v,
                                                                      AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  using Geom = AmRowGeom<LANES>;
  // slot [parity][w] = sum of wavefront w; slot [parity][WAVES] = the block's old v
  __shared__ float xch[2][(Geom::WAVES > 1 ? Geom::WAVES : 1) + 1];
  static_assert(sizeof(xch) <= kCapSlackBytes, "static LDS must fit the slack the occupancy cap leaves");
  uint32_t parity = 0;
  const uint32_t n_groups = (n_items + Geom::TEAMS - 1) / Geom::TEAMS;
  for (uint32_t grp = blockIdx.x; grp < n_groups; grp += gridDim.x, parity ^= 1u) {
    const uint32_t first = am_xcd_swizzle(grp, n_groups, xcd_code) * Geom::TEAMS;
    const AmRowItem it = am_row_decode<LANES>(AM_TABLE_ARGS, n_items, first);
    const AmSeg& S = *it.seg;
    const uint64_t units = S.units_per_block;
    const uint64_t v_idx = S.v_first + it.block;

    float gv[UPT][VEC], mv[UPT][VEC], pv[UPT][VEC];
    float v_old = 0.0f;
    if constexpr (Geom::WAVES <= 1) {
      // team within one wavefront: every lane reads the same scalar (one broadcast request)
      if (it.active) v_old = v[v_idx];
    } else {
      // several wavefronts: only thread 0 touches v, so its later store cannot race a read
      if (threadIdx.x == 0) v_old = v[v_idx];
    }
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_row_unit<LANES, UPT>(k, blocked);
      if (it.active && u < units) {
        const uint64_t e = it.elem0 + u * VEC;
        am_load_grad<G, VEC>(S.g, e, gv[k]);
        am_load_f32<VEC>(S.m, e, mv[k]);
        am_load_f32<VEC>(S.p, e, pv[k]);
      } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) gv[k][j] = 0.0f;
      }
    }
    // block statistic: per lane in unit order, then the fixed reduction tree
    const uint32_t red = S.reducer;
    float ss = 0.0f;
    if (am_red_is_sum_sq(red)) {
      // Algorithm 1's sum of squares (absent units were loaded as zeros)
#pragma unroll
      for (int k = 0; k < UPT; ++k)
#pragma unroll
        for (int j = 0; j < VEC; ++j) ss = fmaf(gv[k][j], gv[k][j], ss);
    } else {
      ss = am_red_identity(red);
#pragma unroll
      for (int k = 0; k < UPT; ++k)
        if (it.active && am_row_unit<LANES, UPT>(k, blocked) < units) {
          ss = am_red_accumulate(red, gv[k], ss);
        }
    }

    if constexpr (LANES == 16) {
      ss = am_row16_reduce(red, ss);  // teams of one wavefront may differ in their reducer
    } else {
      // whole wavefronts share the block, so the choice is uniform
      ss = am_red_is_sum_sq(red) ? am_wave_sum(ss) : am_wave_reduce(red, ss);
      if constexpr (Geom::WAVES > 1) {
        float* slot = xch[parity];
        if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = ss;
        if (threadIdx.x == 0) slot[Geom::WAVES] = v_old;
        __syncthreads();
        ss = slot[0];
        if (am_red_is_sum_sq(red)) {
#pragma unroll
          for (int w = 1; w < Geom::WAVES; ++w) ss += slot[w];
        } else {
#pragma unroll
          for (int w = 1; w < Geom::WAVES; ++w) ss = am_combine(red, ss, slot[w]);
        }
        v_old = slot[Geom::WAVES];
      }
    }

    float v_new, scale;
    am_block_scalars(am_red_finish(red, ss, (float)S.block_numel), v_old, sc, &v_new, &scale);
    const float decay = sc.lr_wd * S.wd_scale;
    if (it.active && (threadIdx.x % LANES) == 0) v[v_idx] = v_new;

#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_row_unit<LANES, UPT>(k, blocked);
      if (it.active && u < units) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) am_update_elem(gv[k][j], mv[k][j], pv[k][j], scale, decay, sc);
        const uint64_t e = it.elem0 + u * VEC;
        am_store_f32<VEC>(S.m, e, mv[k]);
        am_store_f32<VEC>(S.p, e, pv[k]);
      }
    }
  }
}

// Same walk, writing the v index of every element of tensor `tensor`.
template <int VEC, int LANES, int UPT>
__global__ __launch_bounds__(AmRowGeom<LANES>::WG) void am_row_ids(AM_KERNEL_PARAMS,
                                                                   uint32_t n_items, uint32_t blocked,
                                                                   uint32_t tensor,
                                                                   uint64_t* __restrict__ ids) {
  using Geom = AmRowGeom<LANES>;
  const uint32_t n_groups = (n_items + Geom::TEAMS - 1) / Geom::TEAMS;
  for (uint32_t grp = blockIdx.x; grp < n_groups; grp += gridDim.x) {
    const uint32_t first = am_xcd_swizzle(grp, n_groups, xcd_code) * Geom::TEAMS;
    const AmRowItem it = am_row_decode<LANES>(AM_TABLE_ARGS, n_items, first);
    const AmSeg& S = *it.seg;
    if (!it.active || S.tensor != tensor) continue;
    const uint64_t v_idx = S.v_first + it.block;
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_row_unit<LANES, UPT>(k, blocked);
      if (u < S.units_per_block) {
        const uint64_t e = it.elem0 + u * VEC;
#pragma unroll
        for (int j = 0; j < VEC; ++j) ids[e + j] = v_idx;
      }
    }
  }
}

// ===========================================================================
// FUSED family: the whole tensor list of a SMALL layout in one launch.  A step of a small model is
// bound by the number of launches, not by bandwidth, so instead of one launch per kernel variant
// every tensor goes through this one generic kernel: 1024-thread workgroups, each working on one
// item of one tensor.
//   row items   a group of up to 1024 / T whole blocks, each held in the registers of a team of T lanes
//               (T = 16, 64, 256 or 1024: the smallest that holds the block at kFusedUpt units per lane),
//               exactly the single-pass scheme of am_row_kernel
//   tile items  1024 * kFusedUpt units of a tensor whose blocks have one element (AdamW-equivalent)
// T and the number of blocks per item are properties of the tensor (AmSeg::team_lanes, 0 marks a tile
// tensor; AmSeg::blocks_per_item), so they are uniform over a workgroup and the barrier below is too.  The host picks the blocks per item so that a small list makes no more items than the
// chip has compute units: a launch whose workgroups are all resident at once costs little more than an
// empty one (about 6 us back to back), a second round of workgroups nearly doubles it; teams beyond the
// item's blocks simply idle.
// ===========================================================================

template <typename G, int VEC>
__global__ __launch_bounds__(kFusedThreads) void am_fused_kernel(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                 float* __restrict__ v, AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  constexpr int WAVES = kFusedThreads / 64;
  __shared__ float xch[WAVES];     // wavefront results
  __shared__ float xch_v[WAVES];   // a team's old v, left by the team's first wavefront
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    // a later item of a grid-stride pass reuses the exchange slots: everyone must be done reading them
    // (items differ in whether they use the slots at all, so alternating two sets would not be enough)
    if (grp != blockIdx.x) __syncthreads();
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const uint32_t s = am_find_seg(item_keys, n_segs, item);
    const AmSeg& S = segs[s];
    const uint32_t local = item - item_keys[s];
    const uint32_t T = S.team_lanes, per_item = S.blocks_per_item;
    const float decay = sc.lr_wd * S.wd_scale;
    float gv[kFusedUpt][VEC], mv[kFusedUpt][VEC], pv[kFusedUpt][VEC];

    if (T == 0) {
      // tile of a one-element-block tensor: dense v, every statistic of the 1-vector g*g is g*g
      float* __restrict__ vt = v + S.v_first;
      float vv[kFusedUpt][VEC];
      const uint64_t unit0 = (uint64_t)local * (kFusedThreads * kFusedUpt);
#pragma unroll
      for (int k = 0; k < kFusedUpt; ++k) {
        const uint64_t u = unit0 + threadIdx.x + (uint64_t)k * kFusedThreads;
        if (u < S.units_per_block) {
          const uint64_t e = u * VEC;
          am_load_grad<G, VEC>(S.g, e, gv[k]);
          am_load_f32<VEC>(S.m, e, mv[k]);
          am_load_f32<VEC>(S.p, e, pv[k]);
          am_load_f32<VEC>(vt, e, vv[k]);
        }
      }
#pragma unroll
      for (int k = 0; k < kFusedUpt; ++k) {
        const uint64_t u = unit0 + threadIdx.x + (uint64_t)k * kFusedThreads;
        if (u < S.units_per_block) {
#pragma unroll
          for (int j = 0; j < VEC; ++j) {
            float v_new, scale;
            am_block_scalars(gv[k][j] * gv[k][j], vv[k][j], sc, &v_new, &scale);
            vv[k][j] = v_new;
            am_update_elem(gv[k][j], mv[k][j], pv[k][j], scale, decay, sc);
          }
          const uint64_t e = u * VEC;
          am_store_f32<VEC>(S.m, e, mv[k]);
          am_store_f32<VEC>(S.p, e, pv[k]);
          am_store_f32<VEC>(vt, e, vv[k]);
        }
      }
      continue;   // uniform over the workgroup: T belongs to the item
    }

    // row item: team `threadIdx.x / T` takes block local * per_item + team, if the item has that many
    const uint32_t team = threadIdx.x / T, lane = threadIdx.x % T;
    const uint64_t block = (uint64_t)local * per_item + team;
    const bool active = team < per_item && block < S.n_blocks;
    const uint64_t units = S.units_per_block;
    const uint64_t elem0 = block * S.block_numel;
    const uint64_t v_idx = S.v_first + block;
    float v_old = 0.0f;
    if (T <= 64) {
      // a team inside one wavefront: every lane reads the same scalar (one broadcast request); the store
      // below comes later in the same wavefront's program order
      if (active) v_old = v[v_idx];
    } else if (active && lane == 0) {
      v_old = v[v_idx];   // one lane per team touches v: its later store cannot race a read
    }
#pragma unroll
    for (int k = 0; k < kFusedUpt; ++k) {
      const uint64_t u = lane + (uint64_t)k * T;
      if (active && u < units) {
        const uint64_t e = elem0 + u * VEC;
        am_load_grad<G, VEC>(S.g, e, gv[k]);
        am_load_f32<VEC>(S.m, e, mv[k]);
        am_load_f32<VEC>(S.p, e, pv[k]);
      } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) gv[k][j] = 0.0f;
      }
    }
    const uint32_t red = S.reducer;
    float ss;
    if (am_red_is_sum_sq(red)) {
      ss = 0.0f;
#pragma unroll
      for (int k = 0; k < kFusedUpt; ++k)
#pragma unroll
        for (int j = 0; j < VEC; ++j) ss = fmaf(gv[k][j], gv[k][j], ss);
      ss = T == 16 ? am_row16_sum(ss) : am_wave_sum(ss);
    } else {
      ss = am_red_identity(red);
#pragma unroll
      for (int k = 0; k < kFusedUpt; ++k)
        if (active && lane + (uint64_t)k * T < units) ss = am_red_accumulate(red, gv[k], ss);
      ss = T == 16 ? am_row16_reduce(red, ss) : am_wave_reduce(red, ss);
    }
    // T > 64: a team is TW whole wavefronts; the first lane of the team's first wavefront holds v_old
    const uint32_t wave = threadIdx.x >> 6, TW = T >> 6, wave0 = team * TW;
    if (TW > 1) {
      float* slot = xch;
      float* slot_v = xch_v;
      if ((threadIdx.x & 63) == 0) slot[wave] = ss;
      if (lane == 0) slot_v[wave] = v_old;
      __syncthreads();
      ss = slot[wave0];
      if (am_red_is_sum_sq(red)) {
        for (uint32_t w = 1; w < TW; ++w) ss += slot[wave0 + w];
      } else {
        for (uint32_t w = 1; w < TW; ++w) ss = am_combine(red, ss, slot[wave0 + w]);
      }
      v_old = slot_v[wave0];
    }
    float v_new, scale;
    am_block_scalars(am_red_finish(red, ss, (float)S.block_numel), v_old, sc, &v_new, &scale);
    if (active && lane == 0) v[v_idx] = v_new;
#pragma unroll
    for (int k = 0; k < kFusedUpt; ++k) {
      const uint64_t u = lane + (uint64_t)k * T;
      if (active && u < units) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) am_update_elem(gv[k][j], mv[k][j], pv[k][j], scale, decay, sc);
        const uint64_t e = elem0 + u * VEC;
        am_store_f32<VEC>(S.m, e, mv[k]);
        am_store_f32<VEC>(S.p, e, pv[k]);
      }
    }
  }
}

// Same walk, writing the v index of every element of tensor `tensor`.
template <int VEC>
__global__ __launch_bounds__(kFusedThreads) void am_fused_ids(AM_KERNEL_PARAMS, uint32_t n_items, uint32_t tensor,
                                                              uint64_t* __restrict__ ids) {
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const uint32_t s = am_find_seg(item_keys, n_segs, item);
    const AmSeg& S = segs[s];
    if (S.tensor != tensor) continue;
    const uint32_t local = item - item_keys[s];
    const uint32_t T = S.team_lanes, per_item = S.blocks_per_item;
    if (T == 0) {
      const uint64_t unit0 = (uint64_t)local * (kFusedThreads * kFusedUpt);
#pragma unroll
      for (int k = 0; k < kFusedUpt; ++k) {
        const uint64_t u = unit0 + threadIdx.x + (uint64_t)k * kFusedThreads;
        if (u < S.units_per_block)
#pragma unroll
          for (int j = 0; j < VEC; ++j) ids[u * VEC + j] = S.v_first + u * VEC + j;
      }
      continue;
    }
    const uint32_t team = threadIdx.x / T, lane = threadIdx.x % T;
    const uint64_t block = (uint64_t)local * per_item + team;
    if (team >= per_item || block >= S.n_blocks) continue;
#pragma unroll
    for (int k = 0; k < kFusedUpt; ++k) {
      const uint64_t u = lane + (uint64_t)k * T;
      if (u < S.units_per_block)
#pragma unroll
        for (int j = 0; j < VEC; ++j) ids[block * S.block_numel + u * VEC + j] = S.v_first + block;
    }
  }
}

// ===========================================================================
// ROW_LDS family: one block per 1024-thread workgroup, too big for the registers of the team
// but small enough that its gradient fits the compute unit's 160 KB of LDS.  Pass 1 streams g
// from HBM into LDS (as it sits in memory) while summing squares; pass 2 streams m and p,
// taking g back from LDS.  g is read from HBM once, as in the register kernel.
// ===========================================================================
constexpr int kLdsRowThreads = 1024;
constexpr int kLdsRowUnroll = 4;  // independent loads in flight per thread in either pass

// unit handled by a thread at (outer step i, unroll slot j)
__device__ __forceinline__ uint64_t am_lds_unit(uint64_t i, int j) {
  return (i * kLdsRowUnroll + j) * kLdsRowThreads + threadIdx.x;
}

template <typename G, int VEC>
__global__ __launch_bounds__(kLdsRowThreads) void am_row_lds_kernel(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                    float* __restrict__ v, AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  using Raw = typename AmRaw<G, VEC>::T;
  extern __shared__ __attribute__((aligned(16))) unsigned char am_stage_bytes[];
  Raw* stage = reinterpret_cast<Raw*>(am_stage_bytes);
  __shared__ float xch[2][kLdsRowThreads / 64 + 1];
  uint32_t parity = 0;
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x, parity ^= 1u) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const AmRowItem it = am_row_decode<kLdsRowThreads>(AM_TABLE_ARGS, n_items, item);
    const AmSeg& S = *it.seg;
    const uint64_t units = S.units_per_block;
    const uint64_t steps = (units + kLdsRowThreads * kLdsRowUnroll - 1) / (kLdsRowThreads * kLdsRowUnroll);
    const uint64_t v_idx = S.v_first + it.block;
    float v_old = 0.0f;
    if (threadIdx.x == 0) v_old = v[v_idx];

    // pass 1: HBM -> registers -> LDS, block statistic on the way
    const uint32_t red = S.reducer;
    float ss = am_red_identity(red);
    for (uint64_t i = 0; i < steps; ++i) {
      Raw r[kLdsRowUnroll];
#pragma unroll
      for (int j = 0; j < kLdsRowUnroll; ++j) {
        const uint64_t u = am_lds_unit(i, j);
        if (u < units) r[j] = am_load_grad_raw<G, VEC>(S.g, it.elem0 + u * VEC);
      }
#pragma unroll
      for (int j = 0; j < kLdsRowUnroll; ++j) {
        const uint64_t u = am_lds_unit(i, j);
        if (u < units) {
          stage[u] = r[j];
          float gv[VEC];
          am_widen(r[j], gv);
          if (am_red_is_sum_sq(red)) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) ss = fmaf(gv[e], gv[e], ss);
          } else {
            ss = am_red_accumulate(red, gv, ss);
          }
        }
      }
    }
    ss = am_red_is_sum_sq(red) ? am_wave_sum(ss) : am_wave_reduce(red, ss);
    float* slot = xch[parity];
    if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = ss;
    if (threadIdx.x == 0) slot[kLdsRowThreads / 64] = v_old;
    __syncthreads();  // also orders the LDS staging before pass 2 (each thread re-reads only its own units,
                      // but the barrier is needed for the sums anyway)
    ss = slot[0];
    if (am_red_is_sum_sq(red)) {
#pragma unroll
      for (int w = 1; w < kLdsRowThreads / 64; ++w) ss += slot[w];
    } else {
#pragma unroll
      for (int w = 1; w < kLdsRowThreads / 64; ++w) ss = am_combine(red, ss, slot[w]);
    }
    v_old = slot[kLdsRowThreads / 64];

    float v_new, scale;
    am_block_scalars(am_red_finish(red, ss, (float)S.block_numel), v_old, sc, &v_new, &scale);
    const float decay = sc.lr_wd * S.wd_scale;
    if (threadIdx.x == 0) v[v_idx] = v_new;

    // pass 2: m and p from HBM, g from LDS
    for (uint64_t i = 0; i < steps; ++i) {
      float mv[kLdsRowUnroll][VEC], pv[kLdsRowUnroll][VEC];
#pragma unroll
      for (int j = 0; j < kLdsRowUnroll; ++j) {
        const uint64_t u = am_lds_unit(i, j);
        if (u < units) {
          const uint64_t e = it.elem0 + u * VEC;
          am_load_f32<VEC>(S.m, e, mv[j]);
          am_load_f32<VEC>(S.p, e, pv[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < kLdsRowUnroll; ++j) {
        const uint64_t u = am_lds_unit(i, j);
        if (u < units) {
          float gv[VEC];
          am_widen(stage[u], gv);
#pragma unroll
          for (int e = 0; e < VEC; ++e) am_update_elem(gv[e], mv[j][e], pv[j][e], scale, decay, sc);
          const uint64_t e0 = it.elem0 + u * VEC;
          am_store_f32<VEC>(S.m, e0, mv[j]);
          am_store_f32<VEC>(S.p, e0, pv[j]);
        }
      }
    }
    __syncthreads();  // the next item of a grid-stride pass overwrites the stage
  }
}

template <int VEC>
__global__ __launch_bounds__(kLdsRowThreads) void am_row_lds_ids(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                 uint32_t tensor, uint64_t* __restrict__ ids) {
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const AmRowItem it = am_row_decode<kLdsRowThreads>(AM_TABLE_ARGS, n_items, item);
    const AmSeg& S = *it.seg;
    if (S.tensor != tensor) continue;
    const uint64_t units = S.units_per_block;
    const uint64_t steps = (units + kLdsRowThreads * kLdsRowUnroll - 1) / (kLdsRowThreads * kLdsRowUnroll);
    const uint64_t v_idx = S.v_first + it.block;
    for (uint64_t i = 0; i < steps; ++i)
#pragma unroll
      for (int j = 0; j < kLdsRowUnroll; ++j) {
        const uint64_t u = am_lds_unit(i, j);
        if (u < units) {
          const uint64_t e = it.elem0 + u * VEC;
#pragma unroll
          for (int k = 0; k < VEC; ++k) ids[e + k] = v_idx;
        }
      }
  }
}

// ===========================================================================
// LARGE family: a block is cut into chunks of THREADS*UPT units, one per work item
// ===========================================================================
struct AmChunkItem {
  const AmSeg* seg;
  uint32_t block;   // block index inside the tensor
  uint64_t elem0;   // first element of the block inside the tensor
  uint64_t unit0;   // first unit of the chunk inside the block
  uint32_t lblock;  // index of the block among the bucket's large blocks
};

__device__ __forceinline__ AmChunkItem am_chunk_decode(AM_TABLE_PARAMS, uint32_t item, uint32_t chunk_units) {
  const uint32_t s = am_find_seg(item_keys, n_segs, item);
  AmChunkItem it;
  it.seg = segs + s;
  const uint32_t local = item - item_keys[s];
  it.block = local / it.seg->chunks_per_block;
  const uint32_t chunk = local - it.block * it.seg->chunks_per_block;
  it.elem0 = (uint64_t)it.block * it.seg->block_numel;
  it.unit0 = (uint64_t)chunk * chunk_units;
  it.lblock = lblock_keys[s] + it.block;
  return it;
}

template <int THREADS>
__device__ __forceinline__ uint64_t am_chunk_unit(uint64_t unit0, int k) {
  return unit0 + threadIdx.x + (uint64_t)k * THREADS;
}

// Sum of g^2 of one chunk per WAVEFRONT (four chunks per 256-thread workgroup): a wavefront walks its
// chunk of THREADS*UPT units 64 at a time, so there is no LDS traffic and no barrier, and a
// workgroup reads four times the bytes of one update-kernel item.
// ALT: some tensor of the bucket uses one of the ablation's other statistics.  It is a template
// parameter because that path needs the chunk's gradient a second time from the registers, which
// would otherwise cost the plain sum of squares its occupancy (67 -> 120 VGPRs).
template <typename G, int VEC, int THREADS, int UPT, bool ALT>
__global__ __launch_bounds__(256) void am_large_partial(AM_KERNEL_PARAMS, uint32_t item_base,
                                                        uint32_t n_items, uint32_t keep_g,
                                                        float* __restrict__ partials) {
  // work items [item_base, item_base + n_items) of the bucket: the whole bucket, or one slice of it
  constexpr int STEPS = THREADS * UPT / 64;  // units per lane
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const uint32_t n_groups = (n_items + 3) / 4;
  for (uint32_t grp = blockIdx.x; grp < n_groups; grp += gridDim.x) {
    const uint32_t first = am_xcd_swizzle(grp, n_groups, xcd_code) * 4;
    uint32_t item = first + wave;
    const bool active = item < n_items;
    if (!active) item = n_items - 1;
    item = __builtin_amdgcn_readfirstlane(item_base + item);
    const AmChunkItem it = am_chunk_decode(AM_TABLE_ARGS, item, THREADS * UPT);
    const AmSeg& S = *it.seg;
    if constexpr (sizeof(G) == 2 && VEC == 4 && STEPS % 2 == 0) {
      // bf16 units are 8 bytes: where every block is a whole number of unit pairs (16-byte aligned block
      // starts) a lane takes two adjacent units per 128-bit load, which this read-only pass needs to keep
      // up with the fp32 form (6.7 against 5.0 TB/s with 64-bit loads)
      if ((S.units_per_block & 1u) == 0 && (!ALT || am_red_is_sum_sq(S.reducer))) {
        float g8[STEPS / 2][8];
#pragma unroll
        for (int k = 0; k < STEPS / 2; ++k) {
          const uint64_t u = it.unit0 + 2 * ((uint64_t)k * 64 + lane);
          if (active && u < S.units_per_block) {
            am_load_grad_policy<G, 8>(S.g, it.elem0 + u * VEC, keep_g != 0, g8[k]);
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) g8[k][j] = 0.0f;
          }
        }
        float ss = 0.0f;
#pragma unroll
        for (int k = 0; k < STEPS / 2; ++k)
#pragma unroll
          for (int j = 0; j < 8; ++j) ss = fmaf(g8[k][j], g8[k][j], ss);
        ss = am_wave_sum(ss);
        if (active && lane == 0) partials[item] = ss;
        continue;
      }
    }
    float gv[STEPS][VEC];
#pragma unroll
    for (int k = 0; k < STEPS; ++k) {
      const uint64_t u = it.unit0 + (uint64_t)k * 64 + lane;
      if (active && u < S.units_per_block) {
        am_load_grad_policy<G, VEC>(S.g, it.elem0 + u * VEC, keep_g != 0, gv[k]);
      } else {
#pragma unroll
        for (int j = 0; j < VEC; ++j) gv[k][j] = 0.0f;
      }
    }
    float ss = 0.0f;
#pragma unroll
    for (int k = 0; k < STEPS; ++k)
#pragma unroll
      for (int j = 0; j < VEC; ++j) ss = fmaf(gv[k][j], gv[k][j], ss);
    ss = am_wave_sum(ss);
    if constexpr (ALT) {
      const uint32_t red = S.reducer;
      if (!am_red_is_sum_sq(red)) {
        ss = am_red_identity(red);
#pragma unroll
        for (int k = 0; k < STEPS; ++k)
          if (active && it.unit0 + (uint64_t)k * 64 + lane < S.units_per_block) {
            ss = am_red_accumulate(red, gv[k], ss);
          }
        ss = am_wave_reduce(red, ss);
      }
    }
    if (active && lane == 0) partials[item] = ss;
  }
}

// One wavefront per large block: sums the block's chunk partials in a fixed order
// (lane-strided, then butterfly) in double, updates v and stores the step scale.
__global__ __launch_bounds__(256) void am_large_finalize(AM_KERNEL_PARAMS, uint32_t lblock_base,
                                                         uint32_t n_lblocks, const float* __restrict__ partials,
                                                         float* __restrict__ v, float* __restrict__ scales,
                                                         AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  // large blocks [lblock_base, lblock_base + n_lblocks) of the bucket
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t waves_per_grid = gridDim.x * 4;
  for (uint32_t i = blockIdx.x * 4 + (threadIdx.x >> 6); i < n_lblocks; i += waves_per_grid) {
    const uint32_t lb = lblock_base + i;
    const uint32_t s = am_find_seg(lblock_keys, n_segs, lb);
    const AmSeg& S = segs[s];
    const uint32_t block = lb - lblock_keys[s];
    const uint32_t first = item_keys[s] + block * S.chunks_per_block;
    const uint32_t red = S.reducer;
    double acc = (double)am_red_identity(red);
    if (am_red_is_sum_sq(red)) {
      for (uint32_t c = lane; c < S.chunks_per_block; c += 64) acc += (double)partials[first + c];
      acc = am_wave_sum_f64(acc);
    } else {
      for (uint32_t c = lane; c < S.chunks_per_block; c += 64) acc = am_combine(red, acc, (double)partials[first + c]);
      acc = am_wave_reduce_f64(red, acc);
    }
    if (lane == 0) {
      const uint64_t v_idx = S.v_first + block;
      float v_new, scale;
      am_block_scalars(am_red_finish(red, (float)acc, (float)S.block_numel), v[v_idx], sc, &v_new, &scale);
      v[v_idx] = v_new;
      scales[lb] = scale;
    }
  }
}

// The same for blocks cut into MANY chunks (whole-tensor blocks of 10^7..10^8 elements have 10^3..10^5 chunk
// partials; one wavefront per block then spends longer on this walk than the update pass spends on a gigabyte):
// one 1024-thread workgroup per block, each thread summing every 1024th partial in double, then the
// wavefront butterfly, then the 16 wavefront results in wavefront order.  Fixed order, no atomics.
constexpr int kWideFinalizeThreads = 1024;
__global__ __launch_bounds__(kWideFinalizeThreads) void am_large_finalize_wide(
    AM_KERNEL_PARAMS, uint32_t lblock_base, uint32_t n_lblocks, const float* __restrict__ partials,
    float* __restrict__ v, float* __restrict__ scales, AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  constexpr int WAVES = kWideFinalizeThreads / 64;
  __shared__ double xch[WAVES];
  for (uint32_t i = blockIdx.x; i < n_lblocks; i += gridDim.x) {
    if (i != blockIdx.x) __syncthreads();  // the previous block's wavefront results have been read
    const uint32_t lb = lblock_base + i;
    const uint32_t s = am_find_seg(lblock_keys, n_segs, lb);
    const AmSeg& S = segs[s];
    const uint32_t block = lb - lblock_keys[s];
    const uint32_t first = item_keys[s] + block * S.chunks_per_block;
    const uint32_t red = S.reducer;
    double acc = (double)am_red_identity(red);
    if (am_red_is_sum_sq(red)) {
#pragma unroll 4
      for (uint32_t c = threadIdx.x; c < S.chunks_per_block; c += kWideFinalizeThreads) acc += (double)partials[first + c];
      acc = am_wave_sum_f64(acc);
    } else {
#pragma unroll 4
      for (uint32_t c = threadIdx.x; c < S.chunks_per_block; c += kWideFinalizeThreads)
        acc = am_combine(red, acc, (double)partials[first + c]);
      acc = am_wave_reduce_f64(red, acc);
    }
    if ((threadIdx.x & 63) == 0) xch[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      double total = xch[0];
      if (am_red_is_sum_sq(red)) {
        for (int w = 1; w < WAVES; ++w) total += xch[w];
      } else {
        for (int w = 1; w < WAVES; ++w) total = am_combine(red, total, xch[w]);
      }
      const uint64_t v_idx = S.v_first + block;
      float v_new, scale;
      am_block_scalars(am_red_finish(red, (float)total, (float)S.block_numel), v[v_idx], sc, &v_new, &scale);
      v[v_idx] = v_new;
      scales[lb] = scale;
    }
  }
}

template <typename G, int VEC, int THREADS, int UPT>
__global__ __launch_bounds__(THREADS) void am_large_update(AM_KERNEL_PARAMS, uint32_t item_base,
                                                           uint32_t n_items, uint32_t keep_g,
                                                           const float* __restrict__ scales, AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = item_base + am_xcd_swizzle(grp, n_items, xcd_code);
    const AmChunkItem it = am_chunk_decode(AM_TABLE_ARGS, item, THREADS * UPT);
    const AmSeg& S = *it.seg;
    const float scale = scales[it.lblock];
    const float decay = sc.lr_wd * S.wd_scale;
    float gv[UPT][VEC], mv[UPT][VEC], pv[UPT][VEC];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_chunk_unit<THREADS>(it.unit0, k);
      if (u < S.units_per_block) {
        const uint64_t e = it.elem0 + u * VEC;
        am_load_grad_policy<G, VEC>(S.g, e, keep_g != 0, gv[k]);
        am_load_f32<VEC>(S.m, e, mv[k]);
        am_load_f32<VEC>(S.p, e, pv[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_chunk_unit<THREADS>(it.unit0, k);
      if (u < S.units_per_block) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) am_update_elem(gv[k][j], mv[k][j], pv[k][j], scale, decay, sc);
        const uint64_t e = it.elem0 + u * VEC;
        am_store_f32<VEC>(S.m, e, mv[k]);
        am_store_f32<VEC>(S.p, e, pv[k]);
      }
    }
  }
}

template <int VEC, int THREADS, int UPT>
__global__ __launch_bounds__(THREADS) void am_large_ids(AM_KERNEL_PARAMS,
                                                        uint32_t n_items, uint32_t tensor,
                                                        uint64_t* __restrict__ ids) {
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const AmChunkItem it = am_chunk_decode(AM_TABLE_ARGS, item, THREADS * UPT);
    const AmSeg& S = *it.seg;
    if (S.tensor != tensor) continue;
    const uint64_t v_idx = S.v_first + it.block;
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_chunk_unit<THREADS>(it.unit0, k);
      if (u < S.units_per_block) {
        const uint64_t e = it.elem0 + u * VEC;
#pragma unroll
        for (int j = 0; j < VEC; ++j) ids[e + j] = v_idx;
      }
    }
  }
}

// ===========================================================================
// STRIDED family: the tensor is a row-major [R, C] matrix whose blocks are its C columns
// (a weight stored transposed).  A work item is a tile: `rows_per_item` consecutive rows of a group
// of 256 * CPL units (256 * CPL * VEC columns).  Every access is a contiguous 128-bit run along a
// row, and column sums need no cross-lane reduction at all: a lane only ever adds up its own columns.
//   am_strided_partial   per tile: the statistic of g^2 of each column over the tile's rows
//   am_strided_finalize  per column: fixed-order combination over the row chunks (double), v update, step scale
//   am_strided_update    m and p update with the per-column step scales (linear walk, see below)
// CPL = 2 (bf16 gradients in 4-element units, rows of an even number of units): the partial pass gives a
// lane two ADJACENT units, so its 8 bf16 values are one 128-bit load (a read-only pass needs 128-bit
// loads to keep up).  Both passes index the partial sums and the step scales by column, so their unit
// maps never have to agree.
// ===========================================================================
constexpr int kStridedLoads = 8;  // rows in flight per thread in the partial pass

struct AmStridedItem {
  const AmSeg* seg;
  uint64_t row0;       // first row of the tile
  uint64_t unit0;      // first unit (inside a row) of the tile's column group
  uint32_t row_chunk;
};

template <int CPL>
__device__ __forceinline__ AmStridedItem am_strided_decode(AM_TABLE_PARAMS, uint32_t item, uint32_t rows_per_item) {
  const uint32_t s = am_find_seg(item_keys, n_segs, item);
  AmStridedItem it;
  it.seg = segs + s;
  const uint32_t local = item - item_keys[s];
  it.row_chunk = local / it.seg->chunks_per_block;
  const uint32_t group = local - it.row_chunk * it.seg->chunks_per_block;
  it.row0 = (uint64_t)it.row_chunk * rows_per_item;
  it.unit0 = (uint64_t)group * (kStridedThreads * CPL);
  return it;
}

template <typename G, int VEC, int CPL>
__global__ __launch_bounds__(kStridedThreads) void am_strided_partial(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                      uint32_t rows_per_item,
                                                                      float* __restrict__ partials) {
  constexpr int W = VEC * CPL;                 // adjacent columns a lane owns in this pass
  constexpr int ROWS = kStridedLoads;          // rows in flight (one load of W gradients each)
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const AmStridedItem it = am_strided_decode<CPL>(AM_TABLE_ARGS, item, rows_per_item);
    const AmSeg& S = *it.seg;
    const uint64_t rows = S.block_numel, row_len = S.row_len;
    const uint64_t unit = it.unit0 + (uint64_t)threadIdx.x * CPL;   // CPL adjacent units
    const bool lane_on = unit < S.units_per_block;                  // rows hold a whole number of CPL-unit groups
    const uint32_t n_rows = (uint32_t)(rows - it.row0 < rows_per_item ? rows - it.row0 : rows_per_item);
    const uint32_t red = S.reducer;
    float acc[W];
#pragma unroll
    for (int j = 0; j < W; ++j) acc[j] = am_red_identity(red);
    for (uint32_t r = 0; r < n_rows; r += ROWS) {
      float gv[ROWS][W];
#pragma unroll
      for (int q = 0; q < ROWS; ++q) {
        const uint64_t row = it.row0 + r + q;
        if (lane_on && r + q < n_rows) {
          am_load_grad<G, W>(S.g, row * row_len + unit * VEC, gv[q]);
        } else {
#pragma unroll
          for (int j = 0; j < W; ++j) gv[q][j] = 0.0f;
        }
      }
      if (am_red_is_sum_sq(red)) {
#pragma unroll
        for (int q = 0; q < ROWS; ++q)
#pragma unroll
          for (int j = 0; j < W; ++j) acc[j] = fmaf(gv[q][j], gv[q][j], acc[j]);
      } else {
#pragma unroll
        for (int q = 0; q < ROWS; ++q)
          if (lane_on && r + q < n_rows) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
              const float one[1] = {gv[q][j]};  // a lane's W columns are W different blocks
              acc[j] = am_red_accumulate(red, one, acc[j]);
            }
          }
      }
    }
    // plain (cached) stores: the finalize kernel reads these back right away
    if (lane_on) {
      float* dst = partials + S.aux + (uint64_t)it.row_chunk * row_len + unit * VEC;
#pragma unroll
      for (int j = 0; j < W; ++j) dst[j] = acc[j];
    }
  }
}

// One thread per column of the bucket; consecutive threads read consecutive floats of a chunk's partials.
__global__ __launch_bounds__(256) void am_strided_finalize(AM_KERNEL_PARAMS, uint32_t n_cols,
                                                           uint32_t rows_per_item,
                                                           const float* __restrict__ partials,
                                                           float* __restrict__ v, float* __restrict__ scales,
                                                           AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  for (uint32_t gc = blockIdx.x * 256 + threadIdx.x; gc < n_cols; gc += gridDim.x * 256) {
    const uint32_t s = am_find_seg(lblock_keys, n_segs, gc);
    const AmSeg& S = segs[s];
    const uint64_t col = gc - lblock_keys[s];
    const uint64_t rows = S.block_numel, row_len = S.row_len;
    const uint64_t n_chunks = (rows + rows_per_item - 1) / rows_per_item;
    const float* src = partials + S.aux + col;
    const uint32_t red = S.reducer;
    double acc = (double)am_red_identity(red);
    if (am_red_is_sum_sq(red)) {
#pragma unroll 4
      for (uint64_t c = 0; c < n_chunks; ++c) acc += (double)src[c * row_len];
    } else {
      for (uint64_t c = 0; c < n_chunks; ++c) acc = am_combine(red, acc, (double)src[c * row_len]);
    }
    const uint64_t v_idx = S.v_first + col;
    float v_new, scale;
    am_block_scalars(am_red_finish(red, (float)acc, (float)rows), v[v_idx], sc, &v_new, &scale);
    v[v_idx] = v_new;
    scales[gc] = scale;
  }
}

// The update pass walks the stored matrix LINEARLY: a work item is a tile of 256 * kStridedUpdateUpt
// consecutive units of the tensor (whole rows one after the other, as am_large_update walks a block), so
// a workgroup's accesses are one contiguous run per array; the column of a unit, and with it the step
// scale, follows from the unit's position inside its row.  (Tiles shaped like the partial pass's -- a
// column group over many rows -- touch 8 KB pieces 128 KB apart and ran 20 % slower.)  The pass has work
// items of its own: `item_keys` here is the bucket's SECOND key array.
template <typename G, int VEC>
__global__ __launch_bounds__(kStridedThreads) void am_strided_update(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                     const float* __restrict__ scales,
                                                                     AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  constexpr int UPT = kStridedUpdateUpt;
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const uint32_t s = am_find_seg(item_keys, n_segs, item);
    const AmSeg& S = segs[s];
    const uint64_t units_per_row = S.units_per_block;
    const uint64_t total_units = S.block_numel * units_per_row;   // rows * units per row
    const uint64_t unit0 = (uint64_t)(item - item_keys[s]) * (kStridedThreads * UPT);
    const float decay = sc.lr_wd * S.wd_scale;
    const float* __restrict__ tensor_scales = scales + S.lblock_first;
    float gv[UPT][VEC], mv[UPT][VEC], pv[UPT][VEC], scale[UPT][VEC];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = unit0 + threadIdx.x + (uint64_t)k * kStridedThreads;
      if (u < total_units) {
        const uint64_t e = u * VEC;
        am_load_grad<G, VEC>(S.g, e, gv[k]);
        am_load_f32<VEC>(S.m, e, mv[k]);
        am_load_f32<VEC>(S.p, e, pv[k]);
        const uint64_t col = (u % units_per_row) * VEC;            // a unit never straddles rows
        if constexpr (VEC % 4 == 0) {
          // the bucket's scale array is 256-byte aligned and every tensor of the bucket has a multiple of
          // VEC columns, so a unit's scales are whole 16-byte words (cached loads: they are re-read by every row)
#pragma unroll
          for (int q = 0; q < VEC / 4; ++q) {
            const am_f32x4 w = *am_global(reinterpret_cast<const am_f32x4*>(tensor_scales + col) + q);
            scale[k][4 * q + 0] = w.x; scale[k][4 * q + 1] = w.y; scale[k][4 * q + 2] = w.z; scale[k][4 * q + 3] = w.w;
          }
        } else {
#pragma unroll
          for (int j = 0; j < VEC; ++j) scale[k][j] = tensor_scales[col + j];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = unit0 + threadIdx.x + (uint64_t)k * kStridedThreads;
      if (u < total_units) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) am_update_elem(gv[k][j], mv[k][j], pv[k][j], scale[k][j], decay, sc);
        const uint64_t e = u * VEC;
        am_store_f32<VEC>(S.m, e, mv[k]);
        am_store_f32<VEC>(S.p, e, pv[k]);
      }
    }
  }
}

// The update pass's walk, writing the v index of every element of tensor `tensor`.
template <int VEC>
__global__ __launch_bounds__(kStridedThreads) void am_strided_ids(AM_KERNEL_PARAMS, uint32_t n_items,
                                                                  uint32_t tensor, uint64_t* __restrict__ ids) {
  constexpr int UPT = kStridedUpdateUpt;
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const uint32_t s = am_find_seg(item_keys, n_segs, item);
    const AmSeg& S = segs[s];
    if (S.tensor != tensor) continue;
    const uint64_t units_per_row = S.units_per_block;
    const uint64_t total_units = S.block_numel * units_per_row;
    const uint64_t unit0 = (uint64_t)(item - item_keys[s]) * (kStridedThreads * UPT);
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = unit0 + threadIdx.x + (uint64_t)k * kStridedThreads;
      if (u < total_units) {
        const uint64_t col = (u % units_per_row) * VEC;
#pragma unroll
        for (int j = 0; j < VEC; ++j) ids[u * VEC + j] = S.v_first + col + j;
      }
    }
  }
}

// ===========================================================================
// ELEMENTWISE family (block_numel == 1): Algorithm 1 with mean(g*g) = g*g, i.e. AdamW
// ===========================================================================
struct AmTileItem {
  const AmSeg* seg;
  uint64_t unit0;  // first unit of the tile inside the tensor
};

__device__ __forceinline__ AmTileItem am_tile_decode(AM_TABLE_PARAMS, uint32_t item, uint32_t tile_units) {
  const uint32_t s = am_find_seg(item_keys, n_segs, item);
  AmTileItem it;
  it.seg = segs + s;
  it.unit0 = (uint64_t)(item - item_keys[s]) * tile_units;
  return it;
}

template <typename G, int VEC, int THREADS, int UPT>
__global__ __launch_bounds__(THREADS) void am_elementwise(AM_KERNEL_PARAMS,
                                                          uint32_t n_items, float* __restrict__ v, AmScalarsArg sc_arg) {
  const AmScalars sc = am_scalars(sc_arg);
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const AmTileItem it = am_tile_decode(AM_TABLE_ARGS, item, THREADS * UPT);
    const AmSeg& S = *it.seg;
    float* __restrict__ vt = v + S.v_first;
    const float decay = sc.lr_wd * S.wd_scale;
    float gv[UPT][VEC], mv[UPT][VEC], pv[UPT][VEC], vv[UPT][VEC];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_chunk_unit<THREADS>(it.unit0, k);
      if (u < S.units_per_block) {
        const uint64_t e = u * VEC;
        am_load_grad<G, VEC>(S.g, e, gv[k]);
        am_load_f32<VEC>(S.m, e, mv[k]);
        am_load_f32<VEC>(S.p, e, pv[k]);
        am_load_f32<VEC>(vt, e, vv[k]);
      }
    }
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_chunk_unit<THREADS>(it.unit0, k);
      if (u < S.units_per_block) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          float v_new, scale;
          // a block of one element: every statistic of the 1-vector g*g is g*g itself
          am_block_scalars(gv[k][j] * gv[k][j], vv[k][j], sc, &v_new, &scale);
          vv[k][j] = v_new;
          am_update_elem(gv[k][j], mv[k][j], pv[k][j], scale, decay, sc);
        }
        const uint64_t e = u * VEC;
        am_store_f32<VEC>(S.m, e, mv[k]);
        am_store_f32<VEC>(S.p, e, pv[k]);
        am_store_f32<VEC>(vt, e, vv[k]);
      }
    }
  }
}

template <int VEC, int THREADS, int UPT>
__global__ __launch_bounds__(THREADS) void am_elementwise_ids(AM_KERNEL_PARAMS,
                                                              uint32_t n_items, uint32_t tensor,
                                                              uint64_t* __restrict__ ids) {
  for (uint32_t grp = blockIdx.x; grp < n_items; grp += gridDim.x) {
    const uint32_t item = am_xcd_swizzle(grp, n_items, xcd_code);
    const AmTileItem it = am_tile_decode(AM_TABLE_ARGS, item, THREADS * UPT);
    const AmSeg& S = *it.seg;
    if (S.tensor != tensor) continue;
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
      const uint64_t u = am_chunk_unit<THREADS>(it.unit0, k);
      if (u < S.units_per_block) {
        const uint64_t e = u * VEC;
#pragma unroll
        for (int j = 0; j < VEC; ++j) ids[e + j] = S.v_first + e + j;
      }
    }
  }
}

#endif  // AM_KERNELS_H_
