// Device helpers for gfx950: 128-bit global access, bf16 widening, DPP wavefront
// reductions with a fixed combination order, work-table lookup.
#ifndef AM_DEVICE_H_
#define AM_DEVICE_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "am_tables.h"

typedef float am_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int am_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int am_u32x2 __attribute__((ext_vector_type(2)));

// Pointers read out of the work tables have no known address space; all of them point to
// device (global) memory, so say so: the loads and stores become global_* instead of flat_*.
#define AM_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ const AM_GLOBAL T* am_global(const T* p) {
  return (const AM_GLOBAL T*)(uintptr_t)p;
}
template <typename T>
__device__ __forceinline__ AM_GLOBAL T* am_global(T* p) {
  return (AM_GLOBAL T*)(uintptr_t)p;
}

struct am_bf16 {
  uint16_t bits;
};

#ifndef AM_STREAMING
#define AM_STREAMING 1  // 1: mark the bulk loads / stores non-temporal (data is touched once per step)
#endif

// ---------------------------------------------------------------------------
// global memory access: VEC floats at element offset `e` (e is a multiple of VEC)
// ---------------------------------------------------------------------------
template <int VEC>
__device__ __forceinline__ void am_load_f32(const float* __restrict__ base, uint64_t e, float (&out)[VEC]) {
  if constexpr (VEC == 1) {
#if AM_STREAMING
    out[0] = __builtin_nontemporal_load(am_global(base + e));
#else
    out[0] = *am_global(base + e);
#endif
  } else {
#pragma unroll
    for (int j = 0; j < VEC / 4; ++j) {
      const AM_GLOBAL am_f32x4* src = am_global(reinterpret_cast<const am_f32x4*>(base + e) + j);
#if AM_STREAMING
      am_f32x4 t = __builtin_nontemporal_load(src);
#else
      am_f32x4 t = *src;
#endif
      out[4 * j + 0] = t.x;
      out[4 * j + 1] = t.y;
      out[4 * j + 2] = t.z;
      out[4 * j + 3] = t.w;
    }
  }
}

template <int VEC>
__device__ __forceinline__ void am_store_f32(float* __restrict__ base, uint64_t e, const float (&in)[VEC]) {
  if constexpr (VEC == 1) {
#if AM_STREAMING
    __builtin_nontemporal_store(in[0], am_global(base + e));
#else
    *am_global(base + e) = in[0];
#endif
  } else {
#pragma unroll
    for (int j = 0; j < VEC / 4; ++j) {
      am_f32x4 t;
      t.x = in[4 * j + 0];
      t.y = in[4 * j + 1];
      t.z = in[4 * j + 2];
      t.w = in[4 * j + 3];
      AM_GLOBAL am_f32x4* dst = am_global(reinterpret_cast<am_f32x4*>(base + e) + j);
#if AM_STREAMING
      __builtin_nontemporal_store(t, dst);
#else
      *dst = t;
#endif
    }
  }
}

__device__ __forceinline__ float am_bits_to_f32(uint32_t b) { return __builtin_bit_cast(float, b); }

// Gradient units.  AmRaw<G,VEC>::T is the register / LDS form of one unit as it sits in memory
// (VEC fp32 values, or VEC bf16 values packed two to a dword); am_widen turns it into VEC floats.
// bf16 is the upper half of an fp32 word, so widening is a shift or a mask (exact).
template <typename G, int VEC> struct AmRaw;
template <> struct AmRaw<float, 1> { using T = float; };
template <> struct AmRaw<float, 4> { using T = am_f32x4; };
template <> struct AmRaw<am_bf16, 1> { using T = uint16_t; };
template <> struct AmRaw<am_bf16, 4> { using T = am_u32x2; };
template <> struct AmRaw<am_bf16, 8> { using T = am_u32x4; };

template <typename G, int VEC>
__device__ __forceinline__ typename AmRaw<G, VEC>::T am_load_grad_raw(const void* __restrict__ base, uint64_t e) {
  using T = typename AmRaw<G, VEC>::T;
  const AM_GLOBAL T* src = am_global(reinterpret_cast<const T*>(reinterpret_cast<const G*>(base) + e));
#if AM_STREAMING
  return __builtin_nontemporal_load(src);
#else
  return *src;
#endif
}

// The same load with the cache policy chosen at run time (uniform over the launch): `keep` asks for an
// ordinary cached load, so that a second pass over the same bytes soon after may find them on chip.
template <typename G, int VEC>
__device__ __forceinline__ typename AmRaw<G, VEC>::T am_load_grad_raw_policy(const void* __restrict__ base, uint64_t e,
                                                                            bool keep) {
  using T = typename AmRaw<G, VEC>::T;
  const AM_GLOBAL T* src = am_global(reinterpret_cast<const T*>(reinterpret_cast<const G*>(base) + e));
  if (keep) return *src;
  return __builtin_nontemporal_load(src);
}

__device__ __forceinline__ void am_widen(float r, float (&out)[1]) { out[0] = r; }
__device__ __forceinline__ void am_widen(am_f32x4 r, float (&out)[4]) {
  out[0] = r.x; out[1] = r.y; out[2] = r.z; out[3] = r.w;
}
__device__ __forceinline__ void am_widen(uint16_t r, float (&out)[1]) { out[0] = am_bits_to_f32(((uint32_t)r) << 16); }
__device__ __forceinline__ void am_widen(am_u32x2 r, float (&out)[4]) {
  out[0] = am_bits_to_f32(r.x << 16);  // little endian: the low half is the earlier element
  out[1] = am_bits_to_f32(r.x & 0xffff0000u);
  out[2] = am_bits_to_f32(r.y << 16);
  out[3] = am_bits_to_f32(r.y & 0xffff0000u);
}
__device__ __forceinline__ void am_widen(am_u32x4 r, float (&out)[8]) {
  const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    out[2 * j + 0] = am_bits_to_f32(w[j] << 16);
    out[2 * j + 1] = am_bits_to_f32(w[j] & 0xffff0000u);
  }
}

// Gradient load, widened to fp32.
template <typename G, int VEC>
__device__ __forceinline__ void am_load_grad(const void* __restrict__ base, uint64_t e, float (&out)[VEC]) {
  am_widen(am_load_grad_raw<G, VEC>(base, e), out);
}

template <typename G, int VEC>
__device__ __forceinline__ void am_load_grad_policy(const void* __restrict__ base, uint64_t e, bool keep,
                                                    float (&out)[VEC]) {
  am_widen(am_load_grad_raw_policy<G, VEC>(base, e, keep), out);
}

// ---------------------------------------------------------------------------
// reductions.  Every lane ends with the same bits: the combination tree is fixed
// (butterfly inside a row of 16 lanes, then rows 0..3 combined as (r0+r1)+(r2+r3)),
// so results do not depend on scheduling.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float am_dpp(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// Sum over each aligned group of 16 lanes (one DPP row).
__device__ __forceinline__ float am_row16_sum(float x) {
  x += am_dpp<0xB1>(x);   // quad_perm [1,0,3,2]
  x += am_dpp<0x4E>(x);   // quad_perm [2,3,0,1]
  x += am_dpp<0x141>(x);  // row_half_mirror: the other quad of the half row
  x += am_dpp<0x140>(x);  // row_mirror: the other half row
  return x;
}

// Sum over the 64 lanes of the wavefront.
__device__ __forceinline__ float am_wave_sum(float x) {
  x = am_row16_sum(x);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return (r0 + r1) + (r2 + r3);
}

// Sum over a workgroup of WAVES wavefronts; `slots` is WAVES floats of LDS that
// nobody else touches until the next barrier-separated reuse.  Ends with a barrier
// passed by all threads; every thread returns the same value.
template <int WAVES>
__device__ __forceinline__ float am_group_sum(float x, float* slots) {
  x = am_wave_sum(x);
  if constexpr (WAVES == 1) {
    return x;
  } else {
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) slots[wave] = x;
    __syncthreads();
    float total = slots[0];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) total += slots[w];
    return total;
  }
}

// Double-precision wavefront sum with a fixed butterfly (used once per large block).
__device__ __forceinline__ double am_wave_sum_f64(double x) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
  return x;
}

// ---------------------------------------------------------------------------
// Block statistics of s = g .* g that may feed v.  AM_RED_MEAN is Algorithm 1 (Section 2.3);
// the others are the candidates of the appendix's ablation on the design of Adam-mini, read as
// "Algorithm 1 with r(g .* g) in place of mean(g .* g)":
//   1-norm  sum_i |s_i| = sum_i g_i^2      2-norm  sqrt(sum_i s_i^2) = sqrt(sum_i g_i^4)
//   max     largest g_i^2                  min     smallest g_i^2
// A NaN among the g_i makes every statistic NaN (max and min hand it on like the sums do).
// The statistic is a tensor property (AmSeg::reducer); mean and 1-norm share the sum-of-squares
// path, the other three run through the generic accumulate / combine functions below.
// ---------------------------------------------------------------------------
enum : uint32_t { AM_RED_MEAN = 0, AM_RED_NORM1 = 1, AM_RED_NORM2 = 2, AM_RED_MAX = 3, AM_RED_MIN = 4 };

__device__ __forceinline__ bool am_red_is_sum_sq(uint32_t red) { return red <= AM_RED_NORM1; }

template <typename T>
__device__ __forceinline__ T am_nanmax(T a, T b) { return (b > a || b != b) ? b : a; }
template <typename T>
__device__ __forceinline__ T am_nanmin(T a, T b) { return (b < a || b != b) ? b : a; }

// Combination of two partial results (branch-free: lanes of one wavefront may hold different reducers).
template <typename T>
__device__ __forceinline__ T am_combine(uint32_t red, T a, T b) {
  const T sum = a + b, hi = am_nanmax(a, b), lo = am_nanmin(a, b);
  return red < AM_RED_MAX ? sum : (red == AM_RED_MAX ? hi : lo);
}

// Neutral element of the combination.
__device__ __forceinline__ float am_red_identity(uint32_t red) {
  return red == AM_RED_MIN ? __builtin_huge_valf() : 0.0f;
}

// N more gradient elements, in order, into a lane's partial result.
template <int N>
__device__ __forceinline__ float am_red_accumulate(uint32_t red, const float (&g)[N], float acc) {
  if (red == AM_RED_NORM2) {
#pragma unroll
    for (int j = 0; j < N; ++j) { const float s = g[j] * g[j]; acc = fmaf(s, s, acc); }
  } else if (red == AM_RED_MAX) {
#pragma unroll
    for (int j = 0; j < N; ++j) acc = am_nanmax(acc, g[j] * g[j]);
  } else if (red == AM_RED_MIN) {
#pragma unroll
    for (int j = 0; j < N; ++j) acc = am_nanmin(acc, g[j] * g[j]);
  } else {
#pragma unroll
    for (int j = 0; j < N; ++j) acc = fmaf(g[j], g[j], acc);
  }
  return acc;
}

// The statistic from the fully combined result x over a block of n elements.
__device__ __forceinline__ float am_red_finish(uint32_t red, float x, float n) {
  return red == AM_RED_MEAN ? x / n : (red == AM_RED_NORM2 ? sqrtf(x) : x);
}

__device__ __forceinline__ float am_row16_reduce(uint32_t red, float x) {
  x = am_combine(red, x, am_dpp<0xB1>(x));
  x = am_combine(red, x, am_dpp<0x4E>(x));
  x = am_combine(red, x, am_dpp<0x141>(x));
  x = am_combine(red, x, am_dpp<0x140>(x));
  return x;
}

__device__ __forceinline__ float am_wave_reduce(uint32_t red, float x) {
  x = am_row16_reduce(red, x);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
  return am_combine(red, am_combine(red, r0, r1), am_combine(red, r2, r3));
}

__device__ __forceinline__ double am_wave_reduce_f64(uint32_t red, double x) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) x = am_combine(red, x, __shfl_xor(x, off, 64));
  return x;
}

// ---------------------------------------------------------------------------
// work-table lookup: last segment whose first key is <= key
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t am_find_seg(const uint32_t* __restrict__ keys, uint32_t n_segs, uint32_t key) {
  uint32_t lo = 0, hi = n_segs;
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (keys[mid] <= key) lo = mid; else hi = mid;
  }
  return lo;
}

// The step's scalars: the launch argument itself, or the copy in device memory it points to (a uniform
// choice, and a scalar load: every lane of every workgroup reads the same 32 bytes).
__device__ __forceinline__ AmScalars am_scalars(const AmScalarsArg& a) {
  return a.dev ? *a.dev : a.val;
}

// ---------------------------------------------------------------------------
// the arithmetic of Algorithm 1 (Section 2.3), fp32
// ---------------------------------------------------------------------------
// Per-block scalars from the block statistic (mean of g^2 in Algorithm 1): new second moment and
// the step scale s = (lr/bc1) / (sqrt(v/bc2) + eps).
__device__ __forceinline__ void am_block_scalars(float stat, float v_old, const AmScalars& sc,
                                                 float* v_new, float* scale) {
  const float v = fmaf(sc.beta2, v_old, sc.omb2 * stat);
  const float v_hat = v / sc.bc2;
  const float denom = sqrtf(v_hat) + sc.eps;
  *v_new = v;
  *scale = sc.step_size / denom;
}

// Elementwise part: m <- (1-beta1) g + beta1 m ; p <- p - lr*lambda_k*p ; p <- p - scale * m.
__device__ __forceinline__ void am_update_elem(float g, float& m, float& p, float scale, float decay,
                                               const AmScalars& sc) {
  const float m_new = fmaf(sc.beta1, m, sc.omb1 * g);
  float q = fmaf(-decay, p, p);
  q = fmaf(-scale, m_new, q);
  m = m_new;
  p = q;
}

#endif  // AM_DEVICE_H_
