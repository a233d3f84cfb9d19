// Shared device-side helpers of the FastGen HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define FG_WAVE 64

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define FG_LOG2E 1.4426950408889634f

// a finite stand-in for -infinity that survives (x - x) without producing NaN
#define FG_NEG_BIG (-1.0e30f)

__device__ __forceinline__ float fg_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float fg_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float fg_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even float -> bf16 bits (inputs are finite here)
__device__ __forceinline__ uint32_t fg_f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ double fg_shfl_xor_f64(double v, int mask) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __shfl_xor(lo, mask, 64);
  hi = __shfl_xor(hi, mask, 64);
  return __hiloint2double(hi, lo);
}

// ---- cross-lane reductions on the data-parallel-primitive path of the vector ALU (no LDS
// round trip): lane i combines with a lane of its own row of 16.
template <int CTRL>
__device__ __forceinline__ float fg_dpp(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
constexpr int FG_DPP_XOR1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int FG_DPP_XOR2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int FG_DPP_HALF_MIRROR = 0x141; // lane i <-> 7 - i within 8 lanes
constexpr int FG_DPP_MIRROR = 0x140;      // lane i <-> 15 - i within 16 lanes

// Sum over aligned groups of N consecutive lanes (N = 1, 2, 4, 8, 16, 32, 64); every lane of the
// group receives the total. Fixed order: deterministic.
template <int N>
__device__ __forceinline__ float fg_group_sum(float v) {
  if (N >= 2) v += fg_dpp<FG_DPP_XOR1>(v);
  if (N >= 4) v += fg_dpp<FG_DPP_XOR2>(v);
  if (N >= 8) v += fg_dpp<FG_DPP_HALF_MIRROR>(v);
  if (N >= 16) v += fg_dpp<FG_DPP_MIRROR>(v);
  if (N >= 32) v += __shfl_xor(v, 16, 64);
  if (N >= 64) v += __shfl_xor(v, 32, 64);
  return v;
}

// Maximum over the 64 lanes of the wave, as a wave-uniform value.
__device__ __forceinline__ float fg_wave_max(float v) {
  v = fmaxf(v, fg_dpp<FG_DPP_XOR1>(v));
  v = fmaxf(v, fg_dpp<FG_DPP_XOR2>(v));
  v = fmaxf(v, fg_dpp<FG_DPP_HALF_MIRROR>(v));
  v = fmaxf(v, fg_dpp<FG_DPP_MIRROR>(v));
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

template <int CTRL>
__device__ __forceinline__ int fg_dpp_i32(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);  // lanes without a source read 0
}
__device__ __forceinline__ int fg_readlane_i32(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

// Sum over the 64 lanes of the wave, as a wave-uniform value (fixed order).
__device__ __forceinline__ int fg_wave_sum_i32(int v) {
  v += fg_dpp_i32<FG_DPP_XOR1>(v);
  v += fg_dpp_i32<FG_DPP_XOR2>(v);
  v += fg_dpp_i32<FG_DPP_HALF_MIRROR>(v);
  v += fg_dpp_i32<FG_DPP_MIRROR>(v);
  return (fg_readlane_i32(v, 0) + fg_readlane_i32(v, 16)) + (fg_readlane_i32(v, 32) + fg_readlane_i32(v, 48));
}

template <int CTRL>
__device__ __forceinline__ double fg_dpp_f64(double v) {
  return __hiloint2double(fg_dpp_i32<CTRL>(__double2hiint(v)), fg_dpp_i32<CTRL>(__double2loint(v)));
}
// Sum of a double over aligned groups of N consecutive lanes (N <= 32); every lane of the group
// receives the total. Fixed order.
template <int N>
__device__ __forceinline__ double fg_group_sum_f64(double v) {
  static_assert(N <= 32, "groups of up to 32 lanes");
  if (N >= 2) v += fg_dpp_f64<FG_DPP_XOR1>(v);
  if (N >= 4) v += fg_dpp_f64<FG_DPP_XOR2>(v);
  if (N >= 8) v += fg_dpp_f64<FG_DPP_HALF_MIRROR>(v);
  if (N >= 16) v += fg_dpp_f64<FG_DPP_MIRROR>(v);
  if (N >= 32) v += fg_shfl_xor_f64(v, 16);
  return v;
}

__device__ __forceinline__ double fg_wave_sum_f64(double v) {
  v += fg_dpp_f64<FG_DPP_XOR1>(v);
  v += fg_dpp_f64<FG_DPP_XOR2>(v);
  v += fg_dpp_f64<FG_DPP_HALF_MIRROR>(v);
  v += fg_dpp_f64<FG_DPP_MIRROR>(v);
  const int hi = __double2hiint(v), lo = __double2loint(v);
  const double r0 = __hiloint2double(fg_readlane_i32(hi, 0), fg_readlane_i32(lo, 0));
  const double r1 = __hiloint2double(fg_readlane_i32(hi, 16), fg_readlane_i32(lo, 16));
  const double r2 = __hiloint2double(fg_readlane_i32(hi, 32), fg_readlane_i32(lo, 32));
  const double r3 = __hiloint2double(fg_readlane_i32(hi, 48), fg_readlane_i32(lo, 48));
  return (r0 + r1) + (r2 + r3);
}

// Minimum of a double over the wave, wave-uniform (inputs must not be NaN).
__device__ __forceinline__ double fg_wave_min_f64(double v) {
  v = fmin(v, fg_dpp_f64<FG_DPP_XOR1>(v));
  v = fmin(v, fg_dpp_f64<FG_DPP_XOR2>(v));
  v = fmin(v, fg_dpp_f64<FG_DPP_HALF_MIRROR>(v));
  v = fmin(v, fg_dpp_f64<FG_DPP_MIRROR>(v));
  const int hi = __double2hiint(v), lo = __double2loint(v);
  const double r0 = __hiloint2double(fg_readlane_i32(hi, 0), fg_readlane_i32(lo, 0));
  const double r1 = __hiloint2double(fg_readlane_i32(hi, 16), fg_readlane_i32(lo, 16));
  const double r2 = __hiloint2double(fg_readlane_i32(hi, 32), fg_readlane_i32(lo, 32));
  const double r3 = __hiloint2double(fg_readlane_i32(hi, 48), fg_readlane_i32(lo, 48));
  return fmin(fmin(r0, r1), fmin(r2, r3));
}

// Bitwise OR / AND of a 64-bit value over the wave (wave-uniform results).
__device__ __forceinline__ void fg_wave_or_and_u64(unsigned long long v_or, unsigned long long v_and,
                                                   unsigned long long* out_or, unsigned long long* out_and) {
  int olo = (int)(unsigned)v_or, ohi = (int)(unsigned)(v_or >> 32);
  int alo = (int)(unsigned)v_and, ahi = (int)(unsigned)(v_and >> 32);
#define FG_STEP(CTRL)                                                            \
  olo |= fg_dpp_i32<CTRL>(olo); ohi |= fg_dpp_i32<CTRL>(ohi);                    \
  alo &= fg_dpp_i32<CTRL>(alo); ahi &= fg_dpp_i32<CTRL>(ahi);
  FG_STEP(FG_DPP_XOR1) FG_STEP(FG_DPP_XOR2) FG_STEP(FG_DPP_HALF_MIRROR) FG_STEP(FG_DPP_MIRROR)
#undef FG_STEP
  unsigned ro_lo = 0, ro_hi = 0, ra_lo = ~0u, ra_hi = ~0u;
#pragma unroll
  for (int r = 0; r < 64; r += 16) {
    ro_lo |= (unsigned)fg_readlane_i32(olo, r); ro_hi |= (unsigned)fg_readlane_i32(ohi, r);
    ra_lo &= (unsigned)fg_readlane_i32(alo, r); ra_hi &= (unsigned)fg_readlane_i32(ahi, r);
  }
  *out_or = ((unsigned long long)ro_hi << 32) | ro_lo;
  *out_and = ((unsigned long long)ra_hi << 32) | ra_lo;
}

// Inclusive prefix sum over the 64 lanes of the wave.
__device__ __forceinline__ int fg_wave_incscan_i32(int v) {
  v += fg_dpp_i32<0x111>(v);  // row_shr:1
  v += fg_dpp_i32<0x112>(v);  // row_shr:2
  v += fg_dpp_i32<0x114>(v);  // row_shr:4
  v += fg_dpp_i32<0x118>(v);  // row_shr:8   -> inclusive within each row of 16
  const int t0 = fg_readlane_i32(v, 15), t1 = fg_readlane_i32(v, 31), t2 = fg_readlane_i32(v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}

// Deterministic block-wide sums (fixed tree order). `red` is LDS scratch with one slot per
// wave; every thread of the block must call. All threads receive the total.
__device__ __forceinline__ double fg_block_sum_f64(double v, double* red) {
  v = fg_wave_sum_f64(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  double t = 0.0;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

__device__ __forceinline__ int fg_block_sum_i32(int v, int* red) {
  v = fg_wave_sum_i32(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  int t = 0;
  for (int i = 0; i < nw; ++i) t += red[i];
  return t;
}

// Block-wide exclusive prefix sum of one int per thread (blockDim.x <= 1024, multiple of
// 64). `red` needs 17 ints. Returns the exclusive prefix; *total receives the block sum.
__device__ __forceinline__ int fg_block_exscan_i32(int v, int* red, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int inc = fg_wave_incscan_i32(v);
  __syncthreads();
  if (lane == 63) red[wave] = inc;
  __syncthreads();
  int base = 0, tot = 0;
  for (int i = 0; i < nw; ++i) {
    int c = red[i];
    if (i < wave) base += c;
    tot += c;
  }
  *total = tot;
  return base + inc - v;
}

// floor(r * L) in IEEE double: the budget rule of the frequent / local policies.
__device__ __host__ __forceinline__ int fg_budget(double r, int L) {
  double x = r * (double)L;
  return (int)floor(x);
}
