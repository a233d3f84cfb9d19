// Block-wide exact selection of the k largest of m non-negative doubles with the tie rule
// "equal score -> the smaller position is kept" (the frequent policy of Sec. 3.4 keeps the
// tokens with the largest cumulative attention score). MSB-first radix select on the IEEE
// bit patterns (monotone for non-negative doubles), 8 bits per pass, then -- only if the
// boundary value is shared -- the same select on the positions of the tied elements.
#pragma once
#include "fg_common.h"

struct fg_topk {
  uint64_t thr;   // bit pattern of the k-th largest score
  uint32_t pthr;  // among scores == thr, positions <= pthr are inside the top-k
  int mode;       // 0: nothing selected, 1: everything selected, 2: use (thr, pthr)
};

struct fg_select_smem {
  int hist[256];
  int red[20];
  int digit, rem, cnt;
};

__device__ __forceinline__ bool fg_in_topk(const fg_topk& t, double score, uint32_t pos) {
  if (t.mode != 2) return t.mode == 1;
  const uint64_t key = (uint64_t)__double_as_longlong(score);
  return key > t.thr || (key == t.thr && pos <= t.pthr);
}

// One radix pass: histogram of the digit at `shift` over active elements whose key matches
// `prefix` under `mask`, then locate the digit that holds the rem-th largest.
// KeyFn(j, &key) returns false for inactive elements. blockDim.x must be 256.
template <class KeyFn>
__device__ __forceinline__ void fg_radix_pass(KeyFn keyfn, int m, int shift, uint64_t prefix,
                                              uint64_t mask, int rem, fg_select_smem* sm) {
  const int tid = threadIdx.x;
  sm->hist[tid] = 0;
  __syncthreads();
  for (int j = tid; j < m; j += 256) {
    uint64_t key;
    if (keyfn(j, &key) && (key & mask) == prefix) atomicAdd(&sm->hist[(int)((key >> shift) & 255u)], 1);
  }
  __syncthreads();
  // thread t looks at bucket 255 - t: buckets in descending order
  const int h = sm->hist[255 - tid];
  int total;
  const int before = fg_block_exscan_i32(h, sm->red, &total);
  if (before < rem && before + h >= rem) {
    sm->digit = 255 - tid;
    sm->rem = rem - before;
    sm->cnt = h;
  }
  __syncthreads();
}

// ScoreFn(j) -> double (>= 0), PosFn(j) -> uint32 position (unique per element).
template <class ScoreFn, class PosFn>
__device__ __forceinline__ fg_topk fg_select_topk(ScoreFn score, PosFn pos, int m, int k,
                                                  fg_select_smem* sm) {
  fg_topk r;
  r.thr = 0; r.pthr = 0;
  if (k <= 0) { r.mode = 0; return r; }
  if (k >= m) { r.mode = 1; return r; }
  r.mode = 2;
  uint64_t prefix = 0, mask = 0;
  int rem = k;
  auto key1 = [&](int j, uint64_t* key) { *key = (uint64_t)__double_as_longlong(score(j)); return true; };
  for (int shift = 56; shift >= 0; shift -= 8) {
    fg_radix_pass(key1, m, shift, prefix, mask, rem, sm);
    prefix |= (uint64_t)sm->digit << shift;
    mask |= (uint64_t)0xff << shift;
    rem = sm->rem;
  }
  const int n_eq = sm->cnt;  // elements equal to the threshold; `rem` of them are taken
  r.thr = prefix;
  if (rem == n_eq) { r.pthr = 0xffffffffu; return r; }
  // ties at the boundary: keep the `rem` smallest positions among the tied elements,
  // i.e. select the rem-th largest of (~pos)
  const uint64_t thr = prefix;
  auto key2 = [&](int j, uint64_t* key) {
    if ((uint64_t)__double_as_longlong(score(j)) != thr) return false;
    *key = (uint64_t)(0xffffffffu - pos(j));
    return true;
  };
  uint64_t p2 = 0, m2 = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    fg_radix_pass(key2, m, shift, p2, m2, rem, sm);
    p2 |= (uint64_t)sm->digit << shift;
    m2 |= (uint64_t)0xff << shift;
    rem = sm->rem;
  }
  r.pthr = 0xffffffffu - (uint32_t)p2;
  return r;
}
