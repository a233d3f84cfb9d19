// Block-wide exact selection of the k largest of m non-negative doubles with the tie rule
// "equal score -> the smaller position is kept" (the frequent policy of Sec. 3.4 keeps the
// tokens with the largest cumulative attention score). MSB-first radix select on the IEEE
// bit patterns (monotone for non-negative doubles), 8 bits per pass:
//   * keys are held in registers when m <= 256 * FG_SEL_CACHE (else re-read each pass);
//   * passes over the bits that all keys share are skipped (block-wide OR/AND of the keys);
//   * the scan stops as soon as the boundary bucket is taken whole;
//   * only if the boundary value is shared does a second select run on the positions.
// blockDim.x must be 256.
#pragma once
#include "fg_common.h"

#define FG_SEL_CACHE 12

struct fg_topk {
  uint64_t thr;   // keys above thr are in; keys equal to thr are in iff pos <= pthr
  uint32_t pthr;
  int mode;       // 0: nothing selected, 1: everything selected, 2: use (thr, pthr)
};

struct fg_select_smem {
  int hist[256];
  int red[20];
  unsigned long long w_or[4], w_and[4];
  int digit, rem, cnt;
};

__device__ __forceinline__ bool fg_in_topk(const fg_topk& t, double score, uint32_t pos) {
  if (t.mode != 2) return t.mode == 1;
  const uint64_t key = (uint64_t)__double_as_longlong(score);
  return key > t.thr || (key == t.thr && pos <= t.pthr);
}

// hist[digit] += 1 for every lane with `active`; lanes sharing the digit of the first active
// lane are counted with one atomic (keys cluster in few buckets during the first passes).
__device__ __forceinline__ void fg_hist_add(int* hist, bool active, int digit) {
  const unsigned long long act = __ballot(active);
  if (act == 0ull) return;
  const int leader = __ffsll((long long)act) - 1;
  const int d0 = __builtin_amdgcn_readlane(digit, leader);  // `leader` is wave-uniform
  const bool same = active && digit == d0;
  const unsigned long long grp = __ballot(same);
  if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[d0], (int)__popcll(grp));
  if (active && !same) atomicAdd(&hist[digit], 1);
}

// After the histogram of one digit is complete: locate the bucket that holds the rem-th
// largest. Thread t looks at bucket 255 - t (descending order).
__device__ __forceinline__ void fg_radix_locate(int rem, fg_select_smem* sm) {
  const int tid = threadIdx.x;
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

// NC > 0: element tid + 256 i of the block is kc[i] (registers); NC == 0: keys come from score(j).
template <int NC, class ScoreFn, class PosFn>
__device__ __forceinline__ fg_topk fg_select_topk_impl(const uint64_t (&kc)[NC > 0 ? NC : 1], ScoreFn score,
                                                       PosFn pos, int m, int k, fg_select_smem* sm) {
  constexpr bool CACHED = NC > 0;
  fg_topk r;
  r.thr = 0; r.pthr = 0xffffffffu; r.mode = 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // ---- the bits the keys do not all share
  uint64_t k_or = 0, k_and = ~0ull;
  if (CACHED) {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      if (j < m) {
        k_or |= kc[i];
        k_and &= kc[i];
      }
    }
  } else {
    for (int j = tid; j < m; j += 256) {
      const uint64_t key = (uint64_t)__double_as_longlong(score(j));
      k_or |= key;
      k_and &= key;
    }
  }
  {
    unsigned long long wo, wa;
    fg_wave_or_and_u64(k_or, k_and, &wo, &wa);
    k_or = wo;
    k_and = wa;
  }
  __syncthreads();
  if (lane == 0) { sm->w_or[wave] = k_or; sm->w_and[wave] = k_and; }
  __syncthreads();
  k_or = sm->w_or[0] | sm->w_or[1] | sm->w_or[2] | sm->w_or[3];
  k_and = sm->w_and[0] & sm->w_and[1] & sm->w_and[2] & sm->w_and[3];
  const uint64_t diff = k_or ^ k_and;

  uint64_t prefix = 0, mask = 0;
  int rem = k, n_eq = m;
  if (diff != 0) {
    const int top = 63 - __clzll((long long)diff);  // highest bit in which two keys differ
    int shift = (top >> 3) << 3;
    mask = (shift + 8 >= 64) ? 0ull : ~((1ull << (shift + 8)) - 1ull);
    prefix = k_and & mask;
    for (; shift >= 0; shift -= 8) {
      sm->hist[tid] = 0;
      __syncthreads();
      if (CACHED) {
#pragma unroll
        for (int i = 0; i < NC; ++i) {
          const int j = tid + 256 * i;
          fg_hist_add(sm->hist, j < m && (kc[i] & mask) == prefix, (int)((kc[i] >> shift) & 255u));
        }
      } else {
        for (int j = tid; j < m; j += 256) {
          const uint64_t key = (uint64_t)__double_as_longlong(score(j));
          if ((key & mask) == prefix) atomicAdd(&sm->hist[(int)((key >> shift) & 255u)], 1);
        }
      }
      __syncthreads();
      fg_radix_locate(rem, sm);
      prefix |= (uint64_t)sm->digit << shift;
      mask |= (uint64_t)0xff << shift;
      rem = sm->rem;
      n_eq = sm->cnt;
      if (rem == n_eq) {  // the boundary bucket is taken whole: every key >= prefix is in
        r.thr = prefix;
        return r;
      }
    }
  } else {
    prefix = k_and;  // all keys are equal
  }
  r.thr = prefix;
  if (rem == n_eq) return r;
  // ties at the boundary value: keep the `rem` smallest positions among the tied elements,
  // i.e. select the rem-th largest of (~pos) over them
  const uint64_t thr = prefix;
  uint64_t p2 = 0, m2 = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    sm->hist[tid] = 0;
    __syncthreads();
    for (int j = tid; j < m; j += 256) {
      if ((uint64_t)__double_as_longlong(score(j)) != thr) continue;
      const uint64_t key = (uint64_t)(0xffffffffu - pos(j));
      if ((key & m2) == p2) atomicAdd(&sm->hist[(int)((key >> shift) & 255u)], 1);
    }
    __syncthreads();
    fg_radix_locate(rem, sm);
    p2 |= (uint64_t)sm->digit << shift;
    m2 |= (uint64_t)0xff << shift;
    rem = sm->rem;
  }
  r.pthr = 0xffffffffu - (uint32_t)p2;
  return r;
}

// Keys already in registers (element tid + 256 i is kc[i], i < NC, valid while < m).
// score(j) / pos(j) are only consulted if the boundary value is tied.
template <int NC, class ScoreFn, class PosFn>
__device__ __forceinline__ fg_topk fg_select_topk_regs(const uint64_t (&kc)[NC], ScoreFn score, PosFn pos,
                                                       int m, int k, fg_select_smem* sm) {
  fg_topk r;
  r.thr = 0; r.pthr = 0;
  if (k <= 0) { r.mode = 0; return r; }
  if (k >= m) { r.mode = 1; return r; }
  return fg_select_topk_impl<NC>(kc, score, pos, m, k, sm);
}

// Shortcut for the per-step kept-set update. Only tokens that nothing else protects (`prot`
// bit clear) can leave, and they leave lowest score first: a token is outside the top k exactly
// if at least k scores are larger. So instead of locating the k-th largest score, test the
// lowest unprotected score, then the next one, ... until one stays (a step evicts very few
// tokens). Returns false when the shortcut does not apply -- two equal scores at a tested value,
// or more than FG_EVICT_TRIES evictions -- and the caller runs the full selection instead.
// On success every unprotected token with key >= out->thr is in the top k (mode 2, no position
// tie-break needed). Keys of slot tid + 256 i are kc[i] (valid while < m). 256 threads.
#define FG_EVICT_TRIES 6
template <int NC>
__device__ __forceinline__ bool fg_evict_cut_regs(const uint64_t (&kc)[NC], uint32_t prot, int m, int k,
                                                  double* red_d, int* red_i, fg_topk* out) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const double inf = __longlong_as_double(0x7ff0000000000000ll);
  double last = -1.0;  // every evicted score so far is <= last
  for (int it = 0; it < FG_EVICT_TRIES; ++it) {
    double loc = inf;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      const double v = __longlong_as_double((long long)kc[i]);
      if (j < m && !((prot >> i) & 1u) && v > last) loc = fmin(loc, v);
    }
    loc = fg_wave_min_f64(loc);
    __syncthreads();
    if (lane == 0) red_d[wave] = loc;
    __syncthreads();
    const double kmin = fmin(fmin(red_d[0], red_d[1]), fmin(red_d[2], red_d[3]));
    out->mode = 2; out->pthr = 0xffffffffu;
    if (kmin == inf) {  // no unprotected token is left: none of them is in the top k
      out->thr = 0x7ff0000000000000ull;
      return true;
    }
    int cnt = 0;  // scores above kmin in the low half, scores equal to it in the high half
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      const double v = __longlong_as_double((long long)kc[i]);
      if (j < m) cnt += (v > kmin ? 1 : 0) + (v == kmin ? (1 << 16) : 0);
    }
    const int tot = fg_block_sum_i32(cnt, red_i);
    if ((tot >> 16) != 1) return false;       // a tie at the tested value: needs the position rule
    if ((tot & 0xffff) < k) {                  // fewer than k larger scores: it stays, and so do all above it
      out->thr = (uint64_t)__double_as_longlong(kmin);
      return true;
    }
    last = kmin;                               // at least k larger scores: it leaves; test the next one
  }
  return false;
}

// ScoreFn(j) -> double (>= 0), PosFn(j) -> uint32 position (unique per element).
template <class ScoreFn, class PosFn>
__device__ __forceinline__ fg_topk fg_select_topk(ScoreFn score, PosFn pos, int m, int k,
                                                  fg_select_smem* sm) {
  fg_topk r;
  r.thr = 0; r.pthr = 0;
  if (k <= 0) { r.mode = 0; return r; }
  if (k >= m) { r.mode = 1; return r; }
  if (m <= 256 * FG_SEL_CACHE) {
    uint64_t kc[FG_SEL_CACHE];
#pragma unroll
    for (int i = 0; i < FG_SEL_CACHE; ++i) {
      const int j = threadIdx.x + 256 * i;
      kc[i] = (j < m) ? (uint64_t)__double_as_longlong(score(j)) : 0ull;
    }
    return fg_select_topk_impl<FG_SEL_CACHE>(kc, score, pos, m, k, sm);
  }
  const uint64_t none[1] = {0ull};
  return fg_select_topk_impl<0>(none, score, pos, m, k, sm);
}
