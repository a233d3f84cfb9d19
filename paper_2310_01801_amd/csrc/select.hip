// Policy choice and compaction (Alg. 1: "C <- apply Eq. 1 to A", "K^,V^ <- f(K,V,C)").
//
//   fg_classify_kernel token ids -> class bytes (special / punctuation).
//   fg_select_kernel   per unit: the kept sets of the policy family (by default Eq. 2's:
//                      special, +punctuation, +frequent, +local; "+" = union; any table of
//                      component masks is accepted), their recoveries from the column /
//                      band sums, the cheapest policy reaching T (Eq. 1), kept flags and
//                      their prefix scan.
//   fg_offsets_kernel  exclusive scan of the per-unit slot reservations -> pool offsets,
//                      and the static split-KV work list of the decode kernels.
//   fg_gather_kernel   copies the kept rows of K, V with score, position, class.
//   fg_export_kernel   cache state read-back in ascending position order.
#include "fg_common.h"
#include "fg_internal.h"
#include "fg_select.h"

namespace {

// Token ids -> class bytes (Sec. 3.4: which tokens C_special / C_punct. keep). The two id lists
// are small and arrive by value; every thread compares its token with all of them.
__global__ __launch_bounds__(256) void fg_classify_kernel(fg_classify_args a) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= a.count) return;
  const int32_t id = a.token_ids[i];
  int c = 0;
  for (int k = 0; k < a.num_special; ++k) c |= (id == a.special[k]) ? FG_CLASS_SPECIAL : 0;
  for (int k = 0; k < a.num_punct; ++k) c |= (id == a.punct[k]) ? FG_CLASS_PUNCT : 0;
  a.token_class[i] = (uint8_t)c;
}

__global__ __launch_bounds__(256) void fg_select_kernel(fg_select_args a) {
  __shared__ fg_select_smem sm;
  __shared__ double dred[8];
  __shared__ int ired[20];
  const int u = blockIdx.x, tid = threadIdx.x, n = a.n;
  const double* cs = a.colsum + (size_t)u * n;
  const double* bc = a.bandcol + (size_t)u * n;
  const uint8_t* cls = a.token_class + (size_t)(u / a.units_per_seq) * n;
  const int k_f = fg_budget(a.r_f, n);
  const int w = a.w;

  const fg_topk tk = fg_select_topk([&](int j) { return cs[j]; },
                                    [&](int j) { return (uint32_t)j; }, n, k_f, &sm);

  // Recovery of a policy = mean over rows of the kept attention mass. A column in the
  // policy's static set (special / punctuation / frequent) counts in every row: its column
  // sum; any other column is only seen through the local band, if the policy has one.
  double r[4] = {0.0, 0.0, 0.0, 0.0};
  int cnt[4] = {0, 0, 0, 0}, ccnt[4] = {0, 0, 0, 0};
  for (int j = tid; j < n; j += 256) {
    const int c = cls[j];
    const double s = cs[j], b = bc[j];
    const bool top = fg_in_topk(tk, s, (uint32_t)j), tail = j >= n - w;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const int m = a.family[p];
      const bool byclass = ((m & FG_COMP_SPECIAL) && (c & FG_CLASS_SPECIAL)) ||
                           ((m & FG_COMP_PUNCT) && (c & FG_CLASS_PUNCT));
      const bool st = byclass || ((m & FG_COMP_FREQUENT) && top);
      const bool loc = (m & FG_COMP_LOCAL) != 0;
      r[p] += st ? s : (loc ? b : 0.0);
      if (st || (loc && tail)) cnt[p]++;
      if (byclass) ccnt[p]++;
    }
  }
  double R[5];
  int C[5], CC[4];
  for (int c = 0; c < 4; ++c) {
    R[c] = fg_block_sum_f64(r[c], dred) / ((double)n * (double)a.G);  // mean over the rows of all G query heads
    C[c] = fg_block_sum_i32(cnt[c], ired);
    CC[c] = fg_block_sum_i32(ccnt[c], ired);
  }
  R[4] = 1.0;
  C[4] = n;
  // Eq. 1: the cheapest usable policy whose recovery reaches T; equal cost -> smaller id.
  // C_full always qualifies. (For the nested family of Eq. 2 this is the first id reaching T.)
  int policy = 4;
  for (int c = 3; c >= 0; --c)
    if (a.family[c] != 0 && R[c] >= a.T && C[c] <= C[policy]) policy = c;
  if (a.forced_policy >= 0) policy = a.forced_policy;
  const int comp = policy < 4 ? a.family[policy] : 0;

  // kept flags of the chosen policy and their exclusive scan (slot of each kept token)
  int running = 0;
  for (int base = 0; base < n; base += 256) {
    const int j = base + tid;
    int keep = 0, cbyte = 0;
    if (j < n) {
      const int c = cls[j];
      bool k = policy >= 4;
      if (comp & FG_COMP_SPECIAL) k = k || (c & FG_CLASS_SPECIAL) != 0;
      if (comp & FG_COMP_PUNCT) k = k || (c & FG_CLASS_PUNCT) != 0;
      if (comp & FG_COMP_FREQUENT) k = k || fg_in_topk(tk, cs[j], (uint32_t)j);
      if (comp & FG_COMP_LOCAL) k = k || (j >= n - w);
      keep = k ? 1 : 0;
      cbyte = k ? (4 | (c & 3)) : 0;  // kept flag plus the token's class bits
    }
    int total;
    const int ex = fg_block_exscan_i32(keep, ired, &total);
    if (j < n) {
      a.keep[(size_t)u * n + j] = (uint8_t)cbyte;
      a.slot[(size_t)u * n + j] = running + ex;
    }
    running += total;
    __syncthreads();
  }

  if (tid == 0) {
    // slots to reserve: the class-kept prompt tokens, and if a class component is present
    // every later token may be special/punctuation and stay (+S); the frequent budget follows
    // the sequence length; the window is fixed; one extra slot for the new token while it is
    // attended to. Never more than the uncompressed cache.
    const int S = a.S, full = n + S;
    long long cap;
    if (policy == 4) cap = full;
    else {
      cap = CC[policy];
      if (comp & (FG_COMP_SPECIAL | FG_COMP_PUNCT)) cap += S;
      if (comp & FG_COMP_FREQUENT) cap += fg_budget(a.r_f, full);
      if (comp & FG_COMP_LOCAL) cap += w;
      if (comp & (FG_COMP_FREQUENT | FG_COMP_LOCAL)) cap += 1;
      if (cap < running) cap = running;
    }
    if (cap > full) cap = full;
    if (cap < 1) cap = 1;
    a.cap[u] = (int)cap;
    a.len[u] = running;
    a.policy[u] = policy | (comp << 8);  // id in the low byte, component mask above
    if (a.policy_out) a.policy_out[u] = policy;
    for (int c = 0; c < 5; ++c) {
      a.recov[u * 5 + c] = R[c];
      a.kcount[u * 5 + c] = C[c];
      if (a.recov_out) a.recov_out[u * 5 + c] = R[c];
      if (a.kcount_out) a.kcount_out[u * 5 + c] = C[c];
    }
  }
}

// Single workgroup: off[u] = sum_{v<u} cap[v]; chunk_off[u] = sum_{v<u} ceil(cap[v]/chunk).
__global__ __launch_bounds__(1024) void fg_offsets_kernel(const int32_t* __restrict__ cap,
                                                          int64_t* __restrict__ off,
                                                          int32_t* __restrict__ chunk_off,
                                                          int32_t* __restrict__ flags, int U,
                                                          int64_t pool_tokens, int64_t max_chunks, int chunk) {
  __shared__ int red[20];
  __shared__ long long wsum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  long long run_off = 0;
  int run_chunk = 0;
  for (int base = 0; base < U; base += 1024) {
    const int u = base + tid;
    const int c = (u < U) ? cap[u] : 0;
    const int nch = (c + chunk - 1) / chunk;
    int total;
    const int exc = fg_block_exscan_i32(nch, red, &total);
    // 64-bit scan of the capacities: wave scan + serial over the 16 waves
    long long inc = c;
    for (int o = 1; o < 64; o <<= 1) {
      long long t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    long long wbase = 0, wtot = 0;
    for (int i = 0; i < 16; ++i) {
      if (i < wave) wbase += wsum[i];
      wtot += wsum[i];
    }
    if (u < U) {
      off[u] = run_off + wbase + inc - c;
      chunk_off[u] = run_chunk + exc;
    }
    run_off += wtot;
    run_chunk += total;
    __syncthreads();
  }
  if (tid == 0) {
    off[U] = run_off;
    chunk_off[U] = run_chunk;
    flags[0] = (run_off > pool_tokens || (int64_t)run_chunk > max_chunks) ? 1 : 0;
    flags[1] = 0;
  }
}

// Work-item records of the decode attention kernel: item c of unit u covers slots
// [chunk * (c - chunk_off[u]), +chunk) of that unit (chunk = 128 or 256 tokens). 8 ints per item: unit, chunk, cap, tokens held
// by the unit (kept current by the update kernel), off lo, off hi, policy word (id | component
// mask << 8), 0.
__global__ __launch_bounds__(256) void fg_item_map_kernel(const int32_t* __restrict__ chunk_off,
                                                          const int32_t* __restrict__ cap,
                                                          const int64_t* __restrict__ off,
                                                          const int32_t* __restrict__ len,
                                                          const int32_t* __restrict__ policy,
                                                          int32_t* __restrict__ item_rec,
                                                          const int32_t* __restrict__ flags, int U) {
  if (flags[0] != 0) return;
  const int u = blockIdx.x * 256 + threadIdx.x;
  if (u >= U) return;
  const int64_t o = off[u];
  const int c0 = chunk_off[u], c1 = chunk_off[u + 1];
  for (int c = c0; c < c1; ++c) {
    int32_t* r = item_rec + (size_t)c * 8;
    r[0] = u; r[1] = c - c0; r[2] = cap[u]; r[3] = len[u];
    r[4] = (int32_t)(o & 0xffffffffll); r[5] = (int32_t)(o >> 32); r[6] = policy[u]; r[7] = 0;
  }
}

// 16 prompt positions per workgroup; 16-byte chunks of the kept rows are copied by
// consecutive lanes (one 256-byte bf16 row = 16 lanes).
__global__ __launch_bounds__(256) void fg_gather_kernel(fg_compact_args a, int tiles_per_unit) {
  if (a.flags[0] != 0) return;
  const int u = blockIdx.x / tiles_per_unit, tile = blockIdx.x % tiles_per_unit;
  const int n = a.n, tid = threadIdx.x;
  const int rb = a.d * a.esize, cpr = rb / 16;
  const int64_t off = a.off[u];
  const char* Ku = static_cast<const char*>(a.K) + (size_t)u * n * rb;
  const char* Vu = static_cast<const char*>(a.V) + (size_t)u * n * rb;
  char* ck = static_cast<char*>(a.ck);
  char* cv = static_cast<char*>(a.cv);
  for (int q = tid; q < 16 * cpr; q += 256) {
    const int j = tile * 16 + q / cpr, ch = q % cpr;
    if (j >= n) continue;
    const int kb = a.keep[(size_t)u * n + j];
    if (!kb) continue;
    const int64_t dst = off + a.slot[(size_t)u * n + j];
    *reinterpret_cast<u32x4*>(ck + dst * rb + ch * 16) = *reinterpret_cast<const u32x4*>(Ku + (size_t)j * rb + ch * 16);
    *reinterpret_cast<u32x4*>(cv + dst * rb + ch * 16) = *reinterpret_cast<const u32x4*>(Vu + (size_t)j * rb + ch * 16);
    if (ch == 0) {
      a.cscore[dst] = a.colsum[(size_t)u * n + j];
      a.cpos[dst] = j;
      a.ccls[dst] = (uint8_t)(kb & 3);
    }
  }
}

// Single workgroup: offsets[u] = sum_{v<u} len[v].
__global__ __launch_bounds__(1024) void fg_len_scan_kernel(const int32_t* __restrict__ len,
                                                           int64_t* __restrict__ offsets,
                                                           int32_t* __restrict__ lengths,
                                                           const int32_t* __restrict__ flags,
                                                           int32_t* __restrict__ status, int U) {
  __shared__ long long wsum[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  long long run = 0;
  for (int base = 0; base < U; base += 1024) {
    const int u = base + tid;
    const int c = (u < U) ? len[u] : 0;
    long long inc = c;
    for (int o = 1; o < 64; o <<= 1) {
      long long t = __shfl_up(inc, o, 64);
      if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    long long wbase = 0, wtot = 0;
    for (int i = 0; i < 16; ++i) {
      if (i < wave) wbase += wsum[i];
      wtot += wsum[i];
    }
    if (u < U) {
      if (offsets) offsets[u] = run + wbase + inc - c;
      if (lengths) lengths[u] = c;
    }
    run += wtot;
    __syncthreads();
  }
  if (tid == 0) {
    if (offsets) offsets[U] = run;
    if (status) status[0] = flags[0] ? (int)FG_ECAP : 0;
  }
}

// One workgroup per unit. Slots are unordered in the cache; the rank of a held position is
// the number of held positions below it, read off a bitmap of held positions.
__global__ __launch_bounds__(256) void fg_export_kernel(fg_export_args a, const int64_t* __restrict__ dst_off) {
  extern __shared__ uint32_t smem[];  // words bitmap, then words+1 prefix counts
  if (a.flags[0] != 0) return;
  const int u = blockIdx.x, tid = threadIdx.x;
  const int words = (a.max_pos + 31) / 32;
  uint32_t* bits = smem;
  uint32_t* pre = smem + words;
  const int L = a.len[u];
  const int64_t src = a.off[u], dst = dst_off[u];
  for (int i = tid; i < words; i += 256) bits[i] = 0u;
  __syncthreads();
  for (int j = tid; j < L; j += 256) {
    const int p = a.cpos[src + j];
    atomicOr(&bits[p >> 5], 1u << (p & 31));
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t run = 0;
    for (int i = 0; i < words; ++i) { pre[i] = run; run += __popc(bits[i]); }
  }
  __syncthreads();
  const int rb = a.d * a.esize, cpr = rb / 16;
  for (int j = tid; j < L; j += 256) {
    const int p = a.cpos[src + j];
    const int rank = (int)pre[p >> 5] + __popc(bits[p >> 5] & ((1u << (p & 31)) - 1u));
    if (a.positions) a.positions[dst + rank] = p;
    if (a.scores) a.scores[dst + rank] = a.cscore[src + j];
  }
  if (a.keys || a.values) {
    for (int q = tid; q < L * cpr; q += 256) {
      const int j = q / cpr, ch = q % cpr;
      const int p = a.cpos[src + j];
      const int rank = (int)pre[p >> 5] + __popc(bits[p >> 5] & ((1u << (p & 31)) - 1u));
      if (a.keys)
        *reinterpret_cast<u32x4*>(static_cast<char*>(a.keys) + (dst + rank) * rb + ch * 16) =
            *reinterpret_cast<const u32x4*>(static_cast<const char*>(a.ck) + (src + j) * rb + ch * 16);
      if (a.values)
        *reinterpret_cast<u32x4*>(static_cast<char*>(a.values) + (dst + rank) * rb + ch * 16) =
            *reinterpret_cast<const u32x4*>(static_cast<const char*>(a.cv) + (src + j) * rb + ch * 16);
    }
  }
}

}  // namespace

hipError_t fg_launch_classify(const fg_classify_args& a, hipStream_t s) {
  const unsigned blocks = (unsigned)((a.count + 255) / 256);
  hipLaunchKernelGGL(fg_classify_kernel, dim3(blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t fg_launch_select(const fg_select_args& a, hipStream_t s) {
  hipLaunchKernelGGL(fg_select_kernel, dim3((unsigned)a.U), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t fg_launch_compact(const fg_compact_args& a, hipStream_t s) {
  const int tiles = (a.n + 15) / 16;
  hipLaunchKernelGGL(fg_gather_kernel, dim3((unsigned)((size_t)a.U * tiles)), dim3(256), 0, s, a, tiles);
  return hipGetLastError();
}

hipError_t fg_launch_offsets(const int32_t* cap, const int32_t* len, const int32_t* policy, int64_t* off,
                             int32_t* chunk_off, int32_t* item_unit, int32_t* flags, int U, int64_t pool_tokens,
                             int64_t max_chunks, int chunk, hipStream_t s) {
  hipLaunchKernelGGL(fg_offsets_kernel, dim3(1), dim3(1024), 0, s, cap, off, chunk_off, flags, U,
                     pool_tokens, max_chunks, chunk);
  hipLaunchKernelGGL(fg_item_map_kernel, dim3((unsigned)((U + 255) / 256)), dim3(256), 0, s,
                     chunk_off, cap, off, len, policy, item_unit, flags, U);
  return hipGetLastError();
}

hipError_t fg_launch_export(const fg_export_args& a, hipStream_t s) {
  // offsets are needed by the per-unit kernel even if the caller does not want them: the
  // caller-visible array is used when given, else positions cannot be packed
  hipLaunchKernelGGL(fg_len_scan_kernel, dim3(1), dim3(1024), 0, s, a.len, a.offsets, a.lengths,
                     a.flags, a.status, a.U);
  if (a.positions || a.scores || a.keys || a.values) {
    const int words = (a.max_pos + 31) / 32;
    const size_t smem = (size_t)(2 * words + 1) * sizeof(uint32_t);
    hipLaunchKernelGGL(fg_export_kernel, dim3((unsigned)a.U), dim3(256), smem, s, a, a.offsets);
  }
  return hipGetLastError();
}
