// Prompt-time attention profiling for float32 inputs (Alg. 1: A = softmax(Q K^T); Sec. 3.4
// cumulative attention score). Same two sweeps and the same outputs as the bf16 matrix-core
// kernel, on the vector ALU: this is the path of the small float32 correctness workload,
// not a throughput path, so it spends its time on accuracy instead: dot products, exponentials
// and sums in float64 (products of two floats are exact there), only the stored row statistics
// (m, 1/l) are floats. One thread owns one query row (pass 1) or one key column (pass 2)
// with its vector in registers; the other matrix is streamed through LDS in tiles of 32.
#include "fg_common.h"
#include "fg_internal.h"

namespace {

constexpr int kTile = 32;

template <int D, int PASS>
__global__ __launch_bounds__(256) void fg_profile_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, float2* __restrict__ rowstat,
    double* __restrict__ colsum, double* __restrict__ bandcol, int n, int w, float c, int nblk,
    int G) {
  __shared__ __attribute__((aligned(16))) float tile[kTile][D];
  __shared__ float2 stat_t[kTile];

  const int unit = blockIdx.x / nblk, tid = threadIdx.x;
  const int WG0 = (blockIdx.x % nblk) * 256;
  const int own = WG0 + tid;
  // G query heads share a K/V unit: sweep 1 runs per query head (unit = u * G + g) against
  // K of u; sweep 2 runs per K/V unit and streams the rows of its G query heads in turn
  const size_t mat = (size_t)n * D;
  const float* own_mat = (PASS == 1 ? Q : K) + (size_t)unit * mat;
  const float* str_base = (PASS == 1) ? K + (size_t)(unit / G) * mat : Q + (size_t)unit * G * mat;
  const float2* stat_base = rowstat + (size_t)unit * (PASS == 1 ? 1 : G) * n;

  float o[D];
#pragma unroll
  for (int k = 0; k < D; k += 4) {
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (own < n) v = *reinterpret_cast<const f32x4*>(own_mat + (size_t)own * D + k);
    o[k] = v[0]; o[k + 1] = v[1]; o[k + 2] = v[2]; o[k + 3] = v[3];
  }

  int t_begin, t_end;
  if (PASS == 1) { t_begin = 0; t_end = (min(n, WG0 + 256) + kTile - 1) / kTile; }
  else { t_begin = WG0 / kTile; t_end = (n + kTile - 1) / kTile; }

  float m_run = FG_NEG_BIG;
  double l_run = 0.0, col_acc = 0.0, band_acc = 0.0;
  const double c_d = (double)c;

  const int heads = (PASS == 1) ? 1 : G;
  for (int h = 0; h < heads; ++h) {
  const float* str_mat = str_base + (size_t)h * mat;
  const float2* stat_row = stat_base + (size_t)h * n;
  for (int t = t_begin; t < t_end; ++t) {
    const int t0 = t * kTile;
    __syncthreads();
    for (int q = tid; q < kTile * (D / 4); q += 256) {
      const int item = q / (D / 4), ch = q % (D / 4);
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (t0 + item < n) v = *reinterpret_cast<const f32x4*>(str_mat + (size_t)(t0 + item) * D + ch * 4);
      *reinterpret_cast<f32x4*>(&tile[item][ch * 4]) = v;
    }
    if (PASS == 2 && tid < kTile) stat_t[tid] = (t0 + tid < n) ? stat_row[t0 + tid] : make_float2(0.f, 0.f);
    __syncthreads();
    if (own >= n) continue;
    for (int it = 0; it < kTile; ++it) {
      const int s_idx = t0 + it;
      if (s_idx >= n) break;
      if (PASS == 1 && s_idx > own) break;   // causal: column <= row
      if (PASS == 2 && s_idx < own) continue;  // causal: row >= column
      double dot = 0.0;
#pragma unroll
      for (int k = 0; k < D; ++k) dot = fma((double)o[k], (double)tile[it][k], dot);
      const double x = dot * c_d;
      if (PASS == 1) {
        const float m_new = fmaxf(m_run, (float)x);   // a shift near the row's largest logit; any float will do
        l_run = l_run * exp2((double)m_run - (double)m_new) + exp2(x - (double)m_new);
        m_run = m_new;
      } else {
        const double p = exp2(x - (double)stat_t[it].x) * (double)stat_t[it].y;
        col_acc += p;
        if (s_idx - own < w) band_acc += p;
      }
    }
  }
  }
  if (own < n) {
    if (PASS == 1) rowstat[(size_t)unit * n + own] = make_float2(m_run, (float)(1.0 / l_run));
    else {
      colsum[(size_t)unit * n + own] = col_acc;
      bandcol[(size_t)unit * n + own] = band_acc;
    }
  }
}

template <int D>
hipError_t launch(const fg_profile_args& a, int pass, hipStream_t s) {
  const int nblk = (a.n + 255) / 256;
  const dim3 grid((unsigned)((size_t)nblk * a.U * (pass == 1 ? a.G : 1))), block(256);
  const float c = a.scale * FG_LOG2E;
  const float* Q = static_cast<const float*>(a.Q);
  const float* K = static_cast<const float*>(a.K);
  if (pass == 1)
    hipLaunchKernelGGL((fg_profile_f32_kernel<D, 1>), grid, block, 0, s, Q, K, a.rowstat, a.colsum,
                       a.bandcol, a.n, a.w, c, nblk, a.G);
  else
    hipLaunchKernelGGL((fg_profile_f32_kernel<D, 2>), grid, block, 0, s, Q, K, a.rowstat, a.colsum,
                       a.bandcol, a.n, a.w, c, nblk, a.G);
  return hipGetLastError();
}

// A caller-supplied natural-log row log-sum-exp as (m, 1/l): m = the nearest integer to its
// log2 value, 1/l = 2^(m - log2 value) in [0.70, 1.42], so that no bits are lost to the
// magnitude of the log-sum-exp itself.
__global__ void fg_lse_to_rowstat_kernel(const float* __restrict__ in, float2* __restrict__ out, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const double l2 = (double)in[i] * 1.4426950408889634074;
  const double m = rint(l2);
  out[i] = make_float2((float)m, (float)exp2(m - l2));
}

}  // namespace

hipError_t fg_launch_profile_f32(const fg_profile_args& a, int pass, hipStream_t s) {
  if (a.d == 128) return launch<128>(a, pass, s);
  return launch<64>(a, pass, s);
}

hipError_t fg_launch_lse_to_rowstat(const float* lse_nat, float2* rowstat, size_t count, hipStream_t s) {
  const unsigned blocks = (unsigned)((count + 255) / 256);
  hipLaunchKernelGGL(fg_lse_to_rowstat_kernel, dim3(blocks), dim3(256), 0, s, lse_nat, rowstat, count);
  return hipGetLastError();
}
