// Micro-benchmarks behind the roofline figures of the profiling sweeps (measurement aid, not
// part of the FastGen path; built into its own library, libfgubench.so).
//
// One "wave-step" of the sweeps is what a wave does with one streamed tile: 16
// v_mfma_f32_32x32x16_bf16 (two owner fragments x eight k-slabs of head dimension 128) and the
// softmax arithmetic of the 2 x 16 score elements each lane then holds (scale-and-shift,
// exp2, accumulate; plus the running maximum in the first sweep). The kernels below run that
// work from registers only (no LDS, no global loads, no barrier), three waves per SIMD as the
// shipped kernel, and time:
//   mode 1  the 16 MFMAs alone                      -> what the matrix pipe sustains
//   mode 2  the softmax arithmetic alone            -> what the vector ALU needs per wave-step
//   mode 3  both, as the sweep does (MFMAs, then the arithmetic on their result)
//   mode 4  mode 3 of the second sweep (no running maximum, multiply by 1/l folded in)
// If mode 3 takes about mode 1 + mode 2, the two pipes of a SIMD do not overlap for this
// instruction mix and the sweeps cannot exceed  t(mode 1) / t(mode 3)  of the MFMA-only rate.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "fg_common.h"

namespace {

template <int MODE>
__global__ __launch_bounds__(256, 3) void fg_ubench_kernel(float* __restrict__ out, unsigned long long* __restrict__ clk,
                                                           int iters, float c) {
  const int tid = threadIdx.x;
  // shader-clock and constant-rate (100 MHz) counters around the loop: their ratio is the clock
  // the chip actually holds under this instruction mix
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  bf16x8 a[8], b0[8], b1[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      a[kk][e] = (__bf16)(0.01f * (float)((tid + 3 * kk + e) % 17) - 0.08f);
      b0[kk][e] = (__bf16)(0.02f * (float)((tid + 5 * kk + e) % 13) - 0.12f);
      b1[kk][e] = (__bf16)(0.015f * (float)((tid + 7 * kk + e) % 11) - 0.07f);
    }
  }
  f32x16 acc0, acc1;
#pragma unroll
  for (int i = 0; i < 16; ++i) { acc0[i] = 0.001f * (float)(tid + i); acc1[i] = -0.002f * (float)(tid - i); }
  float m_run[2] = {FG_NEG_BIG, FG_NEG_BIG};
  double l_run[2] = {0.0, 0.0};
  float ms[16], il[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { ms[i] = 0.25f * (float)i; il[i] = 1.0f / (float)(i + 1 + tid); }

  for (int it = 0; it < iters; ++it) {
    if (MODE != 2) {
      // the operands are opaque to the compiler each round (no instruction is emitted for this)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(a[kk]));
#pragma unroll
      for (int i = 0; i < 16; ++i) { acc0[i] = 0.f; acc1[i] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], b0[kk], acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], b1[kk], acc1, 0, 0, 0);
      }
    } else {
      asm volatile("" : "+v"(acc0), "+v"(acc1));
    }
    if (MODE == 1) {
      l_run[0] += (double)(acc0[0] + acc1[5]);   // keeps the results alive at the cost of three operations
    } else if (MODE == 2 || MODE == 3) {
      // first sweep, interior tile: running maximum and sum of a row (two owner fragments)
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        const f32x16& ac = f == 0 ? acc0 : acc1;
        const float x0 = fmaxf(fmaxf(ac[0], ac[1]), ac[2]), x1 = fmaxf(fmaxf(ac[3], ac[4]), ac[5]);
        const float x2 = fmaxf(fmaxf(ac[6], ac[7]), ac[8]), x3 = fmaxf(fmaxf(ac[9], ac[10]), ac[11]);
        const float x4 = fmaxf(fmaxf(ac[12], ac[13]), ac[14]);
        const float y0 = fmaxf(fmaxf(x0, x1), x2), y1 = fmaxf(fmaxf(x3, x4), ac[15]);
        const float m_new = fmaxf(fmaxf(y0, y1) * c, m_run[f]);
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s += fg_exp2(fmaf(ac[i], c, -m_new));
        l_run[f] = l_run[f] * (double)fg_exp2(m_run[f] - m_new) + (double)s;
        m_run[f] = m_new;
      }
    } else {
      // second sweep, interior tile: normalised terms summed per column
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        const f32x16& ac = f == 0 ? acc0 : acc1;
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) s = fmaf(fg_exp2(fmaf(ac[i], c, -ms[i])), il[i], s);
        l_run[f] += (double)s;
      }
    }
  }
  out[(size_t)blockIdx.x * 256 + tid] = (float)(l_run[0] + l_run[1]) + m_run[0] + m_run[1];
  if (clk != nullptr && tid == 0) {
    clk[2 * blockIdx.x] = clock64() - c0;
    clk[2 * blockIdx.x + 1] = wall_clock64() - w0;
  }
}

template <int MODE>
hipError_t run(float* out, unsigned long long* clk, int blocks, int iters, hipStream_t s) {
  hipLaunchKernelGGL((fg_ubench_kernel<MODE>), dim3((unsigned)blocks), dim3(256), 0, s, out, clk, iters, 0.1275f);
  return hipGetLastError();
}

}  // namespace

extern "C" {

// Runs one micro-benchmark: `blocks` workgroups of four waves, `iters` wave-steps per wave.
//   mode        1..4, see the head of this file
//   out         device float[blocks * 256], written (results are meaningless, they keep the work alive)
//   clk         device uint64[2 * blocks] or NULL: per workgroup, shader-clock cycles and 100 MHz ticks
//               spent in the loop (written by the timed launch)
//   ns_per_wave_step  host: measured time / iters x (waves per SIMD in flight), i.e. the time one SIMD
//               needs per wave-step when `blocks` fills the chip evenly (a multiple of 768 on 256 CUs)
//   shader_mhz  host or NULL (needs clk): the shader clock held during the timed launch, averaged
//               over the workgroups (cycles / ticks x 100 MHz)
// Returns 0, or a HIP error code. Synchronises the stream.
int fg_ubench_run(int mode, int blocks, int iters, float* out, unsigned long long* clk, void* stream,
                  double* ns_per_wave_step, double* shader_mhz) {
  if (mode < 1 || mode > 4 || blocks < 1 || iters < 1 || !out || !ns_per_wave_step) return -1;
  if (shader_mhz && !clk) return -1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return (int)e; }
  auto launch = [&]() {
    switch (mode) {
      case 1: return run<1>(out, clk, blocks, iters, s);
      case 2: return run<2>(out, clk, blocks, iters, s);
      case 3: return run<3>(out, clk, blocks, iters, s);
      default: return run<4>(out, clk, blocks, iters, s);
    }
  };
  e = launch();  // warm-up
  if (e == hipSuccess) e = hipEventRecord(e0, s);
  if (e == hipSuccess) e = launch();
  if (e == hipSuccess) e = hipEventRecord(e1, s);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (e != hipSuccess) return (int)e;
  // wave-steps per SIMD = iters * (waves per SIMD) = iters * blocks / 256 CUs (one wave of a block per SIMD)
  const double per_simd = (double)iters * (double)blocks / 256.0;
  *ns_per_wave_step = (double)ms * 1e6 / per_simd;
  if (shader_mhz) {
    std::vector<unsigned long long> h(2 * (size_t)blocks);
    e = hipMemcpy(h.data(), clk, h.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost);
    if (e != hipSuccess) return (int)e;
    double cyc = 0.0, ticks = 0.0;
    for (int b = 0; b < blocks; ++b) { cyc += (double)h[2 * b]; ticks += (double)h[2 * b + 1]; }
    *shader_mhz = ticks > 0.0 ? cyc / ticks * 100.0 : 0.0;
  }
  return 0;
}

}  // extern "C"
