// One decode step over the ragged compressed caches (Alg. 2: attend with K^,V^ plus the new
// token, then re-apply f with the head's policy; policies of Sec. 3.4).
//
//   fg_decode_partial_kernel  split-KV attention. The flat work list has one item per 256 (128
//       for short sequences) reserved slots of a unit (static after compaction); an item streams the K and V rows
//       of its held slots with 16-byte-per-lane coalesced loads (a 256-byte bf16 row = 16
//       lanes, 4 rows per wave load), keeps the scaled logits, and emits (max, sum, o) of its
//       chunk. The item that owns the first free slot takes the new token from k_new/v_new
//       and appends it to the cache on the way. With grouped query heads the rows loaded by
//       an item serve every head of the unit (one partial per head).
//   fg_decode_finish_kernel   one workgroup per unit: merges the chunk partials into the
//       attention output; adds this step's attention to the cumulative scores (policies with
//       `frequent`, or every policy when the step is probed); re-derives the kept set from the
//       policy's components  special | punct | TopK(score, k_f(L)) | window  and releases the
//       evicted slots in place (holes below the new length are filled with the kept rows from
//       above it); optionally reports the step's attention mass on every policy's tokens.
#include <type_traits>

#include "fg_common.h"
#include "fg_internal.h"
#include "fg_select.h"

namespace {

constexpr int FG_MOVE_LDS = 64;  // released slots per step whose move lists stay in shared memory

template <int ESIZE>
__device__ __forceinline__ void fg_unpack(const u32x4& v, float* f);
template <>
__device__ __forceinline__ void fg_unpack<2>(const u32x4& v, float* f) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = fg_bf16_lo(v[i]);
    f[2 * i + 1] = fg_bf16_hi(v[i]);
  }
}
template <>
__device__ __forceinline__ void fg_unpack<4>(const u32x4& v, float* f) {
#pragma unroll
  for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(v[i]);
}

// Dot product of the 8 bf16 pairs of two 16-byte chunks with float accumulation: four
// two-element dot instructions instead of eight unpacks and eight multiply-adds. Serves the
// output path only (the cumulative scores use the float64 logits).
__device__ __forceinline__ float fg_dot_bf16x8(const u32x4& a, const u32x4& b) {
  float acc = 0.f;
  // (pairs taken from the 8-element vectors by shuffles: handed bit-cast dwords of the 128-bit
  // vectors, the compiler of ROCm 7.2 selects element 0 for all four instructions)
  const bf16x8 av = __builtin_bit_cast(bf16x8, a), bv = __builtin_bit_cast(bf16x8, b);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(av, av, 0, 1), __builtin_shufflevector(bv, bv, 0, 1), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(av, av, 2, 3), __builtin_shufflevector(bv, bv, 2, 3), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(av, av, 4, 5), __builtin_shufflevector(bv, bv, 4, 5), acc, false);
  acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(av, av, 6, 7), __builtin_shufflevector(bv, bv, 6, 7), acc, false);
  return acc;
}

// GRP: several query heads per unit (a.G > 1); without it G is the constant 1 and the code is
// the plain multi-head path.
template <int ESIZE, int D, bool GRP, int CH>
__global__ __launch_bounds__(256) void fg_decode_partial_kernel(fg_decode_args a) {
  constexpr int RB = D * ESIZE;        // bytes per row
  constexpr int LPR = RB / 16;         // lanes per row
  constexpr int TPL = 64 / LPR;        // rows per wave load
  constexpr int EPL = 16 / ESIZE;      // elements per lane
  constexpr int TPW = CH / 4;          // tokens per wave
  constexpr int ITERS = TPW / TPL;     // loads per wave for its tokens
  __shared__ float s_red[8];
  __shared__ float s_o[GRP ? 1 : 4][D];

  // header: one 32-byte record per item carries everything, the unit's current length included
  const int item = blockIdx.x;
  const int n_items = a.chunk_off[a.U];
  const int overflow = a.flags[0];
  const int4 rec = *reinterpret_cast<const int4*>(a.item_unit + (size_t)item * 8);
  const int4 rec_off = *reinterpret_cast<const int4*>(a.item_unit + (size_t)item * 8 + 4);
  if (overflow != 0 || item >= n_items) return;
  const int u = rec.x, chunk = rec.y;
  const int Lold = rec.w, L = Lold + 1;
  // the logits are kept only where the update kernel needs them: policies with `frequent`
  // (cumulative scores), or every unit when the step is probed
  const bool keep_logits = ((rec_off.z >> 8) & FG_COMP_FREQUENT) != 0 || a.probe != nullptr;
  const int start = chunk * CH;
  if (start >= L) return;
  if (L > rec.z) {  // cannot happen while the host bounds the step count
    if (threadIdx.x == 0) a.flags[0] = 1;
    return;
  }
  const int cnt = min(CH, L - start);
  const int64_t off = ((int64_t)rec_off.y << 32) | (uint32_t)rec_off.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane % LPR, sub = lane / LPR;
  const float c = a.scale * FG_LOG2E;
  // Score path (Sec. 3.4, cumulative attention score): the products of two bf16 (or float32)
  // inputs are exact in float64 and 128 of them add up to ~1e-16 there, so the logit that the
  // update kernel turns into this step's attention is the oracle's to the last bits; the
  // float32 logit (good to ~1e-7 of its size) serves the output only.
  const double c_d = (double)a.scale * 1.4426950408889634074;

  const char* ck = static_cast<const char*>(a.ck);
  const char* cv = static_cast<const char*>(a.cv);
  const char* kn = static_cast<const char*>(a.k_new) + (size_t)u * RB;
  const char* vn = static_cast<const char*>(a.v_new) + (size_t)u * RB;

  // G query heads share the unit's cache: its rows are loaded once and used by every head
  const int G = GRP ? a.G : 1;
  const char* qu = static_cast<const char*>(a.q) + (size_t)u * G * RB;
  float qv[EPL];
  const u32x4 q_raw = *reinterpret_cast<const u32x4*>(qu + g * 16);   // this lane's 16 bytes of the query
  fg_unpack<ESIZE>(q_raw, qv);
  // grouped heads: all G query vectors are staged in LDS while the cache rows are in flight
  __shared__ __attribute__((aligned(16))) unsigned char s_q[GRP ? 16 * RB : 16];
  if (GRP) {
    for (int i = tid; i < G * LPR; i += 256)
      *reinterpret_cast<u32x4*>(&s_q[i * 16]) = *reinterpret_cast<const u32x4*>(qu + (size_t)i * 16);
  }

  // All row loads are issued back to back with no control flow in between (a branch per row
  // makes the compiler wait for each pair of loads before it issues the next). Raw buffer
  // loads over the chunk's cached rows: one per-lane offset, a constant offset per load, and
  // rows past the end read as zeros. The new token is not in the cache yet: its lane group
  // takes it from the step inputs afterwards and appends it.
  u32x4 kv[ITERS], vv[ITERS];
  const int ncached = min(cnt, Lold - start);  // rows of this chunk that are in the cache
  const __amdgpu_buffer_rsrc_t k_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(ck) + (off + start) * RB, 0, ncached * RB, 0x00020000);
  const __amdgpu_buffer_rsrc_t v_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(cv) + (off + start) * RB, 0, ncached * RB, 0x00020000);
  const int voff = (wave * TPW + sub) * RB + g * 16;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    kv[it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, voff, it * TPL * RB, 0));
    vv[it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, voff, it * TPL * RB, 0));
  }
  if (Lold >= start && Lold < start + CH) {  // this item owns the first free slot
    const u32x4 knew = *reinterpret_cast<const u32x4*>(kn + g * 16);
    const u32x4 vnew = *reinterpret_cast<const u32x4*>(vn + g * 16);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
      const int slot = start + wave * TPW + it * TPL + sub;
      if (slot == Lold) {
        kv[it] = knew;
        vv[it] = vnew;
        *reinterpret_cast<u32x4*>(static_cast<char*>(a.ck) + (off + slot) * RB + g * 16) = knew;
        *reinterpret_cast<u32x4*>(static_cast<char*>(a.cv) + (off + slot) * RB + g * 16) = vnew;
        if (g == 0) {
          a.cpos[off + slot] = a.n + a.step;
          a.ccls[off + slot] = a.class_new[u / a.units_per_seq];
          a.cscore[off + slot] = 0.0;
        }
      }
    }
  }

  if (GRP) {
    // ---- grouped heads: each wave keeps its own (max, sum, o) per head for its tokens, so the
    // head loop has no workgroup barrier; the four waves are merged once at the end.
    __shared__ float s_wp[4][16][D + 2];
    __syncthreads();  // s_q is complete
    for (int h = 0; h < G; ++h) {
      {
        const u32x4 t = *reinterpret_cast<const u32x4*>(&s_q[h * RB + g * 16]);
        fg_unpack<ESIZE>(t, qv);
      }
      // keep the cache rows packed across the head loop (unpacking them once for all heads
      // would need twice the register file)
#pragma unroll
      for (int it = 0; it < ITERS; ++it) {
        asm volatile("" : "+v"(kv[it]), "+v"(vv[it]));
      }
      float x[ITERS];
      float mw = FG_NEG_BIG;
#pragma unroll
      for (int it = 0; it < ITERS; ++it) {
        float kf[EPL];
        fg_unpack<ESIZE>(kv[it], kf);
        const int tok = wave * TPW + it * TPL + sub;
        const bool ok = tok < cnt;
        if (keep_logits) {
          double dd = 0.0;
#pragma unroll
          for (int e = 0; e < EPL; ++e) dd = fma((double)qv[e], (double)kf[e], dd);
          dd = fg_group_sum_f64<LPR>(dd) * c_d;
          if (ok && g == 0) a.clogit[(off + start + tok) * G + h] = dd;
          x[it] = ok ? (float)dd : FG_NEG_BIG;
        } else {
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) dot = fmaf(qv[e], kf[e], dot);
          dot = fg_group_sum<LPR>(dot);
          x[it] = ok ? dot * c : FG_NEG_BIG;
        }
        mw = fmaxf(mw, x[it]);
      }
      mw = fg_wave_max(mw);
      float lsum = 0.f;
      float oacc[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) oacc[e] = 0.f;
#pragma unroll
      for (int it = 0; it < ITERS; ++it) {
        const int tok = wave * TPW + it * TPL + sub;
        const float p = (tok < cnt) ? fg_exp2(x[it] - mw) : 0.f;
        lsum += p;
        float vf[EPL];
        fg_unpack<ESIZE>(vv[it], vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) oacc[e] = fmaf(p, vf[e], oacc[e]);
      }
#pragma unroll
      for (int m = LPR; m < 64; m <<= 1) {
        lsum += __shfl_xor(lsum, m, 64);
#pragma unroll
        for (int e = 0; e < EPL; ++e) oacc[e] += __shfl_xor(oacc[e], m, 64);
      }
      if (sub == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) s_wp[wave][h][2 + g * EPL + e] = oacc[e];
      }
      if (lane == 0) { s_wp[wave][h][0] = mw; s_wp[wave][h][1] = lsum; }
    }
    __syncthreads();
    for (int h = 0; h < G; ++h) {
      const float m0 = s_wp[0][h][0], m1 = s_wp[1][h][0], m2 = s_wp[2][h][0], m3 = s_wp[3][h][0];
      const float M = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
      // a wave without tokens carries the lowest max and zero sums: its factor is 0
      const float f0 = fg_exp2(m0 - M), f1 = fg_exp2(m1 - M), f2 = fg_exp2(m2 - M), f3 = fg_exp2(m3 - M);
      float* part = a.part + ((size_t)item * G + h) * (D + 2);
      if (tid < D)
        part[2 + tid] = (s_wp[0][h][2 + tid] * f0 + s_wp[1][h][2 + tid] * f1) +
                        (s_wp[2][h][2 + tid] * f2 + s_wp[3][h][2 + tid] * f3);
      if (tid == 0) {
        part[0] = M;
        part[1] = (s_wp[0][h][1] * f0 + s_wp[1][h][1] * f1) + (s_wp[2][h][1] * f2 + s_wp[3][h][1] * f3);
      }
    }
    return;
  }

  // ---- one query head per unit
  // scaled logits (log2 domain): x = c * q.k, one value per token shared by its LPR lanes
  float x[ITERS];
  float mx = FG_NEG_BIG;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    float kf[EPL];
    fg_unpack<ESIZE>(kv[it], kf);
    const int tok = wave * TPW + it * TPL + sub;
    const bool ok = tok < cnt;
    if (keep_logits) {   // wave-uniform
      double dd = 0.0;
#pragma unroll
      for (int e = 0; e < EPL; ++e) dd = fma((double)qv[e], (double)kf[e], dd);
      dd = fg_group_sum_f64<LPR>(dd) * c_d;
      if (ok && g == 0) a.clogit[off + start + tok] = dd;
      x[it] = ok ? (float)dd : FG_NEG_BIG;
    } else {
      float dot = 0.f;
      if (ESIZE == 2) dot = fg_dot_bf16x8(q_raw, kv[it]);
      else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot = fmaf(qv[e], kf[e], dot);
      }
      dot = fg_group_sum<LPR>(dot);
      x[it] = ok ? dot * c : FG_NEG_BIG;
    }
    mx = fmaxf(mx, x[it]);
  }
  mx = fg_wave_max(mx);
  if (lane == 0) s_red[wave] = mx;
  __syncthreads();
  const float M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));

  float lsum = 0.f;
  float oacc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) oacc[e] = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int tok = wave * TPW + it * TPL + sub;
    const float p = (tok < cnt) ? fg_exp2(x[it] - M) : 0.f;
    lsum += p;
    float vf[EPL];
    fg_unpack<ESIZE>(vv[it], vf);
#pragma unroll
    for (int e = 0; e < EPL; ++e) oacc[e] = fmaf(p, vf[e], oacc[e]);
  }
  // combine the row groups of the wave (lanes with equal g)
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) {
    lsum += __shfl_xor(lsum, m, 64);
#pragma unroll
    for (int e = 0; e < EPL; ++e) oacc[e] += __shfl_xor(oacc[e], m, 64);
  }
  if (sub == 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) s_o[wave][g * EPL + e] = oacc[e];
  }
  if (lane == 0) s_red[4 + wave] = lsum;
  __syncthreads();
  float* part = a.part + (size_t)item * (D + 2);
  if (tid < D) part[2 + tid] = (s_o[0][tid] + s_o[1][tid]) + (s_o[2][tid] + s_o[3][tid]);
  if (tid == 0) {
    part[0] = M;
    part[1] = (s_red[4] + s_red[5]) + (s_red[6] + s_red[7]);
  }
}

template <int ESIZE>
__device__ __forceinline__ void fg_store_out(void* out, size_t idx, float v);
template <>
__device__ __forceinline__ void fg_store_out<2>(void* out, size_t idx, float v) {
  static_cast<uint16_t*>(out)[idx] = (uint16_t)fg_f32_to_bf16_bits(v);
}
template <>
__device__ __forceinline__ void fg_store_out<4>(void* out, size_t idx, float v) {
  static_cast<float*>(out)[idx] = v;
}

template <int ESIZE, int D, bool GRP>
__global__ __launch_bounds__(256, GRP ? 2 : 4) void fg_decode_finish_kernel(fg_decode_args a) {
  constexpr int RB = D * ESIZE, CPR = RB / 16;
  __shared__ fg_select_smem sm;
  __shared__ int ired[20];
  __shared__ double dred[8];
  __shared__ float s_M[16];  // per query head: merged maximum of the scaled logits
  const int u = blockIdx.x, tid = threadIdx.x;
  const int G = GRP ? a.G : 1;
  // Every header word is fetched before the first check, through the constant address space
  // (scalar loads, all in flight together; the empty asm statements pin the order): nothing
  // here writes what they read before the kernel's last step (len[u]), or only 0 -> 1 (the flag).
  typedef const __attribute__((address_space(4))) int32_t* cptr;
  typedef const __attribute__((address_space(4))) int64_t* cptr8;
  const int32_t *flags_p = a.flags, *len_p = a.len + u, *cap_p = a.cap + u, *coff_p = a.chunk_off + u,
                *pol_p = a.policy + u;
  const int64_t* off_p = a.off + u;
  asm volatile("" ::"s"(flags_p), "s"(len_p), "s"(cap_p), "s"(coff_p), "s"(pol_p), "s"(off_p), "s"(a.part), "s"(a.out));
  const int overflow = *(cptr)(uintptr_t)flags_p;
  const int Lold = *(cptr)(uintptr_t)len_p, cap = *(cptr)(uintptr_t)cap_p, c_off = *(cptr)(uintptr_t)coff_p,
            pword = *(cptr)(uintptr_t)pol_p;
  const int64_t off = *(cptr8)(uintptr_t)off_p;
  asm volatile("" ::"s"(overflow), "s"(Lold), "s"(cap), "s"(c_off), "s"(pword), "s"(off));
  // policy word: id in the low byte, the policy's component mask (FG_COMP_*) above it
  const int policy = pword & 0xff, comp = pword >> 8;
  const bool freq = (comp & FG_COMP_FREQUENT) != 0;
  // the stability probe needs the cumulative scores and their top-k for every policy
  const bool probing = a.probe != nullptr;
  const bool scored = freq || probing;
  const int L = Lold + 1;
  if (overflow != 0 || L > cap) return;
  const int CH = a.chunk;                      // a power of two
  const int ch_shift = 31 - __builtin_clz(CH);
  const int nch = (L + CH - 1) >> ch_shift;
  // the new length goes to len[] and into every work-item record of the unit
  auto set_len = [&](int v) {
    if (tid == 0) a.len[u] = v;
    for (int i = tid; i < ((cap + CH - 1) >> ch_shift); i += 256) a.item_unit[(size_t)(c_off + i) * 8 + 3] = v;
  };
  const float* part = a.part + (size_t)c_off * G * (D + 2);

  // ---- merge the chunk partials of every query head:
  //      o = sum_c o_c 2^(M_c - M) / sum_c l_c 2^(M_c - M)
  float M = FG_NEG_BIG;   // of head 0 (the only one without grouping)
  for (int h = 0; h < G; ++h) {
    const float* ph = part + (size_t)h * (D + 2);
    const size_t cs = (size_t)G * (D + 2);  // stride between chunks
    // (max, sum) of the chunks: every wave does it for itself, one chunk per lane, so the loads
    // of all chunks are in flight together and no workgroup barrier is needed
    const int lane = tid & 63;
    float mc = FG_NEG_BIG, lc = 0.f;     // first chunk of this lane
    if (lane < nch) { mc = ph[lane * cs]; lc = ph[lane * cs + 1]; }
    float Mh = mc;
    for (int cix = lane + 64; cix < nch; cix += 64) Mh = fmaxf(Mh, ph[cix * cs]);
    Mh = fg_wave_max(Mh);
    float Lsum = lc * fg_exp2(mc - Mh);
    for (int cix = lane + 64; cix < nch; cix += 64) Lsum += ph[cix * cs + 1] * fg_exp2(ph[cix * cs] - Mh);
    Lsum = fg_group_sum<64>(Lsum);
    const float invh = 1.0f / Lsum;
    if (tid < D) {
      float o = 0.f;
#pragma unroll 4
      for (int cix = 0; cix < nch; ++cix) o += ph[cix * cs + 2 + tid] * fg_exp2(ph[cix * cs] - Mh);
      fg_store_out<ESIZE>(a.out, ((size_t)u * G + h) * D + tid, o * invh);
    }
    if (h == 0) M = Mh;
    if (GRP && tid == 0) s_M[h] = Mh;
  }
  // Score path in float64 (Sec. 3.4, cumulative attention score): this step's attention on held
  // slot j is a_j = 2^(x_j - M) / Z with the float64 logits x_j the attention kernel kept and
  // Z = sum_j 2^(x_j - M) summed here in float64 (M is only a shift: the merged float maximum).
  // Grouped heads: a_j summed over the query heads replaces head 0's logit in place, so that
  // the rest of the kernel reads one ready value per slot (each thread only touches its own slots).
  double inv_d = 0.0;   // 1 / Z of head 0 (the only one without grouping), set below where needed
  if (GRP) {
    __shared__ double s_invd[16];
    __syncthreads();
    if (scored) {
      for (int h = 0; h < G; ++h) {
        const double Mh = (double)s_M[h];
        double z = 0.0;
        for (int j = tid; j < L; j += 256) z += exp2(a.clogit[(off + j) * G + h] - Mh);
        z = fg_block_sum_f64(z, dred);
        if (tid == 0) s_invd[h] = 1.0 / z;
      }
      __syncthreads();
      for (int j = tid; j < L; j += 256) {
        double* lgj = a.clogit + (off + j) * G;
        double sum = 0.0;
        for (int h = 0; h < G; ++h) sum += exp2(lgj[h] - (double)s_M[h]) * s_invd[h];
        lgj[0] = sum;
      }
    }
  }

  if (policy >= 4 && !probing) {
    set_len(L);
    return;
  }
  const int p_new = a.n + a.step;
  double* score = a.cscore + off;
  const int32_t* pos = a.cpos + off;
  const uint8_t* cls = a.ccls + off;
  const int cmask = ((comp & FG_COMP_SPECIAL) ? FG_CLASS_SPECIAL : 0) | ((comp & FG_COMP_PUNCT) ? FG_CLASS_PUNCT : 0);
  const int wlo = (comp & FG_COMP_LOCAL) ? p_new - a.w : 0x7fffffff;  // positions above wlo are inside the window

  // Fast path (L <= 256 * NC): each thread keeps its slots' updated scores and a "protected"
  // bit (special / punctuation / window) in registers, so every later phase is register-only.
  // The code below is straight-line per slot, i.e. executed once per workgroup and bound by
  // instruction fetch: it is instantiated for a few sizes and the smallest one that fits is taken.
  auto update = [&](auto nc_tag) __attribute__((always_inline)) {
  constexpr int NC = decltype(nc_tag)::value;
  uint64_t kc[NC];
  uint32_t prot = 0;
  const bool small = L <= 256 * NC;
  fg_topk tk;
  tk.mode = 0; tk.thr = 0; tk.pthr = 0;
  if (small) {
    // all loads first (they are independent), then the arithmetic, then the stores
    double lg[NC];
    double sc[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      kc[i] = 0;
      lg[i] = 0.0;
      sc[i] = 0.0;
      if (j < L) {
        const int cb = cls[j];
        const int pj = pos[j];
        if ((cb & cmask) != 0 || pj > wlo) prot |= 1u << i;
        if (scored) {
          lg[i] = a.clogit[(off + j) * G];
          sc[i] = score[j];
        }
      }
    }
    if (scored) {
      if (!GRP) {
        // 2^(x_j - M) in place of the logits, their float64 sum over the workgroup
        double z = 0.0;
#pragma unroll
        for (int i = 0; i < NC; ++i) {
          const int j = tid + 256 * i;
          if (j < L) {
            lg[i] = exp2(lg[i] - (double)M);
            z += lg[i];
          }
        }
        inv_d = 1.0 / fg_block_sum_f64(z, dred);
      }
#pragma unroll
      for (int i = 0; i < NC; ++i) {
        const int j = tid + 256 * i;
        if (j < L) {
          // cumulative attention score += this step's attention (Sec. 3.4, frequency policy)
          const double v = sc[i] + (GRP ? lg[i] : lg[i] * inv_d);
          score[j] = v;
          kc[i] = (uint64_t)__double_as_longlong(v);
        }
      }
    }
    if (scored) {
      const int k_f = fg_budget(a.r_f, p_new + 1);
      __syncthreads();  // score[] is re-read by other threads only if the boundary value is tied
      // without the probe only the unprotected tokens' membership matters: try the lowest ones
      bool done = false;
      if (!probing && k_f > 0 && k_f < L && L <= 0xffff) done = fg_evict_cut_regs<NC>(kc, prot, L, k_f, dred, ired, &tk);
      if (!done)
        tk = fg_select_topk_regs<NC>(kc, [&](int j) { return score[j]; },
                                     [&](int j) { return (uint32_t)pos[j]; }, L, k_f, &sm);
    }
  } else if (scored) {
    if (!GRP) {
      double z = 0.0;
      for (int j = tid; j < L; j += 256) z += exp2(a.clogit[off + j] - (double)M);
      inv_d = 1.0 / fg_block_sum_f64(z, dred);
    }
    for (int j = tid; j < L; j += 256) {
      const double aj = GRP ? a.clogit[(off + j) * G] : exp2(a.clogit[off + j] - (double)M) * inv_d;
      score[j] += aj;
    }
    __syncthreads();
    const int k_f = fg_budget(a.r_f, p_new + 1);
    tk = fg_select_topk([&](int j) { return score[j]; }, [&](int j) { return (uint32_t)pos[j]; }, L, k_f, &sm);
  }
  if (probing) {
    // Stability probe (Sec. 4): mass of this step's attention row on every family member's
    // tokens among the held ones (frequent = the top-k just selected, local = last w positions)
    double r[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int j = tid; j < L; j += 256) {
      // the mean of the G heads' rows
      const double aj = GRP ? a.clogit[(off + j) * G] / (double)G
                            : exp2(a.clogit[off + j] - (double)M) * inv_d;
      const int c = cls[j];
      const bool top = fg_in_topk(tk, score[j], (uint32_t)pos[j]), recent = pos[j] > p_new - a.w;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int m = a.family[p];
        const bool in = ((m & FG_COMP_SPECIAL) && (c & FG_CLASS_SPECIAL)) || ((m & FG_COMP_PUNCT) && (c & FG_CLASS_PUNCT)) ||
                        ((m & FG_COMP_FREQUENT) && top) || ((m & FG_COMP_LOCAL) && recent);
        r[p] += in ? aj : 0.0;
      }
      r[4] += aj;
    }
#pragma unroll
    for (int p = 0; p < 5; ++p) {
      const double t = fg_block_sum_f64(r[p], dred);
      if (tid == 0) a.probe[(size_t)u * 5 + p] = t;
    }
    if (policy >= 4) {
      set_len(L);
      return;
    }
  }
  const bool tie_pos = (tk.mode == 2 && tk.pthr != 0xffffffffu);  // rare: boundary value shared
  auto kept = [&](int j) -> bool {  // from memory (large units and the tied case)
    bool k = (cls[j] & cmask) != 0 || pos[j] > wlo;
    if (freq) k = k || fg_in_topk(tk, score[j], (uint32_t)pos[j]);
    return k;
  };
  uint32_t keepbits = 0;  // fast path: bit i = slot tid + 256 i stays
  int mine = 0;
  if (small) {
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      if (j < L) {
        bool k = (prot >> i) & 1u;
        if (freq && !k) {
          if (tk.mode == 1) k = true;
          else if (tk.mode == 2) k = tie_pos ? fg_in_topk(tk, __longlong_as_double((long long)kc[i]), (uint32_t)pos[j])
                                             : (kc[i] >= tk.thr);
        }
        if (k) { keepbits |= 1u << i; ++mine; }
      }
    }
  } else {
    for (int j = tid; j < L; j += 256) mine += kept(j) ? 1 : 0;
  }
  const int new_len = fg_block_sum_i32(mine, ired);
  if (new_len == L) {
    set_len(L);
    return;
  }

  // ---- in-place release: i-th hole (evicted slot below new_len) <- i-th kept slot above it
  int* scratch = reinterpret_cast<int*>(a.clogit + off * G);  // logits are dead from here on (cap ints fit in cap doubles)
  __shared__ int s_move[2 * FG_MOVE_LDS];
  bool in_lds = false;
  __syncthreads();
  int run_h = 0, run_m = 0;
  if (small) {
    // any one-to-one pairing of holes and movers will do: number them thread by thread
    int nh = 0, nm = 0;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      if (j < L) {
        const bool k = (keepbits >> i) & 1u;
        nh += (j < new_len && !k) ? 1 : 0;
        nm += (j >= new_len && k) ? 1 : 0;
      }
    }
    // one scan for both counts (each below 2^16: L <= 256 * NC)
    int tot;
    const int at = fg_block_exscan_i32(nh | (nm << 16), ired, &tot);
    int at_h = at & 0xffff, at_m = at >> 16;
    run_h = tot & 0xffff;
    run_m = tot >> 16;
    // a step releases very few slots: the two lists then stay in shared memory
    in_lds = run_h <= FG_MOVE_LDS;
    int* holes = in_lds ? s_move : scratch;
    int* movers_end = in_lds ? s_move + 2 * FG_MOVE_LDS - 1 : scratch + cap - 1;  // filled downwards
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int j = tid + 256 * i;
      if (j < L) {
        const bool k = (keepbits >> i) & 1u;
        if (j < new_len && !k) holes[at_h++] = j;
        if (j >= new_len && k) *(movers_end - (at_m++)) = j;
      }
    }
    __syncthreads();
  } else {
    for (int base = 0; base < L; base += 256) {
      const int j = base + tid;
      int is_h = 0, is_m = 0;
      if (j < L) {
        const bool k = kept(j);
        is_h = (j < new_len && !k) ? 1 : 0;
        is_m = (j >= new_len && k) ? 1 : 0;
      }
      int tot_h, tot_m;
      const int ex_h = fg_block_exscan_i32(is_h, ired, &tot_h);
      __syncthreads();
      const int ex_m = fg_block_exscan_i32(is_m, ired, &tot_m);
      if (is_h) scratch[run_h + ex_h] = j;
      if (is_m) scratch[cap - 1 - (run_m + ex_m)] = j;
      run_h += tot_h;
      run_m += tot_m;
      __syncthreads();
    }
  }
  const int moves = run_h;  // == run_m
  char* ck = static_cast<char*>(a.ck) + off * RB;
  char* cv = static_cast<char*>(a.cv) + off * RB;
  // the kept() predicate of the large-unit path reads score/pos/cls from memory: there the
  // bookkeeping moves only after every thread is done with it
  if (!small) {
    for (int q = tid; q < moves * CPR; q += 256) {
      const int i = q / CPR, ch = q % CPR;
      const int dst = scratch[i], src = scratch[cap - 1 - i];
      *reinterpret_cast<u32x4*>(ck + (size_t)dst * RB + ch * 16) = *reinterpret_cast<const u32x4*>(ck + (size_t)src * RB + ch * 16);
      *reinterpret_cast<u32x4*>(cv + (size_t)dst * RB + ch * 16) = *reinterpret_cast<const u32x4*>(cv + (size_t)src * RB + ch * 16);
    }
    __syncthreads();
    for (int i = tid; i < moves; i += 256) {
      const int dst = scratch[i], src = scratch[cap - 1 - i];
      score[dst] = score[src];
      a.cpos[off + dst] = pos[src];
      a.ccls[off + dst] = cls[src];
    }
  } else {
    // rows and bookkeeping in one sweep: CPR lanes copy the row, one more moves score/pos/class
    for (int q = tid; q < moves * (CPR + 1); q += 256) {
      const int i = q / (CPR + 1), ch = q % (CPR + 1);
      const int dst = in_lds ? s_move[i] : scratch[i];
      const int src = in_lds ? s_move[2 * FG_MOVE_LDS - 1 - i] : scratch[cap - 1 - i];
      if (ch < CPR) {
        const u32x4 kr = *reinterpret_cast<const u32x4*>(ck + (size_t)src * RB + ch * 16);
        const u32x4 vr = *reinterpret_cast<const u32x4*>(cv + (size_t)src * RB + ch * 16);
        *reinterpret_cast<u32x4*>(ck + (size_t)dst * RB + ch * 16) = kr;
        *reinterpret_cast<u32x4*>(cv + (size_t)dst * RB + ch * 16) = vr;
      } else {
        const double sv = score[src];
        const int pv = pos[src];
        const uint8_t cb = cls[src];
        score[dst] = sv;
        a.cpos[off + dst] = pv;
        a.ccls[off + dst] = cb;
      }
    }
  }
  set_len(new_len);
  };
  if (L <= 256 * 2) update(std::integral_constant<int, 2>{});
  else if (L <= 256 * 4) update(std::integral_constant<int, 4>{});
  else if (L <= 256 * 8) update(std::integral_constant<int, 8>{});
  else if (L <= 256 * 12) update(std::integral_constant<int, 12>{});
  else if (L <= 256 * 16) update(std::integral_constant<int, 16>{});
  else if (L <= 256 * 20) update(std::integral_constant<int, 20>{});
  else update(std::integral_constant<int, 24>{});
}

}  // namespace

template <bool GRP, int CH>
static hipError_t launch_attn(const fg_decode_args& a, hipStream_t s) {
  const dim3 grid((unsigned)a.max_chunks), block(256);
  if (a.dtype == FG_BF16) {
    if (a.d == 128) hipLaunchKernelGGL((fg_decode_partial_kernel<2, 128, GRP, CH>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((fg_decode_partial_kernel<2, 64, GRP, CH>), grid, block, 0, s, a);
  } else {
    if (a.d == 128) hipLaunchKernelGGL((fg_decode_partial_kernel<4, 128, GRP, CH>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((fg_decode_partial_kernel<4, 64, GRP, CH>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

template <bool GRP>
static hipError_t launch_update(const fg_decode_args& a, hipStream_t s) {
  const dim3 grid((unsigned)a.U), block(256);
  if (a.dtype == FG_BF16) {
    if (a.d == 128) hipLaunchKernelGGL((fg_decode_finish_kernel<2, 128, GRP>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((fg_decode_finish_kernel<2, 64, GRP>), grid, block, 0, s, a);
  } else {
    if (a.d == 128) hipLaunchKernelGGL((fg_decode_finish_kernel<4, 128, GRP>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((fg_decode_finish_kernel<4, 64, GRP>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

hipError_t fg_launch_decode_attn(const fg_decode_args& a, hipStream_t s) {
  if (a.chunk == 128) return a.G > 1 ? launch_attn<true, 128>(a, s) : launch_attn<false, 128>(a, s);
  return a.G > 1 ? launch_attn<true, 256>(a, s) : launch_attn<false, 256>(a, s);
}

hipError_t fg_launch_decode_update(const fg_decode_args& a, hipStream_t s) {
  return a.G > 1 ? launch_update<true>(a, s) : launch_update<false>(a, s);
}
