// Prompt-time attention profiling on the bf16 matrix cores (Alg. 1: A = softmax(Q K^T);
// Sec. 3.4: cumulative attention score per token; Sec. 3.3 Eq. 1: recovery of a policy).
//
// The attention map is never stored. Two sweeps over the causal half of Q K^T:
//   PASS 1  row statistics         m_i = max_{j<=i} c * q_i.k_j,   l_i = sum_{j<=i} 2^(c * q_i.k_j - m_i),
//                                  c = scale*log2(e); stored as the pair (m_i, 1/l_i)
//   PASS 2  column reductions      colsum_j  = sum_{i>=j}            2^(c * q_i.k_j - m_i) / l_i
//                                  bandcol_j = sum_{i=j}^{j+w-1}     (same terms)
// (The pair instead of one log-sum-exp value: a float holds m_i + log2 l_i, a number around
// 10..30, only to about 2e-6, which would be a relative error of 1e-6 in every element of the
// row; m_i is exact and 1/l_i is good to 6e-8. The shift costs nothing: the accumulation
// s += p becomes one fused multiply-add s += p~ * (1/l_i).)
// colsum is the "cumulative sum of attention score" of token j (frequent policy and every
// static policy's recovery); bandcol is what the local policy recovers of column j.
//
// Both sweeps use one structure. A workgroup of 4 waves owns 256 consecutive "owner" items
// (query rows in pass 1, key columns in pass 2), 64 per wave, held in registers as the B
// operand of v_mfma_f32_32x32x16_bf16 so that the owner index is the lane index (n = lane%32).
// The other matrix is streamed in tiles of 32 items through double-buffered LDS and read as
// the A operand. Each lane therefore keeps its owner's running statistics privately:
// (max, sum) of its row in pass 1, the column sums in pass 2, and only the two half-waves
// are merged at the end. Reductions run in a fixed order: results are deterministic.
#include "fg_common.h"
#include "fg_internal.h"

namespace {

constexpr int kOwnPerWave = 64;
constexpr int kOwnPerBlock = 256;
constexpr int kTile = 32;

template <int D>
struct Lds {
  static constexpr int kRowBytes = D * 2 + 16;  // +16: consecutive rows land on different banks
  static constexpr int kTileBytes = kTile * kRowBytes;
};

template <int D, int PASS>
__global__ __launch_bounds__(256, 3) void fg_profile_mfma_kernel(
    const __bf16* __restrict__ Q, const __bf16* __restrict__ K, float2* __restrict__ rowstat,
    double* __restrict__ colsum, double* __restrict__ bandcol, int U, int n, int w, float c,
    int nblk, int G) {
  constexpr int KK = D / 16;
  constexpr int RS = Lds<D>::kRowBytes;
  constexpr int CHUNKS_PER_ROW = D / 8;                    // 16-byte chunks per item
  constexpr int LOADS = (kTile * CHUNKS_PER_ROW) / 256;    // per thread per tile (2 or 1)
  static_assert(LOADS >= 1, "tile too small");

  __shared__ __attribute__((aligned(16))) unsigned char tile_lds[2][Lds<D>::kTileBytes];
  __shared__ __attribute__((aligned(16))) float stat_lds[2][kTile * 2];  // [buffer][row][m, 1/l]

  // ---- which (unit, owner block): units of one XCD walk one unit's blocks back to back
  const int idx = blockIdx.x;
  const int xcd = idx & 7, rest = idx >> 3;
  const int npair = (nblk + 1) / 2;
  const int pair_ord = rest % npair;
  const int unit = (rest / npair) * 8 + xcd;
  if (unit >= U) return;
  // A workgroup takes two owner blocks of the unit, the pair_ord-th heaviest and the
  // pair_ord-th lightest one: every workgroup of a unit then has the same amount of work and
  // the start-up of a workgroup is paid once per pair.
  for (int half = 0; half < 2; ++half) {
  const int blk_ord = half == 0 ? pair_ord : nblk - 1 - pair_ord;
  if (half == 1 && blk_ord == pair_ord) break;  // the middle block of an odd count is alone
  const int blk = (PASS == 1) ? (nblk - 1 - blk_ord) : blk_ord;  // heaviest first

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it scalar
  const int ln = lane & 31, lh = lane >> 5;
  // G query heads share a K/V unit. Sweep 1 runs per query head (U counts query heads, unit =
  // u * G + g) against the keys of u; sweep 2 runs per K/V unit and streams the query rows of
  // its G heads one after the other (heads are contiguous: one buffer covers them all).
  const size_t mat = (size_t)n * D;
  const __bf16* own_mat = (PASS == 1 ? Q : K) + (size_t)unit * mat;
  const __bf16* str_mat = (PASS == 1) ? K + (size_t)(unit / G) * mat : Q + (size_t)unit * G * mat;
  const float2* stat_row = rowstat + (size_t)unit * (PASS == 1 ? 1 : G) * n;
  const int heads = (PASS == 1) ? 1 : G;

  const int WG0 = blk * kOwnPerBlock;       // first owner item of the workgroup
  const int O0 = WG0 + wave * kOwnPerWave;  // first owner item of the wave

  // ---- owner fragments (B operand): item O0 + 32 f + ln, k-chunk lh*8 + 16 kk
  bf16x8 own[2][KK];
#pragma unroll
  for (int f = 0; f < 2; ++f) {
    // items past the end are clamped to the last one: their results are never stored
    const int item = min(O0 + 32 * f + ln, n - 1);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(own_mat + (size_t)item * D + lh * 8 + 16 * kk);
      own[f][kk] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- streamed tile range
  int t_begin, t_end;  // in tiles of 32
  if (PASS == 1) {
    t_begin = 0;
    t_end = (min(n, WG0 + kOwnPerBlock) + kTile - 1) / kTile;
  } else {
    t_begin = WG0 / kTile;
    t_end = (n + kTile - 1) / kTile;
  }

  // Streamed tiles come through raw buffer loads: the tile offset is a scalar and rows past the
  // end of the unit read as zeros (every use of them is masked), so a load costs no vector-ALU
  // instruction. In the first sweep at head dimension 128 the loads write straight into LDS (no
  // staging registers, no LDS store instructions): a wave brings eight of the tile's 32 rows,
  // one 256-byte row per instruction (a dword per lane), so that every row lands at its padded
  // position. (Measured: about 3.5 % off the first sweep; the second sweep, which also streams
  // the row statistics, did not gain from it and keeps the register staging.)
  constexpr bool DMA = (D == 128) && (PASS == 1);
  typedef __attribute__((address_space(3))) void* lds_ptr;
  const __amdgpu_buffer_rsrc_t str_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(str_mat), 0, heads * n * D * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t stat_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float2*>(stat_row), 0, heads * n * 8, 0x00020000);
  int voff[LOADS];
#pragma unroll
  for (int r = 0; r < LOADS; ++r) {
    const int q = tid + 256 * r;
    voff[r] = (q / CHUNKS_PER_ROW) * (D * 2) + (q % CHUNKS_PER_ROW) * 16;
  }
  const int voff_stat = (tid & (kTile - 1)) * 8;
  u32x4 stage[LOADS];
  float2 stage_stat = make_float2(0.f, 0.f);
  // `row0` = first streamed row of the tile counted over all heads (head * n + t * 32); a tile
  // that runs past its head's last row reads the next head's rows (or zeros after the last
  // head): those rows are masked wherever they are used. `buf` is the LDS buffer the tile is for.
  auto gload = [&](int row0, int buf) {
    if (DMA) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int row = wave * 8 + r;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(str_rsrc, (lds_ptr)&tile_lds[buf][row * RS], 4, lane * 4,
                                                 (row0 + row) * (D * 2), 0, 0);
      }
      return;
    }
#pragma unroll
    for (int r = 0; r < LOADS; ++r)
      stage[r] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(str_rsrc, voff[r], row0 * (D * 2), 0));
    if (PASS == 2) stage_stat = __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(stat_rsrc, voff_stat, row0 * 8, 0));
  };
  auto lstore = [&](int buf) {
    if (DMA) return;   // the loads have written LDS themselves; the barrier that follows waits for them
#pragma unroll
    for (int r = 0; r < LOADS; ++r) {
      const int q = tid + 256 * r;
      const int item = q / CHUNKS_PER_ROW, ch = q % CHUNKS_PER_ROW;
      *reinterpret_cast<u32x4*>(&tile_lds[buf][item * RS + ch * 16]) = stage[r];
    }
    if (PASS == 2 && tid < kTile) *reinterpret_cast<float2*>(&stat_lds[buf][tid * 2]) = stage_stat;
  };

  // ---- per-lane running statistics
  float m_run[2] = {FG_NEG_BIG, FG_NEG_BIG};                         // pass 1
  double l_run[2] = {0.0, 0.0};
  double col_acc[2] = {0.0, 0.0}, band_acc[2] = {0.0, 0.0};          // pass 2

  // Sweep 1 walks its tiles upwards. Sweep 2 walks the query rows downwards from the end of
  // the prompt: every owner block of a unit then starts at the same tile and the blocks move
  // in step, so a streamed tile is fetched into the XCD's L2 once per unit instead of once per
  // block (walking upwards, block b reads a tile 8 steps after block b - 1 and six units per
  // XCD outgrow the 4 MB L2: 3.5x the algorithmic bytes were fetched at n = 8192).
  const int nt = t_end - t_begin;     // tiles per head
  const int n_it = nt * heads;
  if (n_it > 0) {
    gload((PASS == 2 ? t_end - 1 : t_begin) * kTile, 0);
    lstore(0);
  }
  __syncthreads();

  int t = (PASS == 2) ? t_end - 1 : t_begin, head_row0 = 0;   // current tile and first row of the current head
  for (int it = 0; it < n_it; ++it) {
    const int buf = it & 1;
    const int t0 = t * kTile;
    // next tile: the following one of this head, else the first one of the next head
    int t_next = t + 1, head_next = head_row0;
    if (PASS == 2) {
      t_next = t - 1;
      if (t_next < t_begin) { t_next = t_end - 1; head_next += n; }
    } else if (t_next == t_end) { t_next = t_begin; head_next += n; }
    // unconditional (the load count per iteration is static); the last iteration re-reads its own tile
    gload(it + 1 < n_it ? head_next + t_next * kTile : head_row0 + t0, buf ^ 1);

    // what this wave has to do with the tile, per owner fragment
    bool need[2];
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      const int Of = O0 + 32 * f;
      if (PASS == 1) need[f] = (Of < n) && (t0 <= Of + 31);
      else need[f] = (Of < n) && (t0 + 31 >= Of);
    }

    if (need[0] || need[1]) {  // scalar branch: `wave` is uniform
      f32x16 acc[2];
#pragma unroll
      for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[f][i] = 0.f;
      const unsigned char* a_ptr = &tile_lds[buf][ln * RS + lh * 16];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_ptr + kk * 32);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, own[0][kk], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, own[1][kk], acc[1], 0, 0, 0);
      }

      const int sbase = t0 + lh * 4;  // streamed index of acc[i] = sbase + (i>>2)*8 + (i&3)

      if (PASS == 1) {
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          if (!need[f]) continue;
          const int Of = O0 + 32 * f;
          const int row = Of + ln;
          if (t0 + 31 <= Of) {  // every column of the tile is visible to every row
            // 16 values -> 8 three-operand maxima (c > 0: the max of the raw dot products is enough)
            const f32x16& ac = acc[f];
            const float x0 = fmaxf(fmaxf(ac[0], ac[1]), ac[2]), x1 = fmaxf(fmaxf(ac[3], ac[4]), ac[5]);
            const float x2 = fmaxf(fmaxf(ac[6], ac[7]), ac[8]), x3 = fmaxf(fmaxf(ac[9], ac[10]), ac[11]);
            const float x4 = fmaxf(fmaxf(ac[12], ac[13]), ac[14]);
            const float y0 = fmaxf(fmaxf(x0, x1), x2), y1 = fmaxf(fmaxf(x3, x4), ac[15]);
            const float m_new = fmaxf(fmaxf(y0, y1) * c, m_run[f]);
            float s = fg_exp2(fmaf(acc[f][0], c, -m_new));
#pragma unroll
            for (int i = 1; i < 16; ++i) s += fg_exp2(fmaf(acc[f][i], c, -m_new));
            l_run[f] = l_run[f] * (double)fg_exp2(m_run[f] - m_new) + (double)s;
            m_run[f] = m_new;
          } else {  // diagonal tile: causal mask col <= row
            const int lim = row - sbase;  // valid iff (i>>2)*8 + (i&3) <= lim
            float tmax = FG_NEG_BIG;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const bool ok = ((i >> 2) * 8 + (i & 3)) <= lim;
              tmax = fmaxf(tmax, ok ? acc[f][i] * c : FG_NEG_BIG);
            }
            const float m_new = fmaxf(m_run[f], tmax);
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const bool ok = ((i >> 2) * 8 + (i & 3)) <= lim;
              const float p = fg_exp2(fmaf(acc[f][i], c, -m_new));
              s += ok ? p : 0.f;
            }
            l_run[f] = l_run[f] * (double)fg_exp2(m_run[f] - m_new) + (double)s;
            m_run[f] = m_new;
          }
        }
      } else {
        // (m, 1/l) of the 16 streamed rows this lane sees
        float ms[16], il[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 v = *reinterpret_cast<const f32x4*>(&stat_lds[buf][(g * 8 + lh * 4) * 2]);      // m0 i0 m1 i1
          const f32x4 u = *reinterpret_cast<const f32x4*>(&stat_lds[buf][(g * 8 + lh * 4) * 2 + 4]);  // m2 i2 m3 i3
          ms[g * 4 + 0] = v[0]; ms[g * 4 + 1] = v[2]; ms[g * 4 + 2] = u[0]; ms[g * 4 + 3] = u[2];
          il[g * 4 + 0] = v[1]; il[g * 4 + 1] = v[3]; il[g * 4 + 2] = u[1]; il[g * 4 + 3] = u[3];
        }
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          if (!need[f]) continue;
          const int Cf = O0 + 32 * f;
          const int col = Cf + ln;
          const bool full = (t0 >= Cf + 31) && (t0 + 31 < n);
          const bool inside = (t0 + 31 - Cf) < w;   // every element within the local band
          const bool outside = (t0 - (Cf + 31)) >= w;
          if (full && (inside || outside)) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) s = fmaf(fg_exp2(fmaf(acc[f][i], c, -ms[i])), il[i], s);
            col_acc[f] += (double)s;
            if (inside) band_acc[f] += (double)s;  // the whole tile lies in the local band
          } else if (full) {
            // the band's edge crosses the tile (nothing else to mask): the total needs no
            // mask, the band sum takes the terms with row - col < w
            const int blim = w - (sbase - col);   // row - col < w  iff  (i>>2)*8 + (i&3) < blim
            float s = 0.f, sb = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const float e = fg_exp2(fmaf(acc[f][i], c, -ms[i]));
              s = fmaf(e, il[i], s);
              sb = fmaf(e, ((i >> 2) * 8 + (i & 3)) < blim ? il[i] : 0.f, sb);
            }
            col_acc[f] += (double)s;
            band_acc[f] += (double)sb;
          } else if (inside) {
            // diagonal and / or last tile, wholly within the band: one mask, band sum = total
            const int dbase = sbase - col;
            const int rlim = n - sbase;
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int o = (i >> 2) * 8 + (i & 3);
              const bool ok = (dbase + o >= 0) && (o < rlim);
              const float e = fg_exp2(fmaf(acc[f][i], c, -ms[i]));   // may be huge where masked: select, do not scale
              s = fmaf(ok ? e : 0.f, il[i], s);
            }
            col_acc[f] += (double)s;
            band_acc[f] += (double)s;
          } else {
            const int dbase = sbase - col;        // row - col = dbase + (i>>2)*8 + (i&3)
            const int rlim = n - sbase;           // row < n  iff  (i>>2)*8 + (i&3) < rlim
            float s = 0.f, sb = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int o = (i >> 2) * 8 + (i & 3);
              const int dist = dbase + o;
              const bool ok = (dist >= 0) && (o < rlim);
              const float p = fg_exp2(fmaf(acc[f][i], c, -ms[i])) * il[i];
              s += ok ? p : 0.f;
              sb += (ok && dist < w) ? p : 0.f;
            }
            col_acc[f] += (double)s;
            band_acc[f] += (double)sb;
          }
        }
      }
    }

    lstore(buf ^ 1);
    __syncthreads();
    t = t_next;
    head_row0 = head_next;
  }

  // ---- merge the two half-waves and store
  if (PASS == 1) {
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      const float m_o = __shfl_xor(m_run[f], 32, 64);
      const double l_o = fg_shfl_xor_f64(l_run[f], 32);
      const float M = fmaxf(m_run[f], m_o);
      const double L = l_run[f] * (double)fg_exp2(m_run[f] - M) + l_o * (double)fg_exp2(m_o - M);
      const int row = O0 + 32 * f + ln;
      if (lh == 0 && row < n) rowstat[(size_t)unit * n + row] = make_float2(M, (float)(1.0 / L));
    }
  } else {
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      const double cs = col_acc[f] + fg_shfl_xor_f64(col_acc[f], 32);
      const double bs = band_acc[f] + fg_shfl_xor_f64(band_acc[f], 32);
      const int col = O0 + 32 * f + ln;
      if (lh == 0 && col < n) {
        colsum[(size_t)unit * n + col] = cs;
        bandcol[(size_t)unit * n + col] = bs;
      }
    }
  }
  __syncthreads();  // the tile buffers are reused by the second block
  }
}

template <int D>
hipError_t launch(const fg_profile_args& a, int pass, hipStream_t s) {
  const int nblk = (a.n + kOwnPerBlock - 1) / kOwnPerBlock;
  const int units = (pass == 1) ? a.U * a.G : a.U;  // sweep 1: one unit per query head
  const int ugroups = (units + 7) / 8;
  const dim3 grid((unsigned)(8 * ((nblk + 1) / 2) * ugroups)), block(256);
  const float c = a.scale * FG_LOG2E;
  const __bf16* Q = static_cast<const __bf16*>(a.Q);
  const __bf16* K = static_cast<const __bf16*>(a.K);
  if (pass == 1)
    hipLaunchKernelGGL((fg_profile_mfma_kernel<D, 1>), grid, block, 0, s, Q, K, a.rowstat, a.colsum,
                       a.bandcol, units, a.n, a.w, c, nblk, a.G);
  else
    hipLaunchKernelGGL((fg_profile_mfma_kernel<D, 2>), grid, block, 0, s, Q, K, a.rowstat, a.colsum,
                       a.bandcol, units, a.n, a.w, c, nblk, a.G);
  return hipGetLastError();
}

}  // namespace

hipError_t fg_launch_profile_bf16(const fg_profile_args& a, int pass, hipStream_t s) {
  if (a.d == 128) return launch<128>(a, pass, s);
  return launch<64>(a, pass, s);
}
