// Double-precision variants of the N = 2^16 pass bodies of ntt16.hip.h, for primes q < 2^50.
// On gfx950 the vector FP64 units run at full rate, and a modular multiply by a constant is 6 FP64
// instructions (against ~23 integer instructions for the 64-bit Shoup form), exact because every value is an
// integer below 2^53. Same tiles, lane layouts and LDS transposes as the integer bodies.
//
// Twiddles are single doubles (the quotient estimate uses the rounded product and 1/q, so no companion constant
// is stored). Ranges (in units of q): a multiply returns at most (0.5 + 0.375 |y|) q, so a radix-16 round of four
// forward stages takes |x| <= 1 to |x| <= 7.0 < 8; values are brought back to |x| <= 0.5 after every round. Inverse rounds double the
// sums, so they are brought back after every two stages. Between the two passes of a transform the data lives in
// global memory as reduced doubles.
#pragma once
#include "ntt16.hip.h"

template <class TW>
__device__ __forceinline__ void radix16_fwd_fp(double (&x)[16], double q, double qinv, TW tw) {
#pragma unroll
  for (int s = 0; s < 4; s++) {
    const int half = 8 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      const double w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) {
        double& X = x[g * 2 * half + p];
        double& Y = x[g * 2 * half + p + half];
        const double T = fp_mulmod_var(Y, w, qinv, q);
        Y = X - T;
        X = X + T;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = fp_reduce(x[i], qinv, q);
}
template <class TW>
__device__ __forceinline__ void radix16_inv_fp(double (&x)[16], double q, double qinv, TW tw) {
#pragma unroll
  for (int s = 3; s >= 0; s--) {
    const int half = 8 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      const double w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) {
        double& X = x[g * 2 * half + p];
        double& Y = x[g * 2 * half + p + half];
        const double D = X - Y;
        X = X + Y;
        Y = fp_mulmod_var(D, w, qinv, q);
      }
    }
    if (s == 2 || s == 0) {
#pragma unroll
      for (int i = 0; i < 16; i++) x[i] = fp_reduce(x[i], qinv, q);
    }
  }
}

// Forward, stages 0..7. `x` holds integers of magnitude at most q (residues as doubles) in the row layout of
// ntt16_fwd_rows_loaded; dst receives reduced doubles.
__device__ __forceinline__ void ntt16_fwd_rows_fp_loaded(double (&x)[16], double* __restrict__ dst,
                                                         const double* __restrict__ tw, double q, double qinv, u32 tile,
                                                         double* sm) {
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
  const u32 i0 = r0;
  double twb[15];  // second-round twiddles, requested before the first round
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twb[(1 << s) - 1 + g] = tw[(16 << s) + (i0 << s) + g];
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return tw[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[i * 256 + t] = x[i];
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[(i0 * 16 + j) * 16 + col];
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return twb[(1 << s) - 1 + g]; });
#pragma unroll
  for (int j = 0; j < 16; j++) dst[(size_t)(i0 * 16 + j) * 256 + col0 + col] = x[j];
}
// The same from canonical residues (uint64) in memory.
__device__ __forceinline__ void ntt16_fwd_rows_fp(const u64* __restrict__ src, double* __restrict__ dst,
                                                  const double* __restrict__ tw, double q, double qinv, u32 tile, double* sm) {
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
  double x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = u2d(src[(size_t)(i * 16 + r0) * 256 + col0 + col]);
  ntt16_fwd_rows_fp_loaded(x, dst, tw, q, qinv, tile, sm);
}

// Forward, stages 8..15 on reduced doubles. Leaves x (|x| <= q/2) in the i-layout of ntt16_fwd_blocks.
// `x` must already hold the tile in the i-layout (lane (hb, j0) holds positions i*16 + j0 of block h).
// `between` runs after the first round (its twiddles are dead by then), e.g. to request data the caller needs
// after the transform.
template <class BETWEEN>
__device__ __forceinline__ void ntt16_fwd_blocks_fp_loaded(double (&x)[16], const double* __restrict__ tw, double q,
                                                           double qinv, u32 tile, double* sm, BETWEEN between) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u32 i0 = j0;
  // the second round's 15 twiddles are requested up front so they arrive during the first round
  double twb[15];
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twb[(1 << s) - 1 + g] = tw[(4096 << s) + (h << (4 + s)) + (i0 << s) + g];
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return tw[(256 << s) + (h << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[hb * 272 + i * 17 + j0] = x[i];
  between();
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[hb * 272 + i0 * 17 + j];
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return twb[(1 << s) - 1 + g]; });
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[hb * 272 + i0 * 17 + j] = x[j];
  wave_lds_sync();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[hb * 272 + i * 17 + j0];
}
__device__ __forceinline__ void ntt16_fwd_blocks_fp_loaded(double (&x)[16], const double* __restrict__ tw, double q,
                                                           double qinv, u32 tile, double* sm) {
  ntt16_fwd_blocks_fp_loaded(x, tw, q, qinv, tile, sm, [] {});
}

// The same block pass with its 16 x 16 transposes done in two halves, low words then high words, through a tile of
// 4-byte words (16 groups x 272 words = 17 KB instead of 34 KB): a kernel that wants the rest of its LDS share for
// something else (the prefetched input tiles of ntt16_fwd_blocks_inner_c_kernel) uses this one. `ex` is the
// workgroup's word tile; exchanges stay inside 16-lane groups, so waiting for the wave's own LDS operations orders them.
__device__ __forceinline__ void fp_transpose16_words(double (&x)[16], u32* row_major, u32 wr_stride, u32 wr_lane,
                                                     u32 rd_stride, u32 rd_lane) {
  u32 lo[16], hi[16];
#pragma unroll
  for (int i = 0; i < 16; i++) row_major[i * wr_stride + wr_lane] = (u32)__double2loint(x[i]);
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) lo[j] = row_major[j * rd_stride + rd_lane];
  wave_lds_sync();
#pragma unroll
  for (int i = 0; i < 16; i++) row_major[i * wr_stride + wr_lane] = (u32)__double2hiint(x[i]);
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) hi[j] = row_major[j * rd_stride + rd_lane];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = __hiloint2double((int)hi[j], (int)lo[j]);
}
// `loaded` runs once the loads of all 30 twiddles have been issued and before anything waits for them: memory
// requests a caller starts there are younger than every load the two rounds wait for, so those waits leave them in
// flight. `between` runs after the first round.
// The first round's 15 twiddles are the same for the 16 lanes of a group and for every tile the workgroup transforms:
// `twl` holds them in LDS (group hb at twl + hb * NTT16_TWL_PITCH, filled by ntt16_fwd_blocks_fp_words_twl), so a
// transform starts on a short LDS read instead of a trip to the L2.
#define NTT16_TWL_PITCH 18
// Filling it is split in two so that a caller can put other work between the request and the use of the value:
// wave w fills the rows of its own four groups, lane L < 60 moving twiddle L % 15 of group 4w + L / 15.
__device__ __forceinline__ double ntt16_twl_fetch(const double* __restrict__ tw, u32 tile) {
  const u32 t = threadIdx.x, L = min(t & 63, 59u);
  const u32 hb = (t >> 6) * 4 + L / 15, k = L % 15, h = tile * 16 + hb;
  const u32 s = k >= 7 ? 3 : k >= 3 ? 2 : k >= 1 ? 1 : 0, g = k + 1 - (1u << s);
  return tw[(256 << s) + (h << s) + g];
}
__device__ __forceinline__ void ntt16_twl_store(double v, double* twl) {
  const u32 t = threadIdx.x, L = t & 63;
  if (L < 60) twl[((t >> 6) * 4 + L / 15) * NTT16_TWL_PITCH + L % 15] = v;
}
template <class LOADED, class BETWEEN>
__device__ __forceinline__ void ntt16_fwd_blocks_fp_words(double (&x)[16], const double* __restrict__ tw, double q,
                                                          double qinv, u32 tile, u32* ex, const double* twl, LOADED loaded,
                                                          BETWEEN between) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u32 i0 = j0;
  u32* grp = ex + hb * 272;
  double twa[15], twb[15];
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twb[(1 << s) - 1 + g] = tw[(4096 << s) + (h << (4 + s)) + (i0 << s) + g];
#pragma unroll
  for (int k = 0; k < 15; k++) twa[k] = twl[hb * NTT16_TWL_PITCH + k];
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  loaded();
  __builtin_amdgcn_sched_barrier(0);
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return twa[(1 << s) - 1 + g]; });
  // element (i, j0) -> lane i0 = i holds (i0, j): written at i*17 + j0, read at i0*17 + j
  fp_transpose16_words(x, grp, 17, j0, 1, i0 * 17);
  between();
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return twb[(1 << s) - 1 + g]; });
  // and back: written at i0*17 + j, read at i*17 + j0
  fp_transpose16_words(x, grp, 1, i0 * 17, 17, j0);
}

// Inverse, stages 15..8. In: x = canonical residues as doubles, i-layout. Out: reduced doubles, i-layout.
__device__ __forceinline__ void ntt16_inv_blocks_fp(double (&x)[16], const double* __restrict__ twi, double q, double qinv,
                                                    u32 tile, double* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u32 i0 = j0;
  double twa[15], twb[15];  // both rounds' twiddles, requested before the first transpose
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      twa[(1 << s) - 1 + g] = twi[(4096 << s) + (h << (4 + s)) + (i0 << s) + g];
      twb[(1 << s) - 1 + g] = twi[(256 << s) + (h << s) + g];
    }
#pragma unroll
  for (int i = 0; i < 16; i++) sm[hb * 272 + i * 17 + j0] = x[i];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[hb * 272 + i0 * 17 + j];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twa[(1 << s) - 1 + g]; });
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[hb * 272 + i0 * 17 + j] = x[j];
  wave_lds_sync();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[hb * 272 + i * 17 + j0];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twb[(1 << s) - 1 + g]; });
}

// Inverse, stages 7..0, then multiplication by (sc, sc/q); x receives canonical residues (uint64), row layout.
__device__ __forceinline__ void ntt16_inv_rows_fp(u64 (&out)[16], const double* __restrict__ src, const double* __restrict__ twi,
                                                  double q, double qinv, double sc, double scq, u32 tile, double* sm) {
  const u32 t = threadIdx.x, col = t & 15, i0 = t >> 4, col0 = tile * 16;
  double x[16];
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = src[(size_t)(i0 * 16 + j) * 256 + col0 + col];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twi[(16 << s) + (i0 << s) + g]; });
#pragma unroll
  for (int j = 0; j < 16; j++) sm[(i0 * 16 + j) * 16 + col] = x[j];
  lds_barrier();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[i * 256 + t];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twi[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) out[i] = d2u_canon(fp_mulmod_const(x[i], sc, scq, q), q);
}

__device__ __forceinline__ void ntt16_fwd_blocks_fp(double (&x)[16], const double* __restrict__ src,
                                                    const double* __restrict__ tw, double q, double qinv, u32 tile, double* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, h = tile * 16 + (t >> 4);
  const double* blk = src + (size_t)h * 256;
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = blk[i * 16 + j0];
  ntt16_fwd_blocks_fp_loaded(x, tw, q, qinv, tile, sm);
}

// ---- block pass with 8 values per lane (used where a kernel needs the registers for something else) ----
// One 256-element block is transformed by 32 adjacent lanes: radix-8 on stages 8..10, exchange, radix-8 on stages
// 11..13, exchange, radix-4 on stages 14..15; the exchanges go through the block's own LDS rows (pitch 35 doubles per
// 32 elements: near conflict-free for all three access patterns) and stay inside the half-wave, so no workgroup
// barrier. In: x[i] = element i*32 + l of block h (l = lane & 31), |x| <= q/2. Out: x[c] = element
// (l >> 2)*32 + (l & 3)*8 + c, i.e. 8 consecutive elements per lane, |x| <= q/2. Ranges: reduced after the first
// round; the following five stages take |x| <= 0.5 q to at most 7.7 q < 2^53 / q.
#define NTT8_PITCH 35
#define NTT8_BLOCK_LDS (8 * NTT8_PITCH)

template <class TW>
__device__ __forceinline__ void radix8_fwd_fp(double (&x)[8], double q, double qinv, TW tw) {
#pragma unroll
  for (int s = 0; s < 3; s++) {
    const int half = 4 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      const double w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) {
        double& X = x[g * 2 * half + p];
        double& Y = x[g * 2 * half + p + half];
        const double T = fp_mulmod_var(Y, w, qinv, q);
        Y = X - T;
        X = X + T;
      }
    }
  }
}

template <class BETWEEN>
__device__ __forceinline__ void ntt256_fwd_blocks_fp8(double (&x)[8], const double* __restrict__ tw, double q, double qinv,
                                                      u32 h, u32 l, double* smb, BETWEEN between) {
  const u32 a = l >> 2, b = l & 3;
  // the twiddles of the second and third round are requested up front so they arrive during the first
  double t2[7], t3[6];
#pragma unroll
  for (int s = 0; s < 3; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) t2[(1 << s) - 1 + g] = tw[(2048 << s) + (h << (3 + s)) + (a << s) + g];
#pragma unroll
  for (int u = 0; u < 2; u++) t3[u] = tw[16384 + (h << 6) + (a << 3) + (b << 1) + u];
#pragma unroll
  for (int k = 0; k < 4; k++) t3[2 + k] = tw[32768 + (h << 7) + (a << 4) + (b << 2) + k];
  radix8_fwd_fp(x, q, qinv, [&](int s, int g) { return tw[(256 << s) + (h << s) + g]; });
#pragma unroll
  for (int i = 0; i < 8; i++) smb[i * NTT8_PITCH + l] = fp_reduce(x[i], qinv, q);
  between();
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < 8; r++) x[r] = smb[a * NTT8_PITCH + r * 4 + b];
  radix8_fwd_fp(x, q, qinv, [&](int s, int g) { return t2[(1 << s) - 1 + g]; });
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < 8; r++) smb[a * NTT8_PITCH + r * 4 + b] = x[r];
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 8; c++) x[c] = smb[a * NTT8_PITCH + b * 8 + c];
  // stage 14: pairs (c, c + 2) inside each half; stage 15: pairs (2k, 2k + 1)
#pragma unroll
  for (int u = 0; u < 2; u++)
#pragma unroll
    for (int p = 0; p < 2; p++) {
      double& X = x[u * 4 + p];
      double& Y = x[u * 4 + p + 2];
      const double T = fp_mulmod_var(Y, t3[u], qinv, q);
      Y = X - T;
      X = X + T;
    }
#pragma unroll
  for (int k = 0; k < 4; k++) {
    double& X = x[2 * k];
    double& Y = x[2 * k + 1];
    const double T = fp_mulmod_var(Y, t3[2 + k], qinv, q);
    Y = X - T;
    X = X + T;
  }
#pragma unroll
  for (int c = 0; c < 8; c++) x[c] = fp_reduce(x[c], qinv, q);
}
