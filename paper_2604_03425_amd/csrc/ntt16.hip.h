// Two-pass negacyclic NTT for N = 2^16 on gfx950: each pass does 8 butterfly stages on a 4096-element
// tile held as 16 registers per lane (256 lanes), as two in-register radix-16 rounds with one LDS
// transpose between them. Pass "row" works on 256 rows x 16 adjacent columns of the 256x256 view of a
// limb (stride-256 butterflies, stages 0..7); pass "blk" works on 16 contiguous 256-element blocks
// (stages 8..15). Global loads and stores always have 16 adjacent lanes on 128 contiguous bytes.
//
// Lazy ranges. Every twiddle product is the approximate shoup_lazy4 (below 4q), and the lazy constant the bodies
// pass around is 4q. SMALL primes (q < 2^52): forward butterflies never correct, values grow by 4q per
// stage (< 65q < 2^59 after 16 stages from canonical input) and are reduced once at the end; inverse
// butterflies let sums double for the 8 stages of a pass (inputs < 4q -> < 1024q). BIG primes (q < 2^60)
// use Harvey's butterflies: values are kept in [0,8q) (forward) / [0,4q) (inverse).
#pragma once
#include "modarith.hip.h"

#define NTT16_THREADS 256
#define NTT16_LDS_BYTES (16 * 272 * 8)

// ---- butterflies ----
template <bool BIG>
__device__ __forceinline__ u64 lazy_const(u64 q) { return 4 * q; }
// Forward (Cooley-Tukey), q2 = 4q. BIG: inputs and outputs in [0,8q). SMALL: values grow by 4q per stage.
template <bool BIG>
__device__ __forceinline__ void bf_fwd(u64& X, u64& Y, ulonglong2 w, u64 q, u64 q2) {
  if (BIG) X = csub_neg(X, q2);
  u64 T = shoup_lazy4(Y, w.x, w.y, q);
  Y = X + q2 - T;
  X = X + T;
}
// Inverse (Gentleman-Sande). BIG: c = 4q, inputs in [0,4q), outputs in [0,4q). SMALL: inputs < c (a multiple of q,
// at least 4q), X' < 2c, Y' < 4q.
template <bool BIG>
__device__ __forceinline__ void bf_inv(u64& X, u64& Y, ulonglong2 w, u64 q, u64 c) {
  u64 S = X + Y;
  u64 D = X + c - Y;
  if (BIG) S = csub_neg(S, c);  // c == 4q
  X = S;
  Y = shoup_lazy4(D, w.x, w.y, q);
}

// Four forward stages on 16 registers: stage s pairs (a, a + (8>>s)); tw(s, g) is the twiddle of group g.
template <bool BIG, class TW>
__device__ __forceinline__ void radix16_fwd(u64 (&x)[16], u64 q, u64 q2, TW tw) {
#pragma unroll
  for (int s = 0; s < 4; s++) {
    const int half = 8 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      ulonglong2 w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) bf_fwd<BIG>(x[g * 2 * half + p], x[g * 2 * half + p + half], w, q, q2);
    }
  }
}
// Four inverse stages, in the reverse order (s = 3..0). c0 = bound of the inputs (SMALL) or 4q (BIG).
template <bool BIG, class TW>
__device__ __forceinline__ void radix16_inv(u64 (&x)[16], u64 q, u64 c0, TW tw) {
  u64 c = c0;
#pragma unroll
  for (int s = 3; s >= 0; s--) {
    const int half = 8 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      ulonglong2 w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) bf_inv<BIG>(x[g * 2 * half + p], x[g * 2 * half + p + half], w, q, c);
    }
    if (!BIG) c <<= 1;
  }
}

// The same rounds with a hook after every stage: a pass uses it to request the next round's twiddles as this round's
// die, so that no twiddle is waited for right after it was requested (15 twiddle pairs are 60 registers: two rounds'
// worth do not fit beside the data).
template <bool BIG, class TW, class AFTER>
__device__ __forceinline__ void radix16_fwd_staged(u64 (&x)[16], u64 q, u64 q2, TW tw, AFTER after) {
#pragma unroll
  for (int s = 0; s < 4; s++) {
    const int half = 8 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      ulonglong2 w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) bf_fwd<BIG>(x[g * 2 * half + p], x[g * 2 * half + p + half], w, q, q2);
    }
    after(s);
  }
}
template <bool BIG, class TW, class AFTER>
__device__ __forceinline__ void radix16_inv_staged(u64 (&x)[16], u64 q, u64 c0, TW tw, AFTER after) {
  u64 c = c0;
#pragma unroll
  for (int s = 3; s >= 0; s--) {
    const int half = 8 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      ulonglong2 w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) bf_inv<BIG>(x[g * 2 * half + p], x[g * 2 * half + p + half], w, q, c);
    }
    if (!BIG) c <<= 1;
    after(s);
  }
}
// Slot of the twiddle pair of stage s, group g in a round's table of 15.
#define NTT16_TW_INDEX(s, g) ((1 << (s)) - 1 + (g))
// The 2^s twiddle pairs of stage s, from `src`, into their slots of a round's table. Written out per stage so that
// every index is a constant and the table stays in registers.
__device__ __forceinline__ void ntt16_load_stage(ulonglong2 (&t)[15], const ulonglong2* __restrict__ src, int s) {
  if (s == 0) {
    t[0] = src[0];
  } else if (s == 1) {
    t[1] = src[0], t[2] = src[1];
  } else if (s == 2) {
    t[3] = src[0], t[4] = src[1], t[5] = src[2], t[6] = src[3];
  } else {
    t[7] = src[0], t[8] = src[1], t[9] = src[2], t[10] = src[3];
    t[11] = src[4], t[12] = src[5], t[13] = src[6], t[14] = src[7];
  }
}

__device__ __forceinline__ u64 barrett_lazy(u64 v, u64 mu, u64 q) { return v - mul_hi64(v, mu) * q; }  // [0,2q)

// ---- pass bodies. `base` points at one limb-vector of 65536 words, `tw` at that modulus' table. ----

// Forward, stages 0..7. In: canonical (or < 2q). Out: SMALL < 33q (+in), BIG < 8q.
// `x` holds, for lane (r0 = t>>4, col = t&15), the rows i*16 + r0 (i = 0..15) of column col0 + col.
template <bool BIG>
__device__ __forceinline__ void ntt16_fwd_rows_loaded(u64 (&x)[16], u64* __restrict__ dst, const ulonglong2* __restrict__ tw,
                                                      u64 q, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
  const u64 q2 = lazy_const<BIG>(q);
  const u32 i0 = r0;
  // the second round's twiddles (one set per 16-lane group) are requested here, next to the data loads, and arrive
  // during the first round, whose own twiddles are wave-uniform scalar loads
  ulonglong2 twb[15];
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twb[NTT16_TW_INDEX(s, g)] = tw[(16 << s) + (i0 << s) + g];
  __builtin_amdgcn_sched_barrier(0);
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[i * 256 + t] = x[i];
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[(i0 * 16 + j) * 16 + col];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return twb[NTT16_TW_INDEX(s, g)]; });
#pragma unroll
  for (int j = 0; j < 16; j++) dst[(size_t)(i0 * 16 + j) * 256 + col0 + col] = x[j];
}
template <bool BIG>
__device__ __forceinline__ void ntt16_fwd_rows(const u64* __restrict__ src, u64* __restrict__ dst, const ulonglong2* __restrict__ tw,
                                               u64 q, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
  u64 x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = src[(size_t)(i * 16 + r0) * 256 + col0 + col];
  ntt16_fwd_rows_loaded<BIG>(x, dst, tw, q, tile, sm);
}

// Forward, stages 8..15, then canonical (CANON) or < 2q. `x` is left holding, for lane (hb = t>>4, j0 = t&15), the 16 values at
// block h = tile*16 + hb, positions i*16 + j0 (i = 0..15), ready for a coalesced store or a fused epilogue.
template <bool BIG, bool CANON = true>
__device__ __forceinline__ void ntt16_fwd_blocks_loaded(u64 (&x)[16], const ulonglong2* __restrict__ tw, u64 q, u64 mu,
                                                        u32 tile, u64* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u64 q2 = lazy_const<BIG>(q);
  const u32 i0 = j0;
  // first round's twiddles (one set per group) requested here, next to the caller's data loads; the second round's
  // (one set per lane) take their registers over stage by stage
  ulonglong2 twa[15], twb[15];
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twa[NTT16_TW_INDEX(s, g)] = tw[(256 << s) + (h << s) + g];
  __builtin_amdgcn_sched_barrier(0);
  radix16_fwd_staged<BIG>(
      x, q, q2, [&](int s, int g) { return twa[NTT16_TW_INDEX(s, g)]; },
      [&](int s) {
        __builtin_amdgcn_sched_barrier(0);
        ntt16_load_stage(twb, tw + (4096 << s) + (h << (4 + s)) + (i0 << s), s);
        __builtin_amdgcn_sched_barrier(0);
      });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[hb * 272 + i * 17 + j0] = x[i];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[hb * 272 + i0 * 17 + j];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return twb[NTT16_TW_INDEX(s, g)]; });
#pragma unroll
  for (int j = 0; j < 16; j++) {
    u64 v = x[j];
    if (BIG) v = csub(csub(v, q2), 2 * q);
    else v = barrett_lazy(v, mu, q);
    x[j] = CANON ? csub(v, q) : v;
  }
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[hb * 272 + i0 * 17 + j] = x[j];
  wave_lds_sync();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[hb * 272 + i * 17 + j0];
}

template <bool BIG, bool CANON = true>
__device__ __forceinline__ void ntt16_fwd_blocks(u64 (&x)[16], const u64* __restrict__ src, const ulonglong2* __restrict__ tw,
                                                 u64 q, u64 mu, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, h = tile * 16 + (t >> 4);
  const u64* blk = src + (size_t)h * 256;
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = blk[i * 16 + j0];
  ntt16_fwd_blocks_loaded<BIG, CANON>(x, tw, q, mu, tile, sm);
}

// Forward, stages 8..15 of one 256-element block by 32 adjacent lanes with 8 values each (the layout of
// ntt256_fwd_blocks_fp8: radix-8, exchange, radix-8, exchange, radix-4; LDS rows of pitch 35 words per 32 elements,
// all exchanges inside the half-wave). In: x[i] = element i*32 + l, lazy (BIG: < 8q). Out: x[c] = element
// (l >> 2)*32 + (l & 3)*8 + c, below 2q. `between` runs after the first exchange has been written.
#define NTT8_PITCH_I 35
#define NTT8_BLOCK_LDS_I (8 * NTT8_PITCH_I)
template <bool BIG, class TW>
__device__ __forceinline__ void radix8_fwd(u64 (&x)[8], u64 q, u64 q2, TW tw) {
#pragma unroll
  for (int s = 0; s < 3; s++) {
    const int half = 4 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      const ulonglong2 w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) bf_fwd<BIG>(x[g * 2 * half + p], x[g * 2 * half + p + half], w, q, q2);
    }
  }
}
template <bool BIG, class TW, class AFTER>
__device__ __forceinline__ void radix8_fwd_staged(u64 (&x)[8], u64 q, u64 q2, TW tw, AFTER after) {
#pragma unroll
  for (int s = 0; s < 3; s++) {
    const int half = 4 >> s;
#pragma unroll
    for (int g = 0; g < (1 << s); g++) {
      const ulonglong2 w = tw(s, g);
#pragma unroll
      for (int p = 0; p < half; p++) bf_fwd<BIG>(x[g * 2 * half + p], x[g * 2 * half + p + half], w, q, q2);
    }
    after(s);
  }
}
template <bool BIG, class BETWEEN>
__device__ __forceinline__ void ntt256_fwd_blocks_int8(u64 (&x)[8], const ulonglong2* __restrict__ tw, u64 q, u64 mu, u32 h,
                                                       u32 l, u64* smb, BETWEEN between) {
  const u32 a = l >> 2, b = l & 3;
  const u64 q2 = lazy_const<BIG>(q);
  // The first two rounds' twiddles are requested before `between` runs: the first round's here, the second round's
  // stage by stage as the first round's registers die. Whatever `between` requests is then younger than all of them,
  // so the second round never waits for it. The last two stages' twiddles follow once the second round's registers
  // are free; by then the caller needs what `between` requested anyway.
  ulonglong2 t1[7], t2[7], t3[6];
#pragma unroll
  for (int s = 0; s < 3; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) t1[(1 << s) - 1 + g] = tw[(256 << s) + (h << s) + g];
  __builtin_amdgcn_sched_barrier(0);
  radix8_fwd_staged<BIG>(
      x, q, q2, [&](int s, int g) { return t1[(1 << s) - 1 + g]; },
      [&](int s) {
        __builtin_amdgcn_sched_barrier(0);
        const ulonglong2* ts = tw + (2048 << s) + (h << (3 + s)) + (a << s);
        if (s == 0) {
          t2[0] = ts[0];
        } else if (s == 1) {
          t2[1] = ts[0], t2[2] = ts[1];
        } else {
          t2[3] = ts[0], t2[4] = ts[1], t2[5] = ts[2], t2[6] = ts[3];
        }
        __builtin_amdgcn_sched_barrier(0);
      });
#pragma unroll
  for (int i = 0; i < 8; i++) smb[i * NTT8_PITCH_I + l] = x[i];
  between();
  __builtin_amdgcn_sched_barrier(0);
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < 8; r++) x[r] = smb[a * NTT8_PITCH_I + r * 4 + b];
  radix8_fwd<BIG>(x, q, q2, [&](int s, int g) { return t2[(1 << s) - 1 + g]; });
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < 2; u++) t3[u] = tw[16384 + (h << 6) + (a << 3) + (b << 1) + u];
#pragma unroll
  for (int k = 0; k < 4; k++) t3[2 + k] = tw[32768 + (h << 7) + (a << 4) + (b << 2) + k];
  __builtin_amdgcn_sched_barrier(0);
  wave_lds_sync();
#pragma unroll
  for (int r = 0; r < 8; r++) smb[a * NTT8_PITCH_I + r * 4 + b] = x[r];
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 8; c++) x[c] = smb[a * NTT8_PITCH_I + b * 8 + c];
#pragma unroll
  for (int u = 0; u < 2; u++) {   // stage 14: pairs (c, c + 2) inside each half
#pragma unroll
    for (int p = 0; p < 2; p++) bf_fwd<BIG>(x[u * 4 + p], x[u * 4 + p + 2], t3[u], q, q2);
  }
#pragma unroll
  for (int k = 0; k < 4; k++) bf_fwd<BIG>(x[2 * k], x[2 * k + 1], t3[2 + k], q, q2);   // stage 15: pairs (2k, 2k + 1)
#pragma unroll
  for (int c = 0; c < 8; c++) x[c] = BIG ? csub(csub(x[c], q2), 2 * q) : barrett_lazy(x[c], mu, q);
}

// Inverse, stages 15..8 on contiguous blocks. In: x holds, for lane (hb, j0), the values at positions i*16 + j0
// of block h (any value < 2q). Out: < 2q (BIG: < 4q), same lane layout, ready for a coalesced store.
template <bool BIG>
__device__ __forceinline__ void ntt16_inv_blocks(u64 (&x)[16], const ulonglong2* __restrict__ twi, u64 q, u64 mu, u32 tile,
                                                 u64* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u64 q2 = lazy_const<BIG>(q);
  const u32 i0 = j0;
  // first round's twiddles (one set per lane): requested before the transpose; the second round's (one set per
  // group) take their registers over stage by stage
  ulonglong2 twa[15];
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twa[NTT16_TW_INDEX(s, g)] = twi[(4096 << s) + (h << (4 + s)) + (i0 << s) + g];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 16; i++) sm[hb * 272 + i * 17 + j0] = x[i];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[hb * 272 + i0 * 17 + j];
  ulonglong2 twb[15];
  radix16_inv_staged<BIG>(
      x, q, q2, [&](int s, int g) { return twa[NTT16_TW_INDEX(s, g)]; },
      [&](int s) {
        __builtin_amdgcn_sched_barrier(0);
        ntt16_load_stage(twb, twi + (256 << s) + (h << s), s);
        __builtin_amdgcn_sched_barrier(0);
      });
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[hb * 272 + i0 * 17 + j] = x[j];
  wave_lds_sync();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[hb * 272 + i * 17 + j0];
  radix16_inv<BIG>(x, q, BIG ? q2 : (q2 << 4), [&](int s, int g) { return twb[NTT16_TW_INDEX(s, g)]; });
  if (!BIG) {
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = barrett_lazy(x[i], mu, q);
  }
}

// Inverse, stages 7..0 on 256 rows x 16 columns, then multiplication by the constant (sc, scs) (N^-1, possibly
// merged with another per-limb constant) and canonical output. In: < 2q (BIG: < 4q). x holds for lane (r0 = t>>4, col = t&15)
// the rows i*16 + r0 of column col0 + col.
template <bool BIG>
__device__ __forceinline__ void ntt16_inv_rows(u64 (&x)[16], const u64* __restrict__ src, const ulonglong2* __restrict__ twi,
                                               u64 q, u64 sc, u64 scs, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, col = t & 15, i0 = t >> 4, col0 = tile * 16;
  const u64 q2 = lazy_const<BIG>(q);
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = src[(size_t)(i0 * 16 + j) * 256 + col0 + col];
  // first round's twiddles (one set per group) travel with the data; the second round's are scalar loads
  ulonglong2 twa[15];
#pragma unroll
  for (int s = 0; s < 4; s++)
#pragma unroll
    for (int g = 0; g < (1 << s); g++) twa[NTT16_TW_INDEX(s, g)] = twi[(16 << s) + (i0 << s) + g];
  __builtin_amdgcn_sched_barrier(0);
  radix16_inv<BIG>(x, q, q2, [&](int s, int g) { return twa[NTT16_TW_INDEX(s, g)]; });
#pragma unroll
  for (int j = 0; j < 16; j++) sm[(i0 * 16 + j) * 16 + col] = x[j];
  lds_barrier();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[i * 256 + t];
  radix16_inv<BIG>(x, q, BIG ? q2 : (q2 << 4), [&](int s, int g) { return twi[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = shoup(x[i], sc, scs, q);
}

// Eval-domain Galois map for N = 2^16: out[k] = in[k'], 2*brev(k')+1 = (2*brev(k)+1)*g mod 2N. It maps every aligned
// 16-element segment onto an aligned 16-element segment, so 16 adjacent lanes still read one 128-byte line.
__device__ __forceinline__ u32 galois_src_index16(u32 k, u32 g) {
  u32 e = 2 * (__brev(k) >> 16) + 1;
  u32 t = (e * g) & 0x1FFFFu;
  return __brev(t >> 1) >> 16;
}

// Workgroup -> (poly, tile, slot). mode 0: dispatch order is polynomial-fastest; 1: same, made XCD-contiguous;
// 2: tile-fastest; 3: tile-fastest, XCD-contiguous; 4: all polynomials of one (tile, slot) group run on one XCD
// (they share that group's twiddles and key slices in its L2) while eight consecutive groups, one per XCD, are in
// flight together, which keeps the XCDs evenly loaded. gridDim.y * gridDim.z must be a multiple of 8 for mode 4.
__device__ __forceinline__ void ntt16_map(u32 mode, u32& poly, u32& tile, u32& slot) {
  const u32 lin0 = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  if (mode == 4) {
    const u32 x = lin0 & 7, rest = lin0 >> 3;
    poly = rest % gridDim.x;
    const u32 group = x + 8 * (rest / gridDim.x);
    tile = group % gridDim.y;
    slot = group / gridDim.y;
    return;
  }
  const u32 lin = (mode & 1) ? xcd_swizzled_linear_id() : lin0;
  if (mode & 2) {
    tile = lin % gridDim.y;
    poly = (lin / gridDim.y) % gridDim.x;
  } else {
    poly = lin % gridDim.x;
    tile = (lin / gridDim.x) % gridDim.y;
  }
  slot = lin / (gridDim.x * gridDim.y);
}
