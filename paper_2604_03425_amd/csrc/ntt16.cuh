// Two-pass negacyclic NTT for N = 2^16 on gfx950: each pass does 8 butterfly stages on a 4096-element
// tile held as 16 registers per lane (256 lanes), as two in-register radix-16 rounds with one LDS
// transpose between them. Pass "row" works on 256 rows x 16 adjacent columns of the 256x256 view of a
// limb (stride-256 butterflies, stages 0..7); pass "blk" works on 16 contiguous 256-element blocks
// (stages 8..15). Global loads and stores always have 16 adjacent lanes on 128 contiguous bytes.
//
// Lazy ranges. SMALL primes (q < 2^52): forward butterflies never correct, values grow by 2q per
// stage (< 33q < 2^58 after 16 stages from canonical input) and are reduced once at the end; inverse
// butterflies let sums double for the 8 stages of a pass (inputs < 2q -> < 512q). BIG primes (q < 2^61)
// use Harvey's butterflies with values kept in [0,4q) (forward) / [0,2q) (inverse).
#pragma once
#include "modarith.cuh"

#define NTT16_THREADS 256
#define NTT16_LDS_BYTES (16 * 272 * 8)

// ---- butterflies ----
template <bool BIG>
__device__ __forceinline__ void bf_fwd(u64& X, u64& Y, ulonglong2 w, u64 q, u64 q2) {
  if (BIG) X = csub(X, q2);
  u64 T = shoup_lazy(Y, w.x, w.y, q);
  Y = X + q2 - T;
  X = X + T;
}
// Inverse (Gentleman-Sande). BIG: inputs in [0,2q), outputs in [0,2q). SMALL: inputs < c (a multiple of q),
// X' < 2c, Y' < 2q.
template <bool BIG>
__device__ __forceinline__ void bf_inv(u64& X, u64& Y, ulonglong2 w, u64 q, u64 c) {
  u64 S = X + Y;
  u64 D = X + c - Y;
  if (BIG) S = csub(S, c);  // c == 2q
  X = S;
  Y = shoup_lazy(D, w.x, w.y, q);
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
// Four inverse stages, in the reverse order (s = 3..0). c0 = bound of the inputs (SMALL) or 2q (BIG).
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

__device__ __forceinline__ u64 barrett_lazy(u64 v, u64 mu, u64 q) { return v - mul_hi64(v, mu) * q; }  // [0,2q)

// ---- pass bodies. `base` points at one limb-vector of 65536 words, `tw` at that modulus' table. ----

// Forward, stages 0..7. In: canonical (or < 2q). Out: SMALL < 17q (+in), BIG < 4q.
template <bool BIG>
__device__ __forceinline__ void ntt16_fwd_rows(const u64* __restrict__ src, u64* __restrict__ dst, const ulonglong2* __restrict__ tw,
                                               u64 q, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
  const u64 q2 = 2 * q;
  u64 x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = src[(size_t)(i * 16 + r0) * 256 + col0 + col];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[i * 256 + t] = x[i];
  __syncthreads();
  const u32 i0 = r0;
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[(i0 * 16 + j) * 16 + col];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(16 << s) + (i0 << s) + g]; });
#pragma unroll
  for (int j = 0; j < 16; j++) dst[(size_t)(i0 * 16 + j) * 256 + col0 + col] = x[j];
}

// Forward, stages 8..15, then canonical. `x` is left holding, for lane (hb = t>>4, j0 = t&15), the 16 values at
// block h = tile*16 + hb, positions i*16 + j0 (i = 0..15), ready for a coalesced store or a fused epilogue.
template <bool BIG>
__device__ __forceinline__ void ntt16_fwd_blocks(u64 (&x)[16], const u64* __restrict__ src, const ulonglong2* __restrict__ tw,
                                                 u64 q, u64 mu, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u64 q2 = 2 * q;
  const u64* blk = src + (size_t)h * 256;
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = blk[i * 16 + j0];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(256 << s) + (h << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[hb * 272 + i * 17 + j0] = x[i];
  __syncthreads();
  const u32 i0 = j0;
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[hb * 272 + i0 * 17 + j];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(4096 << s) + (h << (4 + s)) + (i0 << s) + g]; });
#pragma unroll
  for (int j = 0; j < 16; j++) {
    u64 v = x[j];
    if (BIG) v = csub(v, q2);
    else v = barrett_lazy(v, mu, q);
    x[j] = csub(v, q);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[hb * 272 + i0 * 17 + j] = x[j];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[hb * 272 + i * 17 + j0];
}

// Inverse, stages 15..8 on contiguous blocks. In: x holds, for lane (hb, j0), the values at positions i*16 + j0
// of block h (any value < 2q). Out: < 2q, same lane layout, ready for a coalesced store.
template <bool BIG>
__device__ __forceinline__ void ntt16_inv_blocks(u64 (&x)[16], const ulonglong2* __restrict__ twi, u64 q, u64 mu, u32 tile,
                                                 u64* sm) {
  const u32 t = threadIdx.x, j0 = t & 15, hb = t >> 4, h = tile * 16 + hb;
  const u64 q2 = 2 * q;
#pragma unroll
  for (int i = 0; i < 16; i++) sm[hb * 272 + i * 17 + j0] = x[i];
  __syncthreads();
  const u32 i0 = j0;
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[hb * 272 + i0 * 17 + j];
  radix16_inv<BIG>(x, q, q2, [&](int s, int g) { return twi[(4096 << s) + (h << (4 + s)) + (i0 << s) + g]; });
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[hb * 272 + i0 * 17 + j] = x[j];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[hb * 272 + i * 17 + j0];
  radix16_inv<BIG>(x, q, BIG ? q2 : (q2 << 4), [&](int s, int g) { return twi[(256 << s) + (h << s) + g]; });
  if (!BIG) {
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = barrett_lazy(x[i], mu, q);
  }
}

// Inverse, stages 7..0 on 256 rows x 16 columns, then multiplication by the constant (sc, scs) (N^-1, possibly
// merged with another per-limb constant) and canonical output. In: < 2q. x holds for lane (r0 = t>>4, col = t&15)
// the rows i*16 + r0 of column col0 + col.
template <bool BIG>
__device__ __forceinline__ void ntt16_inv_rows(u64 (&x)[16], const u64* __restrict__ src, const ulonglong2* __restrict__ twi,
                                               u64 q, u64 sc, u64 scs, u32 tile, u64* sm) {
  const u32 t = threadIdx.x, col = t & 15, i0 = t >> 4, col0 = tile * 16;
  const u64 q2 = 2 * q;
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = src[(size_t)(i0 * 16 + j) * 256 + col0 + col];
  radix16_inv<BIG>(x, q, q2, [&](int s, int g) { return twi[(16 << s) + (i0 << s) + g]; });
#pragma unroll
  for (int j = 0; j < 16; j++) sm[(i0 * 16 + j) * 16 + col] = x[j];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[i * 256 + t];
  radix16_inv<BIG>(x, q, BIG ? q2 : (q2 << 4), [&](int s, int g) { return twi[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = shoup(x[i], sc, scs, q);
}

// ---- standalone kernels: grid = (polynomials, 16 tiles, limb slots) ----
struct Ntt16Args {
  const u64* src;
  u64* dst;
  const ulonglong2* tw;     // forward or inverse table, [nm][65536]
  const ModInfo* mods;
  u64 src_poly_stride, dst_poly_stride;  // elements between polynomials
  u32 skip_beta, skip_alpha, skip_nq;    // as in the generic pass: digit p % skip_beta leaves its own limbs alone
  unsigned char id[128];
};

__device__ __forceinline__ bool ntt16_skip(const Ntt16Args& a, u32 poly, u32 slot) {
  if (!a.skip_beta) return false;
  u32 j = poly % a.skip_beta, lo = j * a.skip_alpha, hi = min(lo + a.skip_alpha, a.skip_nq);
  return slot >= lo && slot < hi;
}
#define NTT16_PROLOGUE                                                            \
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];                                         \
  const u32 poly = blockIdx.x, tile = blockIdx.y, slot = blockIdx.z;              \
  if (ntt16_skip(a, poly, slot)) return;                                          \
  const u32 id = a.id[slot];                                                      \
  const ModInfo mi = a.mods[id];                                                  \
  const ulonglong2* tw = a.tw + (size_t)id * 65536;                               \
  const u64* src = a.src + (size_t)poly * a.src_poly_stride + (size_t)slot * 65536; \
  u64* dst = a.dst + (size_t)poly * a.dst_poly_stride + (size_t)slot * 65536;     \
  const bool big = (mi.m >> 52) != 0;

__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_rows_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  if (big) ntt16_fwd_rows<true>(src, dst, tw, mi.m, tile, sm);
  else ntt16_fwd_rows<false>(src, dst, tw, mi.m, tile, sm);
}
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_blocks_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  u64 x[16];
  if (big) ntt16_fwd_blocks<true>(x, src, tw, mi.m, mi.mu64, tile, sm);
  else ntt16_fwd_blocks<false>(x, src, tw, mi.m, mi.mu64, tile, sm);
  const u32 t = threadIdx.x, j0 = t & 15, h = tile * 16 + (t >> 4);
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)h * 256 + i * 16 + j0] = x[i];
}
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_inv_blocks_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  const u32 t = threadIdx.x, j0 = t & 15, h = tile * 16 + (t >> 4);
  u64 x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = src[(size_t)h * 256 + i * 16 + j0];
  if (big) ntt16_inv_blocks<true>(x, tw, mi.m, mi.mu64, tile, sm);
  else ntt16_inv_blocks<false>(x, tw, mi.m, mi.mu64, tile, sm);
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)h * 256 + i * 16 + j0] = x[i];
}
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_inv_rows_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  u64 x[16];
  if (big) ntt16_inv_rows<true>(x, src, tw, mi.m, mi.ninv, mi.ninvs, tile, sm);
  else ntt16_inv_rows<false>(x, src, tw, mi.m, mi.ninv, mi.ninvs, tile, sm);
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)(i * 16 + r0) * 256 + col0 + col] = x[i];
}
