// Single-pass negacyclic NTT for N = 2^12 on gfx950: one workgroup of 256 lanes holds a whole limb (4096 residues,
// 16 per lane) and takes it through all 12 stages as three in-register radix-16 rounds with two exchanges through
// LDS; the limb is read and written once. Same butterflies, lazy ranges and modulus classes as the N = 2^16 passes
// (ntt16.hip.h, ntt16fp.hip.h): double precision for q < 2^50, uncorrected integer butterflies for q < 2^52, Harvey
// butterflies for q < 2^60.
//
// Layouts. Round 1 (stages 0..3): lane t holds elements i*256 + t. Round 2 (stages 4..7): lane (i0 = t>>4, col = t&15)
// holds elements (i0*16 + j)*16 + col: a workgroup-wide exchange. Round 3 (stages 8..11): lane (i0, l) holds the 16
// consecutive elements of row R = i0*16 + l: an exchange inside groups of 16 adjacent lanes (no workgroup barrier for
// the data, one to recycle the LDS tile). Memory is always touched one column per lane (16 adjacent lanes on one
// 128-byte line); the row layout exists only between two exchanges.
#pragma once
#include "ntt16fp.hip.h"

#define NTT12_LDS_WORDS (16 * 272)

// ---- integer classes ----
template <bool BIG>
__device__ __forceinline__ void ntt12_fwd_int(const u64* __restrict__ src, u64* __restrict__ dst,
                                              const ulonglong2* __restrict__ tw, u64 q, u64 mu, u64* sm) {
  const u32 t = threadIdx.x, l = t & 15, i0 = t >> 4, R = i0 * 16 + l;
  const u64 q2 = lazy_const<BIG>(q);
  u64 x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = src[i * 256 + t];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[i * 256 + t] = x[i];
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[(i0 * 16 + j) * 16 + l];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(16 << s) + (i0 << s) + g]; });
  lds_barrier();   // every lane has read its round-2 values: the tile can be reused with the padded pitch
#pragma unroll
  for (int j = 0; j < 16; j++) sm[i0 * 272 + j * 17 + l] = x[j];
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) x[c] = sm[i0 * 272 + l * 17 + c];
  radix16_fwd<BIG>(x, q, q2, [&](int s, int g) { return tw[(256 << s) + (R << s) + g]; });
#pragma unroll
  for (int c = 0; c < 16; c++) {
    u64 v = x[c];
    v = BIG ? csub(csub(v, q2), 2 * q) : barrett_lazy(v, mu, q);
    x[c] = csub(v, q);
  }
  // back to one column per lane, so that 16 adjacent lanes store one 128-byte line
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) sm[i0 * 272 + l * 17 + c] = x[c];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) dst[(i0 * 16 + j) * 16 + l] = sm[i0 * 272 + j * 17 + l];
}

// Inverse, with the multiplication by the constant (sc, scs) (N^-1) at the end; canonical in, canonical out.
template <bool BIG>
__device__ __forceinline__ void ntt12_inv_int(const u64* __restrict__ src, u64* __restrict__ dst,
                                              const ulonglong2* __restrict__ twi, u64 q, u64 mu, u64 sc, u64 scs, u64* sm) {
  const u32 t = threadIdx.x, l = t & 15, i0 = t >> 4, R = i0 * 16 + l;
  const u64 q2 = lazy_const<BIG>(q);
  u64 x[16];
  // 16 adjacent lanes load one 128-byte line; an exchange inside the group gives every lane its row
#pragma unroll
  for (int j = 0; j < 16; j++) sm[i0 * 272 + j * 17 + l] = src[(i0 * 16 + j) * 16 + l];
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) x[c] = sm[i0 * 272 + l * 17 + c];
  radix16_inv<BIG>(x, q, q2, [&](int s, int g) { return twi[(256 << s) + (R << s) + g]; });
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) sm[i0 * 272 + l * 17 + c] = x[c];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[i0 * 272 + j * 17 + l];
  radix16_inv<BIG>(x, q, BIG ? q2 : (q2 << 4), [&](int s, int g) { return twi[(16 << s) + (i0 << s) + g]; });
  if (!BIG) {   // eight stages of doubling sums: back below 2q before the last four
#pragma unroll
    for (int j = 0; j < 16; j++) x[j] = barrett_lazy(x[j], mu, q);
  }
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[(i0 * 16 + j) * 16 + l] = x[j];
  lds_barrier();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[i * 256 + t];
  radix16_inv<BIG>(x, q, q2, [&](int s, int g) { return twi[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) dst[i * 256 + t] = shoup(x[i], sc, scs, q);
}

// ---- double-precision class ----
__device__ __forceinline__ void ntt12_fwd_fp(const u64* __restrict__ src, u64* __restrict__ dst, const double* __restrict__ tw,
                                             double q, double qinv, double* sm) {
  const u32 t = threadIdx.x, l = t & 15, i0 = t >> 4, R = i0 * 16 + l;
  double x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = u2d(src[i * 256 + t]);
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return tw[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) sm[i * 256 + t] = x[i];
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[(i0 * 16 + j) * 16 + l];
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return tw[(16 << s) + (i0 << s) + g]; });
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[i0 * 272 + j * 17 + l] = x[j];
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) x[c] = sm[i0 * 272 + l * 17 + c];
  radix16_fwd_fp(x, q, qinv, [&](int s, int g) { return tw[(256 << s) + (R << s) + g]; });
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) sm[i0 * 272 + l * 17 + c] = x[c];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) dst[(i0 * 16 + j) * 16 + l] = d2u_canon(sm[i0 * 272 + j * 17 + l], q);
}

__device__ __forceinline__ void ntt12_inv_fp(const u64* __restrict__ src, u64* __restrict__ dst, const double* __restrict__ twi,
                                             double q, double qinv, double sc, double scq, double* sm) {
  const u32 t = threadIdx.x, l = t & 15, i0 = t >> 4, R = i0 * 16 + l;
  double x[16];
#pragma unroll
  for (int j = 0; j < 16; j++) sm[i0 * 272 + j * 17 + l] = u2d(src[(i0 * 16 + j) * 16 + l]);
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) x[c] = sm[i0 * 272 + l * 17 + c];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twi[(256 << s) + (R << s) + g]; });
  wave_lds_sync();
#pragma unroll
  for (int c = 0; c < 16; c++) sm[i0 * 272 + l * 17 + c] = x[c];
  wave_lds_sync();
#pragma unroll
  for (int j = 0; j < 16; j++) x[j] = sm[i0 * 272 + j * 17 + l];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twi[(16 << s) + (i0 << s) + g]; });
  lds_barrier();
#pragma unroll
  for (int j = 0; j < 16; j++) sm[(i0 * 16 + j) * 16 + l] = x[j];
  lds_barrier();
#pragma unroll
  for (int i = 0; i < 16; i++) x[i] = sm[i * 256 + t];
  radix16_inv_fp(x, q, qinv, [&](int s, int g) { return twi[(1 << s) + g]; });
#pragma unroll
  for (int i = 0; i < 16; i++) dst[i * 256 + t] = d2u_canon(fp_mulmod_const(x[i], sc, scq, q), q);
}

// grid = (polynomials, limb slots). Slot `s` of polynomial `p` is at + p * poly_stride + s * 4096 in src and dst
// (src == dst transforms in place: every lane reads its words before any lane writes, across two barriers).
struct Ntt12Args {
  const u64* src;
  u64* dst;
  const ulonglong2* tw;     // integer table (forward or inverse), [nm][4096]
  const double* twfp;       // double table, same indexing (rows of moduli >= 2^50 unused)
  const ModInfo* mods;
  u64 src_poly_stride, dst_poly_stride;
  u32 skip_beta, skip_alpha, skip_nq;   // digit p % skip_beta leaves its own limbs alone (ModUp'ed digits)
  u32 fp_on;                            // 0: integer bodies for every modulus
  unsigned char id[128];                // slot -> modulus id
};

template <bool INV>
__global__ void __launch_bounds__(256) ntt12_kernel(Ntt12Args a) {
  __shared__ u64 sm[NTT12_LDS_WORDS];
  const u32 poly = blockIdx.x, slot = blockIdx.y;
  if (a.skip_beta) {
    const u32 j = poly % a.skip_beta, lo = j * a.skip_alpha, hi = min(lo + a.skip_alpha, a.skip_nq);
    if (slot >= lo && slot < hi) return;
  }
  const u32 id = a.id[slot];
  const ModInfo mi = a.mods[id];
  const u64* src = a.src + (size_t)poly * a.src_poly_stride + (size_t)slot * 4096;
  u64* dst = a.dst + (size_t)poly * a.dst_poly_stride + (size_t)slot * 4096;
  const ulonglong2* tw = a.tw + (size_t)id * 4096;
  const int cls = mod_class(mi.m, a.fp_on);   // uniform per workgroup
  if (cls == 0) {
    const double* twfp = a.twfp + (size_t)id * 4096;
    if (INV) ntt12_inv_fp(src, dst, twfp, mi.qd, mi.qinv, mi.ninvd, mi.ninvq, (double*)sm);
    else ntt12_fwd_fp(src, dst, twfp, mi.qd, mi.qinv, (double*)sm);
  } else if (cls == 2) {
    if (INV) ntt12_inv_int<true>(src, dst, tw, mi.m, mi.mu64, mi.ninv, mi.ninvs, sm);
    else ntt12_fwd_int<true>(src, dst, tw, mi.m, mi.mu64, sm);
  } else {
    if (INV) ntt12_inv_int<false>(src, dst, tw, mi.m, mi.mu64, mi.ninv, mi.ninvs, sm);
    else ntt12_fwd_int<false>(src, dst, tw, mi.m, mi.mu64, sm);
  }
}
