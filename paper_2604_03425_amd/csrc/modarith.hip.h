// 64-bit modular arithmetic for word-sized primes (< 2^61) on gfx950, built from 32-bit
// integer multiplies (v_mul_lo/hi_u32, v_mad_u64_u32), which issue at full VALU rate on CDNA4.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
typedef unsigned int u32;

// Per-modulus constants, read through scalar loads (the modulus is uniform per workgroup).
struct ModInfo {
  u64 m;      // the prime
  u64 mu64;   // floor(2^64 / m)
  u64 c64;    // 2^64 mod m
  u64 c64s;   // floor(c64 * 2^64 / m)
  u64 ninv;   // N^-1 mod m
  u64 ninvs;  // floor(ninv * 2^64 / m)
  u64 minv;   // -m^-1 mod 2^64 (Montgomery)
  u64 pmod;   // main primes: (p_0 ... p_{K-1}) mod m, the product of all special primes; 0 on special primes
  // double-precision view, used for primes < 2^50 (every residue and every lazy value below 2^53 is exact)
  double qd;     // m
  double qinv;   // 1/m rounded
  double ninvd;  // N^-1 mod m
  double ninvq;  // ninvd / m rounded
};

// ---- exact modular arithmetic in double precision for primes q < 2^50 ----
// Values are integers held in doubles with magnitude < 2^53 = 8q. The product a*w is formed exactly as h + l
// (rounded product + fma error term), the quotient estimate c = rint(a * (w/q)) is off by at most
// 0.5 + |a| 2^-52 from a*w/q, and h - c q + l is exact. All operations are IEEE and deterministic.
__device__ __forceinline__ double fp_mulmod_const(double a, double w, double wq, double q) {
  double h = a * w;
  double l = __builtin_fma(a, w, -h);
  double c = __builtin_rint(a * wq);
  return __builtin_fma(-c, q, h) + l;  // |result| <= (0.5 + |a|/2^52) q
}
// a * e mod q for two variables (no precomputed e/q): quotient from the rounded product.
__device__ __forceinline__ double fp_mulmod_var(double a, double e, double qinv, double q) {
  double h = a * e;
  double l = __builtin_fma(a, e, -h);
  double c = __builtin_rint(h * qinv);
  return __builtin_fma(-c, q, h) + l;
}
__device__ __forceinline__ double fp_reduce(double x, double qinv, double q) {  // |result| <= q/2 (+1)
  return __builtin_fma(-__builtin_rint(x * qinv), q, x);
}
__device__ __forceinline__ double u2d(u64 v) {  // exact for v < 2^52
  return __longlong_as_double((long long)(v | 0x4330000000000000ull)) - 4503599627370496.0;
}
__device__ __forceinline__ u64 d2u_canon(double r, double q) {  // r an integer in (-q, 2q) -> canonical residue
  r = r < 0.0 ? r + q : r;
  r = r >= q ? r - q : r;
  return (u64)__double_as_longlong(r + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
}
// 0: double-precision path (q < 2^50), 1: integer path without butterfly corrections (q < 2^52), 2: Harvey (q < 2^60)
__device__ __forceinline__ int mod_class(u64 m, u32 fp_on) {
  if (fp_on && (m >> 50) == 0) return 0;
  return (m >> 52) == 0 ? 1 : 2;
}

__device__ __forceinline__ u64 mul_hi64(u64 a, u64 b) { return __umul64hi(a, b); }
__device__ __forceinline__ u64 csub(u64 x, u64 m) { return x >= m ? x - m : x; }
__device__ __forceinline__ u64 addmod(u64 a, u64 b, u64 m) { return csub(a + b, m); }
__device__ __forceinline__ u64 submod(u64 a, u64 b, u64 m) { return a >= b ? a - b : a + m - b; }

// x * w mod m for a constant w < m with companion ws = floor(w * 2^64 / m). Any x < 2^64.
// Result in [0, 2m).
__device__ __forceinline__ u64 shoup_lazy(u64 x, u64 w, u64 ws, u64 m) { return x * w - mul_hi64(x, ws) * m; }
__device__ __forceinline__ u64 shoup(u64 x, u64 w, u64 ws, u64 m) { return csub(shoup_lazy(x, w, ws, m), m); }
// Same product with a cheaper quotient estimate: of the four 32 x 32 partial products of x * ws only the top one
// and the high words of the two middle ones are summed (2 multiply-highs, 1 multiply-add and a 64-bit add instead of
// the carry chain of an exact high word). The estimate never exceeds floor(x * ws / 2^64) and falls short of it by
// at most 2, so the result lies in [0, 4m). Any x < 2^64; m < 2^62. The subtraction of estimate * m is done by
// adding estimate * (2^64 - m): both low-word products then share one multiply-add chain and no borrow is needed.
// neg_opaque() hides that the value is a negation, which the compiler would otherwise turn back into a subtraction.
__device__ __forceinline__ u64 neg_opaque(u64 m) {
  u64 nm = 0 - m;
  asm("" : "+s"(nm));
  return nm;
}
__device__ __forceinline__ u64 shoup_lazy4(u64 x, u64 w, u64 ws, u64 m) {
  const u64 nm = neg_opaque(m);
  const u32 x0 = (u32)x, x1 = (u32)(x >> 32), p0 = (u32)ws, p1 = (u32)(ws >> 32);
  const u64 qt = (u64)x1 * p1 + __umulhi(x1, p0) + __umulhi(x0, p1);
  const u32 q0 = (u32)qt, q1 = (u32)(qt >> 32), w0 = (u32)w, w1 = (u32)(w >> 32), n0 = (u32)nm, n1 = (u32)(nm >> 32);
  const u64 t = (u64)x0 * w0 + (u64)q0 * n0;   // modulo 2^64
  const u32 hi = (u32)(t >> 32) + x0 * w1 + x1 * w0 + q0 * n1 + q1 * n0;
  return ((u64)hi << 32) | (u32)t;
}
// x - m if x >= m, computed as x + (2^64 - m): one 64-bit add, no borrow chain.
__device__ __forceinline__ u64 csub_neg(u64 x, u64 m) {
  const u64 d = x + neg_opaque(m);
  return x >= m ? d : x;
}

// 128-bit lazy accumulator for sums of 64x64 products (up to 2^128 - 1 in total).
struct Acc128 {
  u64 lo, hi;
};
__device__ __forceinline__ void mac128(Acc128& a, u64 x, u64 y) {
  u64 l = x * y, h = mul_hi64(x, y);
  a.lo += l;
  a.hi += h + (a.lo < l ? 1ull : 0ull);
}
// Canonical residue of a 128-bit value: fold the high word with 2^64 mod m, Barrett the low word.
__device__ __forceinline__ u64 reduce128(Acc128 a, const ModInfo& mi) {
  u64 t = shoup_lazy(a.hi, mi.c64, mi.c64s, mi.m);  // [0, 2m)
  u64 r = a.lo - mul_hi64(a.lo, mi.mu64) * mi.m;    // [0, 2m)
  u64 s = csub(t + r, 2 * mi.m);
  return csub(s, mi.m);
}
__device__ __forceinline__ u64 mulmod(u64 a, u64 b, const ModInfo& mi) {
  Acc128 acc = {0, 0};
  mac128(acc, a, b);
  return reduce128(acc, mi);
}

// ---- lazy dot products with 30-bit operand halves ----
// A value v < 2^61 is split as v = v1 * 2^30 + v0 (v0 < 2^30, v1 < 2^31). The four partial products of two such
// values are accumulated in four 64-bit sums by v_mad_u64_u32 with no carry handling; up to 16 products of
// operands < 2^60 fit. The sum is then V = s00 + (s01 + s10) * 2^30 + s11 * 2^60.
struct Dot30 {
  u64 s00, s01, s10, s11;
};
__device__ __forceinline__ void dot30_init(Dot30& d) { d.s00 = d.s01 = d.s10 = d.s11 = 0; }
__device__ __forceinline__ void dot30_mac(Dot30& d, u32 y0, u32 y1, u32 c0, u32 c1) {
  d.s00 += (u64)y0 * c0;
  d.s01 += (u64)y0 * c1;
  d.s10 += (u64)y1 * c0;
  d.s11 += (u64)y1 * c1;
}
__device__ __forceinline__ Acc128 dot30_value(const Dot30& d) {
  Acc128 v;
  u64 mid = d.s01 + d.s10;
  u64 carry = mid < d.s01 ? 1ull : 0ull;       // the 65th bit of the middle sum
  u64 mlo = mid << 30, mhi = (mid >> 34) | (carry << 30);
  u64 hlo = d.s11 << 60, hhi = d.s11 >> 4;
  v.lo = d.s00 + mlo;
  v.hi = mhi + (v.lo < mlo ? 1ull : 0ull);
  u64 lo2 = v.lo + hlo;
  v.hi += hhi + (lo2 < hlo ? 1ull : 0ull);
  v.lo = lo2;
  return v;
}
// The same dot product with three sums (the two middle ones share an accumulator) and a word-by-word Montgomery
// reduction in base 2^30: V = a + b * 2^30 + c * 2^60 -> V * 2^-90 mod m in [0, m + 2^34), 22 instructions instead
// of assembling a 128-bit value and reducing that. Valid when no sum can pass 2^64, which the host checks from the
// bit sizes of the two bases and the number of terms (bconv_narrow_ok); constants then carry a factor 2^90.
struct Dot30N {
  u64 a, b, c;
};
__device__ __forceinline__ void dot30n_init(Dot30N& d) { d.a = d.b = d.c = 0; }
__device__ __forceinline__ void dot30n_mac(Dot30N& d, u32 y0, u32 y1, u32 c0, u32 c1) {
  d.a += (u64)y0 * c0;
  d.b += (u64)y0 * c1;
  d.b += (u64)y1 * c0;
  d.c += (u64)y1 * c1;
}
// minv = -m^-1 mod 2^64 (its low 30 bits are -m^-1 mod 2^30).
__device__ __forceinline__ u64 dot30n_redc90(const Dot30N& d, u64 m, u64 minv) {
  const u32 q0 = (u32)m & 0x3FFFFFFFu, q1 = (u32)(m >> 30), qi = (u32)minv & 0x3FFFFFFFu;
  u64 a = d.a, b = d.b, c = d.c;
  u32 u = ((u32)a * qi) & 0x3FFFFFFFu;
  a += (u64)u * q0;              // now a multiple of 2^30
  b += a >> 30;
  b += (u64)u * q1;
  u = ((u32)b * qi) & 0x3FFFFFFFu;
  b += (u64)u * q0;
  c += b >> 30;
  c += (u64)u * q1;
  u = ((u32)c * qi) & 0x3FFFFFFFu;
  c += (u64)u * q0;
  return (c >> 30) + (u64)u * q1;
}
// Montgomery reduction: V * 2^-64 mod m, in [0, V/2^64 + m). minv = -m^-1 mod 2^64.
__device__ __forceinline__ u64 redc(Acc128 v, u64 m, u64 minv) {
  u64 u = v.lo * minv;
  return v.hi + mul_hi64(u, m) + (v.lo != 0 ? 1ull : 0ull);
}

// Workgroup index remapped so that consecutive logical indices run on the same XCD (the dispatcher deals
// workgroups to the 8 XCDs round-robin in linear order). Returns the logical linear index for this workgroup.
__device__ __forceinline__ u32 xcd_swizzled_linear_id() {
  const u32 total = gridDim.x * gridDim.y * gridDim.z;
  const u32 lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const u32 xcd = lin & 7, k = lin >> 3;
  const u32 q = total >> 3, r = total & 7;
  return xcd * q + min(xcd, r) + k;
}

// Workgroup barrier that orders LDS traffic only: waits for this wave's LDS operations, not for its outstanding
// global loads and stores, so those stay in flight across the barrier (a plain __syncthreads() drains them).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Ordering point for LDS exchanges that stay inside one wavefront (here: inside a group of 16 adjacent lanes):
// the wave's own LDS operations complete in order, so waiting for them is enough; no workgroup barrier.
__device__ __forceinline__ void wave_lds_sync() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}
