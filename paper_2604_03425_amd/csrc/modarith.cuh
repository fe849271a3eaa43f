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
};

__device__ __forceinline__ u64 mul_hi64(u64 a, u64 b) { return __umul64hi(a, b); }
__device__ __forceinline__ u64 csub(u64 x, u64 m) { return x >= m ? x - m : x; }
__device__ __forceinline__ u64 addmod(u64 a, u64 b, u64 m) { return csub(a + b, m); }
__device__ __forceinline__ u64 submod(u64 a, u64 b, u64 m) { return a >= b ? a - b : a + m - b; }

// x * w mod m for a constant w < m with companion ws = floor(w * 2^64 / m). Any x < 2^64.
// Result in [0, 2m).
__device__ __forceinline__ u64 shoup_lazy(u64 x, u64 w, u64 ws, u64 m) { return x * w - mul_hi64(x, ws) * m; }
__device__ __forceinline__ u64 shoup(u64 x, u64 w, u64 ws, u64 m) { return csub(shoup_lazy(x, w, ws, m), m); }

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
