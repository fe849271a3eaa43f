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

// Forward, stages 8..15, then canonical (CANON) or < 2q. `x` is left holding, for lane (hb = t>>4, j0 = t&15), the 16 values at
// block h = tile*16 + hb, positions i*16 + j0 (i = 0..15), ready for a coalesced store or a fused epilogue.
template <bool BIG, bool CANON = true>
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
    x[j] = CANON ? csub(v, q) : v;
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

// Eval-domain Galois map for N = 2^16: out[k] = in[k'], 2*brev(k')+1 = (2*brev(k)+1)*g mod 2N. It maps every aligned
// 16-element segment onto an aligned 16-element segment, so 16 adjacent lanes still read one 128-byte line.
__device__ __forceinline__ u32 galois_src_index16(u32 k, u32 g) {
  u32 e = 2 * (__brev(k) >> 16) + 1;
  u32 t = (e * g) & 0x1FFFFu;
  return __brev(t >> 1) >> 16;
}

// ---- standalone kernels: grid = (polynomials, 16 tiles, limb slots) ----
struct Ntt16Args {
  const u64* src;
  u64* dst;
  const ulonglong2* tw;     // forward or inverse table, [nm][65536]
  const ModInfo* mods;
  u64 src_poly_stride, dst_poly_stride;  // elements between polynomials
  u32 skip_beta, skip_alpha, skip_nq;    // as in the generic pass: digit p % skip_beta leaves its own limbs alone
  u32 map_mode;                          // workgroup -> (poly, tile, slot) mapping, see ntt16_map
  u32 galois;                            // inverse first pass only: != 0 reads src through the eval-domain Galois map
  const ulonglong2* scale;               // inverse second pass only: per-slot constant replacing N^-1 (NULL = N^-1)
  unsigned char id[128];
};

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
__device__ __forceinline__ bool ntt16_skip(const Ntt16Args& a, u32 poly, u32 slot) {
  if (!a.skip_beta) return false;
  u32 j = poly % a.skip_beta, lo = j * a.skip_alpha, hi = min(lo + a.skip_alpha, a.skip_nq);
  return slot >= lo && slot < hi;
}
#define NTT16_PROLOGUE                                                            \
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];                                         \
  u32 poly, tile, slot;                                                           \
  ntt16_map(a.map_mode, poly, tile, slot);                                        \
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
  if (a.galois) {
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = src[galois_src_index16(h * 256 + i * 16 + j0, a.galois)];
  } else {
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = src[(size_t)h * 256 + i * 16 + j0];
  }
  if (big) ntt16_inv_blocks<true>(x, tw, mi.m, mi.mu64, tile, sm);
  else ntt16_inv_blocks<false>(x, tw, mi.m, mi.mu64, tile, sm);
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)h * 256 + i * 16 + j0] = x[i];
}
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_inv_rows_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  u64 x[16];
  u64 sc = mi.ninv, scs = mi.ninvs;
  if (a.scale) {
    ulonglong2 v = a.scale[slot];
    sc = v.x;
    scs = v.y;
  }
  if (big) ntt16_inv_rows<true>(x, src, tw, mi.m, sc, scs, tile, sm);
  else ntt16_inv_rows<false>(x, src, tw, mi.m, sc, scs, tile, sm);
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)(i * 16 + r0) * 256 + col0 + col] = x[i];
}

// ---- fused: last forward pass of the ModUp'ed digits + inner product with the evaluation key ----
// For (ciphertext b, extended slot t, tile): acc[b][c][t] = sum_j D_j * evk[j][c][id(t)] * 2^-64, where D_j is the
// forward transform of ext[b][j][t] (slots the digit does not own) or d[b][t] itself (the digit's own limbs,
// already in the evaluation domain). Products are reduced by a Montgomery reduction, hence the 2^-64, which the
// later stages absorb into their constants. Output canonical.
struct FwdInnerArgs {
  const u64* ext;   // [B][beta][next][N], after the row pass
  const u64* d;     // eval domain, limb-vector (b, t) at d + b*d_poly_stride + t*N; read through the Galois map if galois != 0
  u64 d_poly_stride;
  const u64* evk;   // [dnum][2][nm][N]
  u64* acc;         // [B][2][next][N]
  const ulonglong2* tw;
  const ModInfo* mods;
  u32 nlimbs, nq, nm, alpha, beta, next, map_mode, galois;
};

template <bool BIG>
__device__ __forceinline__ void fwd_inner_body(const FwdInnerArgs& a, u32 b, u32 tile, u32 t, u32 id, const ModInfo& mi,
                                               u64* sm) {
  const u32 tid = threadIdx.x, j0 = tid & 15, h = tile * 16 + (tid >> 4);
  const size_t N = 65536;
  const u64 q = mi.m, q2 = 2 * mi.m;
  const ulonglong2* tw = a.tw + (size_t)id * N;
  u64 acc0[16], acc1[16], x[16];
#pragma unroll
  for (int i = 0; i < 16; i++) acc0[i] = acc1[i] = 0;
  for (u32 j = 0; j < a.beta; j++) {
    const u32 lo = j * a.alpha, hi = min(lo + a.alpha, a.nlimbs);
    if (t >= lo && t < hi) {
      const u64* src = a.d + (size_t)b * a.d_poly_stride + (size_t)t * N;
      if (a.galois) {
#pragma unroll
        for (int i = 0; i < 16; i++) x[i] = src[galois_src_index16(h * 256 + i * 16 + j0, a.galois)];
      } else {
#pragma unroll
        for (int i = 0; i < 16; i++) x[i] = src[(size_t)h * 256 + i * 16 + j0];
      }
    } else {
      if (j) __syncthreads();  // the previous digit's transposes are done with the LDS tile
      ntt16_fwd_blocks<BIG, false>(x, a.ext + (((size_t)b * a.beta + j) * a.next + t) * N, tw, q, mi.mu64, tile, sm);
    }
    const u64* kb = a.evk + (((size_t)j * 2 + 0) * a.nm + id) * N + (size_t)h * 256 + j0;
    const u64* ka = kb + (size_t)a.nm * N;
#pragma unroll
    for (int i = 0; i < 16; i++) {
      const u64 eb = kb[i * 16], ea = ka[i * 16];
      Acc128 p0, p1;
      p0.lo = x[i] * eb;
      p0.hi = mul_hi64(x[i], eb);
      p1.lo = x[i] * ea;
      p1.hi = mul_hi64(x[i], ea);
      acc0[i] = csub(acc0[i] + redc(p0, q, mi.minv), q2);
      acc1[i] = csub(acc1[i] + redc(p1, q, mi.minv), q2);
    }
  }
  u64* o0 = a.acc + (((size_t)b * 2 + 0) * a.next + t) * N + (size_t)h * 256 + j0;
  u64* o1 = o0 + (size_t)a.next * N;
#pragma unroll
  for (int i = 0; i < 16; i++) {
    o0[i * 16] = csub(acc0[i], q);
    o1[i * 16] = csub(acc1[i], q);
  }
}

__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_blocks_inner_kernel(FwdInnerArgs a) {
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];
  u32 b, tile, t;
  ntt16_map(a.map_mode, b, tile, t);
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  if ((mi.m >> 52) != 0) fwd_inner_body<true>(a, b, tile, t, id, mi, sm);
  else fwd_inner_body<false>(a, b, tile, t, id, mi, sm);
}

// ---- fused: last forward pass of the ModDown correction + final assembly ----
// out[bc][i] = (acc[bc][i] - NTT(tq[bc][i])) * pinv2[i]  (+ addend), everything in the 2^-64-scaled domain except
// pinv2 = P^-1 * 2^64, so the result is the true key-switch output. addend modes per component c = bc & 1:
// 0 none; 1 the value already in out (in place); 2 add_src read through the Galois map g (HRot's sigma(c0)).
struct FwdFinalArgs {
  const u64* tq;      // [B*2][nlimbs][N], after the row pass
  const u64* acc;     // [B*2][next][N]
  u64* out;           // [B*2][nlimbs][N]
  const u64* add_src; // [B][2][nlimbs][N] (mode 2)
  const ulonglong2* tw;
  const ModInfo* mods;
  const ulonglong2* pinv2;  // [nlimbs]
  u32 nlimbs, next, mode0, mode1, galois, map_mode;
};
template <bool BIG>
__device__ __forceinline__ void fwd_final_body(const FwdFinalArgs& a, u32 bc, u32 tile, u32 i_limb, const ModInfo& mi, u64* sm) {
  const u32 tid = threadIdx.x, j0 = tid & 15, h = tile * 16 + (tid >> 4);
  const size_t N = 65536;
  const u64 q = mi.m, q2 = 2 * mi.m;
  u64 x[16];
  ntt16_fwd_blocks<BIG, false>(x, a.tq + ((size_t)bc * a.nlimbs + i_limb) * N, a.tw + (size_t)i_limb * N, q, mi.mu64, tile, sm);
  const ulonglong2 pv = a.pinv2[i_limb];
  const u64* ac = a.acc + ((size_t)bc * a.next + i_limb) * N + (size_t)h * 256 + j0;
  u64* o = a.out + ((size_t)bc * a.nlimbs + i_limb) * N + (size_t)h * 256 + j0;
  const u32 mode = (bc & 1) ? a.mode1 : a.mode0;
  const u64* as = a.add_src + ((size_t)bc * a.nlimbs + i_limb) * N;
#pragma unroll
  for (int i = 0; i < 16; i++) {
    u64 r = shoup(ac[i * 16] + q2 - x[i], pv.x, pv.y, q);
    if (mode == 1) r = addmod(r, o[i * 16], q);
    else if (mode == 2) r = addmod(r, as[galois_src_index16(h * 256 + i * 16 + j0, a.galois)], q);
    o[i * 16] = r;
  }
}
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_blocks_final_kernel(FwdFinalArgs a) {
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];
  u32 bc, tile, i_limb;
  ntt16_map(a.map_mode, bc, tile, i_limb);
  const ModInfo mi = a.mods[i_limb];
  if ((mi.m >> 52) != 0) fwd_final_body<true>(a, bc, tile, i_limb, mi, sm);
  else fwd_final_body<false>(a, bc, tile, i_limb, mi, sm);
}
