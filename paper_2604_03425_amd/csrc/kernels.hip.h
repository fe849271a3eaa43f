// Device kernels of the RNS-CKKS hot path (gfx950, wave64).
#pragma once
#include "modarith.hip.h"

#define CKKS_MAX_SLOTS 128   // limb slots addressable by one launch (L+1+K <= 128)
#define NTT_THREADS 256

struct LimbMap {
  unsigned char id[CKKS_MAX_SLOTS];
};

// One pass of a multi-pass transform: stages [s0, s0+k) of the logN-stage butterfly network,
// on tiles of 2^tile_log elements = (hi blocks) x (2^k "mid" values) x (2^logC consecutive "lo" values).
struct NttArgs {
  u64* data;
  const ulonglong2* tw;  // [nm][N] (w, floor(w*2^64/m)); entry 2^s + i is the twiddle of group i at stage s
  const ModInfo* mods;
  u64 poly_stride;       // elements between consecutive polynomials
  u32 logN, s0, k, logC, tile_log;
  u32 skip_beta, skip_alpha, skip_nq;  // skip_beta != 0: poly p is digit p % skip_beta; its own limbs are not touched
  LimbMap ids;
};

// Butterflies are done stage by stage in LDS; values stay canonical in [0, m).
template <bool INV>
__global__ void __launch_bounds__(NTT_THREADS) ntt_pass_kernel(NttArgs a) {
  extern __shared__ u64 sm[];
  const u32 poly = blockIdx.x, tile_id = blockIdx.y, slot = blockIdx.z;
  if (a.skip_beta) {
    u32 j = poly % a.skip_beta;
    u32 lo = j * a.skip_alpha, hi = min(lo + a.skip_alpha, a.skip_nq);
    if (slot >= lo && slot < hi) return;
  }
  const u32 id = a.ids.id[slot];
  const ModInfo mi = a.mods[id];
  const u64 m = mi.m;
  const u32 N = 1u << a.logN;
  const ulonglong2* tw = a.tw + (size_t)id * N;
  u64* base = a.data + (size_t)poly * a.poly_stride + (size_t)slot * N;

  const u32 tile = 1u << a.tile_log;
  const u32 k = a.k, logC = a.logC;
  const u32 lo_bits = a.logN - a.s0 - k;          // index bits below the stages of this pass
  const u32 tiles_lo = 1u << (lo_bits - logC);
  const u32 hl_log = a.tile_log - k - logC;        // log2(hi blocks per tile)
  const u32 hi0 = (tile_id / tiles_lo) << hl_log;
  const u32 lo0 = (tile_id % tiles_lo) << logC;
  const u32 cmask = (1u << logC) - 1, kmask = (1u << k) - 1;

  for (u32 e = threadIdx.x; e < tile; e += NTT_THREADS) {
    u32 lo = e & cmask, mid = (e >> logC) & kmask, hl = e >> (logC + k);
    size_t g = ((size_t)(hi0 + hl) << (a.logN - a.s0)) | ((size_t)mid << lo_bits) | (lo0 + lo);
    sm[e] = base[g];
  }
  __syncthreads();

  for (u32 uu = 0; uu < k; uu++) {
    const u32 u = INV ? (k - 1 - uu) : uu;
    const u32 sh = k - 1 - u;
    for (u32 bf = threadIdx.x; bf < tile / 2; bf += NTT_THREADS) {
      u32 lo = bf & cmask, pi = (bf >> logC) & (kmask >> 1), hl = bf >> (logC + k - 1);
      u32 grp = pi >> sh, pos = pi & ((1u << sh) - 1);
      u32 mid_a = (grp << (sh + 1)) | pos;
      u32 ea = (((hl << k) | mid_a) << logC) | lo;
      u32 eb = ea + ((1u << sh) << logC);
      ulonglong2 w = tw[(1u << (a.s0 + u)) + ((hi0 + hl) << u) + grp];
      u64 U = sm[ea], V = sm[eb];
      if (!INV) {
        V = shoup(V, w.x, w.y, m);
        sm[ea] = addmod(U, V, m);
        sm[eb] = submod(U, V, m);
      } else {
        sm[ea] = addmod(U, V, m);
        sm[eb] = shoup(submod(U, V, m), w.x, w.y, m);
      }
    }
    __syncthreads();
  }

  const bool scale = INV && a.s0 == 0;
  for (u32 e = threadIdx.x; e < tile; e += NTT_THREADS) {
    u32 lo = e & cmask, mid = (e >> logC) & kmask, hl = e >> (logC + k);
    size_t g = ((size_t)(hi0 + hl) << (a.logN - a.s0)) | ((size_t)mid << lo_bits) | (lo0 + lo);
    u64 v = sm[e];
    if (scale) v = shoup(v, mi.ninv, mi.ninvs, m);
    base[g] = v;
  }
}

// ---------------------------------------------------------------------------------------------
// Galois automorphism.
// Evaluation domain (bit-reversed order): out[k] = in[k'], 2*brev(k')+1 = (2*brev(k)+1)*g mod 2N.
__device__ __forceinline__ u32 galois_src_index(u32 k, u32 g, u32 logN) {
  u32 e = 2 * (__brev(k) >> (32 - logN)) + 1;
  u32 t = (e * g) & ((2u << logN) - 1);
  return __brev(t >> 1) >> (32 - logN);
}

struct AutoArgs {
  u64* out;
  const u64* in;
  const ModInfo* mods;
  u64 out_poly_stride, in_poly_stride;
  u32 logN, g, g_inv, eval_domain;
  LimbMap ids;
};
__global__ void __launch_bounds__(256) automorph_kernel(AutoArgs a) {
  const u32 poly = blockIdx.z, slot = blockIdx.y;
  const u32 N = 1u << a.logN;
  const u32 k = blockIdx.x * blockDim.x + threadIdx.x;
  const u64* in = a.in + (size_t)poly * a.in_poly_stride + (size_t)slot * N;
  u64* out = a.out + (size_t)poly * a.out_poly_stride + (size_t)slot * N;
  if (a.eval_domain) {
    out[k] = in[galois_src_index(k, a.g, a.logN)];
  } else {
    // out[t] = +-in[j] with t = j*g mod 2N; gather form: j = t*g^-1 mod 2N, sign from whether j*g wraps oddly.
    const u64 m = a.mods[a.ids.id[slot]].m;
    u32 j2 = (k * a.g_inv) & (2 * N - 1);   // index in [0, 2N) whose image is X^k (up to sign)
    u32 j = j2 & (N - 1);
    // X^j -> X^(j*g mod 2N); the image lands on +X^k if (j*g mod 2N) == k, on -X^k if it equals k + N.
    u32 t = (j * a.g) & (2 * N - 1);
    u64 v = in[j];
    out[k] = (t == k) ? v : (v ? m - v : 0);
  }
}

// ---------------------------------------------------------------------------------------------
// Base conversion. For a source basis {c_i} and one coefficient with residues x_i:
//   y_i = [x_i * (C/c_i)^-1]_{c_i};  nneg = #{i : y_i > c_i/2}  (those have centred representative y_i - c_i)
//   out_t = sum_i y_i * [(C/c_i)]_{m_t} + nneg * [-C]_{m_t}   (mod m_t)
// The constants are stored in Montgomery form (times 2^64 mod m_t); the lazy sum of 30-bit partial products is
// reduced once per output by a Montgomery reduction, which gives the plain product sum back.
#define BCONV_THREADS 256
#define M30 0x3FFFFFFFu

// Sum over up to MAXLEN sources (+ the nneg term) for one output, whose MAXLEN + 1 constants are contiguous at
// `crow` (rows beyond the source count are zero, row MAXLEN holds [-C]). Returns the canonical residue.
// NARROW: three-sum accumulation with the base-2^30 reduction (constants carry 2^90); otherwise four sums, a
// 128-bit value and one 2^-64 Montgomery reduction (constants carry 2^64).
template <int MAXLEN, bool NARROW>
__device__ __forceinline__ u64 bconv_dot(const u32 (&y0)[MAXLEN], const u32 (&y1)[MAXLEN], u32 nneg,
                                         const u64* __restrict__ crow, const ModInfo& mi) {
  if (NARROW) {
    u64 r = 0;
#pragma unroll
    for (int i0 = 0; i0 < MAXLEN; i0 += 15) {
      Dot30N dd;
      dot30n_init(dd);
#pragma unroll
      for (int i = i0; i < i0 + 15 && i < MAXLEN; i++) {
        const u64 c = crow[i];
        dot30n_mac(dd, y0[i], y1[i], (u32)c & M30, (u32)(c >> 30));
      }
      if (i0 == 0) {
        const u64 c = crow[MAXLEN];
        dd.a += (u64)nneg * ((u32)c & M30);
        dd.b += (u64)nneg * (u32)(c >> 30);
      }
      r += dot30n_redc90(dd, mi.m, mi.minv);   // each part < m + 2^34
    }
    if (MAXLEN > 15) r = csub(r, 2 * mi.m);   // three chunks: r < 4m
    return csub(r, mi.m);
  }
  Acc128 V = {0, 0};
#pragma unroll
  for (int i0 = 0; i0 < MAXLEN; i0 += 15) {
    Dot30 dd;
    dot30_init(dd);
#pragma unroll
    for (int i = i0; i < i0 + 15 && i < MAXLEN; i++) {
      const u64 c = crow[i];
      dot30_mac(dd, y0[i], y1[i], (u32)c & M30, (u32)(c >> 30));
    }
    if (i0 == 0) {
      const u64 c = crow[MAXLEN];
      dd.s00 += (u64)nneg * ((u32)c & M30);
      dd.s01 += (u64)nneg * (u32)(c >> 30);
    }
    Acc128 part = dot30_value(dd);
    if (i0 == 0) {
      V = part;
    } else {
      V.lo += part.lo;
      V.hi += part.hi + (V.lo < part.lo ? 1ull : 0ull);
    }
  }
  u64 r = redc(V, mi.m, mi.minv);
  if (MAXLEN > 15) r = csub(r, 2 * mi.m);  // three chunks of 15 products: r < 4m
  return csub(r, mi.m);
}

// ModUp: for digit j (limbs [lo_j, hi_j) of the coefficient-domain input), write every other slot of the extended
// basis. Constants: [digit][target][MAXLEN+1]: entry i < len = (Q_j/q_i), entries len..MAXLEN-1 = 0, entry MAXLEN = -Q_j,
// all in Montgomery form.
struct ModUpArgs {
  const u64* dcoef;         // [B][nlimbs][N]
  u64* ext;                 // [B][beta][next][N]
  const ModInfo* mods;
  const ulonglong2* inv;    // [beta][alpha]  ((Q_j/q_i)^-1 mod q_i, shoup)
  const u64* mat;           // [beta][next][MAXLEN+1]
  u32 logN, nlimbs, nq, alpha, beta, next;
};
// PRESCALED: the input already holds y_i (the inverse transform folded (Q_j/q_i)^-1 into its 1/N scaling).
// EPT: adjacent coefficients per lane (16-byte accesses for EPT = 2); the constants of an output are fetched once
// per lane through scalar loads and reused for all of them.
// The tables and buffers are also passed as separate no-alias parameters: only then can the compiler see that the
// stores never touch the constants and fetch those through wave-uniform scalar loads (splitting them on the
// scalar unit as well).
template <int MAXLEN, bool PRESCALED, int EPT, bool NARROW>
__global__ void __launch_bounds__(BCONV_THREADS) modup_kernel(ModUpArgs a, const u64* __restrict__ dcoef,
                                                              u64* __restrict__ ext, const ModInfo* __restrict__ mods,
                                                              const u64* __restrict__ matrix) {
  const u32 N = 1u << a.logN;
  const u32 n = (blockIdx.x * BCONV_THREADS + threadIdx.x) * EPT;
  const u32 j = blockIdx.y, b = blockIdx.z;
  const u32 lo = j * a.alpha, hi = min(lo + a.alpha, a.nlimbs), len = hi - lo;
  const u64* d = dcoef + ((size_t)b * a.nlimbs + lo) * N + n;
  u32 y0[EPT][MAXLEN], y1[EPT][MAXLEN], nneg[EPT];
#pragma unroll
  for (int e = 0; e < EPT; e++) nneg[e] = 0;
#pragma unroll
  for (int i = 0; i < MAXLEN; i++) {
#pragma unroll
    for (int e = 0; e < EPT; e++) y0[e][i] = y1[e][i] = 0;
    if ((u32)i < len) {
      const u64 m = mods[lo + i].m;
      u64 yv[EPT];
      if (EPT == 2) {
        const ulonglong2 v = *(const ulonglong2*)(d + (size_t)i * N);
        yv[0] = v.x;
        yv[EPT - 1] = v.y;
      } else {
        yv[0] = d[(size_t)i * N];
      }
#pragma unroll
      for (int e = 0; e < EPT; e++) {
        u64 y = yv[e];
        if (!PRESCALED) {
          ulonglong2 c = a.inv[j * a.alpha + i];
          y = shoup(y, c.x, c.y, m);
        }
        nneg[e] += (y > (m >> 1)) ? 1u : 0u;
        y0[e][i] = (u32)y & M30;
        y1[e][i] = (u32)(y >> 30);
      }
    }
  }
  const u64* mat = matrix + (size_t)j * a.next * (MAXLEN + 1);
  u64* out = ext + (((size_t)b * a.beta + j) * a.next) * N + n;
  for (u32 t = 0; t < a.next; t++) {
    if (t >= lo && t < hi) continue;
    const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
    const ModInfo mi = mods[id];
    u64 r[EPT];
#pragma unroll
    for (int e = 0; e < EPT; e++) r[e] = bconv_dot<MAXLEN, NARROW>(y0[e], y1[e], nneg[e], mat + (size_t)t * (MAXLEN + 1), mi);
    if (EPT == 2) *(ulonglong2*)(out + (size_t)t * N) = ulonglong2{r[0], r[EPT - 1]};
    else out[(size_t)t * N] = r[0];
  }
}

// Inner product with the evaluation key over the extended basis, eval domain:
// acc[b][c][t][n] = sum_j D_j[t][n] * evk[j][c][id(t)][n], D_j[t] = d[b][t] on digit j's own limbs, ext[b][j][t] else.
struct InnerArgs {
  const u64* d;     // [B][nlimbs][N] eval, polynomial b at d + b*d_stride
  const u64* ext;   // [B][beta][next][N] eval
  const u64* evk;   // [dnum][2][nm][N]
  u64* acc;         // [B][2][next][N]
  const ModInfo* mods;
  u32 logN, nlimbs, nq, nm, alpha, beta, next;
  u64 d_stride;
};
__global__ void __launch_bounds__(256) inner_kernel(InnerArgs a) {
  const u32 N = 1u << a.logN;
  const u32 lin = xcd_swizzled_linear_id();   // batch-innermost, and workgroups sharing a key slice share an XCD
  const u32 b = lin % gridDim.x, t = lin / (gridDim.x * gridDim.y);
  const u32 n = ((lin / gridDim.x) % gridDim.y) * 256 + threadIdx.x;
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  Acc128 sb = {0, 0}, sa = {0, 0};
  for (u32 j = 0; j < a.beta; j++) {
    const u32 lo = j * a.alpha, hi = min(lo + a.alpha, a.nlimbs);
    u64 x = (t >= lo && t < hi) ? a.d[(size_t)b * a.d_stride + (size_t)t * N + n]
                                : a.ext[(((size_t)b * a.beta + j) * a.next + t) * N + n];
    mac128(sb, x, a.evk[(((size_t)j * 2 + 0) * a.nm + id) * N + n]);
    mac128(sa, x, a.evk[(((size_t)j * 2 + 1) * a.nm + id) * N + n]);
  }
  a.acc[(((size_t)b * 2 + 0) * a.next + t) * N + n] = reduce128(sb, mi);
  a.acc[(((size_t)b * 2 + 1) * a.next + t) * N + n] = reduce128(sa, mi);
}

// ModDown base conversion P -> Q_l of the special limbs of acc (coefficient domain after INTT):
// tq[bc][i][n] = sum_k y_k * (P/p_k mod q_i) + nneg * (-P mod q_i), y_k = [x_k (P/p_k)^-1]_{p_k}.
struct ModDownArgs {
  const u64* acc;         // [B*2][next][N]; special limbs at slots nlimbs..next-1, coefficient domain
  u64* tq;                // [B*2][nlimbs][N]
  const ModInfo* mods;
  const ulonglong2* inv;  // [K]
  const u64* mat;         // [nlimbs][MAXLEN+1], Montgomery form
  u32 logN, nlimbs, nq, K, next;
  u32 src_slot;           // slot of the first source limb inside a row of `acc` (nlimbs for a key switch)
  u32 src_id0;            // modulus id of the first source limb (nq for a key switch)
};
template <int MAXLEN, bool PRESCALED, int EPT, bool NARROW>
__global__ void __launch_bounds__(BCONV_THREADS) moddown_kernel(ModDownArgs a, const u64* __restrict__ acc,
                                                                u64* __restrict__ tq, const ModInfo* __restrict__ mods,
                                                                const u64* __restrict__ matrix) {
  const u32 N = 1u << a.logN;
  const u32 n = (blockIdx.x * BCONV_THREADS + threadIdx.x) * EPT;
  const u32 bc = blockIdx.y;
  const u64* x = acc + ((size_t)bc * a.next + a.src_slot) * N + n;
  u32 y0[EPT][MAXLEN], y1[EPT][MAXLEN], nneg[EPT];
#pragma unroll
  for (int e = 0; e < EPT; e++) nneg[e] = 0;
#pragma unroll
  for (int k = 0; k < MAXLEN; k++) {
#pragma unroll
    for (int e = 0; e < EPT; e++) y0[e][k] = y1[e][k] = 0;
    if ((u32)k < a.K) {
      const u64 m = mods[a.src_id0 + k].m;
      u64 yv[EPT];
      if (EPT == 2) {
        const ulonglong2 v = *(const ulonglong2*)(x + (size_t)k * N);
        yv[0] = v.x;
        yv[EPT - 1] = v.y;
      } else {
        yv[0] = x[(size_t)k * N];
      }
#pragma unroll
      for (int e = 0; e < EPT; e++) {
        u64 y = yv[e];
        if (!PRESCALED) {
          ulonglong2 c = a.inv[k];
          y = shoup(y, c.x, c.y, m);
        }
        nneg[e] += (y > (m >> 1)) ? 1u : 0u;
        y0[e][k] = (u32)y & M30;
        y1[e][k] = (u32)(y >> 30);
      }
    }
  }
  u64* out = tq + (size_t)bc * a.nlimbs * N + n;
  for (u32 i = 0; i < a.nlimbs; i++) {
    const ModInfo mi = mods[i];
    u64 r[EPT];
#pragma unroll
    for (int e = 0; e < EPT; e++) r[e] = bconv_dot<MAXLEN, NARROW>(y0[e], y1[e], nneg[e], matrix + (size_t)i * (MAXLEN + 1), mi);
    if (EPT == 2) *(ulonglong2*)(out + (size_t)i * N) = ulonglong2{r[0], r[EPT - 1]};
    else out[(size_t)i * N] = r[0];
  }
}

// Final assembly, eval domain: r = (acc - tq) * P^-1 mod q_i;  out = r (+ out if add_mask bit c is set).
struct FinalArgs {
  const u64* acc;   // [B][2][next][N]
  const u64* tq;    // [B][2][nlimbs][N] (eval domain)
  u64* out;         // [B][2][nlimbs][N]
  const ModInfo* mods;
  const ulonglong2* pinv;  // [nlimbs]
  u32 logN, nlimbs, next, add_mask;
};
__global__ void __launch_bounds__(256) ks_final_kernel(FinalArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = blockIdx.x * 256 + threadIdx.x;
  const u32 i = blockIdx.y, bc = blockIdx.z, c = bc & 1;
  const u64 m = a.mods[i].m;
  ulonglong2 pv = a.pinv[i];
  u64 x = a.acc[((size_t)bc * a.next + i) * N + n];
  u64 t = a.tq[((size_t)bc * a.nlimbs + i) * N + n];
  u64 r = shoup(submod(x, t, m), pv.x, pv.y, m);
  size_t o = ((size_t)bc * a.nlimbs + i) * N + n;
  if ((a.add_mask >> c) & 1) r = addmod(r, a.out[o], m);
  a.out[o] = r;
}

// HMult tensor product: d0 -> out[b][0], d1 -> out[b][1], d2 -> d2[b].
struct TensorArgs {
  const u64 *cta, *ctb;
  u64 *out, *d2;
  const ModInfo* mods;
  u32 logN, nlimbs;
};
__global__ void __launch_bounds__(256) tensor_kernel(TensorArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = blockIdx.x * 256 + threadIdx.x;
  const u32 i = blockIdx.y, b = blockIdx.z;
  const ModInfo mi = a.mods[i];
  size_t o0 = (((size_t)b * 2 + 0) * a.nlimbs + i) * N + n, o1 = o0 + (size_t)a.nlimbs * N;
  u64 a0 = a.cta[o0], a1 = a.cta[o1], b0 = a.ctb[o0], b1 = a.ctb[o1];
  a.out[o0] = mulmod(a0, b0, mi);
  Acc128 s = {0, 0};
  mac128(s, a0, b1);
  mac128(s, a1, b0);
  a.out[o1] = reduce128(s, mi);
  a.d2[((size_t)b * a.nlimbs + i) * N + n] = mulmod(a1, b1, mi);
}

// Three-component product kept for a later relinearisation: out[b] = (a0 b0, a0 b1 + a1 b0, a1 b1) (+ acc[b]).
// acc may be out itself: every lane reads its own words before it writes them.
struct TensorAccArgs {
  const u64 *cta, *ctb, *acc;  // [B][2][nlimbs][N], [B][2][nlimbs][N], null or [B][3][nlimbs][N]
  u64* out;                    // [B][3][nlimbs][N]
  const ModInfo* mods;
  u32 logN, nlimbs;
};
__global__ void __launch_bounds__(256) tensor_acc_kernel(TensorAccArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = blockIdx.x * 256 + threadIdx.x;
  const u32 i = blockIdx.y, b = blockIdx.z;
  const ModInfo mi = a.mods[i];
  const size_t pl = (size_t)a.nlimbs * N;
  const size_t i0 = (size_t)b * 2 * pl + (size_t)i * N + n, i1 = i0 + pl;
  const size_t o0 = (size_t)b * 3 * pl + (size_t)i * N + n;
  u64 a0 = a.cta[i0], a1 = a.cta[i1], b0 = a.ctb[i0], b1 = a.ctb[i1];
  u64 t0 = mulmod(a0, b0, mi);
  Acc128 s = {0, 0};
  mac128(s, a0, b1);
  mac128(s, a1, b0);
  u64 t1 = reduce128(s, mi);
  u64 t2 = mulmod(a1, b1, mi);
  if (a.acc) {
    t0 = addmod(t0, a.acc[o0], mi.m);
    t1 = addmod(t1, a.acc[o0 + pl], mi.m);
    t2 = addmod(t2, a.acc[o0 + 2 * pl], mi.m);
  }
  a.out[o0] = t0;
  a.out[o0 + pl] = t1;
  a.out[o0 + 2 * pl] = t2;
}

// out[b][c] = in[b][c] for c < 2, in holding three components per ciphertext (two adjacent words per lane).
__global__ void __launch_bounds__(256) first_two_components_kernel(const ulonglong2* __restrict__ in,
                                                                   ulonglong2* __restrict__ out, size_t pl2) {
  const size_t k = (size_t)blockIdx.x * 256 + threadIdx.x;   // < 2 * pl2: both kept components of one ciphertext
  if (k >= 2 * pl2) return;
  const size_t b = blockIdx.y;
  out[b * 2 * pl2 + k] = in[b * 3 * pl2 + k];
}

// A ciphertext lifted to the extended basis as (P c0, P c1): out[bc][t] = P * in[bc][t] on the main-prime slots
// t < nlimbs (with the factor 2^-64 on integer-class moduli, the form the key-switch accumulators have there), 0 on
// the special-prime slots. grid = (N/512, next, 2B), two adjacent coefficients per lane.
struct LiftArgs {
  const u64* in;   // [2B][nlimbs][N]
  u64* out;        // [2B][next][N]
  const ModInfo* mods;
  u32 logN, nlimbs, next;
  unsigned char fp[128];   // per main-prime slot: 1 = double-precision class (plain residues)
};
__global__ void __launch_bounds__(256) lift_qp_kernel(LiftArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = (blockIdx.x * 256 + threadIdx.x) * 2, t = blockIdx.y, bc = blockIdx.z;
  ulonglong2 r = {0, 0};
  if (t < a.nlimbs) {
    const ModInfo mi = a.mods[t];
    const ulonglong2 v = *(const ulonglong2*)(a.in + ((size_t)bc * a.nlimbs + t) * N + n);
    if (a.fp[t]) {
      r = ulonglong2{mulmod(v.x, mi.pmod, mi), mulmod(v.y, mi.pmod, mi)};
    } else {
      Acc128 p0 = {v.x * mi.pmod, mul_hi64(v.x, mi.pmod)}, p1 = {v.y * mi.pmod, mul_hi64(v.y, mi.pmod)};
      r = ulonglong2{csub(redc(p0, mi.m, mi.minv), mi.m), csub(redc(p1, mi.m, mi.minv), mi.m)};
    }
  }
  *(ulonglong2*)(a.out + ((size_t)bc * a.next + t) * N + n) = r;
}

// BSGS inner sums for several giant steps and polynomials at once:
//   out_g[b][c][i][n] = sum_{s<n1} src_s[b][c][i][n] * pt[g][s][i][n],  src_0 = ct_in, src_s = baby[s-1].
// One launch covers the limbs of one arithmetic kind (pmacc_fp_kernel, pmacc_int_kernel below).
struct PmaccArgs {
  const u64* ct_in;   // [B][2][nlimbs][N]
  const u64* baby;    // [n1-1][B][2][nlimbs][N]
  const u64* pt;      // [n2][n1][nlimbs][N]
  u64* out0;          // destination of giant step g0 (the caller's output when g0 == 0)
  u64* out_rest;      // [GT-1][B][2][nlimbs][N]: destinations of giant steps g0+1 .. g0+GT-1
  const ModInfo* mods;
  u32 logN, nlimbs, n1, B, g0, ng;  // ng <= GT giant steps are computed
  u32 ngt;                          // pmacc_fp_kernel: the launch covers ngt consecutive tiles of NG giant steps
  unsigned char limbs[128];         // grid.z index -> limb (the launch covers the limbs of one arithmetic kind)
  unsigned char mod_ids[128];       // grid.z index -> modulus of that limb (differs from the limb index when the
                                    // polynomials are in an extended basis: main primes first, then special ones)
};
#define PMACC_TILE 24     // giant steps whose inner sums are held in the workspace at once

// Inner sums on double-precision moduli (q < 2^50), register-tiled like a small matrix product: a lane owns
// one coefficient position and keeps the running sums of PMACC_FP_P polynomials x NG giant steps (one double each:
// every product is reduced on the spot with 5 FP64 instructions), so per baby step it loads P ciphertext words and
// NG plaintext words for P * NG multiply-adds: 8/P + 8/NG bytes per multiply-add instead of 16. grid =
// (ceil(2B / P) * ngt, N / 256, limbs of the class): polynomial groups innermost, then the ngt tiles of NG giant
// steps, so the workgroups that share a plaintext tile or a set of baby-step words run together on one XCD and
// find each other's fetches in its L2 (the HBM read counter equals one pass over the plaintexts and the baby steps).
#define PMACC_FP_P 8
template <int NG>
__global__ void __launch_bounds__(256) pmacc_fp_kernel(PmaccArgs a) {
  constexpr int P = PMACC_FP_P;
  const u32 N = 1u << a.logN;
  const u32 lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  u32 xi, group;
  // when the number of (block, limb) groups allows, a whole group is placed on one XCD (whose L2 then serves the
  // shared words to all of its workgroups) and eight consecutive groups run side by side
  if (((gridDim.y * gridDim.z) & 7) == 0) {
    const u32 rest = lin >> 3;
    xi = rest % gridDim.x;
    group = (lin & 7) + 8 * (rest / gridDim.x);
  } else {
    xi = lin % gridDim.x;
    group = lin / gridDim.x;
  }
  const u32 npg = gridDim.x / a.ngt, pg = xi % npg, gt = xi / npg;
  const u32 nb = group % gridDim.y, i = a.limbs[group / gridDim.y];
  const u32 n = nb * 256 + threadIdx.x;
  const ModInfo mi = a.mods[a.mod_ids[group / gridDim.y]];
  const double q = mi.qd, qinv = mi.qinv;
  const u32 npoly = 2 * a.B;
  const size_t ct_sz = (size_t)npoly * a.nlimbs * N;
  const size_t pt_g = (size_t)a.n1 * a.nlimbs * N;
  size_t o[P];   // the last group may be short: its surplus lanes recompute the last polynomial and store nothing
#pragma unroll
  for (int p = 0; p < P; p++) o[p] = ((size_t)min(pg * P + p, npoly - 1) * a.nlimbs + i) * N + n;
  double s[P][NG];
#pragma unroll
  for (int p = 0; p < P; p++)
#pragma unroll
    for (int g = 0; g < NG; g++) s[p][g] = 0.0;
  for (u32 k = 0; k < a.n1; k++) {
    const u64* src = k == 0 ? a.ct_in : a.baby + (size_t)(k - 1) * ct_sz;
    const u64* w = a.pt + (size_t)(a.g0 + gt * NG) * pt_g + ((size_t)k * a.nlimbs + i) * N + n;
    u64 xr[P], cr[NG];
#pragma unroll
    for (int p = 0; p < P; p++) xr[p] = src[o[p]];
#pragma unroll
    for (int g = 0; g < NG; g++) cr[g] = w[(size_t)g * pt_g];
    double c[NG];
#pragma unroll
    for (int g = 0; g < NG; g++) c[g] = u2d(cr[g]);
#pragma unroll
    for (int p = 0; p < P; p++) {
      const double x = u2d(xr[p]);
#pragma unroll
      for (int g = 0; g < NG; g++) s[p][g] += fp_mulmod_var(x, c[g], qinv, q);
    }
    // each product is below 0.75 q in magnitude: four of them and a folded sum stay below 2^52. A separate
    // (wave-uniform) branch, so that the reduction is not computed and discarded on the other three steps.
    if ((k & 3) == 3) {
#pragma unroll
      for (int p = 0; p < P; p++)
#pragma unroll
        for (int g = 0; g < NG; g++) s[p][g] = fp_reduce(s[p][g], qinv, q);
    }
  }
#pragma unroll
  for (int p = 0; p < P; p++) {
    if (pg * P + p >= npoly) break;
#pragma unroll
    for (int g = 0; g < NG; g++) {
      const u32 rel = gt * NG + g;   // giant step relative to the launch's first one
      u64* dst = (rel == 0 ? a.out0 : a.out_rest + (size_t)(rel - 1) * ct_sz) + o[p];
      *dst = d2u_canon(fp_reduce(s[p][g], qinv, q), q);
    }
  }
}

// The register-tiled form for integer-class moduli (q < 2^60): a lane owns one coefficient position of
// PMACC_INT_P polynomials x NG giant steps, each running sum held as four carry-free sums of 30-bit partial products
// (folded to a canonical residue every 15 baby steps and re-seeded with it: 15 products below 2^60 plus the seed
// stay below 2^64). Per baby step P ciphertext words and NG plaintext words are loaded for P * NG multiply-adds. Grid and
// placement as for pmacc_fp_kernel.
#define PMACC_INT_P 4
template <int NG>
__global__ void __launch_bounds__(256) pmacc_int_kernel(PmaccArgs a) {
  constexpr int P = PMACC_INT_P;
  const u32 N = 1u << a.logN;
  const u32 lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  u32 xi, group;
  if (((gridDim.y * gridDim.z) & 7) == 0) {
    const u32 rest = lin >> 3;
    xi = rest % gridDim.x;
    group = (lin & 7) + 8 * (rest / gridDim.x);
  } else {
    xi = lin % gridDim.x;
    group = lin / gridDim.x;
  }
  const u32 gt = xi % a.ngt, pg = xi / a.ngt;   // the giant tiles of one polynomial group are adjacent
  const u32 nb = group % gridDim.y, i = a.limbs[group / gridDim.y];
  const u32 n = nb * 256 + threadIdx.x;
  const ModInfo mi = a.mods[a.mod_ids[group / gridDim.y]];
  const u32 npoly = 2 * a.B;
  const size_t ct_sz = (size_t)npoly * a.nlimbs * N;
  const size_t pt_g = (size_t)a.n1 * a.nlimbs * N;
  size_t o[P];   // a short last group recomputes the last polynomial in its surplus lanes and stores nothing for them
#pragma unroll
  for (int p = 0; p < P; p++) o[p] = ((size_t)min(pg * P + p, npoly - 1) * a.nlimbs + i) * N + n;
  Dot30 dd[P][NG];
#pragma unroll
  for (int p = 0; p < P; p++)
#pragma unroll
    for (int g = 0; g < NG; g++) dot30_init(dd[p][g]);
  for (u32 k = 0, pending = 0; k < a.n1; k++) {
    const u64* src = k == 0 ? a.ct_in : a.baby + (size_t)(k - 1) * ct_sz;
    const u64* w = a.pt + (size_t)(a.g0 + gt * NG) * pt_g + ((size_t)k * a.nlimbs + i) * N + n;
    u64 xr[P], cr[NG];
#pragma unroll
    for (int p = 0; p < P; p++) xr[p] = src[o[p]];
#pragma unroll
    for (int g = 0; g < NG; g++) cr[g] = w[(size_t)g * pt_g];
    u32 c0[NG], c1[NG];
#pragma unroll
    for (int g = 0; g < NG; g++) {
      c0[g] = (u32)cr[g] & M30;
      c1[g] = (u32)(cr[g] >> 30);
    }
#pragma unroll
    for (int p = 0; p < P; p++) {
      const u32 x0 = (u32)xr[p] & M30, x1 = (u32)(xr[p] >> 30);
#pragma unroll
      for (int g = 0; g < NG; g++) dot30_mac(dd[p][g], x0, x1, c0[g], c1[g]);
    }
    if (++pending == 15) {   // wave-uniform branch
      pending = 0;
#pragma unroll
      for (int p = 0; p < P; p++)
#pragma unroll
        for (int g = 0; g < NG; g++) {
          const u64 r = reduce128(dot30_value(dd[p][g]), mi);
          dot30_init(dd[p][g]);
          dd[p][g].s00 = r;
        }
    }
  }
#pragma unroll
  for (int p = 0; p < P; p++) {
    if (pg * P + p >= npoly) break;
#pragma unroll
    for (int g = 0; g < NG; g++) {
      const u32 rel = gt * NG + g;
      u64* dst = (rel == 0 ? a.out0 : a.out_rest + (size_t)(rel - 1) * ct_sz) + o[p];
      *dst = reduce128(dot30_value(dd[p][g]), mi);
    }
  }
}

// out = out + in (mod q_i) on [npoly][nlimbs][N]
struct AddArgs {
  u64* out;
  const u64* in;
  const ModInfo* mods;
  u32 logN, nlimbs;
};
__global__ void __launch_bounds__(256) addto_kernel(AddArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = blockIdx.x * 256 + threadIdx.x;
  const u32 i = blockIdx.y, p = blockIdx.z;
  const u64 m = a.mods[i].m;
  size_t o = ((size_t)p * a.nlimbs + i) * N + n;
  a.out[o] = addmod(a.out[o], a.in[o], m);
}

// Pointwise helpers of the public calls: out = ct * pt (plaintext broadcast over the polynomials) and out = a + b.
struct PointwiseArgs {
  u64* out;
  const u64 *a, *b;
  const ModInfo* mods;
  u32 logN, nlimbs, b_broadcast;  // b_broadcast: b is [nlimbs][N], shared by every polynomial
};
__global__ void __launch_bounds__(256) pmult_kernel(PointwiseArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = (blockIdx.x * 256 + threadIdx.x) * 2;
  const u32 i = blockIdx.y, p = blockIdx.z;
  const ModInfo mi = a.mods[i];
  const size_t o = ((size_t)p * a.nlimbs + i) * N + n;
  const ulonglong2 x = *(const ulonglong2*)(a.a + o);
  const ulonglong2 y = *(const ulonglong2*)(a.b + (a.b_broadcast ? (size_t)i * N + n : o));
  *(ulonglong2*)(a.out + o) = ulonglong2{mulmod(x.x, y.x, mi), mulmod(x.y, y.y, mi)};
}
__global__ void __launch_bounds__(256) add_kernel(PointwiseArgs a) {
  const u32 N = 1u << a.logN;
  const u32 n = (blockIdx.x * 256 + threadIdx.x) * 2;
  const u32 i = blockIdx.y, p = blockIdx.z;
  const u64 m = a.mods[i].m;
  const size_t o = ((size_t)p * a.nlimbs + i) * N + n;
  const ulonglong2 x = *(const ulonglong2*)(a.a + o);
  const ulonglong2 y = *(const ulonglong2*)(a.b + o);
  *(ulonglong2*)(a.out + o) = ulonglong2{addmod(x.x, y.x, m), addmod(x.y, y.y, m)};
}

// Plain copy of known size (16 bytes per lane): the calibration kernel for the HBM byte counters.
__global__ void __launch_bounds__(256) ckks_prof_copy_kernel(const ulonglong2* __restrict__ in, ulonglong2* __restrict__ out,
                                                              size_t n) {
  const size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  if (i < n) out[i] = in[i];
}
