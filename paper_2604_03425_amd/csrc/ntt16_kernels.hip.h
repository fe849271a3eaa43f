// Kernels of the N = 2^16 path: the four transform passes and the two fused last-pass kernels of key switching.
// Each kernel picks, per modulus (uniform per workgroup), the double-precision bodies (q < 2^50), the integer
// bodies without butterfly corrections (q < 2^52) or the Harvey bodies (q < 2^60). The class also fixes the
// format of the data between the two passes of a transform (reduced doubles / lazy integers) and of the
// constants passed in 16-byte slots (double2 / Shoup pair).
#pragma once
#include "ntt16.hip.h"
#include "ntt16fp.hip.h"

// ---- standalone passes: grid = (polynomials, 16 tiles, limb slots) ----
// A batched rotation may give every ciphertext its own Galois element and key: the kernels then take both from
// small per-ciphertext tables carried in the kernel arguments (at most this many ciphertexts per launch sequence).
#define KS_MULTI_MAX 64

struct Ntt16Args {
  const u64* src;
  u64* dst;
  const ulonglong2* tw;     // integer table (forward or inverse), [nm][65536]
  const double* twfp;       // double table, same indexing (rows of moduli >= 2^50 unused)
  const ModInfo* mods;
  u64 src_poly_stride, dst_poly_stride;  // elements between polynomials
  u32 skip_beta, skip_alpha, skip_nq;    // digit p % skip_beta leaves its own limbs alone (ModUp'ed digits)
  u32 map_mode;                          // workgroup -> (poly, tile, slot) mapping, see ntt16_map
  u32 raw_out;                           // forward last pass, double-precision class only: != 0 leaves reduced doubles
  u32 split_out = 0;                     // inverse second pass only: != 0 writes (y + (q-1)/2) mod q as two 30-bit halves
                                         // (bits 0..29, 32..62), the source form of ntt16_bconv_rows_kernel
  u32 galois;                            // inverse first pass only: != 0 reads src through the eval-domain Galois map
  u32 multi = 0;                         // != 0: polynomial p is read through galois_pc[p] instead (p < KS_MULTI_MAX)
  u32 galois_pc[KS_MULTI_MAX];
  const ulonglong2* scale;               // inverse second pass only: per-slot constant replacing N^-1 (NULL = N^-1);
                                         // a double2 (c, c/q) for double-precision moduli, a Shoup pair otherwise
  unsigned char id[128];                 // slot -> modulus id
  unsigned char slots[128];              // grid.z index -> slot (the launch covers the slots of one modulus class)
};

__device__ __forceinline__ bool ntt16_skip(const Ntt16Args& a, u32 poly, u32 slot) {
  if (!a.skip_beta) return false;
  u32 j = poly % a.skip_beta, lo = j * a.skip_alpha, hi = min(lo + a.skip_alpha, a.skip_nq);
  return slot >= lo && slot < hi;
}
#define NTT16_PROLOGUE                                                              \
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];                                           \
  u32 poly, tile, zi;                                                               \
  ntt16_map(a.map_mode, poly, tile, zi);                                            \
  const u32 slot = a.slots[zi];                                                     \
  if (ntt16_skip(a, poly, slot)) return;                                            \
  const u32 id = a.id[slot];                                                        \
  const ModInfo mi = a.mods[id];                                                    \
  const ulonglong2* tw = a.tw + (size_t)id * 65536;                                 \
  const double* twfp = a.twfp + (size_t)id * 65536;                                 \
  const u64* src = a.src + (size_t)poly * a.src_poly_stride + (size_t)slot * 65536; \
  u64* dst = a.dst + (size_t)poly * a.dst_poly_stride + (size_t)slot * 65536;       \
  const int cls = CLS;

// CLS: modulus class of every slot of the launch (0 double precision, 1 integer uncorrected, 2 Harvey); one
// instantiation per class so that each gets its own register allocation.
template <int CLS>
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_rows_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  if (cls == 0) ntt16_fwd_rows_fp(src, (double*)dst, twfp, mi.qd, mi.qinv, tile, (double*)sm);
  else if (cls == 2) ntt16_fwd_rows<true>(src, dst, tw, mi.m, tile, sm);
  else ntt16_fwd_rows<false>(src, dst, tw, mi.m, tile, sm);
}
template <int CLS>
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_blocks_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  const u32 t = threadIdx.x, j0 = t & 15, h = tile * 16 + (t >> 4);
  u64 x[16];
  if (cls == 0) {
    double xd[16];
    ntt16_fwd_blocks_fp(xd, (const double*)src, twfp, mi.qd, mi.qinv, tile, (double*)sm);
    if (a.raw_out) {
#pragma unroll
      for (int i = 0; i < 16; i++) x[i] = (u64)__double_as_longlong(xd[i]);
    } else {
#pragma unroll
      for (int i = 0; i < 16; i++) x[i] = d2u_canon(xd[i], mi.qd);
    }
  } else if (cls == 2) {
    ntt16_fwd_blocks<true>(x, src, tw, mi.m, mi.mu64, tile, sm);
  } else {
    ntt16_fwd_blocks<false>(x, src, tw, mi.m, mi.mu64, tile, sm);
  }
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)h * 256 + i * 16 + j0] = x[i];
}
template <int CLS>
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_inv_blocks_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  const u32 t = threadIdx.x, j0 = t & 15, h = tile * 16 + (t >> 4);
  u64 x[16];
  const u32 g = a.multi ? a.galois_pc[__builtin_amdgcn_readfirstlane(poly)] : a.galois;
  if (g) {
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = src[galois_src_index16(h * 256 + i * 16 + j0, g)];
  } else {
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = src[(size_t)h * 256 + i * 16 + j0];
  }
  if (cls == 0) {
    double xd[16];
#pragma unroll
    for (int i = 0; i < 16; i++) xd[i] = u2d(x[i]);
    ntt16_inv_blocks_fp(xd, twfp, mi.qd, mi.qinv, tile, (double*)sm);
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = (u64)__double_as_longlong(xd[i]);
  } else if (cls == 2) {
    ntt16_inv_blocks<true>(x, tw, mi.m, mi.mu64, tile, sm);
  } else {
    ntt16_inv_blocks<false>(x, tw, mi.m, mi.mu64, tile, sm);
  }
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)h * 256 + i * 16 + j0] = x[i];
}
template <int CLS>
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_inv_rows_kernel(Ntt16Args a) {
  NTT16_PROLOGUE
  u64 x[16];
  if (cls == 0) {
    double sc = mi.ninvd, scq = mi.ninvq;
    if (a.scale) {
      const double2 v = ((const double2*)a.scale)[slot];
      sc = v.x;
      scq = v.y;
    }
    ntt16_inv_rows_fp(x, (const double*)src, twfp, mi.qd, mi.qinv, sc, scq, tile, (double*)sm);
  } else {
    u64 sc = mi.ninv, scs = mi.ninvs;
    if (a.scale) {
      const ulonglong2 v = a.scale[slot];
      sc = v.x;
      scs = v.y;
    }
    if (cls == 2) ntt16_inv_rows<true>(x, src, tw, mi.m, sc, scs, tile, sm);
    else ntt16_inv_rows<false>(x, src, tw, mi.m, sc, scs, tile, sm);
  }
  if (a.split_out) {   // wave-uniform
    const u64 hq = mi.m >> 1;
#pragma unroll
    for (int i = 0; i < 16; i++) {
      const u64 y = csub(x[i] + hq, mi.m);
      x[i] = (y & 0x3FFFFFFFull) | ((y >> 30) << 32);
    }
  }
  const u32 t = threadIdx.x, col = t & 15, r0 = t >> 4, col0 = tile * 16;
#pragma unroll
  for (int i = 0; i < 16; i++) dst[(size_t)(i * 16 + r0) * 256 + col0 + col] = x[i];
}

// ---- fused: base conversion + first forward pass (ModUp and ModDown) ----
// The coefficient-domain sources arrive in the form the inverse row pass writes when Ntt16Args::split_out is set:
// for a source modulus c with h = (c - 1) / 2, the word holds yt = (y + h) mod c, y = [x (C/c)^-1]_c, as two 30-bit
// halves (bits 0..29 and bits 32..62). Since yt - h is the centred representative of y,
//   sum_k (y_k centred) (C/c_k)  =  sum_k yt_k (C/c_k)  -  sum_k h_k (C/c_k),
// the conversion is one dot product plus a per-target constant (`off`), with no sign handling per coefficient, and
// the halves enter the 32-bit multiply-adds as they are loaded. A workgroup builds the 256 x 16 tile of one target
// limb from the `len` source tiles of its digit and takes it straight through stages 0..7; the converted limb is
// never written in coefficient form. The placement of the workgroups decides which cache serves the re-reads of the
// source tiles: map mode 5 (the default, see the kernel) keeps a polynomial on one XCD with its tiles running side by
// side, target after target; ntt16_map mode 4 with the target index as the fastest dimension puts all targets of one
// (polynomial, tile) next to each other instead, which fetches every source tile once and measured slower.
struct BconvRowsArgs {
  const u64* src;           // source limbs, split form (see above)
  u64* dst;                 // target limbs after the row pass (reduced doubles / lazy integers, by class)
  const u64* mat;           // [beta][ntarget][pitch] constants (C/c_k) mod m_t in Montgomery form (2^90 or 2^64)
  const u64* off;           // [beta][ntarget] the constant -sum_k h_k (C/c_k) mod m_t in the same form
  const ulonglong2* tw;
  const double* twfp;
  const ModInfo* mods;
  u64 src_poly_stride;      // elements between the source rows of consecutive (p / beta)
  u64 dst_poly_stride;      // elements between consecutive destination polynomials p
  u32 src_slot0;            // limb index, inside a source row, of the first source of digit 0
  u32 src_nlimbs, alpha, beta;  // digit j = p % beta owns sources j*alpha .. j*alpha + len - 1, len = min(alpha, src_nlimbs - j*alpha)
  u32 skip_own;             // != 0: target slots j*alpha .. j*alpha + len - 1 are the digit's own limbs: left alone
  u32 ntarget, pitch;
  u32 map_mode;             // ntt16_map modes with the target index as the x dimension, or 5 (see the kernel)
  u32 npoly;                // polynomials (map mode 5 pads the grid to a multiple of 8)
  unsigned char id[128];    // target slot -> modulus id
  unsigned char slots[128]; // grid.x index -> target slot (one modulus class per launch)
};

// A pointer that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ const u64* uniform_ptr(const u64* p) {
  const u64 v = (u64)p;
  const u32 lo = __builtin_amdgcn_readfirstlane((u32)v), hi = __builtin_amdgcn_readfirstlane((u32)(v >> 32));
  return (const u64*)(((u64)hi << 32) | lo);
}
#define BCONV_M30 0x3FFFFFFFu
// Converted values for 8 of the lane's 16 tile positions (those at voff[0..7], offsets inside a limb). Two word
// buffers alternate, so the loads of source k + 1 are in flight while source k is multiplied in.
template <bool NARROW>
struct BconvAcc8 {
  Dot30N n[8];
  Dot30 g[8];
  u64 r[8];
  u32 pending;
  __device__ __forceinline__ void init(u64 offc) {
    pending = 0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
      r[i] = 0;
      if (NARROW) {
        n[i].a = (u32)offc & BCONV_M30;
        n[i].b = offc >> 30;
        n[i].c = 0;
      } else {
        dot30_init(g[i]);
        g[i].s00 = (u32)offc & BCONV_M30;
        g[i].s01 = offc >> 30;
      }
    }
  }
  __device__ __forceinline__ void fold(u64 m, u64 minv) {
#pragma unroll
    for (int i = 0; i < 8; i++) {
      if (NARROW) {
        r[i] += dot30n_redc90(n[i], m, minv);   // each part < m + 2^34
        dot30n_init(n[i]);
      } else {
        r[i] += redc(dot30_value(g[i]), m, minv);   // each part < 2m
        dot30_init(g[i]);
      }
    }
    pending = 0;
  }
  __device__ __forceinline__ void mac(const u64 (&w)[8], u64 c, bool more, u64 m, u64 minv) {
    const u32 c0 = (u32)c & BCONV_M30, c1 = (u32)(c >> 30);
#pragma unroll
    for (int i = 0; i < 8; i++) {
      if (NARROW) dot30n_mac(n[i], (u32)w[i], (u32)(w[i] >> 32), c0, c1);
      else dot30_mac(g[i], (u32)w[i], (u32)(w[i] >> 32), c0, c1);
    }
    if (++pending == 15 && more) fold(m, minv);   // wave-uniform: chunks of 15 terms are reduced separately
  }
};
// boff: byte offsets of the 8 positions inside a limb. The source limbs of the digit are read through a buffer
// resource (scalar base, bounds = the digit's len limbs; scalar offset = the limb, vector offset = the position), so
// addressing costs no vector instructions. The loads are unconditional (a source index past the end is clamped and
// meets the constant 0) and fenced against reordering: the younger buffer's loads stay in flight while the older
// buffer is multiplied in.
typedef u32 bconv_u32x2 __attribute__((ext_vector_type(2)));
template <bool NARROW>
__device__ __forceinline__ void bconv_rows_eight(u64 (&r)[8], const u64* __restrict__ src, const u32 (&boff)[8], u32 len,
                                                 const u64* __restrict__ crow, u64 offc, const ModInfo& mi) {
  const u64 m = mi.m;
  u64 wa[8], wb[8];
  BconvAcc8<NARROW> acc;
  acc.init(offc);
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)src, 0, (int)(len * 524288u), 0x00020000);
  auto load8 = [&](u64 (&w)[8], u32 k) {
    const u32 soff = min(k, len - 1) * 524288u;   // wave-uniform
#pragma unroll
    for (int i = 0; i < 8; i++) {
      const bconv_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rsrc, boff[i], soff, 0);
      w[i] = ((u64)v.y << 32) | v.x;
    }
  };
  // fence: neither the compiler's code motion (memory clobber) nor the instruction scheduler may move a buffer's
  // loads next to their use
#define BCONV_FENCE()                   \
  asm volatile("" ::: "memory");        \
  __builtin_amdgcn_sched_barrier(0)
  load8(wa, 0);
  for (u32 k = 0; k < len; k += 2) {
    load8(wb, k + 1);
    BCONV_FENCE();
    acc.mac(wa, crow[k], k + 1 < len, m, mi.minv);
    BCONV_FENCE();
    load8(wa, k + 2);
    BCONV_FENCE();
    acc.mac(wb, k + 1 < len ? crow[k + 1] : 0, k + 2 < len, m, mi.minv);
    BCONV_FENCE();
  }
#undef BCONV_FENCE
  acc.fold(m, mi.minv);
  // at most three chunks (45 sources): the sum of the parts is below 6m
#pragma unroll
  for (int i = 0; i < 8; i++) {
    u64 v = acc.r[i];
    if (len > 15 || !NARROW) v = csub(csub(v, 4 * m), 2 * m);
    r[i] = csub(v, m);
  }
}

template <int CLS, bool NARROW>
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_bconv_rows_kernel(BconvRowsArgs a) {
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];
  u32 zi, tile, poly;
  if (a.map_mode == 5) {
    // Per XCD (workgroups are dealt to the 8 XCDs round-robin): tiles fastest, then targets, then polynomials, each
    // XCD on polynomials of its own. The 16 tiles of a limb lie on 16 different L2 channels (rows are 2 KiB apart), so
    // the workgroups in flight on an XCD spread their source reads over all channels instead of queueing on one,
    // while the targets that share a polynomial's source tiles still follow each other on the same XCD.
    const u32 lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const u32 r = lin >> 3;
    tile = r & 15;
    zi = (r >> 4) % gridDim.x;
    poly = (lin & 7) + 8 * ((r >> 4) / gridDim.x);
    if (poly >= a.npoly) return;
  } else {
    ntt16_map(a.map_mode, zi, tile, poly);
  }
  const u32 slot = a.slots[zi];
  const u32 j = poly % a.beta, lo = j * a.alpha, len = min(a.alpha, a.src_nlimbs - lo);
  if (a.skip_own && slot >= lo && slot < lo + len) return;
  const u32 id = a.id[slot];
  const ModInfo mi = a.mods[id];
  const u64* src = a.src + (size_t)(poly / a.beta) * a.src_poly_stride + (size_t)(a.src_slot0 + lo) * 65536;
  const u64* crow = a.mat + ((size_t)j * a.ntarget + slot) * a.pitch;
  const u64 offc = a.off[(size_t)j * a.ntarget + slot];
  u64* dst = a.dst + (size_t)poly * a.dst_poly_stride + (size_t)slot * 65536;
  const u32 t = threadIdx.x, pos0 = (t >> 4) * 256 + tile * 16 + (t & 15);   // row r0, column col0 + col
  u64 x[16];
#pragma unroll
  for (int half = 0; half < 2; half++) {
    u32 boff[8];
#pragma unroll
    for (int i = 0; i < 8; i++) boff[i] = (pos0 + (half * 8 + i) * 4096) * 8;   // rows i*16 + r0, in bytes
    u64 r[8];
    bconv_rows_eight<NARROW>(r, src, boff, len, crow, offc, mi);
#pragma unroll
    for (int i = 0; i < 8; i++) x[half * 8 + i] = r[i];
  }
  if (CLS == 0) {
    double xd[16];
#pragma unroll
    for (int i = 0; i < 16; i++) xd[i] = u2d(x[i]);
    ntt16_fwd_rows_fp_loaded(xd, (double*)dst, a.twfp + (size_t)id * 65536, mi.qd, mi.qinv, tile, (double*)sm);
  } else if (CLS == 2) {
    ntt16_fwd_rows_loaded<true>(x, dst, a.tw + (size_t)id * 65536, mi.m, tile, sm);
  } else {
    ntt16_fwd_rows_loaded<false>(x, dst, a.tw + (size_t)id * 65536, mi.m, tile, sm);
  }
}

// ---- fused: last forward pass of the ModUp'ed digits + inner product with the evaluation key ----
// For (ciphertext b, extended slot t, tile): acc[b][c][t] = sum_j D_j * evk[j][c][id(t)], where D_j is the forward
// transform of ext[b][j][t] (slots the digit does not own) or d[b][t] itself (the digit's own limbs, already in
// the evaluation domain). Output canonical. On integer-class moduli the products go through a Montgomery
// reduction, so acc carries a factor 2^-64 there, which the later stages absorb into their constants; on
// double-precision moduli acc is the plain sum.
struct FwdInnerArgs {
  const u64* ext;   // [B][beta][next][N], after the row pass
  const u64* d;     // eval domain, limb-vector (b, t) at d + b*d_poly_stride + t*N; read through the Galois map if galois != 0
  u64 d_poly_stride;
  const u64* evk;   // [dnum][2][nm][N]
  u64* acc;         // [B][2][next][N]
  const ulonglong2* tw;
  const double* twfp; 
  const ModInfo* mods;
  u32 nlimbs, nq, nm, alpha, beta, next, map_mode, galois;
  u32 ext_galois;            // streaming kernels only: != 0 reads ext through the Galois map too (hoisted digits:
                             // ext holds the transform of the un-rotated polynomial, shared by many rotations)
  unsigned char slots[128];  // grid.z index -> extended slot (one modulus class per launch)
  u32 multi = 0;             // != 0: ciphertext b uses galois_pc[b] and evk_pc[b] instead of galois and evk
  u32 galois_pc[KS_MULTI_MAX];
  const u64* evk_pc[KS_MULTI_MAX];
  // streaming kernels only: != null adds P * sigma_g(c0[b][t]) to the first accumulator on the main-prime slots
  // (rotations kept in the extended basis: ModDown of the sum then returns sigma_g(c0) + ModDown(accumulator))
  const u64* c0 = nullptr;   // limb-vector (b, t) at c0 + b*c0_poly_stride + t*N, canonical residues, eval domain
  u64 c0_poly_stride = 0;
  u32 accumulate = 0;        // streaming kernels only: != 0 adds the result to what acc holds instead of overwriting it
  // many-rotation kernels (inner16_rot_*): rotation r < nrot of every ciphertext uses the key evk_pc[r], writes to
  // acc + r * acc_rot_stride, and galois_pc[r] holds the INVERSE of its Galois element modulo 2N
  u32 nrot = 0;
  u64 acc_rot_stride = 0;
  // ntt16_fwd_blocks_inner_c_kernel on main-prime slots only: fin_tq != null finishes the key switch in the same
  // kernel instead of storing the accumulator: out = (sum - NTT(tq)) / P (+ addends), with the arguments of
  // FwdFinalArgs (tq after the row pass, [B*2][nlimbs][N]; pinv [nlimbs] as (1/P, (1/P)/q); addend modes per component)
  const u64* fin_tq = nullptr;
  u64* fin_out = nullptr;
  const u64* fin_add2 = nullptr;
  const u64* fin_add_src = nullptr;
  const ulonglong2* fin_pinv = nullptr;
  u32 fin_mode0 = 0, fin_mode1 = 0, fin_galois = 0, fin_add2_three = 0;
};
// b is the same for the whole workgroup; saying so keeps the table look-ups on the scalar unit and their results
// in scalar registers.
__device__ __forceinline__ u32 fwd_inner_galois(const FwdInnerArgs& a, u32 b) {
  return a.multi ? a.galois_pc[__builtin_amdgcn_readfirstlane(b)] : a.galois;
}
__device__ __forceinline__ const u64* fwd_inner_evk(const FwdInnerArgs& a, u32 b) {
  const u64 v = (u64)(a.multi ? a.evk_pc[__builtin_amdgcn_readfirstlane(b)] : a.evk);
  const u32 lo = __builtin_amdgcn_readfirstlane((u32)v), hi = __builtin_amdgcn_readfirstlane((u32)(v >> 32));
  return (const u64*)(((u64)hi << 32) | lo);
}

__device__ __forceinline__ bool fwd_inner_owns(const FwdInnerArgs& a, u32 t, u32 j) {
  const u32 lo = j * a.alpha, hi = min(lo + a.alpha, a.nlimbs);
  return t >= lo && t < hi;
}

// Double-precision moduli, one key component per workgroup: grid.x = 2B, polynomial index bc = 2b + c. Each of the
// two workgroups of a ciphertext transforms the digit tiles itself (the arithmetic is cheap next to the traffic and
// the second reader finds the tile in its XCD's L2, the pair being adjacent in the launch order) and multiplies by
// its own half of the key: one accumulator tile instead of two, so the kernel keeps 3 waves per SIMD.
// Input tiles are prefetched: the converted digit tiles (and the ModDown correction tile of the fused tail) are
// contiguous 32 KB pieces of memory, so each wave copies its quarter of the NEXT tile straight into LDS with
// direct-to-LDS buffer loads (no registers) while it works on the current one, and starts a tile by reading its
// values from LDS instead of waiting for memory. The own digit, which is read through the Galois map, goes first:
// its loads are in flight together with the first prefetch. The key tile of a digit is requested between the two
// rounds of its transform. LDS: the word tile of the split transposes (17 KB), the image (4 waves x 8 KB) and the
// first-round twiddles (2 KB): 51 KB per workgroup, three workgroups per compute unit.
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef __attribute__((address_space(1))) const void* global_void_ptr;
typedef const __attribute__((address_space(1))) u64* global_u64_ptr;
typedef u64 global_u64x2 __attribute__((ext_vector_type(2)));
#define INNER_C_EX_WORDS (16 * 272)
__device__ __forceinline__ void fwd_inner_c_body_fp(const FwdInnerArgs& a, u32 bc, u32 tile, u32 t, u32 id, const ModInfo& mi,
                                                    u32* ex, double* img, double* twl) {
  const u32 b = bc >> 1, c = bc & 1;
  const size_t N = 65536;
  const double q = mi.qd, qinv = mi.qinv;
  const double* tw = a.twfp + (size_t)id * N;
  const u64* evk = fwd_inner_evk(a, b) + ((size_t)c * a.nm + id) * N;
  const u32 g = __builtin_amdgcn_readfirstlane(fwd_inner_galois(a, b));
  auto lane_pos = [&]() {
    u32 tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    return (tile * 16 + (tid >> 4)) * 256 + (tid & 15);   // position of element 0 of this lane in the limb
  };
  // a wave's quarter of a tile: blocks 4w .. 4w+3, 1024 consecutive words; lane L of request k moves words
  // 128k + 2L and 128k + 2L + 1
  auto request = [&](const u64* limb) {
    u32 tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const u32 wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)uniform_ptr(limb + (size_t)tile * 4096 + wv * 1024), 0, 8192, 0x00020000);
    const int vo = (int)((tid & 63) * 16);
    double* li = img + wv * 1024;
#pragma unroll
    for (int k = 0; k < 8; k++)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(li + k * 128), 16, vo, k * 1024, 0, 0);
  };
  // the requested tile in the i-layout (lane (hb, j0) holds positions i*16 + j0 of block hb); afterwards the image is free
  auto take = [&](double (&x)[16]) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    u32 tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const double* li = img + (tid >> 6) * 1024 + ((tid >> 4) & 3) * 256 + (tid & 15);
#pragma unroll
    for (int i = 0; i < 16; i++) x[i] = li[i * 16];
    wave_lds_sync();
  };
  const u32 beta = a.beta;
  const u32 jo = t < a.nlimbs ? t / a.alpha : 0xFFFFFFFFu;   // the digit that holds limb t itself (none for special slots)
  auto ext_limb = [&](u32 j) { return a.ext + (((size_t)b * beta + j) * a.next + t) * N; };
  const u64* tq_limb = a.fin_tq ? a.fin_tq + ((size_t)bc * a.nlimbs + t) * N : nullptr;
  double acc[16], x[16];
  u64 e[16];
#pragma unroll
  for (int i = 0; i < 16; i++) acc[i] = 0.0;
  u32 jn = jo == 0 ? 1u : 0u;   // next converted digit
  if (jn < beta) request(ext_limb(jn));
  else if (tq_limb) request(tq_limb);
  const double twv = ntt16_twl_fetch(tw, tile);
  u32 cnt = 0;
  if (jo != 0xFFFFFFFFu) {
    const u32 pos = lane_pos();
    const u64* k = evk + (size_t)jo * 2 * a.nm * N + pos;
    const u64* src = a.d + (size_t)b * a.d_poly_stride + (size_t)t * N;
#pragma unroll
    for (int i = 0; i < 16; i++) e[i] = k[i * 16];
    if (g) {
#pragma unroll
      for (int i = 0; i < 16; i++) x[i] = u2d(src[galois_src_index16(pos + i * 16, g)]);
    } else {
#pragma unroll
      for (int i = 0; i < 16; i++) x[i] = u2d(src[pos + i * 16]);
    }
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] += fp_mulmod_var(x[i], u2d(e[i]), qinv, q);
    cnt = 1;
  }
  ntt16_twl_store(twv, twl);   // read by the wave's own lanes from the first transform on
#pragma nounroll
  while (jn < beta) {
    take(x);
    u32 jnext = jn + 1;
    if (jnext == jo) jnext++;
    // (a pointer rebuilt from scalar halves has lost its address space: say "global", or the loads become flat
    // loads, which wait for the prefetch in case it lands where they read)
    const global_u64_ptr k = (global_u64_ptr)(evk + (size_t)jn * 2 * a.nm * N + lane_pos());
    ntt16_fwd_blocks_fp_words(
        x, tw, q, qinv, tile, ex, twl,
        [&] {
          // always issued (the current tile again when nothing follows), so that the waits of the two rounds are
          // the same static counts on every path
          request(jnext < beta ? ext_limb(jnext) : tq_limb ? tq_limb : ext_limb(jn));
        },
        [&] {
#pragma unroll
          for (int i = 0; i < 16; i++) e[i] = k[i * 16];
        });
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] += fp_mulmod_var(x[i], u2d(e[i]), qinv, q);
    if ((++cnt & 3) == 0) {   // each product is below 0.75 q: fold before the sum can reach 2^53
#pragma unroll
      for (int i = 0; i < 16; i++) acc[i] = fp_reduce(acc[i], qinv, q);
    }
    jn = jnext;
  }
  if (a.fin_tq) {
    const u32 mode = c ? a.fin_mode1 : a.fin_mode0;
    const u32 gf = a.multi ? g : a.fin_galois;
    const size_t a2poly = a.fin_add2_three ? (size_t)b * 3 + c : (size_t)bc;
    const u64* a2 = a.fin_add2 + (a2poly * a.nlimbs + t) * N;
    const u64* as = a.fin_add_src + ((size_t)bc * a.nlimbs + t) * N;
    take(x);
    ntt16_fwd_blocks_fp_words(x, tw, q, qinv, tile, ex, twl, [] {}, [&] {
      const u32 pos = lane_pos();
      if (mode & 1) {
#pragma unroll
        for (int i = 0; i < 16; i++) e[i] = a2[pos + i * 16];
      } else if (mode == 2) {
#pragma unroll
        for (int i = 0; i < 16; i++) e[i] = as[galois_src_index16(pos + i * 16, gf)];
      }
    });
    const double2 pv = ((const double2*)a.fin_pinv)[t];
    u64* o = a.fin_out + ((size_t)bc * a.nlimbs + t) * N + lane_pos();
    const u32 pos = lane_pos();
#pragma unroll
    for (int i = 0; i < 16; i++) {
      double r = fp_mulmod_const(fp_reduce(acc[i], qinv, q) - x[i], pv.x, pv.y, q);   // |r| <= 0.75 q
      if (mode) r += u2d(e[i]);
      if (mode == 3) {
        r += u2d(as[galois_src_index16(pos + i * 16, gf)]);
        r = r >= q ? r - q : r;
      }
      o[i * 16] = d2u_canon(r, q);
    }
    return;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy into LDS may outlive the workgroup
  u64* o = a.acc + (((size_t)b * 2 + c) * a.next + t) * N + lane_pos();
  if (a.accumulate) {
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] = fp_reduce(acc[i], qinv, q) + u2d(o[i * 16]);
    if (c == 0 && a.c0 && t < a.nlimbs) {
      const u64* src = a.c0 + (size_t)b * a.c0_poly_stride + (size_t)t * N;
      const double pm = u2d(mi.pmod);
      const u32 pos = lane_pos();
#pragma unroll
      for (int i = 0; i < 16; i++) acc[i] += fp_mulmod_var(u2d(src[galois_src_index16(pos + i * 16, g)]), pm, qinv, q);
    }
  }
#pragma unroll
  for (int i = 0; i < 16; i++) o[i * 16] = d2u_canon(fp_reduce(acc[i], qinv, q), q);
}
__global__ void __launch_bounds__(NTT16_THREADS) __attribute__((amdgpu_waves_per_eu(3, 3)))
ntt16_fwd_blocks_inner_c_kernel(FwdInnerArgs a) {
  // separate arrays, so that the compiler knows the transposes never touch the image a prefetch is landing in
  __shared__ __attribute__((aligned(16))) double img[4096];
  __shared__ u32 ex[INNER_C_EX_WORDS];
  __shared__ double twl[16 * NTT16_TWL_PITCH];
  u32 bc, tile, zi;
  ntt16_map(a.map_mode, bc, tile, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  fwd_inner_c_body_fp(a, bc, tile, t, id, mi, ex, img, twl);
}

// Integer-class moduli (the special primes): both key components per workgroup, 8 values per lane: a workgroup takes
// 8 of the 256-element blocks of a (ciphertext, slot) (grid.y = 32 tiles), each block transformed by 32 lanes
// (ntt256_fwd_blocks_int8), which keeps the kernel at 3 waves per SIMD. After the transform a lane holds 8 consecutive
// coefficients, so key words and accumulators move as 16-byte accesses. Products go through a Montgomery reduction:
// acc carries the factor 2^-64, which the later stages absorb into their constants.
template <int CLS>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
ntt16_fwd_blocks_inner8_kernel(FwdInnerArgs a) {
  constexpr bool BIG = CLS == 2;
  __shared__ u64 sm[8 * NTT8_BLOCK_LDS_I];
  __shared__ __attribute__((aligned(16))) u64 img[2048];
  u32 b, tile, zi;
  ntt16_map(a.map_mode, b, tile, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const size_t N = 65536;
  const u64 q = mi.m, q2 = 2 * mi.m;
  const ulonglong2* tw = a.tw + (size_t)id * N;
  const u32 tid = threadIdx.x, l = tid & 31, hb = tid >> 5, h = tile * 8 + hb;
  u64* smb = sm + hb * NTT8_BLOCK_LDS_I;
  const u64* evk = fwd_inner_evk(a, b) + (size_t)id * N;
  const u32 g = __builtin_amdgcn_readfirstlane(fwd_inner_galois(a, b));
  const u32 posA = h * 256 + l;
  const u32 posC = h * 256 + (l >> 2) * 32 + (l & 3) * 8;
  u64 acc0[8], acc1[8], x[8];
  ulonglong2 e0[4], e1[4];
#pragma unroll
  for (int c = 0; c < 8; c++) acc0[c] = acc1[c] = 0;
  // The converted digit tiles are prefetched: a wave copies its two blocks (4 KB) of the next tile straight into LDS
  // while it multiplies the current one by the key, and starts a tile by reading its values from there.
  auto request = [&](const u64* limb) {
    u32 td = threadIdx.x;
    asm volatile("" : "+v"(td));
    const u32 wv = __builtin_amdgcn_readfirstlane(td >> 6);
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)uniform_ptr(limb + (size_t)tile * 2048 + wv * 512), 0, 4096, 0x00020000);
    const int vo = (int)((td & 63) * 16);
    u64* li = img + wv * 512;
#pragma unroll
    for (int k = 0; k < 4; k++)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(li + k * 128), 16, vo, k * 1024, 0, 0);
  };
  auto take = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    u32 td = threadIdx.x;
    asm volatile("" : "+v"(td));
    const u64* li = img + (td >> 5) * 256 + (td & 31);
#pragma unroll
    for (int i = 0; i < 8; i++) x[i] = li[i * 32];
    wave_lds_sync();
  };
  auto multiply = [&]() {
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const u64 eb[2] = {e0[v].x, e0[v].y}, ea[2] = {e1[v].x, e1[v].y};
#pragma unroll
      for (int k = 0; k < 2; k++) {
        const u64 xv = x[2 * v + k];
        Acc128 p0, p1;
        p0.lo = xv * eb[k];
        p0.hi = mul_hi64(xv, eb[k]);
        p1.lo = xv * ea[k];
        p1.hi = mul_hi64(xv, ea[k]);
        acc0[2 * v + k] = csub(acc0[2 * v + k] + redc(p0, q, mi.minv), q2);
        acc1[2 * v + k] = csub(acc1[2 * v + k] + redc(p1, q, mi.minv), q2);
      }
    }
  };
  auto request_key = [&](u32 j) {
    const global_u64_ptr kb = (global_u64_ptr)(evk + (size_t)j * 2 * a.nm * N + posC);
    const global_u64_ptr ka = kb + (size_t)a.nm * N;
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const global_u64x2 vb = *(const __attribute__((address_space(1))) global_u64x2*)(kb + 2 * v);
      const global_u64x2 va = *(const __attribute__((address_space(1))) global_u64x2*)(ka + 2 * v);
      e0[v] = ulonglong2{vb.x, vb.y};
      e1[v] = ulonglong2{va.x, va.y};
    }
  };
  const u32 beta = a.beta;
  const u32 jo = t < a.nlimbs ? t / a.alpha : 0xFFFFFFFFu;   // the digit that holds limb t itself (none for special slots)
  auto ext_limb = [&](u32 j) { return a.ext + (((size_t)b * beta + j) * a.next + t) * N; };
  u32 jn = jo == 0 ? 1u : 0u;   // next converted digit
  if (jn < beta) request(ext_limb(jn));
  if (jo != 0xFFFFFFFFu) {   // the own digit first: its loads are in flight together with the first prefetch
    const u64* src = a.d + (size_t)b * a.d_poly_stride + (size_t)t * N;
    request_key(jo);
    if (g) {
#pragma unroll
      for (int c = 0; c < 8; c++) x[c] = src[galois_src_index16(posC + c, g)];
    } else {
#pragma unroll
      for (int v = 0; v < 4; v++) {
        const ulonglong2 w = *(const ulonglong2*)(src + posC + 2 * v);
        x[2 * v] = w.x;
        x[2 * v + 1] = w.y;
      }
    }
    multiply();
  }
#pragma nounroll
  while (jn < beta) {
    take();
    u32 jnext = jn + 1;
    if (jnext == jo) jnext++;
    const u32 jcur = jn;
    ntt256_fwd_blocks_int8<BIG>(x, tw, q, mi.mu64, h, l, smb, [&] { request_key(jcur); });
    __builtin_amdgcn_sched_barrier(0);
    // younger than every load the products wait for, so it stays in flight across them (the current tile again when
    // nothing follows: the same static wait counts on every path)
    request(ext_limb(jnext < beta ? jnext : jcur));
    __builtin_amdgcn_sched_barrier(0);
    multiply();
    jn = jnext;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy into LDS may outlive the workgroup
  u64* o0 = a.acc + (((size_t)b * 2 + 0) * a.next + t) * N + posC;
  u64* o1 = o0 + (size_t)a.next * N;
  if (a.accumulate) {   // a rotation kept in the extended basis, added to what acc holds (wave-uniform branch)
#pragma unroll
    for (int v = 0; v < 4; v++) {
      const ulonglong2 p0 = *(const ulonglong2*)(o0 + 2 * v), p1 = *(const ulonglong2*)(o1 + 2 * v);
      acc0[2 * v] = csub(acc0[2 * v] + p0.x, q2);        // old values are canonical: below 3q, back below 2q
      acc0[2 * v + 1] = csub(acc0[2 * v + 1] + p0.y, q2);
      acc1[2 * v] = csub(acc1[2 * v] + p1.x, q2);
      acc1[2 * v + 1] = csub(acc1[2 * v + 1] + p1.y, q2);
    }
    if (a.c0 && t < a.nlimbs) {   // + P * sigma_g(c0) * 2^-64 on the main primes
      const u64* src = a.c0 + (size_t)b * a.c0_poly_stride + (size_t)t * N;
#pragma unroll
      for (int c = 0; c < 8; c++) {
        const u64 v = src[galois_src_index16(posC + c, g)];
        Acc128 p = {v * mi.pmod, mul_hi64(v, mi.pmod)};
        acc0[c] = csub(acc0[c] + redc(p, q, mi.minv), q2);
      }
    }
  }
#pragma unroll
  for (int v = 0; v < 4; v++) {
    *(ulonglong2*)(o0 + 2 * v) = ulonglong2{csub(acc0[2 * v], q), csub(acc0[2 * v + 1], q)};
    *(ulonglong2*)(o1 + 2 * v) = ulonglong2{csub(acc1[2 * v], q), csub(acc1[2 * v + 1], q)};
  }
}

// ---- fused: last forward pass of the ModDown correction + final assembly ----
// out[bc][i] = (acc[bc][i] - NTT(tq[bc][i])) * pinv[i]  (+ addend). On integer-class moduli acc and tq carry the
// factor 2^-64 and pinv = 2^64/P; on double-precision moduli they are plain and pinv = (1/P, (1/P)/q).
// addend modes per component c = bc & 1: 0 none; 1 the plain addend add2 (== out: in place); 2 add_src read
// through the Galois map g (HRot's sigma(c0)); 3 both (an HRot added to another ciphertext or accumulated into out).
struct FwdFinalArgs {
  const u64* tq;      // [B*2][nlimbs][N], after the row pass
  const u64* acc;     // [B*2][next][N]
  u64* out;           // [B*2][nlimbs][N]
  const u64* add2;    // [B*2][nlimbs][N] (mode bit 1); may be out itself
  const u64* add_src; // [B][2][nlimbs][N] (mode bit 2)
  const ulonglong2* tw;
  const double* twfp; 
  const ModInfo* mods;
  const ulonglong2* pinv;  // [nlimbs]
  u32 nlimbs, next, mode0, mode1, galois, map_mode;
  unsigned char slots[128];  // grid.z index -> limb (one modulus class per launch)
  u32 multi = 0;             // != 0: ciphertext b = bc / 2 reads add_src through galois_pc[b]
  u32 galois_pc[KS_MULTI_MAX];
  u32 add2_three = 0;        // != 0: add2 holds three components per ciphertext ([B][3][nlimbs][N]); the first two are added
};
// polynomial index of component bc & 1 of ciphertext bc / 2 inside add2
__device__ __forceinline__ size_t final_add2_poly(const FwdFinalArgs& a, u32 bc) {
  return a.add2_three ? (size_t)(bc >> 1) * 3 + (bc & 1) : (size_t)bc;
}
template <bool BIG>
__device__ __forceinline__ void fwd_final_body(const FwdFinalArgs& a, u32 bc, u32 tile, u32 i_limb, const ModInfo& mi, u64* sm) {
  const u32 tid = threadIdx.x, j0 = tid & 15, h = tile * 16 + (tid >> 4);
  const size_t N = 65536;
  const u64 q = mi.m, q2 = 2 * mi.m;
  u64 x[16];
  ntt16_fwd_blocks<BIG, false>(x, a.tq + ((size_t)bc * a.nlimbs + i_limb) * N, a.tw + (size_t)i_limb * N, q, mi.mu64, tile, sm);
  const ulonglong2 pv = a.pinv[i_limb];
  const u64* ac = a.acc + ((size_t)bc * a.next + i_limb) * N + (size_t)h * 256 + j0;
  u64* o = a.out + ((size_t)bc * a.nlimbs + i_limb) * N + (size_t)h * 256 + j0;
  const u32 mode = (bc & 1) ? a.mode1 : a.mode0;
  const u64* as = a.add_src + ((size_t)bc * a.nlimbs + i_limb) * N;
  const u64* a2 = a.add2 + (final_add2_poly(a, bc) * a.nlimbs + i_limb) * N + (size_t)h * 256 + j0;
  const u32 g = a.multi ? a.galois_pc[__builtin_amdgcn_readfirstlane(bc >> 1)] : a.galois;
#pragma unroll
  for (int i = 0; i < 16; i++) {
    u64 r = shoup(ac[i * 16] + q2 - x[i], pv.x, pv.y, q);
    if (mode & 1) r = addmod(r, a2[i * 16], q);
    if (mode & 2) r = addmod(r, as[galois_src_index16(h * 256 + i * 16 + j0, g)], q);
    o[i * 16] = r;
  }
}
__device__ __forceinline__ void fwd_final_body_fp(const FwdFinalArgs& a, u32 bc, u32 tile, u32 i_limb, const ModInfo& mi,
                                                  double* sm) {
  const u32 tid = threadIdx.x, j0 = tid & 15, h = tile * 16 + (tid >> 4);
  const size_t N = 65536;
  const double q = mi.qd, qinv = mi.qinv;
  double x[16];
  const u64* ac = a.acc + ((size_t)bc * a.next + i_limb) * N + (size_t)h * 256 + j0;
  u64 av[16];  // requested before the transform so that all of the workgroup's reads are in flight together
#pragma unroll
  for (int i = 0; i < 16; i++) av[i] = ac[i * 16];
  u64* o = a.out + ((size_t)bc * a.nlimbs + i_limb) * N + (size_t)h * 256 + j0;
  const u32 mode = (bc & 1) ? a.mode1 : a.mode0;
  const u64* as = a.add_src + ((size_t)bc * a.nlimbs + i_limb) * N;
  const u32 g = a.multi ? a.galois_pc[__builtin_amdgcn_readfirstlane(bc >> 1)] : a.galois;
  u64 ad[16];
  if (mode & 1) {
    const u64* a2 = a.add2 + (final_add2_poly(a, bc) * a.nlimbs + i_limb) * N + (size_t)h * 256 + j0;
#pragma unroll
    for (int i = 0; i < 16; i++) ad[i] = a2[i * 16];
  } else if (mode == 2) {
#pragma unroll
    for (int i = 0; i < 16; i++) ad[i] = as[galois_src_index16(h * 256 + i * 16 + j0, g)];
  }
  ntt16_fwd_blocks_fp(x, (const double*)(a.tq + ((size_t)bc * a.nlimbs + i_limb) * N), a.twfp + (size_t)i_limb * N, q, qinv,
                      tile, sm);
  const double2 pv = ((const double2*)a.pinv)[i_limb];
#pragma unroll
  for (int i = 0; i < 16; i++) {
    double r = fp_mulmod_const(u2d(av[i]) - x[i], pv.x, pv.y, q);  // |r| <= 0.9 q
    if (mode) r += u2d(ad[i]);
    if (mode == 3) {   // two addends: the gathered one is fetched here; bring the sum back below 2q first
      r += u2d(as[galois_src_index16(h * 256 + i * 16 + j0, g)]);
      r = r >= q ? r - q : r;
    }
    o[i * 16] = d2u_canon(r, q);
  }
}
template <int CLS>
__global__ void __launch_bounds__(NTT16_THREADS) ntt16_fwd_blocks_final_kernel(FwdFinalArgs a) {
  __shared__ u64 sm[NTT16_LDS_BYTES / 8];
  u32 bc, tile, zi;
  ntt16_map(a.map_mode, bc, tile, zi);
  const u32 i_limb = a.slots[zi];
  const ModInfo mi = a.mods[i_limb];
  const int cls = CLS;
  if (cls == 0) fwd_final_body_fp(a, bc, tile, i_limb, mi, (double*)sm);
  else if (cls == 2) fwd_final_body<true>(a, bc, tile, i_limb, mi, sm);
  else fwd_final_body<false>(a, bc, tile, i_limb, mi, sm);
}

// ---- streaming inner product for double-precision moduli (hoisted rotations, and the unfused alternative of a
// plain key switch) ----
// acc[b][c][t][n] = sum_j D_j[n] * evk[j][c][id(t)][n] with D_j = ext[b][j][t] (reduced doubles, evaluation domain)
// or d[b][t] (canonical residues, read through the Galois map if asked). One lane per coefficient; grid =
// (B, N/256, slots of the class), batch innermost so that consecutive workgroups share the key slice.
__global__ void __launch_bounds__(256) inner16_fp_kernel(FwdInnerArgs a) {
  // two adjacent coefficients per lane (16-byte accesses); grid.y = N / 512
  const size_t N = 65536;
  u32 b, blk, zi;
  ntt16_map(a.map_mode, b, blk, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const double q = mi.qd, qinv = mi.qinv;
  const u32 n = (blk * 256 + threadIdx.x) * 2;
  double s0[2] = {0.0, 0.0}, s1[2] = {0.0, 0.0};
  const u32 g_own = fwd_inner_galois(a, b);
  const u64* evk = fwd_inner_evk(a, b);
  for (u32 j = 0; j < a.beta; j++) {
    double x[2];
    if (fwd_inner_owns(a, t, j)) {
      const u64* src = a.d + (size_t)b * a.d_poly_stride + (size_t)t * N;
      if (g_own) {
        x[0] = u2d(src[galois_src_index16(n, g_own)]);
        x[1] = u2d(src[galois_src_index16(n + 1, g_own)]);
      } else {
        const ulonglong2 v = *(const ulonglong2*)(src + n);
        x[0] = u2d(v.x);
        x[1] = u2d(v.y);
      }
    } else {
      const u64* e = a.ext + (((size_t)b * a.beta + j) * a.next + t) * N;
      if (a.ext_galois) {
        x[0] = __longlong_as_double((long long)e[galois_src_index16(n, a.ext_galois)]);
        x[1] = __longlong_as_double((long long)e[galois_src_index16(n + 1, a.ext_galois)]);
      } else {
        const double2 v = *(const double2*)(e + n);
        x[0] = v.x;
        x[1] = v.y;
      }
    }
    const u64* kb = evk + (((size_t)j * 2 + 0) * a.nm + id) * N + n;
    const ulonglong2 eb = *(const ulonglong2*)kb;
    const ulonglong2 ea = *(const ulonglong2*)(kb + (size_t)a.nm * N);
    s0[0] += fp_mulmod_var(x[0], u2d(eb.x), qinv, q);
    s0[1] += fp_mulmod_var(x[1], u2d(eb.y), qinv, q);
    s1[0] += fp_mulmod_var(x[0], u2d(ea.x), qinv, q);
    s1[1] += fp_mulmod_var(x[1], u2d(ea.y), qinv, q);
    if ((j & 3) == 3) {
#pragma unroll
      for (int e = 0; e < 2; e++) {
        s0[e] = fp_reduce(s0[e], qinv, q);
        s1[e] = fp_reduce(s1[e], qinv, q);
      }
    }
  }
  if (a.c0 && t < a.nlimbs) {   // at most three products are pending here, a fourth keeps the sum below 2^52
    const u64* src = a.c0 + (size_t)b * a.c0_poly_stride + (size_t)t * N;
    const double pm = u2d(mi.pmod);
    s0[0] += fp_mulmod_var(u2d(src[galois_src_index16(n, g_own)]), pm, qinv, q);
    s0[1] += fp_mulmod_var(u2d(src[galois_src_index16(n + 1, g_own)]), pm, qinv, q);
  }
  u64* o0 = a.acc + (((size_t)b * 2 + 0) * a.next + t) * N + n;
  if (a.accumulate) {   // fold first (|.| <= q/2), then the old canonical values fit under the same bound
    const ulonglong2 p0 = *(const ulonglong2*)o0, p1 = *(const ulonglong2*)(o0 + (size_t)a.next * N);
    s0[0] = fp_reduce(s0[0], qinv, q) + u2d(p0.x);
    s0[1] = fp_reduce(s0[1], qinv, q) + u2d(p0.y);
    s1[0] = fp_reduce(s1[0], qinv, q) + u2d(p1.x);
    s1[1] = fp_reduce(s1[1], qinv, q) + u2d(p1.y);
  }
  *(ulonglong2*)o0 = ulonglong2{d2u_canon(fp_reduce(s0[0], qinv, q), q), d2u_canon(fp_reduce(s0[1], qinv, q), q)};
  *(ulonglong2*)(o0 + (size_t)a.next * N) =
      ulonglong2{d2u_canon(fp_reduce(s1[0], qinv, q), q), d2u_canon(fp_reduce(s1[1], qinv, q), q)};
}

// Same for integer-class moduli (hoisted rotations only): ext holds canonical residues in the evaluation domain;
// products go through a Montgomery reduction, so acc carries the factor 2^-64 like the fused kernel's.
__global__ void __launch_bounds__(256) inner16_int_kernel(FwdInnerArgs a) {
  const size_t N = 65536;
  u32 b, blk, zi;
  ntt16_map(a.map_mode, b, blk, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const u64 q = mi.m, q2 = 2 * mi.m;
  const u32 n = (blk * 256 + threadIdx.x) * 2;
  u64 s0[2] = {0, 0}, s1[2] = {0, 0};
  const u32 g_own = fwd_inner_galois(a, b);
  const u64* evk = fwd_inner_evk(a, b);
  for (u32 j = 0; j < a.beta; j++) {
    const bool own = fwd_inner_owns(a, t, j);
    const u64* src = own ? a.d + (size_t)b * a.d_poly_stride + (size_t)t * N
                         : a.ext + (((size_t)b * a.beta + j) * a.next + t) * N;
    const u32 g = own ? g_own : a.ext_galois;
    u64 x[2];
    if (g) {
      x[0] = src[galois_src_index16(n, g)];
      x[1] = src[galois_src_index16(n + 1, g)];
    } else {
      const ulonglong2 v = *(const ulonglong2*)(src + n);
      x[0] = v.x;
      x[1] = v.y;
    }
    const u64* kb = evk + (((size_t)j * 2 + 0) * a.nm + id) * N + n;
    const ulonglong2 eb = *(const ulonglong2*)kb;
    const ulonglong2 ea = *(const ulonglong2*)(kb + (size_t)a.nm * N);
    const u64 e0[2] = {eb.x, eb.y}, e1[2] = {ea.x, ea.y};
#pragma unroll
    for (int e = 0; e < 2; e++) {
      Acc128 p0, p1;
      p0.lo = x[e] * e0[e];
      p0.hi = mul_hi64(x[e], e0[e]);
      p1.lo = x[e] * e1[e];
      p1.hi = mul_hi64(x[e], e1[e]);
      s0[e] = csub(s0[e] + redc(p0, q, mi.minv), q2);
      s1[e] = csub(s1[e] + redc(p1, q, mi.minv), q2);
    }
  }
  if (a.c0 && t < a.nlimbs) {   // P * c0 with the same factor 2^-64 as the products above
    const u64* src = a.c0 + (size_t)b * a.c0_poly_stride + (size_t)t * N;
#pragma unroll
    for (int e = 0; e < 2; e++) {
      const u64 v = src[galois_src_index16(n + e, g_own)];
      Acc128 p0;
      p0.lo = v * mi.pmod;
      p0.hi = mul_hi64(v, mi.pmod);
      s0[e] = csub(s0[e] + redc(p0, q, mi.minv), q2);
    }
  }
  u64* o0 = a.acc + (((size_t)b * 2 + 0) * a.next + t) * N + n;
  if (a.accumulate) {   // old values are canonical: a sum below 3q comes back below 2q
    const ulonglong2 p0 = *(const ulonglong2*)o0, p1 = *(const ulonglong2*)(o0 + (size_t)a.next * N);
    s0[0] = csub(s0[0] + p0.x, q2);
    s0[1] = csub(s0[1] + p0.y, q2);
    s1[0] = csub(s1[0] + p1.x, q2);
    s1[1] = csub(s1[1] + p1.y, q2);
  }
  *(ulonglong2*)o0 = ulonglong2{csub(s0[0], q), csub(s0[1], q)};
  *(ulonglong2*)(o0 + (size_t)a.next * N) = ulonglong2{csub(s1[0], q), csub(s1[1], q)};
}

// ---- many rotations of the same hoisted digits in one pass (rotations kept in the extended basis) ----
// acc_r[b][c][t][m] = sum_j D_j[pi_r(m)] * evk_r[j][c][id(t)][m]  (+ P * c0[b][t][pi_r(m)] for c = 0 on main primes),
// pi_r the evaluation-domain index map of rotation r. A lane keeps, for one position n and CB ciphertexts (8 on
// double-precision moduli, 4 on integer-class ones),
// the beta digit values and the c0 term in registers and walks over the rotations: for each one it reads the 2 beta
// key words at m = pi_r^-1(n) once for all its ciphertexts and stores the sums there. The map sends aligned
// 16-element segments onto aligned 16-element segments, so a wave's gathered key reads and scattered stores still
// move whole 128-byte lines; the digits, c1 and c0 are read once for all rotations instead of once per rotation, and a
// key word once per CB ciphertexts. grid = (ceil(B / CB), N / 256, slots of the class), mapped like the
// one-rotation kernels. MAXB bounds beta (the host picks 4 or 8).
#define INNER16_ROT_MAX_BETA 8
#define INNER16_ROT_CB 4
#define INNER16_ROT_CB_FP 8
template <int MAXB, bool EXACT>   // EXACT: beta == MAXB (no per-digit tests), else beta <= MAXB
__global__ void __launch_bounds__(256) inner16_rot_fp_kernel(FwdInnerArgs a, u32 B) {
  constexpr int CB = INNER16_ROT_CB_FP;
  const size_t N = 65536;
  u32 bg, blk, zi;
  ntt16_map(a.map_mode, bg, blk, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const double q = mi.qd, qinv = mi.qinv;
  const u32 n = blk * 256 + threadIdx.x;
  u32 bb[CB];   // a short last group recomputes its last ciphertext in the surplus slots and stores nothing for them
#pragma unroll
  for (int k = 0; k < CB; k++) bb[k] = min(bg * CB + k, B - 1);
  double x[MAXB][CB], pc0[CB];
#pragma unroll
  for (int j = 0; j < MAXB; j++)
#pragma unroll
    for (int k = 0; k < CB; k++) {
      x[j][k] = 0.0;
      if (EXACT || (u32)j < a.beta) {
        if (fwd_inner_owns(a, t, j)) x[j][k] = u2d(a.d[(size_t)bb[k] * a.d_poly_stride + (size_t)t * N + n]);
        else x[j][k] = __longlong_as_double((long long)a.ext[(((size_t)bb[k] * a.beta + j) * a.next + t) * N + n]);
      }
    }
#pragma unroll
  for (int k = 0; k < CB; k++) {   // P * c0, reduced, the same for every rotation
    pc0[k] = 0.0;
    if (a.c0 && t < a.nlimbs)
      pc0[k] = fp_reduce(fp_mulmod_var(u2d(a.c0[(size_t)bb[k] * a.c0_poly_stride + (size_t)t * N + n]), u2d(mi.pmod), qinv, q),
                         qinv, q);
  }
  // the key words of rotation r + 1 are requested before the sums of rotation r are formed
  u64 kw[MAXB][2], kn[MAXB][2];
  u32 m_next = galois_src_index16(n, a.galois_pc[0]);
  const size_t comp_stride = (size_t)a.nm * N, id_off = (size_t)id * N;
  auto load_keys = [&](u64 (&w)[MAXB][2], u32 r, u32 m) {
    const u64* kp = uniform_ptr(a.evk_pc[r]) + id_off + m;
#pragma unroll
    for (int j = 0; j < MAXB; j++) {
      w[j][0] = w[j][1] = 0;
      if (EXACT || (u32)j < a.beta) {
        w[j][0] = kp[0];
        w[j][1] = kp[comp_stride];
      }
      kp += 2 * comp_stride;
    }
  };
  load_keys(kn, 0, m_next);
  for (u32 r = 0; r < a.nrot; r++) {
    const u32 m = m_next;
#pragma unroll
    for (int j = 0; j < MAXB; j++) {
      kw[j][0] = kn[j][0];
      kw[j][1] = kn[j][1];
    }
    if (r + 1 < a.nrot) {
      m_next = galois_src_index16(n, a.galois_pc[r + 1]);
      load_keys(kn, r + 1, m_next);
    }
    double s0[CB], s1[CB];
#pragma unroll
    for (int k = 0; k < CB; k++) {
      s0[k] = pc0[k];
      s1[k] = 0.0;
    }
#pragma unroll
    for (int j = 0; j < MAXB; j++) {
      if (EXACT || (u32)j < a.beta) {
        const double kb = u2d(kw[j][0]), ka = u2d(kw[j][1]);
#pragma unroll
        for (int k = 0; k < CB; k++) {
          s0[k] += fp_mulmod_var(x[j][k], kb, qinv, q);
          s1[k] += fp_mulmod_var(x[j][k], ka, qinv, q);
        }
        // P*c0 (|.| <= q/2) and three products stay below 2^52; fold before more are added
        if ((j == 2 || j == 5) && (EXACT ? j + 1 < MAXB : true)) {
#pragma unroll
          for (int k = 0; k < CB; k++) {
            s0[k] = fp_reduce(s0[k], qinv, q);
            s1[k] = fp_reduce(s1[k], qinv, q);
          }
        }
      }
    }
    u64* o = a.acc + (size_t)r * a.acc_rot_stride + (size_t)t * N + m;
#pragma unroll
    for (int k = 0; k < CB; k++) {
      if (bg * CB + k >= B) break;
      u64* o0 = o + ((size_t)bb[k] * 2 + 0) * a.next * N;
      o0[0] = d2u_canon(fp_reduce(s0[k], qinv, q), q);
      o0[(size_t)a.next * N] = d2u_canon(fp_reduce(s1[k], qinv, q), q);
    }
  }
}

// The same for integer-class moduli: products go through a Montgomery reduction (factor 2^-64, as in the
// one-rotation kernel), P * c0 likewise.
template <int MAXB>
__global__ void __launch_bounds__(256) inner16_rot_int_kernel(FwdInnerArgs a, u32 B) {
  constexpr int CB = INNER16_ROT_CB;
  const size_t N = 65536;
  u32 bg, blk, zi;
  ntt16_map(a.map_mode, bg, blk, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const u64 q = mi.m, q2 = 2 * mi.m;
  const u32 n = blk * 256 + threadIdx.x;
  u32 bb[CB];
#pragma unroll
  for (int k = 0; k < CB; k++) bb[k] = min(bg * CB + k, B - 1);
  u64 x[MAXB][CB], pc0[CB];
#pragma unroll
  for (int j = 0; j < MAXB; j++)
#pragma unroll
    for (int k = 0; k < CB; k++) {
      x[j][k] = 0;
      if ((u32)j < a.beta)
        x[j][k] = fwd_inner_owns(a, t, j) ? a.d[(size_t)bb[k] * a.d_poly_stride + (size_t)t * N + n]
                                          : a.ext[(((size_t)bb[k] * a.beta + j) * a.next + t) * N + n];
    }
#pragma unroll
  for (int k = 0; k < CB; k++) {   // P * c0 * 2^-64, below 2q
    pc0[k] = 0;
    if (a.c0 && t < a.nlimbs) {
      const u64 v = a.c0[(size_t)bb[k] * a.c0_poly_stride + (size_t)t * N + n];
      Acc128 p0 = {v * mi.pmod, mul_hi64(v, mi.pmod)};
      pc0[k] = redc(p0, q, mi.minv);
    }
  }
  for (u32 r = 0; r < a.nrot; r++) {
    const u32 m = galois_src_index16(n, a.galois_pc[r]);
    const u64* evk = uniform_ptr(a.evk_pc[r]) + (size_t)id * N + m;
    // up to 8 products below 2^120 summed in 128 bits, one Montgomery reduction per output (result below 2q)
    Acc128 v0[CB], v1[CB];
#pragma unroll
    for (int k = 0; k < CB; k++) v0[k] = v1[k] = Acc128{0, 0};
#pragma unroll
    for (int j = 0; j < MAXB; j++) {
      if ((u32)j < a.beta) {
        const u64 e0 = evk[((size_t)j * 2 + 0) * a.nm * N], e1 = evk[((size_t)j * 2 + 1) * a.nm * N];
#pragma unroll
        for (int k = 0; k < CB; k++) {
          mac128(v0[k], x[j][k], e0);
          mac128(v1[k], x[j][k], e1);
        }
      }
    }
    u64* o = a.acc + (size_t)r * a.acc_rot_stride + (size_t)t * N + m;
#pragma unroll
    for (int k = 0; k < CB; k++) {
      if (bg * CB + k >= B) break;
      u64* o0 = o + ((size_t)bb[k] * 2 + 0) * a.next * N;
      o0[0] = csub(csub(redc(v0[k], q, mi.minv) + pc0[k], q2), q);
      o0[(size_t)a.next * N] = csub(redc(v1[k], q, mi.minv), q);
    }
  }
}

// ---- a ciphertext plus many of its rotations, summed before ModDown (hoisted rotate-and-sum) ----
// acc[b][c][t][n] = P * ct[b][c][t][n] (main primes; or what acc holds, if accumulate)
//                   + sum_r ( sum_j D_j[pi_r(n)] * evk_r[j][c][id(t)][n]  + [c = 0] P * c0[b][t][pi_r(n)] ),
// output-stationary: a lane owns two adjacent positions, walks over the rotations with its sums in registers (digits,
// c1 and c0 read through rotation r's index map, key words read in place) and stores once. galois_pc[r] is the
// Galois element of rotation r, evk_pc[r] its key; d = c1 and c0 are the two components of the input ciphertext.
// Same grid and mapping as inner16_fp_kernel.
__global__ void __launch_bounds__(256) inner16_sum_fp_kernel(FwdInnerArgs a) {
  const size_t N = 65536;
  u32 b, blk, zi;
  ntt16_map(a.map_mode, b, blk, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const double q = mi.qd, qinv = mi.qinv;
  const u32 n = (blk * 256 + threadIdx.x) * 2;
  const bool main_prime = t < a.nlimbs;
  const double pm = u2d(mi.pmod);
  const u64* c0 = a.c0 + (size_t)b * a.c0_poly_stride + (size_t)t * N;
  const u64* c1 = a.d + (size_t)b * a.d_poly_stride + (size_t)t * N;
  u64* o0 = a.acc + (((size_t)b * 2 + 0) * a.next + t) * N + n;
  u64* o1 = o0 + (size_t)a.next * N;
  double s0[2] = {0.0, 0.0}, s1[2] = {0.0, 0.0};
  if (a.accumulate) {
    const ulonglong2 p0 = *(const ulonglong2*)o0, p1 = *(const ulonglong2*)o1;
    s0[0] = u2d(p0.x), s0[1] = u2d(p0.y), s1[0] = u2d(p1.x), s1[1] = u2d(p1.y);
  } else if (main_prime) {
    const ulonglong2 v0 = *(const ulonglong2*)(c0 + n), v1 = *(const ulonglong2*)(c1 + n);
    s0[0] = fp_mulmod_var(u2d(v0.x), pm, qinv, q), s0[1] = fp_mulmod_var(u2d(v0.y), pm, qinv, q);
    s1[0] = fp_mulmod_var(u2d(v1.x), pm, qinv, q), s1[1] = fp_mulmod_var(u2d(v1.y), pm, qinv, q);
  }
  for (u32 r = 0; r < a.nrot; r++) {
    const u32 g = a.galois_pc[r];
    const u64* evk = uniform_ptr(a.evk_pc[r]) + (size_t)id * N + n;
    const u32 m[2] = {galois_src_index16(n, g), galois_src_index16(n + 1, g)};
    // the running sums enter a rotation below 1.5 q in magnitude; three products (0.75 q each) are added between folds
    u32 pending = 0;
    for (u32 j = 0; j < a.beta; j++) {
      double x[2];
      if (fwd_inner_owns(a, t, j)) {
        x[0] = u2d(c1[m[0]]);
        x[1] = u2d(c1[m[1]]);
      } else {
        const u64* e = a.ext + (((size_t)b * a.beta + j) * a.next + t) * N;
        x[0] = __longlong_as_double((long long)e[m[0]]);
        x[1] = __longlong_as_double((long long)e[m[1]]);
      }
      const ulonglong2 eb = *(const ulonglong2*)(evk + ((size_t)j * 2 + 0) * a.nm * N);
      const ulonglong2 ea = *(const ulonglong2*)(evk + ((size_t)j * 2 + 1) * a.nm * N);
      s0[0] += fp_mulmod_var(x[0], u2d(eb.x), qinv, q);
      s0[1] += fp_mulmod_var(x[1], u2d(eb.y), qinv, q);
      s1[0] += fp_mulmod_var(x[0], u2d(ea.x), qinv, q);
      s1[1] += fp_mulmod_var(x[1], u2d(ea.y), qinv, q);
      if (++pending == 3) {
        pending = 0;
#pragma unroll
        for (int e2 = 0; e2 < 2; e2++) {
          s0[e2] = fp_reduce(s0[e2], qinv, q);
          s1[e2] = fp_reduce(s1[e2], qinv, q);
        }
      }
    }
    if (main_prime) {
      s0[0] += fp_mulmod_var(u2d(c0[m[0]]), pm, qinv, q);
      s0[1] += fp_mulmod_var(u2d(c0[m[1]]), pm, qinv, q);
    }
#pragma unroll
    for (int e2 = 0; e2 < 2; e2++) {   // back to |.| <= q/2 before the next rotation
      s0[e2] = fp_reduce(s0[e2], qinv, q);
      s1[e2] = fp_reduce(s1[e2], qinv, q);
    }
  }
  *(ulonglong2*)o0 = ulonglong2{d2u_canon(fp_reduce(s0[0], qinv, q), q), d2u_canon(fp_reduce(s0[1], qinv, q), q)};
  *(ulonglong2*)o1 = ulonglong2{d2u_canon(fp_reduce(s1[0], qinv, q), q), d2u_canon(fp_reduce(s1[1], qinv, q), q)};
}

// The same for integer-class moduli (every term with the factor 2^-64, as in inner16_int_kernel).
__global__ void __launch_bounds__(256) inner16_sum_int_kernel(FwdInnerArgs a) {
  const size_t N = 65536;
  u32 b, blk, zi;
  ntt16_map(a.map_mode, b, blk, zi);
  const u32 t = a.slots[zi];
  const u32 id = t < a.nlimbs ? t : t - a.nlimbs + a.nq;
  const ModInfo mi = a.mods[id];
  const u64 q = mi.m, q2 = 2 * mi.m;
  const u32 n = (blk * 256 + threadIdx.x) * 2;
  const bool main_prime = t < a.nlimbs;
  const u64* c0 = a.c0 + (size_t)b * a.c0_poly_stride + (size_t)t * N;
  const u64* c1 = a.d + (size_t)b * a.d_poly_stride + (size_t)t * N;
  u64* o0 = a.acc + (((size_t)b * 2 + 0) * a.next + t) * N + n;
  u64* o1 = o0 + (size_t)a.next * N;
  auto times_p = [&](u64 v) {   // v * P * 2^-64, below 2q
    Acc128 p = {v * mi.pmod, mul_hi64(v, mi.pmod)};
    return redc(p, q, mi.minv);
  };
  u64 s0[2] = {0, 0}, s1[2] = {0, 0};   // kept below 2q
  if (a.accumulate) {
    const ulonglong2 p0 = *(const ulonglong2*)o0, p1 = *(const ulonglong2*)o1;
    s0[0] = p0.x, s0[1] = p0.y, s1[0] = p1.x, s1[1] = p1.y;
  } else if (main_prime) {
    const ulonglong2 v0 = *(const ulonglong2*)(c0 + n), v1 = *(const ulonglong2*)(c1 + n);
    s0[0] = times_p(v0.x), s0[1] = times_p(v0.y), s1[0] = times_p(v1.x), s1[1] = times_p(v1.y);
  }
  for (u32 r = 0; r < a.nrot; r++) {
    const u32 g = a.galois_pc[r];
    const u64* evk = uniform_ptr(a.evk_pc[r]) + (size_t)id * N + n;
    const u32 m[2] = {galois_src_index16(n, g), galois_src_index16(n + 1, g)};
    for (u32 j = 0; j < a.beta; j++) {
      const u64* src = fwd_inner_owns(a, t, j) ? c1 : a.ext + (((size_t)b * a.beta + j) * a.next + t) * N;
      const u64 x[2] = {src[m[0]], src[m[1]]};
      const ulonglong2 eb = *(const ulonglong2*)(evk + ((size_t)j * 2 + 0) * a.nm * N);
      const ulonglong2 ea = *(const ulonglong2*)(evk + ((size_t)j * 2 + 1) * a.nm * N);
      const u64 e0[2] = {eb.x, eb.y}, e1[2] = {ea.x, ea.y};
#pragma unroll
      for (int e = 0; e < 2; e++) {
        Acc128 p0 = {x[e] * e0[e], mul_hi64(x[e], e0[e])}, p1 = {x[e] * e1[e], mul_hi64(x[e], e1[e])};
        s0[e] = csub(s0[e] + redc(p0, q, mi.minv), q2);
        s1[e] = csub(s1[e] + redc(p1, q, mi.minv), q2);
      }
    }
    if (main_prime) {
      s0[0] = csub(s0[0] + times_p(c0[m[0]]), q2);
      s0[1] = csub(s0[1] + times_p(c0[m[1]]), q2);
    }
  }
  *(ulonglong2*)o0 = ulonglong2{csub(s0[0], q), csub(s0[1], q)};
  *(ulonglong2*)o1 = ulonglong2{csub(s1[0], q), csub(s1[1], q)};
}
