// Host side of libckks_mi355: context tables, argument checks, launch sequences.
#include "../../include/ckks_mi355.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <string>
#include <vector>

#include "kernels.hip.h"
#include "ntt12.hip.h"
#include "ntt16_kernels.hip.h"

typedef unsigned __int128 u128;

// Workspace of ckks_hrot_noalloc, the entry point for callers that cannot allocate: a fixed array in the library's
// own device image (one copy per GPU, held until the process ends). Host code never passes the array's name to a
// kernel or a copy: it uses the per-device address that hipGetSymbolAddress returns (ckks_ctx::scratch_ptr).
#define CKKS_NOALLOC_SCRATCH_BYTES (128ull << 20)
static __device__ __align__(256) unsigned char scratch[CKKS_NOALLOC_SCRATCH_BYTES];

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) {
  g_err = msg;
  return code;
}
#define HIP_TRY(expr)                                                                            \
  do {                                                                                           \
    hipError_t e_ = (expr);                                                                      \
    if (e_ != hipSuccess) return fail(CKKS_EHIP, std::string(#expr ": ") + hipGetErrorString(e_)); \
  } while (0)

// ---- host modular arithmetic (table generation only) ----
inline u64 h_mul(u64 a, u64 b, u64 m) { return (u64)((u128)a * b % m); }
u64 h_pow(u64 a, u64 e, u64 m) {
  u64 r = 1;
  a %= m;
  for (; e; e >>= 1) {
    if (e & 1) r = h_mul(r, a, m);
    a = h_mul(a, a, m);
  }
  return r;
}
inline u64 h_inv(u64 a, u64 m) { return h_pow(a, m - 2, m); }
inline u64 h_shoup(u64 w, u64 m) { return (u64)(((u128)w << 64) / m); }
inline u64 h_mont(u64 v, u64 m) { return (u64)(((u128)v << 64) % m); }  // v * 2^64 mod m
inline u64 h_mont90(u64 v, u64 m) { return h_mul(h_mont(v, m), (u64)(1ull << 26) % m, m); }  // v * 2^90 mod m
inline u32 h_bits(u64 v) {
  u32 b = 0;
  while (v) v >>= 1, b++;
  return b;
}
// Whether a base conversion with at most `n` sources below 2^bs into targets below 2^bt may use the three-sum
// accumulation and the base-2^30 reduction (dot30n_*): none of the three sums, including what the reduction adds
// to them, may reach 2^64.
inline bool bconv_narrow_ok(u32 n, u32 bs, u32 bt, u32 bt_min) {
  if (bs > 60 || bt > 60 || bt_min < 36) return false;  // the result is below m + 2^34 and gets one correction
  if (n > 15) n = 15;  // chunks of 15 terms are reduced separately
  const u128 one = 1, w = (one << 30) - 1;
  const u128 y1 = one << (bs > 30 ? bs - 30 : 0), c1 = one << (bt > 30 ? bt - 30 : 0);
  const u128 amax = (u128)n * w * w + (u128)n * w + w * w;
  const u128 bmax = (u128)n * (w * c1 + y1 * w) + (u128)n * c1 + (one << 34) + w * c1 + w * w;
  const u128 cmax = (u128)n * y1 * c1 + (one << 34) + w * c1 + w * w;
  const u128 lim = one << 64;
  return amax < lim && bmax < lim && cmax < lim;
}
bool h_is_prime(u64 n) {
  if (n < 2) return false;
  const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
  for (u64 b : bases)
    if (n % b == 0) return n == b;
  u64 d = n - 1;
  int r = 0;
  while (!(d & 1)) d >>= 1, r++;
  for (u64 a : bases) {
    u64 x = h_pow(a, d, n);
    if (x == 1 || x == n - 1) continue;
    bool composite = true;
    for (int i = 1; i < r && composite; i++) {
      x = h_mul(x, x, n);
      if (x == n - 1) composite = false;
    }
    if (composite) return false;
  }
  return true;
}
inline u32 h_brev(u32 x, u32 bits) {
  u32 r = 0;
  for (u32 i = 0; i < bits; i++) r |= ((x >> i) & 1) << (bits - 1 - i);
  return r;
}

struct Pass {
  u32 s0, k, logC, tile_log;
};

// Number of source rows the base-conversion kernels are instantiated for (the smallest that covers n).
inline u32 bconv_rows(u32 n) { return n <= 4 ? 4 : n <= 8 ? 8 : n <= 15 ? 15 : n <= 24 ? 24 : n <= 36 ? 36 : 45; }

// Base-conversion constants for ciphertexts at one limb count.
struct LevelTables {
  u32 nlimbs = 0, beta = 0, next = 0;
  bool narrow_up = false, narrow_dn = false, narrow_rs = false;  // which reduction the constants are scaled for
  ulonglong2* up_inv = nullptr;  // [beta][alpha]
  u64* up_mat = nullptr;         // [beta][alpha+1][next]
  ulonglong2* dn_inv = nullptr;  // [K]
  u64* dn_mat = nullptr;         // [K+1][nlimbs]
  ulonglong2* pinv = nullptr;    // [nlimbs]
  // N = 2^16 fused path
  ulonglong2* up_scale = nullptr;  // [nlimbs]  (Q_j/q_i)^-1 / N mod q_i
  ulonglong2* dn_scale = nullptr;  // [K]       2^64 (P/p_k)^-1 / N mod p_k
  u64* dn_mat_plain = nullptr;     // dn_mat without the Montgomery factor
  u64* up_off = nullptr;           // [beta][next] -sum_i ((q_i-1)/2) (Q_j/q_i) mod m_t, scaled like up_mat
  u64* dn_off = nullptr;           // [nlimbs]     -sum_k ((p_k-1)/2) (P/p_k) mod q_i, scaled like dn_mat_plain
  u32 up_pitch = 0, dn_pitch = 0;  // constants per target in up_mat / dn_mat_plain
  ulonglong2* pinv2 = nullptr;     // [nlimbs]  2^64 / P mod q_i
  // rescale from this limb count: drop q_{nlimbs-1}
  ulonglong2* rs_one = nullptr;    // [1]          Shoup pair of 1 (the single source needs no pre-scaling)
  u64* rs_mat = nullptr;           // [nlimbs-1][5] row i = (1, 0, 0, 0, -q_last) mod q_i, Montgomery form
  ulonglong2* rs_qinv = nullptr;   // [nlimbs-1]   q_last^-1 mod q_i, Shoup pair
  ulonglong2* rs_qinv16 = nullptr; // same for the N = 2^16 kernels: (c, c/q) doubles on double-precision moduli
};

}  // namespace

enum ProfKind {
  PK_NTT_FWD = 0, PK_NTT_INV,
  // N = 2^16 kernels: three consecutive kinds each, one per modulus class (the kernel's template argument)
  PK_FWD_ROWS, PK_FWD_BLOCKS = PK_FWD_ROWS + 3, PK_INV_BLOCKS = PK_FWD_BLOCKS + 3, PK_INV_ROWS = PK_INV_BLOCKS + 3,
  PK_FWD_FINAL = PK_INV_ROWS + 3,
  PK_AUTOMORPH = PK_FWD_FINAL + 3, PK_MODUP, PK_INNER, PK_INNER16, PK_INNER16_INT, PK_INNER_C, PK_INNER8, PK_INNER8_BIG, PK_BCONV_ROWS, PK_MODDOWN = PK_BCONV_ROWS + 3, PK_FINAL, PK_TENSOR, PK_PMACC, PK_PMACC_FP, PK_ADD,
  PK_COPY, PK_COUNT
};
static const char* const kProfNames[PK_COUNT] = {
    "ntt_fwd_pass", "ntt_inv_pass",
    "ntt16_fwd_rows_kernel<0>", "ntt16_fwd_rows_kernel<1>", "ntt16_fwd_rows_kernel<2>",
    "ntt16_fwd_blocks_kernel<0>", "ntt16_fwd_blocks_kernel<1>", "ntt16_fwd_blocks_kernel<2>",
    "ntt16_inv_blocks_kernel<0>", "ntt16_inv_blocks_kernel<1>", "ntt16_inv_blocks_kernel<2>",
    "ntt16_inv_rows_kernel<0>", "ntt16_inv_rows_kernel<1>", "ntt16_inv_rows_kernel<2>",
    "ntt16_fwd_blocks_final_kernel<0>", "ntt16_fwd_blocks_final_kernel<1>", "ntt16_fwd_blocks_final_kernel<2>",
    "automorph_kernel", "modup_kernel", "inner_kernel", "inner16_fp_kernel", "inner16_int_kernel", "ntt16_fwd_blocks_inner_c_kernel", "ntt16_fwd_blocks_inner8_kernel<1>", "ntt16_fwd_blocks_inner8_kernel<2>",
    "ntt16_bconv_rows_kernel<0>", "ntt16_bconv_rows_kernel<1>", "ntt16_bconv_rows_kernel<2>", "moddown_kernel", "ks_final_kernel", "tensor_kernel",
    "pmacc_int_kernel", "pmacc_fp_kernel", "addto_kernel", "copy"};
struct ProfRec {
  int kind;
  hipEvent_t start, stop;
};

struct ckks_ctx {
  // Tuning knobs (ckks_tune_set; meanings in the public header). 0: workgroup mapping of the N = 2^16 kernels (-1: per
  // kernel); 1: integer bodies everywhere; 2: 1 = base conversions inside the row passes; 3: 2 = inner product fused
  // with the final assembly on double-precision main limbs, 1 = separate kernels; 4: 0 = fork part of a key switch onto
  // the second stream; 5: general base-conversion reduction; 6: integer PCMM inner sums; 7: cap on giant steps per pass.
  int tune[8] = {-1, 0, 0, 2, 1, 0, 0, 0};
  bool prof_on = false;
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_pool;
  double prof_ms[PK_COUNT] = {0};
  uint64_t prof_n[PK_COUNT] = {0};
  int device = 0;
  u32 logN = 0, N = 0, nq = 0, np = 0, nm = 0, dnum = 0, alpha = 0;
  std::vector<u64> mod, psi;
  ModInfo* d_mods = nullptr;
  ulonglong2* d_tw_fwd = nullptr;
  ulonglong2* d_tw_inv = nullptr;
  double* d_twfp_fwd = nullptr;  // N = 2^16 only: the twiddles as doubles for moduli < 2^50
  double* d_twfp_inv = nullptr;
  hipStream_t side = nullptr;       // second stream for the fork/join inside a key switch (default priority)
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  std::vector<Pass> passes;  // forward order
  // Base-conversion constants of every limb count 1..nq, built when the context is created (and again when knob 1
  // or 5 changes): levels[nlimbs] points into one device allocation, d_levels.
  std::vector<LevelTables> levels;
  char* d_levels = nullptr;
  void* scratch_ptr = nullptr;  // this device's address of `scratch` (hipGetSymbolAddress at context creation)
};

namespace {

template <class T>
int upload(T** dst, const std::vector<T>& src) {
  HIP_TRY(hipMalloc((void**)dst, std::max<size_t>(1, src.size()) * sizeof(T)));
  if (!src.empty()) HIP_TRY(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
  return CKKS_OK;
}

struct DeviceGuard {
  int prev = -1;
  bool ok = false;
  explicit DeviceGuard(int dev) {
    if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true;
  }
  ~DeviceGuard() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

// Brackets the launches made during its lifetime with two events on their stream (only when profiling is on).
struct ProfScope {
  ckks_ctx* c;
  hipStream_t st;
  ProfRec rec;
  bool active = false;
  ProfScope(const ckks_ctx* cc, int kind, hipStream_t s) : c(const_cast<ckks_ctx*>(cc)), st(s) {
    if (!c->prof_on) return;
    auto get = [&](hipEvent_t* e) {
      if (!c->prof_pool.empty()) {
        *e = c->prof_pool.back();
        c->prof_pool.pop_back();
        return true;
      }
      return hipEventCreate(e) == hipSuccess;
    };
    rec.kind = kind;
    if (!get(&rec.start)) return;
    if (!get(&rec.stop)) {
      c->prof_pool.push_back(rec.start);
      return;
    }
    active = hipEventRecord(rec.start, st) == hipSuccess;
  }
  ~ProfScope() {
    if (!active) return;
    (void)hipEventRecord(rec.stop, st);
    c->prof_recs.push_back(rec);
  }
};

// Host image of the device allocation that holds the level tables: every table starts on a 256-byte boundary; the
// LevelTables pointers hold offsets until the image has been uploaded.
struct LevelArena {
  std::vector<char> host;
  template <class T>
  T* add(const std::vector<T>& v) {
    const size_t off = (host.size() + 255) & ~(size_t)255;
    host.resize(off + std::max<size_t>(1, v.size()) * sizeof(T));
    if (!v.empty()) memcpy(host.data() + off, v.data(), v.size() * sizeof(T));
    return (T*)off;
  }
};

// Constants for ciphertexts at `nlimbs` limbs, appended to the arena (pointers are offsets into it).
LevelTables build_level(const ckks_ctx* c, u32 nlimbs, LevelArena& arena) {
  const bool fp_on = c->tune[1] == 0;
  auto is_fp = [&](u64 m) { return fp_on && (m >> 50) == 0; };
  LevelTables t;
  t.nlimbs = nlimbs;
  t.beta = (nlimbs + c->alpha - 1) / c->alpha;
  t.next = nlimbs + c->np;
  const u32 alpha = c->alpha, K = c->np, next = t.next;
  auto ext_mod = [&](u32 s) { return s < nlimbs ? c->mod[s] : c->mod[c->nq + (s - nlimbs)]; };

  // constants of one output are contiguous: [digit][target][R+1], rows >= digit length are zero, row R = -Q_j
  const u32 R = bconv_rows(alpha), RK = bconv_rows(K);
  u32 bq = 0, bq_min = 64, bp = 0, bp_min = 64;
  for (u32 i = 0; i < nlimbs; i++) bq = std::max(bq, h_bits(c->mod[i])), bq_min = std::min(bq_min, h_bits(c->mod[i]));
  for (u32 k = 0; k < K; k++)
    bp = std::max(bp, h_bits(c->mod[c->nq + k])), bp_min = std::min(bp_min, h_bits(c->mod[c->nq + k]));
  t.narrow_up = c->tune[5] == 0 && bconv_narrow_ok(std::min(alpha, nlimbs), bq, std::max(bq, bp), std::min(bq_min, bp_min));
  t.narrow_dn = c->tune[5] == 0 && bconv_narrow_ok(K, bp, bq, bq_min);
  t.narrow_rs = c->tune[5] == 0 && bconv_narrow_ok(1, bq, bq, bq_min);
  auto mont_up = [&](u64 v, u64 m) { return t.narrow_up ? h_mont90(v, m) : h_mont(v, m); };
  auto mont_dn = [&](u64 v, u64 m) { return t.narrow_dn ? h_mont90(v, m) : h_mont(v, m); };
  auto mont_rs = [&](u64 v, u64 m) { return t.narrow_rs ? h_mont90(v, m) : h_mont(v, m); };
  std::vector<ulonglong2> up_inv((size_t)t.beta * alpha, ulonglong2{0, 0});
  std::vector<u64> up_mat((size_t)t.beta * next * (R + 1), 0), up_off((size_t)t.beta * next, 0);
  t.up_pitch = R + 1;
  t.dn_pitch = RK + 1;
  for (u32 j = 0; j < t.beta; j++) {
    u32 lo = j * alpha, hi = std::min(lo + alpha, nlimbs);
    for (u32 i = lo; i < hi; i++) {
      u64 qi = c->mod[i], h = 1;
      for (u32 k = lo; k < hi; k++)
        if (k != i) h = h_mul(h, c->mod[k] % qi, qi);
      u64 inv = h_inv(h, qi);
      up_inv[(size_t)j * alpha + (i - lo)] = ulonglong2{inv, h_shoup(inv, qi)};
      for (u32 s = 0; s < next; s++) {
        u64 m = ext_mod(s), v = 1;
        for (u32 k = lo; k < hi; k++)
          if (k != i) v = h_mul(v, c->mod[k] % m, m);
        up_mat[((size_t)j * next + s) * (R + 1) + (i - lo)] = mont_up(v, m);
      }
    }
    for (u32 s = 0; s < next; s++) {
      u64 m = ext_mod(s), v = 1;
      for (u32 k = lo; k < hi; k++) v = h_mul(v, c->mod[k] % m, m);
      up_mat[((size_t)j * next + s) * (R + 1) + R] = mont_up(v ? m - v : 0, m);
      // offset of the shifted-residue form: -sum_i h_i (Q_j/q_i), h_i = (q_i - 1) / 2
      u64 sum = 0;
      for (u32 i = lo; i < hi; i++) {
        u64 w = 1;
        for (u32 k = lo; k < hi; k++)
          if (k != i) w = h_mul(w, c->mod[k] % m, m);
        sum = (u64)(((u128)sum + h_mul(w, ((c->mod[i] - 1) / 2) % m, m)) % m);
      }
      up_off[(size_t)j * next + s] = mont_up(sum ? m - sum : 0, m);
    }
  }
  std::vector<ulonglong2> dn_inv(K), pinv(nlimbs);
  std::vector<u64> dn_mat((size_t)nlimbs * (RK + 1), 0);
  for (u32 k = 0; k < K; k++) {
    u64 pk = c->mod[c->nq + k], h = 1;
    for (u32 r = 0; r < K; r++)
      if (r != k) h = h_mul(h, c->mod[c->nq + r] % pk, pk);
    u64 inv = h_inv(h, pk);
    dn_inv[k] = ulonglong2{inv, h_shoup(inv, pk)};
    for (u32 i = 0; i < nlimbs; i++) {
      u64 m = c->mod[i], v = 1;
      for (u32 r = 0; r < K; r++)
        if (r != k) v = h_mul(v, c->mod[c->nq + r] % m, m);
      dn_mat[(size_t)i * (RK + 1) + k] = mont_dn(v, m);
    }
  }
  for (u32 i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i], v = 1;
    for (u32 r = 0; r < K; r++) v = h_mul(v, c->mod[c->nq + r] % m, m);
    dn_mat[(size_t)i * (RK + 1) + RK] = mont_dn(v ? m - v : 0, m);
    u64 inv = h_inv(v, m);
    pinv[i] = ulonglong2{inv, h_shoup(inv, m)};
  }
  // Constants of the fused N = 2^16 path. 16-byte slots hold a Shoup pair (integer-class modulus) or the doubles
  // (c, c/q) (double-precision class). Integer-class accumulators carry a factor 2^-64 (Montgomery products), which
  // dn_scale and pinv2 undo; double-precision accumulators are plain.
  std::vector<ulonglong2> up_scale(nlimbs), dn_scale(K), pinv2(nlimbs);
  std::vector<u64> dn_mat_plain(dn_mat.size(), 0), dn_off(nlimbs, 0);
  auto as_fp = [](u64 v, u64 m) {
    double2 d{(double)v, (double)v / (double)m};
    ulonglong2 r;
    memcpy(&r, &d, sizeof(r));
    return r;
  };
  for (u32 i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i], ninv = h_inv(c->N % m, m);
    u64 v = h_mul(up_inv[(size_t)(i / alpha) * alpha + (i % alpha)].x, ninv, m);
    u64 r64_inv = h_inv(h_mont(1, m), m);
    {
      u64 sum = 0;   // -sum_k h_k (P/p_k) mod m, then scaled like the row of constants below
      for (u32 k = 0; k < K; k++) {
        u64 w = 1;
        for (u32 r = 0; r < K; r++)
          if (r != k) w = h_mul(w, c->mod[c->nq + r] % m, m);
        sum = (u64)(((u128)sum + h_mul(w, ((c->mod[c->nq + k] - 1) / 2) % m, m)) % m);
      }
      const u64 neg = mont_dn(sum ? m - sum : 0, m);
      dn_off[i] = is_fp(m) ? neg : h_mul(neg, r64_inv, m);
    }
    if (is_fp(m)) {
      up_scale[i] = as_fp(v, m);
      pinv2[i] = as_fp(pinv[i].x, m);
      for (u32 k = 0; k <= RK; k++) dn_mat_plain[(size_t)i * (RK + 1) + k] = dn_mat[(size_t)i * (RK + 1) + k];
    } else {
      up_scale[i] = ulonglong2{v, h_shoup(v, m)};
      u64 w = h_mont(pinv[i].x, m);
      pinv2[i] = ulonglong2{w, h_shoup(w, m)};
      // stored constants are c * 2^64; multiply by 2^-64 so the Montgomery reduction leaves t * 2^-64
      for (u32 k = 0; k <= RK; k++)
        dn_mat_plain[(size_t)i * (RK + 1) + k] = h_mul(dn_mat[(size_t)i * (RK + 1) + k], r64_inv, m);
    }
  }
  for (u32 k = 0; k < K; k++) {
    u64 m = c->mod[c->nq + k], ninv = h_inv(c->N % m, m);
    u64 v = h_mul(dn_inv[k].x, ninv, m);
    if (is_fp(m)) {
      dn_scale[k] = as_fp(v, m);
    } else {
      u64 w = h_mont(v, m);
      dn_scale[k] = ulonglong2{w, h_shoup(w, m)};
    }
  }
  std::vector<ulonglong2> rs_one(1), rs_qinv(nlimbs > 1 ? nlimbs - 1 : 0), rs_qinv16(rs_qinv.size());
  std::vector<u64> rs_mat(rs_qinv.size() * 5, 0);
  rs_one[0] = ulonglong2{1, 0};  // floor(1 * 2^64 / q) is filled per use below; with x < q the product x*1 needs no reduction
  if (nlimbs > 1) {
    const u64 qL = c->mod[nlimbs - 1];
    rs_one[0] = ulonglong2{1, h_shoup(1, qL)};
    for (u32 i = 0; i + 1 < nlimbs; i++) {
      u64 m = c->mod[i], ql = qL % m, inv = h_inv(ql, m);
      rs_mat[(size_t)i * 5 + 0] = mont_rs(1, m);
      rs_mat[(size_t)i * 5 + 4] = mont_rs(ql ? m - ql : 0, m);
      rs_qinv[i] = ulonglong2{inv, h_shoup(inv, m)};
      rs_qinv16[i] = is_fp(m) ? as_fp(inv, m) : rs_qinv[i];
    }
  }
  t.rs_one = arena.add(rs_one);
  t.rs_mat = arena.add(rs_mat);
  t.rs_qinv = arena.add(rs_qinv);
  t.rs_qinv16 = arena.add(rs_qinv16);
  t.up_scale = arena.add(up_scale);
  t.dn_scale = arena.add(dn_scale);
  t.dn_mat_plain = arena.add(dn_mat_plain);
  t.up_off = arena.add(up_off);
  t.dn_off = arena.add(dn_off);
  t.pinv2 = arena.add(pinv2);
  t.up_inv = arena.add(up_inv);
  t.up_mat = arena.add(up_mat);
  t.dn_inv = arena.add(dn_inv);
  t.dn_mat = arena.add(dn_mat);
  t.pinv = arena.add(pinv);
  return t;
}

// (Re)build the tables of all limb counts under the current knobs 1 and 5: one allocation, one copy. Called from
// ckks_ctx_create and from ckks_tune_set, never from a call that enqueues work.
int build_levels(ckks_ctx* c) {
  LevelArena arena;
  std::vector<LevelTables> lv(c->nq + 1);
  for (u32 nl = 1; nl <= c->nq; nl++) lv[nl] = build_level(c, nl, arena);
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  char* dev = nullptr;
  HIP_TRY(hipMalloc((void**)&dev, arena.host.size()));
  hipError_t e = hipMemcpy(dev, arena.host.data(), arena.host.size(), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(dev);
    return fail(CKKS_EHIP, std::string("uploading the level tables: ") + hipGetErrorString(e));
  }
  auto rebase = [&](auto*& ptr) { ptr = (std::remove_reference_t<decltype(ptr)>)(dev + (size_t)ptr); };
  for (u32 nl = 1; nl <= c->nq; nl++) {
    LevelTables& t = lv[nl];
    rebase(t.up_inv); rebase(t.up_mat); rebase(t.dn_inv); rebase(t.dn_mat); rebase(t.pinv);
    rebase(t.up_scale); rebase(t.dn_scale); rebase(t.dn_mat_plain); rebase(t.pinv2);
    rebase(t.up_off); rebase(t.dn_off);
    rebase(t.rs_one); rebase(t.rs_mat); rebase(t.rs_qinv); rebase(t.rs_qinv16);
  }
  if (c->d_levels) {
    // a knob changed: nothing may still be reading the old tables
    HIP_TRY(hipDeviceSynchronize());
    (void)hipFree(c->d_levels);
  }
  c->d_levels = dev;
  c->levels.swap(lv);
  return CKKS_OK;
}

// Table look-up only: no allocation, no copy, no synchronisation.
int get_level(const ckks_ctx* c, u32 nlimbs, const LevelTables** out) {
  if (nlimbs == 0 || nlimbs >= c->levels.size()) return fail(CKKS_ESHAPE, "nlimbs must be in [1, L+1]");
  *out = &c->levels[nlimbs];
  return CKKS_OK;
}

LimbMap identity_map(u32 n) {
  LimbMap m;
  for (u32 i = 0; i < CKKS_MAX_SLOTS; i++) m.id[i] = (unsigned char)(i < n ? i : 0);
  return m;
}
// slots 0..nlimbs-1 -> q ids, then the K special primes
LimbMap ext_map(const ckks_ctx* c, u32 nlimbs) {
  LimbMap m = identity_map(nlimbs);
  for (u32 k = 0; k < c->np; k++) m.id[nlimbs + k] = (unsigned char)(c->nq + k);
  return m;
}

// Enqueue a transform of npoly polynomials x slots [slot0, slot0+nslots): reads src, writes dst (src == dst for an
// in-place transform; out of place is supported only on the N = 2^16 path). Rows are *_stride elements apart.
// Modulus class on the N = 2^16 path (must match mod_class() on the device).
inline int host_class(const ckks_ctx* c, u64 m) {
  if (c->tune[1] == 0 && (m >> 50) == 0) return 0;
  return (m >> 52) == 0 ? 1 : 2;
}
// Workgroup-to-tile mapping of the N = 2^16 kernels (ntt16_map). Knob 0 >= 0 forces one mode everywhere; by default
// the transform passes and the final assembly, which share nothing but twiddles across polynomials, take the
// XCD-swizzled tile-major order (measured best for them), and the kernels that read the key take the
// group-per-XCD order when the batch shares one key (its slices then stay in that XCD's L2) and the plain
// tile-major order when every ciphertext has its own.
inline u32 map_mode_pass(const ckks_ctx* c) { return c->tune[0] >= 0 ? (u32)c->tune[0] : 3u; }
inline u32 map_mode_inner(const ckks_ctx* c, bool shared_key) {
  return c->tune[0] >= 0 ? (u32)c->tune[0] : shared_key ? 4u : 2u;
}
// Launch KERNEL<cls> once per modulus class present among `nslots` slots, with ARGS.slots listing that class's slots.
#define LAUNCH_BY_CLASS(CTX, PKBASE, KERNEL, ARGS, NX, NSLOTS, CLASS_OF_SLOT, STREAM)                      \
  for (int cls_ = 0; cls_ < 3; cls_++) {                                                                    \
    u32 cnt_ = 0;                                                                                           \
    for (u32 s_ = 0; s_ < (NSLOTS); s_++)                                                                   \
      if ((CLASS_OF_SLOT(s_)) == cls_) (ARGS).slots[cnt_++] = (unsigned char)s_;                            \
    if (!cnt_) continue;                                                                                    \
    dim3 grid_((NX), 16, cnt_), block_(NTT16_THREADS);                                                      \
    ProfScope ps_((CTX), (PKBASE) + cls_, (STREAM));                                                        \
    if (cls_ == 0) hipLaunchKernelGGL((KERNEL<0>), grid_, block_, 0, (STREAM), (ARGS));                     \
    else if (cls_ == 1) hipLaunchKernelGGL((KERNEL<1>), grid_, block_, 0, (STREAM), (ARGS));                \
    else hipLaunchKernelGGL((KERNEL<2>), grid_, block_, 0, (STREAM), (ARGS));                               \
  }

struct NttOpts {
  u32 galois = 0;                     // N = 2^16 inverse only: read src through the eval-domain Galois map
  const u32* galois_pc = nullptr;     // same, one element per polynomial (host array, npoly <= KS_MULTI_MAX entries)
  const ulonglong2* scale = nullptr;  // N = 2^16 inverse only: per-slot constants (from slot0) replacing N^-1
  bool split_out = false;             // N = 2^16 inverse only: write the shifted, split form the fused base conversion reads
  bool rows_only = false;             // N = 2^16 forward only: stop after the row pass (a fused kernel does the rest)
  bool blocks_only = false;           // N = 2^16 forward only: only the block pass, in place on dst
  bool raw_out = false;               // with blocks_only: leave reduced doubles on double-precision moduli
  int only_class = -1;                // >= 0: touch only the slots of this modulus class
  int exclude_class = -1;             // >= 0: leave the slots of this modulus class alone
};
int launch_ntt(const ckks_ctx* c, bool inverse, const u64* src, u64 src_stride, u64* dst, u64 dst_stride, u32 npoly,
               u32 slot0, u32 nslots, const LimbMap& ids_from_slot0, u32 skip_beta, u32 skip_nq, hipStream_t st,
               const NttOpts& opt = NttOpts()) {
  if (npoly == 0 || nslots == 0) return CKKS_OK;
  const int kind = inverse ? PK_NTT_INV : PK_NTT_FWD;
  if (c->logN == 16) {
    Ntt16Args a;
    a.src = src + (size_t)slot0 * c->N;
    a.dst = dst + (size_t)slot0 * c->N;
    a.tw = inverse ? c->d_tw_inv : c->d_tw_fwd;
    a.twfp = inverse ? c->d_twfp_inv : c->d_twfp_fwd;
    a.mods = c->d_mods;
    a.src_poly_stride = src_stride;
    a.dst_poly_stride = dst_stride;
    a.skip_beta = skip_beta;
    a.skip_alpha = c->alpha;
    a.skip_nq = skip_nq;
    for (u32 i = 0; i < 128; i++) a.id[i] = ids_from_slot0.id[i];
    a.map_mode = map_mode_pass(c);
    a.galois = opt.galois;
    if (opt.galois_pc) {
      if (npoly > KS_MULTI_MAX) return fail(CKKS_ESHAPE, "internal: per-polynomial Galois elements for too many polynomials");
      a.multi = 1;
      for (u32 i = 0; i < npoly; i++) a.galois_pc[i] = opt.galois_pc[i];
    }
    a.scale = opt.scale;
    a.raw_out = opt.raw_out ? 1 : 0;
    a.split_out = opt.split_out ? 1 : 0;
    Ntt16Args b = a;  // second pass: in place on dst
    b.src = a.dst;
    b.src_poly_stride = dst_stride;
    auto cls_of = [&](u32 s) {
      int k = host_class(c, c->mod[ids_from_slot0.id[s]]);
      if (opt.only_class >= 0 && k != opt.only_class) return -1;
      if (opt.exclude_class >= 0 && k == opt.exclude_class) return -1;
      return k;
    };
    if (!inverse) {
      if (!opt.blocks_only) {
        LAUNCH_BY_CLASS(c, PK_FWD_ROWS, ntt16_fwd_rows_kernel, a, npoly, nslots, cls_of, st)
      }
      if (!opt.rows_only) {
        LAUNCH_BY_CLASS(c, PK_FWD_BLOCKS, ntt16_fwd_blocks_kernel, b, npoly, nslots, cls_of, st)
      }
    } else {
      LAUNCH_BY_CLASS(c, PK_INV_BLOCKS, ntt16_inv_blocks_kernel, a, npoly, nslots, cls_of, st)
      LAUNCH_BY_CLASS(c, PK_INV_ROWS, ntt16_inv_rows_kernel, b, npoly, nslots, cls_of, st)
    }
    HIP_TRY(hipGetLastError());
    return CKKS_OK;
  }
  if (c->logN == 12) {
    // the whole limb in one workgroup: all 12 stages in one pass over memory, in or out of place
    Ntt12Args a;
    a.src = src + (size_t)slot0 * c->N;
    a.dst = dst + (size_t)slot0 * c->N;
    a.tw = inverse ? c->d_tw_inv : c->d_tw_fwd;
    a.twfp = inverse ? c->d_twfp_inv : c->d_twfp_fwd;
    a.mods = c->d_mods;
    a.src_poly_stride = src_stride;
    a.dst_poly_stride = dst_stride;
    a.skip_beta = skip_beta;
    a.skip_alpha = c->alpha;
    a.skip_nq = skip_nq;
    a.fp_on = c->tune[1] == 0 ? 1u : 0u;
    for (u32 i = 0; i < 128; i++) a.id[i] = ids_from_slot0.id[i];
    const u32 chunk = 65535 - (skip_beta ? 65535 % skip_beta : 0);   // grid.x carries the polynomial index; whole digit groups
    for (u32 p0 = 0; p0 < npoly; p0 += chunk) {
      const u32 np_ = std::min<u32>(chunk, npoly - p0);
      Ntt12Args b = a;
      b.src += (size_t)p0 * src_stride;
      b.dst += (size_t)p0 * dst_stride;
      ProfScope ps(c, kind, st);
      if (inverse) hipLaunchKernelGGL(ntt12_kernel<true>, dim3(np_, nslots), dim3(256), 0, st, b);
      else hipLaunchKernelGGL(ntt12_kernel<false>, dim3(np_, nslots), dim3(256), 0, st, b);
    }
    HIP_TRY(hipGetLastError());
    return CKKS_OK;
  }
  if (src != dst) {
    ProfScope ps(c, PK_COPY, st);
    // generic path is in place: copy the slots first (rows may be strided)
    HIP_TRY(hipMemcpy2DAsync(dst + (size_t)slot0 * c->N, dst_stride * 8, src + (size_t)slot0 * c->N, src_stride * 8,
                             (size_t)nslots * c->N * 8, npoly, hipMemcpyDeviceToDevice, st));
  }
  NttArgs a;
  a.data = dst + (size_t)slot0 * c->N;
  a.tw = inverse ? c->d_tw_inv : c->d_tw_fwd;
  a.mods = c->d_mods;
  a.poly_stride = dst_stride;
  a.logN = c->logN;
  a.skip_beta = skip_beta;
  a.skip_alpha = c->alpha;
  a.skip_nq = skip_nq;
  a.ids = ids_from_slot0;
  const size_t np = c->passes.size();
  for (size_t i = 0; i < np; i++) {
    const Pass& p = c->passes[inverse ? np - 1 - i : i];
    a.s0 = p.s0;
    a.k = p.k;
    a.logC = p.logC;
    a.tile_log = p.tile_log;
    dim3 grid(npoly, c->N >> p.tile_log, nslots);
    size_t lds = sizeof(u64) << p.tile_log;
    ProfScope ps(c, kind, st);
    if (inverse)
      hipLaunchKernelGGL(ntt_pass_kernel<true>, grid, dim3(NTT_THREADS), lds, st, a);
    else
      hipLaunchKernelGGL(ntt_pass_kernel<false>, grid, dim3(NTT_THREADS), lds, st, a);
  }
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}

u32 inv_mod_pow2(u32 g, u32 bits) {  // inverse of odd g modulo 2^bits
  u32 x = 1;
  for (int i = 0; i < 6; i++) x *= 2 - g * x;
  return x & ((bits >= 32) ? 0xFFFFFFFFu : ((1u << bits) - 1));
}

int launch_automorph(const ckks_ctx* c, u64* out, u64 out_stride, const u64* in, u64 in_stride, u32 npoly, u32 nslots,
                     const LimbMap& ids, u32 g, bool eval_domain, hipStream_t st) {
  if (npoly == 0 || nslots == 0) return CKKS_OK;
  AutoArgs a;
  a.out = out;
  a.in = in;
  a.mods = c->d_mods;
  a.out_poly_stride = out_stride;
  a.in_poly_stride = in_stride;
  a.logN = c->logN;
  a.g = g;
  a.g_inv = inv_mod_pow2(g, c->logN + 1);
  a.eval_domain = eval_domain ? 1 : 0;
  a.ids = ids;
  ProfScope ps(c, PK_AUTOMORPH, st);
  hipLaunchKernelGGL(automorph_kernel, dim3(c->N / 256, nslots, npoly), dim3(256), 0, st, a);
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct KsLayout {
  size_t dcoef, ext, acc, tq, total;
};
KsLayout ks_layout(const ckks_ctx* c, u32 B, u32 nlimbs) {
  const size_t N = c->N, next = nlimbs + c->np, beta = (nlimbs + c->alpha - 1) / c->alpha;
  KsLayout L;
  size_t off = 0;
  L.dcoef = off; off += align256((size_t)B * nlimbs * N * 8);
  L.ext = off;   off += align256((size_t)B * beta * next * N * 8);
  L.acc = off;   off += align256((size_t)B * 2 * next * N * 8);
  L.tq = off;    off += align256((size_t)B * 2 * nlimbs * N * 8);
  L.total = off;
  return L;
}

// Base-conversion launches: two adjacent coefficients per lane up to 24 sources, one beyond (register budget).
template <bool PRESCALED, bool NARROW>
void launch_modup_n(const ckks_ctx* c, const ModUpArgs& a, u32 beta, u32 B, hipStream_t st) {
  dim3 block(BCONV_THREADS), g2(c->N / BCONV_THREADS / 2, beta, B), g1(c->N / BCONV_THREADS, beta, B);
#define LAUNCH_MODUP(LEN, EPT, GRID) \
  hipLaunchKernelGGL((modup_kernel<LEN, PRESCALED, EPT, NARROW>), GRID, block, 0, st, a, a.dcoef, a.ext, a.mods, a.mat)
  if (c->alpha <= 4) LAUNCH_MODUP(4, 2, g2);
  else if (c->alpha <= 8) LAUNCH_MODUP(8, 2, g2);
  else if (c->alpha <= 15) LAUNCH_MODUP(15, 2, g2);
  else if (c->alpha <= 24) LAUNCH_MODUP(24, 2, g2);
  else if (c->alpha <= 36) LAUNCH_MODUP(36, 1, g1);
  else LAUNCH_MODUP(45, 1, g1);
#undef LAUNCH_MODUP
}
template <bool PRESCALED>
void launch_modup(const ckks_ctx* c, const ModUpArgs& a, u32 beta, u32 B, bool narrow, hipStream_t st) {
  if (narrow) launch_modup_n<PRESCALED, true>(c, a, beta, B, st);
  else launch_modup_n<PRESCALED, false>(c, a, beta, B, st);
}
template <bool PRESCALED, bool NARROW>
void launch_moddown_n(const ckks_ctx* c, const ModDownArgs& a, u32 B2, hipStream_t st) {
  dim3 block(BCONV_THREADS), g2(c->N / BCONV_THREADS / 2, B2), g1(c->N / BCONV_THREADS, B2);
  const u32 K = a.K;
#define LAUNCH_MODDOWN(LEN, EPT, GRID) \
  hipLaunchKernelGGL((moddown_kernel<LEN, PRESCALED, EPT, NARROW>), GRID, block, 0, st, a, a.acc, a.tq, a.mods, a.mat)
  if (K <= 4) LAUNCH_MODDOWN(4, 2, g2);
  else if (K <= 8) LAUNCH_MODDOWN(8, 2, g2);
  else if (K <= 15) LAUNCH_MODDOWN(15, 2, g2);
  else if (K <= 24) LAUNCH_MODDOWN(24, 2, g2);
  else if (K <= 36) LAUNCH_MODDOWN(36, 1, g1);
  else LAUNCH_MODDOWN(45, 1, g1);
#undef LAUNCH_MODDOWN
}
template <bool PRESCALED>
void launch_moddown(const ckks_ctx* c, const ModDownArgs& a, u32 B2, bool narrow, hipStream_t st) {
  if (narrow) launch_moddown_n<PRESCALED, true>(c, a, B2, st);
  else launch_moddown_n<PRESCALED, false>(c, a, B2, st);
}

// What a key switch reads and how its result is assembled.
struct KsIo {
  const u64* d;          // polynomial to switch, eval domain; limb-vector (b, i) at d + b*d_stride + i*N
  u64 d_stride;
  u32 d_galois;          // != 0: d is read through the eval-domain Galois map (HRot's sigma(c1)); N = 2^16 path only
  u64* out;              // [B][2][nlimbs][N]
  u32 mode[2];           // per component: bit 0: + add2 (out itself when null); bit 1: + sigma_g(add_src) (N = 2^16 path only)
  const u64* add_src;    // [B][2][nlimbs][N]
  u32 add_galois;
  // N = 2^16 path, B <= KS_MULTI_MAX: ciphertext b uses galois_pc[b] (for d and add_src) and the key evk_pc[b]
  const u32* galois_pc = nullptr;
  const u64* const* evk_pc = nullptr;
  const u64* add2 = nullptr;   // [B][2][nlimbs][N] plain addend of mode bit 0 (N = 2^16 path); null = out, in place
  bool add2_three = false;     // add2 is [B][3][nlimbs][N]; its first two components are the addends
};

// Base conversion fused with the first forward pass (ntt16_bconv_rows_kernel): one launch per modulus class among
// the `ntarget` target slots. class_of_slot(slot) < 0 leaves a slot out.
template <class ClassOf>
int launch_bconv_rows(const ckks_ctx* c, BconvRowsArgs a, u32 npoly, bool narrow, ClassOf class_of_slot, hipStream_t st) {
  if (npoly > 65535) return fail(CKKS_ESHAPE, "batch too large for one launch");
  a.tw = c->d_tw_fwd;
  a.twfp = c->d_twfp_fwd;
  a.mods = c->d_mods;
  // the targets of a polynomial on one XCD, whose L2 then serves the shared source tiles, tiles fastest
  a.map_mode = c->tune[0] >= 0 ? (u32)c->tune[0] : 5u;
  a.npoly = npoly;
  const u32 grid_poly = a.map_mode == 5 ? (npoly + 7) / 8 * 8 : npoly;
  for (int cls = 0; cls < 3; cls++) {
    u32 cnt = 0;
    for (u32 s = 0; s < a.ntarget; s++)
      if (class_of_slot(s) == cls) a.slots[cnt++] = (unsigned char)s;
    if (!cnt) continue;
    const dim3 grid(cnt, 16, grid_poly), block(NTT16_THREADS);
    ProfScope ps(c, PK_BCONV_ROWS + cls, st);
#define LAUNCH_BCONV(CLS)                                                                              \
  if (narrow) hipLaunchKernelGGL((ntt16_bconv_rows_kernel<CLS, true>), grid, block, 0, st, a);         \
  else hipLaunchKernelGGL((ntt16_bconv_rows_kernel<CLS, false>), grid, block, 0, st, a)
    if (cls == 0) { LAUNCH_BCONV(0); }
    else if (cls == 1) { LAUNCH_BCONV(1); }
    else { LAUNCH_BCONV(2); }
#undef LAUNCH_BCONV
  }
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}

// ModDown's conversion and the first forward pass of its result on the N = 2^16 path: the special limbs of both
// accumulators back to coefficient form (scaled by (P/p_k)^-1 / N), P -> Q_l, stages 0..7; tq receives the converted
// limbs in row-pass form. Knob 2 = 1 does the conversion inside the row pass (ntt16_bconv_rows_kernel).
int ks16_moddown_rows(ckks_ctx* c, const LevelTables* lt, u32 B, u32 nlimbs, u64* acc, u64* tq, hipStream_t st) {
  int rc;
  const u32 N = c->N, next = lt->next, K = c->np;
  const bool fused = c->tune[2] == 1;
  LimbMap pmap;
  for (u32 k = 0; k < CKKS_MAX_SLOTS; k++) pmap.id[k] = (unsigned char)(k < K ? c->nq + k : 0);
  NttOpts o3;
  o3.scale = lt->dn_scale;
  o3.split_out = fused;
  if ((rc = launch_ntt(c, true, acc, (u64)next * N, acc, (u64)next * N, B * 2, nlimbs, K, pmap, 0, 0, st, o3))) return rc;
  if (!fused) {
    {
      ModDownArgs a{acc, tq, c->d_mods, lt->dn_inv, lt->dn_mat_plain, c->logN, nlimbs, c->nq, K, next, nlimbs, c->nq};
      ProfScope ps(c, PK_MODDOWN, st);
      launch_moddown<true>(c, a, B * 2, lt->narrow_dn, st);
      HIP_TRY(hipGetLastError());
    }
    NttOpts o2;
    o2.rows_only = true;
    return launch_ntt(c, false, tq, (u64)nlimbs * N, tq, (u64)nlimbs * N, B * 2, 0, nlimbs, identity_map(nlimbs), 0, 0, st, o2);
  }
  BconvRowsArgs a;
  a.src = acc;
  a.dst = tq;
  a.mat = lt->dn_mat_plain;
  a.off = lt->dn_off;
  a.src_poly_stride = (u64)next * N;
  a.dst_poly_stride = (u64)nlimbs * N;
  a.src_slot0 = nlimbs;
  a.src_nlimbs = K;
  a.alpha = K;
  a.beta = 1;
  a.skip_own = 0;
  a.ntarget = nlimbs;
  a.pitch = lt->dn_pitch;
  for (u32 i = 0; i < 128; i++) a.id[i] = (unsigned char)(i < nlimbs ? i : 0);
  return launch_bconv_rows(c, a, B * 2, lt->narrow_dn, [&](u32 s) { return host_class(c, c->mod[s]); }, st);
}

// Last kernel of a key switch on the N = 2^16 path: block pass of tq fused with (acc - tq) / P and the addends.
// exclude_class >= 0 leaves the limbs of that modulus class to another kernel.
int ks16_assemble(ckks_ctx* c, const LevelTables* lt, const KsIo& io, u32 B, u32 nlimbs, const u64* acc, const u64* tq,
                  hipStream_t st, int exclude_class = -1) {
  FwdFinalArgs a;
  a.tq = tq;
  a.acc = acc;
  a.out = io.out;
  a.add_src = io.add_src;
  a.add2 = io.add2 ? io.add2 : io.out;
  a.add2_three = io.add2 && io.add2_three ? 1u : 0u;
  a.tw = c->d_tw_fwd;
  a.twfp = c->d_twfp_fwd;
  a.mods = c->d_mods;
  a.pinv = lt->pinv2;
  a.nlimbs = nlimbs;
  a.next = lt->next;
  a.mode0 = io.mode[0];
  a.mode1 = io.mode[1];
  a.galois = io.add_galois;
  if (io.galois_pc) {
    a.multi = 1;
    for (u32 i = 0; i < B; i++) a.galois_pc[i] = io.galois_pc[i];
  }
  a.map_mode = map_mode_pass(c);
  auto cls_of = [&](u32 s) {
    const int k = host_class(c, c->mod[s]);
    return k == exclude_class ? -1 : k;
  };
  LAUNCH_BY_CLASS(c, PK_FWD_FINAL, ntt16_fwd_blocks_final_kernel, a, B * 2, nlimbs, cls_of, st)
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}

// Second half of a key switch on the N = 2^16 path: from the accumulators (all slots) to the assembled output.
// acc_in: accumulators held outside the workspace ([B][2][next][N]; their special-prime slots are overwritten).
int ks16_finish(ckks_ctx* c, const LevelTables* lt, const KsIo& io, u32 B, u32 nlimbs, char* ws, hipStream_t st,
                u64* acc_in = nullptr) {
  int rc;
  KsLayout L = ks_layout(c, B, nlimbs);
  u64* acc = acc_in ? acc_in : (u64*)(ws + L.acc);
  u64* tq = (u64*)(ws + L.tq);
  if ((rc = ks16_moddown_rows(c, lt, B, nlimbs, acc, tq, st))) return rc;
  return ks16_assemble(c, lt, io, B, nlimbs, acc, tq, st);
}

// N = 2^16: transforms fused with their neighbours.
//   1. INTT(d) with (Q_j/q_i)^-1 / N folded in, written in the split form
//   2. ModUp conversion and row pass of every slot a digit does not own (two kernels; knob 2 = 1: one fused kernel)
//   3. integer-class slots (the special primes): [block pass + evk inner product] (x 2^-64 from the Montgomery products)
//   4. INTT of the special limbs with 2^64 (P/p_k)^-1 / N folded in; ModDown conversion and row pass (as step 2)
//   5. double-precision main limbs: [block pass of the digits + evk inner product + block pass of the ModDown
//      correction + (sum - correction) / P + addends] in one kernel, so their accumulators never reach memory;
//      integer-class main limbs take the assembly kernel on the accumulators of step 3.
// With knob 3 = 1 the double-precision slots take a plain block pass, a streaming product and the assembly kernel
// instead of step 5's fusion. With knob 4 = 0 the double-precision part of step 2 runs on the context's second stream
// beside steps 3 and 4, which do not depend on it, and is joined before step 5.
// acc_add != null (knob 3 at its default only): the sequence stops before ModDown and ADDS the two accumulators, plus
// P * sigma(io.add_src component 0) on the main primes of the first, to acc_add ([B][2][next][N]).
int keyswitch_fused16(ckks_ctx* c, const LevelTables* lt, const KsIo& io, u32 B, u32 nlimbs, const u64* evk, char* ws,
                      hipStream_t st, u64* acc_add = nullptr) {
  int rc;
  const u32 N = c->N, next = lt->next, beta = lt->beta;
  KsLayout L = ks_layout(c, B, nlimbs);
  u64* dcoef = (u64*)(ws + L.dcoef);
  u64* ext = (u64*)(ws + L.ext);
  u64* acc = (u64*)(ws + L.acc);
  u64* tq = (u64*)(ws + L.tq);
  const LimbMap qmap = identity_map(nlimbs), emap = ext_map(c, nlimbs);
  if (io.galois_pc && B > KS_MULTI_MAX) return fail(CKKS_ESHAPE, "internal: per-ciphertext keys for too many ciphertexts");
  const bool fused_fp = c->tune[3] != 1;
  if (acc_add && !fused_fp) return fail(CKKS_EINVAL, "internal: accumulation needs the default inner kernels");
  auto ext_class = [&](u32 s) { return host_class(c, c->mod[emap.id[s]]); };
  bool any_fp = false, any_int = false, special_fp = false;
  for (u32 s_ = 0; s_ < next; s_++) {
    const bool fp = ext_class(s_) == 0;
    any_fp |= fp;
    any_int |= !fp;
    if (s_ >= nlimbs) special_fp |= fp;
  }
  const bool fused_up = c->tune[2] == 1;
  // 1.
  NttOpts o1;
  o1.galois = io.d_galois;
  o1.galois_pc = io.galois_pc;
  o1.scale = lt->up_scale;
  o1.split_out = fused_up;
  if ((rc = launch_ntt(c, true, io.d, io.d_stride, dcoef, (u64)nlimbs * N, B, 0, nlimbs, qmap, 0, 0, st, o1))) return rc;
  // 2. The double-precision part of the row pass (memory-bound) may run on the second stream beside the
  // integer-class chain of steps 2-4 (arithmetic-bound), which does not depend on it.
  const bool fork = any_fp && any_int && !special_fp && !acc_add && c->tune[4] == 0;
  hipStream_t sb = st;
  if (!fused_up) {
    ModUpArgs a{dcoef, ext, c->d_mods, lt->up_inv, lt->up_mat, c->logN, nlimbs, c->nq, c->alpha, beta, next};
    ProfScope ps(c, PK_MODUP, st);
    launch_modup<true>(c, a, beta, B, lt->narrow_up, st);
    HIP_TRY(hipGetLastError());
  }
  if (fork) {
    sb = c->side;
    HIP_TRY(hipEventRecord(c->ev_fork, st));
    HIP_TRY(hipStreamWaitEvent(sb, c->ev_fork, 0));
  }
  if (!fused_up) {
    NttOpts o2;
    o2.rows_only = true;
    if (any_fp) {
      NttOpts o = o2;
      o.only_class = 0;
      if ((rc = launch_ntt(c, false, ext, (u64)next * N, ext, (u64)next * N, B * beta, 0, next, emap, beta, nlimbs, sb, o)))
        return rc;
    }
    if (any_int) {
      NttOpts o = o2;
      o.exclude_class = 0;
      if ((rc = launch_ntt(c, false, ext, (u64)next * N, ext, (u64)next * N, B * beta, 0, next, emap, beta, nlimbs, st, o)))
        return rc;
    }
  } else {
    BconvRowsArgs up;
    up.src = dcoef;
    up.dst = ext;
    up.mat = lt->up_mat;
    up.off = lt->up_off;
    up.src_poly_stride = (u64)nlimbs * N;
    up.dst_poly_stride = (u64)next * N;
    up.src_slot0 = 0;
    up.src_nlimbs = nlimbs;
    up.alpha = c->alpha;
    up.beta = beta;
    up.skip_own = 1;
    up.ntarget = next;
    up.pitch = lt->up_pitch;
    for (u32 i = 0; i < 128; i++) up.id[i] = emap.id[i];
    if (any_fp &&
        (rc = launch_bconv_rows(c, up, B * beta, lt->narrow_up, [&](u32 s) { return ext_class(s) == 0 ? 0 : -1; }, sb)))
      return rc;
    if (any_int &&
        (rc = launch_bconv_rows(c, up, B * beta, lt->narrow_up, [&](u32 s) { return ext_class(s) == 0 ? -1 : ext_class(s); }, st)))
      return rc;
  }
  if (fork) HIP_TRY(hipEventRecord(c->ev_join, sb));
  FwdInnerArgs ia;
  ia.ext = ext;
  ia.d = io.d;
  ia.d_poly_stride = io.d_stride;
  ia.evk = evk;
  ia.acc = acc;
  ia.tw = c->d_tw_fwd;
  ia.twfp = c->d_twfp_fwd;
  ia.mods = c->d_mods;
  ia.nlimbs = nlimbs;
  ia.nq = c->nq;
  ia.nm = c->nm;
  ia.alpha = c->alpha;
  ia.beta = beta;
  ia.next = next;
  ia.map_mode = map_mode_inner(c, io.galois_pc == nullptr);
  ia.galois = io.d_galois;
  ia.ext_galois = 0;
  if (io.galois_pc) {
    ia.multi = 1;
    for (u32 i = 0; i < B; i++) ia.galois_pc[i] = io.galois_pc[i], ia.evk_pc[i] = io.evk_pc[i];
  }
  if (acc_add) {
    ia.acc = acc_add;
    ia.accumulate = 1;
    ia.c0 = io.add_src;
    ia.c0_poly_stride = 2 * (u64)nlimbs * N;
  }
  // 3. integer-class slots, 8 values per lane (grid.y = 32 tiles of 8 blocks)
  for (int cls = 1; cls <= 2; cls++) {
    FwdInnerArgs a = ia;
    u32 cnt = 0;
    for (u32 s_ = 0; s_ < next; s_++)
      if (ext_class(s_) == cls) a.slots[cnt++] = (unsigned char)s_;
    if (!cnt) continue;
    ProfScope ps(c, PK_INNER8 + cls - 1, st);
    if (cls == 1) hipLaunchKernelGGL(ntt16_fwd_blocks_inner8_kernel<1>, dim3(B, 32, cnt), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(ntt16_fwd_blocks_inner8_kernel<2>, dim3(B, 32, cnt), dim3(256), 0, st, a);
  }
  HIP_TRY(hipGetLastError());
  // double-precision slots whose accumulators are needed in memory: the special ones always (ModDown reads them),
  // the main ones when the result is accumulated or when the fusion of step 5 is switched off
  auto launch_inner_fp = [&](bool special, bool main_slots, hipStream_t s) -> int {
    FwdInnerArgs a = ia;
    u32 cnt = 0;
    for (u32 s_ = 0; s_ < next; s_++)
      if (ext_class(s_) == 0 && (s_ >= nlimbs ? special : main_slots)) a.slots[cnt++] = (unsigned char)s_;
    if (!cnt) return CKKS_OK;
    if (fused_fp) {
      ProfScope ps(c, PK_INNER_C, s);
      hipLaunchKernelGGL(ntt16_fwd_blocks_inner_c_kernel, dim3(B * 2, 16, cnt), dim3(NTT16_THREADS), 0, s, a);
    } else {
      // plain block pass of every converted double-precision slot (own limbs are skipped), then a streaming product
      NttOpts o;
      o.blocks_only = true;
      o.raw_out = true;
      o.only_class = 0;
      int r2 = launch_ntt(c, false, ext, (u64)next * N, ext, (u64)next * N, B * beta, 0, next, emap, beta, nlimbs, s, o);
      if (r2) return r2;
      ProfScope ps(c, PK_INNER16, s);
      hipLaunchKernelGGL(inner16_fp_kernel, dim3(B, 128, cnt), dim3(256), 0, s, a);
    }
    HIP_TRY(hipGetLastError());
    return CKKS_OK;
  };
  if (special_fp || acc_add || !fused_fp) {
    if ((rc = launch_inner_fp(true, acc_add || !fused_fp, st))) return rc;
  }
  if (acc_add) return CKKS_OK;
  // 4.
  if ((rc = ks16_moddown_rows(c, lt, B, nlimbs, acc, tq, st))) return rc;
  if (fork) HIP_TRY(hipStreamWaitEvent(st, c->ev_join, 0));
  // 5.
  if (fused_fp && any_fp) {
    FwdInnerArgs a = ia;
    u32 cnt = 0;
    for (u32 s_ = 0; s_ < nlimbs; s_++)
      if (ext_class(s_) == 0) a.slots[cnt++] = (unsigned char)s_;
    if (cnt) {
      a.fin_tq = tq;
      a.fin_out = io.out;
      a.fin_add_src = io.add_src;
      a.fin_add2 = io.add2 ? io.add2 : io.out;
      a.fin_add2_three = io.add2 && io.add2_three ? 1u : 0u;
      a.fin_pinv = lt->pinv2;
      a.fin_mode0 = io.mode[0];
      a.fin_mode1 = io.mode[1];
      a.fin_galois = io.add_galois;
      ProfScope ps(c, PK_INNER_C, st);
      hipLaunchKernelGGL(ntt16_fwd_blocks_inner_c_kernel, dim3(B * 2, 16, cnt), dim3(NTT16_THREADS), 0, st, a);
      HIP_TRY(hipGetLastError());
    }
  }
  return ks16_assemble(c, lt, io, B, nlimbs, acc, tq, st, fused_fp ? 0 : -1);
}

// Shared front of the hoisted rotations at N = 2^16: inverse transform, ModUp and forward transform of c1 of ct_in
// ([B][2][nlimbs][N]) into the workspace, and the arguments of the streaming inner-product kernels that read them
// (accumulators default to the workspace's own).
static int hoist_front16(ckks_ctx* c, const LevelTables* lt, const u64* ct_in, u32 B, u32 nlimbs, char* ws, hipStream_t st,
                         FwdInnerArgs& ia) {
  int rc;
  const u32 N = c->N, next = lt->next, beta = lt->beta;
  const u64 polyN = (u64)nlimbs * N;
  KsLayout L = ks_layout(c, B, nlimbs);
  u64* dcoef = (u64*)(ws + L.dcoef);
  u64* ext = (u64*)(ws + L.ext);
  u64* acc = (u64*)(ws + L.acc);
  const LimbMap qmap = identity_map(nlimbs), emap = ext_map(c, nlimbs);
  const u64* c1 = ct_in + polyN;
  NttOpts o1;
  o1.scale = lt->up_scale;
  if ((rc = launch_ntt(c, true, c1, 2 * polyN, dcoef, polyN, B, 0, nlimbs, qmap, 0, 0, st, o1))) return rc;
  {
    ModUpArgs a{dcoef, ext, c->d_mods, lt->up_inv, lt->up_mat, c->logN, nlimbs, c->nq, c->alpha, beta, next};
    ProfScope ps(c, PK_MODUP, st);
    launch_modup<true>(c, a, beta, B, lt->narrow_up, st);
    HIP_TRY(hipGetLastError());
  }
  NttOpts of;
  of.raw_out = true;  // reduced doubles on double-precision moduli, canonical residues elsewhere
  if ((rc = launch_ntt(c, false, ext, (u64)next * N, ext, (u64)next * N, B * beta, 0, next, emap, beta, nlimbs, st, of)))
    return rc;
  ia.ext = ext;
  ia.d = c1;
  ia.d_poly_stride = 2 * polyN;
  ia.acc = acc;
  ia.tw = c->d_tw_fwd;
  ia.twfp = c->d_twfp_fwd;
  ia.mods = c->d_mods;
  ia.nlimbs = nlimbs;
  ia.nq = c->nq;
  ia.nm = c->nm;
  ia.alpha = c->alpha;
  ia.beta = beta;
  ia.next = next;
  ia.map_mode = map_mode_inner(c, true);
  return CKKS_OK;
}

// Hoisted rotations, N = 2^16: out[r] = HRot_{g_r}(ct_in) for r < R. The Galois map commutes exactly with the
// centred base conversion (it permutes coefficients up to sign, and the conversion is odd), so INTT, ModUp and the
// forward transform of c1 are done once on the un-rotated polynomial; each rotation then reads the transformed
// digits through its own index map in the streaming inner product and finishes as usual.
// acc_base != null: rotation r stops before ModDown and leaves its accumulators, with P * sigma(c0) added to the
// first one, at acc_base + r * acc_stride (rotations kept in the extended basis), or adds them to what is there
// (acc_add); out_base is not used then. scratch != null (ordinary rotations): room for the accumulators
// ([B][2][next][N] each) of scratch_rots rotations, which are then computed that many at a time in one pass over the
// digits before each is finished.
int hrot_hoisted16(ckks_ctx* c, u64* out_base, u64 out_stride, const u64* ct_in, u32 B, u32 nlimbs, const u32* galois,
                   const u64* const* evks, u32 R, char* ws, hipStream_t st, u64* acc_base = nullptr, u64 acc_stride = 0,
                   bool acc_add = false, u64* scratch = nullptr, u32 scratch_rots = 0) {
  const LevelTables* lt;
  int rc = get_level(c, nlimbs, &lt);
  if (rc) return rc;
  const u32 N = c->N, next = lt->next, beta = lt->beta;
  const u64 polyN = (u64)nlimbs * N;
  const LimbMap emap = ext_map(c, nlimbs);
  const u64* c1 = ct_in + polyN;
  FwdInnerArgs ia;
  if ((rc = hoist_front16(c, lt, ct_in, B, nlimbs, ws, st, ia))) return rc;
  if (acc_base) {
    ia.c0 = ct_in;
    ia.c0_poly_stride = 2 * polyN;
    ia.accumulate = acc_add ? 1u : 0u;
  }
  // several rotations per pass over the digits (at most KS_MULTI_MAX): accumulators of rotations r0 .. r0+nr-1 to
  // dst + k * stride
  auto launch_rot = [&](u32 r0, u32 nr, u64* dst, u64 stride) -> int {
      ia.acc = dst;
      ia.acc_rot_stride = stride;
      ia.nrot = nr;
      for (u32 r = 0; r < nr; r++) {
        ia.galois_pc[r] = inv_mod_pow2(galois[r0 + r], c->logN + 1);
        ia.evk_pc[r] = evks[r0 + r];
      }
      for (int fp = 1; fp >= 0; fp--) {
        FwdInnerArgs a = ia;
        u32 cnt = 0;
        for (u32 s_ = 0; s_ < next; s_++)
          if ((host_class(c, c->mod[emap.id[s_]]) == 0) == (fp == 1)) a.slots[cnt++] = (unsigned char)s_;
        if (!cnt) continue;
        ProfScope ps(c, fp ? PK_INNER16 : PK_INNER16_INT, st);
        const u32 cb = fp ? INNER16_ROT_CB_FP : INNER16_ROT_CB;
        const dim3 grid((B + cb - 1) / cb, 256, cnt);
        if (fp && beta == 1) hipLaunchKernelGGL((inner16_rot_fp_kernel<1, true>), grid, dim3(256), 0, st, a, B);
        else if (fp && beta == 2) hipLaunchKernelGGL((inner16_rot_fp_kernel<2, true>), grid, dim3(256), 0, st, a, B);
        else if (fp && beta == 3) hipLaunchKernelGGL((inner16_rot_fp_kernel<3, true>), grid, dim3(256), 0, st, a, B);
        else if (fp && beta == 4) hipLaunchKernelGGL((inner16_rot_fp_kernel<4, true>), grid, dim3(256), 0, st, a, B);
        else if (fp) hipLaunchKernelGGL((inner16_rot_fp_kernel<INNER16_ROT_MAX_BETA, false>), grid, dim3(256), 0, st, a, B);
        else if (beta <= 4) hipLaunchKernelGGL(inner16_rot_int_kernel<4>, grid, dim3(256), 0, st, a, B);
        else hipLaunchKernelGGL(inner16_rot_int_kernel<INNER16_ROT_MAX_BETA>, grid, dim3(256), 0, st, a, B);
      }
      HIP_TRY(hipGetLastError());
      return CKKS_OK;
  };
  if (acc_base && !acc_add && beta <= INNER16_ROT_MAX_BETA) {
    for (u32 r0 = 0; r0 < R; r0 += KS_MULTI_MAX) {
      const u32 nr = std::min<u32>(KS_MULTI_MAX, R - r0);
      if ((rc = launch_rot(r0, nr, acc_base + (size_t)r0 * acc_stride, acc_stride))) return rc;
    }
    return CKKS_OK;
  }
  if (!acc_base && scratch && scratch_rots >= 2 && R >= 2 && beta <= INNER16_ROT_MAX_BETA) {
    const u64 one = (u64)B * 2 * next * N;
    const u32 per_pass = std::min<u32>(scratch_rots, KS_MULTI_MAX);
    for (u32 r0 = 0; r0 < R; r0 += per_pass) {
      const u32 nr = std::min<u32>(per_pass, R - r0);
      if ((rc = launch_rot(r0, nr, scratch, one))) return rc;
      for (u32 k = 0; k < nr; k++) {
        const u32 r = r0 + k;
        KsIo io{c1, 2 * polyN, galois[r], out_base + (size_t)r * out_stride, {2, 0}, ct_in, galois[r]};
        if ((rc = ks16_finish(c, lt, io, B, nlimbs, ws, st, scratch + (size_t)k * one))) return rc;
      }
    }
    return CKKS_OK;
  }
  for (u32 r = 0; r < R; r++) {
    ia.evk = evks[r];
    ia.galois = galois[r];
    ia.ext_galois = galois[r];
    if (acc_base) ia.acc = acc_base + (size_t)r * acc_stride;
    for (int fp = 1; fp >= 0; fp--) {
      FwdInnerArgs a = ia;
      u32 cnt = 0;
      for (u32 s_ = 0; s_ < next; s_++)
        if ((host_class(c, c->mod[emap.id[s_]]) == 0) == (fp == 1)) a.slots[cnt++] = (unsigned char)s_;
      if (!cnt) continue;
      ProfScope ps(c, fp ? PK_INNER16 : PK_INNER16_INT, st);
      if (fp) hipLaunchKernelGGL(inner16_fp_kernel, dim3(B, 128, cnt), dim3(256), 0, st, a);
      else hipLaunchKernelGGL(inner16_int_kernel, dim3(B, 128, cnt), dim3(256), 0, st, a);
    }
    HIP_TRY(hipGetLastError());
    if (acc_base) continue;
    KsIo io{c1, 2 * polyN, galois[r], out_base + (size_t)r * out_stride, {2, 0}, ct_in, galois[r]};
    if ((rc = ks16_finish(c, lt, io, B, nlimbs, ws, st))) return rc;
  }
  return CKKS_OK;
}

// Key switch of io.d with evk into io.out (see KsIo). Other ring degrees: one kernel per step.
int keyswitch_impl(ckks_ctx* c, const KsIo& io, u32 B, u32 nlimbs, const u64* evk, char* ws, hipStream_t st) {
  const LevelTables* lt;
  int rc = get_level(c, nlimbs, &lt);
  if (rc) return rc;
  if (c->logN == 16) return keyswitch_fused16(c, lt, io, B, nlimbs, evk, ws, st);
  if (io.d_galois || io.mode[0] >= 2 || io.mode[1] >= 2 || io.add2)
    return fail(CKKS_EINVAL, "internal: gather modes and separate addends need the N = 2^16 path");
  const u64* d = io.d;
  u64* out = io.out;
  const u32 add_mask = (io.mode[0] ? 1u : 0u) | (io.mode[1] ? 2u : 0u);
  const u32 N = c->N, next = lt->next, beta = lt->beta, K = c->np;
  KsLayout L = ks_layout(c, B, nlimbs);
  u64* dcoef = (u64*)(ws + L.dcoef);
  u64* ext = (u64*)(ws + L.ext);
  u64* acc = (u64*)(ws + L.acc);
  u64* tq = (u64*)(ws + L.tq);
  const LimbMap qmap = identity_map(nlimbs), emap = ext_map(c, nlimbs);

  // 1. coefficient form of d
  if ((rc = launch_ntt(c, true, d, io.d_stride, dcoef, (u64)nlimbs * N, B, 0, nlimbs, qmap, 0, 0, st))) return rc;
  // 2. ModUp every digit to the slots it does not own
  {
    ModUpArgs a{dcoef, ext, c->d_mods, lt->up_inv, lt->up_mat, c->logN, nlimbs, c->nq, c->alpha, beta, next};
    ProfScope ps(c, PK_MODUP, st);
    launch_modup<false>(c, a, beta, B, lt->narrow_up, st);
    HIP_TRY(hipGetLastError());
  }
  // 3. forward transform of the converted slots
  if ((rc = launch_ntt(c, false, ext, (u64)next * N, ext, (u64)next * N, B * beta, 0, next, emap, beta, nlimbs, st))) return rc;
  // 4. inner product with the key
  {
    InnerArgs a{d, ext, evk, acc, c->d_mods, c->logN, nlimbs, c->nq, c->nm, c->alpha, beta, next, io.d_stride};
    ProfScope ps(c, PK_INNER, st);
    hipLaunchKernelGGL(inner_kernel, dim3(B, N / 256, next), dim3(256), 0, st, a);
    HIP_TRY(hipGetLastError());
  }
  // 5. special limbs of both accumulators back to coefficient form
  {
    LimbMap pmap;
    for (u32 k = 0; k < CKKS_MAX_SLOTS; k++) pmap.id[k] = (unsigned char)(k < K ? c->nq + k : 0);
    if ((rc = launch_ntt(c, true, acc, (u64)next * N, acc, (u64)next * N, B * 2, nlimbs, K, pmap, 0, 0, st))) return rc;
  }
  // 6. ModDown base conversion P -> Q_l
  {
    ModDownArgs a{acc, tq, c->d_mods, lt->dn_inv, lt->dn_mat, c->logN, nlimbs, c->nq, K, next, nlimbs, c->nq};
    ProfScope ps(c, PK_MODDOWN, st);
    launch_moddown<false>(c, a, B * 2, lt->narrow_dn, st);
    HIP_TRY(hipGetLastError());
  }
  // 7. its forward transform, 8. subtract, scale by P^-1, assemble
  if ((rc = launch_ntt(c, false, tq, (u64)nlimbs * N, tq, (u64)nlimbs * N, B * 2, 0, nlimbs, qmap, 0, 0, st))) return rc;
  {
    FinalArgs a{acc, tq, out, c->d_mods, lt->pinv, c->logN, nlimbs, next, add_mask};
    ProfScope ps(c, PK_FINAL, st);
    hipLaunchKernelGGL(ks_final_kernel, dim3(N / 256, nlimbs, B * 2), dim3(256), 0, st, a);
    HIP_TRY(hipGetLastError());
  }
  return CKKS_OK;
}

int check_common(const ckks_ctx* c, u32 B, u32 nlimbs) {
  if (!c) return fail(CKKS_EINVAL, "null context");
  if (nlimbs == 0 || nlimbs > c->nq) return fail(CKKS_ESHAPE, "nlimbs must be in [1, L+1]");
  if (B == 0 || B > 32767) return fail(CKKS_ESHAPE, "batch must be in [1, 32767]");
  if (c->np == 0) return fail(CKKS_ESHAPE, "key switching needs at least one special prime");
  return CKKS_OK;
}
int check_ws(const ckks_ctx* c, int op, u32 B, u32 nlimbs, u32 n1, const void* ws, size_t ws_bytes) {
  if (!ws || ((uintptr_t)ws & 255)) return fail(CKKS_EWORKSPACE, "workspace is null or not 256-byte aligned");
  size_t need = ckks_workspace_bytes(c, op, B, nlimbs, n1);
  if (ws_bytes < need)
    return fail(CKKS_EWORKSPACE, "workspace too small: need " + std::to_string(need) + " bytes, got " + std::to_string(ws_bytes));
  return CKKS_OK;
}
bool overlap(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

int check_ids(const ckks_ctx* c, const uint32_t* ids, u32 n, LimbMap* out) {
  if (!ids) return fail(CKKS_EINVAL, "null limb_ids");
  if (n == 0 || n > CKKS_MAX_SLOTS) return fail(CKKS_ESHAPE, "nlimbs must be in [1, 128]");
  for (u32 i = 0; i < CKKS_MAX_SLOTS; i++) out->id[i] = 0;
  for (u32 i = 0; i < n; i++) {
    if (ids[i] >= c->nm) return fail(CKKS_EINVAL, "limb id out of range");
    out->id[i] = (unsigned char)ids[i];
  }
  return CKKS_OK;
}

}  // namespace

extern "C" {

const char* ckks_last_error(void) { return g_err.c_str(); }

int ckks_ctx_create(ckks_ctx** out, uint32_t logN, const uint64_t* q, uint32_t nq, const uint64_t* p, uint32_t np,
                    uint32_t dnum, const uint64_t* psi, int device) {
  if (!out || !q || !psi || (np && !p)) return fail(CKKS_EINVAL, "null argument");
  if (logN < 10 || logN > 17) return fail(CKKS_ESHAPE, "logN must be in [10, 17]");
  if (nq == 0 || dnum == 0 || dnum > nq || nq + np > CKKS_MAX_SLOTS || nq > 45 || np > 45)
    return fail(CKKS_ESHAPE, "bad prime or digit count (at most 45 main and 45 special primes)");
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (device < 0 || device >= ndev) return fail(CKKS_EINVAL, "no such device");
  ckks_ctx* c = new ckks_ctx;
  c->device = device;
  c->logN = logN;
  c->N = 1u << logN;
  c->nq = nq;
  c->np = np;
  c->nm = nq + np;
  c->dnum = dnum;
  c->alpha = (nq + dnum - 1) / dnum;
  for (u32 i = 0; i < nq; i++) c->mod.push_back(q[i]);
  for (u32 i = 0; i < np; i++) c->mod.push_back(p[i]);
  c->psi.assign(psi, psi + c->nm);
  const u64 N = c->N;
  for (u32 i = 0; i < c->nm; i++) {
    u64 m = c->mod[i];
    bool ok = m < (1ull << 60) && m > 2 * N && (m - 1) % (2 * N) == 0 && h_is_prime(m) && c->psi[i] < m &&
              h_pow(c->psi[i], N, m) == m - 1;
    for (u32 k = 0; k < i && ok; k++) ok = c->mod[k] != m;
    if (!ok) {
      delete c;
      return fail(CKKS_EINVAL, "modulus " + std::to_string(i) +
                                   " must be a distinct prime < 2^60, = 1 mod 2N, with psi^N = -1");
    }
  }
  // pass plan
  if (logN <= 12) {
    c->passes.push_back(Pass{0, logN, 0, logN});
  } else {
    u32 k1 = logN - 8;
    c->passes.push_back(Pass{0, k1, 12 - k1, 12});
    c->passes.push_back(Pass{k1, 8, 0, 12});
  }
  // tables
  std::vector<ModInfo> mods(c->nm);
  std::vector<ulonglong2> fwd((size_t)c->nm * N), inv((size_t)c->nm * N);
  std::vector<double> fwdfp, invfp;
  if (logN == 16 || logN == 12) {
    fwdfp.assign((size_t)c->nm * N, 0.0);
    invfp.assign((size_t)c->nm * N, 0.0);
  }
  std::vector<u64> pw(N);
  for (u32 i = 0; i < c->nm; i++) {
    u64 m = c->mod[i];
    ModInfo& mi = mods[i];
    mi.m = m;
    mi.mu64 = (u64)((((u128)1) << 64) / m);
    mi.c64 = (u64)((((u128)1) << 64) % m);
    mi.c64s = h_shoup(mi.c64, m);
    mi.ninv = h_inv(N % m, m);
    mi.ninvs = h_shoup(mi.ninv, m);
    {
      u64 x = 1;  // Newton iteration for m^-1 mod 2^64 (m odd)
      for (int it = 0; it < 6; it++) x *= 2 - m * x;
      mi.minv = (u64)0 - x;
      mi.pmod = 0;
      if (i < c->nq) {
        mi.pmod = 1;
        for (u32 k = 0; k < c->np; k++) mi.pmod = h_mul(mi.pmod, c->mod[c->nq + k] % m, m);
      }
    }
    mi.qd = (double)m;
    mi.qinv = 1.0 / (double)m;
    mi.ninvd = (double)mi.ninv;
    mi.ninvq = (double)mi.ninv / (double)m;
    pw[0] = 1;
    for (u64 k = 1; k < N; k++) pw[k] = h_mul(pw[k - 1], c->psi[i], m);
    for (u32 k = 0; k < N; k++) {
      u64 w = pw[h_brev(k, logN)];
      fwd[(size_t)i * N + k] = ulonglong2{w, h_shoup(w, m)};
      // psi^-e = -psi^(N-e)
      u32 e = h_brev(k, logN);
      u64 wi = e == 0 ? 1 : m - pw[N - e];
      inv[(size_t)i * N + k] = ulonglong2{wi, h_shoup(wi, m)};
      if ((logN == 16 || logN == 12) && (m >> 50) == 0) {
        fwdfp[(size_t)i * N + k] = (double)w;
        invfp[(size_t)i * N + k] = (double)wi;
      }
    }
  }
  DeviceGuard guard(device);
  int rc = guard.ok ? CKKS_OK : fail(CKKS_EHIP, "cannot select device");
  if (!rc) rc = upload(&c->d_mods, mods);
  if (!rc) rc = upload(&c->d_tw_fwd, fwd);
  if (!rc) rc = upload(&c->d_tw_inv, inv);
  if (!rc) rc = upload(&c->d_twfp_fwd, fwdfp);
  if (!rc) rc = upload(&c->d_twfp_inv, invfp);
  if (!rc) rc = build_levels(c);
  if (!rc) {
    // device current = the context's: every GPU holds its own copy of the array at its own address
    hipError_t e = hipGetSymbolAddress(&c->scratch_ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !c->scratch_ptr)
      rc = fail(CKKS_EHIP, std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e));
  }
  // the second stream and the events of the fork/join inside a key switch (knob 4) exist from the start, so that
  // no call that enqueues work has to create them
  if (!rc && hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess) rc = fail(CKKS_EHIP, "hipStreamCreate");
  if (!rc && hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess) rc = fail(CKKS_EHIP, "hipEventCreate");
  if (!rc && hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) rc = fail(CKKS_EHIP, "hipEventCreate");
  if (rc) {
    ckks_ctx_destroy(c);
    return rc;
  }
  *out = c;
  return CKKS_OK;
}

int ckks_ctx_destroy(ckks_ctx* c) {
  if (!c) return CKKS_OK;
  DeviceGuard guard(c->device);
  (void)hipFree(c->d_mods);
  (void)hipFree(c->d_tw_fwd);
  (void)hipFree(c->d_tw_inv);
  (void)hipFree(c->d_twfp_fwd);
  (void)hipFree(c->d_twfp_inv);
  if (c->side) (void)hipStreamSynchronize(c->side), (void)hipStreamDestroy(c->side);
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  for (auto& r : c->prof_recs) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  for (auto& e : c->prof_pool) (void)hipEventDestroy(e);
  (void)hipFree(c->d_levels);
  delete c;
  return CKKS_OK;
}

int ckks_tune_set(ckks_ctx* c, int knob, int value) {
  if (!c || knob < 0 || knob >= 8) return fail(CKKS_EINVAL, "bad knob");
  const int old = c->tune[knob];
  c->tune[knob] = value;
  // knobs 1 and 5 select the arithmetic the level tables are scaled for: rebuild them (waits for the device)
  if ((knob == 1 || knob == 5) && (old != 0) != (value != 0)) return build_levels(c);
  return CKKS_OK;
}
int ckks_prof_enable(ckks_ctx* c, int on) {
  if (!c) return fail(CKKS_EINVAL, "null context");
  c->prof_on = on != 0;
  return CKKS_OK;
}
int ckks_prof_copy(ckks_ctx* c, void* dst, const void* src, size_t bytes, void* stream) {
  if (!c || !dst || !src) return fail(CKKS_EINVAL, "null argument");
  if (bytes == 0 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15) || bytes / 16 / 256 >= (1ull << 31))
    return fail(CKKS_ESHAPE, "ckks_prof_copy: size and addresses must be multiples of 16 bytes");
  if (overlap(dst, bytes, src, bytes)) return fail(CKKS_EINVAL, "dst overlaps src");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  const size_t n = bytes / 16;
  ProfScope ps(c, PK_COPY, (hipStream_t)stream);
  hipLaunchKernelGGL(ckks_prof_copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     (const ulonglong2*)src, (ulonglong2*)dst, n);
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}
int ckks_prof_num_kinds(void) { return PK_COUNT; }
const char* ckks_prof_kind_name(int kind) { return kind >= 0 && kind < PK_COUNT ? kProfNames[kind] : ""; }
int ckks_prof_collect(ckks_ctx* c) {
  if (!c) return fail(CKKS_EINVAL, "null context");
  DeviceGuard guard(c->device);
  for (auto& r : c->prof_recs) {
    HIP_TRY(hipEventSynchronize(r.stop));
    float ms = 0;
    HIP_TRY(hipEventElapsedTime(&ms, r.start, r.stop));
    c->prof_ms[r.kind] += ms;
    c->prof_n[r.kind] += 1;
    c->prof_pool.push_back(r.start);
    c->prof_pool.push_back(r.stop);
  }
  c->prof_recs.clear();
  return CKKS_OK;
}
int ckks_prof_read(ckks_ctx* c, int kind, double* total_ms, uint64_t* launches) {
  if (!c || kind < 0 || kind >= PK_COUNT || !total_ms || !launches) return fail(CKKS_EINVAL, "bad argument");
  *total_ms = c->prof_ms[kind];
  *launches = c->prof_n[kind];
  return CKKS_OK;
}
int ckks_prof_reset(ckks_ctx* c) {
  if (!c) return fail(CKKS_EINVAL, "null context");
  int rc = ckks_prof_collect(c);
  for (int k = 0; k < PK_COUNT; k++) c->prof_ms[k] = 0, c->prof_n[k] = 0;
  return rc;
}

size_t ckks_workspace_bytes(const ckks_ctx* c, int op, uint32_t B, uint32_t nlimbs, uint32_t n1) {
  if (!c || B == 0 || nlimbs == 0 || nlimbs > c->nq) return 0;
  const size_t ks = ks_layout(c, B, nlimbs).total;
  const size_t poly = align256((size_t)B * nlimbs * c->N * 8);
  switch (op) {
    case CKKS_OP_KEYSWITCH: return ks;
    case CKKS_OP_HROT: return ks + poly;
    case CKKS_OP_HMULT_RELIN: return ks + poly;
    case CKKS_OP_RESCALE:
      // coefficient form of the dropped limb, its image on the remaining limbs
      return nlimbs < 2 ? 0 : align256((size_t)B * 2 * c->N * 8) + align256((size_t)B * 2 * (nlimbs - 1) * c->N * 8);
    case CKKS_OP_PCMM_BSGS:
      if (n1 == 0) return 0;
      // baby steps 1..n1-1, PMACC_TILE inner sums, rotated inner sum, HRot workspace
      return (size_t)(n1 - 1) * 2 * poly + (size_t)PMACC_TILE * 2 * poly + 2 * poly + ks + poly;
    case CKKS_OP_HROT_SUM:
      // hoisted digits and ModDown scratch, plus the running sum in the extended basis
      return ks + poly + 2 * align256((size_t)B * (nlimbs + c->np) * c->N * 8);
    case CKKS_OP_PCMM_BSGS_DH: {
      if (n1 == 0) return 0;
      // n1 baby steps, PMACC_TILE inner sums and the sum over giant steps in the extended basis, one inner sum
      // after ModDown, HRot workspace
      const size_t ext_poly = align256((size_t)B * (nlimbs + c->np) * c->N * 8);
      return (size_t)(n1 + PMACC_TILE + 1) * 2 * ext_poly + 2 * poly + ks + poly;
    }
    default: return 0;
  }
}

static int transform_entry(ckks_ctx* c, bool inverse, uint64_t* data, uint32_t npoly, const uint32_t* limb_ids,
                           uint32_t nlimbs, void* stream) {
  if (!c || !data) return fail(CKKS_EINVAL, "null argument");
  LimbMap ids;
  int rc = check_ids(c, limb_ids, nlimbs, &ids);
  if (rc) return rc;
  if (npoly == 0) return CKKS_OK;
  if (npoly > 65535 * 16) return fail(CKKS_ESHAPE, "too many polynomials in one call");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  // grid.x carries the polynomial index; split very large batches
  const u32 chunk = 32768;
  for (u32 p0 = 0; p0 < npoly; p0 += chunk) {
    u32 n = std::min(chunk, npoly - p0);
    u64* base = (u64*)data + (size_t)p0 * nlimbs * c->N;
    rc = launch_ntt(c, inverse, base, (u64)nlimbs * c->N, base, (u64)nlimbs * c->N, n, 0, nlimbs, ids, 0, 0,
                    (hipStream_t)stream);
    if (rc) return rc;
  }
  return CKKS_OK;
}

int ckks_ntt(ckks_ctx* c, uint64_t* data, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs, void* stream) {
  return transform_entry(c, false, data, npoly, limb_ids, nlimbs, stream);
}
int ckks_intt(ckks_ctx* c, uint64_t* data, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs, void* stream) {
  return transform_entry(c, true, data, npoly, limb_ids, nlimbs, stream);
}

int ckks_automorph(ckks_ctx* c, uint64_t* out, const uint64_t* in, uint32_t npoly, const uint32_t* limb_ids,
                   uint32_t nlimbs, uint32_t g, int eval_domain, void* stream) {
  if (!c || !out || !in) return fail(CKKS_EINVAL, "null argument");
  LimbMap ids;
  int rc = check_ids(c, limb_ids, nlimbs, &ids);
  if (rc) return rc;
  if (!(g & 1) || g >= 2 * c->N) return fail(CKKS_EINVAL, "galois_elt must be odd and < 2N");
  if (npoly == 0) return CKKS_OK;
  if (npoly > 65535) return fail(CKKS_ESHAPE, "too many polynomials in one call");
  size_t bytes = (size_t)npoly * nlimbs * c->N * 8;
  if (overlap(out, bytes, in, bytes)) return fail(CKKS_EINVAL, "out overlaps in");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  return launch_automorph(c, (u64*)out, (u64)nlimbs * c->N, (const u64*)in, (u64)nlimbs * c->N, npoly, nlimbs, ids, g,
                          eval_domain != 0, (hipStream_t)stream);
}

int ckks_keyswitch(ckks_ctx* c, uint64_t* ks_out, const uint64_t* d, uint32_t B, uint32_t nlimbs, const uint64_t* evk,
                   uint32_t galois_elt, uint32_t dnum, void* ws, size_t ws_bytes, void* stream) {
  (void)galois_elt;
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ks_out || !d || !evk) return fail(CKKS_EINVAL, "null argument");
  if (dnum != c->dnum) return fail(CKKS_ESHAPE, "dnum does not match the context");
  if ((rc = check_ws(c, CKKS_OP_KEYSWITCH, B, nlimbs, 0, ws, ws_bytes))) return rc;
  size_t poly = (size_t)B * nlimbs * c->N * 8;
  if (overlap(ks_out, 2 * poly, d, poly)) return fail(CKKS_EINVAL, "ks_out overlaps d");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  KsIo io{(const u64*)d, (u64)nlimbs * c->N, 0, (u64*)ks_out, {0, 0}, nullptr, 0};
  return keyswitch_impl(c, io, B, nlimbs, (const u64*)evk, (char*)ws, (hipStream_t)stream);
}

static int hrot_impl(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs, uint32_t g,
                     const uint64_t* evk, void* ws, size_t ws_bytes, void* stream, const uint64_t* ct_add);
int ckks_hrot(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs, uint32_t g,
              const uint64_t* evk, void* ws, size_t ws_bytes, void* stream) {
  return hrot_impl(c, ct_out, ct_in, B, nlimbs, g, evk, ws, ws_bytes, stream, nullptr);
}
// ct_add != null: ct_out = ct_add + HRot(ct_in); ct_add == ct_out accumulates in place (N = 2^16 path only).
static int hrot_impl(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs, uint32_t g,
                     const uint64_t* evk, void* ws, size_t ws_bytes, void* stream, const uint64_t* ct_add) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ct_out || !ct_in || !evk) return fail(CKKS_EINVAL, "null argument");
  if (!(g & 1) || g >= 2 * c->N) return fail(CKKS_EINVAL, "galois_elt must be odd and < 2N");
  if ((rc = check_ws(c, CKKS_OP_HROT, B, nlimbs, 0, ws, ws_bytes))) return rc;
  const size_t polyN = (size_t)nlimbs * c->N, ct_bytes = (size_t)B * 2 * polyN * 8;
  if (overlap(ct_out, ct_bytes, ct_in, ct_bytes)) return fail(CKKS_EINVAL, "ct_out overlaps ct_in");
  if (ct_add && ct_add != ct_out && overlap(ct_out, ct_bytes, ct_add, ct_bytes))
    return fail(CKKS_EINVAL, "ct_add must be ct_out itself or not overlap it");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  if (c->logN == 16) {
    // the permutation is applied where the ciphertext is read: by the first inverse pass and the fused inner product
    // (sigma(c1)) and by the final assembly (sigma(c0)), which also adds ct_add
    KsIo io{(const u64*)ct_in + polyN, 2 * polyN, g, (u64*)ct_out, {ct_add ? 3u : 2u, ct_add ? 1u : 0u},
            (const u64*)ct_in, g};
    io.add2 = (const u64*)ct_add;
    return keyswitch_impl(c, io, B, nlimbs, (const u64*)evk, (char*)ws, st);
  }
  if (ct_add && ct_add == ct_out) return fail(CKKS_EINVAL, "internal: accumulating in place needs the N = 2^16 path");
  const size_t ks = ks_layout(c, B, nlimbs).total;
  u64* d = (u64*)((char*)ws + ks);
  const LimbMap qmap = identity_map(nlimbs);
  // sigma(c0) -> out[.,0]; sigma(c1) -> d
  if ((rc = launch_automorph(c, (u64*)ct_out, 2 * polyN, (const u64*)ct_in, 2 * polyN, B, nlimbs, qmap, g, true, st)))
    return rc;
  if ((rc = launch_automorph(c, d, polyN, (const u64*)ct_in + polyN, 2 * polyN, B, nlimbs, qmap, g, true, st))) return rc;
  KsIo io{d, polyN, 0, (u64*)ct_out, {1, 0}, nullptr, 0};
  if ((rc = keyswitch_impl(c, io, B, nlimbs, (const u64*)evk, (char*)ws, st))) return rc;
  if (ct_add) {
    AddArgs ad{(u64*)ct_out, (const u64*)ct_add, c->d_mods, c->logN, nlimbs};
    ProfScope ps(c, PK_ADD, st);
    hipLaunchKernelGGL(addto_kernel, dim3(c->N / 256, nlimbs, 2 * B), dim3(256), 0, st, ad);
    HIP_TRY(hipGetLastError());
  }
  return CKKS_OK;
}

size_t ckks_noalloc_scratch_bytes(void) { return (size_t)CKKS_NOALLOC_SCRATCH_BYTES; }

// ckks_hrot with the library's fixed scratch array as its workspace: no hipMalloc/hipFree here or below (the level
// tables, the second stream and its events exist since ckks_ctx_create). Every region of the workspace is written
// by a kernel of the call before a later kernel reads it, so nothing has to be cleared between calls.
int ckks_hrot_noalloc(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs, uint32_t g,
                      const uint64_t* evk, void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (c->prof_on) return fail(CKKS_EINVAL, "ckks_hrot_noalloc: per-kernel timing creates events; disable it first");
  const size_t need = ckks_workspace_bytes(c, CKKS_OP_HROT, B, nlimbs, 0);
  if (need == 0 || need > (size_t)CKKS_NOALLOC_SCRATCH_BYTES)
    return fail(CKKS_EWORKSPACE, "ckks_hrot_noalloc: this batch needs " + std::to_string(need) +
                                     " bytes of workspace, the fixed scratch array holds " +
                                     std::to_string((size_t)CKKS_NOALLOC_SCRATCH_BYTES));
  return hrot_impl(c, ct_out, ct_in, B, nlimbs, g, evk, c->scratch_ptr, (size_t)CKKS_NOALLOC_SCRATCH_BYTES, stream, nullptr);
}

int ckks_hrot_add(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, const uint64_t* ct_add, uint32_t B, uint32_t nlimbs,
                  uint32_t g, const uint64_t* evk, void* ws, size_t ws_bytes, void* stream) {
  if (!ct_add) return fail(CKKS_EINVAL, "null argument");
  if (c && c->logN != 16 && ct_add == ct_out) return fail(CKKS_EINVAL, "ct_add == ct_out needs N = 2^16");
  return hrot_impl(c, ct_out, ct_in, B, nlimbs, g, evk, ws, ws_bytes, stream, ct_add);
}

int ckks_hrot_multi(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                    const uint32_t* galois_elts, const uint64_t* const* evks, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ct_out || !ct_in || !galois_elts || !evks) return fail(CKKS_EINVAL, "null argument");
  for (u32 b = 0; b < B; b++) {
    if (!evks[b]) return fail(CKKS_EINVAL, "null key");
    if (!(galois_elts[b] & 1) || galois_elts[b] >= 2 * c->N) return fail(CKKS_EINVAL, "galois_elt must be odd and < 2N");
  }
  if ((rc = check_ws(c, CKKS_OP_HROT, B, nlimbs, 0, ws, ws_bytes))) return rc;
  const size_t polyN = (size_t)nlimbs * c->N, ct_bytes = (size_t)B * 2 * polyN * 8;
  if (overlap(ct_out, ct_bytes, ct_in, ct_bytes)) return fail(CKKS_EINVAL, "ct_out overlaps ct_in");
  if (c->logN != 16) {
    // other ring sizes: one rotation at a time through the general path
    for (u32 b = 0; b < B; b++)
      if ((rc = hrot_impl(c, ct_out + b * 2 * polyN, ct_in + b * 2 * polyN, 1, nlimbs, galois_elts[b], evks[b], ws, ws_bytes,
                          stream, nullptr)))
        return rc;
    return CKKS_OK;
  }
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  // the kernels carry the per-ciphertext elements and key pointers in their arguments, KS_MULTI_MAX at a time
  for (u32 b0 = 0; b0 < B; b0 += KS_MULTI_MAX) {
    const u32 nb = std::min<u32>(KS_MULTI_MAX, B - b0);
    const u64* in = (const u64*)ct_in + (size_t)b0 * 2 * polyN;
    KsIo io{in + polyN, 2 * polyN, 0, (u64*)ct_out + (size_t)b0 * 2 * polyN, {2u, 0u}, in, 0};
    io.galois_pc = galois_elts + b0;
    io.evk_pc = (const u64* const*)evks + b0;
    if ((rc = keyswitch_impl(c, io, nb, nlimbs, nullptr, (char*)ws, st))) return rc;
  }
  return CKKS_OK;
}

int ckks_hmult_relin(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_a, const uint64_t* ct_b, uint32_t B,
                     uint32_t nlimbs, const uint64_t* evk, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ct_out || !ct_a || !ct_b || !evk) return fail(CKKS_EINVAL, "null argument");
  if ((rc = check_ws(c, CKKS_OP_HMULT_RELIN, B, nlimbs, 0, ws, ws_bytes))) return rc;
  const size_t ct_bytes = (size_t)B * 2 * nlimbs * c->N * 8;
  if (overlap(ct_out, ct_bytes, ct_a, ct_bytes) || overlap(ct_out, ct_bytes, ct_b, ct_bytes))
    return fail(CKKS_EINVAL, "ct_out overlaps an input");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  const size_t ks = ks_layout(c, B, nlimbs).total;
  u64* d2 = (u64*)((char*)ws + ks);
  TensorArgs a{(const u64*)ct_a, (const u64*)ct_b, (u64*)ct_out, d2, c->d_mods, c->logN, nlimbs};
  {
    ProfScope ps(c, PK_TENSOR, st);
    hipLaunchKernelGGL(tensor_kernel, dim3(c->N / 256, nlimbs, B), dim3(256), 0, st, a);
  }
  HIP_TRY(hipGetLastError());
  KsIo io{d2, (u64)nlimbs * c->N, 0, (u64*)ct_out, {1, 1}, nullptr, 0};
  return keyswitch_impl(c, io, B, nlimbs, (const u64*)evk, (char*)ws, st);
}

int ckks_tensor_acc(ckks_ctx* c, uint64_t* d_out, const uint64_t* ct_a, const uint64_t* ct_b, const uint64_t* d_acc,
                    uint32_t B, uint32_t nlimbs, void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!d_out || !ct_a || !ct_b) return fail(CKKS_EINVAL, "null argument");
  const size_t ct_bytes = (size_t)B * 2 * nlimbs * c->N * 8, d_bytes = ct_bytes / 2 * 3;
  if (overlap(d_out, d_bytes, ct_a, ct_bytes) || overlap(d_out, d_bytes, ct_b, ct_bytes))
    return fail(CKKS_EINVAL, "d_out overlaps an input ciphertext");
  if (d_acc && d_acc != d_out && overlap(d_out, d_bytes, d_acc, d_bytes))
    return fail(CKKS_EINVAL, "d_acc overlaps d_out without being d_out");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  TensorAccArgs a{(const u64*)ct_a, (const u64*)ct_b, (const u64*)d_acc, (u64*)d_out, c->d_mods, c->logN, nlimbs};
  {
    ProfScope ps(c, PK_TENSOR, st);
    hipLaunchKernelGGL(tensor_acc_kernel, dim3(c->N / 256, nlimbs, B), dim3(256), 0, st, a);
  }
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}

int ckks_relin(ckks_ctx* c, uint64_t* ct_out, const uint64_t* d_in, uint32_t B, uint32_t nlimbs, const uint64_t* evk,
               void* ws, size_t ws_bytes, void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ct_out || !d_in || !evk) return fail(CKKS_EINVAL, "null argument");
  if ((rc = check_ws(c, CKKS_OP_KEYSWITCH, B, nlimbs, 0, ws, ws_bytes))) return rc;
  const size_t polyN = (size_t)nlimbs * c->N;
  if (overlap(ct_out, (size_t)B * 2 * polyN * 8, d_in, (size_t)B * 3 * polyN * 8))
    return fail(CKKS_EINVAL, "ct_out overlaps d_in");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  const u64* d = (const u64*)d_in;
  KsIo io{d + 2 * polyN, 3 * (u64)polyN, 0, (u64*)ct_out, {1, 1}, nullptr, 0};
  if (c->logN == 16) {
    // the last kernel of the key switch reads d0 and d1 in place
    io.add2 = d;
    io.add2_three = true;
  } else {
    // general path: d0, d1 are copied into ct_out and the key switch adds to them in place
    const size_t pl2 = polyN / 2;
    ProfScope ps(c, PK_ADD, st);
    hipLaunchKernelGGL(first_two_components_kernel, dim3((unsigned)((2 * pl2 + 255) / 256), B), dim3(256), 0, st,
                       (const ulonglong2*)d, (ulonglong2*)ct_out, pl2);
    HIP_TRY(hipGetLastError());
  }
  return keyswitch_impl(c, io, B, nlimbs, (const u64*)evk, (char*)ws, st);
}

static int pcmm_impl(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                     const uint64_t* pt, uint32_t n1, uint32_t n2, uint32_t stride, const uint64_t* const* evk_baby,
                     const uint64_t* const* evk_giant, void* ws, size_t ws_bytes, void* stream, int mode);
int ckks_pcmm_bsgs(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                   const uint64_t* pt, uint32_t n1, uint32_t n2, uint32_t stride, const uint64_t* const* evk_baby,
                   const uint64_t* const* evk_giant, void* ws, size_t ws_bytes, void* stream) {
  return pcmm_impl(c, ct_out, ct_in, B, nlimbs, pt, n1, n2, stride, evk_baby, evk_giant, ws, ws_bytes, stream, 0);
}
int ckks_pcmm_bsgs_hoisted(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                           const uint64_t* pt, uint32_t n1, uint32_t n2, uint32_t stride,
                           const uint64_t* const* evk_baby, const uint64_t* const* evk_giant, void* ws, size_t ws_bytes,
                           void* stream) {
  return pcmm_impl(c, ct_out, ct_in, B, nlimbs, pt, n1, n2, stride, evk_baby, evk_giant, ws, ws_bytes, stream, 1);
}
int ckks_pcmm_bsgs_double_hoisted(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                                  const uint64_t* pt_ext, uint32_t n1, uint32_t n2, uint32_t stride,
                                  const uint64_t* const* evk_baby, const uint64_t* const* evk_giant, void* ws,
                                  size_t ws_bytes, void* stream) {
  if (c && c->logN != 16) return fail(CKKS_ESHAPE, "the double-hoisted schedule is built for N = 2^16 only");
  return pcmm_impl(c, ct_out, ct_in, B, nlimbs, pt_ext, n1, n2, stride, evk_baby, evk_giant, ws, ws_bytes, stream, 2);
}
int ckks_hrot_hoisted(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                      const uint32_t* galois_elts, const uint64_t* const* evks, uint32_t R, void* ws, size_t ws_bytes,
                      void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ct_out || !ct_in || !galois_elts || !evks) return fail(CKKS_EINVAL, "null argument");
  if (R == 0) return CKKS_OK;
  for (u32 r = 0; r < R; r++) {
    if (!evks[r]) return fail(CKKS_EINVAL, "null key");
    if (!(galois_elts[r] & 1) || galois_elts[r] >= 2 * c->N) return fail(CKKS_EINVAL, "galois_elt must be odd and < 2N");
  }
  if ((rc = check_ws(c, CKKS_OP_HROT, B, nlimbs, 0, ws, ws_bytes))) return rc;
  const size_t ct_elems = (size_t)B * 2 * nlimbs * c->N;
  if (overlap(ct_out, (size_t)R * ct_elems * 8, ct_in, ct_elems * 8)) return fail(CKKS_EINVAL, "ct_out overlaps ct_in");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  if (c->logN == 16) {
    // workspace beyond the required size holds accumulators of rotations that then share a pass over the digits
    const size_t need = ckks_workspace_bytes(c, CKKS_OP_HROT, B, nlimbs, 0);
    const size_t one = (size_t)B * 2 * (nlimbs + c->np) * c->N * 8;
    const u32 fit = (u32)std::min<size_t>((ws_bytes - need) / one, 1u << 20);
    return hrot_hoisted16(c, (u64*)ct_out, ct_elems, (const u64*)ct_in, B, nlimbs, galois_elts, (const u64* const*)evks, R,
                          (char*)ws, (hipStream_t)stream, nullptr, 0, false, (u64*)((char*)ws + need), fit);
  }
  for (u32 r = 0; r < R; r++)  // other ring degrees: the same result, one rotation at a time
    if ((rc = ckks_hrot(c, ct_out + (size_t)r * ct_elems, ct_in, B, nlimbs, galois_elts[r], evks[r], ws, ws_bytes, stream)))
      return rc;
  return CKKS_OK;
}
int ckks_hrot_sum(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                  const uint32_t* galois_elts, const uint64_t* const* evks, uint32_t R, void* ws, size_t ws_bytes,
                  void* stream) {
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (c->logN != 16) return fail(CKKS_ESHAPE, "the hoisted rotate-and-sum is built for N = 2^16 only");
  if (!ct_out || !ct_in || (R && (!galois_elts || !evks))) return fail(CKKS_EINVAL, "null argument");
  if (2 * B > 65535) return fail(CKKS_ESHAPE, "batch too large for one call");
  for (u32 r = 0; r < R; r++) {
    if (!evks[r]) return fail(CKKS_EINVAL, "null key");
    if (!(galois_elts[r] & 1) || galois_elts[r] >= 2 * c->N) return fail(CKKS_EINVAL, "galois_elt must be odd and < 2N");
  }
  if ((rc = check_ws(c, CKKS_OP_HROT_SUM, B, nlimbs, 0, ws, ws_bytes))) return rc;
  const size_t N = c->N, ct_bytes = (size_t)B * 2 * nlimbs * N * 8;
  if (overlap(ct_out, ct_bytes, ct_in, ct_bytes)) return fail(CKKS_EINVAL, "ct_out overlaps ct_in");
  const LevelTables* lt;
  if ((rc = get_level(c, nlimbs, &lt))) return rc;
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  const u32 next = nlimbs + c->np;
  char* hws = (char*)ws;
  u64* total = (u64*)(hws + ckks_workspace_bytes(c, CKKS_OP_HROT, B, nlimbs, 0));
  FwdInnerArgs ia;
  if ((rc = hoist_front16(c, lt, (const u64*)ct_in, B, nlimbs, hws, st, ia))) return rc;
  ia.acc = total;
  ia.c0 = (const u64*)ct_in;
  ia.c0_poly_stride = 2 * (u64)nlimbs * N;
  const LimbMap emap = ext_map(c, nlimbs);
  // up to KS_MULTI_MAX rotations per launch; the first launch starts from P * ct, later ones add to the sum
  for (u32 r0 = 0; r0 == 0 || r0 < R; r0 += KS_MULTI_MAX) {
    const u32 nr = std::min<u32>(KS_MULTI_MAX, R - r0);
    ia.nrot = nr;
    ia.accumulate = r0 ? 1u : 0u;
    for (u32 r = 0; r < nr; r++) {
      ia.galois_pc[r] = galois_elts[r0 + r];
      ia.evk_pc[r] = (const u64*)evks[r0 + r];
    }
    for (int fp = 1; fp >= 0; fp--) {
      FwdInnerArgs a = ia;
      u32 cnt = 0;
      for (u32 s_ = 0; s_ < next; s_++)
        if ((host_class(c, c->mod[emap.id[s_]]) == 0) == (fp == 1)) a.slots[cnt++] = (unsigned char)s_;
      if (!cnt) continue;
      ProfScope ps(c, fp ? PK_INNER16 : PK_INNER16_INT, st);
      if (fp) hipLaunchKernelGGL(inner16_sum_fp_kernel, dim3(B, 128, cnt), dim3(256), 0, st, a);
      else hipLaunchKernelGGL(inner16_sum_int_kernel, dim3(B, 128, cnt), dim3(256), 0, st, a);
    }
    HIP_TRY(hipGetLastError());
  }
  KsIo io{nullptr, 0, 0, (u64*)ct_out, {0, 0}, nullptr, 0};
  return ks16_finish(c, lt, io, B, nlimbs, hws, st, total);
}

static int pcmm_impl(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                     const uint64_t* pt, uint32_t n1, uint32_t n2, uint32_t stride, const uint64_t* const* evk_baby,
                     const uint64_t* const* evk_giant, void* ws, size_t ws_bytes, void* stream, int mode) {
  // mode 0: one rotation at a time; 1: hoisted baby steps; 2: baby steps kept in the extended basis (pt holds the
  // plaintexts in that basis), one ModDown per giant step
  const bool hoisted = mode == 1, dh = mode == 2;
  int rc = check_common(c, B, nlimbs);
  if (rc) return rc;
  if (!ct_out || !ct_in || !pt) return fail(CKKS_EINVAL, "null argument");
  if (n1 == 0 || n2 == 0 || stride == 0) return fail(CKKS_ESHAPE, "n1, n2 and stride must be positive");
  if ((n1 > 1 && !evk_baby) || (n2 > 1 && !evk_giant)) return fail(CKKS_EINVAL, "null key array");
  for (u32 b = 1; b < n1; b++)
    if (!evk_baby[b - 1]) return fail(CKKS_EINVAL, "null baby-step key");
  for (u32 g = 1; g < n2; g++)
    if (!evk_giant[g - 1]) return fail(CKKS_EINVAL, "null giant-step key");
  if (2 * B > 65535) return fail(CKKS_ESHAPE, "batch too large for one call");
  if ((rc = check_ws(c, dh ? CKKS_OP_PCMM_BSGS_DH : CKKS_OP_PCMM_BSGS, B, nlimbs, n1, ws, ws_bytes))) return rc;
  const size_t N = c->N, polyN = (size_t)nlimbs * N, ct_bytes = (size_t)B * 2 * polyN * 8;
  if (overlap(ct_out, ct_bytes, ct_in, ct_bytes)) return fail(CKKS_EINVAL, "ct_out overlaps ct_in");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  const size_t ct_al = 2 * align256((size_t)B * polyN * 8);
  // polynomials the inner sums work on: nlimbs limbs, or the nlimbs + K slots of the extended basis
  const u32 pl_limbs = dh ? nlimbs + c->np : nlimbs;
  const size_t sum_al = dh ? 2 * align256((size_t)B * pl_limbs * N * 8) : ct_al;
  char* w = (char*)ws;
  u64* first = nullptr;                 // double-hoisted: (P c0, P c1), the term of baby step 0
  u64* total = nullptr;                 // double-hoisted: sum over giant steps, extended basis
  if (dh) { first = (u64*)w;            w += sum_al; }
  if (dh) { total = (u64*)w;            w += sum_al; }
  u64* baby = (u64*)w;                  w += (size_t)(n1 - 1) * sum_al;
  u64* inner = (u64*)w;                 w += (size_t)PMACC_TILE * sum_al;   // inner sums of one tile of giant steps
  u64* rot = (u64*)w;                   w += ct_al;
  char* hws = w;
  const size_t hws_bytes = ckks_workspace_bytes(c, CKKS_OP_HROT, B, nlimbs, 0);
  const u64 twoN = 2 * N;
  auto galois = [&](u64 r) {  // 5^r mod 2N
    u64 g = 1, b = 5;
    for (; r; r >>= 1) {
      if (r & 1) g = g * b % twoN;
      b = b * b % twoN;
    }
    return (u32)g;
  };
  const size_t ct_elems = ct_al / 8;  // == B*2*nlimbs*N: a limb-vector is a multiple of 256 bytes
  const size_t sum_elems = sum_al / 8;
  const LevelTables* lt = nullptr;
  if (dh) {
    if ((rc = get_level(c, nlimbs, &lt))) return rc;
    LiftArgs la{(const u64*)ct_in, first, c->d_mods, c->logN, nlimbs, pl_limbs, {}};
    for (u32 i = 0; i < nlimbs; i++) la.fp[i] = host_class(c, c->mod[i]) == 0 ? 1 : 0;
    {
      ProfScope ps(c, PK_ADD, st);
      hipLaunchKernelGGL(lift_qp_kernel, dim3(N / 512, pl_limbs, 2 * B), dim3(256), 0, st, la);
    }
    HIP_TRY(hipGetLastError());
    if (n1 > 1) {
      std::vector<u32> gs(n1 - 1);
      for (u32 b = 1; b < n1; b++) gs[b - 1] = galois((u64)b * stride);
      if ((rc = hrot_hoisted16(c, nullptr, 0, (const u64*)ct_in, B, nlimbs, gs.data(), (const u64* const*)evk_baby, n1 - 1,
                               hws, st, baby, sum_elems)))
        return rc;
    }
  } else if (hoisted && n1 > 1) {
    std::vector<u32> gs(n1 - 1);
    for (u32 b = 1; b < n1; b++) gs[b - 1] = galois((u64)b * stride);
    if (c->logN == 16) {
      // the region of the inner sums is free until the baby steps are done: it holds the accumulators of as many
      // rotations as fit, which then share one pass over the hoisted digits
      const size_t one = (size_t)B * 2 * (nlimbs + c->np) * N * 8;
      const u32 fit = (u32)std::min<size_t>((size_t)PMACC_TILE * ct_al / one, 1u << 20);
      rc = hrot_hoisted16(c, baby, ct_elems, (const u64*)ct_in, B, nlimbs, gs.data(), (const u64* const*)evk_baby, n1 - 1,
                          hws, st, nullptr, 0, false, inner, fit);
    } else {
      rc = ckks_hrot_hoisted(c, (uint64_t*)baby, ct_in, B, nlimbs, gs.data(), evk_baby, n1 - 1, hws, hws_bytes, stream);
    }
    if (rc) return rc;
  } else {
    for (u32 b = 1; b < n1; b++) {
      rc = ckks_hrot(c, (uint64_t*)(baby + (size_t)(b - 1) * ct_elems), ct_in, B, nlimbs, galois((u64)b * stride),
                     evk_baby[b - 1], hws, hws_bytes, stream);
      if (rc) return rc;
    }
  }
  // limbs by arithmetic kind: the double-precision kernel computes up to 6 giant steps x 8 polynomials per pass
  // over the baby-step ciphertexts, the integer kernel up to 3 giant steps x 4 polynomials
  PmaccArgs fa, ia;
  u32 nfp = 0, nint = 0;
  for (u32 i = 0; i < pl_limbs; i++) {
    const u32 id = i < nlimbs ? i : c->nq + (i - nlimbs);
    if (host_class(c, c->mod[id]) == 0 && c->tune[6] == 0) {
      fa.mod_ids[nfp] = (unsigned char)id;
      fa.limbs[nfp++] = (unsigned char)i;
    } else {
      ia.mod_ids[nint] = (unsigned char)id;
      ia.limbs[nint++] = (unsigned char)i;
    }
  }
  const u32 tile_max = c->tune[7] > 0 ? std::min<u32>(PMACC_TILE, (u32)c->tune[7]) : PMACC_TILE;
  for (u32 g0 = 0; g0 < n2;) {
    const u32 ng = std::min<u32>(tile_max, n2 - g0);
    // giant step 0 needs no rotation: its inner sum is written straight into the output
    auto fill = [&](PmaccArgs& a, u32 first_g, u32 count) {
      a.ct_in = dh ? first : (const u64*)ct_in;
      a.baby = baby;
      a.pt = (const u64*)pt;
      a.out0 = first_g == 0 ? (dh ? total : (u64*)ct_out) : inner + (size_t)(first_g - g0) * sum_elems;
      a.out_rest = inner + (size_t)(first_g - g0 + 1) * sum_elems;
      a.mods = c->d_mods;
      a.logN = c->logN;
      a.nlimbs = pl_limbs;
      a.n1 = n1;
      a.B = B;
      a.g0 = first_g;
      a.ng = count;
    };
    for (u32 h0 = g0; nfp && h0 < g0 + ng;) {
      static const u32 kSizes[] = {6, 4, 3, 2, 1};
      u32 cnt = 1;
      for (u32 sz : kSizes)
        if (sz <= g0 + ng - h0) {
          cnt = sz;
          break;
        }
      const u32 ngt = (g0 + ng - h0) / cnt;   // as many whole tiles of this size as remain, in one launch
      fill(fa, h0, cnt);
      fa.ngt = ngt;
      ProfScope ps(c, PK_PMACC_FP, st);
      dim3 grid((2 * B + PMACC_FP_P - 1) / PMACC_FP_P * ngt, N / 256, nfp), block(256);
      switch (cnt) {
        case 6: hipLaunchKernelGGL(pmacc_fp_kernel<6>, grid, block, 0, st, fa); break;
        case 4: hipLaunchKernelGGL(pmacc_fp_kernel<4>, grid, block, 0, st, fa); break;
        case 3: hipLaunchKernelGGL(pmacc_fp_kernel<3>, grid, block, 0, st, fa); break;
        case 2: hipLaunchKernelGGL(pmacc_fp_kernel<2>, grid, block, 0, st, fa); break;
        default: hipLaunchKernelGGL(pmacc_fp_kernel<1>, grid, block, 0, st, fa); break;
      }
      HIP_TRY(hipGetLastError());
      h0 += cnt * ngt;
    }
    for (u32 h0 = g0; nint && h0 < g0 + ng;) {
      static const u32 kSizes[] = {3, 2, 1};
      u32 cnt = 1;
      for (u32 sz : kSizes)
        if (sz <= g0 + ng - h0) {
          cnt = sz;
          break;
        }
      const u32 ngt = (g0 + ng - h0) / cnt;
      fill(ia, h0, cnt);
      ia.ngt = ngt;
      ProfScope ps(c, PK_PMACC, st);
      dim3 grid((2 * B + PMACC_INT_P - 1) / PMACC_INT_P * ngt, N / 256, nint), block(256);
      switch (cnt) {
        case 3: hipLaunchKernelGGL(pmacc_int_kernel<3>, grid, block, 0, st, ia); break;
        case 2: hipLaunchKernelGGL(pmacc_int_kernel<2>, grid, block, 0, st, ia); break;
        default: hipLaunchKernelGGL(pmacc_int_kernel<1>, grid, block, 0, st, ia); break;
      }
      HIP_TRY(hipGetLastError());
      h0 += cnt * ngt;
    }
    for (u32 k = 0; k < ng; k++) {
      const u32 g = g0 + k;
      if (dh) {
        // giant step 0 is already in `total`; the others: ModDown of the inner sum into `rot`, then its rotation
        // (one hoisted rotation that stops before ModDown) added to `total`
        if (g == 0) continue;
        KsIo io{nullptr, 0, 0, rot, {0, 0}, nullptr, 0};
        if ((rc = ks16_finish(c, lt, io, B, nlimbs, hws, st, inner + (size_t)k * sum_elems))) return rc;
        const u32 gg = galois((u64)g * n1 * stride);
        const u64* key = (const u64*)evk_giant[g - 1];
        if (c->tune[3] != 1) {
          // the usual fused sequence of a rotation (c1 read through the Galois map), stopped before ModDown
          KsIo gio{rot + polyN, 2 * (u64)polyN, gg, nullptr, {0, 0}, rot, gg};
          rc = keyswitch_fused16(c, lt, gio, B, nlimbs, key, hws, st, total);
        } else {
          rc = hrot_hoisted16(c, nullptr, 0, rot, B, nlimbs, &gg, &key, 1, hws, st, total, 0, /*acc_add=*/true);
        }
        if (rc) return rc;
        continue;
      }
      if (g == 0) continue;
      const u64* src = inner + (size_t)k * ct_elems;
      if (c->logN == 16) {
        rc = hrot_impl(c, ct_out, (const uint64_t*)src, B, nlimbs, galois((u64)g * n1 * stride), evk_giant[g - 1], hws,
                       hws_bytes, stream, /*ct_add=*/ct_out);
        if (rc) return rc;
      } else {
        rc = ckks_hrot(c, (uint64_t*)rot, (const uint64_t*)src, B, nlimbs, galois((u64)g * n1 * stride), evk_giant[g - 1], hws,
                       hws_bytes, stream);
        if (rc) return rc;
        AddArgs ad{(u64*)ct_out, rot, c->d_mods, c->logN, nlimbs};
        ProfScope ps(c, PK_ADD, st);
        hipLaunchKernelGGL(addto_kernel, dim3(N / 256, nlimbs, 2 * B), dim3(256), 0, st, ad);
        HIP_TRY(hipGetLastError());
      }
    }
    g0 += ng;
  }
  if (dh) {   // one ModDown of the sum over giant steps
    KsIo io{nullptr, 0, 0, (u64*)ct_out, {0, 0}, nullptr, 0};
    if ((rc = ks16_finish(c, lt, io, B, nlimbs, hws, st, total))) return rc;
  }
  return CKKS_OK;
}

int ckks_rescale(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs, void* ws,
                 size_t ws_bytes, void* stream) {
  if (!c || !ct_out || !ct_in) return fail(CKKS_EINVAL, "null argument");
  if (nlimbs < 2 || nlimbs > c->nq) return fail(CKKS_ESHAPE, "rescale needs 2..L+1 limbs");
  if (B == 0 || B > 32767) return fail(CKKS_ESHAPE, "batch must be in [1, 32767]");
  int rc = check_ws(c, CKKS_OP_RESCALE, B, nlimbs, 0, ws, ws_bytes);
  if (rc) return rc;
  const u32 N = c->N, nl1 = nlimbs - 1;
  if (overlap(ct_out, (size_t)B * 2 * nl1 * N * 8, ct_in, (size_t)B * 2 * nlimbs * N * 8))
    return fail(CKKS_EINVAL, "ct_out overlaps ct_in");
  const LevelTables* lt;
  if ((rc = get_level(c, nlimbs, &lt))) return rc;
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  hipStream_t st = (hipStream_t)stream;
  u64* last = (u64*)ws;
  u64* tq = (u64*)((char*)ws + align256((size_t)B * 2 * N * 8));
  // 1. coefficient form of the last limb of every polynomial (rows of ct_in are nlimbs*N apart)
  LimbMap lmap = identity_map(0);
  lmap.id[0] = (unsigned char)nl1;
  if ((rc = launch_ntt(c, true, (const u64*)ct_in + (size_t)nl1 * N, (u64)nlimbs * N, last, (u64)N, B * 2, 0, 1, lmap, 0, 0, st)))
    return rc;
  // 2. its centred representative on the remaining limbs (a one-source base conversion)
  {
    ModDownArgs a{last, tq, c->d_mods, lt->rs_one, lt->rs_mat, c->logN, nl1, c->nq, 1, 1, 0, nl1};
    ProfScope ps(c, PK_MODDOWN, st);
    launch_moddown<true>(c, a, B * 2, lt->narrow_rs, st);
    HIP_TRY(hipGetLastError());
  }
  // 3. back to the evaluation domain, subtract, divide by q_last
  const LimbMap qmap = identity_map(nl1);
  if (c->logN == 16) {
    NttOpts o;
    o.rows_only = true;
    if ((rc = launch_ntt(c, false, tq, (u64)nl1 * N, tq, (u64)nl1 * N, B * 2, 0, nl1, qmap, 0, 0, st, o))) return rc;
    FwdFinalArgs a;
    a.tq = tq;
    a.acc = (const u64*)ct_in;
    a.out = (u64*)ct_out;
    a.add_src = nullptr;
    a.add2 = nullptr;
    a.tw = c->d_tw_fwd;
    a.twfp = c->d_twfp_fwd;
    a.mods = c->d_mods;
    a.pinv = lt->rs_qinv16;
    a.nlimbs = nl1;
    a.next = nlimbs;
    a.mode0 = a.mode1 = 0;
    a.galois = 0;
    a.map_mode = map_mode_pass(c);
    auto cls_of = [&](u32 s) { return host_class(c, c->mod[s]); };
    LAUNCH_BY_CLASS(c, PK_FWD_FINAL, ntt16_fwd_blocks_final_kernel, a, B * 2, nl1, cls_of, st)
    HIP_TRY(hipGetLastError());
    return CKKS_OK;
  }
  if ((rc = launch_ntt(c, false, tq, (u64)nl1 * N, tq, (u64)nl1 * N, B * 2, 0, nl1, qmap, 0, 0, st))) return rc;
  FinalArgs a{(const u64*)ct_in, tq, (u64*)ct_out, c->d_mods, lt->rs_qinv, c->logN, nl1, nlimbs, 0};
  ProfScope ps(c, PK_FINAL, st);
  hipLaunchKernelGGL(ks_final_kernel, dim3(N / 256, nl1, B * 2), dim3(256), 0, st, a);
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}

static int pointwise_entry(ckks_ctx* c, bool mul, uint64_t* out, const uint64_t* a, const uint64_t* b, uint32_t npoly,
                           uint32_t nlimbs, bool broadcast, void* stream) {
  if (!c || !out || !a || !b) return fail(CKKS_EINVAL, "null argument");
  if (nlimbs == 0 || nlimbs > c->nq) return fail(CKKS_ESHAPE, "nlimbs must be in [1, L+1]");
  if (npoly == 0) return CKKS_OK;
  if (npoly > 65535) return fail(CKKS_ESHAPE, "too many polynomials in one call");
  DeviceGuard guard(c->device);
  if (!guard.ok) return fail(CKKS_EHIP, "cannot select the context's device");
  PointwiseArgs pa{(u64*)out, (const u64*)a, (const u64*)b, c->d_mods, c->logN, nlimbs, broadcast ? 1u : 0u};
  ProfScope ps(c, mul ? PK_TENSOR : PK_ADD, (hipStream_t)stream);
  dim3 grid(c->N / 512, nlimbs, npoly), block(256);
  if (mul) hipLaunchKernelGGL(pmult_kernel, grid, block, 0, (hipStream_t)stream, pa);
  else hipLaunchKernelGGL(add_kernel, grid, block, 0, (hipStream_t)stream, pa);
  HIP_TRY(hipGetLastError());
  return CKKS_OK;
}
int ckks_pmult(ckks_ctx* c, uint64_t* ct_out, const uint64_t* ct_in, const uint64_t* pt, uint32_t B, uint32_t nlimbs,
               void* stream) {
  if (B > 32767) return fail(CKKS_ESHAPE, "batch must be in [1, 32767]");
  return pointwise_entry(c, true, ct_out, ct_in, pt, B * 2, nlimbs, true, stream);
}
int ckks_add(ckks_ctx* c, uint64_t* out, const uint64_t* a, const uint64_t* b, uint32_t npoly, uint32_t nlimbs,
             void* stream) {
  return pointwise_entry(c, false, out, a, b, npoly, nlimbs, false, stream);
}

}  // extern "C"
