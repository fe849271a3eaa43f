// CPU oracle for batched RNS-CKKS polynomial arithmetic.
//
// TEST INFRASTRUCTURE ONLY. This file is the slow, plain statement of what the GPU
// library must compute. It shares no code, header, table or constant generator with
// the HIP path; it is called from tests, the smoke check and the CPU-baseline leg of
// the benchmark, never from the product path.
//
// What it follows. The paper fixes the ring Z_q[x]/(x^N+1) with S = N/2 slots, the
// RNS representation over primes q_0..q_L, the RNS-major tensor layout, and the
// operator vocabulary (Sec. 2.1 "Homomorphic Encryption and Operations", Sec. 2.2
// "Data Structure in Homomorphic Encryption", Sec. 3.2.1). It names NTT/INTT,
// automorphism, ModUp/base conversion and key switching over Q*P with special primes,
// but prints no formula for any of them. The definitions below are therefore the
// standard RNS-CKKS ones from the literature the paper cites; every such choice is a
// "reading" and is listed in the design document.
//
// Style: every modular operation is `unsigned __int128` product followed by `%`.
// No lazy ranges, no precomputed Shoup/Barrett/Montgomery constants, no blocking.
// Base conversion is evaluated as an exact multi-precision integer sum and only then
// reduced. The fast transform is "twist, recursive cyclic transform, bit-reverse" and
// is checked against the O(N^2) definition in the tests.
//
// Layouts (host pointers, uint64): polynomial tensors are [npoly][nlimbs][N],
// ciphertexts [B][2][nlimbs][N] with (c0,c1), Dec = c0 + c1*s; evaluation keys
// [dnum][2][nq+np][N] with row 0 = b, row 1 = a. "Eval domain" means the output order
// of ref_ntt: index k holds a(psi^(2*bitrev(k)+1)).

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <string>
#include <thread>
#include <vector>
#include <algorithm>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

namespace {

thread_local std::string g_err;
int g_threads = 1;

inline u64 addm(u64 a, u64 b, u64 m) { u128 s = (u128)a + b; return (u64)(s % m); }
inline u64 subm(u64 a, u64 b, u64 m) { return (u64)(((u128)a + m - (b % m)) % m); }
inline u64 mulm(u64 a, u64 b, u64 m) { return (u64)(((u128)a * b) % m); }
u64 powm(u64 a, u64 e, u64 m) {
  u64 r = 1 % m;
  a %= m;
  while (e) {
    if (e & 1) r = mulm(r, a, m);
    a = mulm(a, a, m);
    e >>= 1;
  }
  return r;
}
inline u64 invm(u64 a, u64 m) { return powm(a, m - 2, m); }  // m prime
inline u64 from_signed(i64 v, u64 m) {
  if (v >= 0) return (u64)v % m;
  u64 r = (u64)(-v) % m;
  return r ? m - r : 0;
}

u64 bitrev(u64 x, int bits) {
  u64 r = 0;
  for (int i = 0; i < bits; i++) r |= ((x >> i) & 1) << (bits - 1 - i);
  return r;
}

// ---- minimal unsigned multi-precision integers (little-endian 64-bit words) ----
typedef std::vector<u64> Big;
void big_mul_word(Big& a, u64 w) {
  u64 carry = 0;
  for (size_t i = 0; i < a.size(); i++) {
    u128 t = (u128)a[i] * w + carry;
    a[i] = (u64)t;
    carry = (u64)(t >> 64);
  }
  if (carry) a.push_back(carry);
}
void big_add(Big& a, const Big& b) {
  if (a.size() < b.size()) a.resize(b.size(), 0);
  u64 carry = 0;
  for (size_t i = 0; i < a.size(); i++) {
    u128 t = (u128)a[i] + (i < b.size() ? b[i] : 0) + carry;
    a[i] = (u64)t;
    carry = (u64)(t >> 64);
  }
  if (carry) a.push_back(carry);
}
u64 big_mod_word(const Big& a, u64 m) {
  u64 r = 0;
  for (size_t i = a.size(); i-- > 0;) r = (u64)((((u128)r << 64) | a[i]) % m);
  return r;
}

}  // namespace

struct RefCtx {
  int logN = 0;
  size_t N = 0;
  int nq = 0, np = 0, dnum = 0, alpha = 0;
  std::vector<u64> mod;  // q then p
  std::vector<u64> psi;
};

namespace {

bool is_prime_u64(u64 n) {
  if (n < 2) return false;
  static const u64 bases[] = {2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37};
  for (u64 b : bases) {
    if (n % b == 0) return n == b;
  }
  u64 d = n - 1;
  int r = 0;
  while ((d & 1) == 0) { d >>= 1; r++; }
  for (u64 a : bases) {
    u64 x = powm(a, d, n);
    if (x == 1 || x == n - 1) continue;
    bool comp = true;
    for (int i = 1; i < r; i++) {
      x = mulm(x, x, n);
      if (x == n - 1) { comp = false; break; }
    }
    if (comp) return false;
  }
  return true;
}

// ---------------- transforms ----------------

// Definition: out[k] = sum_j a[j] * psi^((2*bitrev(k)+1)*j) mod q.   O(N^2).
void ntt_by_definition(const RefCtx* c, u64* a, int id) {
  const size_t N = c->N;
  const u64 q = c->mod[id], psi = c->psi[id];
  std::vector<u64> out(N);
  for (size_t k = 0; k < N; k++) {
    u64 x = powm(psi, 2 * bitrev(k, c->logN) + 1, q);  // evaluation point
    u64 acc = 0, xp = 1;
    for (size_t j = 0; j < N; j++) {
      acc = addm(acc, mulm(a[j], xp, q), q);
      xp = mulm(xp, x, q);
    }
    out[k] = acc;
  }
  std::copy(out.begin(), out.end(), a);
}

// Natural-order cyclic transform A[t] = sum_j b[j] w^(j t), radix-2 recursion on even/odd samples.
void cyclic_rec(u64* b, size_t n, u64 w, u64 q, u64* tmp) {
  if (n == 1) return;
  size_t h = n / 2;
  for (size_t i = 0; i < h; i++) { tmp[i] = b[2 * i]; tmp[h + i] = b[2 * i + 1]; }
  std::copy(tmp, tmp + n, b);
  u64 w2 = mulm(w, w, q);
  cyclic_rec(b, h, w2, q, tmp);
  cyclic_rec(b + h, h, w2, q, tmp);
  u64 wp = 1;
  for (size_t t = 0; t < h; t++) {
    u64 e = b[t], o = mulm(b[h + t], wp, q);
    tmp[t] = addm(e, o, q);
    tmp[t + h] = subm(e, o, q);
    wp = mulm(wp, w, q);
  }
  std::copy(tmp, tmp + n, b);
}

// Forward: twist by psi^j, cyclic transform with w = psi^2, then store A[bitrev(k)] at k.
void ntt_fast(const RefCtx* c, u64* a, int id) {
  const size_t N = c->N;
  const u64 q = c->mod[id], psi = c->psi[id];
  std::vector<u64> b(N), tmp(N);
  u64 pw = 1;
  for (size_t j = 0; j < N; j++) { b[j] = mulm(a[j] % q, pw, q); pw = mulm(pw, psi, q); }
  cyclic_rec(b.data(), N, mulm(psi, psi, q), q, tmp.data());
  for (size_t k = 0; k < N; k++) a[k] = b[bitrev(k, c->logN)];
}

// Inverse of ntt_fast: undo the bit reversal, inverse cyclic transform, scale by 1/N, untwist.
void intt_fast(const RefCtx* c, u64* a, int id) {
  const size_t N = c->N;
  const u64 q = c->mod[id], psi = c->psi[id];
  std::vector<u64> b(N), tmp(N);
  for (size_t k = 0; k < N; k++) b[bitrev(k, c->logN)] = a[k] % q;
  u64 psi_inv = invm(psi, q);
  cyclic_rec(b.data(), N, mulm(psi_inv, psi_inv, q), q, tmp.data());
  u64 ninv = invm((u64)N % q, q), pw = 1;
  for (size_t j = 0; j < N; j++) {
    a[j] = mulm(mulm(b[j], ninv, q), pw, q);
    pw = mulm(pw, psi_inv, q);
  }
}

// Coefficient-domain Galois map a(X) -> a(X^g) in Z_q[X]/(X^N+1).
void automorph_coeff(const RefCtx* c, u64* out, const u64* in, int id, u64 g) {
  const size_t N = c->N;
  const u64 q = c->mod[id];
  for (size_t j = 0; j < N; j++) {
    size_t t = (size_t)(((u128)j * g) % (2 * N));
    u64 v = in[j] % q;
    if (t < N) out[t] = v;
    else out[t - N] = v ? q - v : 0;
  }
}

// ---------------- base conversion ----------------
// Source basis C = {c_i}, target moduli D. For one coefficient with residues x_i:
//   y_i = [x_i * (C/c_i)^-1]_{c_i}, centred to (-c_i/2, c_i/2];
//   V   = sum_i y_i * (C/c_i)  as an exact integer;   result_m = V mod m.
struct BConvPlan {
  std::vector<u64> src, dst;
  std::vector<Big> chat;      // C / c_i
  std::vector<u64> chat_inv;  // (C/c_i)^-1 mod c_i
};
BConvPlan make_bconv(const std::vector<u64>& src, const std::vector<u64>& dst) {
  BConvPlan p;
  p.src = src;
  p.dst = dst;
  for (size_t i = 0; i < src.size(); i++) {
    Big h(1, 1);
    for (size_t k = 0; k < src.size(); k++)
      if (k != i) big_mul_word(h, src[k]);
    p.chat.push_back(h);
    p.chat_inv.push_back(invm(big_mod_word(h, src[i]), src[i]));
  }
  return p;
}
// in: nsrc pointers (coefficient domain), out: ndst pointers; n coefficients.
void bconv_apply(const BConvPlan& p, const std::vector<const u64*>& in, const std::vector<u64*>& out, size_t n) {
  const size_t ns = p.src.size(), nd = p.dst.size();
  for (size_t k = 0; k < n; k++) {
    Big pos(1, 0), neg(1, 0);
    for (size_t i = 0; i < ns; i++) {
      u64 ci = p.src[i];
      u64 y = mulm(in[i][k] % ci, p.chat_inv[i], ci);
      bool negative = y > ci / 2;  // centred representative is y - c_i
      u64 mag = negative ? ci - y : y;
      Big term = p.chat[i];
      big_mul_word(term, mag);
      big_add(negative ? neg : pos, term);
    }
    for (size_t t = 0; t < nd; t++) {
      u64 m = p.dst[t];
      out[t][k] = subm(big_mod_word(pos, m), big_mod_word(neg, m), m);
    }
  }
}

template <class F>
void parallel_for(size_t n, F f) {
  int nt = std::max(1, std::min<int>(g_threads, (int)n));
  if (nt == 1) {
    for (size_t i = 0; i < n; i++) f(i);
    return;
  }
  std::vector<std::thread> th;
  for (int t = 0; t < nt; t++)
    th.emplace_back([=]() {
      for (size_t i = t; i < n; i += nt) f(i);
    });
  for (auto& x : th) x.join();
}

int fail(const std::string& s) {
  g_err = s;
  return -1;
}

bool check_ids(const RefCtx* c, const uint32_t* ids, uint32_t n) {
  for (uint32_t i = 0; i < n; i++)
    if (ids[i] >= (uint32_t)(c->nq + c->np)) return false;
  return true;
}

// First half of the hybrid key switch of ONE polynomial d (eval domain, nlimbs limbs): digit decomposition, ModUp of
// every digit to the extended basis q_0..q_{nlimbs-1}, p_0..p_{K-1}, and the inner product with evk. Returns the two
// accumulators in the evaluation domain, [2][nlimbs + K][N].
std::vector<u64> keyswitch_accumulate(const RefCtx* c, const u64* d, int nlimbs, const u64* evk) {
  const size_t N = c->N;
  const int K = c->np, nm = c->nq + c->np, alpha = c->alpha;
  const int beta = (nlimbs + alpha - 1) / alpha;
  const int next = nlimbs + K;  // extended basis: q_0..q_{nlimbs-1}, p_0..p_{K-1}
  std::vector<int> ext_id(next);
  for (int t = 0; t < nlimbs; t++) ext_id[t] = t;
  for (int k = 0; k < K; k++) ext_id[nlimbs + k] = c->nq + k;

  // coefficient form of d
  std::vector<u64> dc(d, d + (size_t)nlimbs * N);
  for (int i = 0; i < nlimbs; i++) intt_fast(c, &dc[(size_t)i * N], i);

  std::vector<u64> acc((size_t)2 * next * N, 0);
  std::vector<u64> dig((size_t)next * N);
  for (int j = 0; j < beta; j++) {
    int lo = j * alpha, hi = std::min(nlimbs, lo + alpha);
    std::vector<u64> src, dst;
    std::vector<const u64*> in;
    std::vector<u64*> out;
    for (int i = lo; i < hi; i++) { src.push_back(c->mod[i]); in.push_back(&dc[(size_t)i * N]); }
    for (int t = 0; t < next; t++) {
      if (t >= lo && t < hi) {
        std::copy(&dc[(size_t)t * N], &dc[(size_t)(t + 1) * N], &dig[(size_t)t * N]);  // digit's own limbs: as is
      } else {
        dst.push_back(c->mod[ext_id[t]]);
        out.push_back(&dig[(size_t)t * N]);
      }
    }
    BConvPlan plan = make_bconv(src, dst);
    bconv_apply(plan, in, out, N);
    for (int t = 0; t < next; t++) {
      int id = ext_id[t];
      u64 m = c->mod[id];
      u64* x = &dig[(size_t)t * N];
      ntt_fast(c, x, id);
      const u64* kb = evk + (((size_t)j * 2 + 0) * nm + id) * N;
      const u64* ka = evk + (((size_t)j * 2 + 1) * nm + id) * N;
      u64* ab = &acc[((size_t)0 * next + t) * N];
      u64* aa = &acc[((size_t)1 * next + t) * N];
      for (size_t n = 0; n < N; n++) {
        ab[n] = addm(ab[n], mulm(x[n], kb[n] % m, m), m);
        aa[n] = addm(aa[n], mulm(x[n], ka[n] % m, m), m);
      }
    }
  }
  return acc;
}

// Second half: ModDown of both accumulators (evaluation domain, [2][nlimbs + K][N], overwritten):
// x_c = INTT(x); t = BConv_{P->Q_l}(x_c|P); ks_i = NTT((x_c,i - t_i) * P^-1). Writes ks (2 x nlimbs x N).
void moddown_pair(const RefCtx* c, u64* ks, std::vector<u64>& acc, int nlimbs) {
  const size_t N = c->N;
  const int K = c->np, next = nlimbs + K;
  std::vector<int> ext_id(next);
  for (int t = 0; t < nlimbs; t++) ext_id[t] = t;
  for (int k = 0; k < K; k++) ext_id[nlimbs + k] = c->nq + k;
  std::vector<u64> psrc, qdst;
  for (int k = 0; k < K; k++) psrc.push_back(c->mod[c->nq + k]);
  for (int i = 0; i < nlimbs; i++) qdst.push_back(c->mod[i]);
  BConvPlan down = make_bconv(psrc, qdst);
  for (int comp = 0; comp < 2; comp++) {
    u64* x = &acc[(size_t)comp * next * N];
    for (int t = 0; t < next; t++) intt_fast(c, x + (size_t)t * N, ext_id[t]);
    std::vector<u64> tq((size_t)nlimbs * N);
    std::vector<const u64*> in;
    std::vector<u64*> out;
    for (int k = 0; k < K; k++) in.push_back(x + (size_t)(nlimbs + k) * N);
    for (int i = 0; i < nlimbs; i++) out.push_back(&tq[(size_t)i * N]);
    bconv_apply(down, in, out, N);
    for (int i = 0; i < nlimbs; i++) {
      u64 m = c->mod[i];
      u64 pinv = 1;
      for (int k = 0; k < K; k++) pinv = mulm(pinv, c->mod[c->nq + k] % m, m);
      pinv = invm(pinv, m);
      u64* o = ks + ((size_t)comp * nlimbs + i) * N;
      for (size_t n = 0; n < N; n++) o[n] = mulm(subm(x[(size_t)i * N + n], tq[(size_t)i * N + n], m), pinv, m);
      ntt_fast(c, o, i);
    }
  }
}

// Hybrid key switch of ONE polynomial d (eval domain, nlimbs limbs) with evk; writes ks (2 x nlimbs x N).
void keyswitch_one(const RefCtx* c, u64* ks, const u64* d, int nlimbs, const u64* evk) {
  std::vector<u64> acc = keyswitch_accumulate(c, d, nlimbs, evk);
  moddown_pair(c, ks, acc, nlimbs);
}

void automorph_eval(const RefCtx* c, u64* out, const u64* in, int id, u64 g) {
  // defined as NTT o sigma_g o INTT
  const size_t N = c->N;
  std::vector<u64> a(in, in + N), b(N);
  intt_fast(c, a.data(), id);
  automorph_coeff(c, b.data(), a.data(), id, g);
  ntt_fast(c, b.data(), id);
  std::copy(b.begin(), b.end(), out);
}

void hrot_one(const RefCtx* c, u64* out, const u64* ct, int nlimbs, u64 g, const u64* evk) {
  const size_t N = c->N;
  std::vector<u64> r0((size_t)nlimbs * N), r1((size_t)nlimbs * N), ks((size_t)2 * nlimbs * N);
  for (int i = 0; i < nlimbs; i++) {
    automorph_eval(c, &r0[(size_t)i * N], ct + (size_t)i * N, i, g);
    automorph_eval(c, &r1[(size_t)i * N], ct + ((size_t)nlimbs + i) * N, i, g);
  }
  keyswitch_one(c, ks.data(), r1.data(), nlimbs, evk);
  for (int i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i];
    for (size_t n = 0; n < N; n++) {
      out[(size_t)i * N + n] = addm(r0[(size_t)i * N + n], ks[(size_t)i * N + n], m);
      out[((size_t)nlimbs + i) * N + n] = ks[((size_t)nlimbs + i) * N + n];
    }
  }
}

}  // namespace

extern "C" {

const char* ref_last_error() { return g_err.c_str(); }
void ref_set_threads(int n) { g_threads = n < 1 ? 1 : n; }
int ref_get_threads() { return g_threads; }

int ref_ctx_create(RefCtx** out, uint32_t logN, const u64* q, uint32_t nq, const u64* p, uint32_t np, uint32_t dnum,
                   const u64* psi) {
  if (!out || !q || !psi || nq == 0 || dnum == 0 || logN < 1 || logN > 17) return fail("bad argument");
  RefCtx* c = new RefCtx;
  c->logN = logN;
  c->N = (size_t)1 << logN;
  c->nq = nq;
  c->np = np;
  c->dnum = dnum;
  c->alpha = (nq + dnum - 1) / dnum;
  for (uint32_t i = 0; i < nq; i++) c->mod.push_back(q[i]);
  for (uint32_t i = 0; i < np; i++) c->mod.push_back(p[i]);
  for (uint32_t i = 0; i < nq + np; i++) c->psi.push_back(psi[i]);
  for (size_t i = 0; i < c->mod.size(); i++) {
    u64 m = c->mod[i];
    bool ok = m < ((u64)1 << 62) && (m - 1) % (2 * c->N) == 0 && is_prime_u64(m) && powm(c->psi[i], c->N, m) == m - 1;
    for (size_t k = 0; k < i; k++) ok = ok && c->mod[k] != m;
    if (!ok) {
      delete c;
      return fail("modulus " + std::to_string(i) + " is not a distinct prime = 1 mod 2N with a primitive 2N-th root");
    }
  }
  *out = c;
  return 0;
}
int ref_ctx_destroy(RefCtx* c) {
  delete c;
  return 0;
}

// ---- scalar helpers exposed so tests can pin them ----
u64 ref_mulmod(u64 a, u64 b, u64 m) { return mulm(a, b, m); }
u64 ref_powmod(u64 a, u64 e, u64 m) { return powm(a, e, m); }

// c = a * b in Z_q[X]/(X^n + 1), schoolbook.
int ref_negacyclic_schoolbook(u64* c, const u64* a, const u64* b, uint32_t n, u64 q) {
  std::vector<u64> r(n, 0);
  for (uint32_t i = 0; i < n; i++)
    for (uint32_t j = 0; j < n; j++) {
      u64 t = mulm(a[i] % q, b[j] % q, q);
      uint32_t k = i + j;
      if (k < n) r[k] = addm(r[k], t, q);
      else r[k - n] = subm(r[k - n], t, q);
    }
  std::copy(r.begin(), r.end(), c);
  return 0;
}
// Signed integer negacyclic product (no modulus), for s^2; skips zero coefficients of a.
int ref_negacyclic_signed(i64* c, const i64* a, const i64* b, uint32_t n) {
  std::vector<i64> r(n, 0);
  for (uint32_t i = 0; i < n; i++) {
    if (!a[i]) continue;
    for (uint32_t j = 0; j < n; j++) {
      uint32_t k = i + j;
      if (k < n) r[k] += a[i] * b[j];
      else r[k - n] -= a[i] * b[j];
    }
  }
  std::copy(r.begin(), r.end(), c);
  return 0;
}
// Signed coefficient-domain Galois map.
int ref_automorph_signed(i64* out, const i64* in, uint32_t n, uint32_t g) {
  if (!(g & 1) || g >= 2 * n) return fail("galois element must be odd and < 2N");
  for (uint32_t j = 0; j < n; j++) {
    u64 t = ((u64)j * g) % (2 * (u64)n);
    if (t < n) out[t] = in[j];
    else out[t - n] = -in[j];
  }
  return 0;
}

int ref_ntt_definition(const RefCtx* c, u64* data, uint32_t limb_id) {
  if (limb_id >= (uint32_t)(c->nq + c->np)) return fail("bad limb id");
  ntt_by_definition(c, data, limb_id);
  return 0;
}

int ref_ntt(const RefCtx* c, u64* data, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs) {
  if (!check_ids(c, limb_ids, nlimbs)) return fail("bad limb id");
  parallel_for((size_t)npoly * nlimbs, [&](size_t u) { ntt_fast(c, data + u * c->N, limb_ids[u % nlimbs]); });
  return 0;
}
int ref_intt(const RefCtx* c, u64* data, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs) {
  if (!check_ids(c, limb_ids, nlimbs)) return fail("bad limb id");
  parallel_for((size_t)npoly * nlimbs, [&](size_t u) { intt_fast(c, data + u * c->N, limb_ids[u % nlimbs]); });
  return 0;
}

int ref_automorph(const RefCtx* c, u64* out, const u64* in, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs,
                  uint32_t g, int eval_domain) {
  if (!check_ids(c, limb_ids, nlimbs)) return fail("bad limb id");
  if (!(g & 1) || g >= 2 * c->N) return fail("galois element must be odd and < 2N");
  if (out == in) return fail("out must not alias in");
  parallel_for((size_t)npoly * nlimbs, [&](size_t u) {
    int id = limb_ids[u % nlimbs];
    if (eval_domain) automorph_eval(c, out + u * c->N, in + u * c->N, id, g);
    else automorph_coeff(c, out + u * c->N, in + u * c->N, id, g);
  });
  return 0;
}

// Pointwise helpers on [npoly][nlimbs][N]; b may be broadcast over polys (b_npoly == 1).
int ref_pointwise(const RefCtx* c, u64* out, const u64* a, const u64* b, uint32_t npoly, uint32_t b_npoly,
                  const uint32_t* limb_ids, uint32_t nlimbs, int op /*0 add,1 sub,2 mul*/) {
  if (!check_ids(c, limb_ids, nlimbs)) return fail("bad limb id");
  const size_t N = c->N;
  for (size_t u = 0; u < (size_t)npoly * nlimbs; u++) {
    u64 m = c->mod[limb_ids[u % nlimbs]];
    const u64* bb = b + (b_npoly == 1 ? (u % nlimbs) : u) * N;
    for (size_t n = 0; n < N; n++) {
      u64 x = a[u * N + n] % m, y = bb[n] % m;
      out[u * N + n] = op == 0 ? addm(x, y, m) : op == 1 ? subm(x, y, m) : mulm(x, y, m);
    }
  }
  return 0;
}

// Residues of a signed integer polynomial: out[nlimbs][N], coefficient domain.
int ref_signed_to_rns(const RefCtx* c, u64* out, const i64* v, const uint32_t* limb_ids, uint32_t nlimbs) {
  if (!check_ids(c, limb_ids, nlimbs)) return fail("bad limb id");
  for (uint32_t i = 0; i < nlimbs; i++)
    for (size_t n = 0; n < c->N; n++) out[(size_t)i * c->N + n] = from_signed(v[n], c->mod[limb_ids[i]]);
  return 0;
}

// Base conversion exposed for pins: in [nsrc][n], out [ndst][n], coefficient domain.
int ref_bconv(const RefCtx* c, u64* out, const u64* in, const uint32_t* src_ids, uint32_t nsrc, const uint32_t* dst_ids,
              uint32_t ndst, uint32_t n) {
  if (!check_ids(c, src_ids, nsrc) || !check_ids(c, dst_ids, ndst)) return fail("bad limb id");
  std::vector<u64> src, dst;
  std::vector<const u64*> ip;
  std::vector<u64*> op;
  for (uint32_t i = 0; i < nsrc; i++) { src.push_back(c->mod[src_ids[i]]); ip.push_back(in + (size_t)i * n); }
  for (uint32_t i = 0; i < ndst; i++) { dst.push_back(c->mod[dst_ids[i]]); op.push_back(out + (size_t)i * n); }
  bconv_apply(make_bconv(src, dst), ip, op, n);
  return 0;
}

// ModDown exposed for pins: x [nlimbs+K][n] coefficient domain over q_0..q_{nlimbs-1},p_*; out [nlimbs][n]
// = (x_i - BConv_{P->Q}(x|P)_i) * P^-1 mod q_i.
int ref_moddown_coeff(const RefCtx* c, u64* out, const u64* x, uint32_t nlimbs, uint32_t n) {
  const int K = c->np;
  std::vector<uint32_t> s, d;
  for (int k = 0; k < K; k++) s.push_back(c->nq + k);
  for (uint32_t i = 0; i < nlimbs; i++) d.push_back(i);
  std::vector<u64> t((size_t)nlimbs * n);
  if (ref_bconv(c, t.data(), x + (size_t)nlimbs * n, s.data(), K, d.data(), nlimbs, n)) return -1;
  for (uint32_t i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i], pinv = 1;
    for (int k = 0; k < K; k++) pinv = mulm(pinv, c->mod[c->nq + k] % m, m);
    pinv = invm(pinv, m);
    for (uint32_t k = 0; k < n; k++)
      out[(size_t)i * n + k] = mulm(subm(x[(size_t)i * n + k], t[(size_t)i * n + k], m), pinv, m);
  }
  return 0;
}

int ref_keyswitch(const RefCtx* c, u64* ks_out, const u64* d, uint32_t B, uint32_t nlimbs, const u64* evk,
                  uint32_t galois_elt, uint32_t dnum) {
  (void)galois_elt;
  if (dnum != (uint32_t)c->dnum) return fail("dnum does not match the context");
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq) return fail("bad limb count");
  const size_t N = c->N;
  parallel_for(B, [&](size_t b) { keyswitch_one(c, ks_out + b * 2 * nlimbs * N, d + b * nlimbs * N, nlimbs, evk); });
  return 0;
}

int ref_hrot(const RefCtx* c, u64* ct_out, const u64* ct_in, uint32_t B, uint32_t nlimbs, uint32_t g, const u64* evk) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq) return fail("bad limb count");
  if (!(g & 1) || g >= 2 * c->N) return fail("galois element must be odd and < 2N");
  const size_t sz = (size_t)2 * nlimbs * c->N;
  parallel_for(B, [&](size_t b) { hrot_one(c, ct_out + b * sz, ct_in + b * sz, nlimbs, g, evk); });
  return 0;
}

// (c0,c1)x(c0',c1') -> d0 = c0 c0', d1 = c0 c1' + c1 c0', d2 = c1 c1'; out = (d0 + ks.b, d1 + ks.a), ks = KS(d2).
int ref_hmult_relin(const RefCtx* c, u64* ct_out, const u64* ct_a, const u64* ct_b, uint32_t B, uint32_t nlimbs,
                    const u64* evk) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq) return fail("bad limb count");
  const size_t N = c->N, pl = (size_t)nlimbs * N, sz = 2 * pl;
  parallel_for(B, [&](size_t b) {
    const u64 *a0 = ct_a + b * sz, *a1 = a0 + pl, *b0 = ct_b + b * sz, *b1 = b0 + pl;
    std::vector<u64> d0(pl), d1(pl), d2(pl), ks(sz);
    for (uint32_t i = 0; i < nlimbs; i++) {
      u64 m = c->mod[i];
      for (size_t n = 0; n < N; n++) {
        size_t k = (size_t)i * N + n;
        d0[k] = mulm(a0[k] % m, b0[k] % m, m);
        d1[k] = addm(mulm(a0[k] % m, b1[k] % m, m), mulm(a1[k] % m, b0[k] % m, m), m);
        d2[k] = mulm(a1[k] % m, b1[k] % m, m);
      }
    }
    keyswitch_one(c, ks.data(), d2.data(), nlimbs, evk);
    u64* o = ct_out + b * sz;
    for (uint32_t i = 0; i < nlimbs; i++) {
      u64 m = c->mod[i];
      for (size_t n = 0; n < N; n++) {
        size_t k = (size_t)i * N + n;
        o[k] = addm(d0[k], ks[k], m);
        o[pl + k] = addm(d1[k], ks[pl + k], m);
      }
    }
  });
  return 0;
}

// Late relinearisation (Sec. 5.2): products are kept as three components and summed; one key switch follows the sum.
// d_out[b] = (c0 c0', c0 c1' + c1 c0', c1 c1') (+ d_acc[b] when d_acc is given), each [3][nlimbs][N].
int ref_tensor_acc(const RefCtx* c, u64* d_out, const u64* ct_a, const u64* ct_b, const u64* d_acc, uint32_t B,
                   uint32_t nlimbs) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq) return fail("bad limb count");
  const size_t N = c->N, pl = (size_t)nlimbs * N;
  parallel_for(B, [&](size_t b) {
    const u64 *a0 = ct_a + b * 2 * pl, *a1 = a0 + pl, *b0 = ct_b + b * 2 * pl, *b1 = b0 + pl;
    u64* d = d_out + b * 3 * pl;
    const u64* e = d_acc ? d_acc + b * 3 * pl : nullptr;
    for (uint32_t i = 0; i < nlimbs; i++) {
      u64 m = c->mod[i];
      for (size_t n = 0; n < N; n++) {
        size_t k = (size_t)i * N + n;
        u64 t0 = mulm(a0[k] % m, b0[k] % m, m);
        u64 t1 = addm(mulm(a0[k] % m, b1[k] % m, m), mulm(a1[k] % m, b0[k] % m, m), m);
        u64 t2 = mulm(a1[k] % m, b1[k] % m, m);
        if (e) {
          t0 = addm(t0, e[k] % m, m);
          t1 = addm(t1, e[pl + k] % m, m);
          t2 = addm(t2, e[2 * pl + k] % m, m);
        }
        d[k] = t0;
        d[pl + k] = t1;
        d[2 * pl + k] = t2;
      }
    }
  });
  return 0;
}

// Relinearisation of a three-component ciphertext: out = (d0 + ks.b, d1 + ks.a), ks = KS(d2) under the key for s^2.
int ref_relin(const RefCtx* c, u64* ct_out, const u64* d_in, uint32_t B, uint32_t nlimbs, const u64* evk) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq) return fail("bad limb count");
  const size_t N = c->N, pl = (size_t)nlimbs * N;
  parallel_for(B, [&](size_t b) {
    const u64* d = d_in + b * 3 * pl;
    std::vector<u64> d2(pl), ks(2 * pl);
    for (uint32_t i = 0; i < nlimbs; i++)
      for (size_t n = 0; n < N; n++) d2[(size_t)i * N + n] = d[2 * pl + (size_t)i * N + n] % c->mod[i];
    keyswitch_one(c, ks.data(), d2.data(), nlimbs, evk);
    u64* o = ct_out + b * 2 * pl;
    for (uint32_t i = 0; i < nlimbs; i++) {
      u64 m = c->mod[i];
      for (size_t n = 0; n < N; n++) {
        size_t k = (size_t)i * N + n;
        o[k] = addm(d[k] % m, ks[k], m);
        o[pl + k] = addm(d[pl + k] % m, ks[pl + k], m);
      }
    }
  });
  return 0;
}

// y = sum_{g<n2} rot_{g*n1*stride}( sum_{b<n1} pt[g][b] (.) rot_{b*stride}(x) ); rotation by 0 is the identity (no
// key switch). evk_baby[b-1] switches 5^(b*stride), evk_giant[g-1] switches 5^(g*n1*stride). pt: [n2][n1][nlimbs][N].
int ref_pcmm_bsgs(const RefCtx* c, u64* ct_out, const u64* ct_in, uint32_t B, uint32_t nlimbs, const u64* pt,
                  uint32_t n1, uint32_t n2, uint32_t stride, const u64* const* evk_baby, const u64* const* evk_giant) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq || n1 == 0 || n2 == 0) return fail("bad shape");
  const size_t N = c->N, pl = (size_t)nlimbs * N, sz = 2 * pl;
  const u64 twoN = 2 * N;
  parallel_for(B, [&](size_t bi) {
    const u64* x = ct_in + bi * sz;
    std::vector<std::vector<u64>> baby(n1, std::vector<u64>(sz));
    std::copy(x, x + sz, baby[0].begin());
    for (uint32_t b = 1; b < n1; b++) hrot_one(c, baby[b].data(), x, nlimbs, powm(5, (u64)b * stride, twoN), evk_baby[b - 1]);
    std::vector<u64> y(sz, 0), inner(sz), rot(sz);
    for (uint32_t g = 0; g < n2; g++) {
      std::fill(inner.begin(), inner.end(), 0);
      for (uint32_t b = 0; b < n1; b++) {
        const u64* w = pt + ((size_t)g * n1 + b) * pl;
        for (int comp = 0; comp < 2; comp++)
          for (uint32_t i = 0; i < nlimbs; i++) {
            u64 m = c->mod[i];
            for (size_t n = 0; n < N; n++) {
              size_t k = (size_t)comp * pl + (size_t)i * N + n;
              inner[k] = addm(inner[k], mulm(baby[b][k], w[(size_t)i * N + n] % m, m), m);
            }
          }
      }
      const u64* add = inner.data();
      if (g > 0) {
        hrot_one(c, rot.data(), inner.data(), nlimbs, powm(5, (u64)g * n1 * stride, twoN), evk_giant[g - 1]);
        add = rot.data();
      }
      for (int comp = 0; comp < 2; comp++)
        for (uint32_t i = 0; i < nlimbs; i++) {
          u64 m = c->mod[i];
          for (size_t n = 0; n < N; n++) {
            size_t k = (size_t)comp * pl + (size_t)i * N + n;
            y[k] = addm(y[k], add[k], m);
          }
        }
    }
    std::copy(y.begin(), y.end(), ct_out + bi * sz);
  });
  return 0;
}

// Sum of a ciphertext and R of its rotations with one rounding ("hoisted rotate-and-sum", our extension in the spirit
// of the hoisting of Sec. 5.1): with P = p_0 ... p_{K-1},
//   T = (P c0, P c1) on the q-limbs, 0 on the p-limbs
//     + sum_r [ accumulators of the key switch of sigma_r(c1) under evks[r], plus P sigma_r(c0) on the q-limbs ],
//   out = ModDown(T).
// ModDown(x + P z) = z + ModDown(x) exactly, so out = ct + sum_r sigma_r(c0) + ModDown(sum of the accumulators): the
// rotations' key switches share one ModDown (and, all acting on the same c1, one decomposition).
int ref_hrot_sum(const RefCtx* c, u64* ct_out, const u64* ct_in, uint32_t B, uint32_t nlimbs, const uint32_t* galois,
                 const u64* const* evks, uint32_t R) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq) return fail("bad limb count");
  const size_t N = c->N, pl = (size_t)nlimbs * N, sz = 2 * pl;
  const int K = c->np, next = (int)nlimbs + K;
  const size_t el = (size_t)next * N;
  auto ext_mod = [&](int t) { return c->mod[t < (int)nlimbs ? t : c->nq + (t - (int)nlimbs)]; };
  std::vector<u64> pmod(nlimbs);
  for (uint32_t i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i], v = 1;
    for (int k = 0; k < K; k++) v = mulm(v, c->mod[c->nq + k] % m, m);
    pmod[i] = v;
  }
  parallel_for(B, [&](size_t bi) {
    const u64* x = ct_in + bi * sz;
    std::vector<u64> T(2 * el, 0), r0(pl), r1(pl);
    for (int comp = 0; comp < 2; comp++)
      for (uint32_t i = 0; i < nlimbs; i++)
        for (size_t n = 0; n < N; n++)
          T[(size_t)comp * el + (size_t)i * N + n] = mulm(x[(size_t)comp * pl + (size_t)i * N + n] % c->mod[i], pmod[i], c->mod[i]);
    for (uint32_t r = 0; r < R; r++) {
      for (uint32_t i = 0; i < nlimbs; i++) {
        automorph_eval(c, &r0[(size_t)i * N], x + (size_t)i * N, i, galois[r]);
        automorph_eval(c, &r1[(size_t)i * N], x + pl + (size_t)i * N, i, galois[r]);
      }
      std::vector<u64> A = keyswitch_accumulate(c, r1.data(), nlimbs, evks[r]);
      for (uint32_t i = 0; i < nlimbs; i++)
        for (size_t n = 0; n < N; n++) {
          u64& a = A[(size_t)i * N + n];
          a = addm(a, mulm(r0[(size_t)i * N + n], pmod[i], c->mod[i]), c->mod[i]);
        }
      for (int comp = 0; comp < 2; comp++)
        for (int t = 0; t < next; t++) {
          u64 m = ext_mod(t);
          for (size_t n = 0; n < N; n++) {
            size_t k = (size_t)comp * el + (size_t)t * N + n;
            T[k] = addm(T[k], A[k], m);
          }
        }
    }
    moddown_pair(c, ct_out + bi * sz, T, nlimbs);
  });
  return 0;
}

// BSGS matmul with the baby steps kept in the extended basis ("double hoisting": the hoisting the paper discusses
// in Sec. 5.1 taken one step further; not the paper's own schedule, which rotates one at a time). With
// P = p_0 ... p_{K-1} and the basis q_0..q_{nlimbs-1}, p_0..p_{K-1}:
//   A_0 = (P c0, P c1) on the q-limbs, 0 on the p-limbs;
//   A_r = accumulators of the key switch of sigma_r(c1) under evk_baby[r-1] (before ModDown), with P sigma_r(c0)
//         added to the first one on the q-limbs                                  (r = 1..n1-1, sigma_r = 5^(r*stride));
//   S_g = sum_r pt_ext[g][r] (.) A_r  (both components, every limb of the extended basis);
//   u_g = ModDown(S_g) for g >= 1 (an ordinary ciphertext), rotated by sigma'_g = 5^(g*n1*stride) without leaving
//         the extended basis: G_g = accumulators of the key switch of sigma'_g(u_g.c1) under evk_giant[g-1], with
//         P sigma'_g(u_g.c0) added to the first one on the q-limbs;
//   y   = ModDown( S_0 + sum_{g>=1} G_g ).
// ModDown(x + P z) = z + ModDown(x) exactly, so the c0 terms come out as in the plain schedule; what differs is where
// ModDown rounds: once per giant step on the sum over baby steps, and once at the end on the sum over giant steps.
// pt_ext: [n2][n1][nlimbs+K][N], the plaintext's residues for q_0..q_{nlimbs-1} and then p_0..p_{K-1}, eval domain.
int ref_pcmm_bsgs_double_hoisted(const RefCtx* c, u64* ct_out, const u64* ct_in, uint32_t B, uint32_t nlimbs,
                                 const u64* pt_ext, uint32_t n1, uint32_t n2, uint32_t stride,
                                 const u64* const* evk_baby, const u64* const* evk_giant) {
  if (nlimbs == 0 || nlimbs > (uint32_t)c->nq || n1 == 0 || n2 == 0) return fail("bad shape");
  const size_t N = c->N, pl = (size_t)nlimbs * N, sz = 2 * pl;
  const int K = c->np, next = (int)nlimbs + K;
  const size_t el = (size_t)next * N;   // one component in the extended basis
  const u64 twoN = 2 * N;
  auto ext_mod = [&](int t) { return c->mod[t < (int)nlimbs ? t : c->nq + (t - (int)nlimbs)]; };
  std::vector<u64> pmod(nlimbs);        // P mod q_i
  for (uint32_t i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i], v = 1;
    for (int k = 0; k < K; k++) v = mulm(v, c->mod[c->nq + k] % m, m);
    pmod[i] = v;
  }
  parallel_for(B, [&](size_t bi) {
    const u64* x = ct_in + bi * sz;
    std::vector<std::vector<u64>> A(n1);
    A[0].assign(2 * el, 0);
    for (int comp = 0; comp < 2; comp++)
      for (uint32_t i = 0; i < nlimbs; i++)
        for (size_t n = 0; n < N; n++)
          A[0][(size_t)comp * el + (size_t)i * N + n] = mulm(x[(size_t)comp * pl + (size_t)i * N + n] % c->mod[i], pmod[i], c->mod[i]);
    std::vector<u64> r0(pl), r1(pl);
    for (uint32_t r = 1; r < n1; r++) {
      const u64 g = powm(5, (u64)r * stride, twoN);
      for (uint32_t i = 0; i < nlimbs; i++) {
        automorph_eval(c, &r0[(size_t)i * N], x + (size_t)i * N, i, g);
        automorph_eval(c, &r1[(size_t)i * N], x + pl + (size_t)i * N, i, g);
      }
      A[r] = keyswitch_accumulate(c, r1.data(), nlimbs, evk_baby[r - 1]);
      for (uint32_t i = 0; i < nlimbs; i++)
        for (size_t n = 0; n < N; n++) {
          u64& a = A[r][(size_t)i * N + n];
          a = addm(a, mulm(r0[(size_t)i * N + n], pmod[i], c->mod[i]), c->mod[i]);
        }
    }
    std::vector<u64> T(2 * el, 0), S(2 * el), u(sz);
    for (uint32_t g = 0; g < n2; g++) {
      std::fill(S.begin(), S.end(), 0);
      for (uint32_t r = 0; r < n1; r++) {
        const u64* w = pt_ext + ((size_t)g * n1 + r) * el;
        for (int comp = 0; comp < 2; comp++)
          for (int t = 0; t < next; t++) {
            u64 m = ext_mod(t);
            for (size_t n = 0; n < N; n++) {
              size_t k = (size_t)comp * el + (size_t)t * N + n;
              S[k] = addm(S[k], mulm(A[r][k], w[(size_t)t * N + n] % m, m), m);
            }
          }
      }
      if (g > 0) {
        moddown_pair(c, u.data(), S, nlimbs);
        const u64 gg = powm(5, (u64)g * n1 * stride, twoN);
        for (uint32_t i = 0; i < nlimbs; i++) {
          automorph_eval(c, &r0[(size_t)i * N], &u[(size_t)i * N], i, gg);
          automorph_eval(c, &r1[(size_t)i * N], &u[pl + (size_t)i * N], i, gg);
        }
        S = keyswitch_accumulate(c, r1.data(), nlimbs, evk_giant[g - 1]);
        for (uint32_t i = 0; i < nlimbs; i++)
          for (size_t n = 0; n < N; n++) {
            u64& a = S[(size_t)i * N + n];
            a = addm(a, mulm(r0[(size_t)i * N + n], pmod[i], c->mod[i]), c->mod[i]);
          }
      }
      for (int comp = 0; comp < 2; comp++)
        for (int t = 0; t < next; t++) {
          u64 m = ext_mod(t);
          for (size_t n = 0; n < N; n++) {
            size_t k = (size_t)comp * el + (size_t)t * N + n;
            T[k] = addm(T[k], S[k], m);
          }
        }
    }
    moddown_pair(c, ct_out + bi * sz, T, nlimbs);
  });
  return 0;
}

// Rescale (paper Sec. 2.1: divide by the last modulus and drop it). For each polynomial of ct [B][2][nlimbs][N]
// (eval domain): c_L = INTT(last limb), centred to (-q_L/2, q_L/2]; out_i = NTT((INTT(c_i) - c_L) * q_L^-1 mod q_i)
// for i < nlimbs-1. On the integers this is exactly round(c / q_L).
int ref_rescale(const RefCtx* c, u64* out, const u64* ct, uint32_t B, uint32_t nlimbs) {
  if (nlimbs < 2 || nlimbs > (uint32_t)c->nq) return fail("rescale needs 2..L+1 limbs");
  const size_t N = c->N;
  const uint32_t last = nlimbs - 1;
  const u64 qL = c->mod[last];
  parallel_for((size_t)B * 2, [&](size_t p) {
    std::vector<u64> cl(ct + (p * nlimbs + last) * N, ct + (p * nlimbs + last + 1) * N);
    intt_fast(c, cl.data(), last);
    for (uint32_t i = 0; i < last; i++) {
      const u64 m = c->mod[i], qinv = invm(qL % m, m);
      std::vector<u64> x(ct + (p * nlimbs + i) * N, ct + (p * nlimbs + i + 1) * N);
      intt_fast(c, x.data(), i);
      for (size_t n = 0; n < N; n++) {
        u64 v = cl[n];
        u64 t = v > qL / 2 ? subm(v % m, qL % m, m) : v % m;  // centred representative of c_L, reduced mod q_i
        x[n] = mulm(subm(x[n], t, m), qinv, m);
      }
      ntt_fast(c, x.data(), i);
      std::copy(x.begin(), x.end(), out + (p * last + i) * N);
    }
  });
  return 0;
}

// ---- keys, encryption, decryption (harness side of the semantic pins) ----
// evk[j] = (b_j, a_j) over all nq+np moduli, eval domain: b_j = -a_j*s + e_j + W_j*s_from, where W_j = P mod q_i on the
// limbs of digit j (top level digits of width alpha), 0 on every other modulus.
// a_eval: [dnum][nq+np][N] uniform residues taken as already in the eval domain; e: [dnum][N] signed.
int ref_gen_evk(const RefCtx* c, u64* evk, const i64* s, const i64* s_from, const u64* a_eval, const i64* e) {
  const size_t N = c->N;
  const int nm = c->nq + c->np;
  std::vector<uint32_t> ids(nm);
  for (int i = 0; i < nm; i++) ids[i] = i;
  std::vector<u64> s_hat((size_t)nm * N), sf_hat((size_t)nm * N);
  ref_signed_to_rns(c, s_hat.data(), s, ids.data(), nm);
  ref_signed_to_rns(c, sf_hat.data(), s_from, ids.data(), nm);
  for (int i = 0; i < nm; i++) { ntt_fast(c, &s_hat[(size_t)i * N], i); ntt_fast(c, &sf_hat[(size_t)i * N], i); }
  for (int j = 0; j < c->dnum; j++) {
    std::vector<u64> e_hat((size_t)nm * N);
    ref_signed_to_rns(c, e_hat.data(), e + (size_t)j * N, ids.data(), nm);
    for (int i = 0; i < nm; i++) {
      u64 m = c->mod[i];
      ntt_fast(c, &e_hat[(size_t)i * N], i);
      u64 w = 0;
      if (i < c->nq && i / c->alpha == j) {
        w = 1;
        for (int k = 0; k < c->np; k++) w = mulm(w, c->mod[c->nq + k] % m, m);
      }
      const u64* a = a_eval + ((size_t)j * nm + i) * N;
      u64* ob = evk + (((size_t)j * 2 + 0) * nm + i) * N;
      u64* oa = evk + (((size_t)j * 2 + 1) * nm + i) * N;
      for (size_t n = 0; n < N; n++) {
        size_t k = (size_t)i * N + n;
        u64 as = mulm(a[n] % m, s_hat[k], m);
        u64 v = addm(subm(e_hat[k], as, m), mulm(w, sf_hat[k], m), m);
        ob[n] = v;
        oa[n] = a[n] % m;
      }
    }
  }
  return 0;
}

// ct = (-a*s + e + msg, a), eval domain, limbs q_0..q_{nlimbs-1}. a_eval: [nlimbs][N]; msg, e signed coefficients.
int ref_encrypt(const RefCtx* c, u64* ct, const i64* msg, const i64* s, const u64* a_eval, const i64* e, uint32_t nlimbs) {
  const size_t N = c->N;
  std::vector<i64> me(N);
  for (size_t n = 0; n < N; n++) me[n] = msg[n] + e[n];
  for (uint32_t i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i];
    std::vector<u64> sh(N), mh(N);
    uint32_t id = i;
    ref_signed_to_rns(c, sh.data(), s, &id, 1);
    ref_signed_to_rns(c, mh.data(), me.data(), &id, 1);
    ntt_fast(c, sh.data(), i);
    ntt_fast(c, mh.data(), i);
    for (size_t n = 0; n < N; n++) {
      u64 a = a_eval[(size_t)i * N + n] % m;
      ct[(size_t)i * N + n] = subm(mh[n], mulm(a, sh[n], m), m);
      ct[((size_t)nlimbs + i) * N + n] = a;
    }
  }
  return 0;
}

// out[nlimbs][N] = coefficient-domain residues of c0 + c1*s (+ c2*s^2 when ncomp == 3).
int ref_decrypt_rns(const RefCtx* c, u64* out, const u64* ct, const i64* s, uint32_t nlimbs, uint32_t ncomp) {
  const size_t N = c->N;
  for (uint32_t i = 0; i < nlimbs; i++) {
    u64 m = c->mod[i];
    std::vector<u64> sh(N);
    uint32_t id = i;
    ref_signed_to_rns(c, sh.data(), s, &id, 1);
    ntt_fast(c, sh.data(), i);
    u64* o = out + (size_t)i * N;
    for (size_t n = 0; n < N; n++) {
      u64 acc = ct[(size_t)i * N + n] % m, sp = sh[n];
      for (uint32_t k = 1; k < ncomp; k++) {
        acc = addm(acc, mulm(ct[((size_t)k * nlimbs + i) * N + n] % m, sp, m), m);
        sp = mulm(sp, sh[n], m);
      }
      o[n] = acc;
    }
    intt_fast(c, o, i);
  }
  return 0;
}

}  // extern "C"
