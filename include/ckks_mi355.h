/*
 * ckks_mi355 - batched RNS-CKKS polynomial arithmetic on one AMD Instinct MI355X (gfx950).
 *
 * C ABI of the hot path under encrypted Transformer inference: per-limb negacyclic
 * NTT/INTT, Galois automorphism, hybrid key switching (ModUp to the P-extended basis,
 * inner product with the evaluation key, ModDown), and on top of those HRot,
 * HMult+relinearize and the diagonal BSGS ciphertext-plaintext matmul.
 *
 * Conventions common to all calls
 * -------------------------------
 * Ring: Z_q[x]/(x^N+1), N = 2^logN (paper Sec. 2.1). Coefficients are held in RNS form
 * over the main primes q_0..q_L and, during key switching only, the special primes
 * p_0..p_{K-1} (paper Sec. 2.1, last paragraph; Sec. 2.2). A "modulus id" indexes the
 * list q_0..q_L, p_0..p_{K-1} given at context creation.
 *
 * Layout: RNS-major (paper Sec. 2.2): uint64 tensors with the N residues of one modulus
 * contiguous. Polynomial batches are [npoly][nlimbs][N]; ciphertext batches are
 * [B][2][nlimbs][N] holding (c0, c1) with Dec = c0 + c1*s; a ciphertext at nlimbs limbs
 * uses moduli q_0..q_{nlimbs-1}. Evaluation keys are [dnum][2][L+1+K][N] with row 0 = b,
 * row 1 = a, over ALL moduli of the context (q rows first, then p rows).
 *
 * Domain: the "evaluation domain" is the output order of ckks_ntt: index k holds the
 * polynomial's value at psi^(2*bitrev_logN(k)+1). Ciphertexts, keys and pre-encoded
 * plaintexts cross this ABI in the evaluation domain. Every residue crossing the ABI
 * must be canonical (in [0, modulus)) and every output is canonical.
 *
 * Pointers: arguments documented "device" are device addresses on the context's GPU and
 * are owned by the caller (the library never frees or reallocates them); arguments
 * documented "host" are ordinary host pointers read before the call returns. The
 * library owns only the context and its constant tables.
 *
 * Streams: every call enqueues its kernels on `stream` (a hipStream_t passed as void*;
 * NULL = the default stream) and returns without synchronising or allocating: every table a
 * call needs is built by ckks_ctx_create. With tuning knob 4 set to 0 a key switch runs part of its
 * kernels on a second stream owned by the context, forked from and joined back into `stream` with
 * events, so everything is ordered as if it ran on `stream` alone. Calls on one context must not be
 * issued from several host threads at once. Workspace passed to a call must stay untouched until that
 * stream has drained the call. One host thread may keep calls of one context in flight on several
 * streams, each with a workspace of its own (the context holds only constants once it is created),
 * as long as knob 4 keeps its default, profiling is off and none of them is ckks_hrot_noalloc, whose
 * calls share one scratch array per GPU.
 *
 * Errors: calls return CKKS_OK or a negative code; they never throw or abort. After a
 * failure ckks_last_error() returns a thread-local message. Nothing is enqueued when an
 * argument check fails.
 */
#ifndef CKKS_MI355_H
#define CKKS_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CKKS_OK 0
#define CKKS_EINVAL (-1)     /* null pointer, bad modulus, even Galois element, ... */
#define CKKS_ESHAPE (-2)     /* limb count / batch / digit count outside what the context supports */
#define CKKS_EWORKSPACE (-3) /* workspace pointer null, misaligned or smaller than ckks_workspace_bytes() */
#define CKKS_EHIP (-4)       /* a HIP runtime call failed; message holds hipGetErrorString */

#define CKKS_OP_KEYSWITCH 1
#define CKKS_OP_HROT 2
#define CKKS_OP_HMULT_RELIN 3
#define CKKS_OP_PCMM_BSGS 4
#define CKKS_OP_RESCALE 5
#define CKKS_OP_PCMM_BSGS_DH 6
#define CKKS_OP_HROT_SUM 7

typedef struct ckks_ctx ckks_ctx;

/* Thread-local description of the last failure on this thread ("" if none). */
const char* ckks_last_error(void);

/*
 * Create a context on GPU `device` for ring degree 2^logN (10 <= logN <= 17), main primes
 * q[0..nq) (the top level, L+1 = nq), special primes p[0..np), and digit count dnum
 * (digit width alpha = ceil(nq/dnum) limbs; paper Sec. 2.1, last paragraph: the special primes serve the digit
 * decomposition of key switching). psi[i] is a primitive 2N-th root of unity modulo the i-th modulus
 * (q first, then p). All three arrays are host pointers. Every modulus must be a distinct
 * prime < 2^60 congruent to 1 mod 2N, and psi[i]^N must be -1; otherwise CKKS_EINVAL.
 * Builds twiddle tables and base-conversion constants in device memory owned by the context.
 */
int ckks_ctx_create(ckks_ctx** ctx, uint32_t logN, const uint64_t* q, uint32_t nq, const uint64_t* p, uint32_t np,
                    uint32_t dnum, const uint64_t* psi, int device);
int ckks_ctx_destroy(ckks_ctx* ctx);

/*
 * Bytes of device workspace that `op` (CKKS_OP_*) needs for a batch of `batch`
 * ciphertexts at `nlimbs` limbs; n1 is the baby-step count for CKKS_OP_PCMM_BSGS and
 * CKKS_OP_PCMM_BSGS_DH and is ignored otherwise. Returns 0 on a bad argument. Workspace must be
 * 256-byte aligned.
 */
size_t ckks_workspace_bytes(const ckks_ctx* ctx, int op, uint32_t batch, uint32_t nlimbs, uint32_t n1);

/*
 * Forward / inverse negacyclic NTT of every limb-vector of data[npoly][nlimbs][N]
 * (device, in place). Limb slot l uses modulus id limb_ids[l] (host array of nlimbs ids).
 * Forward: coefficient order in, evaluation order (see above) out. Inverse is its exact
 * inverse, including the 1/N factor (paper Sec. 3.2.1: NTT/INTT couple all coefficients
 * within one modulus).
 */
int ckks_ntt(ckks_ctx* ctx, uint64_t* data, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs, void* stream);
int ckks_intt(ckks_ctx* ctx, uint64_t* data, uint32_t npoly, const uint32_t* limb_ids, uint32_t nlimbs, void* stream);

/*
 * Galois automorphism a(X) -> a(X^galois_elt) on in[npoly][nlimbs][N] -> out (device, out
 * must not overlap in). galois_elt must be odd and < 2N. eval_domain != 0: operands are
 * in the evaluation domain (a pure index permutation); eval_domain == 0: coefficient
 * domain (permutation with sign flips). Paper Sec. 3.2.1 (automorphisms, intra-prime
 * coupling); Sec. 2.1 (Rot).
 */
int ckks_automorph(ckks_ctx* ctx, uint64_t* out, const uint64_t* in, uint32_t npoly, const uint32_t* limb_ids,
                   uint32_t nlimbs, uint32_t galois_elt, int eval_domain, void* stream);

/*
 * Hybrid key switch (paper Sec. 2.1: extend to Z_{Q*P}, multiply by the key, reduce back
 * to Z_Q; Sec. 3.2.1: ModUp computes new residues from all residues of a digit).
 *   d      device [B][nlimbs][N], evaluation domain, moduli q_0..q_{nlimbs-1}
 *   evk    device [dnum][2][L+1+K][N]
 *   ks_out device [B][2][nlimbs][N]: ks_out[.,0] + ks_out[.,1]*s = d*s_from + small error
 * The digits are groups of alpha consecutive limbs; at nlimbs < L+1 only the first
 * ceil(nlimbs/alpha) digits exist and the last may be short. Base conversion uses the
 * centred representative. galois_elt is informational (the permutation is NOT applied
 * here); dnum must equal the context's. ks_out must not overlap d.
 */
int ckks_keyswitch(ckks_ctx* ctx, uint64_t* ks_out, const uint64_t* d, uint32_t B, uint32_t nlimbs,
                   const uint64_t* evk, uint32_t galois_elt, uint32_t dnum, void* ws, size_t ws_bytes, void* stream);

/*
 * HRot: ct_out = (sigma_g(c0) + ks.b, ks.a) with ks = keyswitch(sigma_g(c1), evk_rot),
 * g = galois_elt; one (g, key) pair for the whole batch (paper Sec. 2.1: Rot shifts the
 * slots cyclically; g = 5^k mod 2N rotates left by k). ct_in, ct_out: device
 * [B][2][nlimbs][N], must not overlap.
 */
int ckks_hrot(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
              uint32_t galois_elt, const uint64_t* evk_rot, void* ws, size_t ws_bytes, void* stream);

/*
 * HRot for callers that cannot allocate device memory: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc. Same operation, arguments, overlap rules and result as ckks_hrot, but without a
 * workspace argument: the kernels use a fixed array of ckks_noalloc_scratch_bytes() bytes (128 MiB) that lives in
 * the library's device image, one copy per GPU, held until the process ends. The call makes no hipMalloc/hipFree
 * and calls no allocating library routine. A batch whose CKKS_OP_HROT workspace would exceed the array is rejected
 * with CKKS_EWORKSPACE (at N = 2^16, 24 limbs, K = 8, dnum = 3 exactly one ciphertext fits); so is a call while
 * per-kernel timing is enabled (CKKS_EINVAL), because timing creates events. All calls on one GPU share that GPU's
 * array, from every context and every stream: calls that may overlap in time on one GPU race on it, so keep them on
 * one stream or order them with events. Nothing in the array has to be cleared between calls (each region is written
 * before it is read within a call); its contents after a call are unspecified.
 */
size_t ckks_noalloc_scratch_bytes(void);
int ckks_hrot_noalloc(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                      uint32_t galois_elt, const uint64_t* evk_rot, void* stream);

/*
 * Rotate-and-add (the step of the rotate-and-sum reductions and of the rotate-multiply-accumulate loops of the
 * attention and linear layers, paper Sec. 4.2-4.3): ct_out = ct_add + HRot_{galois_elt}(ct_in), with the addition
 * done where the rotation's result is assembled instead of in a pass of its own. ct_add is a device ciphertext
 * batch like ct_in; it may be ct_in (rotate-and-sum) or, at N = 2^16, ct_out itself (accumulate in place);
 * otherwise it must not overlap ct_out. Everything else as for ckks_hrot.
 */
int ckks_hrot_add(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, const uint64_t* ct_add, uint32_t B,
                  uint32_t nlimbs, uint32_t galois_elt, const uint64_t* evk_rot, void* ws, size_t ws_bytes, void* stream);

/*
 * HRot with a Galois element and a rotation key per ciphertext (the batch of the key-switch micro-benchmark is
 * rotated "by seeded Galois elements"; same definition as ckks_hrot, Sec. 2.1 Rot): ct_out[b] =
 * HRot_{galois_elts[b]}(ct_in[b]) with evks[b], i.e. exactly what B calls of ckks_hrot with B = 1 return, but
 * in one launch sequence over the whole batch. galois_elts: HOST array of B odd elements < 2N; evks: HOST array
 * of B device pointers, each laid out like evk_rot of ckks_hrot (pointers may repeat). Buffers, workspace
 * (CKKS_OP_HROT for this B), stream and error behaviour as for ckks_hrot.
 */
int ckks_hrot_multi(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                    const uint32_t* galois_elts, const uint64_t* const* evks, void* ws, size_t ws_bytes, void* stream);

/*
 * HMult + relinearize (paper Sec. 2.1: CMult, Relin): with ct_a = (a0,a1), ct_b = (b0,b1):
 * d0 = a0*b0, d1 = a0*b1 + a1*b0, d2 = a1*b1 (pointwise per limb), ks = keyswitch(d2,
 * evk_mult), ct_out = (d0 + ks.b, d1 + ks.a). No rescale: the output scale is the product
 * of the input scales. ct_out may alias neither input.
 */
int ckks_hmult_relin(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_a, const uint64_t* ct_b, uint32_t B,
                     uint32_t nlimbs, const uint64_t* evk_mult, void* ws, size_t ws_bytes, void* stream);

/*
 * Late relinearisation (paper Sec. 5.2, an optimisation applied to every system compared there): products are kept
 * as three components, summed, and key-switched once. ckks_tensor_acc computes, pointwise per limb,
 *   d_out[b] = (a0*b0, a0*b1 + a1*b0, a1*b1) + d_acc[b]      (d_acc == NULL: no addend)
 * d_out, d_acc: device [B][3][nlimbs][N], canonical residues; d_acc may be d_out itself (accumulate in place) but
 * may not overlap it otherwise; d_out may overlap neither input ciphertext. No workspace. Errors as for ckks_add.
 */
int ckks_tensor_acc(ckks_ctx* ctx, uint64_t* d_out, const uint64_t* ct_a, const uint64_t* ct_b, const uint64_t* d_acc,
                    uint32_t B, uint32_t nlimbs, void* stream);

/*
 * Relinearisation of three-component ciphertexts (paper Sec. 2.1: Relin; Sec. 5.2: late relinearisation):
 *   ks = keyswitch(d2, evk_mult), ct_out[b] = (d0 + ks.b, d1 + ks.a).
 * ckks_relin(ckks_tensor_acc(a, b, NULL)) returns exactly what ckks_hmult_relin(a, b) returns. d_in: device
 * [B][3][nlimbs][N]; ct_out: device [B][2][nlimbs][N], may not overlap d_in. Workspace: CKKS_OP_KEYSWITCH for
 * this B and nlimbs. Key layout, stream and error behaviour as for ckks_hmult_relin.
 */
int ckks_relin(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* d_in, uint32_t B, uint32_t nlimbs,
               const uint64_t* evk_mult, void* ws, size_t ws_bytes, void* stream);

/*
 * Diagonal baby-step/giant-step ciphertext-plaintext matmul, one rotation at a time, no
 * hoisting (paper Sec. 5.1 "Implementation"; Sec. 3.2.2 BSGS matmul):
 *   ct_out = sum_{g<n2} rot_{g*n1*stride}( sum_{b<n1} pt_diag[g][b] (.) rot_{b*stride}(ct_in) )
 * where rot_r is HRot with Galois element 5^r mod 2N and rot_0 is the identity.
 *   pt_diag   device [n2][n1][nlimbs][N], evaluation domain, shared by the whole batch
 *   evk_baby  host array of n1-1 device pointers; evk_baby[b-1] switches 5^(b*stride)
 *   evk_giant host array of n2-1 device pointers; evk_giant[g-1] switches 5^(g*n1*stride)
 * ct_in, ct_out: device [B][2][nlimbs][N], must not overlap. Output scale = input scale
 * times the plaintext scale (no rescale).
 */
int ckks_pcmm_bsgs(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                   const uint64_t* pt_diag, uint32_t n1, uint32_t n2, uint32_t stride,
                   const uint64_t* const* evk_baby, const uint64_t* const* evk_giant, void* ws, size_t ws_bytes,
                   void* stream);

/*
 * Hoisted variants (paper Sec. 5.1 names hoisting as the alternative it switches off by default to save memory on
 * 48 GB GPUs): ckks_hrot_hoisted rotates the SAME batch by R Galois elements, ct_out[r] = HRot_{galois_elts[r]}(ct_in)
 * with key evks[r] (galois_elts, evks: host arrays of R entries; ct_out device [R][B][2][nlimbs][N]), sharing the
 * inverse transform, ModUp and forward transform of c1 among the rotations. ckks_pcmm_bsgs_hoisted is
 * ckks_pcmm_bsgs with its baby steps computed that way. Results are bit-identical to the one-at-a-time calls
 * (the Galois map commutes exactly with the centred base conversion); workspace sizes are those of
 * CKKS_OP_HROT and CKKS_OP_PCMM_BSGS. At N = 2^16 ckks_hrot_hoisted uses whatever the workspace holds beyond that
 * size: every further B*2*(nlimbs+K)*N*8 bytes let one more rotation share a pass over the transformed digits
 * (up to 64 per pass), which saves reading them once per rotation.
 */
int ckks_hrot_hoisted(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                      const uint32_t* galois_elts, const uint64_t* const* evks, uint32_t R, void* ws, size_t ws_bytes,
                      void* stream);
int ckks_pcmm_bsgs_hoisted(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                           const uint64_t* pt_diag, uint32_t n1, uint32_t n2, uint32_t stride,
                           const uint64_t* const* evk_baby, const uint64_t* const* evk_giant, void* ws, size_t ws_bytes,
                           void* stream);

/*
 * BSGS matmul with baby and giant steps kept in the extended basis ("double hoisting"): hoisting as discussed in
 * the paper's Sec. 5.1, taken further; not the paper's own schedule and NOT bit-identical to ckks_pcmm_bsgs.
 * With P the product of the special primes:
 *   A_0 = (P*c0, P*c1) on the main primes, 0 on the special primes;
 *   A_r = the key-switch accumulators of sigma_r(c1) under evk_baby[r-1] before ModDown, plus P*sigma_r(c0) on the
 *         main primes of the first one (r = 1..n1-1, sigma_r = 5^(r*stride));
 *   S_g = sum_r pt_ext[g][r] (.) A_r over all nlimbs + K limbs;
 *   u_g = ModDown(S_g) for g >= 1, and G_g = the accumulators of the key switch of sigma'_g(u_g.c1) under
 *         evk_giant[g-1] plus P*sigma'_g(u_g.c0) as above (sigma'_g = 5^(g*n1*stride));
 *   ct_out = ModDown(S_0 + sum_{g>=1} G_g).
 * ModDown(x + P*z) = z + ModDown(x) exactly, so only the placement of ModDown's rounding differs from the plain
 * schedule: n2 ModDowns per ciphertext instead of n1 + n2 - 2, and baby steps that cost one inner product each.
 *   pt_ext  device [n2][n1][nlimbs + K][N]: the plaintexts' residues for q_0..q_{nlimbs-1}, then p_0..p_{K-1},
 *           evaluation domain
 * N = 2^16 only (CKKS_ESHAPE otherwise). Workspace: CKKS_OP_PCMM_BSGS_DH with n1 (n1 + 25 ciphertexts in the
 * extended basis). Other arguments, overlap rules and errors as for ckks_pcmm_bsgs.
 */
int ckks_pcmm_bsgs_double_hoisted(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                                  const uint64_t* pt_ext, uint32_t n1, uint32_t n2, uint32_t stride,
                                  const uint64_t* const* evk_baby, const uint64_t* const* evk_giant, void* ws,
                                  size_t ws_bytes, void* stream);

/*
 * Hoisted rotate-and-sum (an extension in the spirit of the hoisting of the paper's Sec. 5.1; the rotate-and-sum of
 * Sec. 4.3's score slices in fewer roundings): ct_out[b] = ct_in[b] + sum_{r<R} HRot_{galois_elts[r]}(ct_in[b]) with
 * ONE ModDown for all rotations. With P the product of the special primes,
 *   T = (P*c0, P*c1) + sum_r [ key-switch accumulators of sigma_r(c1) under evks[r], plus P*sigma_r(c0) ],
 *   ct_out = ModDown(T).
 * ModDown(x + P*z) = z + ModDown(x) exactly; for R = 1 the result is bit-identical to ct_in + ckks_hrot(ct_in), for
 * R > 1 it differs from R separate rotations in the rounding only. All rotations share one decomposition of c1.
 * galois_elts, evks: HOST arrays of R entries (R = 0 copies the input through ModDown(P*ct) = ct). ct_out may not
 * overlap ct_in. N = 2^16 only (CKKS_ESHAPE otherwise). Workspace: CKKS_OP_HROT_SUM. Errors as for ckks_hrot.
 */
int ckks_hrot_sum(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs,
                  const uint32_t* galois_elts, const uint64_t* const* evks, uint32_t R, void* ws, size_t ws_bytes,
                  void* stream);

/*
 * Rescale (paper Sec. 2.1: division by the last modulus of the chain, which lowers the scale and drops that prime): for
 * ct_in [B][2][nlimbs][N] (device, evaluation domain, nlimbs >= 2) writes ct_out [B][2][nlimbs-1][N] with
 * every coefficient c replaced by round(c / q_{nlimbs-1}) (centred representatives, exact). ct_out must not
 * overlap ct_in.
 */
int ckks_rescale(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, uint32_t B, uint32_t nlimbs, void* ws,
                 size_t ws_bytes, void* stream);

/*
 * PMult (paper Sec. 2.1): ct_out[b][c][i] = ct_in[b][c][i] (.) pt[i], pt device [nlimbs][N], evaluation domain,
 * pre-encoded (Sec. 2.4). May run in place (ct_out == ct_in).
 * CAdd / PAdd building block: out = a + b on device tensors [npoly][nlimbs][N]. May run in place.
 */
int ckks_pmult(ckks_ctx* ctx, uint64_t* ct_out, const uint64_t* ct_in, const uint64_t* pt, uint32_t B, uint32_t nlimbs,
               void* stream);
int ckks_add(ckks_ctx* ctx, uint64_t* out, const uint64_t* a, const uint64_t* b, uint32_t npoly, uint32_t nlimbs,
             void* stream);

/*
 * Measurement support (not part of the paper's operator set). While enabled, every kernel
 * launch the library makes is bracketed by two HIP events on the stream it is launched on;
 * ckks_prof_collect() waits for the recorded events and adds their elapsed times to
 * per-kernel-kind totals, which ckks_prof_read() returns (total milliseconds and number of
 * launches). Kinds are 0..ckks_prof_num_kinds()-1 with names from ckks_prof_kind_name().
 * Not thread-safe: use one thread per context while profiling.
 */
int ckks_prof_enable(ckks_ctx* ctx, int on);
/* Calibration of hardware byte counters: a plain copy kernel (ckks_prof_copy_kernel) that reads `bytes` from src and
 * writes them to dst (device pointers, multiples of 16 bytes, not overlapping) and nothing else. */
int ckks_prof_copy(ckks_ctx* ctx, void* dst, const void* src, size_t bytes, void* stream);
/* Tuning knobs for experiments (defaults in brackets):
 * knob 0 [-1] workgroup-to-tile mapping of the N = 2^16 kernels: 0..4 forces one mapping everywhere, -1 chooses per kernel;
 * knob 1 [0]  != 0 turns the double-precision bodies for primes < 2^50 off (integer bodies everywhere);
 * knob 2 [0]  1 = the base conversions of ModUp and ModDown run inside the following row pass (one kernel each)
 *             instead of a conversion kernel followed by a row pass; measured slower, kept for the measurement;
 * knob 3 [2]  inner product on double-precision main limbs: 2 = block pass of the digits, product with one key
 *             component, block pass of the ModDown correction and final assembly in one kernel; 1 = plain block
 *             pass, streaming product and a separate assembly kernel;
 * knob 4 [1]  0 lets a key switch run the double-precision row pass of the converted digits on a second stream
 *             owned by the context, beside the special-prime chain, joined before the result is assembled;
 * knob 5 [0]  != 0 makes every base conversion use the general four-sum accumulation with a 128-bit Montgomery
 *             reduction, also where the bit sizes of the bases allow the shorter three-sum form;
 * knob 6 [0]  != 0 computes the inner sums of ckks_pcmm_bsgs with the integer kernel on every limb;
 * knob 7 [0]  > 0 caps the number of giant steps whose inner sums one pass over the baby-step ciphertexts
 *             computes (default and maximum 24).
 * Knobs 1 and 5 rebuild the context's constant tables: the call waits for the device and reallocates them. */
int ckks_tune_set(ckks_ctx* ctx, int knob, int value);
int ckks_prof_num_kinds(void);
const char* ckks_prof_kind_name(int kind);
int ckks_prof_collect(ckks_ctx* ctx);
int ckks_prof_read(ckks_ctx* ctx, int kind, double* total_ms, uint64_t* launches);
int ckks_prof_reset(ckks_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* CKKS_MI355_H */
