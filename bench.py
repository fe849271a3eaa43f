#!/usr/bin/env python3
"""Benchmark of the RNS-CKKS key-switching hot path on one MI355X.

Workload ("keyswitch_micro"): N = 2^16, 24 main primes of 50 bits, 8 special primes of 60
bits, dnum = 3; 64 ciphertexts with uniform residues and seeded uniform evaluation keys.
One step = HRot of all 64 ciphertexts, each by its own seeded Galois element with its own
key (`--groups 64`, one batched ckks_hrot_multi call; `--groups G --hrot-call grouped` shares
an element and key inside each of G groups and makes one ckks_hrot call per group), followed
by HMult+relinearize of 32 ciphertext pairs (one call): 96 key switches. Inputs are resident
in HBM before the timed region.

Prints ONE JSON line: whole-job key switches per second, the roofline figures of the kernel
kind that dominates the timed region (HIP-event durations of every launch, taken by the
library on the launch stream), and the CPU oracle timed on a bounded sample of the same work.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_ALU_TOPS = 256 * 64 * 2.4e9 / 1e12  # 256 CUs x 64 lanes x 2.4 GHz = 39.3 T 32-bit lane-ops/s

# Algorithmic 32-bit lane-op counts: one 64-bit Shoup butterfly = 10 multiply-class
# + 14 add/compare/select ops (the canonical form; the kernels' butterflies execute 21 instructions with their
# approximate quotient, so fractions built on these counts read a little high against executed instructions, which
# profiles/ reports from counters); one 64x64->128 multiply-accumulate = 4 multiplies + 4 adds; one 128->64
# Montgomery reduction = 7 multiplies + 9 adds/selects; one Shoup constant multiply = 10 + 4.
OPS_BUTTERFLY, OPS_MAC, OPS_REDUCE, OPS_SHOUP, OPS_ADD = 24, 8, 16, 14, 4
# Double-precision bodies (primes < 2^50; FP64 instructions issue at the same one-per-lane-per-clock rate):
# butterfly = 6 (exact product, quotient, remainder) + 2 (add, sub) + 1.5 (range reduction every 4 stages);
# variable x variable product reduced = 7; constant multiply = 6.
OPS_BUTTERFLY_FP, OPS_MULRED_FP, OPS_SHOUP_FP = 9.5, 7, 6
# Base-conversion dot product on 30-bit operand halves: 4 multiply-adds per term, and per output a base-2^30
# Montgomery reduction of the three sums (22) plus the final correction (5).
OPS_DOT30, OPS_REDUCE90 = 4, 27


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "keyswitch_micro_traffic.json")


def measured_traffic():
    """HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs on this workload in its default
    configuration, as written by paper_2604_03425_amd/profile_summary.py into profiles/ together with the digest of
    the sources they were taken on. Returns {} when that digest is not the one of the sources in this tree (the
    counters then describe other kernels and the line reports traffic: null)."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return {}
    from paper_2604_03425_amd.srcdigest import source_digest
    if rec.get("source_sha256") != source_digest():
        return {}
    return {k: int(v) for k, v in rec.get("hbm_bytes_per_launch", {}).items()}


def keyswitch_model(p, B, nl, hrot, hmult, fp_inner=2, bconv_fused=False):
    """Algorithmic bytes and lane-ops per kernel kind for ONE key-switch call on a batch of B (N = 2^16 path:
    double-precision bodies on primes < 2^50, with their inner product as a separate streaming kernel)."""
    N, K, alpha = p.N, len(p.p), p.alpha
    nxt, beta = nl + K, p.beta(nl)
    ext_mod = list(p.q[:nl]) + list(p.p)
    fp = [m < (1 << 50) for m in ext_mod]
    digits = [range(j * alpha, min(nl, (j + 1) * alpha)) for j in range(beta)]
    new_fp = sum(1 for dg in digits for t in range(nxt) if t not in dg and fp[t])      # converted limbs per ciphertext
    new_int = sum(1 for dg in digits for t in range(nxt) if t not in dg and not fp[t])
    own_fp = sum(1 for t in range(nl) if fp[t])
    own_int = nl - own_fp
    n_fp, n_int = sum(fp), nxt - sum(fp)
    new_limbs = new_fp + new_int
    limb = 8 * N
    bf_pass = (N / 2) * 8 * OPS_BUTTERFLY          # one 8-stage pass over one limb, integer bodies
    bf_pass_fp = (N / 2) * 8 * OPS_BUTTERFLY_FP    # same, double-precision bodies
    mul_redc = 2 * OPS_MAC + OPS_REDUCE            # one variable x variable product reduced
    m = {}
    kfp = sum(1 for x in p.p if x < (1 << 50))
    inv_fp, inv_int = B * (own_fp + 2 * kfp), B * (own_int + 2 * (K - kfp))

    def put(name, cls, nbytes, nops):
        if nbytes or nops:
            m["%s<%d>" % (name, cls) if cls is not None else name] = dict(bytes=nbytes, ops=nops)
    # class 0 = double-precision bodies; the 60-bit special primes are class 2 (Harvey integer bodies)
    put("ntt16_inv_blocks_kernel", 0, inv_fp * 2 * limb, inv_fp * bf_pass_fp)
    put("ntt16_inv_blocks_kernel", 2, inv_int * 2 * limb, inv_int * bf_pass)
    put("ntt16_inv_rows_kernel", 0, inv_fp * 2 * limb, inv_fp * (bf_pass_fp + N * OPS_SHOUP_FP))
    put("ntt16_inv_rows_kernel", 2, inv_int * 2 * limb, inv_int * (bf_pass + N * OPS_SHOUP))
    fp_main = [t for t in range(nl) if fp[t]]
    fp_t, int_t = [t for t in range(nxt) if fp[t]], [t for t in range(nxt) if not fp[t]]
    dn_fp, dn_int = 2 * own_fp, 2 * own_int     # ModDown targets per ciphertext
    if not bconv_fused:
        # base conversion, as executed: 4 multiply-adds per term on 30-bit halves + a 27-instruction reduction per output
        put("modup_kernel", None, B * (nl + new_limbs) * limb,
            B * N * sum((nxt - len(dg)) * ((len(dg) + 1) * OPS_DOT30 + OPS_REDUCE90) for dg in digits))
        put("moddown_kernel", None, 2 * B * (K + nl) * limb, 2 * B * N * nl * ((K + 1) * OPS_DOT30 + OPS_REDUCE90))
        rows_fp, rows_int = B * (new_fp + dn_fp), B * (new_int + dn_int)
        put("ntt16_fwd_rows_kernel", 0, rows_fp * 2 * limb, rows_fp * bf_pass_fp)
        put("ntt16_fwd_rows_kernel", 2, rows_int * 2 * limb, rows_int * bf_pass)
    else:
        # Knob 2 = 1: base conversion inside the first forward pass: 4 multiply-adds per term and a 27-instruction
        # reduction per output, then 8 butterfly stages. HBM bytes if every source tile is fetched once per
        # (polynomial, tile) group and the other targets of the group find it in L2.
        up_ops = lambda targets: sum(sum(1 for t in targets if t not in dg) * (len(dg) * OPS_DOT30 + OPS_REDUCE90) for dg in digits)
        dn_term = K * OPS_DOT30 + OPS_REDUCE90
        put("ntt16_bconv_rows_kernel", 0, B * ((nl if new_fp else 0) + new_fp + (2 * K if dn_fp else 0) + dn_fp) * limb,
            B * (N * (up_ops(fp_t) + dn_fp * dn_term) + (new_fp + dn_fp) * bf_pass_fp))
        put("ntt16_bconv_rows_kernel", 2, B * ((nl if new_int else 0) + new_int + (2 * K if dn_int else 0) + dn_int) * limb,
            B * (N * (up_ops(int_t) + dn_int * dn_term) + (new_int + dn_int) * bf_pass))
    addend = 1 if hrot else 2 if hmult else 0
    if fp_inner != 1:
        # default on double-precision main limbs: block pass of the digits fused with one key component per workgroup
        # (every converted tile is transformed by both workgroups of its ciphertext: twice in ops, once in bytes, the
        # second read being served by L2), then the block pass of the ModDown correction, the division by P and the
        # addends in the same kernel. Special limbs below 2^50 (none in the benchmark) keep the store of the sums.
        put("ntt16_fwd_blocks_inner_c_kernel", None,
            (B * (new_fp + own_fp + 2 * kfp + (2 + addend + 2) * own_fp) + 2 * beta * n_fp) * limb,
            B * (2 * new_fp * bf_pass_fp + N * n_fp * beta * 2 * OPS_MULRED_FP) +
            2 * B * own_fp * (bf_pass_fp + N * (OPS_SHOUP_FP + 2)))
    else:
        # plain block pass, streaming product and a separate assembly kernel
        put("ntt16_fwd_blocks_kernel", 0, B * new_fp * 2 * limb, B * new_fp * bf_pass_fp)
        put("inner16_fp_kernel", None, (B * (new_fp + own_fp + 2 * n_fp) + 2 * beta * n_fp) * limb,
            B * N * n_fp * beta * 2 * OPS_MULRED_FP)
        put("ntt16_fwd_blocks_final_kernel", 0, B * own_fp * (6 + addend) * limb,
            2 * B * own_fp * (bf_pass_fp + N * (OPS_SHOUP_FP + 2)))
    put("ntt16_fwd_blocks_inner8_kernel", 2, (B * (new_int + own_int + 2 * n_int) + 2 * beta * n_int) * limb,
        B * (new_int * bf_pass + N * n_int * beta * 2 * mul_redc))
    put("ntt16_fwd_blocks_final_kernel", 2, B * own_int * (6 + addend) * limb,
        2 * B * own_int * (bf_pass + N * (OPS_SHOUP + 2 * OPS_ADD)))
    if hmult:
        put("tensor_kernel", None, B * nl * 7 * limb, B * nl * N * 4 * mul_redc)
    return m


def _uniform(torch, gen, dev, prefix, moduli, N):
    t = torch.empty(tuple(prefix) + (len(moduli), N), dtype=torch.int64, device=dev)
    for i, m in enumerate(moduli):
        t[..., i, :] = torch.randint(0, m, tuple(prefix) + (N,), dtype=torch.int64, device=dev, generator=gen)
    return t


def _time(torch, fn, iters):
    fn()
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(iters):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t) / iters


def _time_events(torch, fn, iters, warmup=3):
    """Median of `iters` HIP-event timings of fn (seconds) on torch's current stream, which is the stream the library
    is handed, after `warmup` untimed calls."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        e1.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e-3)
    ts.sort()
    return ts[len(ts) // 2]


def _host(t):
    import numpy as np
    return t.cpu().numpy().view(np.uint64)


def _fail_parity(what):
    print("bench.py: GPU output differs from the oracle on the sample (%s)" % what, file=sys.stderr)
    sys.exit(3)


def _oracle_pcmm_one(rc, ct1, pt, n1, n2, stride, baby, giant, logN, threads):
    """The BSGS definition (one rotation at a time) for ONE ciphertext [1][2][nl][N] through the oracle's HRot and
    pointwise calls, the independent rotations and inner sums spread over host threads."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from ckks_inputs import galois_element
    nl = ct1.shape[2]
    ids = list(range(nl))
    with ThreadPoolExecutor(max_workers=threads) as ex:
        rots = [ct1] + list(ex.map(lambda b: rc.hrot(ct1, galois_element(b * stride, logN), baby[b - 1]), range(1, n1)))

        def inner(g):
            acc = None
            for b in range(n1):
                t = rc.pointwise(rots[b][0], pt[g, b][None], ids, "mul")
                acc = t if acc is None else rc.pointwise(acc, t, ids, "add")
            acc = acc[None]
            return acc if g == 0 else rc.hrot(acc, galois_element(g * n1 * stride, logN), giant[g - 1])
        parts = list(ex.map(inner, range(n2)))
    out = parts[0]
    for part in parts[1:]:
        out = rc.pointwise(out[0], part[0], ids, "add")[None]
    return out


def other_workloads(args):
    """Secondary workloads (not the headline metric): `pcmm` = the FFN layer share, `attention` = QK^T units,
    `sweep` = level/dnum sweep. Each prints its own JSON line(s)."""
    import torch
    import paper_2604_03425_amd as ck
    from ckks_inputs import config_params, galois_element, make_params
    dev = "cuda:0"
    gen = torch.Generator(device=dev).manual_seed(0xFEED)
    if args.workload == "calibrate":
        # the copy kernel of known size the HBM byte counters are calibrated on: 1 GiB read + 1 GiB written per launch
        p = config_params("tiny_hrot")
        ctx = ck.Context(p, 0)
        src = torch.ones(1 << 27, dtype=torch.int64, device=dev)
        dst = torch.zeros_like(src)
        dt = _time_events(torch, lambda: ck.ckks_prof_copy(ctx, dst, src), 3, warmup=0)
        assert torch.equal(dst, src)
        print(json.dumps({"workload": "calibrate", "kernel": "ckks_prof_copy_kernel", "launches": 3,
                          "bytes_read_per_launch": src.numel() * 8, "bytes_written_per_launch": src.numel() * 8,
                          "copy_GBps": round(2 * src.numel() * 8 / dt / 1e9, 1)}))
    elif args.workload == "ntt":
        # the transforms alone on the batch of the key-switch micro-benchmark: [64 * 2][24] limb-vectors of 2^16
        # residues (50-bit primes), forward then inverse, `--steps` times; --int-only forces the integer bodies
        # (64-bit Shoup butterflies from 32-bit multiplies) that the double-precision bodies replace by default
        p = config_params("keyswitch_micro" if args.ntt_logn == 16 else "tiny_hrot_k2")
        N, nl, B = p.N, len(p.q), 64 if args.ntt_logn == 16 else 4096
        ctx = ck.Context(p, 0)
        if args.int_only:
            ck.ckks_tune_set(ctx, 1, 1)
        x = _uniform(torch, gen, dev, (B * 2,), p.q, N)
        x0 = x[:2].clone()
        ids = list(range(nl))
        for _ in range(max(1, args.warmup)):
            ck.ckks_ntt(ctx, x, B * 2, ids)
            ck.ckks_intt(ctx, x, B * 2, ids)
        torch.cuda.synchronize()
        ck.ckks_prof_reset(ctx)
        ck.ckks_prof_enable(ctx, True)
        for _ in range(args.steps):
            ck.ckks_ntt(ctx, x, B * 2, ids)
            ck.ckks_intt(ctx, x, B * 2, ids)
        torch.cuda.synchronize()
        ck.ckks_prof_enable(ctx, False)
        prof = ck.ckks_prof_collect(ctx)
        assert torch.equal(x[:2], x0), "INTT(NTT(x)) != x"
        limbs = B * 2 * nl
        ops_bf = OPS_BUTTERFLY if args.int_only else OPS_BUTTERFLY_FP
        kinds = {}
        npass = 2 if args.ntt_logn == 16 else 1   # passes over memory per transform
        for k, (ms, n) in prof.items():
            t = ms * 1e-3 / n                    # one pass over every limb
            kinds[k] = dict(avg_launch_us=round(t * 1e6, 2), GBps=round(limbs * 2 * 8 * N / t / 1e9, 1),
                            modelled_Tops=round(limbs * (N / 2) * (p.logN / npass) * ops_bf / t / 1e12, 2))
        fwd = sum(ms for k, (ms, n) in prof.items() if "fwd" in k) * 1e-3 / args.steps
        inv = sum(ms for k, (ms, n) in prof.items() if "inv" in k) * 1e-3 / args.steps
        print(json.dumps({"workload": "ntt", "arithmetic": "int32 (Shoup butterflies; utilisation counts the canonical 24 operations per butterfly)" if args.int_only
                          else "fp64 (utilisation counts 9.5 operations per butterfly)", "limb_vectors": limbs,
                          "ntt_limbs_per_s": round(limbs / fwd), "intt_limbs_per_s": round(limbs / inv),
                          "ring": "N = 2^%d" % p.logN,
                          "ntt_hbm_frac": round(limbs * 2 * npass * 8 * N / fwd / 1e9 / PEAK_HBM_GBS, 4),
                          "ntt_alu_frac_modelled_ops": round(limbs * (N / 2) * p.logN * ops_bf / fwd / 1e12 / PEAK_ALU_TOPS, 4),
                          "kernels": kinds}))
    elif args.workload == "pcmm":
        # 2048 tokens x 768 hidden in 128 ciphertexts (16 tokens each), 768x768 weight slice as 32 x 24 diagonals,
        # processed in calls of `--pcmm-batch` ciphertexts; 31 baby + 23 giant rotation keys shared by all
        p = config_params("keyswitch_micro")
        N, nl, n1, n2, total = p.N, len(p.q), args.pcmm_n1, args.pcmm_n2, 128
        Bc = args.pcmm_batch
        ctx = ck.Context(p, 0)
        for kv in filter(None, args.tune.split(",")):
            k, v = kv.split("=")
            ck.ckks_tune_set(ctx, int(k), int(v))
        ct = _uniform(torch, gen, dev, (Bc, 2), p.q, N)
        pt = _uniform(torch, gen, dev, (n2, n1), p.q, N)
        baby = [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(n1 - 1)]
        giant = [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(n2 - 1)]
        out = torch.empty_like(ct)
        ws = ctx.workspace(ck.OP_PCMM_BSGS, Bc, nl, n1)
        dt = _time(torch, lambda: ck.ckks_pcmm_bsgs(ctx, out, ct, Bc, nl, pt, n1, n2, 1, baby, giant, ws), 2)
        ck.ckks_prof_reset(ctx)
        ck.ckks_prof_enable(ctx, True)
        ck.ckks_pcmm_bsgs(ctx, out, ct, Bc, nl, pt, n1, n2, 1, baby, giant, ws)
        ck.ckks_prof_enable(ctx, False)
        prof = {k: round(v[0], 2) for k, v in ck.ckks_prof_collect(ctx).items()}
        dth = _time(torch, lambda: ck.ckks_pcmm_bsgs_hoisted(ctx, out, ct, Bc, nl, pt, n1, n2, 1, baby, giant, ws), 2)
        ck.ckks_prof_reset(ctx)
        ck.ckks_prof_enable(ctx, True)
        ck.ckks_pcmm_bsgs_hoisted(ctx, out, ct, Bc, nl, pt, n1, n2, 1, baby, giant, ws)
        ck.ckks_prof_enable(ctx, False)
        prof_h = {k: round(v[0], 2) for k, v in ck.ckks_prof_collect(ctx).items()}
        # baby steps kept in the extended basis (one ModDown per giant step); plaintexts in that basis. Baby steps
        # are cheap there, so the same n1*n2 diagonals are split with more baby and fewer giant steps
        del ws
        d1, d2 = args.pcmm_dh_n1, args.pcmm_dh_n2
        if d1 * d2 != n1 * n2:
            d1, d2 = n1, n2
        pt_ext = _uniform(torch, gen, dev, (d2, d1), list(p.q) + list(p.p), N)
        baby += [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(d1 - n1)]
        giant += [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(d2 - n2)]
        ws2 = ctx.workspace(ck.OP_PCMM_BSGS_DH, Bc, nl, d1)
        dh_call = lambda: ck.ckks_pcmm_bsgs_double_hoisted(ctx, out, ct, Bc, nl, pt_ext, d1, d2, 1, baby[:d1 - 1],
                                                           giant[:d2 - 1], ws2)
        dtd = _time(torch, dh_call, 2)
        ck.ckks_prof_reset(ctx)
        ck.ckks_prof_enable(ctx, True)
        dh_call()
        ck.ckks_prof_enable(ctx, False)
        prof_d = {k: round(v[0], 2) for k, v in ck.ckks_prof_collect(ctx).items()}
        # parity of what was timed: ciphertext `Bc - 1` of the plain and of the hoisted call against the oracle
        checked = None
        if not args.no_cpu_baseline:
            from oracle import ref
            threads = min(16, os.cpu_count() or 1)
            rc = ref.RefContext(p)
            ref.set_threads(1)
            b1 = Bc - 1
            t_or = time.perf_counter()
            want = _oracle_pcmm_one(rc, _host(ct[b1:b1 + 1]), _host(pt), n1, n2, 1, [_host(k) for k in baby[:n1 - 1]],
                                    [_host(k) for k in giant[:n2 - 1]], p.logN, threads)
            t_or = time.perf_counter() - t_or
            for name, fn in (("ckks_pcmm_bsgs", ck.ckks_pcmm_bsgs), ("ckks_pcmm_bsgs_hoisted", ck.ckks_pcmm_bsgs_hoisted)):
                wsc = ctx.workspace(ck.OP_PCMM_BSGS, Bc, nl, n1)
                fn(ctx, out, ct, Bc, nl, pt, n1, n2, 1, baby[:n1 - 1], giant[:n2 - 1], wsc)
                torch.cuda.synchronize()
                if not (_host(out[b1:b1 + 1]) == want).all():
                    _fail_parity(name)
                del wsc
            checked = "ciphertext %d of the plain and the hoisted call equals the oracle's BSGS (%.0f s on %d threads)" % (b1, t_or, threads)
        rots = Bc * (n1 - 1 + n2 - 1)
        # inner sums on the double-precision limbs: 7 FP64 instructions per multiply-add (exact product in two
        # parts, quotient, remainder, accumulate), against the chip's FP64 vector issue rate
        nfp = sum(1 for m in p.q if m < (1 << 50))
        macs = Bc * 2 * nfp * N * n1 * n2
        pm_ms = prof.get("pmacc_fp_kernel", 0.0)
        pm_roof = None
        if pm_ms:
            tops = macs * OPS_MULRED_FP / (pm_ms * 1e-3) / 1e12
            pm_roof = {"bound": "alu", "kernel": "pmacc_fp_kernel", "achieved": round(tops, 2), "peak": round(PEAK_ALU_TOPS, 1),
                       "unit": "T lane-instructions/s", "frac": round(tops / PEAK_ALU_TOPS, 3)}
        print(json.dumps({"workload": "pcmm_ffn_share", "gpu_matches_oracle_on_sample": checked, "inner_sum_roofline": pm_roof, "ciphertexts_per_call": Bc, "seconds_per_call": round(dt, 4),
                          "seconds_for_128_ciphertexts": round(dt * total / Bc, 3), "hrot_per_s": round(rots / dt, 1),
                          "hoisted_seconds_per_call": round(dth, 4),
                          "hoisted_seconds_for_128_ciphertexts": round(dth * total / Bc, 3),
                          "pmult_acc_per_s": round(Bc * n1 * n2 / dt, 1), "kernel_ms_per_call": prof,
                          "hoisted_kernel_ms_per_call": prof_h,
                          "double_hoisted_split": [d1, d2],
                          "double_hoisted_seconds_per_call": round(dtd, 4),
                          "double_hoisted_seconds_for_128_ciphertexts": round(dtd * total / Bc, 3),
                          "double_hoisted_kernel_ms_per_call": prof_d,
                          "note": "%d x %d diagonals: %d HRot + %d PMult-acc per ciphertext (32 x 24 = 2048 tokens x 768 -> "
                                  "768 slice of the FFN; the QKV / W_o projections are the same call with their own "
                                  "diagonals)" % (n1, n2, n1 + n2 - 2, n1 * n2)}))
    elif args.workload == "attention":
        # one (a,b) block pair per head, 3 heads: unit = HMult+relin + 6 rotate-and-sum HRots; 20 limbs, dnum 4, K 5
        p = config_params("attention_qk")
        N, nl, B = p.N, len(p.q), args.att_batch
        ctx = ck.Context(p, 0)
        qa = _uniform(torch, gen, dev, (B, 2), p.q, N)
        kb = _uniform(torch, gen, dev, (B, 2), p.q, N)
        relin = _uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N)
        rot = [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(6)]
        acc = torch.empty_like(qa)
        tmp = torch.empty_like(qa)
        ws = ctx.workspace(ck.OP_HROT, B, nl)
        mods = torch.tensor(list(p.q), dtype=torch.int64, device=dev).view(1, 1, nl, 1)

        def units():
            ck.ckks_hmult_relin(ctx, acc, qa, kb, B, nl, relin, ws)
            cur, nxt = acc, tmp
            for i in range(6):   # rotate-and-sum: next = cur + HRot(cur)
                ck.ckks_hrot_add(ctx, nxt, cur, cur, B, nl, galois_element(1 << i, p.logN), rot[i], ws)
                cur, nxt = nxt, cur
            return cur
        dt = _time(torch, units, 2)
        # the same slot sums as two hoisted sums (rotations by 1..7, then by 8, 16, .., 56): 2 decompositions and 2
        # ModDowns instead of 6 key switches, 14 rotation keys instead of 6
        rot14 = rot + [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(8)]
        ws_sum = ctx.workspace(ck.OP_HROT_SUM, B, nl)
        g_in = [galois_element(k, p.logN) for k in range(1, 8)]
        g_out = [galois_element(8 * j, p.logN) for j in range(1, 8)]

        def units_hoisted():
            ck.ckks_hmult_relin(ctx, acc, qa, kb, B, nl, relin, ws)
            ck.ckks_hrot_sum(ctx, tmp, acc, B, nl, g_in, rot14[:7], ws_sum)
            ck.ckks_hrot_sum(ctx, acc, tmp, B, nl, g_out, rot14[7:], ws_sum)
            return acc
        dth = _time(torch, units_hoisted, 2)
        # parity of what was timed: the first two units of both forms against the same sequences on the oracle
        checked = None
        if not args.no_cpu_baseline:
            from oracle import ref
            ns = min(2, B)
            rc = ref.RefContext(p)
            ref.set_threads(ns)
            ids = list(range(nl))
            t_or = time.perf_counter()
            w = rc.hmult_relin(_host(qa[:ns]), _host(kb[:ns]), _host(relin))
            prod = w
            for i in range(6):
                w = rc.pointwise(w, rc.hrot(w, galois_element(1 << i, p.logN), _host(rot[i])), ids, "add")
            wh = rc.hrot_sum(prod, g_in, [_host(k) for k in rot14[:7]])
            wh = rc.hrot_sum(wh, g_out, [_host(k) for k in rot14[7:]])
            t_or = time.perf_counter() - t_or
            got = units()
            torch.cuda.synchronize()
            if not (_host(got[:ns]) == w).all():
                _fail_parity("attention unit")
            got = units_hoisted()
            torch.cuda.synchronize()
            if not (_host(got[:ns]) == wh).all():
                _fail_parity("attention unit, hoisted sums")
            checked = "units 0..%d of both forms equal the oracle's (%.0f s on %d threads)" % (ns - 1, t_or, ns)
        print(json.dumps({"workload": "attention_qk_units", "gpu_matches_oracle_on_sample": checked,
                          "units_per_call": B, "units_per_s": round(B / dt, 1),
                          "units_per_s_hoisted_sums": round(B / dth, 1),
                          "key_switches_per_s": round(7 * B / dt, 1),
                          "note": "unit = HMult+relin + 6 rotate-and-sum HRot at 20 limbs, dnum=4, K=5; "
                                  "1536 units per (head, block pair) x 3 heads scale linearly; hoisted_sums: the "
                                  "sum over a token's 64 slots as two ckks_hrot_sum calls (7 rotations and one "
                                  "ModDown each) instead of 6 key switches"}))
    elif args.workload == "attention_av":
        # second attention workload: score diagonal (as above), mask-and-pack (Rescale, PMult by the slot mask,
        # Rescale, 6 replicating right rotations) and the product with V two limbs lower; 14 key switches per unit
        p = config_params("attention_qk")
        N, nl, B = p.N, len(p.q), args.att_batch
        ctx = ck.Context(p, 0)
        qa = _uniform(torch, gen, dev, (B, 2), p.q, N)
        kb = _uniform(torch, gen, dev, (B, 2), p.q, N)
        vb = _uniform(torch, gen, dev, (B, 2), p.q[:nl - 2], N)
        mask = _uniform(torch, gen, dev, (), p.q[:nl - 1], N)
        relin = _uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N)
        rot = [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(12)]
        ws = ctx.workspace(ck.OP_HROT, B, nl)
        new = lambda n: torch.empty((B, 2, n, N), dtype=torch.int64, device=dev)
        d, tmp, d1, m1, m, tmp2, out = new(nl), new(nl), new(nl - 1), new(nl - 1), new(nl - 2), new(nl - 2), new(nl - 2)

        def units():
            ck.ckks_hmult_relin(ctx, d, qa, kb, B, nl, relin, ws)
            cur, nxt = d, tmp
            for i in range(6):
                ck.ckks_hrot_add(ctx, nxt, cur, cur, B, nl, galois_element(1 << i, p.logN), rot[i], ws)
                cur, nxt = nxt, cur
            ck.ckks_rescale(ctx, d1, cur, B, nl, ws)
            ck.ckks_pmult(ctx, m1, d1, mask, B, nl - 1)
            ck.ckks_rescale(ctx, m, m1, B, nl - 1, ws)
            cur, nxt = m, tmp2
            for i in range(6):
                ck.ckks_hrot_add(ctx, nxt, cur, cur, B, nl - 2, galois_element(-(1 << i), p.logN), rot[6 + i], ws)
                cur, nxt = nxt, cur
            if late[0]:
                ck.ckks_tensor_acc(ctx, acc3, cur, vb, acc3, B, nl - 2)
            else:
                ck.ckks_hmult_relin(ctx, out, cur, vb, B, nl - 2, relin, ws)
        late = [False]
        acc3 = torch.zeros((B, 3, nl - 2, N), dtype=torch.int64, device=dev)
        dt = _time(torch, units, 2)
        # parity of what was timed: the first two units against the same sequence of calls on the oracle
        checked = None
        if not args.no_cpu_baseline:
            from oracle import ref
            ns = min(2, B)
            rc = ref.RefContext(p)
            ref.set_threads(ns)
            t_or = time.perf_counter()
            w = rc.hmult_relin(_host(qa[:ns]), _host(kb[:ns]), _host(relin))
            for i in range(6):
                w = rc.pointwise(w, rc.hrot(w, galois_element(1 << i, p.logN), _host(rot[i])), list(range(nl)), "add")
            w = rc.rescale(rc.pmult(rc.rescale(w), _host(mask)))
            for i in range(6):
                w = rc.pointwise(w, rc.hrot(w, galois_element(-(1 << i), p.logN), _host(rot[6 + i])), list(range(nl - 2)), "add")
            w = rc.hmult_relin(w, _host(vb[:ns]), _host(relin))
            t_or = time.perf_counter() - t_or
            units()
            torch.cuda.synchronize()
            if not (_host(out[:ns]) == w).all():
                _fail_parity("attention A x V unit")
            checked = "units 0..%d equal the oracle's (%.0f s on %d threads)" % (ns - 1, t_or, ns)
        # late relinearisation (Sec. 5.2): the products with V of a block's 64 diagonals stay in three components
        # and share one key switch, timed here as 64 calls of the unit followed by one ckks_relin
        late[0] = True

        def block():
            for _ in range(64):
                units()
            ck.ckks_relin(ctx, out, acc3, B, nl - 2, relin, ws)
        dt_late = _time(torch, block, 1) / 64
        # every slot sum as two hoisted sums (rotations by +-1..7, then +-8..56), late relinearisation as above
        rot28 = rot + [_uniform(torch, gen, dev, (p.dnum, 2), p.moduli, N) for _ in range(16)]
        ws_sum = ctx.workspace(ck.OP_HROT_SUM, B, nl)
        gin = [galois_element(k, p.logN) for k in range(1, 8)]
        gout = [galois_element(8 * j, p.logN) for j in range(1, 8)]
        gin_r = [galois_element(-k, p.logN) for k in range(1, 8)]
        gout_r = [galois_element(-8 * j, p.logN) for j in range(1, 8)]

        def units_hoisted():
            ck.ckks_hmult_relin(ctx, d, qa, kb, B, nl, relin, ws)
            ck.ckks_hrot_sum(ctx, tmp, d, B, nl, gin, rot28[:7], ws_sum)
            ck.ckks_hrot_sum(ctx, d, tmp, B, nl, gout, rot28[7:14], ws_sum)
            ck.ckks_rescale(ctx, d1, d, B, nl, ws)
            ck.ckks_pmult(ctx, m1, d1, mask, B, nl - 1)
            ck.ckks_rescale(ctx, m, m1, B, nl - 1, ws)
            ck.ckks_hrot_sum(ctx, tmp2, m, B, nl - 2, gin_r, rot28[14:21], ws_sum)
            ck.ckks_hrot_sum(ctx, m, tmp2, B, nl - 2, gout_r, rot28[21:28], ws_sum)
            ck.ckks_tensor_acc(ctx, acc3, m, vb, acc3, B, nl - 2)

        def block_hoisted():
            for _ in range(64):
                units_hoisted()
            ck.ckks_relin(ctx, out, acc3, B, nl - 2, relin, ws)
        dt_h = _time(torch, block_hoisted, 1) / 64
        print(json.dumps({"workload": "attention_av_units", "gpu_matches_oracle_on_sample": checked,
                          "units_per_call": B, "units_per_s": round(B / dt, 1),
                          "key_switches_per_s": round(14 * B / dt, 1),
                          "units_per_s_late_relin": round(B / dt_late, 1),
                          "units_per_s_hoisted_sums": round(B / dt_h, 1),
                          "note": "unit = score diagonal (HMult+relin + 6 HRot) + mask-and-pack (2 Rescale, PMult, "
                                  "6 HRot) + HMult+relin with V, 20 -> 18 limbs, dnum=4, K=5; late_relin: the "
                                  "product with V accumulated in three components, one key switch per 64 units; "
                                  "hoisted_sums: also every sum over a token's 64 slots as two ckks_hrot_sum calls "
                                  "(7 rotations each, one ModDown each)"}))
    elif args.workload == "sweep":
        B = 32
        for limbs in (4, 8, 12, 16, 20, 24, 28, 32, 36):
            for dnum in (1, 2, 3, 4, 6):
                if dnum > limbs:
                    continue
                K = -(-limbs // dnum)
                p = make_params(16, limbs, 50, K, 60, dnum)
                ctx = ck.Context(p, 0)
                for kv in filter(None, args.tune.split(",")):
                    k, v = kv.split("=")
                    ck.ckks_tune_set(ctx, int(k), int(v))
                d = _uniform(torch, gen, dev, (B,), p.q, p.N)
                evk = _uniform(torch, gen, dev, (p.dnum, 2), p.moduli, p.N)
                out = torch.empty((B, 2, limbs, p.N), dtype=torch.int64, device=dev)
                ws = ctx.workspace(ck.OP_KEYSWITCH, B, limbs)
                dt = _time_events(torch, lambda: ck.ckks_keyswitch(ctx, out, d, B, limbs, evk, 0, dnum, ws), 20)
                x = _uniform(torch, gen, dev, (B * 2,), p.q, p.N)
                ids = list(range(limbs))
                dn = _time_events(torch, lambda: ck.ckks_ntt(ctx, x, B * 2, ids), 20)
                if not args.no_cpu_baseline:   # parity of what was timed: ciphertext 0 of the key switch
                    from oracle import ref
                    rc = ref.RefContext(p)
                    ref.set_threads(1)
                    torch.cuda.synchronize()
                    if not (_host(out[:1]) == rc.keyswitch(_host(d[:1]), _host(evk))).all():
                        _fail_parity("sweep point %d limbs, dnum %d" % (limbs, dnum))
                model = keyswitch_model(p, B, limbs, False, False)
                nbytes = sum(v["bytes"] for v in model.values())
                nops = sum(v["ops"] for v in model.values())
                print(json.dumps({"workload": "sweep", "limbs": limbs, "dnum": dnum, "K": K, "batch": B,
                                  "timing": "median of 20 HIP-event iterations after 3 warm-ups",
                                  "gpu_matches_oracle_on_sample": not args.no_cpu_baseline,
                                  "key_switches_per_s": round(B / dt, 1), "ntt_limbs_per_s": round(B * 2 * limbs / dn),
                                  "hbm_frac_modelled_bytes": round(nbytes / dt / 1e9 / PEAK_HBM_GBS, 3),
                                  "alu_frac_modelled_ops": round(nops / dt / 1e12 / PEAK_ALU_TOPS, 3),
                                  "ntt_hbm_frac": round(B * 2 * limbs * 4 * 8 * p.N / dn / 1e9 / PEAK_HBM_GBS, 3)}), flush=True)
                ctx.close()
                del d, evk, out, ws, x
                torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--groups", type=int, default=64, help="distinct (Galois element, key) groups among the 64 HRots")
    ap.add_argument("--hrot-call", default="multi", choices=["grouped", "multi"],
                    help="grouped: one ckks_hrot per group; multi: one ckks_hrot_multi over all 64 ciphertexts")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--map-mode", type=int, default=None, help="experiment: workgroup mapping mode of the 2^16 transforms")
    ap.add_argument("--int-only", action="store_true", help="experiment: integer bodies for every modulus")
    ap.add_argument("--tune", type=str, default="", help="experiment: comma-separated knob=value pairs")
    ap.add_argument("--streams", type=int, default=1, help="HIP streams the independent calls of a step are spread over")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="experiment: time the steps without the per-kernel HIP events (no phases, no roofline)")
    ap.add_argument("--no-extras", action="store_true", help="skip the separate NTT / HRot / HMult timings (profiling runs)")
    ap.add_argument("--workload", default="keyswitch_micro", choices=["keyswitch_micro", "pcmm", "attention", "attention_av", "sweep", "ntt", "calibrate"])
    ap.add_argument("--pcmm-batch", type=int, default=32)
    ap.add_argument("--pcmm-n1", type=int, default=32, help="baby steps (32 x 24 = the FFN share; 8 x 8 = a 64-slot block)")
    ap.add_argument("--pcmm-n2", type=int, default=24, help="giant steps")
    ap.add_argument("--pcmm-dh-n1", type=int, default=64, help="baby steps of the double-hoisted schedule (same product n1*n2, else the plain split is used)")
    ap.add_argument("--pcmm-dh-n2", type=int, default=12)
    ap.add_argument("--att-batch", type=int, default=32)
    ap.add_argument("--ntt-logn", type=int, default=16, choices=[12, 16],
                    help="ring degree of the `ntt` workload (12: the tiny configuration's primes, 4096 x 2 polynomials)")
    ap.add_argument("--cpu-sample", type=int, default=32, help="ciphertexts the CPU oracle rotates (half as many HMult pairs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build covers one GPU's share of the work; --gpus %d is not supported (use --gpus 1)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_03425_amd as ck
    from ckks_inputs import config_params, galois_element, seeded_rotation_steps

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.workload != "keyswitch_micro":
        other_workloads(args)
        return
    dev = "cuda:0"
    p = config_params("keyswitch_micro")
    N, nl, B, G = p.N, len(p.q), 64, args.groups
    assert B % G == 0
    ctx = ck.Context(p, 0)
    if args.map_mode is not None:
        ck.ckks_tune_set(ctx, 0, args.map_mode)
    if args.int_only:
        ck.ckks_tune_set(ctx, 1, 1)
    fp_inner, bconv_fused = 2, False   # library defaults of knobs 3 and 2
    for kv in filter(None, args.tune.split(",")):
        k, v = kv.split("=")
        ck.ckks_tune_set(ctx, int(k), int(v))
        if int(k) == 3:
            fp_inner = int(v)
        if int(k) == 2:
            bconv_fused = int(v) == 1
    gen = torch.Generator(device=dev).manual_seed(0xC0FFEE)

    def uniform(prefix, moduli):
        t = torch.empty(tuple(prefix) + (len(moduli), N), dtype=torch.int64, device=dev)
        for i, m in enumerate(moduli):
            t[..., i, :] = torch.randint(0, m, tuple(prefix) + (N,), dtype=torch.int64, device=dev, generator=gen)
        return t

    ct = uniform((B, 2), p.q)
    evks = [uniform((p.dnum, 2), p.moduli) for _ in range(G)]
    evk_mult = uniform((p.dnum, 2), p.moduli)
    steps_r = seeded_rotation_steps(7, G, 1, N // 2 - 1)
    gal = [galois_element(r, p.logN) for r in steps_r]
    ct_a = ct[0::2].contiguous()
    ct_b = ct[1::2].contiguous()
    out_rot = torch.empty_like(ct)
    out_mul = torch.empty_like(ct_a)
    Bg = B // G
    # the calls of a step are independent of each other; with more than one stream they are dealt round-robin to
    # the streams (default priority), each stream with its own workspace, so one call's tail overlaps another's start
    nstreams = max(1, args.streams)
    streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(nstreams - 1)]
    multi = args.hrot_call == "multi"
    wss = [ctx.workspace(ck.OP_HROT, B if multi else max(Bg, B // 2), nl) for _ in range(nstreams)]
    ws = wss[0]
    gal_pc = [gal[b // Bg] for b in range(B)]
    evk_pc = [evks[b // Bg] for b in range(B)]

    def step():
        if nstreams > 1:
            for s_ in streams[1:]:
                s_.wait_stream(streams[0])
        if multi:   # all 64 rotations in one call, each ciphertext with its group's element and key
            ck.ckks_hrot_multi(ctx, out_rot, ct, B, nl, gal_pc, evk_pc, ws)
        for g in range(0 if multi else G):
            with torch.cuda.stream(streams[g % nstreams]):
                ck.ckks_hrot(ctx, out_rot[g * Bg:(g + 1) * Bg], ct[g * Bg:(g + 1) * Bg], Bg, nl, gal[g], evks[g],
                             wss[g % nstreams])
        with torch.cuda.stream(streams[G % nstreams]):
            ck.ckks_hmult_relin(ctx, out_mul, ct_a, ct_b, B // 2, nl, evk_mult, wss[G % nstreams])
        if nstreams > 1:
            for s_ in streams[1:]:
                streams[0].wait_stream(s_)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ck.ckks_prof_reset(ctx)
    ck.ckks_prof_enable(ctx, not args.no_kernel_events)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ck.ckks_prof_enable(ctx, False)
    prof = ck.ckks_prof_collect(ctx)
    sec = t1 - t0
    ks_per_step = B + B // 2
    value = ks_per_step * args.steps / sec

    # --- per-kind roofline figures from the event durations of the timed region ---
    model = {}
    for (b, hrot, hmult, calls) in ((Bg, True, False, G), (B // 2, False, True, 1)):
        for kind, v in keyswitch_model(p, b, nl, hrot, hmult, fp_inner, bconv_fused).items():
            acc = model.setdefault(kind, dict(bytes=0.0, ops=0.0))
            acc["bytes"] += v["bytes"] * calls
            acc["ops"] += v["ops"] * calls
    phases = {}
    for kind, (ms, n) in prof.items():
        per_step_ms = ms / args.steps
        mdl = model.get(kind, dict(bytes=0.0, ops=0.0))
        phases[kind] = dict(ms_per_step=round(per_step_ms, 4), launches_per_step=n / args.steps,
                            avg_launch_us=round(1e3 * ms / n, 2),
                            GBps=round(mdl["bytes"] / per_step_ms / 1e6, 1) if per_step_ms else None,
                            Tops=round(mdl["ops"] / per_step_ms / 1e9, 2) if per_step_ms else None)
    # the counter runs were made in the default configuration only
    default_cfg = (G == 64 and multi and not args.tune and not args.int_only and args.map_mode is None and nstreams == 1)
    traffic_tab = measured_traffic() if default_cfg else {}
    dom = max(prof.items(), key=lambda kv: kv[1][0])[0] if prof else None
    d = phases[dom] if dom else dict(GBps=None, Tops=None, avg_launch_us=None)
    hbm_frac = (d["GBps"] or 0) / PEAK_HBM_GBS
    alu_frac = (d["Tops"] or 0) / PEAK_ALU_TOPS
    if dom is None:
        roofline = None
    elif alu_frac >= hbm_frac:
        roofline = dict(bound="alu", kernel=dom, achieved=d["Tops"], peak=round(PEAK_ALU_TOPS, 1), unit="Tlane-op/s",
                        frac=round(alu_frac, 4), traffic=traffic_tab.get(dom) if default_cfg else None, avg_launch_us=d["avg_launch_us"])
    else:
        roofline = dict(bound="hbm", kernel=dom, achieved=d["GBps"], peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(hbm_frac, 4), traffic=traffic_tab.get(dom) if default_cfg else None, avg_launch_us=d["avg_launch_us"])
    total_bytes = sum(v["bytes"] for v in model.values())
    total_ops = sum(v["ops"] for v in model.values())
    # compulsory traffic of a step: read every input ciphertext and key once, write every output once
    compulsory = (G * (Bg * (2 * nl + 2 * nl) + 2 * p.dnum * (nl + len(p.p))) +
                  (B // 2) * (4 * nl + 2 * nl) + 2 * p.dnum * (nl + len(p.p))) * 8 * N

    # --- separate short measurements: transforms alone, HRot alone, HMult alone ---
    def timed(fn, iters):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(iters):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / iters
    extra = None
    if not args.no_extras:
      ids = list(range(nl))
      scratch = ct.clone()
      t_ntt = timed(lambda: ck.ckks_ntt(ctx, scratch, B * 2, ids), 5)
      t_intt = timed(lambda: ck.ckks_intt(ctx, scratch, B * 2, ids), 5)
      ctx_int = ck.Context(p, 0)
      ck.ckks_tune_set(ctx_int, 1, 1)
      t_ntt_int = timed(lambda: ck.ckks_ntt(ctx_int, scratch, B * 2, ids), 5)
      ctx_int.close()
      t_rot = timed(lambda: [ck.ckks_hrot(ctx, out_rot[g * Bg:(g + 1) * Bg], ct[g * Bg:(g + 1) * Bg], Bg, nl, gal[g], evks[g], ws)
                             for g in range(G)], 3)
      t_rot1 = timed(lambda: ck.ckks_hrot(ctx, out_rot, ct, B, nl, gal[0], evks[0],
                                          ctx.workspace(ck.OP_HROT, B, nl)), 3)
      t_mul = timed(lambda: ck.ckks_hmult_relin(ctx, out_mul, ct_a, ct_b, B // 2, nl, evk_mult, ws), 3)
      # every ciphertext with its own element and key (64 keys, 6 GiB), one batched call
      ws_b = ctx.workspace(ck.OP_HROT, B, nl)
      evk64 = evks + [uniform((p.dnum, 2), p.moduli) for _ in range(B - G)]
      gal64 = [galois_element(r, p.logN) for r in seeded_rotation_steps(8, B, 1, N // 2 - 1)]
      t_rot64 = timed(lambda: ck.ckks_hrot_multi(ctx, out_rot, ct, B, nl, gal64, evk64, ws_b), 3)
      # the paper's one-rotation-at-a-time style (Sec. 5.1) without launch overhead: the same 64 rotations as 64
      # calls on one ciphertext each, captured once into a HIP graph through the entry point that allocates nothing
      # and replayed (they share the library's scratch array, so the graph is one chain)
      graph = torch.cuda.CUDAGraph()
      ck.ckks_hrot_noalloc(ctx, out_rot[:1], ct[:1], 1, nl, gal64[0], evk64[0])
      torch.cuda.synchronize()
      with torch.cuda.graph(graph):
          for b in range(B):
              ck.ckks_hrot_noalloc(ctx, out_rot[b:b + 1], ct[b:b + 1], 1, nl, gal64[b], evk64[b])
      t_rot_graph = timed(graph.replay, 3)
      del graph
      # the same 64 single-ciphertext rotations issued round-robin on four streams (a workspace each): what a caller
      # that cannot batch gets by keeping several calls in flight (default-priority streams; one context serves them all)
      side = [torch.cuda.Stream() for _ in range(4)]
      ws4 = [ctx.workspace(ck.OP_HROT, 1, nl) for _ in range(4)]
      def rot_streams():
          cur = torch.cuda.current_stream()
          for s_ in side:
              s_.wait_stream(cur)
          for b in range(B):
              with torch.cuda.stream(side[b % 4]):
                  ck.ckks_hrot(ctx, out_rot[b:b + 1], ct[b:b + 1], 1, nl, gal64[b], evk64[b], ws4[b % 4])
          for s_ in side:
              cur.wait_stream(s_)
      t_rot_streams = timed(rot_streams, 3)
      del evk64, ws4
      # the step after a product: Rescale (and the PMult / Add building blocks), same batch
      ws_rs = ctx.workspace(ck.OP_RESCALE, B, nl)
      out_rs = torch.empty((B, 2, nl - 1, N), dtype=torch.int64, device=dev)
      t_rs = timed(lambda: ck.ckks_rescale(ctx, out_rs, ct, B, nl, ws_rs), 3)
      pt1 = ct[0, 0].contiguous()
      # the Galois automorphism as a call of its own (inside HRot it is a gather fused into the loads)
      g_auto = galois_element(4321, p.logN)
      t_au = timed(lambda: ck.ckks_automorph(ctx, out_rot, ct, B * 2, ids, g_auto, True), 3)
      t_auc = timed(lambda: ck.ckks_automorph(ctx, out_rot, ct, B * 2, ids, g_auto, False), 3)
      t_pm = timed(lambda: ck.ckks_pmult(ctx, out_rot, ct, pt1, B, nl), 3)
      t_ad = timed(lambda: ck.ckks_add(ctx, out_rot, ct, out_rot, B * 2, nl), 3)
      extra = dict(ntt_limbs_per_s=round(B * 2 * nl / t_ntt), intt_limbs_per_s=round(B * 2 * nl / t_intt),
                   hrot_per_s=round(B / t_rot, 1), hrot_per_s_one_group=round(B / t_rot1, 1),
                   hrot_per_s_own_key_each=round(B / t_rot64, 1),
                   hrot_per_s_one_by_one_hip_graph=round(B / t_rot_graph, 1),
                   hrot_per_s_one_by_one_4_streams=round(B / t_rot_streams, 1),
                   hmult_relin_per_s=round(B / 2 / t_mul, 1),
                 rescale_per_s=round(B / t_rs, 1),
                 rescale_hbm_frac=round(B * 2 * (4 + 3 * (nl - 1) + 4 * (nl - 1)) * 8 * N / t_rs / 1e9 / PEAK_HBM_GBS, 4),
                 automorph_eval_GBps=round(B * 2 * nl * 2 * 8 * N / t_au / 1e9, 1),
                 automorph_coeff_GBps=round(B * 2 * nl * 2 * 8 * N / t_auc / 1e9, 1),
                 pmult_hbm_frac=round(B * 2 * nl * 2 * 8 * N / t_pm / 1e9 / PEAK_HBM_GBS, 4),
                 add_hbm_frac=round(B * 2 * nl * 3 * 8 * N / t_ad / 1e9 / PEAK_HBM_GBS, 4),
                   # executed arithmetic of the standalone NTT against the 39.3 T lane-ops/s vector issue rate: the
                   # default path runs 9.5 FP64 instructions per butterfly on these 50-bit limbs; the integer bodies
                   # (knob 1, timed on a context of their own) 24 32-bit integer instructions per butterfly
                   ntt_fp64_issue_frac=round(B * 2 * nl * (N / 2) * p.logN * OPS_BUTTERFLY_FP / t_ntt / 1e12 / PEAK_ALU_TOPS, 4),
                   ntt_int_limbs_per_s=round(B * 2 * nl / t_ntt_int),
                   ntt_int32_alu_frac=round(B * 2 * nl * (N / 2) * p.logN * OPS_BUTTERFLY / t_ntt_int / 1e12 / PEAK_ALU_TOPS, 4),
                 ntt_hbm_frac=round(B * 2 * nl * 4 * 8 * N / t_ntt / 1e9 / PEAK_HBM_GBS, 4),
                   hbm_frac_compulsory_bytes=round(compulsory * args.steps / sec / 1e9 / PEAK_HBM_GBS, 4),
                   hbm_frac_modelled_bytes=round(total_bytes * args.steps / sec / 1e9 / PEAK_HBM_GBS, 4),
                 alu_frac_modelled_ops=round(total_ops * args.steps / sec / 1e12 / PEAK_ALU_TOPS, 4))

    # --- CPU oracle on a bounded sample of the same workload ---
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ref
        import numpy as np
        ns = max(2, args.cpu_sample // 2 * 2)
        threads = min(16, os.cpu_count() or 1, ns)
        ref.set_threads(threads)
        rctx = ref.RefContext(p)
        h_ct = ct[:ns].cpu().numpy().view(np.uint64)
        h_evk = evks[0].cpu().numpy().view(np.uint64)
        h_mul = evk_mult.cpu().numpy().view(np.uint64)
        t = time.perf_counter()
        r1 = rctx.hrot(h_ct, gal[0], h_evk)
        r2 = rctx.hmult_relin(h_ct[0::2], h_ct[1::2], h_mul)
        cpu_sec = time.perf_counter() - t
        ref.set_threads(1)
        t = time.perf_counter()
        r1_one = rctx.hrot(h_ct[:1], gal[0], h_evk)
        one_sec = time.perf_counter() - t
        assert (r1_one == r1[:1]).all()
        cpu = dict(value=round((ns + ns // 2) / cpu_sec, 3), unit="key-switches/s", cores=threads, kind="oracle",
                   sample="%d HRot + %d HMult+relin of the same workload (N=2^16, 24 limbs, dnum=3), %.1f s on %d threads; "
                          "single thread: 1 HRot in %.1f s" % (ns, ns // 2, cpu_sec, threads, one_sec),
                   single_thread_value=round(1.0 / one_sec, 3), host_cpus=os.cpu_count())
        # the sample doubles as an end-of-run parity check of the timed configuration
        chk = torch.empty_like(ct[:ns])
        ck.ckks_hrot(ctx, chk, ct[:ns].contiguous(), ns, nl, gal[0], evks[0], ctx.workspace(ck.OP_HROT, ns, nl))
        ck.ckks_hmult_relin(ctx, out_mul, ct_a, ct_b, B // 2, nl, evk_mult, ws)
        torch.cuda.synchronize()
        ok = bool((chk.cpu().numpy().view(np.uint64) == r1).all() and
                  (out_mul[:ns // 2].cpu().numpy().view(np.uint64) == r2).all())
        if multi:   # the batched call as timed: one ciphertext of another group against the oracle
            b1 = B - 1
            ck.ckks_hrot_multi(ctx, out_rot, ct, B, nl, gal_pc, evk_pc, ws)
            torch.cuda.synchronize()
            r3 = rctx.hrot(ct[b1:b1 + 1].cpu().numpy().view(np.uint64), gal_pc[b1], evk_pc[b1].cpu().numpy().view(np.uint64))
            ok = ok and bool((out_rot[b1:b1 + 1].cpu().numpy().view(np.uint64) == r3).all())
        cpu["gpu_matches_oracle_on_sample"] = ok
        if not ok:
            print("bench.py: GPU output differs from the oracle on the sample", file=sys.stderr)
            sys.exit(3)

    line = {
        "metric": "key_switches_per_s (HRot x64 + HMult+relin x32 per step; N=2^16, 24 limbs, dnum=3)",
        "value": round(value, 2), "unit": "key-switches/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(1e3 * sec / args.steps, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "keyswitch_micro: N=2^16, 24x50-bit + 8x60-bit primes, dnum=3, 64 cts, %d HRot groups (%s), 32 HMult pairs" % (G, "one batched call" if multi else "one call per group"),
                   "global_batch": B, "parallelism": "single-gpu",
                   "arithmetic": "64-bit residues; the 50-bit limbs are computed exactly on the FP64 units, the 60-bit ones on "
                                 "the integer units"},
        "roofline": roofline, "cpu_baseline": cpu, "phases": phases, "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
