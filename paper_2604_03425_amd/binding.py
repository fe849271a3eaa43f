"""ctypes binding of include/ckks_mi355.h. Argument marshalling only; every step runs in the HIP kernels.

Tensors are torch CUDA tensors with 8-byte elements (torch.int64 or torch.uint64 storage of the
uint64 residues), contiguous, on the context's device. Calls are enqueued on torch's current stream.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libckks_mi355.so")

OP_KEYSWITCH, OP_HROT, OP_HMULT_RELIN, OP_PCMM_BSGS, OP_RESCALE, OP_PCMM_BSGS_DH, OP_HROT_SUM = 1, 2, 3, 4, 5, 6, 7

_SYMBOLS = ["ckks_last_error", "ckks_ctx_create", "ckks_ctx_destroy", "ckks_workspace_bytes", "ckks_ntt", "ckks_intt",
            "ckks_automorph", "ckks_keyswitch", "ckks_hrot", "ckks_hmult_relin", "ckks_pcmm_bsgs",
            "ckks_prof_enable", "ckks_prof_num_kinds", "ckks_prof_kind_name", "ckks_prof_collect", "ckks_prof_read",
            "ckks_prof_reset", "ckks_prof_copy", "ckks_tune_set", "ckks_rescale", "ckks_pmult", "ckks_add",
            "ckks_hrot_hoisted", "ckks_pcmm_bsgs_hoisted", "ckks_hrot_multi", "ckks_hrot_add", "ckks_tensor_acc",
            "ckks_relin", "ckks_pcmm_bsgs_double_hoisted", "ckks_hrot_sum", "ckks_hrot_noalloc",
            "ckks_noalloc_scratch_bytes"]


class CkksError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("ckks_mi355 error %d: %s" % (code, msg))
        self.code = code


def library_path():
    return _LIB_PATH


def exported_symbols():
    return list(_SYMBOLS)


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libckks_mi355.so is not built: run `python paper_2604_03425_amd/build.py` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    u64p, u32p, vp = C.c_void_p, C.POINTER(C.c_uint32), C.c_void_p
    lib.ckks_last_error.restype = C.c_char_p
    lib.ckks_ctx_create.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint64), C.c_uint32,
                                    C.POINTER(C.c_uint64), C.c_uint32, C.c_uint32, C.POINTER(C.c_uint64), C.c_int]
    lib.ckks_ctx_destroy.argtypes = [vp]
    lib.ckks_workspace_bytes.restype = C.c_size_t
    lib.ckks_workspace_bytes.argtypes = [vp, C.c_int, C.c_uint32, C.c_uint32, C.c_uint32]
    lib.ckks_ntt.argtypes = [vp, u64p, C.c_uint32, u32p, C.c_uint32, vp]
    lib.ckks_intt.argtypes = [vp, u64p, C.c_uint32, u32p, C.c_uint32, vp]
    lib.ckks_automorph.argtypes = [vp, u64p, u64p, C.c_uint32, u32p, C.c_uint32, C.c_uint32, C.c_int, vp]
    lib.ckks_keyswitch.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, u64p, C.c_uint32, C.c_uint32, vp,
                                   C.c_size_t, vp]
    lib.ckks_hrot.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, C.c_uint32, u64p, vp, C.c_size_t, vp]
    lib.ckks_hrot_noalloc.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, C.c_uint32, u64p, vp]
    lib.ckks_noalloc_scratch_bytes.restype = C.c_size_t
    lib.ckks_noalloc_scratch_bytes.argtypes = []
    lib.ckks_hmult_relin.argtypes = [vp, u64p, u64p, u64p, C.c_uint32, C.c_uint32, u64p, vp, C.c_size_t, vp]
    lib.ckks_tensor_acc.argtypes = [vp, u64p, u64p, u64p, u64p, C.c_uint32, C.c_uint32, vp]
    lib.ckks_relin.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, u64p, vp, C.c_size_t, vp]
    lib.ckks_pcmm_bsgs.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, u64p, C.c_uint32, C.c_uint32, C.c_uint32,
                                   C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), vp, C.c_size_t, vp]
    lib.ckks_hrot_hoisted.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, u32p, C.POINTER(C.c_void_p), C.c_uint32, vp,
                                      C.c_size_t, vp]
    lib.ckks_hrot_sum.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, u32p, C.POINTER(C.c_void_p), C.c_uint32, vp,
                                  C.c_size_t, vp]
    lib.ckks_hrot_add.argtypes = [vp, u64p, u64p, u64p, C.c_uint32, C.c_uint32, C.c_uint32, u64p, vp, C.c_size_t, vp]
    lib.ckks_hrot_multi.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, u32p, C.POINTER(C.c_void_p), vp, C.c_size_t, vp]
    lib.ckks_pcmm_bsgs_hoisted.argtypes = lib.ckks_pcmm_bsgs.argtypes
    lib.ckks_pcmm_bsgs_double_hoisted.argtypes = lib.ckks_pcmm_bsgs.argtypes
    lib.ckks_rescale.argtypes = [vp, u64p, u64p, C.c_uint32, C.c_uint32, vp, C.c_size_t, vp]
    lib.ckks_pmult.argtypes = [vp, u64p, u64p, u64p, C.c_uint32, C.c_uint32, vp]
    lib.ckks_add.argtypes = [vp, u64p, u64p, u64p, C.c_uint32, C.c_uint32, vp]
    lib.ckks_prof_enable.argtypes = [vp, C.c_int]
    lib.ckks_prof_copy.argtypes = [vp, vp, vp, C.c_size_t, vp]
    lib.ckks_tune_set.argtypes = [vp, C.c_int, C.c_int]
    lib.ckks_prof_kind_name.restype = C.c_char_p
    lib.ckks_prof_kind_name.argtypes = [C.c_int]
    lib.ckks_prof_collect.argtypes = [vp]
    lib.ckks_prof_reset.argtypes = [vp]
    lib.ckks_prof_read.argtypes = [vp, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    for name in _SYMBOLS:
        getattr(lib, name)
    return lib


_lib = _load()


def _check(rc):
    if rc != 0:
        raise CkksError(rc, _lib.ckks_last_error().decode())


def _ptr(t, name, ctx=None, elems=None):
    """Device address of `t`. With ctx/elems: also refuse a tensor on another GPU than the context's or with fewer
    than `elems` elements, so that a wrong shape raises here instead of becoming an out-of-bounds device access."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.element_size() != 8 or not t.is_contiguous():
        raise TypeError("%s must be a contiguous CUDA tensor with 8-byte elements" % name)
    if ctx is not None and t.device.index != ctx.device:
        raise ValueError("%s is on cuda:%d, the context on cuda:%d" % (name, t.device.index, ctx.device))
    if elems is not None and t.numel() < elems:
        raise ValueError("%s has %d elements, the call reads or writes %d" % (name, t.numel(), elems))
    return C.c_void_p(t.data_ptr())


def _key_elems(ctx):
    return ctx.params.dnum * 2 * (ctx.nq + ctx.np_) * ctx.N


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ids(ids):
    arr = (C.c_uint32 * len(ids))(*[int(i) for i in ids])
    return arr, C.c_uint32(len(ids))


class Context:
    """Owns a ckks_ctx. `params` needs logN, q, p, dnum, psi (see ckks_inputs.CkksParams)."""

    def __init__(self, params, device=0):
        self.params = params
        self.N = 1 << params.logN
        self.nq, self.np_ = len(params.q), len(params.p)
        q = (C.c_uint64 * self.nq)(*params.q)
        p = (C.c_uint64 * max(1, self.np_))(*(params.p or [0]))
        psi = (C.c_uint64 * (self.nq + self.np_))(*params.psi)
        self.handle = C.c_void_p()
        self.device = device
        _check(_lib.ckks_ctx_create(C.byref(self.handle), params.logN, q, self.nq, p, self.np_, params.dnum, psi, device))

    def close(self):
        if self.handle:
            _lib.ckks_ctx_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace(self, op, batch, nlimbs, n1=0):
        n = ckks_workspace_bytes(self, op, batch, nlimbs, n1)
        if n == 0:
            raise CkksError(-2, "bad shape for workspace query")
        return torch.empty(n // 8, dtype=torch.int64, device="cuda:%d" % self.device)


def ckks_tune_set(ctx, knob, value):
    _check(_lib.ckks_tune_set(ctx.handle, knob, value))


def ckks_prof_enable(ctx, on):
    _check(_lib.ckks_prof_enable(ctx.handle, 1 if on else 0))


def ckks_prof_copy(ctx, dst, src):
    """Plain copy of src into dst (same size), the calibration kernel for the HBM byte counters."""
    n = src.numel() * 8
    _check(_lib.ckks_prof_copy(ctx.handle, _ptr(dst, "dst", ctx, src.numel()), _ptr(src, "src", ctx), n, _stream()))


def ckks_prof_reset(ctx):
    _check(_lib.ckks_prof_reset(ctx.handle))


def ckks_prof_collect(ctx):
    """Per-kernel-kind totals since the last reset: {name: (total_ms, launches)}."""
    _check(_lib.ckks_prof_collect(ctx.handle))
    out = {}
    for k in range(_lib.ckks_prof_num_kinds()):
        ms, n = C.c_double(), C.c_uint64()
        _check(_lib.ckks_prof_read(ctx.handle, k, C.byref(ms), C.byref(n)))
        if n.value:
            out[_lib.ckks_prof_kind_name(k).decode()] = (ms.value, n.value)
    return out


def ckks_workspace_bytes(ctx, op, batch, nlimbs, n1=0):
    return int(_lib.ckks_workspace_bytes(ctx.handle, op, batch, nlimbs, n1))


def ckks_ntt(ctx, data, npoly, limb_ids):
    ids, n = _ids(limb_ids)
    _check(_lib.ckks_ntt(ctx.handle, _ptr(data, "data", ctx, npoly * len(limb_ids) * ctx.N), npoly, ids, n, _stream()))


def ckks_intt(ctx, data, npoly, limb_ids):
    ids, n = _ids(limb_ids)
    _check(_lib.ckks_intt(ctx.handle, _ptr(data, "data", ctx, npoly * len(limb_ids) * ctx.N), npoly, ids, n, _stream()))


def ckks_automorph(ctx, out, inp, npoly, limb_ids, galois_elt, eval_domain):
    ids, n = _ids(limb_ids)
    e = npoly * len(limb_ids) * ctx.N
    _check(_lib.ckks_automorph(ctx.handle, _ptr(out, "out", ctx, e), _ptr(inp, "in", ctx, e), npoly, ids, n, galois_elt,
                               1 if eval_domain else 0, _stream()))


def ckks_keyswitch(ctx, ks_out, d, B, nlimbs, evk, galois_elt, dnum, ws):
    e = B * nlimbs * ctx.N
    _check(_lib.ckks_keyswitch(ctx.handle, _ptr(ks_out, "ks_out", ctx, 2 * e), _ptr(d, "d", ctx, e), B, nlimbs,
                               _ptr(evk, "evk", ctx, _key_elems(ctx)), galois_elt, dnum, _ptr(ws, "ws", ctx),
                               ws.numel() * 8, _stream()))


def ckks_hrot(ctx, ct_out, ct_in, B, nlimbs, galois_elt, evk_rot, ws):
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hrot(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e), B, nlimbs, galois_elt,
                          _ptr(evk_rot, "evk_rot", ctx, _key_elems(ctx)), _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_noalloc_scratch_bytes():
    return int(_lib.ckks_noalloc_scratch_bytes())


def ckks_hrot_noalloc(ctx, ct_out, ct_in, B, nlimbs, galois_elt, evk_rot):
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hrot_noalloc(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e), B, nlimbs,
                                  galois_elt, _ptr(evk_rot, "evk_rot", ctx, _key_elems(ctx)), _stream()))


def ckks_hmult_relin(ctx, ct_out, ct_a, ct_b, B, nlimbs, evk_mult, ws):
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hmult_relin(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_a, "ct_a", ctx, e),
                                 _ptr(ct_b, "ct_b", ctx, e), B, nlimbs, _ptr(evk_mult, "evk_mult", ctx, _key_elems(ctx)),
                                 _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_tensor_acc(ctx, d_out, ct_a, ct_b, d_acc, B, nlimbs):
    e = B * nlimbs * ctx.N
    _check(_lib.ckks_tensor_acc(ctx.handle, _ptr(d_out, "d_out", ctx, 3 * e), _ptr(ct_a, "ct_a", ctx, 2 * e),
                                _ptr(ct_b, "ct_b", ctx, 2 * e),
                                None if d_acc is None else _ptr(d_acc, "d_acc", ctx, 3 * e), B, nlimbs, _stream()))


def ckks_relin(ctx, ct_out, d_in, B, nlimbs, evk_mult, ws):
    e = B * nlimbs * ctx.N
    _check(_lib.ckks_relin(ctx.handle, _ptr(ct_out, "ct_out", ctx, 2 * e), _ptr(d_in, "d_in", ctx, 3 * e), B, nlimbs,
                           _ptr(evk_mult, "evk_mult", ctx, _key_elems(ctx)), _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_hrot_hoisted(ctx, ct_out, ct_in, B, nlimbs, galois_elts, evks, ws):
    R = len(galois_elts)
    if len(evks) != R:
        raise ValueError("need one key per Galois element")
    gs, _ = _ids(galois_elts)
    keys = (C.c_void_p * max(1, R))(*[_ptr(k, "evk", ctx, _key_elems(ctx)).value for k in evks])
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hrot_hoisted(ctx.handle, _ptr(ct_out, "ct_out", ctx, R * e), _ptr(ct_in, "ct_in", ctx, e), B, nlimbs,
                                  gs, keys, R, _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_hrot_sum(ctx, ct_out, ct_in, B, nlimbs, galois_elts, evks, ws):
    R = len(galois_elts)
    if len(evks) != R:
        raise ValueError("need one key per Galois element")
    gs, _ = _ids(galois_elts)
    keys = (C.c_void_p * max(1, R))(*[_ptr(k, "evk", ctx, _key_elems(ctx)).value for k in evks])
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hrot_sum(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e), B, nlimbs, gs, keys,
                              R, _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_hrot_add(ctx, ct_out, ct_in, ct_add, B, nlimbs, galois_elt, evk_rot, ws):
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hrot_add(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e),
                              _ptr(ct_add, "ct_add", ctx, e), B, nlimbs, galois_elt,
                              _ptr(evk_rot, "evk_rot", ctx, _key_elems(ctx)), _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_hrot_multi(ctx, ct_out, ct_in, B, nlimbs, galois_elts, evks, ws):
    if len(galois_elts) != B or len(evks) != B:
        raise ValueError("need one Galois element and one key per ciphertext")
    gs, _ = _ids(galois_elts)
    keys = (C.c_void_p * max(1, B))(*[_ptr(k, "evk", ctx, _key_elems(ctx)).value for k in evks])
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_hrot_multi(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e), B, nlimbs, gs, keys,
                                _ptr(ws, "ws", ctx), ws.numel() * 8, _stream()))


def ckks_pcmm_bsgs(ctx, ct_out, ct_in, B, nlimbs, pt_diag, n1, n2, stride, evk_baby, evk_giant, ws, hoisted=False):
    baby = (C.c_void_p * max(1, n1 - 1))(*[_ptr(k, "evk_baby", ctx, _key_elems(ctx)).value for k in evk_baby])
    giant = (C.c_void_p * max(1, n2 - 1))(*[_ptr(k, "evk_giant", ctx, _key_elems(ctx)).value for k in evk_giant])
    if len(evk_baby) != n1 - 1 or len(evk_giant) != n2 - 1:
        raise ValueError("need n1-1 baby-step keys and n2-1 giant-step keys")
    fn = {False: _lib.ckks_pcmm_bsgs, True: _lib.ckks_pcmm_bsgs_hoisted, "double": _lib.ckks_pcmm_bsgs_double_hoisted}[hoisted]
    e = B * 2 * nlimbs * ctx.N
    pt_limbs = nlimbs + ctx.np_ if hoisted == "double" else nlimbs   # the extended-basis schedule takes extended plaintexts
    _check(fn(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e), B, nlimbs,
              _ptr(pt_diag, "pt_diag", ctx, n1 * n2 * pt_limbs * ctx.N), n1, n2, stride, baby, giant, _ptr(ws, "ws", ctx),
              ws.numel() * 8, _stream()))


def ckks_rescale(ctx, ct_out, ct_in, B, nlimbs, ws):
    _check(_lib.ckks_rescale(ctx.handle, _ptr(ct_out, "ct_out", ctx, B * 2 * (nlimbs - 1) * ctx.N),
                             _ptr(ct_in, "ct_in", ctx, B * 2 * nlimbs * ctx.N), B, nlimbs, _ptr(ws, "ws", ctx),
                             ws.numel() * 8, _stream()))


def ckks_pmult(ctx, ct_out, ct_in, pt, B, nlimbs):
    e = B * 2 * nlimbs * ctx.N
    _check(_lib.ckks_pmult(ctx.handle, _ptr(ct_out, "ct_out", ctx, e), _ptr(ct_in, "ct_in", ctx, e),
                           _ptr(pt, "pt", ctx, nlimbs * ctx.N), B, nlimbs, _stream()))


def ckks_add(ctx, out, a, b, npoly, nlimbs):
    e = npoly * nlimbs * ctx.N
    _check(_lib.ckks_add(ctx.handle, _ptr(out, "out", ctx, e), _ptr(a, "a", ctx, e), _ptr(b, "b", ctx, e), npoly, nlimbs,
                         _stream()))


def ckks_pcmm_bsgs_hoisted(ctx, ct_out, ct_in, B, nlimbs, pt_diag, n1, n2, stride, evk_baby, evk_giant, ws):
    ckks_pcmm_bsgs(ctx, ct_out, ct_in, B, nlimbs, pt_diag, n1, n2, stride, evk_baby, evk_giant, ws, hoisted=True)


def ckks_pcmm_bsgs_double_hoisted(ctx, ct_out, ct_in, B, nlimbs, pt_ext, n1, n2, stride, evk_baby, evk_giant, ws):
    ckks_pcmm_bsgs(ctx, ct_out, ct_in, B, nlimbs, pt_ext, n1, n2, stride, evk_baby, evk_giant, ws, hoisted="double")
