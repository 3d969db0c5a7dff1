"""ctypes binding of libcachemir: argument marshalling only.

Function names follow include/cachemir.h without the cm_ prefix.  Device memory of
ciphertexts and plaintexts is owned by torch tensors (int64 views of the 64-bit words); the
library is handed their data pointers and the current torch HIP stream.  Nothing here computes:
if libcachemir.so is missing the import fails (build it with python -m
paper_2602_11470_amd.build)."""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcachemir.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not built: run python -m paper_2602_11470_amd.build")
lib = C.CDLL(LIB_PATH)

CM_QK, CM_SV, CM_QK_GROUP, CM_SV_GROUP, CM_KV_INDEX = 0, 1, 2, 3, 4
CM_VMM_RAISED_SUMS, CM_VMM_DIRECT_GIANTS, CM_VMM_TOKEN_BATCH, CM_VMM_UNROLLED_LADDERS = 1, 2, 4, 8
CM_KV_UNROLLED_LADDERS, CM_KV_KEY_INDEX = 1, 2
CM_OPT_EVK_STORED_A, CM_OPT_TWO_STEP_MASKS = 1, 2


class cm_params(C.Structure):
    _fields_ = [("n", C.c_int32), ("n_q", C.c_int32), ("n_p", C.c_int32), ("alpha", C.c_int32),
                ("q0_bits", C.c_int32), ("qi_bits", C.c_int32), ("p_bits", C.c_int32),
                ("hamming", C.c_int32), ("scale", C.c_double), ("sigma", C.c_double)]


class cm_ct(C.Structure):
    _fields_ = [("dev", C.c_void_p), ("level", C.c_int32), ("ncomp", C.c_int32), ("scale", C.c_double)]


class cm_pt(C.Structure):
    _fields_ = [("dev", C.c_void_p), ("level", C.c_int32), ("mont", C.c_int32), ("scale", C.c_double)]


_vp, _i32, _u64, _f64, _sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_double, C.c_size_t
_P = C.POINTER
_SIGS = {
    "cm_strerror": ([_i32], C.c_char_p),
    "cm_last_hip_error": ([], _i32),
    "cm_ctx_create": ([_P(cm_params), _P(_vp)], _i32),
    "cm_ctx_destroy": ([_vp], None),
    "cm_ctx_set_option": ([_vp, _i32, _i32], _i32),
    "cm_ctx_moduli": ([_vp, _vp], _i32),
    "cm_ct_words": ([_vp, _i32, _i32], _sz),
    "cm_pt_words": ([_vp, _i32], _sz),
    "cm_ctx_gauss_table": ([_vp, _vp], _i32),
    "cm_keygen_secret": ([_vp, _u64, _P(_vp)], _i32),
    "cm_sk_destroy": ([_vp], None),
    "cm_sk_coeffs": ([_vp, _vp, _vp], _i32),
    "cm_keygen_rotations": ([_vp, _vp, _vp, _sz, _i32, _u64, _P(_vp)], _i32),
    "cm_evk_destroy": ([_vp], None),
    "cm_evk_export": ([_vp, _vp, _i32, _i32, _i32, _i32, _vp], _i32),
    "cm_encode_coeffs": ([_vp, _vp, _vp, _sz, _f64, _vp], _i32),
    "cm_pt_from_coeffs": ([_vp, _vp, _i32, _f64, _P(cm_pt)], _i32),
    "cm_encode": ([_vp, _vp, _vp, _sz, _i32, _f64, _P(cm_pt)], _i32),
    "cm_encrypt": ([_vp, _vp, _P(cm_pt), _u64, _P(cm_ct)], _i32),
    "cm_decrypt": ([_vp, _vp, _P(cm_ct), _P(cm_pt)], _i32),
    "cm_decode": ([_vp, _P(cm_pt), _vp, _vp, _sz], _i32),
    "cm_ct_export": ([_vp, _P(cm_ct), _vp], _i32),
    "cm_pt_export": ([_vp, _P(cm_pt), _vp], _i32),
    "cm_add": ([_vp, _P(cm_ct), _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_mul_pt": ([_vp, _P(cm_ct), _P(cm_pt), _P(cm_ct), _vp], _i32),
    "cm_mul_ct": ([_vp, _P(cm_ct), _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_relinearize": ([_vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_rescale": ([_vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_rescale_static": ([_vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_level_drop": ([_vp, _P(cm_ct), _i32, _P(cm_ct), _vp], _i32),
    "cm_rotate": ([_vp, _vp, _P(cm_ct), _i32, _P(cm_ct), _vp], _i32),
    "cm_rotate_hoisted": ([_vp, _vp, _P(cm_ct), _vp, _sz, _P(cm_ct), _vp], _i32),
    "cm_vmm_plan_create": ([_vp, _i32, _i32, _i32, _i32, _i32, _f64, _vp, _P(_vp)], _i32),
    "cm_vmm_plan_create_from_coeffs": ([_vp, _i32, _i32, _i32, _i32, _i32, _f64, _vp, _P(_vp)], _i32),
    "cm_vmm_plan_create_ex": ([_vp, _i32, _i32, _i32, _i32, _i32, _f64, _vp, _vp, C.c_uint32, _P(_vp)], _i32),
    "cm_vmm_plan_destroy": ([_vp], None),
    "cm_vmm_plan_steps": ([_vp, _vp, _i32], _i32),
    "cm_vmm_plan_info": ([_vp, _P(_i32), _P(_i32), _P(_i32)], _i32),
    "cm_vmm_plan_diag_export": ([_vp, _vp, _i32, _i32, _vp], _i32),
    "cm_vmm_pt": ([_vp, _vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_vmm_pt_multi": ([_vp, _vp, _vp, _i32, _P(cm_ct), _vp, _vp], _i32),
    "cm_rope_create": ([_vp, _i32, _i32, _i32, _i32, _i32, _f64, _vp, _P(_vp)], _i32),
    "cm_inner_rot_create": ([_vp, _i32, _i32, _i32, _vp, _P(_vp)], _i32),
    "cm_rope_destroy": ([_vp], None),
    "cm_rope_steps": ([_vp, _vp, _i32], _i32),
    "cm_rope_apply": ([_vp, _vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_kv_create": ([_vp, _i32, _i32, _i32, _i32, _f64, _i32, _P(_vp)], _i32),
    "cm_kv_destroy": ([_vp], None),
    "cm_kv_steps": ([_vp, _vp, _i32], _i32),
    "cm_kv_tokens": ([_vp], _i32),
    "cm_kv_load": ([_vp, _vp, _i32, _i32, _P(cm_ct), _vp], _i32),
    "cm_kv_set_tokens": ([_vp, _i32], _i32),
    "cm_kv_set_shared_dims": ([_vp, _i32], _i32),
    "cm_kv_export": ([_vp, _vp, _i32, _i32, _vp], _i32),
    "cm_kv_set_mask": ([_vp, _i32, _vp], _i32),
    "cm_kv_append": ([_vp, _vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_kv_create_ex": ([_vp, _i32, _i32, _i32, _i32, _f64, _i32, C.c_uint32, _P(_vp)], _i32),
    "cm_kv_append_group": ([_vp, _vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_vmm_kv": ([_vp, _vp, _vp, _i32, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_gqa_create": ([_vp, _vp, _i32, _vp, _P(_vp)], _i32),
    "cm_gqa_destroy": ([_vp], None),
    "cm_gqa_steps": ([_vp, _vp, _i32], _i32),
    "cm_gqa_qk": ([_vp, _vp, _vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_gqa_sv": ([_vp, _vp, _vp, _vp, _P(cm_ct), _P(cm_ct), _vp], _i32),
    "cm_profile_enable": ([_vp, _i32], _i32),
    "cm_profile_get": ([_vp, _i32, _P(_f64), _P(_f64), _P(_f64)], _i32),
    "cm_ntt": ([_vp, _vp, _vp, _i32, _i32, _vp], _i32),
    "cm_keyswitch": ([_vp, _vp, _i32, _i32, _vp, _i32, _vp, _vp, _vp], _i32),
    "cm_hbm_probe": ([_i32, _u64, _i32, _P(_f64)], _i32),
}
for _name, (_args, _res) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.argtypes, _f.restype = _args, _res
EXPORTS = sorted(_SIGS)


class CachemirError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(f"libcachemir: {lib.cm_strerror(status).decode()} (status {status}, "
                         f"hip {lib.cm_last_hip_error()})")


def _chk(status):
    if status != 0:
        raise CachemirError(status)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _np(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


class Ct:
    """Ciphertext: torch-owned device words + the descriptor the library reads and writes."""

    def __init__(self, ctx, level, ncomp=2):
        self.ctx = ctx
        self.buf = torch.empty(lib.cm_ct_words(ctx.h, ctx.L, max(ncomp, 2)), dtype=torch.int64, device="cuda")
        self.d = cm_ct(self.buf.data_ptr(), level, ncomp, 0.0)

    level = property(lambda s: s.d.level)
    scale = property(lambda s: s.d.scale)
    ncomp = property(lambda s: s.d.ncomp)


class Pt:
    def __init__(self, ctx, level, mont):
        self.ctx = ctx
        self.buf = torch.empty(lib.cm_pt_words(ctx.h, level), dtype=torch.int64, device="cuda")
        self.d = cm_pt(self.buf.data_ptr(), level, 1 if mont else 0, 0.0)

    level = property(lambda s: s.d.level)
    scale = property(lambda s: s.d.scale)


class Context:
    def __init__(self, n, n_q, n_p, alpha, q0_bits, qi_bits, p_bits, scale, hamming=0, sigma=3.2):
        self.prm = cm_params(n, n_q, n_p, alpha, q0_bits, qi_bits, p_bits, hamming, scale, sigma)
        h = _vp()
        torch.cuda.init()
        _chk(lib.cm_ctx_create(C.byref(self.prm), C.byref(h)))
        self.h, self.n, self.S, self.L, self.K = h, n, n // 2, n_q - 1, n_p
        self.scale = scale

    def close(self):
        if self.h:
            lib.cm_ctx_destroy(self.h)
            self.h = None

    def set_option(self, option, value):
        _chk(lib.cm_ctx_set_option(self.h, option, int(value)))

    def moduli(self):
        out = np.empty(self.L + 1 + self.K, dtype=np.uint64)
        _chk(lib.cm_ctx_moduli(self.h, out.ctypes.data))
        return out

    def gauss_table(self):
        out = np.empty(19, dtype=np.uint64)
        _chk(lib.cm_ctx_gauss_table(self.h, out.ctypes.data))
        return out

    # keys
    def keygen_secret(self, seed):
        return SecretKey(self, seed)

    def keygen_rotations(self, sk, steps, seed, with_relin=False):
        return Evk(self, sk, steps, seed, with_relin)

    # plaintexts
    def encode_coeffs(self, z, scale):
        z = np.asarray(z)
        re = _np(z.real, np.float64)
        im = _np(z.imag, np.float64) if np.iscomplexobj(z) else None
        out = np.empty(self.n, dtype=np.int64)
        _chk(lib.cm_encode_coeffs(self.h, re.ctypes.data, im.ctypes.data if im is not None else None,
                                  len(re), scale, out.ctypes.data))
        return out

    def pt_from_coeffs(self, coeffs, level, scale, mont=False):
        pt = Pt(self, level, mont)
        c = _np(coeffs, np.int64)
        assert c.shape == (self.n,)
        _chk(lib.cm_pt_from_coeffs(self.h, c.ctypes.data, level, scale, C.byref(pt.d)))
        return pt

    def encode(self, z, level, scale=0.0, mont=False):
        pt = Pt(self, level, mont)
        z = np.asarray(z)
        re = _np(z.real, np.float64)
        im = _np(z.imag, np.float64) if np.iscomplexobj(z) else None
        _chk(lib.cm_encode(self.h, re.ctypes.data, im.ctypes.data if im is not None else None, len(re),
                           level, scale, C.byref(pt.d)))
        return pt

    def encrypt(self, sk, pt, seed):
        ct = Ct(self, pt.level)
        _chk(lib.cm_encrypt(self.h, sk.h, C.byref(pt.d), seed, C.byref(ct.d)))
        return ct

    def decrypt(self, sk, ct, nslots=None):
        """decrypt + decode: complex slot values."""
        pt = Pt(self, 1, False)
        _chk(lib.cm_decrypt(self.h, sk.h, C.byref(ct.d), C.byref(pt.d)))
        nslots = self.S if nslots is None else nslots
        re, im = np.empty(nslots), np.empty(nslots)
        _chk(lib.cm_decode(self.h, C.byref(pt.d), re.ctypes.data, im.ctypes.data, nslots))
        return re + 1j * im

    def ct_export(self, ct):
        out = np.empty((ct.ncomp, ct.level + 1, self.n), dtype=np.uint64)
        _chk(lib.cm_ct_export(self.h, C.byref(ct.d), out.ctypes.data))
        return out

    def pt_export(self, pt):
        out = np.empty((pt.level + 1, self.n), dtype=np.uint64)
        _chk(lib.cm_pt_export(self.h, C.byref(pt.d), out.ctypes.data))
        return out

    # ciphertext operations
    def add(self, a, b, out=None):
        out = out or Ct(self, a.level, a.ncomp)
        _chk(lib.cm_add(self.h, C.byref(a.d), C.byref(b.d), C.byref(out.d), _stream()))
        return out

    def mul_pt(self, a, pt, out=None):
        out = out or Ct(self, a.level, a.ncomp)
        _chk(lib.cm_mul_pt(self.h, C.byref(a.d), C.byref(pt.d), C.byref(out.d), _stream()))
        return out

    def mul_ct(self, a, b):
        out = Ct(self, a.level, 3)
        _chk(lib.cm_mul_ct(self.h, C.byref(a.d), C.byref(b.d), C.byref(out.d), _stream()))
        return out

    def relinearize(self, evk, a):
        out = Ct(self, a.level, 2)
        _chk(lib.cm_relinearize(self.h, evk.h, C.byref(a.d), C.byref(out.d), _stream()))
        return out

    def rescale(self, a):
        out = Ct(self, a.level - 1, a.ncomp)
        _chk(lib.cm_rescale(self.h, C.byref(a.d), C.byref(out.d), _stream()))
        return out

    def rescale_static(self, a, out=None):
        out = out or Ct(self, a.level - 1, a.ncomp)
        _chk(lib.cm_rescale_static(self.h, C.byref(a.d), C.byref(out.d), _stream()))
        return out

    def level_drop(self, a, level):
        out = Ct(self, level, a.ncomp)
        _chk(lib.cm_level_drop(self.h, C.byref(a.d), level, C.byref(out.d), _stream()))
        return out

    def rotate(self, evk, a, step, out=None):
        out = out or Ct(self, a.level)
        _chk(lib.cm_rotate(self.h, evk.h, C.byref(a.d), step, C.byref(out.d), _stream()))
        return out

    def rotate_hoisted(self, evk, a, steps):
        outs = [Ct(self, a.level) for _ in steps]
        arr = (cm_ct * len(steps))(*[o.d for o in outs])
        st = _np(steps, np.int32)
        _chk(lib.cm_rotate_hoisted(self.h, evk.h, C.byref(a.d), st.ctypes.data, len(steps), arr, _stream()))
        for o, d in zip(outs, arr):
            o.d = cm_ct(d.dev, d.level, d.ncomp, d.scale)
        return outs

    def keyswitch(self, evk, d, level, step=0, relin=False):
        """d: torch int64 [level+1, n] evaluation-domain polynomial; returns (ks0, ks1) tensors."""
        ks0, ks1 = torch.empty_like(d), torch.empty_like(d)
        _chk(lib.cm_keyswitch(self.h, evk.h, step, int(relin), d.data_ptr(), level, ks0.data_ptr(),
                              ks1.data_ptr(), _stream()))
        return ks0, ks1

    def ntt(self, data, mod_idx, inverse=False):
        idx = _np(mod_idx, np.int32)
        _chk(lib.cm_ntt(self.h, data.data_ptr(), idx.ctypes.data, len(idx), int(inverse), _stream()))

    def profile_enable(self, on=True):
        _chk(lib.cm_profile_enable(self.h, int(on)))

    def profile_get(self, family):
        """(launches, units, milliseconds) of one kernel family since profile_enable(True)."""
        a, b, c = _f64(), _f64(), _f64()
        _chk(lib.cm_profile_get(self.h, family, C.byref(a), C.byref(b), C.byref(c)))
        return a.value, b.value, c.value

    def vmm_plan(self, d_in, d_out, W=None, level=None, r_i=0, tau=0, pt_scale=0.0, coeffs=None, raised_sums=False,
                 direct_giants=False, token_batch=False, unrolled_ladders=False):
        return VmmPlan(self, d_in, d_out, W, self.L if level is None else level, r_i, tau, pt_scale, coeffs,
                       raised_sums, direct_giants, token_batch, unrolled_ladders)

    def vmm_pt(self, evk, plan, x, out=None):
        out = out or Ct(self, x.level - 1)
        _chk(lib.cm_vmm_pt(self.h, evk.h, plan.h, C.byref(x.d), C.byref(out.d), _stream()))
        return out

    def vmm_pt_multi(self, evk, plans, x, outs=None):
        """Products of one input with several plans of the same shape; the baby steps run once."""
        outs = outs or [Ct(self, x.level - 1) for _ in plans]
        hp = (_vp * len(plans))(*[p.h for p in plans])
        yp = (C.POINTER(cm_ct) * len(plans))(*[C.pointer(o.d) for o in outs])
        _chk(lib.cm_vmm_pt_multi(self.h, evk.h, hp, len(plans), C.byref(x.d), yp, _stream()))
        return outs

    def rope(self, heads, dim, level, token, tau=0, base=10000.0, coeffs=None):
        return Rope(self, heads, dim, level, token, tau, base, coeffs)

    def inner_rot(self, t, delta, level, coeffs=None):
        """Inner rotation by delta of the residues of every block of t slots; applied with rope_apply."""
        return Rope(self, 0, 0, level, 0, 0, 0.0, coeffs, inner=(t, delta))

    def rope_apply(self, evk, rope, x, out=None):
        out = out or Ct(self, x.level - 1)
        _chk(lib.cm_rope_apply(self.h, evk.h, rope.h, C.byref(x.d), C.byref(out.d), _stream()))
        return out

    def kv_create(self, heads, dim, level, scale=0.0, max_tokens=None, r_i=0, unrolled_ladders=False, shared_dims=1,
                  key_index=False):
        return KvCache(self, heads, dim, r_i, level, scale, max_tokens, unrolled_ladders, shared_dims, key_index)

    def gqa(self, kv, group, coeffs=None):
        return Gqa(self, kv, group, coeffs)

    def gqa_qk(self, evk, gqa, q):
        """group score ciphertexts (pass delta at index delta), two levels below the cache."""
        outs = [Ct(self, q.level - (2 if gqa.kv.key_index else 3)) for _ in range(gqa.group)]
        arr = (cm_ct * gqa.group)(*[o.d for o in outs])
        _chk(lib.cm_gqa_qk(self.h, evk.h, gqa.h, gqa.kv.h, C.byref(q.d), arr, _stream()))
        for o, d in zip(outs, arr):
            o.d = cm_ct(d.dev, d.level, d.ncomp, d.scale)
        return outs

    def gqa_sv(self, evk, gqa, scores):
        out = Ct(self, scores[0].level - 2)
        arr = (cm_ct * gqa.group)(*[s.d for s in scores])
        _chk(lib.cm_gqa_sv(self.h, evk.h, gqa.h, gqa.kv.h, arr, C.byref(out.d), _stream()))
        return out

    def vmm_kv(self, evk, kv, which, x):
        out = Ct(self, x.level - (1 if which in (CM_SV, CM_SV_GROUP) or kv.key_index else 2))
        _chk(lib.cm_vmm_kv(self.h, evk.h, kv.h, which, C.byref(x.d), C.byref(out.d), _stream()))
        return out


class SecretKey:
    def __init__(self, ctx, seed):
        self.ctx, self.h = ctx, _vp()
        _chk(lib.cm_keygen_secret(ctx.h, seed, C.byref(self.h)))

    def coeffs(self):
        out = np.empty(self.ctx.n, dtype=np.int8)
        _chk(lib.cm_sk_coeffs(self.ctx.h, self.h, out.ctypes.data))
        return out

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.cm_sk_destroy(self.h)
            self.h = None


class Evk:
    def __init__(self, ctx, sk, steps, seed, with_relin):
        self.ctx, self.h = ctx, _vp()
        st = _np(list(steps), np.int32)
        _chk(lib.cm_keygen_rotations(ctx.h, sk.h, st.ctypes.data, len(st), int(with_relin), seed, C.byref(self.h)))

    def export(self, step=0, relin=False, digit=0, comp=0):
        out = np.empty((self.ctx.L + 1 + self.ctx.K, self.ctx.n), dtype=np.uint64)
        _chk(lib.cm_evk_export(self.ctx.h, self.h, step, int(relin), digit, comp, out.ctypes.data))
        return out

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.cm_evk_destroy(self.h)
            self.h = None


class VmmPlan:
    def __init__(self, ctx, d_in, d_out, W, level, r_i, tau, pt_scale, coeffs, raised_sums=False, direct_giants=False,
                 token_batch=False, unrolled_ladders=False):
        self.ctx, self.h, self.level = ctx, _vp(), level
        direct_giants = direct_giants or unrolled_ladders
        raised_sums = raised_sums or direct_giants
        self.limbs = level + 1 + (ctx.K if raised_sums else 0)
        flags = (CM_VMM_RAISED_SUMS if raised_sums else 0) | (CM_VMM_DIRECT_GIANTS if direct_giants else 0) | \
                (CM_VMM_TOKEN_BATCH if token_batch else 0) | (CM_VMM_UNROLLED_LADDERS if unrolled_ladders else 0)
        if coeffs is not None:
            c = _np(coeffs, np.int64)
            _chk(lib.cm_vmm_plan_create_ex(ctx.h, d_in, d_out, r_i, tau, level, pt_scale, None, c.ctypes.data,
                                           flags, C.byref(self.h)))
        else:
            w = _np(W, np.float64)
            assert w.shape == (d_in, d_out)
            _chk(lib.cm_vmm_plan_create_ex(ctx.h, d_in, d_out, r_i, tau, level, pt_scale, w.ctypes.data, None,
                                           flags, C.byref(self.h)))
        a, b, c = _i32(), _i32(), _i32()
        _chk(lib.cm_vmm_plan_info(self.h, C.byref(a), C.byref(b), C.byref(c)))
        self.r_i, self.r_o, self.n_rotations = a.value, b.value, c.value

    def steps(self):
        n = lib.cm_vmm_plan_steps(self.h, None, 0)
        out = np.empty(n, dtype=np.int32)
        lib.cm_vmm_plan_steps(self.h, out.ctypes.data, n)
        return out.tolist()

    def diag_export(self, j, k):
        out = np.empty((self.limbs, self.ctx.n), dtype=np.uint64)
        _chk(lib.cm_vmm_plan_diag_export(self.ctx.h, self.h, j, k, out.ctypes.data))
        return out

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.cm_vmm_plan_destroy(self.h)
            self.h = None


class Rope:
    """The rotary embedding of a layout, or (inner=(t, delta)) the inner rotation of the residues of every block."""

    def __init__(self, ctx, heads, dim, level, token, tau, base, coeffs, inner=None):
        self.ctx, self.h = ctx, _vp()
        c = _np(coeffs, np.int64) if coeffs is not None else None
        cp = c.ctypes.data if c is not None else None
        if inner is not None:
            _chk(lib.cm_inner_rot_create(ctx.h, inner[0], inner[1], level, cp, C.byref(self.h)))
        else:
            _chk(lib.cm_rope_create(ctx.h, heads, dim, level, token, tau, base, cp, C.byref(self.h)))

    def steps(self):
        out = np.empty(2, dtype=np.int32)
        lib.cm_rope_steps(self.h, out.ctypes.data, 2)
        return out.tolist()

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.cm_rope_destroy(self.h)
            self.h = None


class Gqa:
    """Grouped-query attention on a cache of the KV heads (cm_gqa_*)."""

    def __init__(self, ctx, kv, group, coeffs=None):
        self.ctx, self.kv, self.group, self.h = ctx, kv, group, _vp()
        c = _np(coeffs, np.int64) if coeffs is not None else None
        _chk(lib.cm_gqa_create(ctx.h, kv.h, group, c.ctypes.data if c is not None else None, C.byref(self.h)))

    def steps(self):
        n = lib.cm_gqa_steps(self.h, None, 0)
        out = np.empty(n, dtype=np.int32)
        lib.cm_gqa_steps(self.h, out.ctypes.data, n)
        return out.tolist()

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.cm_gqa_destroy(self.h)
            self.h = None


class KvCache:
    def __init__(self, ctx, heads, dim, r_i, level, scale, max_tokens, unrolled_ladders=False, shared_dims=1, key_index=False):
        self.ctx, self.h, self.level, self.key_index = ctx, _vp(), level, key_index
        t = ctx.S // ((1 << (heads - 1).bit_length()) * dim)
        max_tokens = dim * t if max_tokens is None else max_tokens
        _chk(lib.cm_kv_create_ex(ctx.h, heads, dim, r_i, level, scale, max_tokens,
                                 (CM_KV_UNROLLED_LADDERS if unrolled_ladders else 0) | (CM_KV_KEY_INDEX if key_index else 0),
                                 C.byref(self.h)))
        if shared_dims != 1:
            self.set_shared_dims(shared_dims)

    def set_shared_dims(self, shared):
        _chk(lib.cm_kv_set_shared_dims(self.h, shared))

    def steps(self):
        n = lib.cm_kv_steps(self.h, None, 0)
        out = np.empty(n, dtype=np.int32)
        lib.cm_kv_steps(self.h, out.ctypes.data, n)
        return out.tolist()

    def tokens(self):
        return lib.cm_kv_tokens(self.h)

    def set_tokens(self, n):
        _chk(lib.cm_kv_set_tokens(self.h, n))

    def load(self, which, idx, ct):
        _chk(lib.cm_kv_load(self.ctx.h, self.h, which, idx, C.byref(ct.d), _stream()))

    def export(self, which, idx):
        out = np.empty((2, self.level + 1, self.ctx.n), dtype=np.uint64)
        _chk(lib.cm_kv_export(self.ctx.h, self.h, which, idx, out.ctypes.data))
        return out

    def set_mask(self, kind, coeffs):
        c = _np(coeffs, np.int64)
        _chk(lib.cm_kv_set_mask(self.h, kind, c.ctypes.data))

    def append(self, evk, k_new, v_new):
        _chk(lib.cm_kv_append(self.ctx.h, evk.h, self.h, C.byref(k_new.d), C.byref(v_new.d), _stream()))

    def append_group(self, evk, k_grp, v_grp):
        _chk(lib.cm_kv_append_group(self.ctx.h, evk.h, self.h, C.byref(k_grp.d), C.byref(v_grp.d), _stream()))

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.cm_kv_destroy(self.h)
            self.h = None


def config1():
    """Benchmark configuration 1: n = 4096, a 50-bit base prime, four 40-bit primes, one 60-bit
    special prime, one prime per key-switch digit, scale 2^40, uniform ternary secret."""
    return Context(4096, 5, 1, 1, 50, 40, 60, 2.0 ** 40, hamming=0)


CM_PROBE_READ, CM_PROBE_COPY, CM_PROBE_READ3_WRITE1 = 0, 1, 2


def hbm_probe(kind, nbytes=4 << 30, reps=5):
    """GB/s a plain streaming kernel of the given read/write mix reaches on the current device."""
    r = _f64()
    _chk(lib.cm_hbm_probe(kind, nbytes, reps, C.byref(r)))
    return r.value


def llama_ring(n_q=24, n_p=4, n=65536):
    """Configurations 2-4 (24 + 4 primes) and 5 (36 + 6): 50-bit primes, 60-bit special primes,
    six digits, scale 2^50, secret of Hamming weight 192."""
    return Context(n, n_q, n_p, n_q // 6, 50, 50, 60, 2.0 ** 50, hamming=192)
