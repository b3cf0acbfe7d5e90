"""ctypes binding of libckks_hip.so: argument marshalling only.

Every function has the name of the C entry point it calls (see include/ckks.h).
Device buffers are torch tensors on the current HIP device (dtype int64 used as
raw 64-bit storage for uint64 residues); the stream is torch's current stream.
The library is loaded at import and the import fails loudly if it is missing:
there is no fallback path.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckks_hip.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2604_09975_amd.build` (hipcc, gfx950)")
lib = C.CDLL(LIB_PATH)

STEP_CONJ = -(2 ** 31)
_u64p, _u32p, _i32p, _vp = C.POINTER(C.c_uint64), C.POINTER(C.c_uint32), C.POINTER(C.c_int32), C.c_void_p


class Counters(C.Structure):
    _fields_ = [("key_switches", C.c_uint64), ("ptmuls", C.c_uint64), ("limb_ntts", C.c_uint64)]


class CkksError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"ckks error {code}: {msg}")
        self.code = code


lib.ckks_last_error.restype = C.c_char_p
_SIGS = {
    "ckks_find_primes": [C.c_uint32, C.c_uint32, C.c_uint32, _u64p],
    "ckks_params_create": [C.c_uint32, _u64p, C.c_uint32, _u64p, C.c_uint32, C.c_uint32, C.POINTER(_vp)],
    "ckks_params_root": [_vp, C.c_uint32, _u64p],
    "ckks_params_reserve": [_vp, C.c_uint64],
    "ckks_params_scratch_bytes": [_vp, _u64p],
    "ckks_ntt": [_vp, _vp, _u32p, C.c_uint32, C.c_uint32, _vp],
    "ckks_intt": [_vp, _vp, _u32p, C.c_uint32, C.c_uint32, _vp],
    "ckks_galois_elt": [_vp, C.c_int32, _u64p],
    "ckks_galois_key_load": [_vp, C.c_uint64, _vp, _vp, C.POINTER(_vp)],
    "ckks_galois_key_adopt": [_vp, C.c_uint64, _vp, _vp, C.POINTER(_vp)],
    "ckks_rotate_hoisted": [_vp, _vp, C.c_uint32, _i32p, C.c_uint32, C.POINTER(_vp), _vp, _vp],
    "ckks_weights_create": [_vp] + [C.c_uint32] * 6 + [C.POINTER(_vp)],
    "ckks_weights_set_diagonals": [_vp, C.c_uint32, C.c_uint32, _vp, _vp],
    "ckks_weights_set_bias": [_vp, _vp, C.c_uint64, _vp],
    "ckks_weights_load": [_vp] + [C.c_uint32] * 6 + [_vp, _vp, C.c_uint64, _vp, C.POINTER(_vp)],
    "ckks_ctpt_matmul": [_vp, _vp, _vp, C.POINTER(_vp), C.POINTER(_vp), _vp, C.c_uint32, _vp, C.POINTER(Counters),
                         _vp],
    "ckks_rescale": [_vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp],
    "ckks_rescale_static": [_vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp],
    "ckks_relin_key_load": [_vp, _vp, _vp, C.POINTER(_vp)],
    "ckks_ctmul": [_vp, _vp, _vp, C.c_uint32, _vp, _vp, _vp],
    "ckks_plain_expand": [_vp, C.c_uint32, _vp, C.c_uint32, _vp, _vp],
    "ckks_add": [_vp, _vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp],
    "ckks_ptmul": [_vp, _vp, C.c_uint32, _vp, _vp, _vp],
    "ckks_mod_switch_to_next": [_vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp],
    "ckks_shift_bank": [_vp, _vp, C.c_uint32, C.c_uint32, C.POINTER(C.c_int32), C.POINTER(_vp), _vp, _vp, _vp],
    "ckks_rot_first": [_vp, _vp, C.c_uint32, C.c_uint32, C.c_uint32, _vp, _vp, _vp, _vp, _vp, _vp],
    "ckks_probe_stream": [_vp, _vp, C.c_uint64, C.c_uint32, _vp],
    "ckks_probe_mulmod": [_vp, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, _vp, _vp],
    "ckks_encode": [_vp, _vp, C.c_uint32, C.c_double, C.c_uint32, _vp, _vp],
    "ckks_decode": [_vp, _vp, C.c_uint32, C.c_uint32, C.c_double, _vp, _vp],
}
for _n, _a in _SIGS.items():
    getattr(lib, _n).argtypes = _a
    getattr(lib, _n).restype = C.c_int
for _n in ("ckks_params_destroy", "ckks_galois_key_destroy", "ckks_weights_destroy"):
    getattr(lib, _n).argtypes = [_vp]
    getattr(lib, _n).restype = None


def _check(rc):
    if rc != 0:
        raise CkksError(rc, lib.ckks_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.element_size() == 8):
        raise TypeError("expected a contiguous 64-bit device tensor")
    return C.c_void_p(t.data_ptr())


def _u64arr(v):
    return (C.c_uint64 * max(len(v), 1))(*[int(x) for x in v])


def ckks_find_primes(bits, logN, count):
    out = (C.c_uint64 * count)()
    _check(lib.ckks_find_primes(bits, logN, count, out))
    return [int(x) for x in out]


class Handle:
    """Owns one library handle and destroys it once."""
    _destroy = None

    def __init__(self, h):
        self.h = h

    def close(self):
        if self.h:
            getattr(lib, self._destroy)(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Params(Handle):
    _destroy = "ckks_params_destroy"


class GaloisKey(Handle):
    _destroy = "ckks_galois_key_destroy"


class Weights(Handle):
    _destroy = "ckks_weights_destroy"


def ckks_params_create(logN, q, p, dnum):
    h = _vp()
    _check(lib.ckks_params_create(logN, _u64arr(q), len(q), _u64arr(p), len(p), dnum, C.byref(h)))
    P = Params(h)
    P.logN, P.N, P.L, P.K, P.dnum = logN, 1 << logN, len(q), len(p), dnum
    P.q, P.p = [int(x) for x in q], [int(x) for x in p]
    return P


def ckks_params_reserve(P, nbytes):
    _check(lib.ckks_params_reserve(P.h, int(nbytes)))


def ckks_params_scratch_bytes(P):
    out = C.c_uint64()
    _check(lib.ckks_params_scratch_bytes(P.h, C.byref(out)))
    return int(out.value)


def ckks_params_root(P, limb):
    out = C.c_uint64()
    _check(lib.ckks_params_root(P.h, limb, C.byref(out)))
    return int(out.value)


def _ntt(fn, P, d_data, limb_ids, batch):
    ids = (C.c_uint32 * max(len(limb_ids), 1))(*[int(x) for x in limb_ids])
    if d_data.numel() != batch * len(limb_ids) * P.N:
        raise ValueError("tensor size does not match batch * n_limbs * N")
    _check(fn(P.h, _dev(d_data), ids, len(limb_ids), batch, _stream()))
    return d_data


def ckks_ntt(P, d_data, limb_ids, batch):
    return _ntt(lib.ckks_ntt, P, d_data, limb_ids, batch)


def ckks_intt(P, d_data, limb_ids, batch):
    return _ntt(lib.ckks_intt, P, d_data, limb_ids, batch)


def ckks_galois_elt(P, step):
    out = C.c_uint64()
    _check(lib.ckks_galois_elt(P.h, STEP_CONJ if step == "conj" else int(step), C.byref(out)))
    return int(out.value)


def ckks_galois_key_load(P, galois_elt, d_key):
    if d_key.numel() != P.dnum * 2 * (P.L + P.K) * P.N:
        raise ValueError("key tensor must be [dnum][2][L+K][N]")
    h = _vp()
    _check(lib.ckks_galois_key_load(P.h, galois_elt, _dev(d_key), _stream(), C.byref(h)))
    k = GaloisKey(h)
    k.galois_elt = galois_elt
    return k


def ckks_galois_key_adopt(P, galois_elt, d_key):
    """Borrowing form: d_key is rewritten in place and must stay alive (the handle keeps a reference to it)."""
    if d_key.numel() != P.dnum * 2 * (P.L + P.K) * P.N:
        raise ValueError("key tensor must be [dnum][2][L+K][N]")
    h = _vp()
    _check(lib.ckks_galois_key_adopt(P.h, galois_elt, _dev(d_key), _stream(), C.byref(h)))
    k = GaloisKey(h)
    k.galois_elt = galois_elt
    k.buffer = d_key
    return k


def ckks_relin_key_load(P, d_key):
    if d_key.numel() != P.dnum * 2 * (P.L + P.K) * P.N:
        raise ValueError("key tensor must be [dnum][2][L+K][N]")
    h = _vp()
    _check(lib.ckks_relin_key_load(P.h, _dev(d_key), _stream(), C.byref(h)))
    k = GaloisKey(h)
    k.galois_elt = 1
    return k


def ckks_ctmul(P, d_ct_a, d_ct_b, level, relin_key, d_ct_out=None):
    if d_ct_a.numel() != 2 * level * P.N or d_ct_b.numel() != 2 * level * P.N:
        raise ValueError("ciphertexts must be [2][level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty((2, level, P.N), dtype=torch.int64, device=d_ct_a.device)
    _check(lib.ckks_ctmul(P.h, _dev(d_ct_a), _dev(d_ct_b), level, relin_key.h if relin_key is not None else None,
                          _dev(d_ct_out), _stream()))
    return d_ct_out


def _keyarr(keys):
    arr = (_vp * max(len(keys), 1))()
    for i, k in enumerate(keys):
        arr[i] = k.h if k is not None else None
    return arr


def ckks_rotate_hoisted(P, d_ct_in, level, steps, keys, d_ct_out=None):
    n = len(steps)
    if d_ct_in.numel() != 2 * level * P.N:
        raise ValueError("ciphertext must be [2][level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty((n, 2, level, P.N), dtype=torch.int64, device=d_ct_in.device)
    elif d_ct_out.numel() != n * 2 * level * P.N:
        raise ValueError("output must be [n_steps][2][level][N]")
    st = (C.c_int32 * max(n, 1))(*[STEP_CONJ if s == "conj" else int(s) for s in steps])
    _check(lib.ckks_rotate_hoisted(P.h, _dev(d_ct_in), level, st, n, _keyarr(keys), _dev(d_ct_out), _stream()))
    return d_ct_out


def ckks_weights_create(P, level, m, Cc, G, B_out, N1):
    h = _vp()
    _check(lib.ckks_weights_create(P.h, level, m, Cc, G, B_out, N1, C.byref(h)))
    w = Weights(h)
    w.level, w.m, w.C, w.G, w.B_out, w.N1, w.N2 = level, m, Cc, G, B_out, N1, Cc // N1
    w.N = P.N
    return w


def ckks_weights_set_diagonals(w, first, d_coeffs):
    count = d_coeffs.numel() // w.N
    if d_coeffs.numel() != count * w.N:
        raise ValueError("coefficients must be [count][N]")
    _check(lib.ckks_weights_set_diagonals(w.h, first, count, _dev(d_coeffs), _stream()))


def ckks_weights_set_bias(w, d_bias_coeffs, bias_mul):
    if d_bias_coeffs.numel() != w.B_out * w.N:
        raise ValueError("bias coefficients must be [B_out][N]")
    _check(lib.ckks_weights_set_bias(w.h, _dev(d_bias_coeffs), int(bias_mul), _stream()))


def ckks_weights_load(P, level, m, Cc, G, B_out, N1, d_coeffs, d_bias_coeffs=None, bias_mul=0):
    N2 = Cc // max(N1, 1)
    if d_coeffs.numel() != B_out * N2 * G * N1 * P.N:
        raise ValueError("coefficients must be [B_out][N2][G][N1][N]")
    if d_bias_coeffs is not None and d_bias_coeffs.numel() != B_out * P.N:
        raise ValueError("bias coefficients must be [B_out][N]")
    h = _vp()
    _check(lib.ckks_weights_load(P.h, level, m, Cc, G, B_out, N1, _dev(d_coeffs),
                                 _dev(d_bias_coeffs) if d_bias_coeffs is not None else None, int(bias_mul),
                                 _stream(), C.byref(h)))
    w = Weights(h)
    w.level, w.m, w.C, w.G, w.B_out, w.N1, w.N2 = level, m, Cc, G, B_out, N1, N2
    w.N = P.N
    return w


MATMUL_MERGED_GIANT = 1
MATMUL_RESCALE = 2
MATMUL_CONJ_PER_ACC = 4


def ckks_ctpt_matmul(P, w, d_ct_x, baby_keys, giant_keys, d_ct_y=None, conj_key=None, flags=0):
    if d_ct_x.numel() != w.G * 2 * w.level * P.N:
        raise ValueError("input must be [G][2][level][N]")
    if len(baby_keys) != w.N1 - 1 or len(giant_keys) != w.N2 - 1:
        raise ValueError("need N1-1 baby keys and N2-1 giant keys")
    out_level = w.level - 1 if flags & MATMUL_RESCALE else w.level
    if d_ct_y is None:
        d_ct_y = torch.empty((w.B_out, 2, max(out_level, 1), P.N), dtype=torch.int64, device=d_ct_x.device)
    elif d_ct_y.numel() != w.B_out * 2 * out_level * P.N:
        raise ValueError("output must be [B_out][2][level][N] ([B_out][2][level-1][N] with MATMUL_RESCALE)")
    cnt = Counters()
    _check(lib.ckks_ctpt_matmul(P.h, w.h, _dev(d_ct_x), _keyarr(baby_keys), _keyarr(giant_keys),
                                conj_key.h if conj_key is not None else None, flags, _dev(d_ct_y), C.byref(cnt),
                                _stream()))
    return d_ct_y, cnt


def ckks_rescale(P, d_ct_in, level_in, n_ct, d_ct_out=None):
    if d_ct_in.numel() != n_ct * 2 * level_in * P.N:
        raise ValueError("input must be [n_ct][2][level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty((n_ct, 2, max(level_in - 1, 1), P.N), dtype=torch.int64, device=d_ct_in.device)
    _check(lib.ckks_rescale(P.h, _dev(d_ct_in), level_in, n_ct, _dev(d_ct_out), _stream()))
    return d_ct_out


def ckks_rescale_static(P, d_ct_in, level_in, n_ct, d_ct_out):
    """ckks_rescale for callers that may not allocate: the caller passes the output, the library's scratch is a
    static device array (2 * n_ct * N words must fit it)."""
    if d_ct_in.numel() != n_ct * 2 * level_in * P.N or d_ct_out.numel() != n_ct * 2 * (level_in - 1) * P.N:
        raise ValueError("input must be [n_ct][2][level][N], output [n_ct][2][level-1][N]")
    _check(lib.ckks_rescale_static(P.h, _dev(d_ct_in), level_in, n_ct, _dev(d_ct_out), _stream()))
    return d_ct_out


def ckks_plain_expand(P, level, d_coeffs, d_out=None):
    count = d_coeffs.numel() // P.N
    if d_coeffs.numel() != count * P.N:
        raise ValueError("coefficients must be [count][N]")
    if d_out is None:
        d_out = torch.empty((count, level, P.N), dtype=torch.int64, device=d_coeffs.device)
    _check(lib.ckks_plain_expand(P.h, level, _dev(d_coeffs), count, _dev(d_out), _stream()))
    return d_out


def ckks_add(P, d_ct_a, d_ct_b, level, n_ct, d_ct_out=None):
    if d_ct_a.numel() != n_ct * 2 * level * P.N or d_ct_b.numel() != d_ct_a.numel():
        raise ValueError("ciphertexts must be [n_ct][2][level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty_like(d_ct_a)
    _check(lib.ckks_add(P.h, _dev(d_ct_a), _dev(d_ct_b), level, n_ct, _dev(d_ct_out), _stream()))
    return d_ct_out


def ckks_ptmul(P, d_ct, level, d_plain, d_ct_out=None):
    if d_ct.numel() != 2 * level * P.N or d_plain.numel() != level * P.N:
        raise ValueError("ciphertext must be [2][level][N], plaintext [level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty_like(d_ct)
    _check(lib.ckks_ptmul(P.h, _dev(d_ct), level, _dev(d_plain), _dev(d_ct_out), _stream()))
    return d_ct_out


def ckks_mod_switch_to_next(P, d_ct_in, level_in, n_ct, d_ct_out=None):
    if d_ct_in.numel() != n_ct * 2 * level_in * P.N:
        raise ValueError("input must be [n_ct][2][level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty((n_ct, 2, max(level_in - 1, 1), P.N), dtype=torch.int64, device=d_ct_in.device)
    _check(lib.ckks_mod_switch_to_next(P.h, _dev(d_ct_in), level_in, n_ct, _dev(d_ct_out), _stream()))
    return d_ct_out


def ckks_shift_bank(P, d_ct_in, level, steps, keys, d_masks, d_ct_out=None):
    """steps, keys: flat lists of 2*n_out entries (pair i at 2i, 2i+1); d_masks [n_out][2][level][N]."""
    n_out = len(steps) // 2
    if len(steps) != 2 * n_out or len(keys) != len(steps):
        raise ValueError("steps and keys must hold one pair per output")
    if d_ct_in.numel() != 2 * level * P.N or d_masks.numel() != n_out * 2 * level * P.N:
        raise ValueError("ciphertext must be [2][level][N], masks [n_out][2][level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty((n_out, 2, level, P.N), dtype=torch.int64, device=d_ct_in.device)
    st = (C.c_int32 * max(len(steps), 1))(*[STEP_CONJ if s == "conj" else int(s) for s in steps])
    _check(lib.ckks_shift_bank(P.h, _dev(d_ct_in), level, n_out, st, _keyarr(keys), _dev(d_masks), _dev(d_ct_out),
                               _stream()))
    return d_ct_out


def ckks_rot_first(P, d_ct_in, level, L_slots, tau, key_tau, key_wrap, d_mask_a, d_mask_b, d_ct_out=None):
    if d_ct_in.numel() != 2 * level * P.N or d_mask_a.numel() != level * P.N or d_mask_b.numel() != level * P.N:
        raise ValueError("ciphertext must be [2][level][N], masks [level][N]")
    if d_ct_out is None:
        d_ct_out = torch.empty((2, level, P.N), dtype=torch.int64, device=d_ct_in.device)
    _check(lib.ckks_rot_first(P.h, _dev(d_ct_in), level, L_slots, tau, key_tau.h if key_tau is not None else None,
                              key_wrap.h if key_wrap is not None else None, _dev(d_mask_a), _dev(d_mask_b),
                              _dev(d_ct_out), _stream()))
    return d_ct_out


lib.ckks_profile_begin.argtypes = [_vp]
lib.ckks_profile_begin.restype = C.c_int
lib.ckks_profile_end.argtypes = [_vp, _vp, C.POINTER(C.c_double), C.POINTER(C.c_uint32)]
lib.ckks_profile_end.restype = C.c_int


def ckks_profile_begin(P):
    _check(lib.ckks_profile_begin(P.h))


def ckks_profile_end(P):
    """-> (total ms of the diagonal multiply-accumulate kernel, launches) since ckks_profile_begin."""
    ms, n = C.c_double(), C.c_uint32()
    _check(lib.ckks_profile_end(P.h, _stream(), C.byref(ms), C.byref(n)))
    return ms.value, n.value


PROBE_COPY, PROBE_READ, PROBE_WRITE = 0, 1, 2
PROBE_INT64, PROBE_FP64, PROBE_INT64_LAZY = 0, 1, 2


def ckks_probe_stream(d_dst, d_src, mode):
    """One launch of the plain copy / read / write kernel over the whole of d_dst (and d_src)."""
    n = d_dst.numel() if mode == PROBE_WRITE else d_src.numel()
    if mode == PROBE_COPY and d_dst.numel() != d_src.numel():
        raise ValueError("copy needs equal sizes")
    _check(lib.ckks_probe_stream(_dev(d_dst), _dev(d_src) if d_src is not None else None, n, mode, _stream()))


def ckks_probe_mulmod(P, limb, kind, n_threads, iters, d_out=None):
    """-> d_out [n_threads]: XOR over c < 4 of ((4t + c + 1) mod 2^20) * psi^iters mod q."""
    if d_out is None:
        d_out = torch.empty(n_threads, dtype=torch.int64, device="cuda")
    elif d_out.numel() != n_threads:
        raise ValueError("d_out must hold n_threads words")
    _check(lib.ckks_probe_mulmod(P.h, limb, kind, n_threads, iters, _dev(d_out), _stream()))
    return d_out


ENCODE_REAL = 1


def _cdev(t):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == torch.complex128):
        raise TypeError("expected a contiguous complex128 device tensor")
    return C.c_void_p(t.data_ptr())


def ckks_encode(P, d_slots, scale, flags=0, d_coeffs=None):
    """d_slots complex128 [count][n] -> int64 [count][N], nearest integers to scale * m_k."""
    n = P.N // 2
    if d_slots.numel() % n:
        raise ValueError("slot vectors must have N/2 entries")
    count = d_slots.numel() // n
    if d_coeffs is None:
        d_coeffs = torch.empty((count, P.N), dtype=torch.int64, device=d_slots.device)
    elif d_coeffs.numel() != count * P.N:
        raise ValueError("d_coeffs must be [count][N]")
    _check(lib.ckks_encode(P.h, _cdev(d_slots), count, float(scale), flags, _dev(d_coeffs), _stream()))
    return d_coeffs


def ckks_decode(P, d_res, nlimbs, scale, d_slots=None):
    """d_res [count][nlimbs][N] coefficient-domain residues -> complex128 [count][n], m(zeta^(5^j)) / scale."""
    if nlimbs < 1 or d_res.numel() % (nlimbs * P.N):
        raise ValueError("d_res must be [count][nlimbs][N]")
    count = d_res.numel() // (nlimbs * P.N)
    if d_slots is None:
        d_slots = torch.empty((count, P.N // 2), dtype=torch.complex128, device=d_res.device)
    elif d_slots.numel() != count * (P.N // 2):
        raise ValueError("d_slots must be [count][N/2]")
    _check(lib.ckks_decode(P.h, _dev(d_res), nlimbs, count, float(scale), _cdev(d_slots), _stream()))
    return d_slots


# ---- key holder's side -------------------------------------------------------
class Secret(Handle):
    _destroy = "ckks_client_secret_destroy"


_i8p = C.POINTER(C.c_int8)
for _n, _a in {
    "ckks_client_secret_load": [_vp, _i8p, _vp, C.POINTER(_vp)],
    "ckks_client_galois_keygen": [_vp, _vp, C.c_uint64, _vp, _vp, _vp, _vp],
    "ckks_client_relin_keygen": [_vp, _vp, _vp, _vp, _vp, _vp],
    "ckks_client_encrypt": [_vp, _vp, C.c_uint32, _vp, _vp, _vp, _vp, _vp],
    "ckks_client_decrypt": [_vp, _vp, _vp, C.c_uint32, C.c_uint32, _vp, _vp],
}.items():
    getattr(lib, _n).argtypes = _a
    getattr(lib, _n).restype = C.c_int
lib.ckks_client_secret_destroy.argtypes = [_vp]
lib.ckks_client_secret_destroy.restype = None


def ckks_client_secret_load(P, s):
    """s: numpy int8 [N] ternary."""
    import numpy as np
    s = np.ascontiguousarray(s, dtype=np.int8)
    if s.shape != (P.N,):
        raise ValueError("secret must be int8 [N]")
    h = _vp()
    _check(lib.ckks_client_secret_load(P.h, s.ctypes.data_as(_i8p), _stream(), C.byref(h)))
    return Secret(h)


def ckks_client_galois_keygen(P, S, galois_elt, d_a, d_e, d_key=None):
    W = P.L + P.K
    if d_a.numel() != P.dnum * W * P.N or d_e.numel() != P.dnum * P.N:
        raise ValueError("a must be [dnum][L+K][N], e [dnum][N]")
    if d_key is None:
        d_key = torch.empty((P.dnum, 2, W, P.N), dtype=torch.int64, device=d_a.device)
    _check(lib.ckks_client_galois_keygen(P.h, S.h, galois_elt, _dev(d_a), _dev(d_e), _dev(d_key), _stream()))
    return d_key


def ckks_client_relin_keygen(P, S, d_a, d_e, d_key=None):
    W = P.L + P.K
    if d_a.numel() != P.dnum * W * P.N or d_e.numel() != P.dnum * P.N:
        raise ValueError("a must be [dnum][L+K][N], e [dnum][N]")
    if d_key is None:
        d_key = torch.empty((P.dnum, 2, W, P.N), dtype=torch.int64, device=d_a.device)
    _check(lib.ckks_client_relin_keygen(P.h, S.h, _dev(d_a), _dev(d_e), _dev(d_key), _stream()))
    return d_key


def ckks_client_encrypt(P, S, level, d_m, d_a, d_e, d_ct=None):
    if d_m.numel() != P.N or d_e.numel() != P.N or d_a.numel() != level * P.N:
        raise ValueError("m, e must be [N], a [level][N]")
    if d_ct is None:
        d_ct = torch.empty((2, level, P.N), dtype=torch.int64, device=d_a.device)
    _check(lib.ckks_client_encrypt(P.h, S.h, level, _dev(d_m), _dev(d_a), _dev(d_e), _dev(d_ct), _stream()))
    return d_ct


def ckks_client_decrypt(P, S, d_ct, level, nlimbs):
    if d_ct.numel() != 2 * level * P.N:
        raise ValueError("ciphertext must be [2][level][N]")
    out = torch.empty((nlimbs, P.N), dtype=torch.int64, device=d_ct.device)
    _check(lib.ckks_client_decrypt(P.h, S.h, _dev(d_ct), level, nlimbs, _dev(out), _stream()))
    return out
