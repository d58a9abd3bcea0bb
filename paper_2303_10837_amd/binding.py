"""Thin ctypes binding over libhe_fedavg.so (argument marshalling only).

Every function has the name and meaning of the C entry point declared in
include/he_fedavg.h; torch tensors supply device memory and the current HIP
stream.  There is no CPU fallback: if the library is missing, `load()` raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_LIB = None
LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhe_fedavg.so")


class HeError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"he_status {code}: {msg}")
        self.code = code


class he_params(C.Structure):
    _fields_ = [("log2_n", C.c_uint32), ("n_limbs", C.c_uint32), ("scale_bits", C.c_uint32),
                ("cbd_eta", C.c_uint32), ("primes", C.POINTER(C.c_uint32))]


_P = C.c_void_p
_SIGS = {
    "he_last_error": (C.c_char_p, []),
    "he_ctx_create": (C.c_int32, [C.POINTER(he_params), C.c_int, C.POINTER(_P)]),
    "he_ctx_destroy": (None, [_P]),
    "he_ctx_primes": (C.c_int32, [_P, C.POINTER(C.c_uint32)]),
    "he_ctx_ring_degree": (C.c_uint32, [_P]),
    "he_ctx_n_limbs": (C.c_uint32, [_P]),
    "he_ct_bytes": (C.c_uint64, [_P, C.c_uint32]),
    "he_keygen": (C.c_int32, [_P, C.c_uint64, C.POINTER(_P), C.POINTER(_P), _P]),
    "he_pk_destroy": (None, [_P]),
    "he_sk_destroy": (None, [_P]),
    "he_mask_create": (C.c_int32, [_P, C.c_uint64, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.c_uint64, C.POINTER(_P)]),
    "he_mask_from_bytes": (C.c_int32, [_P, C.c_uint64, _P, C.POINTER(_P), _P]),
    "he_mask_select_top": (C.c_int32, [_P, C.c_uint64, _P, C.c_double, C.POINTER(_P), _P]),
    "he_mask_n_runs": (C.c_uint64, [_P]),
    "he_mask_runs": (C.c_int32, [_P, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "he_mask_destroy": (None, [_P]),
    "he_mask_n_params": (C.c_uint64, [_P]),
    "he_mask_n_enc": (C.c_uint64, [_P]),
    "he_n_ct": (C.c_uint64, [_P, _P]),
    "he_encrypt_masked": (C.c_int32, [_P, _P, _P, C.c_uint64, C.c_uint32, _P, _P, _P, _P]),
    "he_encrypt_masked_static": (C.c_int32, [_P, _P, _P, C.c_uint64, C.c_uint32, _P, _P, _P, _P]),
    "he_aggregate": (C.c_int32, [_P, C.c_uint32, C.POINTER(C.c_double), C.POINTER(_P), C.POINTER(_P),
                                 C.c_uint64, C.c_uint64, _P, _P, _P]),
    "he_aggregate_begin": (C.c_int32, [_P, C.c_uint64, C.c_uint64, _P, _P, _P]),
    "he_aggregate_add": (C.c_int32, [_P, C.c_uint32, C.POINTER(C.c_double), C.POINTER(_P), C.POINTER(_P),
                                     C.c_uint64, C.c_uint64, _P, _P, _P]),
    "he_aggregate_add_first": (C.c_int32, [_P, C.c_uint32, C.POINTER(C.c_double), C.POINTER(_P), C.POINTER(_P),
                                           C.c_uint64, C.c_uint64, _P, _P, _P]),
    "he_aggregate_add_last": (C.c_int32, [_P, C.c_uint32, C.POINTER(C.c_double), C.POINTER(_P), C.POINTER(_P),
                                          C.c_uint64, C.c_uint64, _P, _P, _P, _P, _P]),
    "he_aggregate_finalize": (C.c_int32, [_P, C.c_uint64, C.c_uint64, _P, _P, _P, _P, _P]),
    "he_decrypt_merge": (C.c_int32, [_P, _P, _P, _P, _P, _P, _P]),
    "he_encrypt_masked_weighted": (C.c_int32, [_P, _P, _P, C.c_uint64, C.c_uint32, C.c_double, _P, _P, _P, _P]),
    "he_aggregate_sum": (C.c_int32, [_P, C.c_uint32, C.POINTER(_P), C.POINTER(_P), C.c_uint64, C.c_uint64, _P, _P, _P]),
    "he_decrypt_merge_level": (C.c_int32, [_P, _P, _P, C.c_uint32, _P, _P, _P, _P]),
    "he_debug_encode": (C.c_int32, [_P, _P, C.c_uint64, _P, _P]),
    "he_debug_encrypt_plain": (C.c_int32, [_P, _P, C.c_uint64, C.c_uint32, C.c_uint64, _P, C.c_uint64, _P, _P]),
    "he_debug_decrypt_residues": (C.c_int32, [_P, _P, _P, C.c_uint64, C.c_uint32, _P, _P]),
    "he_debug_decode": (C.c_int32, [_P, _P, C.c_uint64, C.c_uint32, _P, _P]),
    "he_debug_ntt": (C.c_int32, [_P, C.c_int, C.c_uint32, _P, C.c_uint64, _P]),
    "he_debug_export_keys": (C.c_int32, [_P, _P, _P, _P, _P, _P]),
    "he_debug_count_out_of_range": (C.c_int32, [_P, _P, C.c_uint64, C.POINTER(C.c_uint64), _P]),
    "he_debug_count_noncanonical": (C.c_int32, [_P, _P, C.c_uint64, C.c_uint32, C.POINTER(C.c_uint64), _P]),
    "he_debug_timing_enable": (C.c_int32, [_P, C.c_int]),
    "he_debug_timing_kernels": (C.c_uint32, []),
    "he_debug_timing_name": (C.c_char_p, [C.c_uint32]),
    "he_debug_timing_read": (C.c_int32, [_P, C.POINTER(C.c_double), C.POINTER(C.c_uint64)]),
}

EXPORTED_SYMBOLS = tuple(_SIGS)
HE_STATIC_SCRATCH_BYTES = 32 << 20      # include/he_fedavg.h


def load():
    """Loads the built library (raises if it has not been built)."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def _check(code):
    if code != 0:
        raise HeError(code, load().he_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous"
    if dtype is not None:
        assert t.dtype == dtype, f"expected {dtype}, got {t.dtype}"
    return C.c_void_p(t.data_ptr())


class Context:
    def __init__(self, log2_n, n_limbs, scale_bits=30, cbd_eta=21, primes=None, device=0):
        lib = load()
        arr = (C.c_uint32 * n_limbs)(*primes) if primes else None
        p = he_params(log2_n, n_limbs, scale_bits, cbd_eta, arr)
        h = _P()
        _check(lib.he_ctx_create(C.byref(p), device, C.byref(h)))
        self.h, self.device = h, torch.device("cuda", device)
        self.N, self.L = lib.he_ctx_ring_degree(h), lib.he_ctx_n_limbs(h)
        self.n_slots, self.scale_bits = self.N // 2, scale_bits
        out = (C.c_uint32 * self.L)()
        _check(lib.he_ctx_primes(h, out))
        self.primes = tuple(out)

    def close(self):
        if self.h:
            load().he_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def ct_words(self, level):
        return 2 * level * self.N


class KeyPair:
    def __init__(self, ctx, pk, sk):
        self.ctx, self.pk, self.sk = ctx, pk, sk

    def close(self):
        lib = load()
        if self.pk:
            lib.he_pk_destroy(self.pk)
            lib.he_sk_destroy(self.sk)
            self.pk = self.sk = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Mask:
    def __init__(self, ctx, h):
        lib = load()
        self.ctx, self.h = ctx, h
        self.P, self.P_enc = lib.he_mask_n_params(h), lib.he_mask_n_enc(h)
        self.n_ct = lib.he_n_ct(ctx.h, h)
        self.n_plain = self.P - self.P_enc

    def close(self):
        if self.h:
            load().he_mask_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def he_keygen(ctx, seed):
    pk, sk = _P(), _P()
    _check(load().he_keygen(ctx.h, seed, C.byref(pk), C.byref(sk), _stream()))
    return KeyPair(ctx, pk, sk)


def he_mask_create(ctx, P, starts, lens):
    n = len(starts)
    a = (C.c_uint64 * max(n, 1))(*[int(x) for x in starts])
    b = (C.c_uint64 * max(n, 1))(*[int(x) for x in lens])
    h = _P()
    _check(load().he_mask_create(ctx.h, P, a, b, n, C.byref(h)))
    return Mask(ctx, h)


def he_mask_from_bytes(ctx, mask_bytes):
    h = _P()
    _check(load().he_mask_from_bytes(ctx.h, mask_bytes.numel(), _ptr(mask_bytes, torch.uint8), C.byref(h), _stream()))
    return Mask(ctx, h)


def he_mask_select_top(ctx, sens, ratio):
    h = _P()
    _check(load().he_mask_select_top(ctx.h, sens.numel(), _ptr(sens, torch.float32), float(ratio), C.byref(h), _stream()))
    return Mask(ctx, h)


def he_mask_runs(mask):
    """(starts, lens) of the mask's run list as Python lists."""
    n = load().he_mask_n_runs(mask.h)
    a, b = (C.c_uint64 * max(n, 1))(), (C.c_uint64 * max(n, 1))()
    _check(load().he_mask_runs(mask.h, a, b))
    return list(a[:n]), list(b[:n])


def he_encrypt_masked(ctx, keys, mask, seed, client_id, w, ct_out=None, plain_out=None):
    """Returns (ct int32-viewed-uint32 [n_ct,2,L,N], plain float32[P-P_enc]).

    (seed, client_id) must be fresh for every call under one key pair (a new seed every round) and unrelated to the
    he_keygen seed: the encryption randomness depends on nothing else, and reusing a pair leaks the difference of the
    two plaintexts (see include/he_fedavg.h)."""
    if ct_out is None:
        ct_out = torch.empty((mask.n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device=ctx.device)
    if plain_out is None:
        plain_out = torch.empty((mask.n_plain,), dtype=torch.float32, device=ctx.device)
    assert w.numel() == mask.P and ct_out.numel() == mask.n_ct * 2 * ctx.L * ctx.N and plain_out.numel() == mask.n_plain
    _check(load().he_encrypt_masked(ctx.h, keys.pk, mask.h, seed, client_id, _ptr(w, torch.float32),
                                    _ptr(ct_out, torch.int32), _ptr(plain_out, torch.float32), _stream()))
    return ct_out, plain_out


def he_encrypt_masked_static(ctx, keys, mask, seed, client_id, w, ct_out, plain_out):
    """he_encrypt_masked that allocates nothing: the caller passes both outputs."""
    assert w.numel() == mask.P and ct_out.numel() == mask.n_ct * 2 * ctx.L * ctx.N and plain_out.numel() == mask.n_plain
    _check(load().he_encrypt_masked_static(ctx.h, keys.pk, mask.h, seed, client_id, _ptr(w, torch.float32),
                                           _ptr(ct_out, torch.int32) if mask.n_ct else None,
                                           _ptr(plain_out, torch.float32) if mask.n_plain else None, _stream()))
    return ct_out, plain_out


def he_encrypt_masked_weighted(ctx, keys, mask, seed, client_id, alpha, w, ct_out=None, plain_out=None):
    if ct_out is None:
        ct_out = torch.empty((mask.n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device=ctx.device)
    if plain_out is None:
        plain_out = torch.empty((mask.n_plain,), dtype=torch.float32, device=ctx.device)
    assert w.numel() == mask.P and ct_out.numel() == mask.n_ct * 2 * ctx.L * ctx.N and plain_out.numel() == mask.n_plain
    _check(load().he_encrypt_masked_weighted(ctx.h, keys.pk, mask.h, seed, client_id, float(alpha), _ptr(w, torch.float32),
                                             _ptr(ct_out, torch.int32), _ptr(plain_out, torch.float32), _stream()))
    return ct_out, plain_out


def _ptr_array(tensors, dtype):
    arr = (_P * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = t.data_ptr() if t is not None and t.numel() else 0
        if t is not None and t.numel():
            assert t.is_cuda and t.is_contiguous() and t.dtype == dtype
    return arr


def he_aggregate(ctx, alphas, cts, plains, ct_out=None, plain_out=None):
    K = len(alphas)
    n_ct = cts[0].shape[0] if cts and cts[0] is not None else 0
    n_plain = plains[0].numel() if plains and plains[0] is not None else 0
    if ct_out is None:
        ct_out = torch.empty((n_ct, 2, ctx.L - 1, ctx.N), dtype=torch.int32, device=ctx.device)
    if plain_out is None:
        plain_out = torch.empty((n_plain,), dtype=torch.float32, device=ctx.device)
    a = (C.c_double * K)(*[float(x) for x in alphas])
    cp = _ptr_array(cts, torch.int32) if n_ct else None
    pp = _ptr_array(plains, torch.float32) if n_plain else None
    _check(load().he_aggregate(ctx.h, K, a, cp, pp, n_ct, n_plain, _ptr(ct_out) if n_ct else None,
                               _ptr(plain_out) if n_plain else None, _stream()))
    return ct_out, plain_out


def he_aggregate_sum(ctx, cts, plains, ct_out=None, plain_out=None):
    K = len(cts)
    n_ct = cts[0].shape[0] if cts and cts[0] is not None else 0
    n_plain = plains[0].numel() if plains and plains[0] is not None else 0
    if ct_out is None:
        ct_out = torch.empty((n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device=ctx.device)
    if plain_out is None:
        plain_out = torch.empty((n_plain,), dtype=torch.float32, device=ctx.device)
    cp = _ptr_array(cts, torch.int32) if n_ct else None
    pp = _ptr_array(plains, torch.float32) if n_plain else None
    _check(load().he_aggregate_sum(ctx.h, K, cp, pp, n_ct, n_plain, _ptr(ct_out) if n_ct else None,
                                   _ptr(plain_out) if n_plain else None, _stream()))
    return ct_out, plain_out


def he_aggregate_begin(ctx, n_ct, n_plain, acc_ct=None, acc_plain=None):
    if acc_ct is None:
        acc_ct = torch.empty((n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device=ctx.device)
    if acc_plain is None:
        acc_plain = torch.empty((n_plain,), dtype=torch.float64, device=ctx.device)
    _check(load().he_aggregate_begin(ctx.h, n_ct, n_plain, _ptr(acc_ct) if n_ct else None,
                                     _ptr(acc_plain) if n_plain else None, _stream()))
    return acc_ct, acc_plain


def he_aggregate_add(ctx, alphas, cts, plains, acc_ct, acc_plain):
    K = len(alphas)
    n_ct, n_plain = acc_ct.shape[0], acc_plain.numel()
    a = (C.c_double * K)(*[float(x) for x in alphas])
    cp = _ptr_array(cts, torch.int32) if n_ct else None
    pp = _ptr_array(plains, torch.float32) if n_plain else None
    _check(load().he_aggregate_add(ctx.h, K, a, cp, pp, n_ct, n_plain, _ptr(acc_ct) if n_ct else None,
                                   _ptr(acc_plain) if n_plain else None, _stream()))


def he_aggregate_add_first(ctx, alphas, cts, plains, acc_ct, acc_plain):
    """begin + add in one: the accumulators are written without being read."""
    K = len(alphas)
    n_ct, n_plain = acc_ct.shape[0], acc_plain.numel()
    a = (C.c_double * K)(*[float(x) for x in alphas])
    cp = _ptr_array(cts, torch.int32) if n_ct else None
    pp = _ptr_array(plains, torch.float32) if n_plain else None
    _check(load().he_aggregate_add_first(ctx.h, K, a, cp, pp, n_ct, n_plain, _ptr(acc_ct) if n_ct else None,
                                         _ptr(acc_plain) if n_plain else None, _stream()))


def he_aggregate_add_last(ctx, alphas, cts, plains, acc_ct, acc_plain, ct_out=None, plain_out=None):
    """add + finalize in one: returns (ct_out, plain_out); the accumulators hold nothing defined afterwards."""
    K = len(alphas)
    n_ct, n_plain = acc_ct.shape[0], acc_plain.numel()
    if ct_out is None:
        ct_out = torch.empty((n_ct, 2, ctx.L - 1, ctx.N), dtype=torch.int32, device=ctx.device)
    if plain_out is None:
        plain_out = torch.empty((n_plain,), dtype=torch.float32, device=ctx.device)
    a = (C.c_double * K)(*[float(x) for x in alphas])
    cp = _ptr_array(cts, torch.int32) if n_ct else None
    pp = _ptr_array(plains, torch.float32) if n_plain else None
    _check(load().he_aggregate_add_last(ctx.h, K, a, cp, pp, n_ct, n_plain, _ptr(acc_ct) if n_ct else None,
                                        _ptr(acc_plain) if n_plain else None, _ptr(ct_out) if n_ct else None,
                                        _ptr(plain_out) if n_plain else None, _stream()))
    return ct_out, plain_out


def he_aggregate_finalize(ctx, acc_ct, acc_plain, ct_out=None, plain_out=None):
    n_ct, n_plain = acc_ct.shape[0], acc_plain.numel()
    if ct_out is None:
        ct_out = torch.empty((n_ct, 2, ctx.L - 1, ctx.N), dtype=torch.int32, device=ctx.device)
    if plain_out is None:
        plain_out = torch.empty((n_plain,), dtype=torch.float32, device=ctx.device)
    _check(load().he_aggregate_finalize(ctx.h, n_ct, n_plain, _ptr(acc_ct) if n_ct else None,
                                        _ptr(acc_plain) if n_plain else None, _ptr(ct_out) if n_ct else None,
                                        _ptr(plain_out) if n_plain else None, _stream()))
    return ct_out, plain_out


def he_decrypt_merge(ctx, keys, mask, ct_glob, plain_glob, w_out=None):
    if w_out is None:
        w_out = torch.empty((mask.P,), dtype=torch.float32, device=ctx.device)
    assert ct_glob.numel() == mask.n_ct * 2 * (ctx.L - 1) * ctx.N
    assert (plain_glob.numel() if plain_glob is not None else 0) == mask.n_plain
    _check(load().he_decrypt_merge(ctx.h, keys.sk, mask.h, _ptr(ct_glob, torch.int32) if mask.n_ct else None,
                                   _ptr(plain_glob, torch.float32) if mask.n_plain else None,
                                   _ptr(w_out, torch.float32), _stream()))
    return w_out


def he_decrypt_merge_level(ctx, keys, mask, level, ct_glob, plain_glob, w_out=None):
    if w_out is None:
        w_out = torch.empty((mask.P,), dtype=torch.float32, device=ctx.device)
    assert ct_glob.numel() == mask.n_ct * 2 * level * ctx.N
    assert (plain_glob.numel() if plain_glob is not None else 0) == mask.n_plain
    _check(load().he_decrypt_merge_level(ctx.h, keys.sk, mask.h, level, _ptr(ct_glob, torch.int32) if mask.n_ct else None,
                                         _ptr(plain_glob, torch.float32) if mask.n_plain else None,
                                         _ptr(w_out, torch.float32), _stream()))
    return w_out


def he_debug_encode(ctx, slots):
    n_ct = slots.shape[0]
    out = torch.empty((n_ct, ctx.N), dtype=torch.int32, device=ctx.device)
    _check(load().he_debug_encode(ctx.h, _ptr(slots, torch.float32), n_ct, _ptr(out), _stream()))
    return out


def he_debug_encrypt_plain(ctx, keys, seed, client_id, first_ct, m):
    n_ct = m.shape[0]
    out = torch.empty((n_ct, 2, ctx.L, ctx.N), dtype=torch.int32, device=ctx.device)
    _check(load().he_debug_encrypt_plain(ctx.h, keys.pk, seed, client_id, first_ct, _ptr(m, torch.int32), n_ct,
                                         _ptr(out), _stream()))
    return out


def he_debug_decrypt_residues(ctx, keys, ct, level):
    n_ct = ct.shape[0]
    out = torch.empty((n_ct, level, ctx.N), dtype=torch.int32, device=ctx.device)
    _check(load().he_debug_decrypt_residues(ctx.h, keys.sk, _ptr(ct, torch.int32), n_ct, level, _ptr(out), _stream()))
    return out


def he_debug_decode(ctx, d, level):
    n_ct = d.shape[0]
    out = torch.empty((n_ct, ctx.n_slots), dtype=torch.float64, device=ctx.device)
    _check(load().he_debug_decode(ctx.h, _ptr(d, torch.int32), n_ct, level, _ptr(out), _stream()))
    return out


def he_debug_ntt(ctx, inverse, limb, polys):
    """In place on polys int32[batch, N]."""
    _check(load().he_debug_ntt(ctx.h, int(inverse), limb, _ptr(polys, torch.int32), polys.shape[0], _stream()))
    return polys


def he_debug_export_keys(ctx, keys):
    pk = torch.empty((2, ctx.L, ctx.N), dtype=torch.int32, device=ctx.device)
    sk = torch.empty((ctx.N,), dtype=torch.int32, device=ctx.device)
    _check(load().he_debug_export_keys(ctx.h, keys.pk, keys.sk, _ptr(pk), _ptr(sk), _stream()))
    return pk, sk


def he_debug_count_out_of_range(ctx, w):
    n = C.c_uint64(0)
    _check(load().he_debug_count_out_of_range(ctx.h, _ptr(w, torch.float32) if w.numel() else None, w.numel(), C.byref(n), _stream()))
    return int(n.value)


def he_debug_count_noncanonical(ctx, ct, level):
    n = C.c_uint64(0)
    _check(load().he_debug_count_noncanonical(ctx.h, _ptr(ct, torch.int32) if ct.numel() else None, ct.shape[0], level, C.byref(n), _stream()))
    return int(n.value)


def he_debug_timing_enable(ctx, on):
    _check(load().he_debug_timing_enable(ctx.h, int(on)))


def he_debug_timing_read(ctx):
    """{kernel name: (total ms, launches)} since the last read."""
    lib = load()
    n = lib.he_debug_timing_kernels()
    ms, cnt = (C.c_double * n)(), (C.c_uint64 * n)()
    _check(lib.he_debug_timing_read(ctx.h, ms, cnt))
    return {lib.he_debug_timing_name(i).decode(): (ms[i], cnt[i]) for i in range(n)}
