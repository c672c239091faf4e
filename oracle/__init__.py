"""CPU oracle for Gumbel-max list sampling -- TEST INFRASTRUCTURE, not product.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It wraps oracle/libllc_ref.so (scalar fp64 C++, built by
oracle/build.py) and holds two small pure-Python companions used to pin it:
philox_py (big-integer Philox) and lml (the list matching lemma's bounds).
It imports nothing from the HIP package.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
LOGITS, PROBS, LOGW = 0, 1, 2

_lib = None


class _Args(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("K", ctypes.c_int64), ("V", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32),
        ("draft", ctypes.c_void_p),
        ("draft_stride_b", ctypes.c_int64), ("draft_stride_k", ctypes.c_int64),
        ("target", ctypes.c_void_p), ("target_stride_b", ctypes.c_int64),
        ("temp_target", ctypes.c_float),
        ("temp_draft", ctypes.c_void_p),
        ("temp_draft_all", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("accept", ctypes.c_void_p),
        ("match_k", ctypes.c_void_p),
        ("keyX", ctypes.c_void_p), ("keyY", ctypes.c_void_p),
        ("Yk", ctypes.c_void_p), ("keyYk", ctypes.c_void_p),
        ("gapX", ctypes.c_void_p), ("gapY", ctypes.c_void_p), ("gapYk", ctypes.c_void_p),
        ("threads", ctypes.c_int32), ("min_first", ctypes.c_int32),
    ]


class _VerifyArgs(ctypes.Structure):
    _fields_ = [
        ("S", ctypes.c_int64), ("L", ctypes.c_int64), ("K", ctypes.c_int64), ("V", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32),
        ("target", ctypes.c_void_p),
        ("stride_s", ctypes.c_int64), ("stride_j", ctypes.c_int64), ("stride_k", ctypes.c_int64),
        ("temp_target", ctypes.c_float),
        ("tokens", ctypes.c_void_p),
        ("tok_stride_s", ctypes.c_int64), ("tok_stride_j", ctypes.c_int64),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("row_stride_s", ctypes.c_int64), ("row_stride_j", ctypes.c_int64),
        ("strong", ctypes.c_int32),
        ("Y", ctypes.c_void_p), ("n_out", ctypes.c_void_p), ("active", ctypes.c_void_p),
        ("key", ctypes.c_void_p), ("gap", ctypes.c_void_p),
        ("threads", ctypes.c_int32), ("min_first", ctypes.c_int32),
    ]


class _TopmArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("K", ctypes.c_int64), ("Md", ctypes.c_int64), ("Mt", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32),
        ("draft_ids", ctypes.c_void_p), ("draft_val", ctypes.c_void_p),
        ("draft_stride_b", ctypes.c_int64), ("draft_stride_k", ctypes.c_int64),
        ("target_ids", ctypes.c_void_p), ("target_val", ctypes.c_void_p),
        ("target_stride_b", ctypes.c_int64),
        ("temp_target", ctypes.c_float),
        ("temp_draft", ctypes.c_void_p),
        ("temp_draft_all", ctypes.c_float),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("accept", ctypes.c_void_p),
        ("match_k", ctypes.c_void_p),
        ("keyX", ctypes.c_void_p), ("keyY", ctypes.c_void_p),
        ("gapX", ctypes.c_void_p), ("gapY", ctypes.c_void_p),
        ("threads", ctypes.c_int32),
    ]


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = ctypes.CDLL(path)
        _lib.llc_couple_ref.argtypes = [ctypes.POINTER(_Args)]
        _lib.llc_couple_ref.restype = ctypes.c_int
        _lib.llc_ref_philox4x32_10.argtypes = [ctypes.c_void_p] * 3
        _lib.llc_ref_philox4x32_10.restype = None
        _lib.llc_ref_shared_word.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32,
                                             ctypes.c_uint64]
        _lib.llc_ref_shared_word.restype = ctypes.c_uint32
        _lib.llc_ref_race_time.argtypes = [ctypes.c_uint32]
        _lib.llc_ref_race_time.restype = ctypes.c_double
        _lib.llc_ref_threads.restype = ctypes.c_int
        _lib.llc_ref_aux_word.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32]
        _lib.llc_ref_aux_word.restype = ctypes.c_uint32
        _lib.llc_ref_race_times.argtypes = [ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64,
                                            ctypes.c_uint64, ctypes.c_int64, ctypes.c_void_p]
        _lib.llc_ref_race_times.restype = None
        _lib.llc_couple_is_ref.argtypes = (
            [ctypes.c_int64] * 3 + [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                    ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64,
                                    ctypes.c_uint64] + [ctypes.c_void_p] * 8 + [ctypes.c_int32, ctypes.c_int32])
        _lib.llc_couple_is_ref.restype = ctypes.c_int
        _lib.llc_verify_ref.argtypes = [ctypes.POINTER(_VerifyArgs)]
        _lib.llc_verify_ref.restype = ctypes.c_int
        _lib.llc_compress_select_ref.argtypes = (
            [ctypes.c_int64] * 3 + [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64,
                                    ctypes.c_int64, ctypes.c_void_p, ctypes.c_int64, ctypes.c_uint64,
                                    ctypes.c_uint64] + [ctypes.c_void_p] * 9 + [ctypes.c_int32, ctypes.c_int32])
        _lib.llc_compress_select_ref.restype = ctypes.c_int
        _lib.llc_couple_topm_ref.argtypes = [ctypes.POINTER(_TopmArgs)]
        _lib.llc_couple_topm_ref.restype = ctypes.c_int
    return _lib


def philox4x32_10(ctr, key):
    """The C++ oracle's Philox4x32-10 block function: 4 counter words, 2 key words -> 4 words."""
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().llc_ref_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def shared_word(seed, row, k, i):
    return int(lib().llc_ref_shared_word(seed, row, k, i))


def race_time(x):
    return float(lib().llc_ref_race_time(x))


def threads():
    return int(lib().llc_ref_threads())


def aux_word(seed, row, i, which):
    return int(lib().llc_ref_aux_word(seed, row, i, which))


def race_times(seed, row0, n_rows, i, K, *, min_first=False):
    """S_i^(k) of rows row0 .. row0 + n_rows - 1 at index i: [n_rows, K] (see row_race_time)."""
    out = np.zeros((n_rows, K))
    lib().llc_ref_race_times(1 if min_first else 0, seed, row0, n_rows, i, K, out.ctypes.data)
    return out


def _check_input(arr, dtype):
    arr = np.asarray(arr)
    if dtype == F32:
        assert arr.dtype == np.float32, arr.dtype
    else:
        assert arr.dtype == np.uint16, "bf16 inputs are passed as their uint16 bit patterns"
    assert arr.strides[-1] == arr.itemsize, "last dimension must be contiguous"
    return arr


def couple(draft, target, K, *, dtype=F32, kind=LOGITS, temp_target=1.0, temp_draft=None,
           temp_draft_all=1.0, seed=0, row_offset=0, threads=0, partials=False, min_first=False):
    """Algorithm 1 on host arrays.

    draft: [B,V] (one proposal per row, shared by the K drafts) or [B,K,V];
    target: [B,V].  Returns a dict of numpy arrays: X [B,K], Y [B], accept [B],
    match_k [B], keyX [B,K], keyY [B], gapX [B,K], gapY [B] (relative gap to the
    runner-up), and with partials=True also Yk, keyYk, gapYk [B,K].
    min_first: the K race times of an index are drawn through their minimum (llc_ref.cpp,
    row_race_time) instead of one word per (k, i).
    """
    draft = _check_input(draft, dtype)
    target = _check_input(target, dtype)
    B, V = target.shape
    it = draft.itemsize
    if draft.ndim == 2:
        assert draft.shape == (B, V)
        sb, sk = draft.strides[0] // it, 0
    else:
        assert draft.shape == (B, K, V)
        sb, sk = draft.strides[0] // it, draft.strides[1] // it
    out = {
        "X": np.full((B, K), -2, np.int32), "Y": np.full(B, -2, np.int32),
        "accept": np.zeros(B, np.uint8), "match_k": np.full(B, -2, np.int32),
        "keyX": np.zeros((B, K)), "keyY": np.zeros(B),
        "gapX": np.zeros((B, K)), "gapY": np.zeros(B),
    }
    if partials:
        out.update(Yk=np.full((B, K), -2, np.int32), keyYk=np.zeros((B, K)),
                   gapYk=np.zeros((B, K)))
    a = _Args()
    a.B, a.K, a.V = B, K, V
    a.dtype, a.kind = dtype, kind
    a.draft, a.draft_stride_b, a.draft_stride_k = draft.ctypes.data, sb, sk
    a.target, a.target_stride_b = target.ctypes.data, target.strides[0] // it
    a.temp_target = temp_target
    td = None
    if temp_draft is not None:
        td = np.ascontiguousarray(temp_draft, dtype=np.float32)
        assert td.shape == (K,)
        a.temp_draft = td.ctypes.data
    a.temp_draft_all = temp_draft_all
    a.seed, a.row_offset = seed, row_offset
    for name in out:
        setattr(a, name, out[name].ctypes.data)
    a.threads = threads
    a.min_first = 1 if min_first else 0
    rc = lib().llc_couple_ref(ctypes.byref(a))
    if rc != 0:
        raise ValueError("llc_couple_ref rejected its arguments")
    return out


def couple_is(logw_enc, logw_dec, *, seed=0, row_offset=0, threads=0, min_first=False):
    """Importance-weight form (Appendix C): logw_enc [B,N], logw_dec [B,L,N], fp32."""
    enc = _check_input(logw_enc, F32)
    dec = _check_input(logw_dec, F32)
    B, N = enc.shape
    L = dec.shape[1]
    assert dec.shape == (B, L, N)
    out = {
        "X": np.full((B, L), -2, np.int32), "Y": np.full(B, -2, np.int32),
        "accept": np.zeros(B, np.uint8), "match_k": np.full(B, -2, np.int32),
        "keyX": np.zeros((B, L)), "keyY": np.zeros(B),
        "gapX": np.zeros((B, L)), "gapY": np.zeros(B),
    }
    rc = lib().llc_couple_is_ref(
        B, L, N, enc.ctypes.data, enc.strides[0] // 4, dec.ctypes.data, dec.strides[0] // 4,
        dec.strides[1] // 4, seed, row_offset, out["X"].ctypes.data, out["Y"].ctypes.data,
        out["accept"].ctypes.data, out["match_k"].ctypes.data, out["keyX"].ctypes.data,
        out["keyY"].ctypes.data, out["gapX"].ctypes.data, out["gapY"].ctypes.data, threads,
        1 if min_first else 0)
    if rc != 0:
        raise ValueError("llc_couple_is_ref rejected its arguments")
    return out


def verify(target, tokens, *, dtype=F32, kind=LOGITS, temp_target=1.0, seed=0, row_offset=0,
           row_stride_s=None, row_stride_j=1, strong=False, threads=0, min_first=False):
    """Algorithm 2's verification loop on host arrays.

    target: [S, L+1, K, V] (q^(j,k), position L is the bonus position); tokens: [S, L, K] int32
    draft tokens.  Position j of sequence s uses the stream of row
    row_offset + s*row_stride_s + j*row_stride_j (default row_stride_s = L+1).
    Returns Y [S, L+1] (-1 where not reached), n_out [S], active [S, K], key, gap [S, L+1].
    """
    target = _check_input(target, dtype)
    S, L1, K, V = target.shape
    L = L1 - 1
    tokens = np.ascontiguousarray(tokens, dtype=np.int32).reshape(S, L, K)
    it = target.itemsize
    out = {"Y": np.full((S, L1), -2, np.int32), "n_out": np.zeros(S, np.int32),
           "active": np.zeros((S, K), np.uint8), "key": np.zeros((S, L1)), "gap": np.zeros((S, L1))}
    a = _VerifyArgs()
    a.S, a.L, a.K, a.V = S, L, K, V
    a.dtype, a.kind = dtype, kind
    a.target = target.ctypes.data
    a.stride_s, a.stride_j, a.stride_k = (target.strides[0] // it, target.strides[1] // it,
                                          target.strides[2] // it)
    a.temp_target = temp_target
    a.tokens, a.tok_stride_s, a.tok_stride_j = tokens.ctypes.data, L * K, K
    a.seed, a.row_offset = seed, row_offset
    a.row_stride_s = L1 if row_stride_s is None else row_stride_s
    a.row_stride_j = row_stride_j
    a.strong = 1 if strong else 0
    for name in out:
        setattr(a, name, out[name].ctypes.data)
    a.threads = threads
    a.min_first = 1 if min_first else 0
    if lib().llc_verify_ref(ctypes.byref(a)) != 0:
        raise ValueError("llc_verify_ref rejected its arguments")
    return out


def couple_topm(draft_ids, draft_val, target_ids, target_val, K, *, dtype=F32, kind=LOGITS,
                temp_target=1.0, temp_draft=None, temp_draft_all=1.0, seed=0, row_offset=0, threads=0):
    """Algorithm 1 on candidate lists (Section 4.4).

    draft_ids / draft_val: [B,Md] (one list per row, shared by the K drafts) or [B,K,Md];
    target_ids / target_val: [B,Mt].  ids are int32 token ids (negative = empty slot).  Returns
    X [B,K], Y [B] (token ids), accept, match_k, keyX, keyY, gapX, gapY.
    """
    draft_val, target_val = _check_input(draft_val, dtype), _check_input(target_val, dtype)
    draft_ids = np.asarray(draft_ids)
    target_ids = np.asarray(target_ids)
    assert draft_ids.dtype == np.int32 and target_ids.dtype == np.int32
    assert draft_ids.shape == draft_val.shape and target_ids.shape == target_val.shape
    B, Mt = target_val.shape
    Md = draft_val.shape[-1]
    it = draft_val.itemsize
    assert draft_ids.strides[-1] == 4 and target_ids.strides[-1] == 4
    if draft_val.ndim == 2:
        sb, sk = draft_val.strides[0] // it, 0
        assert draft_ids.strides[0] // 4 == sb
    else:
        assert draft_val.shape[:2] == (B, K)
        sb, sk = draft_val.strides[0] // it, draft_val.strides[1] // it
        assert (draft_ids.strides[0] // 4, draft_ids.strides[1] // 4) == (sb, sk)
    assert target_ids.strides[0] // 4 == target_val.strides[0] // it
    out = {
        "X": np.full((B, K), -2, np.int32), "Y": np.full(B, -2, np.int32),
        "accept": np.zeros(B, np.uint8), "match_k": np.full(B, -2, np.int32),
        "keyX": np.zeros((B, K)), "keyY": np.zeros(B),
        "gapX": np.zeros((B, K)), "gapY": np.zeros(B),
    }
    a = _TopmArgs()
    a.B, a.K, a.Md, a.Mt = B, K, Md, Mt
    a.dtype, a.kind = dtype, kind
    a.draft_ids, a.draft_val = draft_ids.ctypes.data, draft_val.ctypes.data
    a.draft_stride_b, a.draft_stride_k = sb, sk
    a.target_ids, a.target_val = target_ids.ctypes.data, target_val.ctypes.data
    a.target_stride_b = target_val.strides[0] // it
    a.temp_target = temp_target
    td = None
    if temp_draft is not None:
        td = np.ascontiguousarray(temp_draft, dtype=np.float32)
        assert td.shape == (K,)
        a.temp_draft = td.ctypes.data
    a.temp_draft_all = temp_draft_all
    a.seed, a.row_offset = seed, row_offset
    for name in out:
        setattr(a, name, out[name].ctypes.data)
    a.threads = threads
    if lib().llc_couple_topm_ref(ctypes.byref(a)) != 0:
        raise ValueError("llc_couple_topm_ref rejected its arguments")
    return out


def compress_select(logw_enc, logw_dec, bins, *, seed=0, row_offset=0, threads=0, shared_race=False):
    """Index selection of the compression scheme with bins (Section 5.1 / Appendix C).

    logw_enc [B,N], logw_dec [B,L,N] fp32, bins [B,N] uint8.  Returns Y, message (the bin of Y),
    X [B,L] (drawn among the candidates of that bin), accept, match_k, keys and gaps.
    shared_race=True: the baseline of Section 5.3 (all decoders use the first set of race times)."""
    enc = _check_input(logw_enc, F32)
    dec = _check_input(logw_dec, F32)
    bins = np.asarray(bins)
    assert bins.dtype == np.uint8 and bins.strides[-1] == 1
    B, N = enc.shape
    L = dec.shape[1]
    assert dec.shape == (B, L, N) and bins.shape == (B, N)
    out = {
        "X": np.full((B, L), -2, np.int32), "Y": np.full(B, -2, np.int32),
        "message": np.full(B, -2, np.int32),
        "accept": np.zeros(B, np.uint8), "match_k": np.full(B, -2, np.int32),
        "keyX": np.zeros((B, L)), "keyY": np.zeros(B),
        "gapX": np.zeros((B, L)), "gapY": np.zeros(B),
    }
    rc = lib().llc_compress_select_ref(
        B, L, N, enc.ctypes.data, enc.strides[0] // 4, dec.ctypes.data, dec.strides[0] // 4,
        dec.strides[1] // 4, bins.ctypes.data, bins.strides[0], seed, row_offset,
        out["X"].ctypes.data, out["Y"].ctypes.data, out["message"].ctypes.data,
        out["accept"].ctypes.data, out["match_k"].ctypes.data, out["keyX"].ctypes.data,
        out["keyY"].ctypes.data, out["gapX"].ctypes.data, out["gapY"].ctypes.data, threads,
        1 if shared_race else 0)
    if rc != 0:
        raise ValueError("llc_compress_select_ref rejected its arguments")
    return out
