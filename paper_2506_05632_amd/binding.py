"""ctypes binding of libllc_hip.so: argument marshalling only.

Every step of the sampler runs in the HIP kernels; torch supplies device
memory and the current stream.  There is no CPU fallback: if the library is
missing, `load()` raises.
"""
import ctypes
import os
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libllc_hip.so")

F32, BF16 = 0, 1
LOGITS, PROBS, LOGW = 0, 1, 2
FLAG_EXACT_SCAN = 1
FLAG_STRONG = 2
FLAG_DRY_RUN = 4
FLAG_SHARED_RACE = 8
FLAG_MIN_FIRST = 16  # the K race times of an index are drawn through their minimum (see llc.h)
FLAG_DRAFT_ONLY = 32  # the draft side alone: no target, no Y, no accept test

_KINDS = {"logits": LOGITS, "probs": PROBS, "logw": LOGW}
EXPORTS = ["llc_couple", "llc_couple_static", "llc_couple_is", "llc_couple_topm", "llc_compress_select", "llc_verify", "llc_lml_bound",
           "llc_couple_workspace_size", "llc_verify_workspace_size", "llc_lml_workspace_size", "llc_status_string",
           "llc_version"]


class LlcStats(ctypes.Structure):
    _fields_ = [("survivors", ctypes.c_ulonglong), ("exact_evals", ctypes.c_ulonglong),
                ("slow_blocks", ctypes.c_ulonglong), ("degenerate", ctypes.c_ulonglong),
                ("near_ties", ctypes.c_ulonglong)]


STATS_FIELDS = ("survivors", "exact_evals", "slow_blocks", "degenerate", "near_ties")


class CoupleArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("K", ctypes.c_int64), ("V", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32),
        ("draft", ctypes.c_void_p),
        ("draft_stride_b", ctypes.c_int64), ("draft_stride_k", ctypes.c_int64),
        ("target", ctypes.c_void_p), ("target_stride_b", ctypes.c_int64),
        ("temp_target", ctypes.c_float), ("temp_draft_all", ctypes.c_float),
        ("temp_draft", ctypes.c_void_p),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("accept", ctypes.c_void_p),
        ("match_k", ctypes.c_void_p), ("keyX", ctypes.c_void_p), ("keyY", ctypes.c_void_p),
        ("stats", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("flags", ctypes.c_int32), ("v_chunks", ctypes.c_int32), ("k_tile", ctypes.c_int32),
        ("ev_scan_begin", ctypes.c_void_p), ("ev_scan_end", ctypes.c_void_p),
    ]


class CoupleIsArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("L", ctypes.c_int64), ("N", ctypes.c_int64),
        ("logw_enc", ctypes.c_void_p), ("enc_stride_b", ctypes.c_int64),
        ("logw_dec", ctypes.c_void_p),
        ("dec_stride_b", ctypes.c_int64), ("dec_stride_l", ctypes.c_int64),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("accept", ctypes.c_void_p),
        ("match_l", ctypes.c_void_p), ("keyX", ctypes.c_void_p), ("keyY", ctypes.c_void_p),
        ("stats", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("flags", ctypes.c_int32), ("v_chunks", ctypes.c_int32), ("k_tile", ctypes.c_int32),
        ("ev_scan_begin", ctypes.c_void_p), ("ev_scan_end", ctypes.c_void_p),
    ]


class CompressSelectArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("L", ctypes.c_int64), ("N", ctypes.c_int64),
        ("logw_enc", ctypes.c_void_p), ("enc_stride_b", ctypes.c_int64),
        ("logw_dec", ctypes.c_void_p),
        ("dec_stride_b", ctypes.c_int64), ("dec_stride_l", ctypes.c_int64),
        ("bins", ctypes.c_void_p), ("bins_stride_b", ctypes.c_int64),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("accept", ctypes.c_void_p),
        ("message", ctypes.c_void_p), ("match_l", ctypes.c_void_p),
        ("keyX", ctypes.c_void_p), ("keyY", ctypes.c_void_p),
        ("stats", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("flags", ctypes.c_int32), ("v_chunks", ctypes.c_int32), ("k_tile", ctypes.c_int32),
        ("ev_scan_begin", ctypes.c_void_p), ("ev_scan_end", ctypes.c_void_p),
        ("cand", ctypes.c_void_p), ("cand_stride_b", ctypes.c_int64),
        ("side", ctypes.c_void_p), ("side_stride_b", ctypes.c_int64),
        ("source", ctypes.c_void_p),
        ("var_w_given_a", ctypes.c_float), ("var_t_given_a", ctypes.c_float),
        ("W", ctypes.c_void_p), ("A_hat", ctypes.c_void_p), ("sq_err", ctypes.c_void_p),
    ]


class TopmArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("K", ctypes.c_int64), ("Md", ctypes.c_int64), ("Mt", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32),
        ("draft_ids", ctypes.c_void_p), ("draft_val", ctypes.c_void_p),
        ("draft_stride_b", ctypes.c_int64), ("draft_stride_k", ctypes.c_int64),
        ("target_ids", ctypes.c_void_p), ("target_val", ctypes.c_void_p),
        ("target_stride_b", ctypes.c_int64),
        ("temp_target", ctypes.c_float), ("temp_draft_all", ctypes.c_float),
        ("temp_draft", ctypes.c_void_p),
        ("seed", ctypes.c_uint64), ("row_offset", ctypes.c_uint64),
        ("X", ctypes.c_void_p), ("Y", ctypes.c_void_p), ("accept", ctypes.c_void_p),
        ("match_k", ctypes.c_void_p), ("keyX", ctypes.c_void_p), ("keyY", ctypes.c_void_p),
        ("stats", ctypes.c_void_p), ("stream", ctypes.c_void_p),
        ("ev_begin", ctypes.c_void_p), ("ev_end", ctypes.c_void_p),
    ]


class VerifyArgs(ctypes.Structure):
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
        ("Y", ctypes.c_void_p), ("n_out", ctypes.c_void_p), ("active", ctypes.c_void_p),
        ("keyY", ctypes.c_void_p), ("Yk", ctypes.c_void_p), ("keyYk", ctypes.c_void_p),
        ("stats", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("flags", ctypes.c_int32), ("v_chunks", ctypes.c_int32), ("k_tile", ctypes.c_int32),
        ("ev_scan_begin", ctypes.c_void_p), ("ev_scan_end", ctypes.c_void_p),
    ]


LML_MAX_K = 8


class LmlArgs(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int64), ("V", ctypes.c_int64),
        ("dtype", ctypes.c_int32), ("kind", ctypes.c_int32),
        ("draft", ctypes.c_void_p), ("draft_stride_b", ctypes.c_int64),
        ("target", ctypes.c_void_p), ("target_stride_b", ctypes.c_int64),
        ("temp_target", ctypes.c_float), ("temp_draft", ctypes.c_float),
        ("n_k", ctypes.c_int32), ("k", ctypes.c_int32 * LML_MAX_K),
        ("bound", ctypes.c_void_p), ("relaxed", ctypes.c_void_p), ("tv", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("ev_begin", ctypes.c_void_p), ("ev_end", ctypes.c_void_p),
    ]


_lib = None


def load():
    """Load the HIP library (built by paper_2506_05632_amd/build.py); raise if it is not there."""
    global _lib
    if _lib is None:
        path = LIB_PATH
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run `python -m paper_2506_05632_amd.build` "
                               "(there is no CPU fallback)")
        lib = ctypes.CDLL(path)
        lib.llc_couple.argtypes = [ctypes.POINTER(CoupleArgs)]
        lib.llc_couple.restype = ctypes.c_int
        lib.llc_couple_static.argtypes = [ctypes.POINTER(CoupleArgs)]
        lib.llc_couple_static.restype = ctypes.c_int
        lib.llc_couple_is.argtypes = [ctypes.POINTER(CoupleIsArgs)]
        lib.llc_couple_is.restype = ctypes.c_int
        lib.llc_compress_select.argtypes = [ctypes.POINTER(CompressSelectArgs)]
        lib.llc_compress_select.restype = ctypes.c_int
        lib.llc_couple_topm.argtypes = [ctypes.POINTER(TopmArgs)]
        lib.llc_couple_topm.restype = ctypes.c_int
        lib.llc_verify.argtypes = [ctypes.POINTER(VerifyArgs)]
        lib.llc_verify.restype = ctypes.c_int
        lib.llc_lml_bound.argtypes = [ctypes.POINTER(LmlArgs)]
        lib.llc_lml_bound.restype = ctypes.c_int
        lib.llc_lml_workspace_size.argtypes = [ctypes.c_int64] * 2
        lib.llc_lml_workspace_size.restype = ctypes.c_size_t
        lib.llc_couple_workspace_size.argtypes = [ctypes.c_int64] * 3
        lib.llc_couple_workspace_size.restype = ctypes.c_size_t
        lib.llc_verify_workspace_size.argtypes = [ctypes.c_int64] * 4
        lib.llc_verify_workspace_size.restype = ctypes.c_size_t
        lib.llc_status_string.argtypes = [ctypes.c_int]
        lib.llc_status_string.restype = ctypes.c_char_p
        lib.llc_version.restype = ctypes.c_int
        _lib = lib
    return _lib


class LlcError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"llc error {code}: {load().llc_status_string(code).decode()}")


def llc_version() -> int:
    return load().llc_version()


def llc_status_string(code: int) -> str:
    return load().llc_status_string(code).decode()


def llc_couple_workspace_size(B: int, K: int, V: int) -> int:
    return load().llc_couple_workspace_size(B, K, V)


def llc_verify_workspace_size(S: int, L: int, K: int, V: int) -> int:
    return load().llc_verify_workspace_size(S, L, K, V)


def llc_lml_workspace_size(B: int, V: int) -> int:
    return load().llc_lml_workspace_size(B, V)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream_handle(device):
    return torch.cuda.current_stream(device).cuda_stream


def new_stats(device) -> torch.Tensor:
    """Zeroed 64-bit device counters laid out as llc_stats (survivors, exact_evals, slow_blocks,
    degenerate, near_ties)."""
    return torch.zeros(len(STATS_FIELDS), dtype=torch.int64, device=device)


def llc_couple(draft: torch.Tensor, target: torch.Tensor, K: int, *, kind="logits",
               temp_target: float = 1.0, temp_draft: float = 1.0,
               temp_draft_per_k: Optional[torch.Tensor] = None, seed: int = 0, row_offset: int = 0,
               want_keys: bool = False, want_match: bool = True, stats: Optional[torch.Tensor] = None,
               workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None,
               flags: int = 0, v_chunks: int = 0, k_tile: int = 0, scan_events=None,
               _static: bool = False) -> dict:
    """Algorithm 1 on device tensors.

    draft: [B,V] (the K drafts of a row share it) or [B,K,V]; target: [B,V]; both
    float32 or bfloat16 with a contiguous last dimension.  Returns device tensors
    X [B,K] int32, Y [B] int32, accept [B] uint8 and, if asked, match_k, keyX, keyY.
    With flags & FLAG_DRAFT_ONLY the target may be None: only X (and keyX) come back.
    The call is asynchronous on torch's current stream.
    """
    lib = load()
    draft_only = (flags & FLAG_DRAFT_ONLY) != 0
    if draft_only:
        target = None
    if not (draft.is_cuda and (draft_only or target.is_cuda)):
        raise ValueError("llc_couple needs device tensors (there is no CPU path)")
    if draft.dtype not in (torch.float32, torch.bfloat16) or not (draft_only or draft.dtype == target.dtype):
        raise ValueError("draft and target must both be float32 or both bfloat16")
    if draft.stride(-1) != 1 or not (draft_only or (target.stride(-1) == 1 and target.dim() == 2)):
        raise ValueError("last dimension must be contiguous; target must be [B,V]")
    B, V = (draft.shape[0], draft.shape[-1]) if draft_only else target.shape
    if draft.dim() == 2:
        if tuple(draft.shape) != (B, V):
            raise ValueError("draft must be [B,V] or [B,K,V]")
        sb, sk = draft.stride(0), 0
    else:
        if tuple(draft.shape) != (B, K, V):
            raise ValueError("draft must be [B,V] or [B,K,V]")
        sb, sk = draft.stride(0), draft.stride(1)
    dev = draft.device
    if out is None:
        out = {"X": torch.empty(B, K, dtype=torch.int32, device=dev)}
        if not draft_only:
            out["Y"] = torch.empty(B, dtype=torch.int32, device=dev)
            out["accept"] = torch.empty(B, dtype=torch.uint8, device=dev)
            if want_match:
                out["match_k"] = torch.empty(B, dtype=torch.int32, device=dev)
        if want_keys:
            out["keyX"] = torch.empty(B, K, dtype=torch.float32, device=dev)
            if not draft_only:
                out["keyY"] = torch.empty(B, dtype=torch.float32, device=dev)
    if workspace is None and not _static:
        workspace = new_workspace(B, K, V, dev)
    a = CoupleArgs()
    a.B, a.K, a.V = B, K, V
    a.dtype = F32 if draft.dtype == torch.float32 else BF16
    a.kind = _KINDS[kind]
    a.draft, a.draft_stride_b, a.draft_stride_k = draft.data_ptr(), sb, sk
    if not draft_only:
        a.target, a.target_stride_b = target.data_ptr(), target.stride(0)
    a.temp_target, a.temp_draft_all = temp_target, temp_draft
    if temp_draft_per_k is not None:
        if temp_draft_per_k.dtype != torch.float32 or temp_draft_per_k.numel() != K or not temp_draft_per_k.is_cuda:
            raise ValueError("temp_draft_per_k must be K float32 values on the device")
        a.temp_draft = temp_draft_per_k.data_ptr()
    a.seed, a.row_offset = seed, row_offset
    a.X, a.Y, a.accept = out["X"].data_ptr(), _ptr(out.get("Y")), _ptr(out.get("accept"))
    a.match_k = _ptr(out.get("match_k"))
    a.keyX, a.keyY = _ptr(out.get("keyX")), _ptr(out.get("keyY"))
    a.stats = _ptr(stats)
    if not _static:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream_handle(dev)
    a.flags, a.v_chunks, a.k_tile = flags, v_chunks, k_tile
    if scan_events is not None:
        a.ev_scan_begin, a.ev_scan_end = scan_events
    rc = lib.llc_couple_static(ctypes.byref(a)) if _static else lib.llc_couple(ctypes.byref(a))
    if rc != 0:
        raise LlcError(rc)
    return out


def llc_couple_static(draft: torch.Tensor, target: torch.Tensor, K: int, *, out: dict, **kw) -> dict:
    """llc_couple without a workspace and without any allocation: the partial results live in the
    library's own static device array (LLC_STATIC_SCRATCH_BYTES).  The caller passes the output
    tensors (`out` with X, Y, accept and optionally match_k, keyX, keyY), so that this wrapper
    allocates nothing either; the tensors' device must be the current device.  Calls on one GPU
    that may overlap in time race on the array."""
    if kw.get("workspace") is not None:
        raise ValueError("llc_couple_static takes no workspace")
    with torch.cuda.device(draft.device):
        return llc_couple(draft, target, K, out=out, _static=True, **kw)


def llc_couple_is(logw_enc: torch.Tensor, logw_dec: torch.Tensor, *, seed: int = 0,
                  row_offset: int = 0, want_keys: bool = False,
                  stats: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                  flags: int = 0, v_chunks: int = 0, k_tile: int = 0, scan_events=None) -> dict:
    """Importance-weight form: logw_enc [B,N], logw_dec [B,L,N], float32 device tensors."""
    lib = load()
    if not (logw_enc.is_cuda and logw_dec.is_cuda):
        raise ValueError("llc_couple_is needs device tensors (there is no CPU path)")
    if logw_enc.dtype != torch.float32 or logw_dec.dtype != torch.float32:
        raise ValueError("log-weights must be float32")
    B, N = logw_enc.shape
    L = logw_dec.shape[1]
    if tuple(logw_dec.shape) != (B, L, N) or logw_enc.stride(-1) != 1 or logw_dec.stride(-1) != 1:
        raise ValueError("logw_dec must be [B,L,N] with a contiguous last dimension")
    dev = logw_enc.device
    out = {"X": torch.empty(B, L, dtype=torch.int32, device=dev),
           "Y": torch.empty(B, dtype=torch.int32, device=dev),
           "accept": torch.empty(B, dtype=torch.uint8, device=dev),
           "match_k": torch.empty(B, dtype=torch.int32, device=dev)}
    if want_keys:
        out["keyX"] = torch.empty(B, L, dtype=torch.float32, device=dev)
        out["keyY"] = torch.empty(B, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = new_workspace(B, L, N, dev)
    a = CoupleIsArgs()
    a.B, a.L, a.N = B, L, N
    a.logw_enc, a.enc_stride_b = logw_enc.data_ptr(), logw_enc.stride(0)
    a.logw_dec, a.dec_stride_b, a.dec_stride_l = logw_dec.data_ptr(), logw_dec.stride(0), logw_dec.stride(1)
    a.seed, a.row_offset = seed, row_offset
    a.X, a.Y, a.accept = out["X"].data_ptr(), out["Y"].data_ptr(), out["accept"].data_ptr()
    a.match_l = out["match_k"].data_ptr()
    a.keyX, a.keyY = _ptr(out.get("keyX")), _ptr(out.get("keyY"))
    a.stats = _ptr(stats)
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream_handle(dev)
    a.flags, a.v_chunks, a.k_tile = flags, v_chunks, k_tile
    if scan_events is not None:
        a.ev_scan_begin, a.ev_scan_end = scan_events
    rc = lib.llc_couple_is(ctypes.byref(a))
    if rc != 0:
        raise LlcError(rc)
    return out


def llc_compress_select(logw_enc: torch.Tensor, logw_dec: torch.Tensor, bins: torch.Tensor, *,
                        seed: int = 0, row_offset: int = 0, want_keys: bool = False,
                        stats: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                        out: Optional[dict] = None, flags: int = 0, v_chunks: int = 0, k_tile: int = 0,
                        scan_events=None, shared_race: bool = False,
                        cand: Optional[torch.Tensor] = None, side: Optional[torch.Tensor] = None,
                        source: Optional[torch.Tensor] = None, var_w_given_a: float = 0.0,
                        var_t_given_a: float = 0.0) -> dict:
    """Binned index selection of the compression scheme: logw_enc [B,N], logw_dec [B,L,N]
    float32, bins [B,N] uint8, all on the device.  Returns Y, message, X [B,L], accept, match_k
    and, if asked, keyX, keyY.  shared_race: the baseline in which all decoders share one set of
    race times.  With cand [B,N] (the candidates U_i) also W [B,L]; with side [B,L] and the two
    variances also the MMSE estimates A_hat [B,L]; with source [B] also sq_err [B], the least
    squared error among the decoders.  Asynchronous on torch's current stream."""
    lib = load()
    if not (logw_enc.is_cuda and logw_dec.is_cuda and bins.is_cuda):
        raise ValueError("llc_compress_select needs device tensors (there is no CPU path)")
    if logw_enc.dtype != torch.float32 or logw_dec.dtype != torch.float32 or bins.dtype != torch.uint8:
        raise ValueError("log-weights must be float32, bins uint8")
    B, N = logw_enc.shape
    L = logw_dec.shape[1]
    if (tuple(logw_dec.shape) != (B, L, N) or tuple(bins.shape) != (B, N) or logw_enc.stride(-1) != 1
            or logw_dec.stride(-1) != 1 or bins.stride(-1) != 1):
        raise ValueError("logw_dec must be [B,L,N], bins [B,N], last dimensions contiguous")
    dev = logw_enc.device
    if out is None:
        out = {"X": torch.empty(B, L, dtype=torch.int32, device=dev),
               "Y": torch.empty(B, dtype=torch.int32, device=dev),
               "message": torch.empty(B, dtype=torch.int32, device=dev),
               "accept": torch.empty(B, dtype=torch.uint8, device=dev),
               "match_k": torch.empty(B, dtype=torch.int32, device=dev)}
        if want_keys:
            out["keyX"] = torch.empty(B, L, dtype=torch.float32, device=dev)
            out["keyY"] = torch.empty(B, dtype=torch.float32, device=dev)
        if cand is not None:
            out["W"] = torch.empty(B, L, dtype=torch.float32, device=dev)
            if side is not None:
                out["A_hat"] = torch.empty(B, L, dtype=torch.float32, device=dev)
                if source is not None:
                    out["sq_err"] = torch.empty(B, dtype=torch.float32, device=dev)
    for t, shape in ((cand, (B, N)), (side, (B, L)), (source, (B,))):
        if t is not None and (not t.is_cuda or t.dtype != torch.float32 or tuple(t.shape) != shape
                              or t.stride(-1) != 1):
            raise ValueError("cand [B,N], side [B,L], source [B]: float32 device tensors, last dimension contiguous")
    if workspace is None:
        workspace = new_workspace(B, L, N, dev)
    a = CompressSelectArgs()
    a.B, a.L, a.N = B, L, N
    a.logw_enc, a.enc_stride_b = logw_enc.data_ptr(), logw_enc.stride(0)
    a.logw_dec, a.dec_stride_b, a.dec_stride_l = logw_dec.data_ptr(), logw_dec.stride(0), logw_dec.stride(1)
    a.bins, a.bins_stride_b = bins.data_ptr(), bins.stride(0)
    a.seed, a.row_offset = seed, row_offset
    a.X, a.Y, a.accept = out["X"].data_ptr(), out["Y"].data_ptr(), out["accept"].data_ptr()
    a.message, a.match_l = _ptr(out.get("message")), _ptr(out.get("match_k"))
    a.keyX, a.keyY = _ptr(out.get("keyX")), _ptr(out.get("keyY"))
    a.stats = _ptr(stats)
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream_handle(dev)
    a.flags, a.v_chunks, a.k_tile = flags, v_chunks, k_tile
    if scan_events is not None:
        a.ev_scan_begin, a.ev_scan_end = scan_events
    if shared_race:
        a.flags |= FLAG_SHARED_RACE
    if cand is not None:
        a.cand, a.cand_stride_b = cand.data_ptr(), cand.stride(0)
    if side is not None:
        a.side, a.side_stride_b = side.data_ptr(), side.stride(0)
    a.source = _ptr(source)
    a.var_w_given_a, a.var_t_given_a = var_w_given_a, var_t_given_a
    a.W, a.A_hat, a.sq_err = _ptr(out.get("W")), _ptr(out.get("A_hat")), _ptr(out.get("sq_err"))
    rc = lib.llc_compress_select(ctypes.byref(a))
    if rc != 0:
        raise LlcError(rc)
    return out


def llc_couple_topm(draft_ids: torch.Tensor, draft_val: torch.Tensor, target_ids: torch.Tensor,
                    target_val: torch.Tensor, K: int, *, kind="logits", temp_target: float = 1.0,
                    temp_draft: float = 1.0, temp_draft_per_k: Optional[torch.Tensor] = None,
                    seed: int = 0, row_offset: int = 0, want_keys: bool = False,
                    stats: Optional[torch.Tensor] = None, out: Optional[dict] = None,
                    events=None) -> dict:
    """Algorithm 1 on candidate lists (top-M form) on device tensors.

    draft_ids / draft_val: [B,Md] (one list per row, shared by the K drafts) or [B,K,Md];
    target_ids / target_val: [B,Mt]; ids int32 (negative = empty slot), values float32 or
    bfloat16, ids and values of one side with identical strides.  Returns token ids X [B,K],
    Y [B], accept [B] uint8, match_k [B] and, if asked, keyX, keyY.  Asynchronous.
    """
    lib = load()
    for t in (draft_ids, draft_val, target_ids, target_val):
        if not t.is_cuda:
            raise ValueError("llc_couple_topm needs device tensors (there is no CPU path)")
    if draft_ids.dtype != torch.int32 or target_ids.dtype != torch.int32:
        raise ValueError("ids must be int32")
    if draft_val.dtype != target_val.dtype or draft_val.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("values must both be float32 or both bfloat16")
    if draft_ids.shape != draft_val.shape or target_ids.shape != target_val.shape or target_val.dim() != 2:
        raise ValueError("ids and values must have the same shape; the target side is [B,Mt]")
    if draft_ids.stride() != draft_val.stride() or target_ids.stride() != target_val.stride():
        raise ValueError("ids and values of one side must have identical strides")
    if draft_val.stride(-1) != 1 or target_val.stride(-1) != 1:
        raise ValueError("last dimension must be contiguous")
    B, Mt = target_val.shape
    Md = draft_val.shape[-1]
    if draft_val.dim() == 2:
        if draft_val.shape[0] != B:
            raise ValueError("draft lists must be [B,Md] or [B,K,Md]")
        sb, sk = draft_val.stride(0), 0
    else:
        if tuple(draft_val.shape[:2]) != (B, K):
            raise ValueError("draft lists must be [B,Md] or [B,K,Md]")
        sb, sk = draft_val.stride(0), draft_val.stride(1)
    dev = target_val.device
    if out is None:
        out = {"X": torch.empty(B, K, dtype=torch.int32, device=dev),
               "Y": torch.empty(B, dtype=torch.int32, device=dev),
               "accept": torch.empty(B, dtype=torch.uint8, device=dev),
               "match_k": torch.empty(B, dtype=torch.int32, device=dev)}
        if want_keys:
            out["keyX"] = torch.empty(B, K, dtype=torch.float32, device=dev)
            out["keyY"] = torch.empty(B, dtype=torch.float32, device=dev)
    a = TopmArgs()
    a.B, a.K, a.Md, a.Mt = B, K, Md, Mt
    a.dtype = F32 if draft_val.dtype == torch.float32 else BF16
    a.kind = _KINDS[kind]
    a.draft_ids, a.draft_val = draft_ids.data_ptr(), draft_val.data_ptr()
    a.draft_stride_b, a.draft_stride_k = sb, sk
    a.target_ids, a.target_val = target_ids.data_ptr(), target_val.data_ptr()
    a.target_stride_b = target_val.stride(0)
    a.temp_target, a.temp_draft_all = temp_target, temp_draft
    if temp_draft_per_k is not None:
        if temp_draft_per_k.dtype != torch.float32 or temp_draft_per_k.numel() != K or not temp_draft_per_k.is_cuda:
            raise ValueError("temp_draft_per_k must be K float32 values on the device")
        a.temp_draft = temp_draft_per_k.data_ptr()
    a.seed, a.row_offset = seed, row_offset
    a.X, a.Y, a.accept = out["X"].data_ptr(), _ptr(out.get("Y")), _ptr(out.get("accept"))
    a.match_k = _ptr(out.get("match_k"))
    a.keyX, a.keyY = _ptr(out.get("keyX")), _ptr(out.get("keyY"))
    a.stats = _ptr(stats)
    a.stream = _stream_handle(dev)
    if events is not None:
        a.ev_begin, a.ev_end = events
    rc = lib.llc_couple_topm(ctypes.byref(a))
    if rc != 0:
        raise LlcError(rc)
    return out


def llc_verify(target: torch.Tensor, tokens: torch.Tensor, *, kind="logits", temp_target: float = 1.0,
               seed: int = 0, row_offset: int = 0, row_stride_s: Optional[int] = None,
               row_stride_j: int = 1, want_keys: bool = False, want_partials: bool = False,
               stats: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
               out: Optional[dict] = None, flags: int = 0, v_chunks: int = 0, k_tile: int = 0,
               scan_events=None, strong: bool = False) -> dict:
    """Algorithm 2's verification loop on device tensors.

    target: [S, L+1, K, V] float32 or bfloat16 (q^(j,k); position L is the bonus position),
    tokens: [S, L, K] int32 draft tokens.  Position j of sequence s uses the random stream of
    row row_offset + s*row_stride_s + j*row_stride_j (default row_stride_s = L+1).  Returns
    device tensors Y [S, L+1] int32 (-1 where not reached), n_out [S] int32, active [S, K]
    uint8 and, if asked, keyY [S, L+1], Yk and keyYk [S, L+1, K].  Asynchronous on torch's
    current stream.
    """
    lib = load()
    if not target.is_cuda:
        raise ValueError("llc_verify needs device tensors (there is no CPU path)")
    if target.dtype not in (torch.float32, torch.bfloat16) or target.dim() != 4 or target.stride(-1) != 1:
        raise ValueError("target must be [S, L+1, K, V], float32 or bfloat16, last dimension contiguous")
    S, L1, K, V = target.shape
    L = L1 - 1
    dev = target.device
    if L > 0:
        if (not tokens.is_cuda or tokens.dtype != torch.int32 or tuple(tokens.shape) != (S, L, K)
                or tokens.stride(2) != 1):
            raise ValueError("tokens must be [S, L, K] int32 on the device, last dimension contiguous")
    if out is None:
        out = {"Y": torch.empty(S, L1, dtype=torch.int32, device=dev),
               "n_out": torch.empty(S, dtype=torch.int32, device=dev),
               "active": torch.empty(S, K, dtype=torch.uint8, device=dev)}
        if want_keys:
            out["keyY"] = torch.empty(S, L1, dtype=torch.float32, device=dev)
        if want_partials:
            out["Yk"] = torch.empty(S, L1, K, dtype=torch.int32, device=dev)
            out["keyYk"] = torch.empty(S, L1, K, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(llc_verify_workspace_size(S, L, K, V), 256), dtype=torch.uint8, device=dev)
    a = VerifyArgs()
    a.S, a.L, a.K, a.V = S, L, K, V
    a.dtype = F32 if target.dtype == torch.float32 else BF16
    a.kind = _KINDS[kind]
    a.target = target.data_ptr()
    a.stride_s, a.stride_j, a.stride_k = target.stride(0), target.stride(1), target.stride(2)
    a.temp_target = temp_target
    if L > 0:
        a.tokens, a.tok_stride_s, a.tok_stride_j = tokens.data_ptr(), tokens.stride(0), tokens.stride(1)
    a.seed, a.row_offset = seed, row_offset
    a.row_stride_s = L1 if row_stride_s is None else row_stride_s
    a.row_stride_j = row_stride_j
    a.Y, a.n_out = out["Y"].data_ptr(), out["n_out"].data_ptr()
    a.active, a.keyY = _ptr(out.get("active")), _ptr(out.get("keyY"))
    a.Yk, a.keyYk = _ptr(out.get("Yk")), _ptr(out.get("keyYk"))
    a.stats = _ptr(stats)
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream_handle(dev)
    if strong:
        flags |= FLAG_STRONG  # Appendix B: the pool runs over all K drafts' race times
    a.flags, a.v_chunks, a.k_tile = flags, v_chunks, k_tile
    if scan_events is not None:
        a.ev_scan_begin, a.ev_scan_end = scan_events
    rc = lib.llc_verify(ctypes.byref(a))
    if rc != 0:
        raise LlcError(rc)
    return out


def llc_lml_bound(draft: torch.Tensor, target: torch.Tensor, ks, *, kind="logits", temp_target: float = 1.0,
                  temp_draft: float = 1.0, want_relaxed: bool = True, want_tv: bool = True,
                  workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None, events=None) -> dict:
    """Theorem 1's lower bound on the matching probability for the list sizes `ks`, per row.

    draft, target: [B,V] device tensors (float32 or bfloat16, last dimension contiguous).
    Returns float64 tensors bound [B,len(ks)] and, if asked, relaxed [B,len(ks)] and tv [B].
    Asynchronous on the current stream; the workspace belongs to the call until it has finished.
    """
    lib = load()
    if not (draft.is_cuda and target.is_cuda):
        raise ValueError("llc_lml_bound needs device tensors (there is no CPU path)")
    if draft.dtype != target.dtype or draft.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("draft and target must both be float32 or both bfloat16")
    if draft.dim() != 2 or draft.shape != target.shape or draft.stride(1) != 1 or target.stride(1) != 1:
        raise ValueError("draft and target must be [B,V] with a contiguous last dimension")
    ks = [int(k) for k in ks]
    if not 1 <= len(ks) <= LML_MAX_K:
        raise ValueError(f"between 1 and {LML_MAX_K} list sizes")
    B, V = target.shape
    dev = target.device
    if out is None:
        out = {"bound": torch.empty(B, len(ks), dtype=torch.float64, device=dev)}
        if want_relaxed:
            out["relaxed"] = torch.empty(B, len(ks), dtype=torch.float64, device=dev)
        if want_tv:
            out["tv"] = torch.empty(B, dtype=torch.float64, device=dev)
    if workspace is None:
        workspace = torch.empty(max(llc_lml_workspace_size(B, V), 256), dtype=torch.uint8, device=dev)
    a = LmlArgs()
    a.B, a.V = B, V
    a.dtype = F32 if draft.dtype == torch.float32 else BF16
    a.kind = _KINDS[kind]
    a.draft, a.draft_stride_b = draft.data_ptr(), draft.stride(0)
    a.target, a.target_stride_b = target.data_ptr(), target.stride(0)
    a.temp_target, a.temp_draft = temp_target, temp_draft
    a.n_k = len(ks)
    for n, k in enumerate(ks):
        a.k[n] = k
    a.bound = out["bound"].data_ptr()
    a.relaxed, a.tv = _ptr(out.get("relaxed")), _ptr(out.get("tv"))
    a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
    a.stream = _stream_handle(dev)
    if events is not None:
        a.ev_begin, a.ev_end = events
    rc = lib.llc_lml_bound(ctypes.byref(a))
    if rc != 0:
        raise LlcError(rc)
    out["_workspace"] = workspace  # keeps the scratch alive until the caller drops the result
    return out


def new_workspace(B: int, K: int, V: int, device, v_chunks: int = 0) -> torch.Tensor:
    """Device scratch for one call; larger explicit v_chunks need proportionally more."""
    n = llc_couple_workspace_size(B, K, V)
    if v_chunks > 16:
        n = n * ((v_chunks + 15) // 16)
    return torch.empty(max(n, 256), dtype=torch.uint8, device=device)
