"""Thin ctypes binding over the C ABI in include/tli.h and include/tli_bench.h (same names, argument marshalling only).

torch is used for device buffers and the current HIP stream; every step of the path runs in the
library's kernels.  There is no CPU fallback: if libtli.so is missing or fails to load, the first
call raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtli.so")

TLI_F32, TLI_BF16 = 0, 1
FLAG_NONFINITE, FLAG_ZERO_MASS, FLAG_BAD_DRAFT, FLAG_DEGENERATE = 1, 2, 4, 8

EXPORTS = (
    "tli_build_map", "tli_free_map", "tli_map_info", "tli_workspace_bytes", "tli_draft_sample", "tli_verify",
    "tli_status_string", "tli_profile_enable", "tli_profile_collect", "tli_profile_disable", "tli_calib_copy",
    "tli_union_draft_sample", "tli_union_verify", "tli_acceptance_rates_workspace_bytes", "tli_acceptance_rates",
    "tli_sample_rows_workspace_bytes", "tli_sample_rows", "tli_greedy_draft", "tli_exact_match_workspace_bytes",
    "tli_exact_match_verify", "tli_draft_sample_compact", "tli_verify_compact",
    "tli_warp_workspace_bytes", "tli_warp_rows", "tli_map_dry_run", "tli_calib_read", "tli_device_info",
    "tli_d2t_from_strings", "tli_verify_static", "tli_verify_static_max_bytes",
    "tli_tune_final_path", "tli_sample_rows_warped", "tli_draft_sample_warped",
)
KERNELS = ("lse", "accept", "final_scan", "final_pick", "draft_scan", "draft_pick")

_lib = None


class TliError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


def load_library() -> ctypes.CDLL:
    """Load libtli.so built in-tree (see build.py).  Raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2502_05202_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    lib.tli_build_map.argtypes = [vp, i32, i32, ctypes.POINTER(vp), ctypes.POINTER(i32)]
    lib.tli_build_map.restype = ctypes.c_int
    lib.tli_free_map.argtypes = [vp]
    lib.tli_free_map.restype = None
    lib.tli_map_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.tli_map_info.restype = ctypes.c_int
    lib.tli_workspace_bytes.argtypes = [i32, i32, i32, i32, ctypes.c_int]
    lib.tli_workspace_bytes.restype = ctypes.c_size_t
    lib.tli_draft_sample.argtypes = [vp, vp, ctypes.c_int, i64, i32, f32, vp, vp, vp, vp, vp, vp, i64, vp,
                                     ctypes.c_size_t, vp]
    lib.tli_draft_sample.restype = ctypes.c_int
    lib.tli_verify.argtypes = [vp, vp, vp, ctypes.c_int, i32, i32, f32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                               vp, vp, vp, ctypes.c_size_t, vp]
    lib.tli_verify.restype = ctypes.c_int
    lib.tli_verify_static.argtypes = [vp, vp, vp, ctypes.c_int, i32, i32, f32, f32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                      vp, vp, vp]
    lib.tli_verify_static.restype = ctypes.c_int
    lib.tli_verify_static_max_bytes.argtypes = []
    lib.tli_verify_static_max_bytes.restype = ctypes.c_size_t
    lib.tli_tune_final_path.argtypes = [i32]
    lib.tli_tune_final_path.restype = ctypes.c_int
    lib.tli_draft_sample_compact.argtypes = lib.tli_draft_sample.argtypes
    lib.tli_draft_sample_compact.restype = ctypes.c_int
    lib.tli_verify_compact.argtypes = [vp, vp, vp, i64, ctypes.c_int, i32, i32, f32, f32, vp, vp, vp, vp, vp, vp, vp, vp,
                                       vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.tli_verify_compact.restype = ctypes.c_int
    lib.tli_warp_workspace_bytes.argtypes = [i32, i32, ctypes.c_int]
    lib.tli_warp_workspace_bytes.restype = ctypes.c_size_t
    lib.tli_warp_rows.argtypes = [vp, vp, ctypes.c_int, i64, i32, i32, f32, i32, f32, vp, i64, vp, vp, vp, vp,
                                  ctypes.c_size_t, vp]
    lib.tli_warp_rows.restype = ctypes.c_int
    lib.tli_union_draft_sample.argtypes = lib.tli_draft_sample.argtypes
    lib.tli_union_draft_sample.restype = ctypes.c_int
    lib.tli_union_verify.argtypes = lib.tli_verify.argtypes
    lib.tli_union_verify.restype = ctypes.c_int
    lib.tli_acceptance_rates_workspace_bytes.argtypes = [vp, i32, i32, ctypes.c_int]
    lib.tli_acceptance_rates_workspace_bytes.restype = ctypes.c_size_t
    lib.tli_acceptance_rates.argtypes = [vp, vp, vp, ctypes.c_int, i32, i32, f32, f32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.tli_acceptance_rates.restype = ctypes.c_int
    lib.tli_sample_rows_workspace_bytes.argtypes = [i32, i32, ctypes.c_int]
    lib.tli_sample_rows_workspace_bytes.restype = ctypes.c_size_t
    lib.tli_sample_rows.argtypes = [vp, ctypes.c_int, i64, i32, i32, f32, vp, vp, vp, vp, vp, i64, vp, ctypes.c_size_t, vp]
    lib.tli_sample_rows.restype = ctypes.c_int
    lib.tli_sample_rows_warped.argtypes = [vp, ctypes.c_int, i64, i32, i32, f32, vp, vp, vp, vp, vp, vp, i64, vp,
                                           ctypes.c_size_t, vp]
    lib.tli_sample_rows_warped.restype = ctypes.c_int
    lib.tli_draft_sample_warped.argtypes = [vp, vp, ctypes.c_int, i64, i32, f32, vp, vp, vp, vp, vp, vp, vp, i64, vp,
                                            ctypes.c_size_t, vp]
    lib.tli_draft_sample_warped.restype = ctypes.c_int
    lib.tli_greedy_draft.argtypes = [vp, vp, ctypes.c_int, i64, i32, vp, vp, vp, i64, vp, ctypes.c_size_t, vp]
    lib.tli_greedy_draft.restype = ctypes.c_int
    lib.tli_exact_match_workspace_bytes.argtypes = [i32, i32, i32, ctypes.c_int]
    lib.tli_exact_match_workspace_bytes.restype = ctypes.c_size_t
    lib.tli_exact_match_verify.argtypes = [vp, ctypes.c_int, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp,
                                           ctypes.c_size_t, vp]
    lib.tli_exact_match_verify.restype = ctypes.c_int
    lib.tli_profile_enable.argtypes = [ctypes.c_uint32, i32, i32]
    lib.tli_profile_enable.restype = ctypes.c_int
    lib.tli_profile_collect.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    lib.tli_profile_collect.restype = ctypes.c_int
    lib.tli_profile_disable.argtypes = []
    lib.tli_profile_disable.restype = None
    lib.tli_calib_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.tli_calib_copy.restype = ctypes.c_int
    lib.tli_calib_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_size_t, i32, vp, vp]
    lib.tli_calib_read.restype = ctypes.c_int
    lib.tli_device_info.argtypes = [ctypes.POINTER(i32)]
    lib.tli_device_info.restype = ctypes.c_int
    lib.tli_map_dry_run.argtypes = [vp, i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.tli_map_dry_run.restype = ctypes.c_int
    lib.tli_d2t_from_strings.argtypes = [ctypes.c_char_p, vp, i32, ctypes.c_char_p, vp, i32, vp, ctypes.POINTER(i32)]
    lib.tli_d2t_from_strings.restype = ctypes.c_int
    lib.tli_status_string.argtypes = [ctypes.c_int]
    lib.tli_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def tli_tune_final_path(path: int) -> None:
    """Form of tli_verify's first steps: 0 by batch size, 1 split, 2 a workgroup per sequence (see tli_bench.h)."""
    rc = load_library().tli_tune_final_path(int(path))
    if rc != 0:
        raise TliError(rc, "tli_tune_final_path")


def status_string(code: int) -> str:
    return load_library().tli_status_string(int(code)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TLI_F32
    if t.dtype == torch.bfloat16:
        return TLI_BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


class TliMap:
    """Owner of a tli_map (device tables of the vocabulary intersection)."""

    def __init__(self, handle: int, Vd: int, Vt: int, num_shared: int):
        self._h = ctypes.c_void_p(handle)
        self.Vd, self.Vt, self.num_shared = Vd, Vt, num_shared

    @property
    def handle(self):
        if self._h is None:
            raise RuntimeError("tli_map already freed")
        return self._h

    def free(self):
        if self._h is not None:
            load_library().tli_free_map(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def tli_build_map(d2t, Vt: int) -> TliMap:
    """d2t: host int32 array [Vd], target id of each drafter id or -1."""
    lib = load_library()
    arr = np.ascontiguousarray(np.asarray(d2t), dtype=np.int32)
    out = ctypes.c_void_p()
    S = ctypes.c_int32()
    rc = lib.tli_build_map(arr.ctypes.data_as(ctypes.c_void_p), arr.shape[0], int(Vt), ctypes.byref(out),
                           ctypes.byref(S))
    if rc != 0:
        raise TliError(rc, "tli_build_map")
    return TliMap(out.value, int(arr.shape[0]), int(Vt), S.value)


def _pack_tokens(tokens):
    raw = [t.encode("utf-8") if isinstance(t, str) else bytes(t) for t in tokens]
    offs = np.zeros(len(raw) + 1, np.int64)
    np.cumsum([len(r) for r in raw], out=offs[1:])
    return b"".join(raw), offs


def tli_d2t_from_strings(tokens_d, tokens_t) -> np.ndarray:
    """d2t (int32 [Vd]) from the two vocabularies' token strings (str or bytes) by exact equality; host only."""
    lib = load_library()
    bd, od = _pack_tokens(tokens_d)
    bt, ot = _pack_tokens(tokens_t)
    out = np.empty(len(tokens_d), np.int32)
    S = ctypes.c_int32()
    rc = lib.tli_d2t_from_strings(bd, od.ctypes.data_as(ctypes.c_void_p), len(tokens_d), bt,
                                  ot.ctypes.data_as(ctypes.c_void_p), len(tokens_t), out.ctypes.data_as(ctypes.c_void_p),
                                  ctypes.byref(S))
    if rc != 0:
        raise TliError(rc, "tli_d2t_from_strings")
    return out


def tli_map_dry_run(d2t, Vt: int) -> dict:
    """Host-only rehearsal of tli_build_map: same checks and tables, no device, plus the library's replay of what
    the residual-scan kernel does with them.  Returns status, num_shared, nparts (per dtype) and failed_check."""
    lib = load_library()
    arr = np.ascontiguousarray(np.asarray(d2t), dtype=np.int32)
    S, bad = ctypes.c_int32(), ctypes.c_int32()
    nparts = (ctypes.c_int32 * 2)()
    rc = lib.tli_map_dry_run(arr.ctypes.data_as(ctypes.c_void_p), arr.shape[0], int(Vt), ctypes.byref(S), nparts,
                             ctypes.byref(bad))
    return dict(status=int(rc), num_shared=S.value, nparts=(nparts[0], nparts[1]), failed_check=bad.value)


def tli_workspace_bytes(B: int, K: int, Vt: int, Vd: int, dtype: int) -> int:
    return int(load_library().tli_workspace_bytes(B, K, Vt, Vd, dtype))


def alloc_workspace(B: int, K: int, m: TliMap, dtype: int, device) -> torch.Tensor:
    n = tli_workspace_bytes(B, K, m.Vt, m.Vd, dtype)
    if n == 0:
        raise TliError(-1, "tli_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def tli_draft_sample(m: TliMap, logits_d: torch.Tensor, temp_d: float, u_draft: torch.Tensor,
                     workspace: torch.Tensor, out: dict | None = None, stream=None, column=None,
                     _entry: str = "tli_draft_sample") -> dict:
    """logits_d [..., Vd] with contiguous last dim; leading dims are flattened into R rows.

    column=(k, K): the per-step form.  logits_d is then the [B, Vd] view logits[:, k, :] of a [B,K,Vd]
    tensor, u_draft and the tensors of `out` are the full [B,K] arrays, and the call reads / fills their
    column k (io_stride = K, pointers advanced by k)."""
    lib = load_library()
    assert logits_d.is_cuda and logits_d.stride(-1) == 1
    ld = logits_d.reshape(-1, logits_d.shape[-1]) if logits_d.dim() != 2 else logits_d
    R, Vd = ld.shape
    k, io = (0, 1) if column is None else (int(column[0]), int(column[1]))
    assert 0 <= k < io
    want_v = m.num_shared if _entry == "tli_draft_sample_compact" else m.Vd
    assert Vd == want_v and u_draft.numel() == R * io and u_draft.dtype == torch.float32 and u_draft.is_contiguous()
    dev = ld.device
    if out is None:
        out = dict(tok_d=torch.empty(R * io, dtype=torch.int32, device=dev),
                   tok_t=torch.empty(R * io, dtype=torch.int32, device=dev),
                   q_tok=torch.empty(R * io, dtype=torch.float64, device=dev),
                   lse_q=torch.empty(R * io, dtype=torch.float64, device=dev),
                   status=torch.empty(R * io, dtype=torch.int32, device=dev))

    def at(t):
        if t is None:
            return None
        assert t.numel() == R * io and t.is_contiguous()
        return ctypes.c_void_p(t.data_ptr() + k * t.element_size())

    rc = getattr(lib, _entry)(m.handle, _ptr(ld), _dtype_code(ld), ld.stride(0), R, float(temp_d), at(u_draft),
                              at(out["tok_d"]), at(out["tok_t"]), at(out.get("q_tok")), at(out["lse_q"]),
                              at(out["status"]), io, _ptr(workspace), workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, _entry)
    return out


def tli_draft_sample_compact(m: TliMap, logits_c, temp_d, u_draft, workspace, out=None, stream=None, column=None) -> dict:
    """tli_draft_sample on rows in compact layout: logits_c [..., S] (a view with a wider row stride is fine),
    entry r = logit of the shared token of rank r."""
    return tli_draft_sample(m, logits_c, temp_d, u_draft, workspace, out, stream, column, _entry="tli_draft_sample_compact")


def tli_verify_compact(m: TliMap, logits_t: torch.Tensor, logits_c: torch.Tensor, temp_t: float, temp_d: float,
                       tok_d: torch.Tensor, lse_q, u_acc: torch.Tensor, u_fin: torch.Tensor, workspace: torch.Tensor,
                       out: dict | None = None, stream=None) -> dict:
    """tli_verify with the drafter logits in compact layout: logits_c [B, K, S] with stride(1) = row stride."""
    lib = load_library()
    B, K1, Vt = logits_t.shape
    K = K1 - 1
    assert logits_t.is_cuda and logits_t.is_contiguous() and Vt == m.Vt and logits_t.dtype == logits_c.dtype
    assert tuple(logits_c.shape) == (B, K, m.num_shared) and logits_c.stride(2) == 1
    stride = logits_c.stride(1)
    assert logits_c.stride(0) == K * stride
    if out is None:
        out = alloc_verify_outputs(B, K, logits_t.device)
    rc = lib.tli_verify_compact(m.handle, _ptr(logits_t), _ptr(logits_c), stride, _dtype_code(logits_t), B, K,
                                float(temp_t), float(temp_d), _ptr(tok_d), _ptr(lse_q), _ptr(u_acc), _ptr(u_fin),
                                _ptr(out["n_accepted"]), _ptr(out["out_tok"]), _ptr(out.get("accept")),
                                _ptr(out.get("p_tok")), _ptr(out.get("q_tok")), _ptr(out.get("lse_p")), _ptr(out["status"]),
                                _ptr(workspace), workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_verify_compact")
    return out


def tli_union_draft_sample(m: TliMap, logits_d, temp_d, u_draft, workspace, out=None, stream=None, column=None) -> dict:
    """Draft step of the union algorithm: same call as tli_draft_sample, drawn from q over all of D."""
    return tli_draft_sample(m, logits_d, temp_d, u_draft, workspace, out, stream, column, _entry="tli_union_draft_sample")


def alloc_verify_outputs(B: int, K: int, device) -> dict:
    return dict(n_accepted=torch.empty(B, dtype=torch.int32, device=device),
                out_tok=torch.empty((B, K + 1), dtype=torch.int32, device=device),
                accept=torch.empty((B, K), dtype=torch.uint8, device=device),
                p_tok=torch.empty((B, K), dtype=torch.float64, device=device),
                q_tok=torch.empty((B, K), dtype=torch.float64, device=device),
                lse_p=torch.empty((B, K + 1), dtype=torch.float64, device=device),
                status=torch.empty(B, dtype=torch.int32, device=device))


def tli_verify(m: TliMap, logits_t: torch.Tensor, logits_d: torch.Tensor, temp_t: float, temp_d: float,
               tok_d: torch.Tensor, lse_q: torch.Tensor, u_acc: torch.Tensor, u_fin: torch.Tensor,
               workspace: torch.Tensor, out: dict | None = None, stream=None, _entry: str = "tli_verify") -> dict:
    """logits_t [B,K+1,Vt], logits_d [B,K,Vd] dense; tok_d int32 [B,K]; lse_q float64 [B,K] or None
    (None: the library recomputes the drafter normalisers)."""
    lib = load_library()
    B, K1, Vt = logits_t.shape
    K = K1 - 1
    assert logits_t.is_cuda and logits_t.is_contiguous() and logits_d.is_contiguous()
    assert tuple(logits_d.shape) == (B, K, m.Vd) and Vt == m.Vt and logits_t.dtype == logits_d.dtype
    assert tok_d.dtype == torch.int32 and tok_d.numel() == B * K and tok_d.is_contiguous()
    assert lse_q is None or (lse_q.dtype == torch.float64 and lse_q.numel() == B * K and lse_q.is_contiguous())
    assert u_acc.dtype == torch.float32 and u_acc.numel() == B * K and u_acc.is_contiguous()
    assert u_fin.dtype == torch.float32 and u_fin.numel() == B and u_fin.is_contiguous()
    if out is None:
        out = alloc_verify_outputs(B, K, logits_t.device)
    rc = getattr(lib, _entry)(m.handle, _ptr(logits_t), _ptr(logits_d), _dtype_code(logits_t), B, K, float(temp_t),
                        float(temp_d), _ptr(tok_d), _ptr(lse_q), _ptr(u_acc), _ptr(u_fin), _ptr(out["n_accepted"]),
                        _ptr(out["out_tok"]), _ptr(out.get("accept")), _ptr(out.get("p_tok")), _ptr(out.get("q_tok")),
                        _ptr(out.get("lse_p")), _ptr(out["status"]), _ptr(workspace), workspace.numel(),
                        _stream(stream))
    if rc != 0:
        raise TliError(rc, _entry)
    return out


def tli_verify_static(m: TliMap, logits_t: torch.Tensor, logits_d: torch.Tensor, temp_t: float, temp_d: float,
                      tok_d: torch.Tensor, lse_q, u_acc: torch.Tensor, u_fin: torch.Tensor, out: dict,
                      stream=None) -> dict:
    """tli_verify without a workspace (the library's fixed scratch); `out` must be given: nothing is allocated."""
    lib = load_library()
    B, K1, Vt = logits_t.shape
    K = K1 - 1
    assert logits_t.is_cuda and logits_t.is_contiguous() and logits_d.is_contiguous()
    assert tuple(logits_d.shape) == (B, K, m.Vd) and Vt == m.Vt and logits_t.dtype == logits_d.dtype
    assert tok_d.dtype == torch.int32 and tok_d.numel() == B * K and tok_d.is_contiguous()
    assert lse_q is None or (lse_q.dtype == torch.float64 and lse_q.numel() == B * K and lse_q.is_contiguous())
    assert u_acc.dtype == torch.float32 and u_acc.numel() == B * K and u_acc.is_contiguous()
    assert u_fin.dtype == torch.float32 and u_fin.numel() == B and u_fin.is_contiguous()
    rc = lib.tli_verify_static(m.handle, _ptr(logits_t), _ptr(logits_d), _dtype_code(logits_t), B, K, float(temp_t),
                               float(temp_d), _ptr(tok_d), _ptr(lse_q), _ptr(u_acc), _ptr(u_fin), _ptr(out["n_accepted"]),
                               _ptr(out["out_tok"]), _ptr(out.get("accept")), _ptr(out.get("p_tok")),
                               _ptr(out.get("q_tok")), _ptr(out.get("lse_p")), _ptr(out["status"]), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_verify_static")
    return out


def tli_union_verify(m: TliMap, logits_t, logits_d, temp_t, temp_d, tok_d, lse_q, u_acc, u_fin, workspace, out=None,
                     stream=None) -> dict:
    """Verification of the union algorithm: same call as tli_verify with q over all of D (lse_q over all of D)."""
    return tli_verify(m, logits_t, logits_d, temp_t, temp_d, tok_d, lse_q, u_acc, u_fin, workspace, out, stream,
                      _entry="tli_union_verify")


def tli_acceptance_rates(m: TliMap, logits_t: torch.Tensor, logits_d: torch.Tensor, temp_t: float, temp_d: float,
                         workspace: torch.Tensor | None = None, stream=None) -> dict:
    """alpha_tli, alpha_union [B,K] fp64 and pos_status [B,K] for logits_t [B,K+1,Vt], logits_d [B,K,Vd]."""
    lib = load_library()
    B, K1, Vt = logits_t.shape
    K = K1 - 1
    assert logits_t.is_contiguous() and logits_d.is_contiguous() and tuple(logits_d.shape) == (B, K, m.Vd) and Vt == m.Vt
    code = _dtype_code(logits_t)
    if workspace is None:
        n = int(lib.tli_acceptance_rates_workspace_bytes(m.handle, B, K, code))
        if n == 0:
            raise TliError(-1, "tli_acceptance_rates_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=logits_t.device)
    dev = logits_t.device
    out = dict(alpha_tli=torch.empty((B, K), dtype=torch.float64, device=dev),
               alpha_union=torch.empty((B, K), dtype=torch.float64, device=dev),
               status=torch.empty((B, K), dtype=torch.int32, device=dev))
    rc = lib.tli_acceptance_rates(m.handle, _ptr(logits_t), _ptr(logits_d), code, B, K, float(temp_t), float(temp_d),
                                  _ptr(out["alpha_tli"]), _ptr(out["alpha_union"]), _ptr(out["status"]), _ptr(workspace),
                                  workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_acceptance_rates")
    out["workspace"] = workspace
    return out


def tli_sample_rows(logits: torch.Tensor, temp: float, u: torch.Tensor | None, workspace: torch.Tensor | None = None,
                    stream=None, thr: torch.Tensor | None = None) -> dict:
    """One token per row of logits [R, V] (contiguous last dim): softmax draw, or argmax at temp == 0.
    thr [R] fp32: the rows warped by threshold (tli_sample_rows_warped; temp > 0)."""
    lib = load_library()
    assert logits.is_cuda and logits.dim() == 2 and logits.stride(-1) == 1
    R, V = logits.shape
    code = _dtype_code(logits)
    if workspace is None:
        workspace = torch.empty(int(lib.tli_sample_rows_workspace_bytes(R, V, code)), dtype=torch.uint8, device=logits.device)
    dev = logits.device
    out = dict(tok=torch.empty(R, dtype=torch.int32, device=dev), p_tok=torch.empty(R, dtype=torch.float64, device=dev),
               lse=torch.empty(R, dtype=torch.float64, device=dev), status=torch.empty(R, dtype=torch.int32, device=dev))
    if thr is not None:
        assert thr.dtype == torch.float32 and thr.numel() == R and thr.is_contiguous()
        rc = lib.tli_sample_rows_warped(_ptr(logits), code, logits.stride(0), R, V, float(temp), _ptr(thr), _ptr(u),
                                        _ptr(out["tok"]), _ptr(out["p_tok"]), _ptr(out["lse"]), _ptr(out["status"]), 1,
                                        _ptr(workspace), workspace.numel(), _stream(stream))
    else:
        rc = lib.tli_sample_rows(_ptr(logits), code, logits.stride(0), R, V, float(temp), _ptr(u), _ptr(out["tok"]),
                                 _ptr(out["p_tok"]), _ptr(out["lse"]), _ptr(out["status"]), 1, _ptr(workspace),
                                 workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_sample_rows")
    return out


def tli_draft_sample_warped(m: TliMap, logits_d: torch.Tensor, temp_d: float, thr: torch.Tensor, u_draft: torch.Tensor,
                            workspace: torch.Tensor, stream=None) -> dict:
    """tli_draft_sample on rows logits_d [R, Vd] warped by the thresholds thr [R] (from tli_warp_rows(..., m=m,
    rewrite=False) on the same rows)."""
    lib = load_library()
    assert logits_d.is_cuda and logits_d.dim() == 2 and logits_d.stride(-1) == 1 and logits_d.shape[1] == m.Vd
    R = logits_d.shape[0]
    assert thr.dtype == torch.float32 and thr.numel() == R and thr.is_contiguous()
    assert u_draft.dtype == torch.float32 and u_draft.numel() == R and u_draft.is_contiguous()
    dev = logits_d.device
    out = dict(tok_d=torch.empty(R, dtype=torch.int32, device=dev), tok_t=torch.empty(R, dtype=torch.int32, device=dev),
               q_tok=torch.empty(R, dtype=torch.float64, device=dev), lse_q=torch.empty(R, dtype=torch.float64, device=dev),
               status=torch.empty(R, dtype=torch.int32, device=dev))
    rc = lib.tli_draft_sample_warped(m.handle, _ptr(logits_d), _dtype_code(logits_d), logits_d.stride(0), R, float(temp_d),
                                     _ptr(thr), _ptr(u_draft), _ptr(out["tok_d"]), _ptr(out["tok_t"]), _ptr(out["q_tok"]),
                                     _ptr(out["lse_q"]), _ptr(out["status"]), 1, _ptr(workspace), workspace.numel(),
                                     _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_draft_sample_warped")
    return out


def tli_warp_rows(logits: torch.Tensor, temp: float, top_k: int, top_p: float, m: TliMap | None = None,
                  out: torch.Tensor | None = None, workspace: torch.Tensor | None = None, stream=None,
                  rewrite: bool = True) -> dict:
    """top-k / top-p on rows logits [R, V]: returns the warped rows (dropped = -inf; `out` may be `logits` itself),
    thr, kept, status.  With a map only the shared drafter ids compete.  rewrite=False: thresholds and status only
    (thr = the lowest value kept, -inf if no warper is active for the row)."""
    lib = load_library()
    assert logits.is_cuda and logits.dim() == 2 and logits.stride(-1) == 1
    R, V = logits.shape
    code = _dtype_code(logits)
    dev = logits.device
    if workspace is None:
        workspace = torch.empty(int(lib.tli_warp_workspace_bytes(R, V, code)), dtype=torch.uint8, device=dev)
    res = dict(thr=torch.empty(R, dtype=torch.float32, device=dev), status=torch.empty(R, dtype=torch.int32, device=dev))
    if rewrite:
        if out is None:  # rows start on 16-byte boundaries: the row stride is V rounded up to whole vectors
            epv = 16 // logits.element_size()
            out = torch.empty((R, (V + epv - 1) // epv * epv), dtype=logits.dtype, device=dev)[:, :V]
        assert out.shape == logits.shape and out.dtype == logits.dtype and out.stride(-1) == 1
        res["logits"] = out
        res["kept"] = torch.empty(R, dtype=torch.int32, device=dev)
    rc = lib.tli_warp_rows(None if m is None else m.handle, _ptr(logits), code, logits.stride(0), R, V, float(temp),
                           int(top_k), float(top_p), _ptr(out) if rewrite else None, out.stride(0) if rewrite else 0,
                           _ptr(res["thr"]), _ptr(res.get("kept")), _ptr(res["status"]), _ptr(workspace),
                           workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_warp_rows")
    return res


def tli_greedy_draft(m: TliMap, logits_d: torch.Tensor, workspace: torch.Tensor, stream=None) -> dict:
    """TLI draft at temperature zero for logits_d [..., Vd]: argmax over the shared ids."""
    lib = load_library()
    ld = logits_d.reshape(-1, logits_d.shape[-1]) if logits_d.dim() != 2 else logits_d
    R, Vd = ld.shape
    assert Vd == m.Vd and ld.stride(-1) == 1
    dev = ld.device
    out = dict(tok_d=torch.empty(R, dtype=torch.int32, device=dev), tok_t=torch.empty(R, dtype=torch.int32, device=dev),
               status=torch.empty(R, dtype=torch.int32, device=dev))
    rc = lib.tli_greedy_draft(m.handle, _ptr(ld), _dtype_code(ld), ld.stride(0), R, _ptr(out["tok_d"]), _ptr(out["tok_t"]),
                              _ptr(out["status"]), 1, _ptr(workspace), workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_greedy_draft")
    return out


def tli_exact_match_verify(logits_t: torch.Tensor, temp_t: float, draft_t: torch.Tensor, u: torch.Tensor | None,
                           workspace: torch.Tensor | None = None, out: dict | None = None, stream=None) -> dict:
    """logits_t [B, m+1, Vt] dense, draft_t int32 [B, m] target ids, u fp32 [B, m+1] (None at temp_t == 0)."""
    lib = load_library()
    B, m1, Vt = logits_t.shape
    mm = m1 - 1
    assert logits_t.is_cuda and logits_t.is_contiguous()
    assert draft_t.dtype == torch.int32 and draft_t.numel() == B * mm and draft_t.is_contiguous()
    assert u is None or (u.dtype == torch.float32 and u.numel() == B * m1 and u.is_contiguous())
    code = _dtype_code(logits_t)
    if workspace is None:
        workspace = torch.empty(int(lib.tli_exact_match_workspace_bytes(B, mm, Vt, code)), dtype=torch.uint8,
                                device=logits_t.device)
    dev = logits_t.device
    if out is None:
        out = dict(n_accepted=torch.empty(B, dtype=torch.int32, device=dev),
                   out_tok=torch.empty((B, m1), dtype=torch.int32, device=dev),
                   tgt_tok=torch.empty((B, m1), dtype=torch.int32, device=dev),
                   status=torch.empty(B, dtype=torch.int32, device=dev))
    rc = lib.tli_exact_match_verify(_ptr(logits_t), code, B, mm, Vt, float(temp_t), _ptr(draft_t), _ptr(u),
                                    _ptr(out["n_accepted"]), _ptr(out["out_tok"]), _ptr(out["tgt_tok"]),
                                    _ptr(out["status"]), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_exact_match_verify")
    return out


def tli_profile_enable(kernels, max_calls: int, every: int = 1) -> None:
    """kernels: iterable of names from KERNELS; one launch in `every` is timed."""
    mask = 0
    for k in kernels:
        mask |= 1 << KERNELS.index(k)
    rc = load_library().tli_profile_enable(mask, int(max_calls), int(every))
    if rc != 0:
        raise TliError(rc, "tli_profile_enable")


def tli_profile_collect(kernel: str):
    """-> (total milliseconds, launches) of one kernel since the last collect."""
    ms, n = ctypes.c_double(), ctypes.c_int32()
    rc = load_library().tli_profile_collect(KERNELS.index(kernel), ctypes.byref(ms), ctypes.byref(n))
    if rc != 0:
        raise TliError(rc, "tli_profile_collect")
    return ms.value, n.value


def tli_profile_disable() -> None:
    load_library().tli_profile_disable()


def tli_calib_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """Plain copy of src into dst (same byte size) by the library's calibration kernel."""
    n = src.numel() * src.element_size()
    assert n == dst.numel() * dst.element_size()
    rc = load_library().tli_calib_copy(_ptr(src), _ptr(dst), n, _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_calib_copy")


def tli_calib_read(src: torch.Tensor, slab_bytes: int, nontemporal: bool, out: torch.Tensor, nbytes: int | None = None,
                   stream=None) -> None:
    """Read-only streaming pass over the first nbytes of src (default: all) in slabs of slab_bytes, one workgroup each;
    out: uint32/int32 device scratch with a word per slab."""
    n = src.numel() * src.element_size() if nbytes is None else int(nbytes)
    assert out.numel() >= n // slab_bytes
    rc = load_library().tli_calib_read(_ptr(src), n, int(slab_bytes), int(bool(nontemporal)), _ptr(out), _stream(stream))
    if rc != 0:
        raise TliError(rc, "tli_calib_read")


def tli_device_info() -> dict:
    """Memory clock (kHz), memory bus width (bits), compute units and engine clock (kHz) as the HIP runtime reports
    them for the current device (0 where it reports nothing)."""
    out = (ctypes.c_int32 * 4)()
    rc = load_library().tli_device_info(out)
    if rc != 0:
        raise TliError(rc, "tli_device_info")
    return dict(memory_clock_khz=int(out[0]), memory_bus_bits=int(out[1]), compute_units=int(out[2]), clock_khz=int(out[3]))
