"""CPU oracle for the TLI draft-and-verify step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``tli_oracle.c`` (plain fp64 C).  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; the product package never does, and this
package imports nothing from the product.

Logit arrays are numpy ``float32`` (fp32 logits) or ``uint16`` (the raw bits of bf16 logits).
Uniforms are passed as float64 (fp32 uniforms convert exactly).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tli_oracle.c")
_LIB = os.path.join(_HERE, "libtli_oracle.so")

NONFINITE, ZERO_MASS, BAD_DRAFT, DEGENERATE = 1, 2, 4, 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math: IEEE semantics are the point)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.tlo_inverse_cdf.restype = ctypes.c_int64
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError(f"logits must be float32 or uint16 (bf16 bits), got {a.dtype}")


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def softmax(logits_row: np.ndarray, tau: float):
    """p = softmax(logits / tau) for one row -> (prob[n] float64, log_norm, status)."""
    lib = _load()
    row = np.ascontiguousarray(logits_row)
    n = row.shape[0]
    prob = np.empty(n, np.float64)
    lse = ctypes.c_double()
    st = lib.tlo_softmax(_p(row), _dtype_code(row), ctypes.c_int64(n), ctypes.c_double(tau), _p(prob),
                         ctypes.byref(lse))
    return prob, lse.value, st


def adjusted_drafter(logits_row: np.ndarray, tau_d: float, d2t: np.ndarray):
    """TLI's q and q' for one drafter row -> (q[Vd], qprime[Vd], log_norm_shared, status)."""
    lib = _load()
    row = np.ascontiguousarray(logits_row)
    d2t = _c(d2t, np.int32)
    Vd = row.shape[0]
    assert d2t.shape[0] == Vd
    q = np.empty(Vd, np.float64)
    qp = np.empty(Vd, np.float64)
    lse = ctypes.c_double()
    st = lib.tlo_adjusted_drafter(_p(row), _dtype_code(row), ctypes.c_int64(Vd), ctypes.c_double(tau_d),
                                  _p(d2t), _p(q), _p(qp), ctypes.byref(lse))
    return q, qp, lse.value, st


def inverse_cdf(w: np.ndarray, u: float):
    """First id whose running sum exceeds u * total -> (id, margin)."""
    lib = _load()
    w = _c(w, np.float64)
    mg = ctypes.c_double()
    x = lib.tlo_inverse_cdf(_p(w), ctypes.c_int64(w.shape[0]), ctypes.c_double(u), ctypes.byref(mg))
    return int(x), mg.value


def draft_sample(logits_d: np.ndarray, tau_d: float, d2t: np.ndarray, u_draft: np.ndarray, threads: int = 1):
    """Draft sampling for rows [R, Vd] (the row stride is the array's own)."""
    lib = _load()
    ld = np.ascontiguousarray(logits_d)
    R, Vd = ld.shape
    d2t = _c(d2t, np.int32)
    u = _c(np.asarray(u_draft).reshape(-1), np.float64)
    assert u.shape[0] == R and d2t.shape[0] == Vd
    out = dict(
        tok_d=np.empty(R, np.int32), tok_t=np.empty(R, np.int32), q_tok=np.empty(R, np.float64),
        lse_q=np.empty(R, np.float64), status=np.empty(R, np.int32), margin=np.empty(R, np.float64),
    )
    code = _dtype_code(ld)
    esz = ld.dtype.itemsize

    def run(lo, hi):
        if hi <= lo:
            return
        work = np.empty(2 * Vd, np.float64)
        off = lambda a: ctypes.c_void_p(a.ctypes.data + lo * a.dtype.itemsize)
        lib.tlo_draft_sample(
            ctypes.c_void_p(ld.ctypes.data + lo * Vd * esz), code, ctypes.c_int64(Vd), ctypes.c_int64(hi - lo),
            ctypes.c_int64(Vd), ctypes.c_double(tau_d), _p(d2t), off(u), off(out["tok_d"]), off(out["tok_t"]),
            off(out["q_tok"]), off(out["lse_q"]), off(out["status"]), off(out["margin"]), _p(work))

    _fan_out(run, R, threads)
    return out


def verify(logits_t: np.ndarray, logits_d: np.ndarray, tau_t: float, tau_d: float, d2t: np.ndarray,
           tok_d: np.ndarray, u_acc: np.ndarray, u_fin: np.ndarray, want_weights: bool = False,
           threads: int = 1, _fn: str = "tlo_verify"):
    """One TLI verification for B sequences; logits_t [B,K+1,Vt], logits_d [B,K,Vd], tok_d [B,K]."""
    lib = _load()
    lt = np.ascontiguousarray(logits_t)
    ld = np.ascontiguousarray(logits_d)
    B, K1, Vt = lt.shape
    K = K1 - 1
    assert ld.shape[0] == B and ld.shape[1] == K and lt.dtype == ld.dtype
    Vd = ld.shape[2]
    d2t = _c(d2t, np.int32)
    tok = _c(np.asarray(tok_d).reshape(B, K), np.int32)
    ua = _c(np.asarray(u_acc).reshape(B, K), np.float64)
    uf = _c(np.asarray(u_fin).reshape(B), np.float64)
    out = dict(
        n_acc=np.empty(B, np.int32), out_tok=np.empty((B, K + 1), np.int32), accept=np.empty((B, K), np.uint8),
        p_tok=np.empty((B, K), np.float64), q_tok=np.empty((B, K), np.float64),
        lse_p=np.empty((B, K + 1), np.float64), lse_q=np.empty((B, K), np.float64),
        status=np.empty(B, np.int32), acc_margin=np.empty((B, K), np.float64), fin_margin=np.empty(B, np.float64),
    )
    if want_weights:
        out["fin_weights"] = np.empty((B, Vt), np.float64)
    code = _dtype_code(lt)
    esz = lt.dtype.itemsize

    def run(lo, hi):
        if hi <= lo:
            return
        work = np.empty(3 * Vt + 2 * Vd, np.float64)

        def off(a):
            per = int(np.prod(a.shape[1:])) if a.ndim > 1 else 1
            return ctypes.c_void_p(a.ctypes.data + lo * per * a.dtype.itemsize)

        fw = off(out["fin_weights"]) if want_weights else ctypes.c_void_p(0)
        getattr(lib, _fn)(
            ctypes.c_void_p(lt.ctypes.data + lo * (K + 1) * Vt * esz),
            ctypes.c_void_p(ld.ctypes.data + lo * K * Vd * esz), code,
            ctypes.c_int64(hi - lo), ctypes.c_int64(K), ctypes.c_int64(Vt), ctypes.c_int64(Vd),
            ctypes.c_double(tau_t), ctypes.c_double(tau_d), _p(d2t), off(tok), off(ua), off(uf),
            off(out["n_acc"]), off(out["out_tok"]), off(out["accept"]), off(out["p_tok"]), off(out["q_tok"]),
            off(out["lse_p"]), off(out["lse_q"]), off(out["status"]), off(out["acc_margin"]),
            off(out["fin_margin"]), fw, _p(work))

    _fan_out(run, B, threads)
    return out


def _rows_call(fn_name, logits, R, V, threads, make_args, out):
    """Shared driver of the per-row entry points: rows [R, V] split over host threads."""
    lib = _load()
    code = _dtype_code(logits)
    esz = logits.dtype.itemsize

    def run(lo, hi):
        if hi <= lo:
            return
        off = lambda a: ctypes.c_void_p(a.ctypes.data + lo * (a.size // R) * a.dtype.itemsize)
        getattr(lib, fn_name)(*make_args(ctypes.c_void_p(logits.ctypes.data + lo * V * esz), code, hi - lo, off))

    _fan_out(run, R, threads)
    return out


def union_draft_sample(logits_d: np.ndarray, tau_d: float, d2t: np.ndarray, u_draft: np.ndarray, threads: int = 1):
    """Draft step of the union algorithm: d ~ softmax over ALL of D; tok_t = -1 for tokens outside T."""
    ld = np.ascontiguousarray(logits_d)
    R, Vd = ld.shape
    d2t = _c(d2t, np.int32)
    u = _c(np.asarray(u_draft).reshape(-1), np.float64)
    assert u.shape[0] == R and d2t.shape[0] == Vd
    out = dict(tok_d=np.empty(R, np.int32), tok_t=np.empty(R, np.int32), q_tok=np.empty(R, np.float64),
               lse_q=np.empty(R, np.float64), status=np.empty(R, np.int32), margin=np.empty(R, np.float64))

    def args(row0, code, n, off):
        work = np.empty(Vd, np.float64)
        return (row0, code, ctypes.c_int64(Vd), ctypes.c_int64(n), ctypes.c_int64(Vd), ctypes.c_double(tau_d), _p(d2t),
                off(u), off(out["tok_d"]), off(out["tok_t"]), off(out["q_tok"]), off(out["lse_q"]), off(out["status"]),
                off(out["margin"]), _p(work))

    return _rows_call("tlo_union_draft_sample", ld, R, Vd, threads, args, out)


def union_verify(logits_t: np.ndarray, logits_d: np.ndarray, tau_t: float, tau_d: float, d2t: np.ndarray,
                 tok_d: np.ndarray, u_acc: np.ndarray, u_fin: np.ndarray, want_weights: bool = False,
                 threads: int = 1):
    """Verification of the union algorithm (standard SD with p, q extended by zeros to T ∪ D)."""
    return verify(logits_t, logits_d, tau_t, tau_d, d2t, tok_d, u_acc, u_fin, want_weights, threads,
                  _fn="tlo_union_verify")


def acceptance_rates(logits_t: np.ndarray, logits_d: np.ndarray, tau_t: float, tau_d: float, d2t: np.ndarray,
                     threads: int = 1):
    """alpha_tli, alpha_union per row pair; logits_t [R, Vt], logits_d [R, Vd]."""
    lib = _load()
    lt = np.ascontiguousarray(logits_t)
    ld = np.ascontiguousarray(logits_d)
    R, Vt = lt.shape
    Vd = ld.shape[1]
    assert ld.shape[0] == R and lt.dtype == ld.dtype
    d2t = _c(d2t, np.int32)
    out = dict(alpha_tli=np.empty(R, np.float64), alpha_union=np.empty(R, np.float64), status=np.empty(R, np.int32))
    code = _dtype_code(lt)
    esz = lt.dtype.itemsize

    def run(lo, hi):
        if hi <= lo:
            return
        work = np.empty(Vt + Vd, np.float64)
        off = lambda a: ctypes.c_void_p(a.ctypes.data + lo * a.dtype.itemsize)
        lib.tlo_acceptance_rates(ctypes.c_void_p(lt.ctypes.data + lo * Vt * esz), ctypes.c_int64(Vt),
                                 ctypes.c_void_p(ld.ctypes.data + lo * Vd * esz), ctypes.c_int64(Vd), code,
                                 ctypes.c_int64(hi - lo), ctypes.c_int64(Vt), ctypes.c_int64(Vd), ctypes.c_double(tau_t),
                                 ctypes.c_double(tau_d), _p(d2t), off(out["alpha_tli"]), off(out["alpha_union"]),
                                 off(out["status"]), _p(work))

    _fan_out(run, R, threads)
    return out


def sample_rows(logits: np.ndarray, tau: float, u: np.ndarray, threads: int = 1):
    """One token per row of [R, V]: inverse CDF of softmax(logits/tau) with u[r], or the argmax at tau == 0."""
    lg = np.ascontiguousarray(logits)
    R, V = lg.shape
    u = _c(np.asarray(u).reshape(-1), np.float64)
    assert u.shape[0] == R
    out = dict(tok=np.empty(R, np.int32), p_tok=np.empty(R, np.float64), lse=np.empty(R, np.float64),
               status=np.empty(R, np.int32), margin=np.empty(R, np.float64))

    def args(row0, code, n, off):
        work = np.empty(V, np.float64)
        return (row0, code, ctypes.c_int64(V), ctypes.c_int64(n), ctypes.c_int64(V), ctypes.c_double(tau), off(u),
                off(out["tok"]), off(out["p_tok"]), off(out["lse"]), off(out["status"]), off(out["margin"]), _p(work))

    return _rows_call("tlo_sample_rows", lg, R, V, threads, args, out)


def exact_match_verify(logits_t: np.ndarray, tau_t: float, draft_t: np.ndarray, u: np.ndarray, threads: int = 1):
    """Tail of string-level exact matching: logits_t [B, m+1, Vt], draft_t [B, m] target ids, u [B, m+1]."""
    lib = _load()
    lt = np.ascontiguousarray(logits_t)
    B, m1, Vt = lt.shape
    m = m1 - 1
    dr = _c(np.asarray(draft_t).reshape(B, m), np.int32)
    uu = _c(np.asarray(u).reshape(B, m1), np.float64)
    out = dict(n_acc=np.empty(B, np.int32), out_tok=np.empty((B, m1), np.int32), tgt_tok=np.empty((B, m1), np.int32),
               status=np.empty(B, np.int32), margin=np.empty((B, m1), np.float64))
    code = _dtype_code(lt)
    esz = lt.dtype.itemsize

    def run(lo, hi):
        if hi <= lo:
            return
        work = np.empty(Vt, np.float64)

        def off(a):
            per = int(np.prod(a.shape[1:])) if a.ndim > 1 else 1
            return ctypes.c_void_p(a.ctypes.data + lo * per * a.dtype.itemsize)

        lib.tlo_exact_match_verify(ctypes.c_void_p(lt.ctypes.data + lo * m1 * Vt * esz), code, ctypes.c_int64(hi - lo),
                                   ctypes.c_int64(m), ctypes.c_int64(Vt), ctypes.c_double(tau_t), off(dr), off(uu),
                                   off(out["n_acc"]), off(out["out_tok"]), off(out["tgt_tok"]), off(out["status"]),
                                   off(out["margin"]), _p(work))

    _fan_out(run, B, threads)
    return out


def greedy_draft(logits_d: np.ndarray, d2t: np.ndarray, threads: int = 1):
    """TLI draft at temperature zero: argmax over the shared ids of each row of [R, Vd]."""
    ld = np.ascontiguousarray(logits_d)
    R, Vd = ld.shape
    d2t = _c(d2t, np.int32)
    out = dict(tok_d=np.empty(R, np.int32), tok_t=np.empty(R, np.int32), status=np.empty(R, np.int32))

    def args(row0, code, n, off):
        return (row0, code, ctypes.c_int64(Vd), ctypes.c_int64(n), ctypes.c_int64(Vd), _p(d2t), off(out["tok_d"]),
                off(out["tok_t"]), off(out["status"]))

    return _rows_call("tlo_greedy_draft", ld, R, Vd, threads, args, out)


def warp_rows(logits: np.ndarray, tau: float, top_k: int, top_p: float, d2t=None, threads: int = 1):
    """top-k / top-p thresholds of rows [R, V]: thr, kept, keep_mask [R, V] uint8, status, margin."""
    lib = _load()
    lg = np.ascontiguousarray(logits)
    R, V = lg.shape
    dd = None if d2t is None else _c(d2t, np.int32)
    out = dict(thr=np.empty(R, np.float64), kept=np.empty(R, np.int32), keep_mask=np.empty((R, V), np.uint8),
               status=np.empty(R, np.int32), margin=np.empty(R, np.float64))
    code = _dtype_code(lg)
    esz = lg.dtype.itemsize

    def run(lo, hi):
        if hi <= lo:
            return
        work = np.empty(V, np.float64)

        def off(a):
            per = int(np.prod(a.shape[1:])) if a.ndim > 1 else 1
            return ctypes.c_void_p(a.ctypes.data + lo * per * a.dtype.itemsize)

        lib.tlo_warp_rows(ctypes.c_void_p(lg.ctypes.data + lo * V * esz), code, ctypes.c_int64(V), ctypes.c_int64(hi - lo),
                          ctypes.c_int64(V), ctypes.c_double(tau), ctypes.c_void_p(0) if dd is None else _p(dd),
                          ctypes.c_int64(int(top_k)), ctypes.c_double(float(top_p)), off(out["thr"]), off(out["kept"]),
                          off(out["keep_mask"]), off(out["status"]), off(out["margin"]), _p(work))

    _fan_out(run, R, threads)
    return out


def _fan_out(run, n, threads):
    """Independent rows / sequences split over `threads` host threads (ctypes drops the GIL)."""
    threads = max(1, min(int(threads), n))
    if threads == 1:
        run(0, n)
        return
    bounds = [(i * n // threads, (i + 1) * n // threads) for i in range(threads)]
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda b: run(*b), bounds))
