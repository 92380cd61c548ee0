"""Seeded random rows through the row-level entry points against the oracle: one token per row and the argmax, the
warpers (rewritten rows, thresholds alone, draws from rows given with thresholds), greedy and union drafts -- rows of a
few ids to forty chunks, one row to a thousand, ties everywhere (values rounded to halves), stretches of -inf, NaN
inside such stretches, +inf, rows without mass, one dominant logit, uniforms at both ends of [0, 1).  Every case
prints what it is before it runs."""
import numpy as np
import pytest
import torch

from paper_2502_05202_amd import binding, synth

import parity
from test_gpu_next import _check_warp

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _rows(rng, gen, R, V, stride, dtype, allow_bad=True):
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    buf = (torch.randn(R, stride, generator=gen, device=DEV) * float(rng.choice([0.3, 3.0, 12.0]))).to(tdt)
    if rng.integers(3) == 0:
        buf = (torch.round(buf.float() * 2) / 2).to(tdt)
    buf[:, V:] = 60.0  # padding beyond V must be ignored
    for _ in range(int(rng.integers(0, 4))):
        r, ev = int(rng.integers(R)), int(rng.integers(6))
        a, n = int(rng.integers(0, V)), int(rng.integers(1, V))
        if ev == 0:
            buf[r, a:min(V, a + n)] = float("-inf")
        elif ev == 1:
            buf[r, :V] = float(rng.choice([1.25, -3.0, 0.0]))
        elif ev == 2 and allow_bad:
            buf[r, a:min(V, a + n)] = float("-inf")
            buf[r, min(V - 1, a + int(rng.integers(0, 40)))] = float("nan")
        elif ev == 3 and allow_bad:
            buf[r, a] = float("inf")
        elif ev == 4:
            buf[r, :V] = float("-inf")
        elif ev == 5:
            buf[r, a] = 40.0
    return buf


def _one_case(oracle, seed):
    rng = np.random.default_rng(seed)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    dtype = ["bf16", "f32"][rng.integers(2)]
    chunk, epv = (2048, 8) if dtype == "bf16" else (1024, 4)
    V = int(rng.choice([rng.integers(4, 200), rng.integers(200, 3 * chunk), rng.integers(chunk, 40 * chunk), chunk * rng.integers(1, 6)]))
    R = int(rng.choice([1, rng.integers(1, 12), rng.integers(12, 300), rng.integers(300, 1200)]))
    R = min(R, max(1, 4_000_000 // V))
    stride = (V + epv - 1) // epv * epv + epv * int(rng.integers(0, 3))
    tau = float(rng.choice([0.05, 0.3, 0.8, 1.0, 2.5]))
    what = int(rng.integers(4))
    print(f"seed {seed}: case {what} {dtype} V={V} R={R} stride={stride} tau={tau}", flush=True)
    buf = _rows(rng, gen, R, V, stride, dtype)
    view = buf[:, :V]
    rows = synth.logits_to_numpy(view.contiguous())
    u = synth._uniform24(R, gen, DEV)
    if rng.integers(4) == 0:
        u[: max(1, R // 3)] = 0.0
    if rng.integers(4) == 0:
        u[-max(1, R // 3):] = 1.0 - 2.0 ** -24
    un = u.cpu().numpy().astype(np.float64)
    if what == 0:  # one token per row, and the argmax
        for t in (tau, 0.0):
            g = parity.to_host(binding.tli_sample_rows(view, t, u))
            ref = oracle.sample_rows(rows, parity.f32(t), un, threads=8)
            if t == 0.0:
                assert np.array_equal(g["tok"], ref["tok"]) and np.array_equal(g["status"], ref["status"])
                continue
            rep = parity.compare_row_tokens(oracle, rows, t, un, g["tok"], g["status"], ref,
                                            lambda r: oracle.softmax(rows[r], parity.f32(t))[0])
            assert rep["hard"] == 0
            same = (g["tok"] == ref["tok"]) & (ref["status"] == 0) & (ref["p_tok"] >= 1e-290)
            if same.any():
                assert np.abs(g["lse"][same] - ref["lse"][same]).max() < parity.REL_TOL
                assert (np.abs(g["p_tok"][same] - ref["p_tok"][same]) / ref["p_tok"][same]).max() < parity.REL_TOL
        return
    top_k = int(rng.choice([0, 1, 5, 50, 1000, 10 ** 7]))
    top_p = float(rng.choice([1.0, 0.9, 0.5, 1e-7, 0.999]))
    if top_k == 0 and top_p == 1.0:
        top_k = 3
    if what == 1:  # warpers on rows of any vocabulary
        _check_warp(oracle, view, rows, tau, top_k, top_p, None, None)
        return
    # with a map (the oracle wants the unshared drafter logits finite or -inf: no NaN / +inf rows here)
    Vt = int(rng.integers(8, 3 * chunk)) // 8 * 8 + 8
    S = int(rng.choice([1, rng.integers(1, min(V, Vt) + 1), min(V, Vt)]))
    d2t = synth.make_d2t(V, Vt, S, seed)
    buf = _rows(rng, gen, R, V, stride, dtype, allow_bad=False)
    view = buf[:, :V]
    rows = synth.logits_to_numpy(view.contiguous())
    m = binding.tli_build_map(d2t, Vt)
    ws = binding.alloc_workspace(R, 1, m, binding.TLI_F32 if dtype == "f32" else binding.TLI_BF16, DEV)
    if what == 2:  # greedy and union drafts
        g = parity.to_host(binding.tli_greedy_draft(m, view, ws))
        ref = oracle.greedy_draft(rows, d2t, threads=8)
        for k in ("tok_d", "tok_t", "status"):
            assert np.array_equal(g[k], ref[k]), k
        g = parity.to_host(binding.tli_union_draft_sample(m, view, tau, u, ws))
        ref = oracle.union_draft_sample(rows, parity.f32(tau), d2t, un, threads=8)
        rep = parity.compare_row_tokens(oracle, rows, tau, un, g["tok_d"], g["status"], ref,
                                        lambda r: oracle.softmax(rows[r], parity.f32(tau))[0])
        assert rep["hard"] == 0
    else:  # warpers over the shared ids, and TLI drafts from the rows given with their thresholds
        _check_warp(oracle, view, rows, tau, top_k, top_p, d2t, m)
        gw = binding.tli_warp_rows(view, tau, top_k, top_p, m=m, rewrite=False)
        gd = parity.to_host(binding.tli_draft_sample_warped(m, view, tau, gw["thr"], u, ws))
        rw = oracle.warp_rows(rows, parity.f32(tau), top_k, float(np.float32(top_p)), d2t=d2t, threads=8)
        ninf = 0xFF80 if rows.dtype == np.uint16 else np.float32(-np.inf)
        ref = oracle.draft_sample(np.where(rw["keep_mask"].astype(bool), rows, ninf), parity.f32(tau), d2t, un, threads=8)
        for r in np.nonzero((rw["status"] == 0) & (rw["margin"] > parity.NEAR_TIE))[0]:  # (rows whose cut is not itself a near-tie)
            assert gd["status"][r] == ref["status"][r], r
            assert ref["status"][r] or gd["tok_d"][r] == ref["tok_d"][r] or ref["margin"][r] < parity.NEAR_TIE, r
    m.free()


@pytest.mark.parametrize("block", range(8))
def test_random_rows_sample_warp_greedy_union(oracle, block):
    for seed in range(61000 + 25 * block, 61000 + 25 * (block + 1)):
        _one_case(oracle, seed)
