"""Seeded random structures through the whole path against the oracle: vocabulary sizes from a few ids to a dozen
chunks, intersections from one shared token to all of them (scattered or in one stretch), temperatures from 0.05 to 8,
value distributions of all three kinds, and on top of them stretches of -inf, NaN / +inf inside such stretches,
constant rows, identical models (every draft accepted) and uniforms at both ends of [0, 1).  Both forms of
tli_verify's first steps are taken.  Every case prints what it is before it runs."""
import numpy as np
import pytest
import torch

from paper_2502_05202_amd import binding, synth

import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _restore_choice():
    yield
    binding.tli_tune_final_path(0)


def _draw_case(seed):
    rng = np.random.default_rng(seed)
    dtype = ["bf16", "f32"][rng.integers(2)]
    chunk = 2048 if dtype == "bf16" else 1024

    def size():
        v = int(rng.choice([rng.integers(8, 200), rng.integers(200, 3 * chunk), rng.integers(chunk, 12 * chunk),
                            chunk * rng.integers(1, 6)]))
        return max(8, v // 8 * 8)  # contiguous rows must be whole 16-byte vectors

    Vt, Vd = size(), size()
    smax = min(Vt, Vd)
    S = max(1, min(smax, int(rng.choice([1, rng.integers(1, smax // 50 + 2), rng.integers(1, smax + 1), smax]))))
    B, K = int(rng.integers(1, 10)), int(rng.integers(1, 7))
    tau_t, tau_d = (float(rng.choice([0.05, 0.3, 0.7, 1.0, 1.5, 8.0])) for _ in range(2))
    kind = ["noise", "corr", "zipf"][rng.integers(3)]
    w = synth.Workload("random", 99, B, K, Vt, Vd, S, dtype, tau_t, tau_d, kind, sigma=float(rng.choice([0.5, 3.0, 10.0])),
                       noise=float(rng.choice([0.0, 0.01, 1.0])), only_mu=float(rng.choice([0.0, -5.0, -40.0])),
                       rho=float(rng.choice([0.0, 0.7, 0.99, 1.0])))
    inp = synth.make_inputs(w, DEV, seed=seed)
    if rng.integers(4) == 1:  # the intersection in one stretch on either side
        d2t = np.full(Vd, -1, np.int32)
        d0, t0 = int(rng.integers(0, Vd - S + 1)), int(rng.integers(0, Vt - S + 1))
        d2t[d0:d0 + S] = (t0 + rng.permutation(S)).astype(np.int32)
        inp["d2t"] = d2t
    d2t = inp["d2t"]
    lt, ld = inp["logits_t"], inp["logits_d"]
    sh = np.nonzero(d2t >= 0)[0]
    ev = int(rng.integers(6))
    b, k = int(rng.integers(B)), int(rng.integers(K))
    if ev == 1:  # stretches of -inf
        a = int(rng.integers(0, Vt)); lt[b, k, a:a + int(rng.integers(1, Vt))] = float("-inf")
        a = int(rng.integers(0, Vd)); ld[b, k, a:a + int(rng.integers(1, Vd))] = float("-inf")
    elif ev == 2:  # NaN / +inf anywhere in a target row or on a shared drafter id, possibly inside a stretch of -inf
        if rng.integers(2):
            a = int(rng.integers(0, Vt)); lt[b, k, a:a + int(rng.integers(1, Vt))] = float("-inf")
            lt[b, k, min(Vt - 1, a + int(rng.integers(0, 50)))] = float(["nan", "inf"][rng.integers(2)])
        else:
            x = int(sh[rng.integers(len(sh))])
            if rng.integers(2):
                ld[b, k, max(0, x - 3000):x + 3000] = float("-inf")
            ld[b, k, x] = float(["nan", "inf"][rng.integers(2)])
    elif ev == 3:  # constant rows
        lt[b, k, :] = 1.25
        ld[b, k, :] = -0.5
    elif ev == 4:  # the two models agree on the shared ids and the target has nothing else: everything is accepted
        t_idx = torch.from_numpy(d2t[sh].astype(np.int64)).to(DEV)
        d_idx = torch.from_numpy(sh).to(DEV)
        lt[:, :K, :] = float("-inf") if rng.integers(2) else -60.0
        lt[:, :K, t_idx] = ld[:, :, d_idx]
        w = w.scaled(tau_t=w.tau_d)
        inp["workload"], inp["tau_t"] = w, w.tau_d
    elif ev == 5:  # uniforms at the ends
        inp["u_draft"][b, :] = 0.0
        inp["u_acc"][b, :] = 0.0
        inp["u_fin"][b] = 1.0 - 2.0 ** -24
    path = int(rng.integers(3))
    return w, inp, path, f"seed {seed}: {dtype} Vt={Vt} Vd={Vd} S={S} B={B} K={K} tau=({w.tau_t}, {w.tau_d}) {kind} extra={ev} form={path}"


@pytest.mark.parametrize("block", range(8))
def test_random_structures_draft_verify_and_rates(oracle, block):
    for seed in range(52000 + 40 * block, 52000 + 40 * (block + 1)):
        w, inp, path, what = _draw_case(seed)
        print(what, flush=True)
        binding.tli_tune_final_path(path)
        res = parity.run_case(oracle, inp, threads=8, chain=True)
        for name in ("draft", "verify", "chained"):
            assert res[name]["hard"] == 0, (what, name, dict(res[name]))
        if seed % 3 == 0:
            m = binding.tli_build_map(inp["d2t"], w.Vt)
            lt, ld = inp["logits_t"], inp["logits_d"]
            g = parity.to_host(binding.tli_acceptance_rates(m, lt, ld, w.tau_t, w.tau_d))
            ref = oracle.acceptance_rates(synth.logits_to_numpy(lt)[:, :w.K].reshape(w.B * w.K, w.Vt),
                                          synth.logits_to_numpy(ld).reshape(w.B * w.K, w.Vd), parity.f32(w.tau_t),
                                          parity.f32(w.tau_d), inp["d2t"], threads=8)
            assert np.array_equal(g["status"].reshape(-1), ref["status"]), what
            ok = ref["status"] == 0
            for name in ("alpha_tli", "alpha_union"):
                gg, rr = g[name].reshape(-1)[ok], ref[name][ok]
                big = rr >= 1e-290
                rel = np.abs(gg[big] - rr[big]) / rr[big]
                assert rel.size == 0 or rel.max() < 1e-5, (what, name, rel.max())
                assert np.all(gg[~big] < 1e-289), (what, name)
            m.free()
