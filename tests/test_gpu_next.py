"""GPU parity of the entry points beyond the TLI step -- union algorithm, expected acceptance rates, one
token per row / argmax, greedy TLI draft, exact-match tail -- against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2502_05202_amd import binding, synth

import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

SHAPES = [
    # (B, K, Vt, Vd, S, dtype, tau_t, tau_d)
    (5, 3, 2048 * 3 + 40, 2048 * 2 + 24, 1500, "bf16", 0.7, 0.9),
    (3, 4, 1024 * 4 + 28, 1024 + 4, 700, "f32", 1.0, 1.0),
    (40, 2, 10000, 30000, 9000, "bf16", 0.8, 1.1),
    (2, 2, 2048 * 30 + 16, 2048 * 27 + 8, 50000, "bf16", 0.9, 1.0),
    (2, 2, 70000, 60000, 50000, "f32", 1.0, 0.9),  # three parts in the residual scan
]
IDS = [f"B{c[0]}_Vt{c[2]}_{c[5]}" for c in SHAPES]


def _inputs(shape, cfg=70):
    B, K, Vt, Vd, S, dtype, tt, td = shape
    w = synth.WORKLOADS[3].scaled(B=B, K=K, Vt=Vt, Vd=Vd, S=S, dtype=dtype, tau_t=tt, tau_d=td, cfg=cfg)
    return w, synth.make_inputs(w, DEV)


def _rates_close(got, want):
    """Expected acceptance rates: one rule, 1e-5 relative (the tolerance the probabilities are held to), for every
    rate down to 1e-290; what is smaller still must come out below 1e-289."""
    got, want = np.asarray(got, np.float64).reshape(-1), np.asarray(want, np.float64).reshape(-1)
    big = want >= 1e-290
    rel = np.abs(got[big] - want[big]) / want[big]
    assert rel.size == 0 or rel.max() < 1e-5, (rel.max(), want[big][rel.argmax()], got[big][rel.argmax()])
    assert np.all(got[~big] < 1e-289)
    return float(rel.max()) if rel.size else 0.0


@pytest.mark.parametrize("shape", SHAPES, ids=IDS)
def test_union_draft_and_verify(oracle, shape):
    w, inp = _inputs(shape)
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    code = binding.TLI_F32 if w.dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(w.B, w.K, m, code, DEV)
    lt_np, ld_np = synth.logits_to_numpy(inp["logits_t"]), synth.logits_to_numpy(inp["logits_d"])
    rows = ld_np.reshape(w.B * w.K, w.Vd)
    ud = inp["u_draft"].cpu().numpy().astype(np.float64).reshape(-1)
    ua = inp["u_acc"].cpu().numpy().astype(np.float64)
    uf = inp["u_fin"].cpu().numpy().astype(np.float64)
    td, tt = parity.f32(w.tau_d), parity.f32(w.tau_t)
    g = parity.to_host(binding.tli_union_draft_sample(m, inp["logits_d"], w.tau_d, inp["u_draft"].reshape(-1), ws))
    ref = oracle.union_draft_sample(rows, td, inp["d2t"], ud, threads=8)
    rep = parity.compare_row_tokens(oracle, rows, td, ud, g["tok_d"], g["status"], ref,
                                    lambda r: oracle.softmax(rows[r], td)[0])
    same = (ref["status"] == 0) & (g["tok_d"] == ref["tok_d"])
    assert np.array_equal(g["tok_t"][same], ref["tok_t"][same])
    assert w.B * w.K < 12 or (ref["tok_t"] < 0).any()  # some drafts fall outside T
    assert np.abs(g["lse_q"][same] - ref["lse_q"][same]).max() < 5e-7
    assert (np.abs(g["q_tok"][same] - ref["q_tok"][same]) / ref["q_tok"][same]).max() < 1e-6
    assert rep["hard"] == 0, dict(rep)
    # verify on the oracle's union drafts (some lie outside T), with and without the normalisers
    tok = torch.from_numpy(ref["tok_d"]).to(DEV)
    for lse_q in (torch.from_numpy(ref["lse_q"]).to(DEV), None):
        gv = binding.tli_union_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d, tok, lse_q,
                                      inp["u_acc"].reshape(-1), inp["u_fin"], ws)
        torch.cuda.synchronize()
        rv, refv = parity.compare_verify(oracle, lt_np, ld_np, w.tau_t, w.tau_d, inp["d2t"], ref["tok_d"], ua, uf,
                                         parity.to_host(gv), threads=8, fn="union_verify")
        print(dict(rv))
        assert rv["hard"] == 0 and rv["max_lse_err"] < 5e-7 and rv["max_prob_rel"] < 1e-6
    m.free()


def test_union_flags(oracle):
    w, inp = _inputs((6, 3, 6000, 4104, 2000, "bf16", 0.8, 0.8), cfg=71)
    d2t = inp["d2t"]
    unshared = np.nonzero(d2t < 0)[0]
    ld = inp["logits_d"]
    ld[0, 1, int(unshared[3])] = float("nan")      # an unshared logit matters to the union algorithm
    ld[1, 0, :] = float("-inf")
    m = binding.tli_build_map(d2t, w.Vt)
    ws = binding.alloc_workspace(w.B, w.K, m, binding.TLI_BF16, DEV)
    rows = synth.logits_to_numpy(ld).reshape(w.B * w.K, w.Vd)
    ud = inp["u_draft"].cpu().numpy().astype(np.float64).reshape(-1)
    g = parity.to_host(binding.tli_union_draft_sample(m, ld, w.tau_d, inp["u_draft"].reshape(-1), ws))
    ref = oracle.union_draft_sample(rows, parity.f32(w.tau_d), d2t, ud, threads=4)
    assert np.array_equal(g["status"], ref["status"]) and ref["status"][1] == oracle.NONFINITE and ref["status"][3] == oracle.ZERO_MASS
    # verify: a valid draft id on the NaN row flags the sequence; out-of-range ids are BAD_DRAFT
    tok = ref["tok_d"].reshape(w.B, w.K).copy()
    tok[0, 1] = 5
    tok[2, 0] = w.Vd + 3
    tok[3, 2] = int(unshared[0])
    gv = binding.tli_union_verify(m, inp["logits_t"], ld, w.tau_t, w.tau_d, torch.from_numpy(tok).to(DEV), None,
                                  inp["u_acc"].reshape(-1), inp["u_fin"], ws)
    torch.cuda.synchronize()
    rv, refv = parity.compare_verify(oracle, synth.logits_to_numpy(inp["logits_t"]), synth.logits_to_numpy(ld), w.tau_t,
                                     w.tau_d, d2t, tok, inp["u_acc"].cpu().numpy().astype(np.float64),
                                     inp["u_fin"].cpu().numpy().astype(np.float64), parity.to_host(gv), threads=4,
                                     fn="union_verify")
    assert rv["hard"] == 0
    assert refv["status"][0] & oracle.NONFINITE and refv["status"][2] & oracle.BAD_DRAFT and refv["status"][3] == 0
    m.free()


@pytest.mark.parametrize("shape", SHAPES, ids=IDS)
def test_acceptance_rates(oracle, shape):
    w, inp = _inputs(shape, cfg=72)
    lt, ld = inp["logits_t"], inp["logits_d"]
    d2t = inp["d2t"]
    if w.B >= 3:  # flags: NaN in an unshared drafter logit, zero shared mass, -inf stretch in a target row
        ld[0, 0, int(np.nonzero(d2t < 0)[0][0])] = float("nan")
        ld[1, 1, torch.from_numpy(np.nonzero(d2t >= 0)[0]).to(DEV)] = float("-inf")
        lt[2, 0, : w.Vt // 2] = float("-inf")
    if w.B >= 4:  # a NaN with nothing but -inf around it still flags its position (target row; shared drafter id)
        lt[3, 0, : w.Vt // 2] = float("-inf")
        lt[3, 0, 11] = float("nan")
        sh_ = np.nonzero(d2t >= 0)[0]
        ld[3, 1, : w.Vd // 2] = float("-inf")
        ld[3, 1, int(sh_[0])] = float("nan")
    m = binding.tli_build_map(d2t, w.Vt)
    g = parity.to_host(binding.tli_acceptance_rates(m, lt, ld, w.tau_t, w.tau_d))
    lt_np = synth.logits_to_numpy(lt)[:, : w.K].reshape(w.B * w.K, w.Vt)
    ld_np = synth.logits_to_numpy(ld).reshape(w.B * w.K, w.Vd)
    ref = oracle.acceptance_rates(lt_np, ld_np, parity.f32(w.tau_t), parity.f32(w.tau_d), d2t, threads=8)
    assert np.array_equal(g["status"].reshape(-1), ref["status"])
    ok = ref["status"] == 0
    for name in ("alpha_tli", "alpha_union"):
        gg, rr = g[name].reshape(-1), ref[name]
        assert np.all(np.isnan(gg[ref["status"] == oracle.NONFINITE]))
        assert np.all(gg[ref["status"] == oracle.ZERO_MASS] == 0.0)
        print(name, "max rel err", _rates_close(gg[ok], rr[ok]), "range", rr[ok].min(), rr[ok].max())
    assert np.all(g["alpha_union"].reshape(-1)[ok] <= g["alpha_tli"].reshape(-1)[ok] * (1 + 1e-9))
    m.free()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_acceptance_rates_when_unshared_logits_dwarf_the_shared(oracle, dtype):
    """Both drafter normalisers come from one pass that shares its exponentials; where the shared ids of a chunk lie
    far below its largest logit (here: one unshared logit of +80 in the first chunk of every other row), or a chunk
    holds no shared id at all (every chunk but the first), the shared ones are reduced on their own."""
    chunk = 2048 if dtype == "bf16" else 1024
    Vd, Vt, B, K, S = chunk * 3 + 24, 5000, 4, 3, 400
    rng = np.random.default_rng(11)
    d2t = np.full(Vd, -1, np.int32)
    sh = np.sort(rng.permutation(chunk)[:S])                      # shared drafter ids: first chunk only
    d2t[sh] = rng.permutation(Vt)[:S].astype(np.int32)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(12)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    lt = (torch.randn(B, K + 1, Vt, generator=gen, device=DEV) * 3).to(tdt)
    ld = (torch.randn(B, K, Vd, generator=gen, device=DEV) * 3).to(tdt)
    big = int(np.setdiff1d(np.arange(chunk), sh)[5])
    ld[::2, :, big] = 80.0
    m = binding.tli_build_map(d2t, Vt)
    g = parity.to_host(binding.tli_acceptance_rates(m, lt, ld, 0.9, 1.0))
    ref = oracle.acceptance_rates(synth.logits_to_numpy(lt)[:, :K].reshape(B * K, Vt),
                                  synth.logits_to_numpy(ld).reshape(B * K, Vd), parity.f32(0.9), parity.f32(1.0), d2t, threads=4)
    assert np.all(ref["status"] == 0) and np.all(g["status"] == 0)
    for name in ("alpha_tli", "alpha_union"):
        print(name, "max rel err", _rates_close(g[name], ref[name]), "range", ref[name].min(), ref[name].max())
        rel = np.abs(g[name].reshape(-1) - ref[name]) / ref[name]
        assert rel.max() < 1e-5  # these vanishing rates (1e-31) are still normal fp32 numbers: the path's general 1e-5
    assert ref["alpha_union"].reshape(B, K)[0].max() < 1e-20 < ref["alpha_union"].reshape(B, K)[1].min()
    m.free()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_acceptance_rates_of_a_cold_drafter_whose_favourite_is_unshared(oracle, dtype):
    """A drafter at temperature 0.05 with one unshared logit 8 to 14 above every shared one: q = q' * 2^-dq with dq
    between 230 and 400 binary orders, alpha_union between 1e-70 and 1e-120.  dq has to enter the sums with more than
    the 24 bits of an fp32 (2^-24 of 300 is 1.2e-5 of the rate)."""
    chunk = 2048 if dtype == "bf16" else 1024
    Vd, Vt, B, K, S = chunk * 2 + 40, chunk * 2 + 24, 5, 3, 900
    rng = np.random.default_rng(41)
    d2t = np.full(Vd, -1, np.int32)
    sh = np.sort(rng.permutation(Vd)[:S])
    d2t[sh] = rng.permutation(Vt)[:S].astype(np.int32)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(42)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ld = (torch.randn(B, K, Vd, generator=gen, device=DEV) * 0.5).to(tdt)
    lt = (torch.randn(B, K + 1, Vt, generator=gen, device=DEV) * 2).to(tdt)
    un = int(np.setdiff1d(np.arange(Vd), sh)[7])
    for b in range(B):
        for k in range(K):
            ld[b, k, un] = 10.0 + 2.0 * ((b * K + k) % 4)
    m = binding.tli_build_map(d2t, Vt)
    g = parity.to_host(binding.tli_acceptance_rates(m, lt, ld, 1.0, 0.05))
    ref = oracle.acceptance_rates(synth.logits_to_numpy(lt)[:, :K].reshape(B * K, Vt),
                                  synth.logits_to_numpy(ld).reshape(B * K, Vd), 1.0, parity.f32(0.05), d2t, threads=4)
    assert np.all(ref["status"] == 0) and np.all(g["status"] == 0)
    assert 1e-130 < ref["alpha_union"].min() and ref["alpha_union"].max() < 1e-60
    for name in ("alpha_tli", "alpha_union"):
        print(name, "max rel err", _rates_close(g[name], ref[name]), "range", ref[name].min(), ref[name].max())
    m.free()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_acceptance_rates_of_nearly_disjoint_models(oracle, dtype):
    """Drafter and target that put their mass on different shared tokens: the rates run from 1e-3 down to 1e-200,
    far below what an fp32 term holds, and every one of them must still be good to 1e-5 relative."""
    chunk = 2048 if dtype == "bf16" else 1024
    Vd, Vt, B, K, S = chunk * 2 + 40, chunk * 3 + 24, 6, 4, 1500
    rng = np.random.default_rng(31)
    d2t = np.full(Vd, -1, np.int32)
    sh = np.sort(rng.permutation(Vd)[:S])
    d2t[sh] = rng.permutation(Vt)[:S].astype(np.int32)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(32)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    ld = (torch.randn(B, K, Vd, generator=gen, device=DEV) * 2).to(tdt)
    lt = (torch.randn(B, K + 1, Vt, generator=gen, device=DEV) * 2).to(tdt)
    # sequence 0: the target repeats the drafter on the shared ids; sequence b > 0: it is the drafter's mirror image
    # there, scaled up with b
    sh_d = torch.from_numpy(sh).to(DEV)
    sh_t = torch.from_numpy(d2t[sh].astype(np.int64)).to(DEV)
    lt[0, :K, sh_t] = ld[0, :, sh_d]
    for b in range(1, B):
        lt[b, :K, sh_t] = (-(4.0 ** b) * ld[b, :, sh_d].float()).to(tdt)
    m = binding.tli_build_map(d2t, Vt)
    g = parity.to_host(binding.tli_acceptance_rates(m, lt, ld, 0.1, 0.1))
    ref = oracle.acceptance_rates(synth.logits_to_numpy(lt)[:, :K].reshape(B * K, Vt),
                                  synth.logits_to_numpy(ld).reshape(B * K, Vd), parity.f32(0.1), parity.f32(0.1), d2t, threads=4)
    assert np.all(ref["status"] == 0) and np.all(g["status"] == 0)
    for name in ("alpha_tli", "alpha_union"):
        print(name, "max rel err", _rates_close(g[name], ref[name]), "range", ref[name].min(), ref[name].max())
    assert ref["alpha_tli"].min() < 1e-60 and ref["alpha_tli"].max() > 1e-3  # both passes of the scan are taken
    m.free()


@pytest.mark.parametrize("dtype,V,R,stride", [("bf16", 2048 * 3 + 40, 9, 2048 * 3 + 48), ("f32", 5000, 3, 5000),
                                               ("bf16", 151936, 2, 151936), ("bf16", 4104, 1500, 4104)])
def test_sample_rows_and_argmax(oracle, dtype, V, R, stride):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(V + R)
    buf = (torch.randn(R, stride, generator=gen, device=DEV) * 3).to(torch.bfloat16 if dtype == "bf16" else torch.float32)
    buf[:, V:] = 60.0  # padding beyond V must be ignored
    view = buf[:, :V]
    u = synth._uniform24(R, gen, DEV)
    rows = synth.logits_to_numpy(view.contiguous())
    un = u.cpu().numpy().astype(np.float64)
    for tau in (0.8, 0.0):
        g = parity.to_host(binding.tli_sample_rows(view, tau, u))
        ref = oracle.sample_rows(rows, parity.f32(tau), un, threads=8)
        if tau == 0.0:
            assert np.array_equal(g["tok"], ref["tok"]) and np.array_equal(g["status"], ref["status"])
            assert np.all(g["p_tok"] == 1.0) and np.all(np.isnan(g["lse"]))
        else:
            rep = parity.compare_row_tokens(oracle, rows, tau, un, g["tok"], g["status"], ref,
                                            lambda r: oracle.softmax(rows[r], parity.f32(tau))[0])
            assert rep["hard"] == 0
            same = g["tok"] == ref["tok"]
            assert np.abs(g["lse"][same] - ref["lse"][same]).max() < 5e-7
            assert (np.abs(g["p_tok"][same] - ref["p_tok"][same]) / ref["p_tok"][same]).max() < 1e-6


def test_argmax_ties_and_flags(oracle):
    V, R = 2048 * 2 + 16, 6
    x = torch.zeros(R, V, dtype=torch.bfloat16, device=DEV)
    x[0, [5, 4000, 2049]] = 7.0          # equal maxima in different chunks and lanes: the lowest id wins
    x[1, V - 1] = 1.0                    # the last id of the ragged tail
    x[2, :] = float("-inf")              # nothing to choose from
    x[3, 77] = float("nan")
    x[4, 3000] = float("inf")
    x[5, :] = float("-inf"); x[5, 2048] = -3.0
    g = parity.to_host(binding.tli_sample_rows(x, 0.0, None))
    ref = oracle.sample_rows(synth.logits_to_numpy(x), 0.0, np.zeros(R))
    assert np.array_equal(g["tok"], ref["tok"]) and list(g["tok"]) == [5, V - 1, -1, -1, -1, 2048]
    assert np.array_equal(g["status"], ref["status"])


@pytest.mark.parametrize("shape", SHAPES, ids=IDS)
def test_greedy_draft_and_temperature_zero_verify(oracle, shape):
    w, inp = _inputs(shape, cfg=73)
    d2t = inp["d2t"]
    lt, ld = inp["logits_t"], inp["logits_d"]
    sh = np.nonzero(d2t >= 0)[0]
    # make the target agree with the drafter's shared argmax on a prefix of length b % (K+1)
    ld_h = ld.float().cpu().numpy()
    for b in range(w.B):
        for k in range(b % (w.K + 1)):
            d = sh[np.argmax(ld_h[b, k, sh])]
            lt[b, k, int(d2t[d])] = 50.0
    if w.B >= 3:
        ld[1, 0, torch.from_numpy(sh).to(DEV)] = float("-inf")
        ld[2, 1, int(sh[0])] = float("nan")
    m = binding.tli_build_map(d2t, w.Vt)
    code = binding.TLI_F32 if w.dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(w.B, w.K, m, code, DEV)
    g = binding.tli_greedy_draft(m, ld, ws)
    gh = parity.to_host(g)
    ref = oracle.greedy_draft(synth.logits_to_numpy(ld).reshape(w.B * w.K, w.Vd), d2t, threads=8)
    for k in ("tok_d", "tok_t", "status"):
        assert np.array_equal(gh[k], ref[k]), k
    v = parity.to_host(binding.tli_exact_match_verify(lt, 0.0, g["tok_t"], None))
    rv = oracle.exact_match_verify(synth.logits_to_numpy(lt), 0.0, ref["tok_t"].reshape(w.B, w.K),
                                   np.zeros((w.B, w.K + 1)), threads=8)
    assert np.array_equal(v["n_accepted"], rv["n_acc"]) and np.array_equal(v["out_tok"], rv["out_tok"])
    assert np.array_equal(v["tgt_tok"], rv["tgt_tok"]) and np.array_equal(v["status"], rv["status"])
    if w.B > w.K:
        assert len(set(rv["n_acc"])) >= 3  # several prefix lengths are exercised
    m.free()


def test_greedy_draft_many_rows_several_chunks_per_wave(oracle):
    """Enough rows for one workgroup per row: every wave then owns several chunks, and the lanes of a wave find
    their maxima in different chunks (the shared-id mask of the final look-up is per lane)."""
    R, Vd, Vt, S = 2100, 2048 * 9 + 24, 4104, 3000
    d2t = synth.make_d2t(Vd, Vt, S, 321)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(12)
    for dt in (torch.bfloat16, torch.float32):
        ld = (torch.randn(R, Vd, generator=gen, device=DEV) * 3).to(dt)
        m = binding.tli_build_map(d2t, Vt)
        ws = binding.alloc_workspace(R, 1, m, binding._dtype_code(ld), DEV)
        g = parity.to_host(binding.tli_greedy_draft(m, ld, ws))
        ref = oracle.greedy_draft(synth.logits_to_numpy(ld), d2t, threads=8)
        for k in ("tok_d", "tok_t", "status"):
            assert np.array_equal(g[k], ref[k]), k
        u = synth._uniform24(R, gen, DEV)
        g0 = parity.to_host(binding.tli_sample_rows(ld, 0.0, None))
        assert np.array_equal(g0["tok"], oracle.sample_rows(synth.logits_to_numpy(ld), 0.0, np.zeros(R), threads=8)["tok"])
        m.free()


@pytest.mark.parametrize("shape", SHAPES, ids=IDS)
def test_exact_match_tail_sampled(oracle, shape):
    w, inp = _inputs(shape, cfg=74)
    lt = inp["logits_t"]
    B, m = w.B, w.K
    gen = torch.Generator(device=DEV)
    gen.manual_seed(99)
    u = synth._uniform24(B * (m + 1), gen, DEV).reshape(B, m + 1)
    lt_np = synth.logits_to_numpy(lt)
    un = u.cpu().numpy().astype(np.float64)
    tau = parity.f32(w.tau_t)
    own = oracle.sample_rows(lt_np.reshape(-1, w.Vt), tau, un.reshape(-1), threads=8)
    draft = own["tok"].reshape(B, m + 1)[:, :m].copy()
    for b in range(B):  # break the match at position b % (m+2) (m: a missing draft token, m+1: nowhere)
        j = b % (m + 2)
        if j < m:
            draft[b, j] = (draft[b, j] + 1) % w.Vt
        elif j == m:
            draft[b, m - 1] = -1
    if B >= 3:
        lt[2, 1, 9] = float("nan")
        lt[1, 0, : w.Vt // 2] = float("-inf")  # a NaN with nothing but -inf around it
        lt[1, 0, 3] = float("nan")
        lt_np = synth.logits_to_numpy(lt)
    g = parity.to_host(binding.tli_exact_match_verify(lt, w.tau_t, torch.from_numpy(draft).to(DEV), u))
    ref = oracle.exact_match_verify(lt_np, tau, draft, un, threads=8)
    assert np.array_equal(g["status"], ref["status"])
    near = 0
    for b in range(B):
        if ref["status"][b]:
            assert g["n_accepted"][b] == 0 and np.all(g["out_tok"][b] == -1)
            continue
        diff = np.nonzero(g["tgt_tok"][b] != ref["tgt_tok"][b])[0]
        if diff.size:  # a drawn id may differ only inside the near-tie window; the sequence is then compared no further
            for j in diff:
                p = oracle.softmax(lt_np[b, j], tau)[0]
                assert ref["margin"][b, j] < parity.NEAR_TIE and parity._cdf_distance(p, int(g["tgt_tok"][b, j]), un[b, j]) < parity.NEAR_TIE
            near += 1
            continue
        assert g["n_accepted"][b] == ref["n_acc"][b] and np.array_equal(g["out_tok"][b], ref["out_tok"][b])
    print("sequences with a near-tie draw:", near)


# ---------------------------------------------------------------- full size, in the launch configuration the benchmark times
def test_full_size_large_vocab_next_rows(oracle):
    """Workload 4 (B=256, K=8, Vt=256000, Vd=128256, bf16) through every neighbouring entry point; every output
    is compared (the oracle is fanned out over the host cores)."""
    w = synth.WORKLOADS[4]
    inp = synth.make_inputs(w, DEV)
    d2t = inp["d2t"]
    lt, ld = inp["logits_t"], inp["logits_d"]
    m = binding.tli_build_map(d2t, w.Vt)
    ws = binding.alloc_workspace(w.B, w.K, m, binding.TLI_BF16, DEV)
    lt_np, ld_np = synth.logits_to_numpy(lt), synth.logits_to_numpy(ld)
    rows_d = ld_np.reshape(w.B * w.K, w.Vd)
    tt, td = parity.f32(w.tau_t), parity.f32(w.tau_d)
    ud = inp["u_draft"].cpu().numpy().astype(np.float64).reshape(-1)
    ua = inp["u_acc"].cpu().numpy().astype(np.float64)
    uf = inp["u_fin"].cpu().numpy().astype(np.float64)
    # union algorithm
    g = parity.to_host(binding.tli_union_draft_sample(m, ld, w.tau_d, inp["u_draft"].reshape(-1), ws))
    ref = oracle.union_draft_sample(rows_d, td, d2t, ud, threads=16)
    rep = parity.compare_row_tokens(oracle, rows_d, td, ud, g["tok_d"], g["status"], ref,
                                    lambda r: oracle.softmax(rows_d[r], td)[0])
    assert rep["hard"] == 0 and np.abs(g["lse_q"] - ref["lse_q"]).max() < 5e-7
    gv = binding.tli_union_verify(m, lt, ld, w.tau_t, w.tau_d, torch.from_numpy(ref["tok_d"]).to(DEV),
                                  torch.from_numpy(ref["lse_q"]).to(DEV), inp["u_acc"].reshape(-1), inp["u_fin"], ws)
    torch.cuda.synchronize()
    rv, _ = parity.compare_verify(oracle, lt_np, ld_np, w.tau_t, w.tau_d, d2t, ref["tok_d"], ua, uf, parity.to_host(gv),
                                  threads=16, fn="union_verify")
    print("union verify", dict(rv))
    assert rv["hard"] == 0 and rv["max_lse_err"] < 5e-7
    # expected acceptance rates of all 2048 positions
    ga = parity.to_host(binding.tli_acceptance_rates(m, lt, ld, w.tau_t, w.tau_d))
    ra = oracle.acceptance_rates(lt_np[:, : w.K].reshape(-1, w.Vt), rows_d, tt, td, d2t, threads=16)
    assert np.all(ra["status"] == 0) and np.all(ga["status"] == 0)
    for name in ("alpha_tli", "alpha_union"):
        print(name, "max rel", _rates_close(ga[name], ra[name]), "mean", ra[name].mean())
    # exact-match tail over the 2304 target rows, sampled and at temperature zero; greedy drafts
    gen = torch.Generator(device=DEV)
    gen.manual_seed(404)
    u = synth._uniform24(w.B * (w.K + 1), gen, DEV).reshape(w.B, w.K + 1)
    un = u.cpu().numpy().astype(np.float64)
    gd = binding.tli_greedy_draft(m, ld, ws)
    rd = oracle.greedy_draft(rows_d, d2t, threads=16)
    assert np.array_equal(parity.to_host(gd)["tok_d"], rd["tok_d"]) and np.all(rd["status"] == 0)
    for tau in (w.tau_t, 0.0):
        own = oracle.sample_rows(lt_np.reshape(-1, w.Vt), parity.f32(tau), un.reshape(-1), threads=16)
        draft = own["tok"].reshape(w.B, w.K + 1)[:, : w.K].copy()
        for b in range(w.B):
            j = b % (w.K + 2)
            if j < w.K:
                draft[b, j] = (draft[b, j] + 1) % w.Vt
        ge = parity.to_host(binding.tli_exact_match_verify(lt, tau, torch.from_numpy(draft).to(DEV), u))
        re_ = oracle.exact_match_verify(lt_np, parity.f32(tau), draft, un, threads=16)
        near = 0
        for b in range(w.B):
            diff = np.nonzero(ge["tgt_tok"][b] != re_["tgt_tok"][b])[0]
            if diff.size:
                assert tau > 0
                for j in diff:
                    p = oracle.softmax(lt_np[b, j], parity.f32(tau))[0]
                    assert re_["margin"][b, j] < parity.NEAR_TIE and \
                        parity._cdf_distance(p, int(ge["tgt_tok"][b, j]), un[b, j]) < parity.NEAR_TIE
                near += 1
                continue
            assert ge["n_accepted"][b] == re_["n_acc"][b] and np.array_equal(ge["out_tok"][b], re_["out_tok"][b])
        print(f"exact match tau={tau}: near-tie sequences {near}, mean accepted {re_['n_acc'].mean():.2f}")
    m.free()


# ---------------------------------------------------------------- logit warpers
WARP = [("bf16", 2048 * 3 + 40, 9, 2048 * 3 + 48), ("f32", 5000, 4, 5000), ("bf16", 151936, 3, 151936), ("f32", 33000, 2, 33000),
        # rows that do not end on a vector boundary (the warped copy gets a row stride of whole vectors)
        ("bf16", 18847, 3, 18848), ("f32", 5001, 2, 5008)]


def _check_warp(oracle, view, rows, tau, top_k, top_p, d2t, m, pick=None):
    """pick: compare only these rows of `view` (then `rows` holds just those, in that order)."""
    g = binding.tli_warp_rows(view, tau, top_k, top_p, m=m)
    torch.cuda.synchronize()
    if pick is not None:
        at = torch.as_tensor(pick, device=view.device)
        g = {k: v[at] for k, v in g.items()}
    ref = oracle.warp_rows(rows, parity.f32(tau), top_k, float(np.float32(top_p)), d2t=d2t, threads=8)
    gs, gk, gt = g["status"].cpu().numpy(), g["kept"].cpu().numpy(), g["thr"].cpu().numpy().astype(np.float64)
    assert np.array_equal(gs, ref["status"])
    out = synth.logits_to_numpy(g["logits"])
    ninf = 0xFF80 if rows.dtype == np.uint16 else np.float32(-np.inf)
    near = 0
    for r in range(rows.shape[0]):
        if ref["status"][r]:
            assert gk[r] == 0 and np.isnan(gt[r])
            continue
        if gk[r] != ref["kept"][r]:
            # a top-p cut may move by one group of equal logits only if the oracle's own decision was within 1e-6
            assert ref["margin"][r] < parity.NEAR_TIE, (r, gk[r], ref["kept"][r], ref["margin"][r])
            near += 1
            continue
        assert gt[r] == ref["thr"][r] or (np.isinf(gt[r]) and np.isinf(ref["thr"][r])), (r, gt[r], ref["thr"][r])
        want = np.where(ref["keep_mask"][r].astype(bool), rows[r], ninf)
        if rows.dtype == np.float32:
            assert np.array_equal(out[r].view(np.uint32), want.view(np.uint32)) or np.array_equal(out[r], want)
        else:
            assert np.array_equal(out[r], want)
    # thresholds only (no rewrite): the rows at or above the threshold are the oracle's kept set
    g2 = binding.tli_warp_rows(view, tau, top_k, top_p, m=m, rewrite=False)
    torch.cuda.synchronize()
    if pick is not None:
        g2 = {k: v[at] for k, v in g2.items()}
    t2 = g2["thr"].cpu().numpy().astype(np.float64)
    assert np.array_equal(g2["status"].cpu().numpy(), ref["status"])
    fl = (rows.astype(np.uint32) << 16).view(np.float32) if rows.dtype == np.uint16 else rows
    competes = fl > -np.inf
    if d2t is not None:
        competes &= (np.asarray(d2t) >= 0)[None, :]
    for r in range(rows.shape[0]):
        if ref["status"][r]:
            assert np.isnan(t2[r])
            continue
        if gk[r] != ref["kept"][r]:
            continue  # the near-tie rows counted above
        assert np.array_equal(competes[r] & (fl[r] >= t2[r]), ref["keep_mask"][r].astype(bool)), (r, t2[r], gt[r])
    return near


@pytest.mark.parametrize("dtype,V,R,stride", WARP, ids=[f"{c[0]}_V{c[1]}" for c in WARP])
def test_warp_rows(oracle, dtype, V, R, stride):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(V + 7 * R)
    buf = (torch.randn(R, stride, generator=gen, device=DEV) * 3).to(torch.bfloat16 if dtype == "bf16" else torch.float32)
    buf[:, V:] = 60.0
    buf[0, 10:300] = float("-inf")
    buf[R - 1, 5] = -0.0
    buf[R - 1, 6] = 0.0
    if R >= 3:
        buf[1, :V] = 1.25  # a constant row: top-p reaches the bottom and drops nothing (threshold -inf), top-k keeps all ties
    view = buf[:, :V]
    rows = synth.logits_to_numpy(view.contiguous())
    near = 0
    for top_k, top_p, tau in [(50, 1.0, 1.0), (1, 1.0, 1.0), (0, 0.9, 0.8), (0, 0.3, 1.2), (200, 0.95, 0.7), (10 ** 7, 0.999, 1.0),
                              (0, 1e-7, 1.0), (7, 0.5, 1.0)]:
        near += _check_warp(oracle, view, rows, tau, top_k, top_p, None, None)
    print("top-p cuts inside the near-tie window:", near)
    # padding beyond V is left as the caller had it when the warp is done in place
    g = binding.tli_warp_rows(view, 1.0, 5, 1.0, out=view)
    torch.cuda.synchronize()
    assert torch.all(buf[:, V:] == 60.0) and int((buf[:, :V] > float("-inf")).sum()) == int(g["kept"].sum())


def test_warp_rows_flags_and_map(oracle):
    w = synth.WORKLOADS[3].scaled(B=4, K=3, Vt=6000, Vd=4104, S=2000, cfg=75)
    inp = synth.make_inputs(w, DEV)
    d2t = inp["d2t"]
    ld = inp["logits_d"].reshape(12, w.Vd).clone()
    sh = np.nonzero(d2t >= 0)[0]
    ld[1, int(sh[3])] = float("nan")
    ld[2, torch.from_numpy(sh).to(DEV)] = float("-inf")
    ld[3, int(np.nonzero(d2t < 0)[0][0])] = float("nan")  # unshared: ignored
    ld[5, :2048 + 100] = float("-inf")  # a NaN with nothing but -inf around it
    ld[5, int(sh[1])] = float("nan")
    m = binding.tli_build_map(d2t, w.Vt)
    rows = synth.logits_to_numpy(ld)
    for top_k, top_p in [(20, 1.0), (0, 0.9), (40, 0.8)]:
        _check_warp(oracle, ld, rows, 0.9, top_k, top_p, d2t, m)
    # the warped rows feed the TLI draft: only surviving shared ids can be drawn
    g = binding.tli_warp_rows(ld, 0.9, 3, 1.0, m=m)
    ws = binding.alloc_workspace(4, 3, m, binding.TLI_BF16, DEV)
    u = inp["u_draft"].reshape(-1)
    d = binding.tli_draft_sample(m, g["logits"], 0.9, u, ws)
    torch.cuda.synchronize()
    dr = oracle.draft_sample(synth.logits_to_numpy(g["logits"]), parity.f32(0.9), d2t, u.cpu().numpy().astype(np.float64))
    assert np.array_equal(d["tok_d"].cpu().numpy(), dr["tok_d"])
    m.free()


@pytest.mark.parametrize("dtype,V,R", [("bf16", 2048 * 5 + 24, 40), ("f32", 1024 * 9 + 4, 24), ("bf16", 151936, 6)])
def test_draws_from_rows_warped_by_threshold(oracle, dtype, V, R):
    """One token per row from rows given with their thresholds (no rewrite) against the oracle's draw from the rows the
    oracle warped; the same for TLI drafts with a map (only shared ids compete for the threshold and for the draw).
    Small batches run the split kernels, R = 40 x 28 rows of the first case the one-workgroup-per-row kernel."""
    gen = torch.Generator(device=DEV)
    gen.manual_seed(V + R)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    reps = 28 if V < 20000 and dtype == "bf16" else 1
    rows_t = (torch.randn(R * reps, V, generator=gen, device=DEV) * 3).to(tdt)
    rows_t[0, 10:300] = float("-inf")
    rows_t[1, :] = 1.25  # a constant row: nothing is dropped
    u = synth._uniform24(R * reps, gen, DEV)
    rows = synth.logits_to_numpy(rows_t)
    un = u.cpu().numpy().astype(np.float64)
    near = 0
    for top_k, top_p, tau in [(50, 0.9, 0.8), (0, 0.7, 1.1), (5, 1.0, 1.0), (300, 0.99, 0.6)]:
        wr = oracle.warp_rows(rows, parity.f32(tau), top_k, float(np.float32(top_p)), threads=8)
        ninf = 0xFF80 if rows.dtype == np.uint16 else np.float32(-np.inf)
        warped = np.where(wr["keep_mask"].astype(bool), rows, ninf)
        ref = oracle.sample_rows(warped, parity.f32(tau), un, threads=8)
        gw = binding.tli_warp_rows(rows_t, tau, top_k, top_p, rewrite=False)
        g = parity.to_host(binding.tli_sample_rows(rows_t, tau, u, thr=gw["thr"]))
        ok = wr["margin"] >= parity.NEAR_TIE  # rows whose top-p cut the oracle itself decided inside the window aside
        rep = parity.compare_row_tokens(oracle, warped[ok], tau, un[ok], g["tok"][ok], g["status"][ok],
                                        {k: v[ok] for k, v in ref.items()},
                                        lambda r: oracle.softmax(warped[ok][r], parity.f32(tau))[0])
        assert rep["hard"] == 0, dict(rep)
        near += rep["token_near_ties"] + int((~ok).sum())
        assert np.abs(g["lse"][ok] - ref["lse"][ok]).max() < 5e-7
    # TLI drafts from warped drafter rows
    w = synth.WORKLOADS[3].scaled(B=1, K=1, Vt=V + 1000, Vd=V, S=V // 2, cfg=77)
    d2t = synth.make_d2t(w.Vd, w.Vt, w.S, 77)
    m = binding.tli_build_map(d2t, w.Vt)
    ws = binding.alloc_workspace(R * reps, 1, m, binding.TLI_BF16 if dtype == "bf16" else binding.TLI_F32, DEV)
    for top_k, top_p, tau in [(20, 0.9, 0.9), (0, 0.8, 1.0)]:
        wr = oracle.warp_rows(rows, parity.f32(tau), top_k, float(np.float32(top_p)), d2t=d2t, threads=8)
        warped = np.where(wr["keep_mask"].astype(bool), rows, ninf)
        gw = binding.tli_warp_rows(rows_t, tau, top_k, top_p, m=m, rewrite=False)
        g = parity.to_host(binding.tli_draft_sample_warped(m, rows_t, tau, gw["thr"], u, ws))
        ok = wr["margin"] >= parity.NEAR_TIE
        repd, _ = parity.compare_draft(oracle, warped[ok], tau, d2t, un[ok], {k: v[ok] for k, v in g.items()}, threads=8)
        assert repd["hard"] == 0, dict(repd)
        near += repd["token_near_ties"] + int((~ok).sum())
    print("near-tie draws or cuts:", near)
    m.free()


def test_next_rows_beyond_32_bit_offsets(oracle):
    """The neighbouring entry points on buffers that pass 2^31 elements and 2^32 bytes (rows of the large-vocabulary
    shape, rotated copies of 8 drawn sequences): the oracle runs on the rows and sequences either side of every
    offset where a 30-, 31- or 32-bit element count wraps, the first and the last."""
    base = synth.WORKLOADS[4].scaled(B=8)
    inp = synth.make_inputs(base, DEV)
    K, Vt, Vd, d2t = base.K, base.Vt, base.Vd, inp["d2t"]
    tt, td = parity.f32(base.tau_t), parity.f32(base.tau_d)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(8496)
    # ---- one token per row, argmax, exact-match tail, warpers: 8496 rows of 256000 bf16 (4.35 GB)
    lt = parity.rolled_copies(inp["logits_t"], 118)
    B, m1 = lt.shape[0], K + 1
    R = B * m1
    assert R * Vt > 2 ** 31
    flat = lt.reshape(R, Vt)
    u = synth._uniform24(R, gen, DEV)
    un = u.cpu().numpy().astype(np.float64)
    pick = parity.around_wraps(R, [Vt])
    rows = synth.logits_to_numpy(flat[torch.tensor(pick, device=DEV)])
    seqs = parity.around_wraps(B, [m1 * Vt])
    lt_np = synth.logits_to_numpy(lt[torch.tensor(seqs, device=DEV)])
    for tau in (base.tau_t, 0.0):
        g = parity.to_host(binding.tli_sample_rows(flat, tau, u))
        ref = oracle.sample_rows(rows, parity.f32(tau), un[pick], threads=8)
        gp = {k: v[pick] for k, v in g.items()}
        if tau == 0.0:
            assert np.array_equal(gp["tok"], ref["tok"]) and np.array_equal(gp["status"], ref["status"])
        else:
            rep = parity.compare_row_tokens(oracle, rows, tau, un[pick], gp["tok"], gp["status"], ref,
                                            lambda r: oracle.softmax(rows[r], parity.f32(tau))[0])
            assert rep["hard"] == 0 and rep["token_near_ties"] == 0
            assert np.abs(gp["lse"] - ref["lse"]).max() < 5e-7
        assert np.all(g["status"] == 0) and np.all((0 <= g["tok"]) & (g["tok"] < Vt))
        # drafts: the target's own tokens, one of them changed in most sequences
        draft = g["tok"].reshape(B, m1)[:, :K].copy()
        for b in range(B):
            if b % (K + 2) < K:
                draft[b, b % (K + 2)] = (draft[b, b % (K + 2)] + 1) % Vt
        ge = parity.to_host(binding.tli_exact_match_verify(lt, tau, torch.from_numpy(draft).to(DEV), u.reshape(B, m1)))
        re_ = oracle.exact_match_verify(lt_np, parity.f32(tau), draft[seqs], un.reshape(B, m1)[seqs], threads=8)
        for i, b in enumerate(seqs):
            diff = np.nonzero(ge["tgt_tok"][b] != re_["tgt_tok"][i])[0]
            if diff.size:  # only a draw inside the oracle's near-tie window may differ
                assert tau > 0 and np.all(re_["margin"][i, diff] < parity.NEAR_TIE), (tau, b, diff)
                continue
            assert ge["n_accepted"][b] == re_["n_acc"][i] and np.array_equal(ge["out_tok"][b], re_["out_tok"][i])
        want_n = np.array([b % (K + 2) if b % (K + 2) < K else K for b in range(B)])
        assert np.array_equal(ge["n_accepted"], want_n)
    near = _check_warp(oracle, flat, rows, base.tau_t, 50, 0.9, None, None, pick=pick)
    assert near == 0
    del lt, flat
    torch.cuda.empty_cache()
    # ---- union algorithm, acceptance rates, greedy drafts: B = 2104 (target 9.7 GB, drafter 4.3 GB)
    reps = 263
    lt, ld = parity.rolled_copies(inp["logits_t"], reps), parity.rolled_copies(inp["logits_d"], reps)
    B = 8 * reps
    assert B * K * Vd > 2 ** 31
    u_draft, u_acc = synth._uniform24(B * K, gen, DEV), synth._uniform24(B * K, gen, DEV)
    u_fin = synth._uniform24(B, gen, DEV)
    mp = binding.tli_build_map(d2t, Vt)
    ws = binding.alloc_workspace(B, K, mp, binding.TLI_BF16, DEV)
    seqs = parity.around_wraps(B, [m1 * Vt, K * Vd])
    sel = torch.tensor(seqs, device=DEV)
    prow = (sel[:, None] * K + torch.arange(K, device=DEV)[None, :]).reshape(-1)
    prow_h = prow.cpu().numpy()
    lt_np, ld_np = synth.logits_to_numpy(lt[sel]), synth.logits_to_numpy(ld[sel])
    rows_d = ld_np.reshape(len(seqs) * K, Vd)
    ud = u_draft[prow].cpu().numpy().astype(np.float64)
    g_all = binding.tli_union_draft_sample(mp, ld, base.tau_d, u_draft, ws)
    g = {k: v[prow_h] for k, v in parity.to_host(g_all).items()}
    ref = oracle.union_draft_sample(rows_d, td, d2t, ud, threads=8)
    rep = parity.compare_row_tokens(oracle, rows_d, td, ud, g["tok_d"], g["status"], ref,
                                    lambda r: oracle.softmax(rows_d[r], td)[0])
    assert rep["hard"] == 0 and np.abs(g["lse_q"] - ref["lse_q"]).max() < 5e-7
    gv = binding.tli_union_verify(mp, lt, ld, base.tau_t, base.tau_d, g_all["tok_d"], g_all["lse_q"], u_acc, u_fin, ws)
    torch.cuda.synchronize()
    gvp = {k: v[seqs] for k, v in parity.to_host(gv).items()}
    rv, _ = parity.compare_verify(oracle, lt_np, ld_np, base.tau_t, base.tau_d, d2t, g["tok_d"],
                                  u_acc[prow].cpu().numpy().astype(np.float64).reshape(len(seqs), K),
                                  u_fin[sel].cpu().numpy().astype(np.float64), gvp, threads=8, fn="union_verify")
    print("union verify", seqs, dict(rv))
    assert rv["hard"] == 0 and rv["max_lse_err"] < 5e-7
    ga = parity.to_host(binding.tli_acceptance_rates(mp, lt, ld, base.tau_t, base.tau_d))
    ra = oracle.acceptance_rates(lt_np[:, :K].reshape(-1, Vt), rows_d, tt, td, d2t, threads=8)
    assert np.all(ga["status"] == 0) and np.all(ra["status"] == 0)
    for name in ("alpha_tli", "alpha_union"):
        print(name, "max rel", _rates_close(ga[name].reshape(-1)[prow_h], ra[name]))
    assert np.all(ga["alpha_union"] <= ga["alpha_tli"] * (1 + 1e-9)) and np.all(ga["alpha_tli"] <= 1 + 1e-9)
    gd = parity.to_host(binding.tli_greedy_draft(mp, ld, ws))
    rd = oracle.greedy_draft(rows_d, d2t, threads=8)
    assert np.array_equal(gd["tok_d"][prow_h], rd["tok_d"]) and np.all(gd["status"] == 0)
    mp.free()
    del lt, ld, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("i", range(8))
def test_random_shapes_next_rows(oracle, i):
    """Seeded random vocabulary sizes, overlaps, storage types, temperatures and batch shapes through the parity
    checks above (union algorithm, acceptance rates, exact-match tail, one token per row, warpers), within what those
    checks assume of a shape (unshared drafter ids exist, two positions or more, rows longer than the stretch the warp
    test blanks out)."""
    rng = np.random.default_rng(7000 + i)
    dtype = "bf16" if rng.random() < 0.6 else "f32"
    epv = 8 if dtype == "bf16" else 4
    Vt, Vd = int(rng.integers(40, 12000)) * epv, int(rng.integers(40, 9000)) * epv
    if rng.random() < 0.3:
        Vt, Vd = Vd, Vt
    S = int(rng.integers(1, int(0.8 * min(Vt, Vd)) + 1))
    shape = (int(rng.integers(1, 7)), int(rng.integers(2, 6)), Vt, Vd, S, dtype, float(rng.uniform(0.4, 1.4)),
             float(rng.uniform(0.4, 1.4)))
    V, R = int(rng.integers(300, 60000)), int(rng.integers(1, 12))
    stride = (V + epv - 1) // epv * epv + epv * int(rng.integers(0, 3))
    print(shape, (V, R, stride))
    test_union_draft_and_verify(oracle, shape)
    test_acceptance_rates(oracle, shape)
    test_exact_match_tail_sampled(oracle, shape)
    test_sample_rows_and_argmax(oracle, dtype, V, R, stride)
    test_warp_rows(oracle, dtype, V, R, stride)
