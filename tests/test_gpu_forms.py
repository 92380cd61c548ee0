"""The two forms of tli_verify's first steps -- a workgroup per target row plus the accept kernel (split), and a
persistent workgroup per sequence that streams its rows and takes the accept tests as they complete -- must agree:
the same decisions, tokens and flags, normalisers equal to rounding of the last fp64 sum.  The library chooses by
batch size; here both are forced on the same inputs, at sizes where either is taken in production and at small ones."""
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


CASES = [
    # (workload, B, K, Vt, Vd, S, union)
    (3, 40, 5, 2048 * 7 + 264, 2048 * 3 + 8, 4000, False),
    (2, 9, 3, 1024 * 5 + 20, 1024 * 2 + 4, 1500, False),
    (4, 300, 8, 2048 * 2 + 8, 2048 + 16, 1300, False),
    (5, 33, 10, 2048 * 4, 2048 * 2, 2048 * 2, True),
    (3, 7, 64, 2048 + 8, 1024 + 8, 600, False),
]


@pytest.mark.parametrize("wl,B,K,Vt,Vd,S,union", CASES)
def test_split_and_per_sequence_forms_agree(oracle, wl, B, K, Vt, Vd, S, union):
    w = synth.WORKLOADS[wl].scaled(B=B, K=K, Vt=Vt, Vd=Vd, S=S)
    inp = synth.make_inputs(w, DEV, seed=4100 + wl)
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    code = binding.TLI_F32 if w.dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(w.B, w.K, m, code, DEV)
    draft = binding.tli_union_draft_sample if union else binding.tli_draft_sample
    verify = binding.tli_union_verify if union else binding.tli_verify
    d = draft(m, inp["logits_d"], w.tau_d, inp["u_draft"].reshape(-1), ws)
    res = {}
    for path in (1, 2):
        binding.tli_tune_final_path(path)
        for lse_q in (d["lse_q"], None):  # None: the library recomputes the drafter normalisers first
            out = verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d, d["tok_d"], lse_q,
                         inp["u_acc"].reshape(-1), inp["u_fin"], ws)
            torch.cuda.synchronize()
            res[(path, lse_q is None)] = parity.to_host(out)
    ref = res[(1, False)]
    for key, got in res.items():
        for name in ("n_accepted", "out_tok", "accept", "status"):
            assert np.array_equal(ref[name], got[name]), (key, name)
        for name in ("p_tok", "q_tok"):
            np.testing.assert_allclose(got[name], ref[name], rtol=1e-9, atol=0, err_msg=str((key, name)))
        np.testing.assert_allclose(got["lse_p"][:, :K], ref["lse_p"][:, :K], rtol=0, atol=1e-9, err_msg=str(key))
        bonus = ref["n_accepted"] == K
        np.testing.assert_allclose(got["lse_p"][bonus, K], ref["lse_p"][bonus, K], rtol=0, atol=1e-9)
        assert np.isnan(got["lse_p"][~bonus, K]).all()
    m.free()


def test_forms_agree_on_flagged_sequences(oracle):
    """NaN / +inf rows, unusable drafts: the flags and the blanked outputs are the same in both forms."""
    w = synth.WORKLOADS[3].scaled(B=12, K=4, Vt=2048 * 2 + 40, Vd=2048 + 24, S=900)
    inp = synth.make_inputs(w, DEV, seed=4177)
    lt, ld = inp["logits_t"].clone(), inp["logits_d"]
    lt[1, 2, 77] = float("nan")
    lt[2, 0, 5] = float("inf")
    lt[4, 4, 100] = float("nan")  # the bonus row: matters only if every draft is accepted
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    ws = binding.alloc_workspace(w.B, w.K, m, binding.TLI_BF16, DEV)
    d = binding.tli_draft_sample(m, ld, w.tau_d, inp["u_draft"].reshape(-1), ws)
    tok = d["tok_d"].clone()
    tok[5 * w.K + 1] = -1
    tok[6 * w.K + 0] = w.Vd + 3
    unshared = int(np.nonzero(inp["d2t"] < 0)[0][0])
    tok[7 * w.K + 2] = unshared
    res = []
    for path in (1, 2):
        binding.tli_tune_final_path(path)
        out = binding.tli_verify(m, lt, ld, w.tau_t, w.tau_d, tok, d["lse_q"], inp["u_acc"].reshape(-1), inp["u_fin"], ws)
        torch.cuda.synchronize()
        res.append(parity.to_host(out))
    for name in ("n_accepted", "out_tok", "accept", "status"):
        assert np.array_equal(res[0][name], res[1][name]), name
    assert res[0]["status"][1] & binding.FLAG_NONFINITE and res[0]["status"][2] & binding.FLAG_NONFINITE
    assert res[0]["status"][5] & binding.FLAG_BAD_DRAFT and res[0]["status"][6] & binding.FLAG_BAD_DRAFT
    assert res[0]["status"][7] & binding.FLAG_BAD_DRAFT
    # and the oracle sees the same sequences the same way
    rep, _ = parity.compare_verify(oracle, synth.logits_to_numpy(lt), synth.logits_to_numpy(ld), w.tau_t, w.tau_d,
                                   inp["d2t"], tok.cpu().numpy(), inp["u_acc"].cpu().numpy().astype(np.float64),
                                   inp["u_fin"].cpu().numpy().astype(np.float64), res[1])
    assert rep["hard"] == 0
    m.free()


@pytest.mark.parametrize("dtype,Vd", [("bf16", 2048 * 5 + 72), ("f32", 1024 * 32), ("f32", 1024 * 2 + 4)])
def test_draft_forms_agree_on_flagged_and_plain_rows(oracle, dtype, Vd):
    """Few short rows are drawn by one kernel that keeps a row in a workgroup's registers, more rows by a scan kernel
    and a draw kernel: the same tokens, normalisers and flags bit for bit -- NaN, +inf and massless rows included --
    and both as the oracle has them."""
    R = 300  # one call: the two-kernel form; three calls of 100 rows: the single-kernel form
    w = synth.WORKLOADS[3].scaled(B=R, K=1, Vt=5000, Vd=Vd, S=min(Vd, 5000) // 2, dtype=dtype, cfg=61)
    inp = synth.make_inputs(w, DEV, seed=4300)
    ld = inp["logits_d"].reshape(R, Vd).clone()
    shared = np.nonzero(inp["d2t"] >= 0)[0]
    unshared = np.nonzero(inp["d2t"] < 0)[0]
    ld[3, int(shared[5])] = float("nan")
    ld[7, int(shared[-1])] = float("inf")
    ld[11, int(unshared[0])] = float("-inf")     # outside the intersection (the oracle wants those finite or -inf)
    ld[13, torch.from_numpy(shared).to(DEV)] = float("-inf")  # no mass on the shared ids
    ld[17, int(shared[0])] = float("-inf")
    ld[250, int(shared[len(shared) // 2])] = float("nan")
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    code = binding.TLI_F32 if dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(R, 1, m, code, DEV)
    u = inp["u_draft"].reshape(-1)
    whole = parity.to_host(binding.tli_draft_sample(m, ld, w.tau_d, u, ws))
    parts = [parity.to_host(binding.tli_draft_sample(m, ld[i:i + 100], w.tau_d, u[i:i + 100].contiguous(), ws))
             for i in range(0, R, 100)]
    torch.cuda.synchronize()
    for k in ("tok_d", "tok_t", "status", "lse_q", "q_tok"):
        joined = np.concatenate([p[k] for p in parts])
        assert np.array_equal(joined, whole[k], equal_nan=k in ("lse_q", "q_tok")), k
    assert whole["status"][3] == oracle.NONFINITE and whole["status"][7] == oracle.NONFINITE
    assert whole["status"][13] == oracle.ZERO_MASS and whole["status"][11] == 0 and whole["status"][17] == 0
    rep, _ = parity.compare_draft(oracle, synth.logits_to_numpy(ld), w.tau_d, inp["d2t"],
                                  u.cpu().numpy().astype(np.float64), whole, threads=8)
    assert rep["hard"] == 0
    m.free()
