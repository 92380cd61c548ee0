"""GPU-vs-oracle comparison rules for the TLI path (used by the -m gpu tests).

Decisions and token ids must be bit-exact for the same uniforms.  The only tolerated differences are
near-ties, which are counted and returned, never silently forgiven:
  * an accept decision may differ only if the oracle's margin |u - p/q'| is below NEAR_TIE;
  * a sampled id may differ only if the oracle's CDF margin for that sample is below NEAR_TIE and u
    lies within NEAR_TIE of the GPU-chosen id's interval of the oracle's CDF; for an extra token drawn from a
    residual whose total mass R is small (the models nearly agree at the rejected position) the window is
    ABS_TIE / R instead, counted separately (see _small_residual_tie).
A sequence whose accept flags differ (inside the window) is compared no further.
Normalisers and probabilities must agree to REL_TOL relative.
"""
from __future__ import annotations

import numpy as np
import torch

from paper_2502_05202_amd import binding, synth

NEAR_TIE = 1e-6
TIGHT = 1e-8
REL_TOL = 1e-5


class Report(dict):
    def __init__(self):
        super().__init__(accept_near_ties=0, accept_near_ties_tight=0, token_near_ties=0, token_near_ties_tight=0,
                         token_small_residual_ties=0, hard=0, compared_positions=0, compared_tokens=0, max_lse_err=0.0, max_prob_rel=0.0)

    def merge(self, other):
        for k, v in other.items():
            self[k] = max(self[k], v) if k.startswith("max_") else self[k] + v
        return self


def _cdf_distance(weights: np.ndarray, tok: int, u: float) -> float:
    """distance from u to the interval of id `tok` in the oracle's CDF (0 if inside)."""
    C = np.cumsum(weights)
    tot = C[-1]
    lo = (C[tok - 1] if tok > 0 else 0.0) / tot
    hi = C[tok] / tot
    if weights[tok] <= 0:
        return np.inf
    return max(lo - u, u - hi, 0.0)


ABS_TIE = 5e-7


def _small_residual_tie(oracle_mod, lt_row, ld_row, tau_t, tau_d, d2t, margin, dist) -> bool:
    """The margins of an extra token drawn from a residual are relative to the residual's total mass R = 1 - sum min(p, q').
    The normalisers of p and q' are good to 5e-7 (asserted beside every comparison), which moves every CDF edge of
    max(0, p - q') by up to that much PROBABILITY MASS, i.e. by 5e-7 / R of the residual: when the two models nearly
    agree at the rejected position (R small) a draw may differ although its relative margin exceeds NEAR_TIE.  Such a
    draw is tolerated -- and counted on its own -- only if margin and distance are below ABS_TIE in units of mass."""
    ar = oracle_mod.acceptance_rates(lt_row[None], ld_row[None], tau_t, tau_d, d2t)
    R = 1.0 - float(ar["alpha_tli"][0])
    return R < 0.5 and margin * R < ABS_TIE and dist * R < ABS_TIE


def f32(x) -> float:
    """The C ABI takes temperatures as fp32: the oracle must be given the same (rounded) number."""
    return float(np.float32(x))


def compare_draft(oracle_mod, ld_np, tau_d, d2t, u_draft, gpu: dict, ref: dict | None = None, threads=16):
    """gpu: dict of host numpy arrays tok_d, tok_t, q_tok, lse_q, status [R]."""
    tau_d = f32(tau_d)
    R = ld_np.shape[0]
    if ref is None:
        ref = oracle_mod.draft_sample(ld_np, tau_d, d2t, u_draft, threads=threads)
    rep = Report()
    rep["compared_tokens"] = R
    assert np.array_equal(gpu["status"], ref["status"]), "draft row status differs"
    ok = ref["status"] == 0
    flagged = ~ok
    assert np.all(gpu["tok_d"][flagged] == -1) and np.all(gpu["tok_t"][flagged] == -1)
    err = np.abs(gpu["lse_q"][ok] - ref["lse_q"][ok])
    if err.size:
        rep["max_lse_err"] = float(err.max())
        assert err.max() < REL_TOL, f"lse_q differs by {err.max()}"
    diff = np.nonzero(ok & (gpu["tok_d"] != ref["tok_d"]))[0]
    for r in diff:
        m = ref["margin"][r]
        _, qp, _, _ = oracle_mod.adjusted_drafter(ld_np[r], tau_d, d2t)
        dist = _cdf_distance(qp, int(gpu["tok_d"][r]), float(u_draft.reshape(-1)[r]))
        if m < NEAR_TIE and dist < NEAR_TIE:
            rep["token_near_ties"] += 1
            rep["token_near_ties_tight"] += int(m < TIGHT)
        else:
            rep["hard"] += 1
            print(f"HARD draft mismatch row {r}: gpu {gpu['tok_d'][r]} oracle {ref['tok_d'][r]} margin {m} dist {dist}")
    same = ok & (gpu["tok_d"] == ref["tok_d"])
    assert np.array_equal(gpu["tok_t"][same], ref["tok_t"][same])
    same &= ref["q_tok"] >= 1e-290  # (below that fp64 no longer holds a probability with all its bits)
    rel = np.abs(gpu["q_tok"][same] - ref["q_tok"][same]) / ref["q_tok"][same]
    if rel.size:
        rep["max_prob_rel"] = float(rel.max())
        assert rel.max() < REL_TOL, f"q_tok relative error {rel.max()}"
    return rep, ref


def compare_verify(oracle_mod, lt_np, ld_np, tau_t, tau_d, d2t, tok_d, u_acc, u_fin, gpu: dict, threads=16,
                   fn="verify"):
    """gpu: dict of host numpy arrays n_accepted, out_tok, accept, p_tok, q_tok, lse_p, status.
    fn: the oracle entry to compare with ("verify" = TLI, "union_verify" = the union algorithm)."""
    tau_t, tau_d = f32(tau_t), f32(tau_d)
    B, K1, Vt = lt_np.shape
    K = K1 - 1
    oracle_verify = getattr(oracle_mod, fn)
    ref = oracle_verify(lt_np, ld_np, tau_t, tau_d, d2t, tok_d, u_acc, u_fin, threads=threads)
    rep = Report()
    u_fin = np.asarray(u_fin, np.float64).reshape(B)
    for b in range(B):
        st_ref, st_gpu = int(ref["status"][b]), int(gpu["status"][b])
        if st_ref & oracle_mod.NONFINITE:
            assert st_gpu & binding.FLAG_NONFINITE, f"seq {b}: oracle NONFINITE, gpu status {st_gpu}"
            assert gpu["n_accepted"][b] == 0 and np.all(gpu["out_tok"][b] == -1)
            continue
        rep["compared_positions"] += K
        # normalisers and per-position probabilities
        e = np.abs(gpu["lse_p"][b, :K] - ref["lse_p"][b, :K]).max()
        rep["max_lse_err"] = max(rep["max_lse_err"], float(e))
        assert e < REL_TOL, f"seq {b}: lse_p differs by {e}"
        for name in ("p_tok", "q_tok"):
            r_, g_ = ref[name][b], gpu[name][b]
            # the relative bound is for probabilities that fp64 holds with all its bits; at 1e-290 and below (a
            # subnormal has as few as one) both sides only have to be that small
            nz = r_ >= 1e-290
            assert np.all(g_[~nz] < 1e-289)
            if nz.any():
                rel = (np.abs(g_[nz] - r_[nz]) / r_[nz]).max()
                rep["max_prob_rel"] = max(rep["max_prob_rel"], float(rel))
                assert rel < REL_TOL, f"seq {b}: {name} relative error {rel}"
        # accept flags: every position is tested on its own
        flips = np.nonzero(gpu["accept"][b] != ref["accept"][b])[0]
        if flips.size:
            for k in flips:
                m = ref["acc_margin"][b, k]
                if m < NEAR_TIE:
                    rep["accept_near_ties"] += 1
                    rep["accept_near_ties_tight"] += int(m < TIGHT)
                else:
                    rep["hard"] += 1
                    print(f"HARD accept mismatch seq {b} pos {k}: margin {m}")
            continue  # downstream outputs legitimately differ after a near-tie flip
        assert (st_gpu & ~binding.FLAG_DEGENERATE) == (st_ref & ~oracle_mod.DEGENERATE), \
            f"seq {b}: status gpu {st_gpu} oracle {st_ref}"
        n = int(ref["n_acc"][b])
        assert gpu["n_accepted"][b] == n, f"seq {b}: n_accepted gpu {gpu['n_accepted'][b]} oracle {n}"
        assert np.array_equal(gpu["out_tok"][b, :n], ref["out_tok"][b, :n])
        assert np.all(gpu["out_tok"][b, n + 1:] == -1)
        rep["compared_tokens"] += 1
        if n == K:
            e = abs(gpu["lse_p"][b, K] - ref["lse_p"][b, K])
            assert e < REL_TOL
        else:
            assert np.isnan(gpu["lse_p"][b, K])
        g_tok, r_tok = int(gpu["out_tok"][b, n]), int(ref["out_tok"][b, n])
        if g_tok != r_tok:
            one = oracle_verify(lt_np[b:b + 1], ld_np[b:b + 1], tau_t, tau_d, d2t, tok_d.reshape(B, K)[b:b + 1],
                                    np.asarray(u_acc).reshape(B, K)[b:b + 1], u_fin[b:b + 1], want_weights=True)
            m = ref["fin_margin"][b]
            dist = _cdf_distance(one["fin_weights"][0], g_tok, float(u_fin[b])) if 0 <= g_tok < Vt else np.inf
            if m < NEAR_TIE and dist < NEAR_TIE:
                rep["token_near_ties"] += 1
                rep["token_near_ties_tight"] += int(m < TIGHT)
            elif n < K and fn == "verify" and _small_residual_tie(oracle_mod, lt_np[b, n], ld_np[b, n], tau_t, tau_d, d2t,
                                                                  m, dist):
                rep["token_small_residual_ties"] += 1
            else:
                rep["hard"] += 1
                print(f"HARD extra-token mismatch seq {b}: gpu {g_tok} oracle {r_tok} margin {m} dist {dist}")
    return rep, ref


def compare_row_tokens(oracle_mod, rows_np, tau, u, gpu_tok, gpu_status, ref: dict, weights_of_row):
    """One sampled id per row: equal to the oracle's, or a counted near-tie (oracle CDF margin below NEAR_TIE and u
    within NEAR_TIE of the GPU id's interval of the oracle's distribution `weights_of_row(r)`)."""
    rep = Report()
    R = rows_np.shape[0]
    rep["compared_tokens"] = R
    assert np.array_equal(gpu_status, ref["status"]), "row status differs"
    ok = ref["status"] == 0
    assert np.all(gpu_tok[~ok] == -1)
    key = "tok_d" if "tok_d" in ref else "tok"
    for r in np.nonzero(ok & (gpu_tok != ref[key]))[0]:
        m = ref["margin"][r]
        dist = _cdf_distance(weights_of_row(r), int(gpu_tok[r]), float(np.asarray(u).reshape(-1)[r]))
        if m < NEAR_TIE and dist < NEAR_TIE:
            rep["token_near_ties"] += 1
            rep["token_near_ties_tight"] += int(m < TIGHT)
        else:
            rep["hard"] += 1
            print(f"HARD row-token mismatch row {r}: gpu {gpu_tok[r]} oracle {ref[key][r]} margin {m} dist {dist}")
    return rep


def to_host(d: dict) -> dict:
    return {k: v.detach().cpu().numpy() for k, v in d.items() if isinstance(v, torch.Tensor)}


def run_case(oracle_mod, inp: dict, threads=16, chain=True):
    """Full draft + verify parity for one drawn batch (tensors already on the GPU).
    Verify is fed the ORACLE's draft tokens (so a draft near-tie cannot confound it); if `chain`, the
    GPU's own draft tokens and lse_q are fed to a second verify and compared with the oracle again."""
    w = inp["workload"]
    dev = inp["logits_t"].device
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    assert m.num_shared == w.S
    code = binding.TLI_F32 if w.dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(w.B, w.K, m, code, dev)
    lt_np = synth.logits_to_numpy(inp["logits_t"])
    ld_np = synth.logits_to_numpy(inp["logits_d"])
    ud = inp["u_draft"].cpu().numpy().astype(np.float64)
    ua = inp["u_acc"].cpu().numpy().astype(np.float64)
    uf = inp["u_fin"].cpu().numpy().astype(np.float64)
    g_draft = binding.tli_draft_sample(m, inp["logits_d"], w.tau_d, inp["u_draft"].reshape(-1), ws)
    torch.cuda.synchronize()
    g_draft_h = to_host(g_draft)
    rep_d, ref_d = compare_draft(oracle_mod, ld_np.reshape(w.B * w.K, w.Vd), w.tau_d, inp["d2t"], ud, g_draft_h,
                                 threads=threads)
    # verify on the oracle's drafts
    tok = torch.from_numpy(ref_d["tok_d"]).to(dev)
    lse_q = torch.from_numpy(ref_d["lse_q"]).to(dev)
    g_ver = binding.tli_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d, tok, lse_q,
                               inp["u_acc"].reshape(-1), inp["u_fin"], ws)
    torch.cuda.synchronize()
    rep_v, ref_v = compare_verify(oracle_mod, lt_np, ld_np, w.tau_t, w.tau_d, inp["d2t"], ref_d["tok_d"], ua, uf,
                                  to_host(g_ver), threads=threads)
    rep_c = None
    if chain:
        g_ver2 = binding.tli_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d, g_draft["tok_d"],
                                    g_draft["lse_q"], inp["u_acc"].reshape(-1), inp["u_fin"], ws)
        torch.cuda.synchronize()
        rep_c, _ = compare_verify(oracle_mod, lt_np, ld_np, w.tau_t, w.tau_d, inp["d2t"], g_draft_h["tok_d"], ua, uf,
                                  to_host(g_ver2), threads=threads)
    m.free()
    return dict(draft=rep_d, verify=rep_v, chained=rep_c, ref_draft=ref_d, ref_verify=ref_v, gpu_verify=to_host(g_ver))


def rolled_copies(x: torch.Tensor, reps: int) -> torch.Tensor:
    """[n, ...] -> [n * reps, ...]: copy i is x rotated by i ids along the last (vocabulary) axis, so that no two
    blocks hold the same rows (for buffers larger than any drawn input)."""
    out = torch.empty((x.shape[0] * reps,) + tuple(x.shape[1:]), dtype=x.dtype, device=x.device)
    n = x.shape[0]
    for i in range(reps):
        out[n * i:n * (i + 1)] = torch.roll(x, i, dims=-1)
    return out


def around_wraps(n_items: int, item_elems: list[int], bits=(30, 31, 32)) -> list[int]:
    """Indices of the items (sequences, rows) either side of every offset where an element count of `bits` bits
    wraps (for 2-byte storage the byte count is one bit on), for each per-item size given; plus the first two and
    the last two."""
    pick = {0, 1, n_items - 2, n_items - 1}
    for b in bits:
        for per in item_elems:
            i = (1 << b) // per
            pick |= {i - 1, i, i + 1}
    return sorted(i for i in pick if 0 <= i < n_items)
