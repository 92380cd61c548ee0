"""Pins for the oracle functions beyond the TLI step (union algorithm, expected acceptance rates, the
exact-match tail, temperature zero): each is checked against something other than itself -- the paper's
tiny-vocabulary examples, its table of expected acceptance rates, its theorems, numpy/scipy routines,
exact enumeration of output distributions measured on the samplers as black boxes.  CPU only."""
import numpy as np
import pytest
import scipy.special as sps

from paper_2502_05202_amd import synth

from test_oracle_pins import d2t_from_strings, ref_qprime, ref_softmax, small_case


def bisect_threshold(pred):
    """sup{u in [0,1) : pred(u)} for a predicate that is true on [0, thr) (1.0 if true everywhere)."""
    if pred(1.0 - 1e-16):
        return 1.0
    if not pred(0.0):
        return 0.0
    lo, hi = 0.0, 1.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        lo, hi = (mid, hi) if pred(mid) else (lo, mid)
    return 0.5 * (lo + hi)


def interval_lengths(sample, edges, n, eps=1e-10):
    """Confirm that the black-box sampler `sample(u) -> id` returns id x exactly on [edges[x], edges[x+1])
    (probing the midpoint and just inside both edges) and return the interval lengths."""
    out = np.zeros(n)
    for x in range(n):
        lo, hi = edges[x], edges[x + 1]
        if hi - lo <= 4 * eps:
            continue
        for u in (0.5 * (lo + hi), lo + eps, hi - eps):
            assert sample(u) == x, (x, u)
        out[x] = hi - lo
    return out


# ---------------------------------------------------------------- union algorithm
def union_output_distribution(oracle, lt, ld, d2t, K):
    """Exact distribution of the token emitted at each position by union draft + union verify (B = 1),
    from interval lengths measured on the oracle's samplers; also the per-position acceptance rates."""
    Vt, Vd = lt.shape[2], ld.shape[2]
    marg = np.zeros((K + 1, Vt))
    alpha = np.zeros(K)
    reach = 1.0
    tok = np.zeros((1, K), np.int32)
    ua = np.zeros((1, K))
    some_ok = [None] * K
    for k in range(K):
        q = ref_softmax(ld[0, k], 1.0)
        p = ref_softmax(lt[0, k], 1.0)
        rows = ld[0, k][None]
        Q = interval_lengths(lambda u: oracle.union_draft_sample(rows, 1.0, d2t, [u])["tok_d"][0],
                             np.concatenate([[0.0], np.cumsum(q) / q.sum()]), Vd)
        A = np.zeros(Vd)
        for d in range(Vd):
            def acc(u, d=d):
                tok[0, :] = d
                ua[:] = 0.0
                ua[0, k] = u
                return oracle.union_verify(lt, ld, 1.0, 1.0, d2t, tok, ua, [0.5])["accept"][0, k]
            A[d] = bisect_threshold(acc)
            if d2t[d] < 0:
                assert A[d] == 0.0  # a draft outside T is rejected for every u
            elif A[d] > 0 and some_ok[k] is None:
                some_ok[k] = d
        alpha[k] = (Q * A).sum()
        # extra-token intervals after a rejection at k (earlier positions accepted with u = 0)
        qt = np.zeros(Vt)
        sh = np.nonzero(d2t >= 0)[0]
        qt[d2t[sh]] = q[sh]
        r = np.maximum(0.0, p - qt)
        d_rej = int(np.argmin(np.where(A < 0.9, A, 2.0)))
        def extra(u):
            for j in range(K):
                tok[0, j] = some_ok[j] if j < k else d_rej
                ua[0, j] = 0.0 if j < k else 0.5 * (A[d_rej] + 1.0)
            v = oracle.union_verify(lt, ld, 1.0, 1.0, d2t, tok, ua, [u])
            assert v["n_acc"][0] == k
            return v["out_tok"][0, k]
        R = interval_lengths(extra, np.concatenate([[0.0], np.cumsum(r) / r.sum()]), Vt)
        emitted = np.zeros(Vt)
        np.add.at(emitted, d2t[sh], (Q * A)[sh])
        marg[k] = reach * (emitted + (1.0 - alpha[k]) * R)
        reach *= alpha[k]
    return marg, alpha


@pytest.mark.parametrize("name", ["disjoint", "drafter_subset", "target_subset"])
def test_union_preserves_the_target_on_the_papers_tiny_vocabularies(oracle, name):
    """Section 'Motivating Examples': T={a},D={b} (every draft rejected); T={a,b},D={b}; T={a},D={a,b}:
    the union algorithm preserves the target distribution in all three."""
    T, D = {"disjoint": (["a"], ["b"]), "drafter_subset": (["a", "b"], ["b"]), "target_subset": (["a"], ["a", "b"])}[name]
    d2t = d2t_from_strings(D, T)
    rng = np.random.default_rng(3)
    lt = rng.standard_normal((1, 2, len(T))).astype(np.float32)
    ld = rng.standard_normal((1, 1, len(D))).astype(np.float32)
    marg, alpha = union_output_distribution(oracle, lt, ld, d2t, 1)
    np.testing.assert_allclose(marg[0], ref_softmax(lt[0, 0], 1.0), atol=1e-12)
    if name == "disjoint":
        assert alpha[0] == 0.0


@pytest.mark.parametrize("seed", [51, 52])
def test_union_lossless_and_acceptance_rate(oracle, seed):
    """Table of expected acceptance rates, union row: sum_{T∩D} min{p, q}; the emitted tokens are
    distributed according to p at every position (K = 2, exact, from measured interval lengths)."""
    inp, lt, ld = small_case(seed, K=2, Vt=23, Vd=17, S=9)
    d2t = inp["d2t"]
    sh = np.nonzero(d2t >= 0)[0]
    marg, alpha = union_output_distribution(oracle, lt, ld, d2t, 2)
    reach = 1.0
    for k in range(2):
        p, q = ref_softmax(lt[0, k], 1.0), ref_softmax(ld[0, k], 1.0)
        assert abs(alpha[k] - np.minimum(p[d2t[sh]], q[sh]).sum()) < 1e-12
        np.testing.assert_allclose(marg[k], reach * p, atol=1e-12)
        reach *= alpha[k]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_acceptance_rates_match_the_table_and_the_theorem(oracle, dtype):
    """alpha_union = sum min{p,q}, alpha_tli = sum min{p, q/sum_{T∩D} q} (table), alpha_union <= alpha_tli
    (theorem), both written here with scipy from the raw logits."""
    w = synth.WORKLOADS[1].scaled(B=3, K=2, Vt=500, Vd=300, S=120, dtype=dtype, tau_t=0.9, tau_d=1.3)
    inp = synth.make_inputs(w)
    lt, ld = synth.logits_to_numpy(inp["logits_t"]), synth.logits_to_numpy(inp["logits_d"])
    ltf, ldf = inp["logits_t"].double().numpy(), inp["logits_d"].double().numpy()
    d2t = inp["d2t"]
    sh = np.nonzero(d2t >= 0)[0]
    got = oracle.acceptance_rates(lt[:, :2].reshape(6, -1), ld.reshape(6, -1), 0.9, 1.3, d2t)
    for r in range(6):
        b, k = divmod(r, 2)
        p, q = ref_softmax(ltf[b, k], 0.9), ref_softmax(ldf[b, k], 1.3)
        qp, _ = ref_qprime(ldf[b, k], 1.3, d2t)
        assert abs(got["alpha_union"][r] - np.minimum(p[d2t[sh]], q[sh]).sum()) < 1e-13
        assert abs(got["alpha_tli"][r] - np.minimum(p[d2t[sh]], qp[sh]).sum()) < 1e-13
        assert got["alpha_union"][r] <= got["alpha_tli"][r] + 1e-15
    # identical vocabularies and models: both rates are one; disjoint mass: TLI flags zero mass
    V = 40
    lg = np.random.default_rng(1).standard_normal((2, V)).astype(np.float32)
    same = oracle.acceptance_rates(lg, lg, 1.0, 1.0, np.arange(V, dtype=np.int32))
    np.testing.assert_allclose(same["alpha_tli"], 1.0, atol=1e-14)
    np.testing.assert_allclose(same["alpha_union"], 1.0, atol=1e-14)
    d2 = np.full(V, -1, np.int32)
    d2[3] = 0
    l2 = lg.copy()
    l2[:, 3] = -np.inf
    z = oracle.acceptance_rates(lg, l2, 1.0, 1.0, d2)
    assert np.all(z["status"] == oracle.ZERO_MASS) and np.all(z["alpha_tli"] == 0) and np.all(z["alpha_union"] == 0)


def test_union_draft_is_searchsorted_and_flags(oracle):
    rng = np.random.default_rng(8)
    Vd = 300
    ld = (rng.standard_normal((5, Vd)) * 2).astype(np.float32)
    d2t = synth.make_d2t(Vd, 400, 100, 5)
    u = rng.random(5)
    got = oracle.union_draft_sample(ld, 0.8, d2t, u)
    for r in range(5):
        q = ref_softmax(ld[r], 0.8)
        C = np.cumsum(q)
        d = int(np.searchsorted(C, u[r] * C[-1], side="right"))
        assert got["tok_d"][r] == d and got["tok_t"][r] == d2t[d]
        assert abs(got["q_tok"][r] - q[d]) < 1e-15 and abs(got["lse_q"][r] - sps.logsumexp(ld[r].astype(np.float64) / 0.8)) < 1e-13
    bad = ld.copy()
    bad[0, int(np.nonzero(d2t < 0)[0][0])] = np.nan   # an unshared logit matters here
    bad[1, :] = -np.inf
    g = oracle.union_draft_sample(bad, 0.8, d2t, u)
    assert g["status"][0] == oracle.NONFINITE and g["status"][1] == oracle.ZERO_MASS and g["tok_d"][0] == -1


def test_union_verify_conventions(oracle):
    inp, lt, ld = small_case(61, K=3)
    d2t = inp["d2t"]
    unshared = int(np.nonzero(d2t < 0)[0][0])
    shared = int(np.nonzero(d2t >= 0)[0][0])
    tok = np.array([[shared, unshared, shared]], np.int32)
    v = oracle.union_verify(lt, ld, 1.0, 1.0, d2t, tok, np.zeros((1, 3)), [0.4], want_weights=True)
    assert v["n_acc"][0] == 1 and v["status"][0] == 0 and list(v["accept"][0]) == [1, 0, 1]
    assert v["p_tok"][0, 1] == 0.0 and v["q_tok"][0, 1] > 0.0
    # the residual after rejecting a token outside T still subtracts q on the shared ids
    p, q = ref_softmax(lt[0, 1], 1.0), ref_softmax(ld[0, 1], 1.0)
    sh = np.nonzero(d2t >= 0)[0]
    qt = np.zeros_like(p)
    qt[d2t[sh]] = q[sh]
    r = np.maximum(0.0, p - qt)
    np.testing.assert_allclose(v["fin_weights"][0], r / r.sum(), rtol=1e-12, atol=1e-18)
    for bad in (-1, 10 ** 6):
        t2 = tok.copy()
        t2[0, 0] = bad
        v = oracle.union_verify(lt, ld, 1.0, 1.0, d2t, t2, np.zeros((1, 3)), [0.4], want_weights=True)
        assert v["status"][0] & oracle.BAD_DRAFT and v["n_acc"][0] == 0
        np.testing.assert_allclose(v["fin_weights"][0], ref_softmax(lt[0, 0], 1.0), rtol=1e-12)
    l2 = ld.copy()
    l2[0, 0, unshared] = np.inf
    v = oracle.union_verify(lt, l2, 1.0, 1.0, d2t, tok, np.zeros((1, 3)), [0.4])
    assert v["status"][0] & oracle.NONFINITE and v["n_acc"][0] == 0 and np.all(v["out_tok"] == -1)


# ---------------------------------------------------------------- one token per row, temperature zero
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sample_rows_is_searchsorted_and_argmax(oracle, dtype):
    w = synth.WORKLOADS[1].scaled(B=4, K=2, Vt=700, Vd=64, S=10, dtype=dtype)
    inp = synth.make_inputs(w)
    rows = synth.logits_to_numpy(inp["logits_t"]).reshape(12, 700)
    rf = inp["logits_t"].double().numpy().reshape(12, 700)
    u = np.random.default_rng(2).random(12)
    got = oracle.sample_rows(rows, 0.7, u)
    for r in range(12):
        p = ref_softmax(rf[r], 0.7)
        C = np.cumsum(p)
        t = int(np.searchsorted(C, u[r] * C[-1], side="right"))
        assert got["tok"][r] == t and abs(got["p_tok"][r] - p[t]) < 1e-15
        assert abs(got["lse"][r] - sps.logsumexp(rf[r] / 0.7)) < 1e-13
    g0 = oracle.sample_rows(rows, 0.0, u)
    assert np.array_equal(g0["tok"], rf.argmax(1)) and np.all(g0["p_tok"] == 1.0)
    # ties: the lowest id; and the argmax is the tau -> 0 limit of the sampler (distinct maxima)
    tie = np.zeros((1, 9), np.float32)
    tie[0, [2, 5]] = 3.0
    assert oracle.sample_rows(tie, 0.0, [0.99])["tok"][0] == 2
    cold = oracle.sample_rows(rows, 1e-3, u)
    gap = np.sort(rf, 1)[:, -1] - np.sort(rf, 1)[:, -2]
    assert np.array_equal(cold["tok"][gap > 0.05], g0["tok"][gap > 0.05])
    bad = rows.copy()
    bad[0, 5] = np.float32(np.nan).view(rows.dtype) if rows.dtype == np.float32 else 0x7FC0
    assert oracle.sample_rows(bad, 0.0, u)["status"][0] == oracle.NONFINITE


def test_greedy_draft_is_masked_argmax_and_cold_limit(oracle):
    w = synth.WORKLOADS[1].scaled(B=5, K=1, Vt=300, Vd=200, S=70)
    inp = synth.make_inputs(w)
    ld = synth.logits_to_numpy(inp["logits_d"]).reshape(5, 200)
    d2t = inp["d2t"]
    g = oracle.greedy_draft(ld, d2t)
    masked = np.where(d2t >= 0, ld.astype(np.float64), -np.inf)
    assert np.array_equal(g["tok_d"], masked.argmax(1)) and np.array_equal(g["tok_t"], d2t[masked.argmax(1)])
    # cold limit of the sampling oracle (tau = 0.02: cold enough to sit on a maximum that leads by 0.5, warm
    # enough that the shared mass does not underflow next to a larger unshared logit)
    cold = oracle.draft_sample(ld, 0.02, d2t, np.full(5, 0.37))
    top2 = np.sort(masked, 1)[:, -2:]
    sep = top2[:, 1] - top2[:, 0] > 0.5
    assert sep.any() and np.array_equal(cold["tok_d"][sep], g["tok_d"][sep])
    l2 = ld.copy()
    l2[0, np.nonzero(d2t >= 0)[0]] = -np.inf
    l2[1, int(np.nonzero(d2t >= 0)[0][0])] = np.inf
    l2[2, int(np.nonzero(d2t < 0)[0][0])] = np.nan  # unshared: ignored
    g2 = oracle.greedy_draft(l2, d2t)
    assert list(g2["status"][:3]) == [oracle.ZERO_MASS, oracle.NONFINITE, 0] and g2["tok_d"][0] == -1


# ---------------------------------------------------------------- exact-match tail
def test_exact_match_acceptance_is_p_of_the_draft(oracle):
    """Table of expected acceptance rates, exact-match row: sum_t p(t) psi(t); for a given draft token t the
    acceptance probability is p(t) (measured as the length of the set of uniforms that match), and with the
    drafter equal to the target the rate is sum p^2 < 1 = the rate of standard SD (theorem on exact matching
    versus speculative decoding)."""
    rng = np.random.default_rng(17)
    V, m = 30, 2
    lt = (rng.standard_normal((1, m + 1, V)) * 1.5).astype(np.float32)
    for j in range(m):
        p = ref_softmax(lt[0, j], 1.0)
        edges = np.concatenate([[0.0], np.cumsum(p) / p.sum()])
        total = 0.0
        for t in range(V):
            draft = np.array([[0] * m], np.int32)
            u = np.zeros((1, m + 1))
            # earlier positions must match: use their own sampled token at u = 0
            first = oracle.exact_match_verify(lt, 1.0, draft, u)["tgt_tok"][0]
            draft[0, :j] = first[:j]
            draft[0, j] = t
            def matched(uu):
                u[0, j] = uu
                return oracle.exact_match_verify(lt, 1.0, draft, u)["n_acc"][0] > j
            # the matching set must be exactly the interval of t in the CDF of p_j: probe both sides of both edges
            for probe, want in ((edges[t] + 1e-10, True), (edges[t + 1] - 1e-10, True), (edges[t] - 1e-10, False),
                                (edges[t + 1] + 1e-10, False)):
                if 0.0 <= probe < 1.0 and edges[t + 1] - edges[t] > 1e-9:
                    assert matched(probe) == want, (j, t, probe)
            total += p[t] * (edges[t + 1] - edges[t])
        assert abs(total - (p ** 2).sum()) < 1e-12 and total < 1.0


def test_exact_match_output_is_the_targets_own_tokens(oracle):
    rng = np.random.default_rng(23)
    B, m, V = 40, 4, 25
    lt = (rng.standard_normal((B, m + 1, V)) * 3).astype(np.float32)
    u = rng.random((B, m + 1))
    own = oracle.sample_rows(lt.reshape(-1, V), 0.8, u.reshape(-1))["tok"].reshape(B, m + 1)
    draft = own[:, :m].copy()
    for b in range(B):  # break the match at a chosen place (or nowhere)
        j = b % (m + 2)
        if j < m:
            draft[b, j] = (draft[b, j] + 1) % V
        elif j == m:
            draft[b, m - 1] = -1   # "no draft token here" ends the match as well
    v = oracle.exact_match_verify(lt, 0.8, draft, u)
    assert np.array_equal(v["tgt_tok"], own)
    for b in range(B):
        n = v["n_acc"][b]
        j = b % (m + 2)
        assert n == (j if j < m else (m - 1 if j == m else m))
        assert np.array_equal(v["out_tok"][b, :n + 1], own[b, :n + 1]) and np.all(v["out_tok"][b, n + 1:] == -1)


def test_temperature_zero_tli_is_exact_match_on_argmax(oracle):
    """TLI as both temperatures go to zero: drafts are the argmax over the shared ids, a draft is accepted
    iff it is the target's argmax, the extra token is the target's argmax of the first rejected row (or of
    the last row).  The cold limit of the sampling oracle (tau = 1e-3, separated maxima) must agree."""
    rng = np.random.default_rng(29)
    B, K, Vt, Vd, S = 30, 3, 60, 50, 35
    d2t = synth.make_d2t(Vd, Vt, S, 77)
    sh = np.nonzero(d2t >= 0)[0]
    ld = (rng.standard_normal((B, K, Vd)) * 4).astype(np.float32)
    lt = (rng.standard_normal((B, K + 1, Vt)) * 4).astype(np.float32)
    for b in range(B):  # make the target agree with the drafter's shared argmax on a prefix of length b % (K+1)
        for k in range(b % (K + 1)):
            d = sh[np.argmax(ld[b, k, sh])]
            lt[b, k, d2t[d]] = lt[b, k].max() + 1.0
    gd = oracle.greedy_draft(ld.reshape(B * K, Vd), d2t)
    v0 = oracle.exact_match_verify(lt, 0.0, gd["tok_t"].reshape(B, K), np.zeros((B, K + 1)))
    u = rng.random((3, B, K)) * 0.98 + 0.01
    tau = 0.02  # cold enough for maxima that lead by 0.5, warm enough that nothing underflows to zero mass
    cold_d = oracle.draft_sample(ld.reshape(B * K, Vd), tau, d2t, u[0].reshape(-1))
    cold_v = oracle.verify(lt, ld, tau, tau, d2t, cold_d["tok_d"], u[1], u[2, :, 0])
    lead_d = np.sort(np.where(d2t >= 0, ld.astype(np.float64), -np.inf), 2)
    lead_t = np.sort(lt.astype(np.float64), 2)
    sep = ((lead_d[:, :, -1] - lead_d[:, :, -2] > 0.5).all(1)) & ((lead_t[:, :, -1] - lead_t[:, :, -2] > 0.5).all(1))
    assert sep.sum() >= 5
    assert np.array_equal(cold_d["tok_d"].reshape(B, K)[sep], gd["tok_d"].reshape(B, K)[sep])
    assert np.array_equal(cold_v["n_acc"][sep], v0["n_acc"][sep]) and np.array_equal(cold_v["out_tok"][sep], v0["out_tok"][sep])
    assert set(v0["n_acc"]) == set(range(K + 1))


# ---------------------------------------------------------------- logit warpers (top-k, top-p)
def ref_warp(x, tau, top_k, top_p, comp):
    """numpy statement of the warpers: grouped by distinct value (np.unique), independent of the oracle's loop."""
    xs = np.where(comp, x, -np.inf)
    vals, counts = np.unique(xs[np.isfinite(xs)], return_counts=True)
    vals, counts = vals[::-1], counts[::-1]  # descending
    n_above = np.concatenate([[0], np.cumsum(counts)[:-1]])
    keep_g = np.ones(len(vals), bool)
    if 0 < top_k < counts.sum():
        keep_g &= n_above < top_k
    if top_p < 1.0:
        w = np.where(keep_g, counts * np.exp((vals - vals[0]) / tau), 0.0)
        frac_above = np.concatenate([[0.0], np.cumsum(w)[:-1]]) / w.sum()
        keep_g &= frac_above < top_p
    thr = vals[keep_g].min() if not keep_g.all() else -np.inf
    return thr, np.isfinite(xs) & (xs >= thr)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_warp_rows_matches_numpy_and_its_defining_properties(oracle, dtype):
    w = synth.WORKLOADS[1].scaled(B=3, K=2, Vt=900, Vd=600, S=250, dtype=dtype)
    inp = synth.make_inputs(w)
    rows = synth.logits_to_numpy(inp["logits_t"]).reshape(9, 900)
    rf = inp["logits_t"].double().numpy().reshape(9, 900)
    rf[0, :50] = -np.inf
    rows[0, :50] = 0xFF80 if dtype == "bf16" else np.float32(-np.inf)
    all_ids = np.ones(900, bool)
    for top_k, top_p, tau in [(0, 1.0, 1.0), (5, 1.0, 1.0), (50, 0.9, 0.7), (0, 0.5, 1.3), (1, 0.3, 1.0), (2000, 0.999, 1.0),
                              (0, 1e-9, 1.0)]:
        got = oracle.warp_rows(rows, tau, top_k, top_p)
        for r in range(9):
            thr, mask = ref_warp(rf[r], tau, top_k, top_p, all_ids)
            assert np.array_equal(got["keep_mask"][r].astype(bool), mask), (top_k, top_p, r)
            assert got["kept"][r] == mask.sum() and (got["thr"][r] == thr)
            x = rf[r]
            kept, fin = mask, np.isfinite(rf[r])
            assert kept.any() and kept[np.argmax(x)]                      # the largest logit always survives
            assert x[kept].min() >= x[fin & ~kept].max() if (fin & ~kept).any() else True
            if 0 < top_k < fin.sum():
                assert (x > x[kept].min()).sum() < max(top_k, 1) or top_p < 1.0
                assert kept.sum() >= min(top_k, fin.sum()) or top_p < 1.0
            if top_p < 1.0:
                # minimality: the survivors reach top_p of the top-k mass, and without their lowest value they do not
                tk = ref_warp(x, tau, top_k, 1.0, all_ids)[1]
                p = np.where(tk, np.exp((x - x[fin].max()) / tau), 0.0)
                p /= p.sum()
                assert p[kept].sum() >= top_p - 1e-12 or kept.sum() == tk.sum()
                lowest = kept & (x == x[kept].min())
                assert p[kept & ~lowest].sum() < top_p
    # restricted to the shared ids of a map (TLI drafter rows): unshared ids never survive
    ld = synth.logits_to_numpy(inp["logits_d"]).reshape(6, 600)
    lf = inp["logits_d"].double().numpy().reshape(6, 600)
    d2t = inp["d2t"]
    got = oracle.warp_rows(ld, 0.8, 20, 0.95, d2t=d2t)
    for r in range(6):
        thr, mask = ref_warp(lf[r], 0.8, 20, 0.95, d2t >= 0)
        assert np.array_equal(got["keep_mask"][r].astype(bool), mask) and not mask[d2t < 0].any()


def test_warp_rows_ties_margin_and_flags(oracle):
    x = np.array([[1.0, 3.0, 2.0, 3.0, 0.5, -1.0, 2.0]], np.float32)
    g = oracle.warp_rows(x, 1.0, 1, 1.0)
    assert list(g["keep_mask"][0]) == [0, 1, 0, 1, 0, 0, 0] and g["kept"][0] == 2 and g["thr"][0] == 3.0  # ties stay together
    g = oracle.warp_rows(x, 1.0, 3, 1.0)
    assert g["kept"][0] == 4 and g["thr"][0] == 2.0
    p = np.exp(x[0].astype(np.float64))
    p /= p.sum()
    top = p[[1, 3]].sum()
    g = oracle.warp_rows(x, 1.0, 0, top + 1e-9)      # just above the mass of the top group: the next group is needed
    assert g["kept"][0] == 4 and abs(g["margin"][0] - 1e-9) < 1e-12
    g = oracle.warp_rows(x, 1.0, 0, top - 1e-9)
    assert g["kept"][0] == 2 and abs(g["margin"][0] - 1e-9) < 1e-12
    bad = x.copy()
    bad[0, 2] = np.nan
    assert oracle.warp_rows(bad, 1.0, 2, 0.9)["status"][0] == oracle.NONFINITE
    none = np.full((1, 5), -np.inf, np.float32)
    g = oracle.warp_rows(none, 1.0, 2, 0.9)
    assert g["status"][0] == oracle.ZERO_MASS and g["kept"][0] == 0
