"""The drafting loop at its real shape: tli_draft_sample called once per lookahead position on the B rows
logits_d[:, k, :] (after each drafter forward), filling column k of the [B,K] arrays that tli_verify takes;
and the K + 1 calls of one iteration captured in a HIP graph and replayed."""
import numpy as np
import pytest
import torch

from paper_2502_05202_amd import binding, synth

import parity

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _per_step_draft(m, inp, w, ws, out=None):
    u = inp["u_draft"].reshape(-1)
    for k in range(w.K):
        out = binding.tli_draft_sample(m, inp["logits_d"][:, k, :], w.tau_d, u, ws, out=out, column=(k, w.K))
    return out


@pytest.mark.parametrize("shape", [(1, 5, 9000, 7000, 2500, "f32"), (37, 4, 30000, 2048 * 5 + 64, 4000, "bf16"),
                                   (300, 3, 5000, 4104, 1500, "bf16"),
                                   # per position the single-kernel form (rows held in registers), batched the split one
                                   (100, 3, 5000, 2048 * 9 + 264, 1500, "bf16"), (90, 4, 6000, 1024 * 31 + 4, 2500, "f32")])
def test_per_step_drafts_match_oracle_and_batched_call(oracle, shape):
    B, K, Vt, Vd, S, dtype = shape
    w = synth.WORKLOADS[3].scaled(B=B, K=K, Vt=Vt, Vd=Vd, S=S, dtype=dtype, cfg=60)
    inp = synth.make_inputs(w, DEV)
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    code = binding.TLI_F32 if dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(w.B, w.K, m, code, DEV)
    step = _per_step_draft(m, inp, w, ws)
    torch.cuda.synchronize()
    step_h = parity.to_host(step)
    whole = parity.to_host(binding.tli_draft_sample(m, inp["logits_d"], w.tau_d, inp["u_draft"].reshape(-1), ws))
    for k in ("tok_d", "tok_t", "status"):
        assert np.array_equal(step_h[k], whole[k]), k
    assert np.allclose(step_h["lse_q"], whole["lse_q"], rtol=0, atol=1e-12)
    ld_np = synth.logits_to_numpy(inp["logits_d"]).reshape(B * K, Vd)
    rep, ref = parity.compare_draft(oracle, ld_np, w.tau_d, inp["d2t"],
                                    inp["u_draft"].cpu().numpy().astype(np.float64), step_h, threads=8)
    print(dict(rep))
    assert rep["hard"] == 0 and rep["max_lse_err"] < 5e-7
    # the columns feed tli_verify as they are
    g = binding.tli_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d, step["tok_d"], step["lse_q"],
                           inp["u_acc"].reshape(-1), inp["u_fin"], ws)
    torch.cuda.synchronize()
    rep_v, _ = parity.compare_verify(oracle, synth.logits_to_numpy(inp["logits_t"]),
                                     synth.logits_to_numpy(inp["logits_d"]), w.tau_t, w.tau_d, inp["d2t"],
                                     step_h["tok_d"], inp["u_acc"].cpu().numpy().astype(np.float64),
                                     inp["u_fin"].cpu().numpy().astype(np.float64), parity.to_host(g), threads=8)
    assert rep_v["hard"] == 0
    m.free()


def test_iteration_in_a_hip_graph_replays_exactly():
    """K per-step draft calls + tli_verify captured once; every replay (with new uniforms copied into the
    captured buffers and unrelated eager work in between) must reproduce the eager result bit for bit."""
    w = synth.WORKLOADS[3].scaled(B=24, K=4, Vt=20000, Vd=12000, S=5000, cfg=61)
    inp = synth.make_inputs(w, DEV)
    m = binding.tli_build_map(inp["d2t"], w.Vt)
    ws = binding.alloc_workspace(w.B, w.K, m, binding.TLI_BF16, DEV)
    R = w.B * w.K
    d_out = dict(tok_d=torch.empty(R, dtype=torch.int32, device=DEV), tok_t=torch.empty(R, dtype=torch.int32, device=DEV),
                 q_tok=torch.empty(R, dtype=torch.float64, device=DEV), lse_q=torch.empty(R, dtype=torch.float64, device=DEV),
                 status=torch.empty(R, dtype=torch.int32, device=DEV))
    v_out = binding.alloc_verify_outputs(w.B, w.K, DEV)
    u_draft = inp["u_draft"].reshape(-1).clone()
    u_acc = inp["u_acc"].reshape(-1).clone()
    u_fin = inp["u_fin"].clone()
    static = dict(inp, u_draft=u_draft)

    def iteration():
        _per_step_draft(m, static, w, ws, out=d_out)
        binding.tli_verify(m, inp["logits_t"], inp["logits_d"], w.tau_t, w.tau_d, d_out["tok_d"], d_out["lse_q"],
                           u_acc, u_fin, ws, out=v_out)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        iteration()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        iteration()
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)
    for rep in range(4):
        u_draft.copy_(synth._uniform24(R, gen, DEV))
        u_acc.copy_(synth._uniform24(R, gen, DEV))
        u_fin.copy_(synth._uniform24(w.B, gen, DEV))
        for t in list(d_out.values()) + list(v_out.values()):
            t.view(torch.uint8).fill_(0xA5)  # stale results must not survive a replay
        graph.replay()
        torch.cuda.synchronize()
        got = {**{"d_" + k: t.clone() for k, t in d_out.items()}, **{k: t.clone() for k, t in v_out.items()}}
        _ = (torch.randn(1 << 20, device=DEV) * 2).sum().item()  # unrelated eager work between replays
        iteration()
        torch.cuda.synchronize()
        want = {**{"d_" + k: t for k, t in d_out.items()}, **{k: t for k, t in v_out.items()}}
        for k in want:
            assert torch.equal(got[k].view(torch.uint8), want[k].view(torch.uint8)), (rep, k)
    m.free()


COMPACT = [(5, 3, 2048 * 3 + 40, 2048 * 2 + 24, 1500, "bf16"), (3, 4, 1024 * 4 + 28, 1024 + 4, 700, "f32"),
           (300, 2, 5000, 4104, 1501, "bf16"), (2, 2, 2048 * 30 + 16, 2048 * 27 + 8, 50000, "bf16"),
           (2, 2, 70000, 60000, 50000, "f32")]  # the last two: 2 and 3 parts in the residual scan


@pytest.mark.parametrize("shape", COMPACT, ids=[f"B{c[0]}_S{c[4]}_{c[5]}" for c in COMPACT])
def test_compact_drafter_layout(oracle, shape):
    """Drafter rows that hold only the shared tokens' logits (rank order): draft and verify must give what the
    full-layout oracle gives on the original rows (q' does not depend on the logits outside the intersection)."""
    B, K, Vt, Vd, S, dtype = shape
    w = synth.WORKLOADS[3].scaled(B=B, K=K, Vt=Vt, Vd=Vd, S=S, dtype=dtype, cfg=62)
    inp = synth.make_inputs(w, DEV)
    d2t = inp["d2t"]
    m = binding.tli_build_map(d2t, w.Vt)
    code = binding.TLI_F32 if dtype == "f32" else binding.TLI_BF16
    ws = binding.alloc_workspace(w.B, w.K, m, code, DEV)
    sh_x = torch.from_numpy(np.nonzero(d2t >= 0)[0]).to(DEV)
    epv = 4 if dtype == "f32" else 8
    stride = (S + epv - 1) // epv * epv + epv  # a wider row than needed; the padding holds large values
    buf = torch.full((B, K, stride), 40.0, dtype=inp["logits_d"].dtype, device=DEV)
    buf[:, :, :S] = inp["logits_d"].index_select(2, sh_x)
    ldc = buf[:, :, :S]
    ld_np, lt_np = synth.logits_to_numpy(inp["logits_d"]), synth.logits_to_numpy(inp["logits_t"])
    ud = inp["u_draft"].cpu().numpy().astype(np.float64)
    g = binding.tli_draft_sample_compact(m, buf.reshape(B * K, stride)[:, :S], w.tau_d, inp["u_draft"].reshape(-1), ws)
    torch.cuda.synchronize()
    gh = parity.to_host(g)
    rep, ref = parity.compare_draft(oracle, ld_np.reshape(B * K, Vd), w.tau_d, d2t, ud, gh, threads=8)
    assert rep["hard"] == 0 and rep["max_lse_err"] < 5e-7
    full = parity.to_host(binding.tli_draft_sample(m, inp["logits_d"], w.tau_d, inp["u_draft"].reshape(-1), ws))
    # the two layouts cut a row into different chunks: only a draw inside the oracle's near-tie window may differ
    differ = gh["tok_d"] != full["tok_d"]
    assert np.all(ref["margin"][differ] < parity.NEAR_TIE), np.nonzero(differ)[0]
    assert np.array_equal(gh["tok_t"][~differ], full["tok_t"][~differ])
    ua = inp["u_acc"].cpu().numpy().astype(np.float64)
    uf = inp["u_fin"].cpu().numpy().astype(np.float64)
    tok = torch.from_numpy(ref["tok_d"]).to(DEV)
    for lse_q in (torch.from_numpy(ref["lse_q"]).to(DEV), None):
        gv = binding.tli_verify_compact(m, inp["logits_t"], ldc, w.tau_t, w.tau_d, tok, lse_q, inp["u_acc"].reshape(-1),
                                        inp["u_fin"], ws)
        torch.cuda.synchronize()
        rv, _ = parity.compare_verify(oracle, lt_np, ld_np, w.tau_t, w.tau_d, d2t, ref["tok_d"], ua, uf, parity.to_host(gv),
                                      threads=8)
        print(dict(rv))
        assert rv["hard"] == 0 and rv["max_lse_err"] < 5e-7 and rv["max_prob_rel"] < 1e-6
    m.free()
