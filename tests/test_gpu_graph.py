"""The library only enqueues kernels on the caller's stream (no allocation, no synchronisation, no memset), so a
decode step can be captured into a HIP graph and replayed: every replay, with eager work and synchronisations
in between and with new inputs written into the same buffers, must give the bits of the eager call."""
import math

import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    hx_.load_library()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return hx_


@pytest.mark.parametrize("kind", ["gqa", "mla", "mla_fp8"])
def test_captured_decode_replays_like_eager(hx, kind):
    from paper_2507_07120_amd import harness
    if kind == "gqa":
        w = synth.Workload("graph_gqa", B=2, Q=16, K=2, dk=128, dv=128, n_shards=3, scale=1 / math.sqrt(128), seed=930, seq_len=1500)
    else:
        w = synth.Workload("graph_mla", B=2, Q=128, K=1, dk=576, dv=512, n_shards=2, scale=1 / math.sqrt(192), seed=931, seq_len=400,
                           mla=True, fp8=(kind == "mla_fp8"))
    inp = synth.make_inputs(w, "cuda")
    lens = torch.tensor([w.seq_len, w.seq_len // 3], dtype=torch.int32, device="cuda")
    prob = harness.problem_for(w)
    cache = hx.KVShard.from_padded(inp.k, inp.v, lens, w.seq_len, kv_scale=inp.kv_scale)
    ws = harness.workspace_for(prob, w.n_shards, w.seq_len, "cuda")
    q = inp.q.clone()
    o = torch.empty((w.B, w.Q, w.dv), device="cuda")
    lse = torch.empty((w.B, w.Q), device="cuda")

    def step():
        hx.helix_attn_decode_kvp(prob, q, cache, w.n_shards, o, ws, lse_out=lse)

    step()                                              # warm-up outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        q.copy_(synth.normal_bf16(w.seed, 5000 + rep, tuple(q.shape), "cuda"))     # new query in the captured buffer
        lens[1] = w.seq_len // 3 + 17 * rep                                         # and a grown sequence
        graph.replay()
        torch.cuda.synchronize()
        o_g, lse_g = o.clone(), lse.clone()
        o.fill_(float("nan"))
        lse.fill_(float("nan"))
        step()                                          # the same step, eagerly
        torch.cuda.synchronize()
        assert torch.equal(o_g, o) and torch.equal(lse_g, lse), f"replay {rep} differs from the eager call"
