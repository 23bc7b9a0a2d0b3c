"""The shard descriptor carries element strides: the same values behind other memory layouts (token-major
storage with interleaved KV heads, rows padded to a wider pitch, a cache that is a window of a larger
allocation) must give bit-identical results to the dense [B, K, S, d] layout."""
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


def decode(hx, w, q, k, v, lens_dev, n_shards, kv_scale=None):
    from paper_2507_07120_amd import harness
    prob = harness.problem_for(w)
    max_len = int(lens_dev.max().item())
    cache = hx.KVShard.from_padded(k, v, lens_dev, max_len, kv_scale=kv_scale)
    ws = harness.workspace_for(prob, n_shards, max_len, "cuda")
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device="cuda")
    lse = torch.full((w.B, w.Q), float("nan"), device="cuda")
    hx.helix_attn_decode_kvp(prob, q, cache, n_shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("D", [64, 128])
def test_gqa_token_major_and_padded_rows(hx, D):
    w = synth.Workload("strides_gqa", B=2, Q=16, K=4, dk=D, dv=D, n_shards=3, scale=1 / math.sqrt(D), seed=900 + D, seq_len=777)
    inp = synth.make_inputs(w, "cuda")
    lens = torch.tensor([777, 300], dtype=torch.int32, device="cuda")
    o_ref, lse_ref = decode(hx, w, inp.q, inp.k, inp.v, lens, 3)
    # token-major storage [B, S, K, D]: KV heads interleaved inside a token
    k_tm = inp.k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    v_tm = inp.v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert k_tm.stride(2) == w.K * D and k_tm.stride(1) == D
    o, lse = decode(hx, w, inp.q, k_tm, v_tm, lens, 3)
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    # rows padded to a pitch of D + 24 elements (a multiple of 16 bytes), inside a larger allocation
    pitch = D + 24
    kp = torch.full((w.B, w.K, 800, pitch), float("nan"), dtype=torch.bfloat16, device="cuda")
    vp = torch.full((w.B, w.K, 800, pitch), float("nan"), dtype=torch.bfloat16, device="cuda")
    kp[:, :, :777, :D] = inp.k
    vp[:, :, :777, :D] = inp.v
    o, lse = decode(hx, w, inp.q, kp[:, :, :, :D], vp[:, :, :, :D], lens, 3)
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)


@pytest.mark.parametrize("fp8", [False, True])
def test_mla_padded_row_pitch(hx, fp8):
    w = synth.Workload("strides_mla", B=2, Q=128, K=1, dk=576, dv=512, n_shards=2, scale=1 / math.sqrt(192), seed=910,
                       seq_len=500, mla=True, fp8=fp8)
    inp = synth.make_inputs(w, "cuda")
    lens = torch.tensor([500, 129], dtype=torch.int32, device="cuda")
    o_ref, lse_ref = decode(hx, w, inp.q, inp.k, None, lens, 2, kv_scale=inp.kv_scale)
    pitch = 576 + 64                                  # a multiple of 16 bytes for both element sizes
    kp = torch.zeros((w.B, 1, 520, pitch), dtype=inp.k.dtype, device="cuda")
    kp[:, :, :500, :576] = inp.k
    sc = None
    if fp8:
        sc = torch.zeros((w.B, 1, 520), dtype=torch.float32, device="cuda")
        sc[:, :, :500] = inp.kv_scale
    o, lse = decode(hx, w, inp.q, kp[:, :, :, :576], None, lens, 2, kv_scale=sc)
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)


def test_calls_on_a_side_stream(hx):
    """Every entry point enqueues on the stream it is given: work issued on a side stream (default priority)
    while the default stream is busy with something else gives the same bits as on the default stream."""
    w = synth.Workload("side_stream", B=2, Q=16, K=1, dk=128, dv=128, n_shards=2, scale=1 / math.sqrt(128), seed=920, seq_len=2000)
    inp = synth.make_inputs(w, "cuda")
    lens = torch.tensor([2000, 1234], dtype=torch.int32, device="cuda")
    o_ref, lse_ref = decode(hx, w, inp.q, inp.k, inp.v, lens, 2)
    from paper_2507_07120_amd import harness
    prob = harness.problem_for(w)
    cache = hx.KVShard.from_padded(inp.k, inp.v, lens, 2000)
    ws = harness.workspace_for(prob, 2, 2000, "cuda")
    o = torch.full((2, 16, 128), float("nan"), device="cuda")
    lse = torch.full((2, 16), float("nan"), device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    busy = torch.empty(1 << 26, device="cuda")
    for _ in range(4):
        busy.normal_()                                 # keeps the default stream occupied
    with torch.cuda.stream(side):
        hx.helix_attn_decode_kvp(prob, inp.q, cache, 2, o, ws, lse_out=lse, stream=side)
    side.synchronize()
    assert torch.equal(o, o_ref) and torch.equal(lse, lse_ref)
    torch.cuda.synchronize()
