"""The entry point that cuts the KVP slices (Sec. 2.1.1) inside the attention kernel instead of in a
launch of its own.  The cut it reports must be bit-exact against the oracle's layout, the per-slice
fragments and the combined output must meet the same bars against the fp64 oracle as the two-call
path, and both paths must agree to the sharded-vs-unsharded bound (their split plans may differ)."""
import math

import numpy as np
import pytest
import torch

import synth
from test_gpu_parity_gqa import SHARD_VS_UNSHARDED, check_lse, check_o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    hx_.load_library()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return hx_


def whole_cache(hx, w, inp, lens_dev, seq_base):
    max_len = int(inp.lens.max())
    if getattr(w, "fp4", False):
        return hx.KVShard.from_mxfp4(inp.k, inp.v, inp.k_mx, inp.v_mx, lens_dev, max_len, tok_off=seq_base)
    if inp.k.dim() == 2:
        return hx.KVShard.from_packed(inp.k, lens_dev, max_len, seq_base, kv_scale=inp.kv_scale)
    return hx.KVShard.from_padded(inp.k, inp.v, lens_dev, max_len, kv_scale=inp.kv_scale)


def run_both(hx, oracle, w, inp, N, split_tokens=0):
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w, split_tokens)
    lens_dev = inp.lens.to(dev)
    packed = inp.seq_off is not None
    seq_base = inp.seq_off[:-1].to(dev) if packed else None
    mx = (inp.k_mx, inp.v_mx) if getattr(w, "fp4", False) else None
    max_len = int(inp.lens.max())
    ws = harness.workspace_for(prob, N, max_len, dev)

    def outputs():
        return (torch.full((w.B, w.Q, w.dv), float("nan"), device=dev), torch.full((w.B, w.Q), float("nan"), device=dev),
                torch.full((N, w.B, w.Q, w.dv), float("nan"), device=dev), torch.full((N, w.B, w.Q), float("nan"), device=dev))

    # two calls: layout kernel, then decode over slice descriptors
    ss = harness.make_shards(inp.k, inp.v, lens_dev, N, kv_scale=inp.kv_scale, seq_base=seq_base, mx=mx)
    o2, lse2, p2, l2 = outputs()
    hx.helix_attn_decode(prob, inp.q, ss.shards, o2, ws, lse_out=lse2, o_partials=p2, lses=l2)
    # one call: the cut happens in the kernel
    o1, lse1, p1, l1 = outputs()
    off = torch.full((N, w.B), -7, dtype=torch.int64, device=dev)
    ln = torch.full((N, w.B), -7, dtype=torch.int32, device=dev)
    cache = whole_cache(hx, w, inp, lens_dev, seq_base)
    hx.helix_attn_decode_kvp(prob, inp.q, cache, N, o1, ws, lse_out=lse1, o_partials=p1, lses=l1, shard_off=off, shard_len=ln)
    torch.cuda.synchronize()

    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), N)
    base = inp.seq_off[:-1].numpy()[None, :] if packed else 0
    assert np.array_equal(off.cpu().numpy(), off_ref + base), "slice offsets must be bit-exact"
    assert np.array_equal(ln.cpu().numpy(), len_ref), "slice lengths must be bit-exact"
    assert torch.equal(off, ss.shard_off) and torch.equal(ln, ss.shard_len)

    assert (o1 - o2).abs().max().item() <= SHARD_VS_UNSHARDED
    assert (p1 - p2).abs().max().item() <= SHARD_VS_UNSHARDED
    fin = torch.isfinite(l2)
    assert torch.equal(torch.isfinite(l1), fin)
    assert (l1[fin] - l2[fin]).abs().max().item() <= 1e-5 if fin.any() else True
    assert torch.equal(torch.isfinite(lse1), torch.isfinite(lse2))

    # and against the oracle directly
    qb = synth.bits(inp.q)
    lens = inp.lens.numpy()
    if mx is not None:
        o_ref, lse_ref = oracle.attention(qb, inp.k.cpu().numpy(), None if w.mla else inp.v.cpu().numpy(), lens, w.scale, kv_heads=w.K,
                                          dv=w.dv, mx=(inp.k_mx.cpu().numpy(), None if w.mla else inp.v_mx.cpu().numpy()),
                                          tok_off=inp.seq_off[:-1].numpy() if packed else None)
    else:
        sc = None if inp.kv_scale is None else inp.kv_scale.cpu().numpy()
        o_ref, lse_ref = oracle.attention(qb, synth.bits(inp.k), None if w.mla else synth.bits(inp.v), lens, w.scale,
                                          kv_heads=w.K, dv=w.dv, kv_scale=sc,
                                          tok_off=inp.seq_off[:-1].numpy() if packed else None)
    has = lens > 0
    check_o(o1.cpu().numpy()[has], o_ref[has], f"{w.name} fused cut, combined O")
    check_lse(lse1.cpu().numpy(), lse_ref, f"{w.name} fused cut, combined LSE")
    assert np.all(o1.cpu().numpy()[~has] == 0)
    return o1


@pytest.mark.parametrize("B,Q,K,D,S,N,lens,split", [
    (3, 32, 2, 128, 1000, 3, [1000, 517, 33], 0),        # ragged lengths, uneven last slices
    (2, 16, 1, 128, 4200, 5, [4200, 4100], 256),         # forced small splits
    (4, 8, 8, 64, 300, 8, [300, 0, 17, 128], 128),       # an empty sequence and empty slices, d=64
    (1, 16, 1, 128, 16, 4, [16], 0),                     # fewer 16-token blocks than slices
    (2, 8, 2, 128, 1500, 20, [1500, 640], 0),            # more slices than one launch carries
])
def test_gqa_bf16_fused_cut(hx, oracle, B, Q, K, D, S, N, lens, split):
    w = synth.Workload("kvp_gqa", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=177 + S, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    run_both(hx, oracle, w, inp, N, split_tokens=split)


def test_equal_lengths_give_identical_bits(hx, oracle):
    """With every slice equally long both paths plan the same splits, so the outputs are the same bits."""
    w = synth.Workload("kvp_eq", B=2, Q=16, K=1, dk=128, dv=128, n_shards=4, scale=1 / math.sqrt(128), seed=9, seq_len=4096)
    inp = synth.make_inputs(w, "cuda")
    from paper_2507_07120_amd import harness
    prob = harness.problem_for(w)
    lens_dev = inp.lens.to("cuda")
    ws = harness.workspace_for(prob, 4, 4096, "cuda")
    ss = harness.make_shards(inp.k, inp.v, lens_dev, 4)
    o2 = torch.empty((2, 16, 128), device="cuda")
    o1 = torch.empty_like(o2)
    hx.helix_attn_decode(prob, inp.q, ss.shards, o2, ws)
    hx.helix_attn_decode_kvp(prob, inp.q, hx.KVShard.from_padded(inp.k, inp.v, lens_dev, 4096), 4, o1, ws)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)


@pytest.mark.parametrize("B,lo,hi,N,split", [
    (4, 40, 900, 8, 0),                        # ragged packed e4m3 with per-sequence base rows
    (2, 1500, 3000, 3, 256),
])
def test_mla_fp8_packed_fused_cut(hx, oracle, B, lo, hi, N, split):
    w = synth.scaled(synth.WORKLOADS["mla_fp8_ragged"], B=B, len_range=(lo, hi), n_shards=N, seed=600 + hi)
    inp = synth.make_inputs(w, "cuda")
    run_both(hx, oracle, w, inp, N, split_tokens=split)


def test_mla_bf16_fused_cut(hx, oracle):
    w = synth.Workload("kvp_mla", B=2, Q=128, K=1, dk=576, dv=512, n_shards=3, scale=1 / math.sqrt(192), seed=43,
                       seq_len=700, mla=True)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor([700, 333], dtype=torch.int32)
    run_both(hx, oracle, w, inp, 3)


def test_mxfp4_fused_cut(hx, oracle):
    w = synth.Workload("kvp_mx", B=3, Q=32, K=2, dk=128, dv=128, n_shards=3, scale=1 / math.sqrt(128), seed=311,
                       seq_len=1000, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor([1000, 517, 33], dtype=torch.int32)
    run_both(hx, oracle, w, inp, 3)


def test_fused_cut_of_a_ragged_batch(hx, oracle):
    """helix_attn_decode_kvp on a ragged batch (the host knows only the longest sequence): the cut and the results
    are those of the oracle."""
    from paper_2507_07120_amd import harness
    lens = [50000, 1000, 0, 333, 20000, 4096, 77, 15000]
    w = synth.Workload("kvp_ragged", B=8, Q=16, K=1, dk=128, dv=128, n_shards=4, scale=1 / math.sqrt(128), seed=71, seq_len=50000)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    prob = harness.problem_for(w)
    lens_dev = inp.lens.cuda()
    cache = hx.KVShard.from_padded(inp.k, inp.v, lens_dev, 50000)
    ws = harness.workspace_for(prob, 4, 50000, "cuda")
    o = torch.full((8, 16, 128), float("nan"), device="cuda")
    lse = torch.full((8, 16), float("nan"), device="cuda")
    off = torch.full((4, 8), -7, dtype=torch.int64, device="cuda")
    ln = torch.full((4, 8), -7, dtype=torch.int32, device="cuda")
    hx.helix_attn_decode_kvp(prob, inp.q, cache, 4, o, ws, lse_out=lse, shard_off=off, shard_len=ln)
    torch.cuda.synchronize()
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), 4)
    assert np.array_equal(off.cpu().numpy(), off_ref) and np.array_equal(ln.cpu().numpy(), len_ref)
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), synth.bits(inp.k), synth.bits(inp.v), inp.lens.numpy(), w.scale, kv_heads=1, dv=128)
    has = np.array(lens) > 0
    check_o(o.cpu().numpy()[has], o_ref[has], "fused cut, declared ragged O")
    check_lse(lse.cpu().numpy(), lse_ref, "fused cut, declared ragged LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
