"""GPU parity of the GQA path, the shard combine and the integer metadata against the CPU oracle.
Every call goes through the C ABI (ctypes binding); tolerances are the benchmark's:
O max-abs 2e-3 and relative L2 1e-3 against the fp64 oracle, sharded-vs-unsharded max-abs 1e-5,
integers bit-exact.  LSE: max-abs 1e-4 (|lse| < 64 in fp32 leaves 4e-6 per rounding)."""
import math

import numpy as np
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu

O_MAX_ABS, O_REL_L2, LSE_MAX_ABS, SHARD_VS_UNSHARDED = 2e-3, 1e-3, 1e-4, 1e-5


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    hx_.load_library()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return hx_


def check_o(got, ref, what, max_abs=O_MAX_ABS):
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - ref).max()
    rel = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
    assert err <= max_abs and rel <= O_REL_L2, f"{what}: max-abs {err:.3e} rel-L2 {rel:.3e}"
    return err, rel


def check_lse(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    both_inf = np.isneginf(got) & np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), np.isneginf(ref)), f"{what}: -inf pattern differs"
    err = np.abs(np.where(both_inf, 0.0, got - ref)).max()
    assert err <= LSE_MAX_ABS, f"{what}: lse max-abs {err:.3e}"


def run_sharded(hx, oracle, w, inp, n_shards, split_tokens=0, check_partials=True):
    """decode over n_shards on the GPU, compared with the oracle; returns the GPU output."""
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w, split_tokens)
    lens_dev = inp.lens.to(dev)
    ss = harness.make_shards(inp.k, inp.v, lens_dev, n_shards, kv_scale=inp.kv_scale)
    # integer metadata: bit-exact against the oracle's layout
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), n_shards)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref)
    assert np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    ws = harness.workspace_for(prob, n_shards, max(ss.max_lens), dev)
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device=dev)
    lse = torch.full((w.B, w.Q), float("nan"), device=dev)
    o_parts = torch.full((n_shards, w.B, w.Q, w.dv), float("nan"), device=dev)
    lses = torch.full((n_shards, w.B, w.Q), float("nan"), device=dev)
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse, o_partials=o_parts, lses=lses)
    torch.cuda.synchronize()

    qb, kb, vb = synth.bits(inp.q), synth.bits(inp.k), synth.bits(inp.v)
    lens = inp.lens.numpy()
    o_ref, lse_ref = oracle.attention(qb, kb, vb, lens, w.scale, kv_heads=w.K, dv=w.dv)
    has = lens > 0
    check_o(o.cpu().numpy()[has], o_ref[has], f"{w.name} N={n_shards} combined O")
    check_lse(lse.cpu().numpy(), lse_ref, f"{w.name} N={n_shards} combined LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
    if check_partials:
        for i in range(n_shards):
            lo, hi = off_ref[i], off_ref[i] + len_ref[i]
            op_ref, lp_ref = oracle.attention(qb, kb, vb, lens, w.scale, kv_heads=w.K, dv=w.dv, t_lo=lo, t_hi=hi)
            nz = len_ref[i] > 0
            gp = o_parts[i].cpu().numpy()
            if nz.any():
                check_o(gp[nz], op_ref[nz], f"{w.name} shard {i} partial O")
            assert np.all(gp[~nz] == 0), "empty shard must emit a zero partial"
            check_lse(lses[i].cpu().numpy(), lp_ref, f"{w.name} shard {i} partial LSE")
    # the public combine on the stored fragments: same O, and the argmax bookkeeping bit-exact
    o2 = torch.empty_like(o)
    lse2 = torch.empty_like(lse)
    amax = torch.empty((w.B, w.Q), dtype=torch.int32, device=dev)
    hx.helix_attn_combine(prob, o_parts, lses, o2, lse_out=lse2, argmax_shard=amax)
    torch.cuda.synchronize()
    assert torch.equal(o2, o) and torch.equal(lse2, lse)
    assert np.array_equal(amax.cpu().numpy(), oracle.argmax_f32(lses.cpu().numpy()))
    return o, lse


@pytest.mark.parametrize("B,Q,K,D,S,N,lens", [
    (8, 16, 1, 128, 40000, 1, [40000, 3000, 17, 0, 9000, 128, 20000, 511], ),     # runs sized for 72k tokens, not 320k
    (8, 16, 1, 128, 40000, 3, [40000, 3000, 17, 0, 9000, 128, 20000, 511], ),
    (5, 40, 2, 64, 9000, 2, [9000, 100, 4000, 1, 2500]),                           # two head tiles, d=64
    (3, 16, 2, 128, 20000, 20, [20000, 700, 5000]),                                # more shards than one launch carries
])
def test_gqa_ragged_batch(hx, oracle, B, Q, K, D, S, N, lens):
    """A ragged batch: the workgroups cut the tokens that exist evenly among themselves from the device-side lengths
    (the host only knows the longest); the result does not depend on the upper bound the launch was sized from."""
    w = synth.Workload("ragged", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=55 + N, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    o_t, lse_t = run_sharded(hx, oracle, w, inp, N)
    o_p, lse_p = run_sharded(hx, oracle, w, inp, N, check_partials=False)
    assert torch.equal(o_t, o_p) and torch.equal(lse_t, lse_p)


@pytest.mark.parametrize("B,Q,K,D,N,S,split", [
    (40, 8, 2, 64, 3, 700, 0),          # 120 pairs: every thread of the planning scan has at most one
    (5, 16, 1, 128, 16, 3000, 0),       # 80 pairs in one launch of 16 shards
    (300, 4, 1, 64, 4, 500, 128),       # 1200 pairs: several per thread; short forced runs
    (70, 40, 2, 128, 1, 260, 0),        # 70 pairs, two head tiles per KV head
])
def test_gqa_many_pairs_plan_through_shared_memory(hx, oracle, B, Q, K, D, N, S, split):
    """More than 64 (shard, sequence) pairs in a launch: the workgroups scan the lengths in chunks through shared
    memory instead of one pair per lane.  Lengths from 0 to S incl. 1-token sequences; the workspace is filled with
    NaN, so a record that nobody wrote, or a row served twice or not at all, shows in the result."""
    from paper_2507_07120_amd import harness
    w = synth.Workload("gqa_many", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=900 + B, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    lens = synth.uniform_lengths(13, 5, B, 0, S)
    lens[:4] = torch.tensor([0, S, 1, 129], dtype=torch.int32)
    inp.lens = lens
    prob = harness.problem_for(w, split)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.cuda(), N)
    ws = harness.workspace_for(prob, N, max(ss.max_lens), "cuda")
    ws.view(torch.float32)[: ws.numel() // 4].fill_(float("nan"))
    o = torch.full((B, Q, D), float("nan"), device="cuda")
    lse = torch.full((B, Q), float("nan"), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    ln = inp.lens.numpy()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), synth.bits(inp.k), synth.bits(inp.v), ln, w.scale, kv_heads=K, dv=D)
    has = ln > 0
    check_o(o.cpu().numpy()[has], o_ref[has], f"{B * N} pairs O")
    check_lse(lse.cpu().numpy(), lse_ref, f"{B * N} pairs LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
    # the fused cut on the unsharded cache (sized from another bound, so cut at other tokens): fp32 summation order apart
    cache = hx.KVShard.from_padded(inp.k, inp.v, inp.lens.cuda(), S)
    ws2 = harness.workspace_for(prob, N, S, "cuda")
    ws2.view(torch.float32)[: ws2.numel() // 4].fill_(float("nan"))
    o2 = torch.full_like(o, float("nan"))
    lse2 = torch.full_like(lse, float("nan"))
    hx.helix_attn_decode_kvp(prob, inp.q, cache, N, o2, ws2, lse_out=lse2)
    torch.cuda.synchronize()
    assert (o2 - o).abs().max().item() <= SHARD_VS_UNSHARDED
    assert (lse2[torch.from_numpy(has).cuda()] - lse[torch.from_numpy(has).cuda()]).abs().max().item() <= 1e-5


@pytest.mark.parametrize("fmt", ["bf16", "e4m3", "mxfp4"])
@pytest.mark.parametrize("B,Q,K,N,S,split", [
    (3, 80, 2, 2, 9000, 0),             # three head tiles (the last with 8 heads), sets of 80 workgroups: ids 8 apart share tokens
    (1, 128, 1, 1, 40000, 0),           # multi-query attention with 128 heads: eight sets of 32
    (2, 34, 1, 3, 700, 0),              # a small launch: sets of fewer than 8 workgroups, head tile after head tile
    (2, 64, 2, 1, 5000, 384),           # forced short runs
])
def test_gqa_head_tiles_side_by_side(hx, oracle, fmt, B, Q, K, N, S, split):
    """More than 16 query heads per KV head: the launch is head_tiles equal sets of workgroups that are cut alike, so
    that the workgroups of different head tiles read the same tokens at the same time (through one XCD's L2 where
    the sets are multiples of 8).  Ragged lengths incl. an empty sequence where the batch allows; the workspace is
    filled with NaN, so a record nobody wrote, or a row served twice or not at all, shows in the result."""
    from paper_2507_07120_amd import harness
    D = 128
    w = synth.Workload("gqa_tiles", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=1300 + Q, seq_len=S,
                       fp8=fmt == "e4m3", fp4=fmt == "mxfp4")
    inp = synth.make_inputs(w, "cuda")
    lens = [S, S // 3 + 1, 0][:B]
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    prob = harness.problem_for(w, split)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.cuda(), N, kv_scale=inp.kv_scale, mx=(inp.k_mx, inp.v_mx) if fmt == "mxfp4" else None)
    ws = harness.workspace_for(prob, N, max(ss.max_lens), "cuda")
    ws.view(torch.float32)[: ws.numel() // 4].fill_(float("nan"))
    o = torch.full((B, Q, D), float("nan"), device="cuda")
    lse = torch.full((B, Q), float("nan"), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    ln = inp.lens.numpy()
    if fmt == "mxfp4":
        o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), ln, w.scale, kv_heads=K,
                                          mx=(inp.k_mx.cpu().numpy(), inp.v_mx.cpu().numpy()))
    elif fmt == "e4m3":
        o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), ln, w.scale, kv_heads=K,
                                          kv_scale=inp.kv_scale.cpu().numpy())
    else:
        o_ref, lse_ref = oracle.attention(synth.bits(inp.q), synth.bits(inp.k), synth.bits(inp.v), ln, w.scale, kv_heads=K, dv=D)
    has = ln > 0
    check_o(o.cpu().numpy()[has], o_ref[has], f"{fmt} g={Q // K} O")
    check_lse(lse.cpu().numpy(), lse_ref, f"{fmt} g={Q // K} LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)


@pytest.mark.parametrize("B,Q,K,D,N,S,split", [
    (600, 8, 2, 64, 3, 400, 0),         # 4800 rows of one or two records, three shards, d=64
    (150, 16, 1, 128, 1, 3000, 128),    # 2400 rows of up to 24 records each: several per sub-lane of the fold
    (300, 8, 1, 128, 20, 2000, 0),      # more shards than one launch carries: fragments per launch, then the combine
])
def test_gqa_many_rows_are_finished_by_thread_groups(hx, oracle, B, Q, K, D, N, S, split):
    """From 2048 (b, h) rows on, the records of a row are folded and the shards combined by one thread group per row
    instead of one workgroup per row (a workgroup per row is bound by the rate at which workgroups start).  Same
    operations on the same values: the usual bars against the oracle for output, fragments and LSEs, and the public
    combine on the stored fragments reproduces the fused output bit for bit (run_sharded checks both)."""
    w = synth.Workload("many_rows", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=700 + B, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    lens = synth.uniform_lengths(17, 3, B, 0, S)
    lens[:4] = torch.tensor([0, S, 1, 129], dtype=torch.int32)
    inp.lens = lens
    run_sharded(hx, oracle, w, inp, N, split_tokens=split)


def test_gqa_partial_of_many_rows(hx, oracle):
    """helix_attn_partial on a batch with 2400 (b, h) rows: the split records are merged by thread groups."""
    from paper_2507_07120_amd import harness
    B, Q, S = 300, 8, 1500
    w = synth.Workload("many_rows_partial", B=B, Q=Q, K=1, dk=128, dv=128, n_shards=1, scale=1 / math.sqrt(128), seed=41, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    lens = synth.uniform_lengths(19, 3, B, 0, S)
    lens[:3] = torch.tensor([0, S, 1], dtype=torch.int32)
    inp.lens = lens
    prob = harness.problem_for(w)
    shard = hx.KVShard.from_padded(inp.k, inp.v, inp.lens.cuda(), S)
    ws = harness.workspace_for(prob, 1, S, "cuda")
    ws.view(torch.float32)[: ws.numel() // 4].fill_(float("nan"))
    o = torch.full((B, Q, 128), float("nan"), device="cuda")
    lse = torch.full((B, Q), float("nan"), device="cuda")
    hx.helix_attn_partial(prob, inp.q, shard, o, lse, ws)
    torch.cuda.synchronize()
    ln = inp.lens.numpy()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), synth.bits(inp.k), synth.bits(inp.v), ln, w.scale, kv_heads=1, dv=128)
    has = ln > 0
    check_o(o.cpu().numpy()[has], o_ref[has], "partial of many rows O")
    check_lse(lse.cpu().numpy(), lse_ref, "partial of many rows LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)


def test_tiny_gqa_config(hx, oracle):
    """B=1, 8 query / 2 KV heads, d=64, S=4096 in 4 equal shards: the full first configuration."""
    w = synth.WORKLOADS["tiny_gqa"]
    inp = synth.make_inputs(w, "cuda")
    o4, lse4 = run_sharded(hx, oracle, w, inp, 4)
    o1, lse1 = run_sharded(hx, oracle, w, inp, 1)
    assert (o4 - o1).abs().max().item() <= SHARD_VS_UNSHARDED
    assert (lse4 - lse1).abs().max().item() <= 1e-5


@pytest.mark.parametrize("B,Q,K,D,S,N,lens,split", [
    (3, 32, 2, 128, 1000, 3, [1000, 517, 33], 0),        # group of 16, ragged, several blocks + tail
    (2, 16, 1, 128, 4200, 5, [4200, 4100], 256),         # forced small splits -> many records
    (2, 10, 2, 128, 700, 2, [700, 1], 0),                # group of 5 (padded tile), a 1-token sequence
    (1, 40, 2, 64, 900, 4, [900], 0),                    # group of 20 -> two head tiles, d=64
    (4, 8, 8, 64, 300, 8, [300, 0, 17, 128], 128),       # MHA (group 1), an empty sequence, empty shards
    (1, 16, 1, 128, 16, 4, [16], 0),                     # fewer 16-token blocks than shards
    (2, 16, 2, 128, 2049, 1, [2049, 2048], 512),         # one shard, tail of one token
    (2, 8, 2, 128, 1500, 20, [1500, 640], 0),            # more shards than one launch carries
])
def test_gqa_shapes_against_oracle(hx, oracle, B, Q, K, D, S, N, lens, split):
    w = synth.Workload("case", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=77 + S, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    o_n, lse_n = run_sharded(hx, oracle, w, inp, N, split_tokens=split)
    o_1, lse_1 = run_sharded(hx, oracle, w, inp, 1, split_tokens=split, check_partials=False)
    assert (o_n - o_1).abs().max().item() <= SHARD_VS_UNSHARDED


def test_maximum_shard_count(hx, oracle):
    """HELIX_MAX_SHARDS = 1024 slices of one cache (64 launches of 16 descriptors each, then the
    stand-alone combine over 1024 fragments): layout bit-exact, combined result and argmax against the oracle."""
    w = synth.Workload("max_shards", B=2, Q=16, K=1, dk=128, dv=128, n_shards=1024, scale=1 / math.sqrt(128), seed=88, seq_len=20000)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor([20000, 9000], dtype=torch.int32)
    o_n, lse_n = run_sharded(hx, oracle, w, inp, 1024, check_partials=False)
    o_1, lse_1 = run_sharded(hx, oracle, w, inp, 1, check_partials=False)
    assert (o_n - o_1).abs().max().item() <= SHARD_VS_UNSHARDED
    from paper_2507_07120_amd import harness
    with pytest.raises(hx.HelixError):                      # one more than the limit is refused before any launch
        hx.helix_shard_layout(inp.lens.cuda(), 1025, torch.empty((1025, 2), dtype=torch.int64, device="cuda"),
                              torch.empty((1025, 2), dtype=torch.int32, device="cuda"))


def test_peaked_softmax_sharded_vs_unsharded(hx, oracle):
    """The sharp-peak recipe of the 16-shard configuration (1% of keys x8) at a reduced length."""
    w = synth.scaled(synth.WORKLOADS["gqa_full"], B=2, seq_len=16384)
    inp = synth.make_inputs(w, "cuda")
    o16, _ = run_sharded(hx, oracle, w, inp, 16, check_partials=False)
    o1, _ = run_sharded(hx, oracle, w, inp, 1, check_partials=False)
    assert (o16 - o1).abs().max().item() <= SHARD_VS_UNSHARDED


def test_partial_entry_point_matches_decode_fragment(hx, oracle):
    from paper_2507_07120_amd import harness
    w = synth.Workload("case", B=2, Q=16, K=2, dk=128, dv=128, n_shards=3, scale=0.09, seed=5, seq_len=777)
    inp = synth.make_inputs(w, "cuda")
    prob = harness.problem_for(w)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.cuda(), 3)
    ws = harness.workspace_for(prob, 3, max(ss.max_lens), "cuda")
    o = torch.empty((2, 16, 128), device="cuda")
    o_parts = torch.empty((3, 2, 16, 128), device="cuda")
    lses = torch.empty((3, 2, 16), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, o_partials=o_parts, lses=lses)
    for i in range(3):
        op = torch.empty((2, 16, 128), device="cuda")
        lp = torch.empty((2, 16), device="cuda")
        hx.helix_attn_partial(prob, inp.q, ss.shards[i], op, lp, ws)
        torch.cuda.synchronize()
        assert torch.equal(op, o_parts[i]) and torch.equal(lp, lses[i])


def test_combine_against_oracle_and_edge_cases(hx, oracle):
    rng = np.random.default_rng(3)
    N, B, Q, dv = 5, 3, 7, 128
    o_p = rng.standard_normal((N, B, Q, dv)).astype(np.float32)
    lse_p = (rng.standard_normal((N, B, Q)) * 5).astype(np.float32)
    lse_p[1] = -np.inf                      # a whole empty shard
    lse_p[:, 0, 0] = -np.inf                # a row with no tokens anywhere
    lse_p[2, 1, 1] = lse_p[4, 1, 1] = 9.0   # a tie for the argmax: lowest index wins
    o_p[1] = np.nan                         # an empty shard's partial must not be read into the sum
    prob = hx.Problem(B, Q, 1, dv, dv, 1.0)
    o = torch.empty((B, Q, dv), device="cuda")
    lse = torch.empty((B, Q), device="cuda")
    am = torch.empty((B, Q), dtype=torch.int32, device="cuda")
    hx.helix_attn_combine(prob, torch.tensor(o_p).cuda(), torch.tensor(lse_p).cuda(), o, lse_out=lse, argmax_shard=am)
    torch.cuda.synchronize()
    o_clean = np.where(np.isnan(o_p), 0.0, o_p).astype(np.float64)
    o_ref, lse_ref = oracle.combine(o_clean, lse_p.astype(np.float64))
    assert np.abs(o.cpu().numpy() - o_ref).max() <= 1e-5
    check_lse(lse.cpu().numpy(), lse_ref, "combine LSE")
    assert np.array_equal(am.cpu().numpy(), oracle.argmax_f32(lse_p))
    assert am[1, 1].item() == 2 and am[0, 0].item() == 0
    assert torch.all(o[0, 0] == 0) and lse[0, 0].item() == -math.inf


def test_shard_layout_bit_exact(hx, oracle):
    lens = np.concatenate([[0, 1, 15, 16, 17, 4096, 262144, 16384], np.random.default_rng(1).integers(1, 300000, 56)]).astype(np.int32)
    base = np.concatenate([[0], np.cumsum(lens.astype(np.int64))[:-1]])
    for N in [1, 3, 8, 16]:
        off = torch.empty((N, len(lens)), dtype=torch.int64, device="cuda")
        ln = torch.empty((N, len(lens)), dtype=torch.int32, device="cuda")
        hx.helix_shard_layout(torch.tensor(lens).cuda(), N, off, ln, seq_base=torch.tensor(base).cuda())
        off_ref, len_ref = oracle.shard_layout(lens, N)
        assert np.array_equal(off.cpu().numpy(), off_ref + base[None, :])
        assert np.array_equal(ln.cpu().numpy(), len_ref)
