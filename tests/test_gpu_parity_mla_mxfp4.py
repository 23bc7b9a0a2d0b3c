"""GPU parity of the MLA path on an MXFP4 latent (Sec. 3: the evaluation keeps KV states in FP4; Sec. 1:
MLA keeps one latent per token for key and value) against the CPU oracle, through the C ABI.  The bars
of the e4m3 latent apply -- the kernel widens both to fp16 entries times a per-token power of two and
hands the matrix cores one fp16 weight per token: O max-abs max(2e-3, 2^-11 max|v|) and relative L2
1e-3 against the fp64 oracle on the same codes and scales, sharded-vs-unsharded max-abs 1e-5."""
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


def mla_mx(B, Q, S, N, seed):
    return synth.Workload("mla_mx_case", B=B, Q=Q, K=1, dk=576, dv=512, n_shards=N, scale=1 / math.sqrt(192), seed=seed,
                          seq_len=S, mla=True, fp4=True)


def value_bar(inp):
    """2^-11 of the largest value magnitude (one fp16 rounding of a weight that the normaliser does not share)."""
    top = float(2.0 ** (inp.k_mx.max().item() - 127) * 6.0)
    return max(2e-3, top * 2.0 ** -11)


def run(hx, oracle, w, inp, n_shards, split_tokens=0, check_partials=True):
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w, split_tokens)
    ss = harness.make_shards(inp.k, None, inp.lens.to(dev), n_shards, mx=(inp.k_mx, None))
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), n_shards)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref) and np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    ws = harness.workspace_for(prob, n_shards, max(ss.max_lens), dev)
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device=dev)
    lse = torch.full((w.B, w.Q), float("nan"), device=dev)
    o_parts = torch.full((n_shards, w.B, w.Q, w.dv), float("nan"), device=dev)
    lses = torch.full((n_shards, w.B, w.Q), float("nan"), device=dev)
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse, o_partials=o_parts, lses=lses)
    torch.cuda.synchronize()
    qb, kc, km = synth.bits(inp.q), inp.k.cpu().numpy(), inp.k_mx.cpu().numpy()
    lens = inp.lens.numpy()
    bar = value_bar(inp)
    o_ref, lse_ref = oracle.attention(qb, kc, None, lens, w.scale, kv_heads=1, dv=w.dv, mx=(km, None))
    has = lens > 0
    check_o(o.cpu().numpy()[has], o_ref[has], f"{w.name} N={n_shards} combined O", bar)
    check_lse(lse.cpu().numpy(), lse_ref, f"{w.name} N={n_shards} combined LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
    if check_partials:
        for i in range(n_shards):
            lo, hi = off_ref[i], off_ref[i] + len_ref[i]
            op_ref, lp_ref = oracle.attention(qb, kc, None, lens, w.scale, kv_heads=1, dv=w.dv, mx=(km, None), t_lo=lo, t_hi=hi)
            nz = len_ref[i] > 0
            gp = o_parts[i].cpu().numpy()
            if nz.any():
                check_o(gp[nz], op_ref[nz], f"{w.name} shard {i} partial O", bar)
            assert np.all(gp[~nz] == 0)
            check_lse(lses[i].cpu().numpy(), lp_ref, f"{w.name} shard {i} partial LSE")
    return o, lse


@pytest.mark.parametrize("B,Q,S,N,lens,split", [
    (2, 128, 700, 2, [700, 333], 0),          # several tiles and a ragged tail
    (1, 128, 2100, 3, [2100], 128),           # forced small splits -> many records
    (2, 64, 98, 1, [97, 1], 0),               # 64 heads (padded head tile), a 1-token sequence
    (3, 128, 300, 4, [300, 0, 35], 64),       # an empty sequence, tails of 3 and 12 rows (partial scale dwords)
    (1, 16, 16, 4, [16], 0),                  # fewer 16-token blocks than shards
    (1, 200, 130, 1, [130], 0),               # two head tiles
])
def test_mla_mxfp4_shapes_against_oracle(hx, oracle, B, Q, S, N, lens, split):
    w = mla_mx(B, Q, S, N, 800 + S)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    oN, lN = run(hx, oracle, w, inp, N, split)
    o1, l1 = run(hx, oracle, w, inp, 1, split, check_partials=False)
    has = np.array(lens) > 0
    assert (oN - o1).abs().cpu().numpy()[has].max() <= SHARD_VS_UNSHARDED
    assert (lN - l1).abs().cpu().numpy()[has].max() <= 1e-5


@pytest.mark.parametrize("first", [[1, 7], [2, 5], [33, 0]])
def test_mla_mxfp4_views_that_start_on_any_row(hx, oracle, first):
    """A token row's 18 scale bytes start on an even address that is a multiple of 4 only for even rows:
    views whose first rows are odd, even, or mixed must give the oracle's result on the same rows."""
    from paper_2507_07120_amd import harness
    w = mla_mx(2, 128, 260, 1, 91)
    inp = synth.make_inputs(w, "cuda")
    lens = [200, 77]
    prob = harness.problem_for(w, 64)
    s = hx.KVShard.from_mxfp4(inp.k, None, inp.k_mx, None, torch.tensor(lens, dtype=torch.int32, device="cuda"), max(lens),
                              tok_off=torch.tensor(first, dtype=torch.int64, device="cuda"))
    ws = harness.workspace_for(prob, 1, max(lens), "cuda")
    o = torch.full((2, 128, 512), float("nan"), device="cuda")
    lse = torch.full((2, 128), float("nan"), device="cuda")
    hx.helix_attn_decode(prob, inp.q, [s], o, ws, lse_out=lse)
    torch.cuda.synchronize()
    lo = np.array(first, dtype=np.int64)
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), None, np.array([260, 260], np.int32), w.scale,
                                      kv_heads=1, dv=512, mx=(inp.k_mx.cpu().numpy(), None), t_lo=lo, t_hi=lo + np.array(lens))
    check_o(o.cpu().numpy(), o_ref, f"views from rows {first}", value_bar(inp))
    check_lse(lse.cpu().numpy(), lse_ref, f"views from rows {first} LSE")


@pytest.mark.parametrize("B,lo,hi,N,split", [
    (4, 40, 900, 8, 0),                        # ragged packed rows, sequences starting on odd and even rows
    (3, 1, 70, 2, 0),
    (2, 1500, 3000, 3, 256),
])
def test_mla_mxfp4_ragged_packed_against_oracle(hx, oracle, B, lo, hi, N, split):
    from test_gpu_decode_kvp import run_both
    w = synth.scaled(synth.WORKLOADS["mla_mxfp4_ragged"], B=B, len_range=(lo, hi), n_shards=N, seed=900 + hi)
    inp = synth.make_inputs(w, "cuda")
    assert inp.k.dim() == 2 and inp.k_mx.shape == (inp.k.shape[0], 18)
    run_both(hx, oracle, w, inp, N, split_tokens=split)


def test_mla_mxfp4_block_scales_spread(hx, oracle):
    """Block scales that differ inside a row (up to 6 octaves) and between rows (14 more): every entry stays
    exact in the widened tile, the per-token powers of two spread the weights over fp16's range; the
    absolute bar scales with the largest value."""
    from paper_2507_07120_amd import harness
    w = synth.Workload("mla_mx_scales", B=1, Q=128, K=1, dk=576, dv=512, n_shards=2, scale=2.0 ** -16, seed=47, seq_len=330,
                       mla=True, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    g = torch.Generator().manual_seed(8)
    row = torch.randint(120, 135, (1, 1, 330, 1), generator=g, dtype=torch.int32)
    blk = torch.randint(0, 7, (1, 1, 330, 18), generator=g, dtype=torch.int32)
    inp.k_mx = (row + blk).to(torch.uint8).cuda()
    prob = harness.problem_for(w)
    ss = harness.make_shards(inp.k, None, inp.lens.cuda(), 2, mx=(inp.k_mx, None))
    ws = harness.workspace_for(prob, 2, max(ss.max_lens), "cuda")
    o = torch.empty((1, 128, 512), device="cuda")
    lse = torch.empty((1, 128), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), None, inp.lens.numpy(), w.scale,
                                      kv_heads=1, dv=512, mx=(inp.k_mx.cpu().numpy(), None))
    got = o.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(got - o_ref) / np.linalg.norm(o_ref)
    assert rel <= 1e-3, rel
    assert np.abs(got - o_ref).max() <= value_bar(inp), "one fp16 rounding of the weights, relative to the largest value"
    check_lse(lse.cpu().numpy(), lse_ref, "spread block scales LSE")


def test_mla_mxfp4_blocks_far_below_the_row_maximum(hx, oracle):
    """Blocks more than 21 octaves below their row's largest scale leave fp16's normal range in the widened
    tile (and vanish beyond 32): the documented error, 2^-24 of the row's largest magnitude per entry, is
    far inside the bars."""
    w = mla_mx(1, 128, 160, 1, 55)
    inp = synth.make_inputs(w, "cuda")
    mxs = inp.k_mx.cpu().clone()
    mxs[0, 0, :, 3] -= 23          # denormal fp16 entries
    mxs[0, 0, :, 9] -= 30
    mxs[0, 0, :, 17] -= 60         # flushed to zero
    mxs[0, 0, ::3, 0] -= 22
    inp.k_mx = mxs.cuda()
    run(hx, oracle, w, inp, 1)


def test_mla_mxfp4_fused_cut(hx, oracle):
    from test_gpu_decode_kvp import run_both
    w = mla_mx(2, 128, 700, 3, 43)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor([700, 333], dtype=torch.int32)
    run_both(hx, oracle, w, inp, 3)


def test_mla_mxfp4_rejects_bad_descriptors(hx):
    from paper_2507_07120_amd import harness
    w = mla_mx(1, 128, 64, 1, 3)
    inp = synth.make_inputs(w, "cuda")
    prob = harness.problem_for(w)
    lens = inp.lens.cuda()
    ws = harness.workspace_for(prob, 1, 64, "cuda")
    o = torch.empty((1, 128, 512), device="cuda")
    good = hx.KVShard.from_mxfp4(inp.k, None, inp.k_mx, None, lens, 64)
    hx.helix_attn_decode(prob, inp.q, [good], o, ws)
    bad = hx.KVShard.from_mxfp4(inp.k, None, inp.k_mx, None, lens, 64)
    bad.v_scale_mx = inp.k_mx                      # a latent has no value scales of its own
    with pytest.raises(hx.HelixError) as e:
        hx.helix_attn_decode(prob, inp.q, [bad], o, ws)
    assert e.value.status == 2
    bad = hx.KVShard.from_mxfp4(inp.k, None, inp.k_mx, None, lens, 64)
    bad.k_scale_mx = None
    with pytest.raises(hx.HelixError) as e:
        hx.helix_attn_decode(prob, inp.q, [bad], o, ws)
    assert e.value.status == 1
    torch.cuda.synchronize()


def test_mla_mxfp4_decode_loop_round_robin(hx, oracle):
    """Sec. 2.3 append on an MXFP4 latent cache: codes and block scales land in the owner shard, attention
    over the grown shards equals the oracle on the logical sequence."""
    from paper_2507_07120_amd import harness
    dev = "cuda"
    B, Q, D, N, cap = 2, 128, 576, 2, 64
    w = mla_mx(B, Q, 40, N, 67)
    base = synth.make_inputs(w, dev)
    prefill = [40, 23]
    prob = harness.problem_for(w)
    off = torch.empty((N, B), dtype=torch.int64, device=dev)
    ln = torch.empty((N, B), dtype=torch.int32, device=dev)
    hx.helix_shard_layout(torch.tensor(prefill, dtype=torch.int32, device=dev), N, off, ln)
    off_h, ln_h = off.cpu().numpy(), ln.cpu().numpy()
    store = [[torch.zeros((B, 1, cap, D // 2), dtype=torch.uint8, device=dev), torch.full((B, 1, cap, D // 32), 127, dtype=torch.uint8, device=dev)]
             for _ in range(N)]
    for i in range(N):
        for b in range(B):
            lo, n = int(off_h[i, b]), int(ln_h[i, b])
            for dst, src in zip(store[i], (base.k, base.k_mx)):
                dst[b, :, :n] = src[b, :, lo:lo + n]
    shards = [hx.KVShard.from_mxfp4(store[i][0], None, store[i][1], None, ln[i], int(ln_h[i].max())) for i in range(N)]
    ws = harness.workspace_for(prob, N, cap, dev)
    log = [[t[b, :, :prefill[b]].cpu().numpy() for t in (base.k, base.k_mx)] for b in range(B)]
    model_len = ln_h.copy()
    o = torch.empty((B, Q, 512), device=dev)
    lse = torch.empty((B, Q), device=dev)
    overflow = torch.zeros(1, dtype=torch.int32, device=dev)
    steps = 16 * N + 5
    for t in range(steps):
        q = synth.normal_bf16(w.seed, 1000 + t, (B, Q, D), dev)
        kc, ks = synth.normal_mxfp4_rows(w.seed, 2000 + t, B, D, dev)
        new = [kc.view(B, 1, D // 2), ks.view(B, 1, D // 32)]
        owner = oracle.round_robin_owner(t, N)
        hx.helix_kv_append_mxfp4(prob, shards, t, new[0], None, new[1], None, cap, overflow=overflow)
        model_len[owner] += 1
        shards[owner].max_len += 1
        for b in range(B):
            log[b] = [np.concatenate([old, n_[b].cpu().numpy()[:, None, :]], axis=1) for old, n_ in zip(log[b], new)]
        hx.helix_attn_decode(prob, q, shards, o, ws, lse_out=lse)
        torch.cuda.synchronize()
        if t % 7 == 0 or t % 16 in (0, 15) or t == steps - 1:
            assert np.array_equal(ln.cpu().numpy(), model_len)
            for b in range(B):
                pos = int(model_len[owner, b]) - 1
                for dst, n_ in zip(store[owner], new):
                    assert torch.equal(dst[b, :, pos], n_[b])
                kcb, kmb = (np.ascontiguousarray(x[None]) for x in log[b])
                ob, lb = oracle.attention(synth.bits(q[b:b + 1]), kcb, None, np.array([prefill[b] + t + 1], np.int32), w.scale,
                                          kv_heads=1, dv=512, mx=(kmb, None))
                check_o(o[b:b + 1].cpu().numpy(), ob, f"step {t} seq {b} O")
                check_lse(lse[b:b + 1].cpu().numpy(), lb, f"step {t} seq {b} LSE")
    assert overflow.item() == 0
