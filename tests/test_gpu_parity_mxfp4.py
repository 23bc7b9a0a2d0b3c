"""GPU parity of the MXFP4-KV GQA path (the FP4 of the paper's evaluation, Sec. 3) against the CPU
oracle, through the C ABI.  Same bars as the bf16 path: O max-abs 2e-3 and relative L2 1e-3 against
the fp64 oracle on the same codes and scales, sharded-vs-unsharded max-abs 1e-5, integers bit-exact."""
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


def run_mx(hx, oracle, w, inp, n_shards, split_tokens=0):
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w, split_tokens)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.to(dev), n_shards, mx=(inp.k_mx, inp.v_mx))
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), n_shards)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref) and np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    ws = harness.workspace_for(prob, n_shards, max(ss.max_lens), dev)
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device=dev)
    lse = torch.full((w.B, w.Q), float("nan"), device=dev)
    o_parts = torch.full((n_shards, w.B, w.Q, w.dv), float("nan"), device=dev)
    lses = torch.full((n_shards, w.B, w.Q), float("nan"), device=dev)
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse, o_partials=o_parts, lses=lses)
    torch.cuda.synchronize()
    qb = synth.bits(inp.q)
    kc, vc, km, vm = (t.cpu().numpy() for t in (inp.k, inp.v, inp.k_mx, inp.v_mx))
    lens = inp.lens.numpy()
    o_ref, lse_ref = oracle.attention(qb, kc, vc, lens, w.scale, kv_heads=w.K, mx=(km, vm))
    has = lens > 0
    check_o(o.cpu().numpy()[has], o_ref[has], f"{w.name} N={n_shards} combined O")
    check_lse(lse.cpu().numpy(), lse_ref, f"{w.name} N={n_shards} combined LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
    for i in range(n_shards):
        lo, hi = off_ref[i], off_ref[i] + len_ref[i]
        op_ref, lp_ref = oracle.attention(qb, kc, vc, lens, w.scale, kv_heads=w.K, mx=(km, vm), t_lo=lo, t_hi=hi)
        nz = len_ref[i] > 0
        gp = o_parts[i].cpu().numpy()
        if nz.any():
            check_o(gp[nz], op_ref[nz], f"{w.name} shard {i} partial O")
        assert np.all(gp[~nz] == 0)
        check_lse(lses[i].cpu().numpy(), lp_ref, f"{w.name} shard {i} partial LSE")
    return o, lse


@pytest.mark.parametrize("B,Q,K,S,N,lens,split", [
    (3, 32, 2, 1000, 3, [1000, 517, 33], 0),       # group of 16, ragged, several blocks + tails
    (2, 16, 1, 4200, 5, [4200, 4100], 256),        # forced small splits -> many records
    (2, 10, 2, 700, 2, [700, 1], 0),               # group of 5 (padded head tile), a 1-token sequence
    (2, 40, 2, 900, 4, [900, 0], 0),               # two head tiles, an empty sequence
    (1, 16, 1, 16, 4, [16], 0),                    # fewer 16-token blocks than shards
    (2, 16, 2, 2049, 1, [2049, 2048], 512),        # one shard, tail of one token
    (1, 16, 1, 131, 1, [131], 0),                  # one wave gets several blocks, others none: clamped prefetch
    (2, 8, 2, 1500, 20, [1500, 640], 0),           # more shards than one launch carries
])
def test_mxfp4_shapes_against_oracle(hx, oracle, B, Q, K, S, N, lens, split):
    w = synth.Workload("mx_case", B=B, Q=Q, K=K, dk=128, dv=128, n_shards=N, scale=1 / math.sqrt(128), seed=300 + S,
                       seq_len=S, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    oN, lN = run_mx(hx, oracle, w, inp, N, split)
    o1, l1 = run_mx(hx, oracle, w, inp, 1, split)
    has = np.array(lens) > 0
    assert (oN - o1).abs().cpu().numpy()[has].max() <= SHARD_VS_UNSHARDED
    assert (lN - l1).abs().cpu().numpy()[has].max() <= 1e-5


def test_mxfp4_extreme_block_scales(hx, oracle):
    """Block scales far from 1 on both sides (2^-20 .. 2^20): the dequantised operands stay exact, so
    the result still meets the bar relative to its own magnitude."""
    w = synth.Workload("mx_scales", B=1, Q=16, K=1, dk=128, dv=128, n_shards=2, scale=2.0 ** -10, seed=41, seq_len=300, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    g = torch.Generator().manual_seed(5)
    inp.k_mx = (inp.k_mx.cpu().to(torch.int32) + torch.randint(-6, 7, inp.k_mx.shape, generator=g)).to(torch.uint8).cuda()
    inp.v_mx = torch.randint(107, 148, inp.v_mx.shape, generator=g, dtype=torch.int32).to(torch.uint8).cuda()
    from paper_2507_07120_amd import harness
    prob = harness.problem_for(w)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.cuda(), 2, mx=(inp.k_mx, inp.v_mx))
    ws = harness.workspace_for(prob, 2, max(ss.max_lens), "cuda")
    o = torch.empty((1, 16, 128), device="cuda")
    lse = torch.empty((1, 16), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), inp.lens.numpy(), w.scale,
                                      kv_heads=1, mx=(inp.k_mx.cpu().numpy(), inp.v_mx.cpu().numpy()))
    got = o.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(got - o_ref) / np.linalg.norm(o_ref)
    assert rel <= 1e-3 and np.abs(got - o_ref).max() <= 2e-3 * max(1.0, np.abs(o_ref).max())
    check_lse(lse.cpu().numpy(), lse_ref, "extreme scales LSE")


def test_mxfp4_rejects_what_it_does_not_implement(hx):
    from paper_2507_07120_amd import harness
    w = synth.Workload("mx_bad", B=1, Q=8, K=1, dk=64, dv=64, n_shards=1, scale=0.125, seed=1, seq_len=64, fp4=True)
    prob = harness.problem_for(w)
    assert hx.helix_attn_workspace_bytes(prob, 1, 64) == 0                 # head width 64 is not built for MXFP4


def test_mxfp4_decode_loop_round_robin(hx, oracle):
    """Sec. 2.3 append on an MXFP4 cache: rows and block scales land in the owner shard, attention over
    the grown shards equals the oracle on the logical sequence."""
    from paper_2507_07120_amd import harness
    dev = "cuda"
    B, Q, K, D, N, cap = 2, 16, 2, 128, 3, 96
    w = synth.Workload("mx_loop", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=63, seq_len=40, fp4=True)
    base = synth.make_inputs(w, dev)
    prefill = [40, 23]
    prob = harness.problem_for(w)
    off = torch.empty((N, B), dtype=torch.int64, device=dev)
    ln = torch.empty((N, B), dtype=torch.int32, device=dev)
    hx.helix_shard_layout(torch.tensor(prefill, dtype=torch.int32, device=dev), N, off, ln)
    off_h, ln_h = off.cpu().numpy(), ln.cpu().numpy()
    store = [[torch.zeros((B, K, cap, D // 2), dtype=torch.uint8, device=dev), torch.zeros((B, K, cap, D // 2), dtype=torch.uint8, device=dev),
              torch.full((B, K, cap, D // 32), 127, dtype=torch.uint8, device=dev), torch.full((B, K, cap, D // 32), 127, dtype=torch.uint8, device=dev)]
             for _ in range(N)]
    for i in range(N):
        for b in range(B):
            lo, n = int(off_h[i, b]), int(ln_h[i, b])
            for dst, src in zip(store[i], (base.k, base.v, base.k_mx, base.v_mx)):
                dst[b, :, :n] = src[b, :, lo:lo + n]
    shards = [hx.KVShard.from_mxfp4(*store[i], ln[i], int(ln_h[i].max())) for i in range(N)]
    ws = harness.workspace_for(prob, N, cap, dev)
    log = [[t[b, :, :prefill[b]].cpu().numpy() for t in (base.k, base.v, base.k_mx, base.v_mx)] for b in range(B)]
    model_len = ln_h.copy()
    o = torch.empty((B, Q, D), device=dev)
    lse = torch.empty((B, Q), device=dev)
    overflow = torch.zeros(1, dtype=torch.int32, device=dev)
    for t in range(16 * N + 7):
        q = synth.normal_bf16(w.seed, 1000 + t, (B, Q, D), dev)
        kc, ks = synth.normal_mxfp4_rows(w.seed, 2000 + t, B * K, D, dev)
        vc, vs = synth.normal_mxfp4_rows(w.seed, 3000 + t, B * K, D, dev)
        new = [kc.view(B, K, D // 2), vc.view(B, K, D // 2), ks.view(B, K, D // 32), vs.view(B, K, D // 32)]
        owner = oracle.round_robin_owner(t, N)
        hx.helix_kv_append_mxfp4(prob, shards, t, new[0], new[1], new[2], new[3], cap, overflow=overflow)
        model_len[owner] += 1
        shards[owner].max_len += 1
        for b in range(B):
            log[b] = [np.concatenate([old, n_[b].cpu().numpy()[:, None, :]], axis=1) for old, n_ in zip(log[b], new)]
        hx.helix_attn_decode(prob, q, shards, o, ws, lse_out=lse)
        torch.cuda.synchronize()
        if t % 5 == 0 or t % 16 in (0, 15) or t == 16 * N + 6:
            assert np.array_equal(ln.cpu().numpy(), model_len)
            for b in range(B):
                pos = int(model_len[owner, b]) - 1
                for dst, n_ in zip(store[owner], new):
                    assert torch.equal(dst[b, :, pos], n_[b])
                kcb, vcb, kmb, vmb = (np.ascontiguousarray(x[None]) for x in log[b])
                ob, lb = oracle.attention(synth.bits(q[b:b + 1]), kcb, vcb, np.array([prefill[b] + t + 1], np.int32), w.scale,
                                          kv_heads=K, mx=(kmb, vmb))
                check_o(o[b:b + 1].cpu().numpy(), ob, f"step {t} seq {b} O")
                check_lse(lse[b:b + 1].cpu().numpy(), lb, f"step {t} seq {b} LSE")
    assert overflow.item() == 0


def test_mxfp4_many_pairs_plan_through_shared_memory(hx, oracle):
    """The MXFP4 streaming kernel with more than 64 (shard, sequence) pairs in a launch (the chunked planning scan),
    lengths from 0 up, NaN-filled workspace."""
    from paper_2507_07120_amd import harness
    B, N, S = 45, 2, 900
    w = synth.Workload("mx_many", B=B, Q=16, K=1, dk=128, dv=128, n_shards=N, scale=1 / math.sqrt(128), seed=31, seq_len=S, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    lens = synth.uniform_lengths(17, 3, B, 0, S)
    lens[:3] = torch.tensor([0, S, 1], dtype=torch.int32)
    inp.lens = lens
    prob = harness.problem_for(w)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.cuda(), N, mx=(inp.k_mx, inp.v_mx))
    ws = harness.workspace_for(prob, N, max(ss.max_lens), "cuda")
    ws.view(torch.float32)[: ws.numel() // 4].fill_(float("nan"))
    o = torch.full((B, 16, 128), float("nan"), device="cuda")
    lse = torch.full((B, 16), float("nan"), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    ln = inp.lens.numpy()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), ln, w.scale,
                                      kv_heads=1, mx=(inp.k_mx.cpu().numpy(), inp.v_mx.cpu().numpy()))
    has = ln > 0
    check_o(o.cpu().numpy()[has], o_ref[has], "MXFP4 90 pairs O")
    check_lse(lse.cpu().numpy(), lse_ref, "MXFP4 90 pairs LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)


def test_mxfp4_ragged_batch(hx, oracle):
    """The MXFP4 streaming kernel on a ragged batch: the workgroups share the tokens that exist evenly."""
    from paper_2507_07120_amd import harness
    lens = [30000, 2000, 0, 700, 12000, 64]
    w = synth.Workload("mx_ragged", B=6, Q=16, K=1, dk=128, dv=128, n_shards=2, scale=1 / math.sqrt(128), seed=29,
                       seq_len=30000, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    prob = harness.problem_for(w)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.cuda(), 2, mx=(inp.k_mx, inp.v_mx))
    ws = harness.workspace_for(prob, 2, max(ss.max_lens), "cuda")
    o = torch.full((6, 16, 128), float("nan"), device="cuda")
    lse = torch.full((6, 16), float("nan"), device="cuda")
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), inp.lens.numpy(), w.scale,
                                      kv_heads=1, mx=(inp.k_mx.cpu().numpy(), inp.v_mx.cpu().numpy()))
    has = np.array(lens) > 0
    check_o(o.cpu().numpy()[has], o_ref[has], "MXFP4 ragged O")
    check_lse(lse.cpu().numpy(), lse_ref, "MXFP4 ragged LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
