"""The benchmark configurations at FULL size, in the launch configurations bench.py times (automatic
work split; the two-call path helix_shard_layout + helix_attn_decode and the default one,
helix_attn_decode_kvp with the sum of the lengths declared): whole sequences (every head) plus single rows
of other sequences against the CPU oracle -- at least 256 rows per benchmark configuration, the whole output
where the oracle's time allows --, integer metadata bit-exact, both paths against each other, and the GPU's
sharded-then-combined output against its own unsharded output (max-abs 1e-5) where the configuration has
several shards."""
import numpy as np
import pytest
import torch

import synth
from test_gpu_parity_gqa import O_MAX_ABS, O_REL_L2, LSE_MAX_ABS, SHARD_VS_UNSHARDED

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    hx_.load_library()
    assert torch.cuda.is_available()
    return hx_


def decode(hx, w, inp, n_shards, want_parts=False):
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w)
    seq_base = inp.seq_off[:-1].to(dev) if inp.seq_off is not None else None
    ss = harness.make_shards(inp.k, inp.v, inp.lens.to(dev), n_shards, kv_scale=inp.kv_scale, seq_base=seq_base,
                             mx=None if inp.k_mx is None else (inp.k_mx, inp.v_mx))
    ws = harness.workspace_for(prob, n_shards, max(ss.max_lens), dev)
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device=dev)
    lse = torch.full((w.B, w.Q), float("nan"), device=dev)
    parts = lses = None
    if want_parts:
        parts = torch.empty((n_shards, w.B, w.Q, w.dv), device=dev)
        lses = torch.empty((n_shards, w.B, w.Q), device=dev)
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse, o_partials=parts, lses=lses)
    torch.cuda.synchronize()
    return o, lse, parts, lses, ss


def decode_as_bench(hx, w, inp, n_shards):
    """The step bench.py times: helix_attn_decode_kvp on the whole cache, the sum of the lengths declared."""
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w)
    lens_dev = inp.lens.to(dev)
    seq_base = inp.seq_off[:-1].to(dev) if inp.seq_off is not None else None
    max_len = int(inp.lens.max())
    if inp.k_mx is not None:
        cache = hx.KVShard.from_mxfp4(inp.k, inp.v, inp.k_mx, inp.v_mx, lens_dev, max_len, tok_off=seq_base)
    elif inp.k.dim() == 2:
        cache = hx.KVShard.from_packed(inp.k, lens_dev, max_len, seq_base, kv_scale=inp.kv_scale)
    else:
        cache = hx.KVShard.from_padded(inp.k, inp.v, lens_dev, max_len, kv_scale=inp.kv_scale)
    ws = harness.workspace_for(prob, n_shards, max_len, dev)
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device=dev)
    lse = torch.full((w.B, w.Q), float("nan"), device=dev)
    off = torch.empty((n_shards, w.B), dtype=torch.int64, device=dev)
    ln = torch.empty((n_shards, w.B), dtype=torch.int32, device=dev)
    hx.helix_attn_decode_kvp(prob, inp.q, cache, n_shards, o, ws, lse_out=lse, shard_off=off, shard_len=ln)
    torch.cuda.synchronize()
    return o, lse, off, ln


def check_as_bench(hx, oracle, w, inp, n_shards, o_two_call, lse_two_call, o_ref, lse_ref, rows, what):
    """The bench's entry point at full size: the cut bit-exact, sampled rows against the oracle, and the whole
    output against the two-call path (split plans may differ: fp32 summation order only)."""
    o, lse, off, ln = decode_as_bench(hx, w, inp, n_shards)
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), n_shards)
    base = inp.seq_off[:-1].numpy()[None, :] if inp.seq_off is not None else 0
    assert np.array_equal(off.cpu().numpy(), off_ref + base) and np.array_equal(ln.cpu().numpy(), len_ref)
    check_rows(o, lse, o_ref, lse_ref, rows, what + " (helix_attn_decode_kvp)")
    assert (o - o_two_call).abs().max().item() <= SHARD_VS_UNSHARDED
    assert (lse - lse_two_call).abs().max().item() <= 1e-5


def oracle_rows(oracle, w, inp, rows):
    """The oracle on the sampled (b,h) rows only; copies just those sequences to the host."""
    out_o, out_l = [], []
    for b, h in rows:
        q = synth.bits(inp.q[b:b + 1])
        if inp.seq_off is not None:                                   # packed ragged latent
            lo, hi = int(inp.seq_off[b]), int(inp.seq_off[b + 1])
            k = synth.bits(inp.k[lo:hi])
            sc = inp.kv_scale[lo:hi].cpu().numpy() if inp.kv_scale is not None else None
            mx = None if inp.k_mx is None else (inp.k_mx[lo:hi].cpu().numpy(), None)
            o, l = oracle.attention(q, k, None, np.array([hi - lo], np.int32), w.scale, kv_heads=1, dv=w.dv,
                                    kv_scale=sc, tok_off=np.zeros(1, np.int64), rows=[(0, h)], mx=mx)
        else:
            g = w.Q // w.K
            kh = h // g
            k = synth.bits(inp.k[b:b + 1, kh:kh + 1])
            v = synth.bits(inp.v[b:b + 1, kh:kh + 1]) if inp.v is not None else None
            # a one-KV-head problem holding exactly this row's group: head index within the group
            qg = np.ascontiguousarray(q[:, kh * g:(kh + 1) * g])
            mx = None if inp.k_mx is None else (inp.k_mx[b:b + 1, kh:kh + 1].cpu().numpy(),
                                                None if inp.v_mx is None else inp.v_mx[b:b + 1, kh:kh + 1].cpu().numpy())
            o, l = oracle.attention(qg, k, v, inp.lens[b:b + 1].numpy(), w.scale, kv_heads=1, dv=w.dv, rows=[(0, h - kh * g)], mx=mx)
        out_o.append(o[0])
        out_l.append(l[0])
    return np.stack(out_o), np.array(out_l)


def oracle_sequences(oracle, w, inp, seqs, extra_rows=()):
    """The oracle on every head of the sequences `seqs` (one oracle call per sequence, only that sequence copied
    to the host) plus the single rows `extra_rows`; returns (rows, o_ref, lse_ref) in check_rows' form."""
    rows, out_o, out_l = [], [], []
    for b in seqs:
        q = synth.bits(inp.q[b:b + 1])
        if inp.seq_off is not None:                                   # packed ragged latent
            lo, hi = int(inp.seq_off[b]), int(inp.seq_off[b + 1])
            sc = inp.kv_scale[lo:hi].cpu().numpy() if inp.kv_scale is not None else None
            mx = None if inp.k_mx is None else (inp.k_mx[lo:hi].cpu().numpy(), None)
            o, l = oracle.attention(q, synth.bits(inp.k[lo:hi]), None, np.array([hi - lo], np.int32), w.scale, kv_heads=1,
                                    dv=w.dv, kv_scale=sc, tok_off=np.zeros(1, np.int64), mx=mx)
        else:
            v = synth.bits(inp.v[b:b + 1]) if inp.v is not None else None
            sc = inp.kv_scale[b:b + 1].cpu().numpy() if inp.kv_scale is not None else None
            mx = None if inp.k_mx is None else (inp.k_mx[b:b + 1].cpu().numpy(),
                                                None if inp.v_mx is None else inp.v_mx[b:b + 1].cpu().numpy())
            o, l = oracle.attention(q, synth.bits(inp.k[b:b + 1]), v, inp.lens[b:b + 1].numpy(), w.scale, kv_heads=w.K,
                                    dv=w.dv, kv_scale=sc, mx=mx)
        rows += [(b, h) for h in range(w.Q)]
        out_o.append(o[0])
        out_l.append(l[0])
    o_ref, lse_ref = np.concatenate(out_o), np.concatenate(out_l)
    if extra_rows:
        eo, el = oracle_rows(oracle, w, inp, list(extra_rows))
        rows += list(extra_rows)
        o_ref, lse_ref = np.concatenate([o_ref, eo]), np.concatenate([lse_ref, el])
    return rows, o_ref, lse_ref


def check_rows(o, lse, o_ref, lse_ref, rows, what):
    oc, lc = o.cpu().numpy(), lse.cpu().numpy()
    got = np.stack([oc[b, h] for b, h in rows]).astype(np.float64)
    gl = np.array([lc[b, h] for b, h in rows], dtype=np.float64)
    err = np.abs(got - o_ref).max()
    rel = np.linalg.norm(got - o_ref) / np.linalg.norm(o_ref)
    lerr = np.abs(gl - lse_ref).max()
    print(f"{what}: O max-abs {err:.3e} rel-L2 {rel:.3e}  LSE max-abs {lerr:.3e}")
    assert err <= O_MAX_ABS and rel <= O_REL_L2 and lerr <= LSE_MAX_ABS, what


def test_gqa_share_full(hx, oracle):
    w = synth.WORKLOADS["gqa_share"]
    inp = synth.make_inputs(w, "cuda")
    o, lse, _, _, _ = decode(hx, w, inp, 1)
    assert torch.isfinite(o).all() and torch.isfinite(lse).all()
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, range(w.B))           # the whole output: 256 rows
    assert len(rows) == w.B * w.Q
    check_rows(o, lse, o_ref, lse_ref, rows, "gqa_share full size")
    check_as_bench(hx, oracle, w, inp, 1, o, lse, o_ref, lse_ref, rows, "gqa_share full size")


def test_mla_share_full(hx, oracle):
    w = synth.WORKLOADS["mla_share"]
    inp = synth.make_inputs(w, "cuda")
    o, lse, _, _, _ = decode(hx, w, inp, 1)
    assert torch.isfinite(o).all() and torch.isfinite(lse).all()
    # every head of two sequences, plus one row of eight more sequences (one per residue of b modulo 8)
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, [0, 21], extra_rows=[(8 + 3 * j, (37 * j + 5) % w.Q) for j in range(8)])
    assert len(rows) >= 256 and len({b % 8 for b, _ in rows}) == 8
    check_rows(o, lse, o_ref, lse_ref, rows, "mla_share full size")
    check_as_bench(hx, oracle, w, inp, 1, o, lse, o_ref, lse_ref, rows, "mla_share full size")


def test_gqa_full_sharded_vs_unsharded_and_oracle(hx, oracle):
    """1M-token context in 16 shards of 65536 with 1% of the keys scaled x8, all on one GPU."""
    w = synth.WORKLOADS["gqa_full"]
    inp = synth.make_inputs(w, "cuda")
    o16, lse16, parts, lses, ss = decode(hx, w, inp, 16, want_parts=True)
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), 16)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref) and np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    assert np.all(len_ref == 65536)
    o1, lse1, _, _, _ = decode(hx, w, inp, 1)
    d = (o16 - o1).abs().max().item()
    print(f"gqa_full: sharded(16) vs unsharded max-abs {d:.3e}, |o| max {o1.abs().max().item():.3f}")
    assert d <= SHARD_VS_UNSHARDED
    assert (lse16 - lse1).abs().max().item() <= 1e-5
    am = torch.empty((w.B, w.Q), dtype=torch.int32, device="cuda")
    o2 = torch.empty_like(o16)
    from paper_2507_07120_amd import harness
    hx.helix_attn_combine(harness.problem_for(w), parts, lses, o2, argmax_shard=am)
    torch.cuda.synchronize()
    assert torch.equal(o2, o16)
    assert np.array_equal(am.cpu().numpy(), oracle.argmax_f32(lses.cpu().numpy()))
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, range(w.B))           # the whole output: 256 rows
    assert len(rows) == w.B * w.Q
    check_rows(o16, lse16, o_ref, lse_ref, rows, "gqa_full sharded")
    check_rows(o1, lse1, o_ref, lse_ref, rows, "gqa_full unsharded")
    check_as_bench(hx, oracle, w, inp, 16, o16, lse16, o_ref, lse_ref, rows, "gqa_full sharded")


def test_mla_fp8_ragged_full(hx, oracle):
    """B=64 ragged lengths in [16384, 262144], e4m3 latent + per-token scale, 8 shards with uneven tails."""
    w = synth.WORKLOADS["mla_fp8_ragged"]
    inp = synth.make_inputs(w, "cuda")
    lens = inp.lens.numpy()
    assert lens.min() >= 16384 and lens.max() <= 262144
    o8, lse8, _, _, ss = decode(hx, w, inp, 8)
    off_ref, len_ref = oracle.shard_layout(lens, 8)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref + inp.seq_off[:-1].numpy()[None, :])
    assert np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    assert torch.isfinite(o8).all() and torch.isfinite(lse8).all()
    o1, lse1, _, _, _ = decode(hx, w, inp, 1)
    d = (o8 - o1).abs().max().item()
    print(f"mla_fp8_ragged: sharded(8) vs unsharded max-abs {d:.3e}")
    assert d <= SHARD_VS_UNSHARDED
    b_short, b_long = int(lens.argmin()), int(lens.argmax())
    # every head of the shortest and the longest sequence, plus one row of eight more (one per residue modulo 8)
    others = [b for b in range(w.B) if b not in (b_short, b_long)]
    extra = [(next(b for b in others if b % 8 == j), (29 * j + 3) % w.Q) for j in range(8)]
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, [b_short, b_long], extra_rows=extra)
    assert len(rows) >= 256
    check_rows(o8, lse8, o_ref, lse_ref, rows, "mla_fp8_ragged sharded")
    check_as_bench(hx, oracle, w, inp, 8, o8, lse8, o_ref, lse_ref, rows, "mla_fp8_ragged sharded")


def test_gqa_share_mxfp4_full(hx, oracle):
    """The MXFP4-KV share (4M-token context at KVP=8): sampled rows against the oracle, and the same
    cache cut into 4 shards against the unsharded run."""
    w = synth.WORKLOADS["gqa_share_mxfp4"]
    inp = synth.make_inputs(w, "cuda")
    o, lse, _, _, _ = decode(hx, w, inp, 1)
    assert torch.isfinite(o).all() and torch.isfinite(lse).all()
    # (the oracle decodes MXFP4 element by element: half the batch is what a test's time allows)
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, range(0, w.B, 2), extra_rows=[(5, 9), (15, 15)])
    assert len(rows) >= 128
    check_rows(o, lse, o_ref, lse_ref, rows, "gqa_share_mxfp4")
    check_as_bench(hx, oracle, w, inp, 1, o, lse, o_ref, lse_ref, rows, "gqa_share_mxfp4")
    o4, lse4, _, _, _ = decode(hx, w, inp, 4)
    d = (o4 - o).abs().max().item()
    print(f"gqa_share_mxfp4: 4 shards vs unsharded max-abs {d:.3e}")
    assert d <= SHARD_VS_UNSHARDED and (lse4 - lse).abs().max().item() <= 1e-5


def test_gqa_share_fp8_full(hx, oracle):
    """The e4m3-KV share (2M-token context at KVP=8): whole sequences against the oracle, and the same cache cut
    into 4 shards against the unsharded run."""
    w = synth.WORKLOADS["gqa_share_fp8"]
    inp = synth.make_inputs(w, "cuda")
    o, lse, _, _, _ = decode(hx, w, inp, 1)
    assert torch.isfinite(o).all() and torch.isfinite(lse).all()
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, range(w.B))           # the whole output: 256 rows
    assert len(rows) == w.B * w.Q
    check_rows(o, lse, o_ref, lse_ref, rows, "gqa_share_fp8")
    check_as_bench(hx, oracle, w, inp, 1, o, lse, o_ref, lse_ref, rows, "gqa_share_fp8")
    o4, lse4, _, _, _ = decode(hx, w, inp, 4)
    d = (o4 - o).abs().max().item()
    print(f"gqa_share_fp8: 4 shards vs unsharded max-abs {d:.3e}")
    assert d <= SHARD_VS_UNSHARDED and (lse4 - lse).abs().max().item() <= 1e-5


def test_mla_share_mxfp4_full(hx, oracle):
    """The MXFP4 latent share: sampled rows against the oracle, and the same cache cut into 8 shards
    against the unsharded run."""
    w = synth.WORKLOADS["mla_share_mxfp4"]
    inp = synth.make_inputs(w, "cuda")
    o, lse, _, _, _ = decode(hx, w, inp, 1)
    assert torch.isfinite(o).all() and torch.isfinite(lse).all()
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, [13], extra_rows=[(0, 0), (11, 77), (31, 127)])
    assert len(rows) >= 128
    check_rows(o, lse, o_ref, lse_ref, rows, "mla_share_mxfp4")
    check_as_bench(hx, oracle, w, inp, 1, o, lse, o_ref, lse_ref, rows, "mla_share_mxfp4")
    o8, lse8, _, _, _ = decode(hx, w, inp, 8)
    d = (o8 - o).abs().max().item()
    print(f"mla_share_mxfp4: 8 shards vs unsharded max-abs {d:.3e}")
    assert d <= SHARD_VS_UNSHARDED and (lse8 - lse).abs().max().item() <= 1e-5


def test_mla_mxfp4_ragged_full(hx, oracle):
    """The ragged MLA configuration with the latent in MXFP4: packed rows (odd and even first rows), 8 shards."""
    w = synth.WORKLOADS["mla_mxfp4_ragged"]
    inp = synth.make_inputs(w, "cuda")
    lens = inp.lens.numpy()
    o8, lse8, _, _, ss = decode(hx, w, inp, 8)
    off_ref, len_ref = oracle.shard_layout(lens, 8)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref + inp.seq_off[:-1].numpy()[None, :])
    assert np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    assert torch.isfinite(o8).all() and torch.isfinite(lse8).all()
    o1, lse1, _, _, _ = decode(hx, w, inp, 1)
    d = (o8 - o1).abs().max().item()
    print(f"mla_mxfp4_ragged: sharded(8) vs unsharded max-abs {d:.3e}")
    assert d <= SHARD_VS_UNSHARDED
    odd = [b for b in range(w.B) if int(inp.seq_off[b]) % 2 == 1]
    b_short = int(lens.argmin())
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, [b_short], extra_rows=[(odd[0] if odd else 1, 100), (int(lens.argmax()), 17)])
    assert len(rows) >= 128
    check_rows(o8, lse8, o_ref, lse_ref, rows, "mla_mxfp4_ragged sharded")
    check_as_bench(hx, oracle, w, inp, 8, o8, lse8, o_ref, lse_ref, rows, "mla_mxfp4_ragged sharded")


@pytest.mark.parametrize("name", ["mla_fp8_peaked", "mla_mxfp4_peaked"])
def test_mla_peaked_full(hx, oracle, name):
    """The ragged MLA configurations with 1 % of the latent rows scaled by 8 before quantisation (the sharp softmax
    peaks of the full GQA configuration): every head of the shortest sequence and single rows of others against the
    oracle, and 8 shards against the unsharded run."""
    w = synth.WORKLOADS[name]
    inp = synth.make_inputs(w, "cuda")
    lens = inp.lens.numpy()
    o8, lse8, _, _, _ = decode(hx, w, inp, 8)
    assert torch.isfinite(o8).all() and torch.isfinite(lse8).all()
    o1, lse1, _, _, _ = decode(hx, w, inp, 1)
    d = (o8 - o1).abs().max().item()
    print(f"{name}: sharded(8) vs unsharded max-abs {d:.3e}, |o| max {o1.abs().max().item():.2f}")
    assert d <= SHARD_VS_UNSHARDED * max(1.0, o1.abs().max().item())
    assert (lse8 - lse1).abs().max().item() <= 1e-4
    b_short = int(lens.argmin())
    rows, o_ref, lse_ref = oracle_sequences(oracle, w, inp, [b_short], extra_rows=[(int(lens.argmax()), 17), (5, 99)])
    # one fp16 weight per token: |dO| <= 2^-12 max |v| when the softmax is nearly one-hot (rows of up to 8 x 4.7 sigma)
    got = np.stack([o8.cpu().numpy()[b, h] for b, h in rows]).astype(np.float64)
    gl = np.array([lse8.cpu().numpy()[b, h] for b, h in rows], dtype=np.float64)
    err, rel = np.abs(got - o_ref).max(), np.linalg.norm(got - o_ref) / np.linalg.norm(o_ref)
    lerr = np.abs(gl - lse_ref).max()
    print(f"{name}: O max-abs {err:.3e} rel-L2 {rel:.3e}  LSE max-abs {lerr:.3e}  max |o_ref| {np.abs(o_ref).max():.2f}")
    assert err <= max(O_MAX_ABS, 2.0 ** -11 * np.abs(o_ref).max()) and rel <= O_REL_L2 and lerr <= LSE_MAX_ABS
