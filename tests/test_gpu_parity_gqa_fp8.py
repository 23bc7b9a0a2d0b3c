"""GPU parity of the fp8 GQA path (e4m3 codes, one fp32 scale per token shared by its key and value row) against
the CPU oracle, through the C ABI.  Same bars as the bf16 path: the converted operands are exact and the scale acts
in fp32, so O max-abs 2e-3 and relative L2 1e-3 against the fp64 oracle on the same codes and scales,
sharded-vs-unsharded max-abs 1e-5, integers bit-exact."""
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


def run_f8(hx, oracle, w, inp, n_shards, split_tokens=0, value_bar=None):
    from paper_2507_07120_amd import harness
    dev = "cuda"
    prob = harness.problem_for(w, split_tokens)
    ss = harness.make_shards(inp.k, inp.v, inp.lens.to(dev), n_shards, kv_scale=inp.kv_scale)
    off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), n_shards)
    assert np.array_equal(ss.shard_off.cpu().numpy(), off_ref) and np.array_equal(ss.shard_len.cpu().numpy(), len_ref)
    ws = harness.workspace_for(prob, n_shards, max(ss.max_lens), dev)
    ws.view(torch.float32)[: ws.numel() // 4].fill_(float("nan"))
    o = torch.full((w.B, w.Q, w.dv), float("nan"), device=dev)
    lse = torch.full((w.B, w.Q), float("nan"), device=dev)
    o_parts = torch.full((n_shards, w.B, w.Q, w.dv), float("nan"), device=dev)
    lses = torch.full((n_shards, w.B, w.Q), float("nan"), device=dev)
    hx.helix_attn_decode(prob, inp.q, ss.shards, o, ws, lse_out=lse, o_partials=o_parts, lses=lses)
    torch.cuda.synchronize()
    qb, kc, vc, sc = synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), inp.kv_scale.cpu().numpy()
    lens = inp.lens.numpy()
    bar = 2e-3 if value_bar is None else value_bar
    o_ref, lse_ref = oracle.attention(qb, kc, vc, lens, w.scale, kv_heads=w.K, kv_scale=sc)
    has = lens > 0
    check_o(o.cpu().numpy()[has], o_ref[has], f"{w.name} N={n_shards} combined O", bar)
    check_lse(lse.cpu().numpy(), lse_ref, f"{w.name} N={n_shards} combined LSE")
    assert np.all(o.cpu().numpy()[~has] == 0)
    for i in range(n_shards):
        lo, hi = off_ref[i], off_ref[i] + len_ref[i]
        op_ref, lp_ref = oracle.attention(qb, kc, vc, lens, w.scale, kv_heads=w.K, kv_scale=sc, t_lo=lo, t_hi=hi)
        nz = len_ref[i] > 0
        gp = o_parts[i].cpu().numpy()
        if nz.any():
            check_o(gp[nz], op_ref[nz], f"{w.name} shard {i} partial O", bar)
        assert np.all(gp[~nz] == 0)
        check_lse(lses[i].cpu().numpy(), lp_ref, f"{w.name} shard {i} partial LSE")
    return o, lse


def _w(name, B, Q, K, S, N, seed):
    return synth.Workload(name, B=B, Q=Q, K=K, dk=128, dv=128, n_shards=N, scale=1 / math.sqrt(128), seed=seed, seq_len=S, fp8=True)


@pytest.mark.parametrize("B,Q,K,S,N,lens,split", [
    (3, 32, 2, 1000, 3, [1000, 517, 33], 0),       # group of 16, ragged, several blocks + tails
    (2, 16, 1, 4200, 5, [4200, 4100], 256),        # forced small splits -> many records
    (2, 10, 2, 700, 2, [700, 1], 0),               # group of 5 (padded head tile), a 1-token sequence
    (1, 40, 2, 900, 4, [900], 0),                  # group of 20 -> two head tiles
    (4, 8, 8, 300, 8, [300, 0, 17, 128], 128),     # MHA (group 1), an empty sequence, empty shards
    (1, 16, 1, 16, 4, [16], 0),                    # fewer 16-token blocks than shards
    (3, 16, 2, 20000, 20, [20000, 700, 5000], 0),  # more shards than one launch carries
])
def test_gqa_fp8_shapes_against_oracle(hx, oracle, B, Q, K, S, N, lens, split):
    w = _w("gqa_fp8_case", B, Q, K, S, N, 300 + B + N)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    o_n, _ = run_f8(hx, oracle, w, inp, N, split)
    o_1, _ = run_f8(hx, oracle, w, inp, 1, split)
    assert (o_n - o_1).abs().max().item() <= SHARD_VS_UNSHARDED


def test_gqa_fp8_conversion_is_exact_for_every_code(hx, oracle):
    """Every e4m3 code as a key entry and as a value entry (a one-hot query and a one-token sequence read them back):
    the kernel's conversion must give the format's value, the scale must multiply it in fp32."""
    w = _w("gqa_fp8_codes", 1, 16, 1, 256, 1, 5)
    inp = synth.make_inputs(w, "cuda")
    # token t carries code t in every key and value entry; NaN codes (0x7f, 0xff) are left out
    codes = torch.arange(256, dtype=torch.uint8, device="cuda")
    codes[0x7f] = 0
    codes[0xff] = 0
    inp.k[0, 0, :, :] = codes[:, None]
    inp.v[0, 0, :, :] = codes[:, None]
    inp.kv_scale[0, 0, :] = torch.linspace(0.37, 2.9, 256, device="cuda")
    inp.lens = torch.tensor([256], dtype=torch.int32)
    run_f8(hx, oracle, w, inp, 1, value_bar=2e-3 * 448 * 2.9)
    # one token at a time: O is that token's value times its scale (a single weight: the scale, carried by the bf16
    # hi/lo pair to within 2^-17 of itself)
    from paper_2507_07120_amd import harness
    prob = harness.problem_for(w)
    vals = np.array([oracle.e4m3_value(int(c)) for c in codes.cpu().numpy()])
    for t in (0, 1, 7, 8, 0x38, 0x77, 0x7e, 0x80, 0x81, 0xc0, 0xfe):
        k1 = inp.k[:, :, t:t + 1].contiguous()
        v1 = inp.v[:, :, t:t + 1].contiguous()
        s1 = inp.kv_scale[:, :, t:t + 1].contiguous()
        sh = hx.KVShard.from_padded(k1, v1, torch.tensor([1], dtype=torch.int32, device="cuda"), 1, kv_scale=s1)
        ws = harness.workspace_for(prob, 1, 1, "cuda")
        o = torch.empty((1, 16, 128), device="cuda")
        hx.helix_attn_decode(prob, inp.q, [sh], o, ws)
        torch.cuda.synchronize()
        want = float(vals[t]) * float(s1.item())
        assert np.all(np.abs(o.cpu().numpy().astype(np.float64) - want) <= 2.0 ** -16 * abs(want)), (t, o[0, 0, :4], want)


def test_gqa_fp8_token_scales_spread_over_octaves(hx, oracle):
    """Per-token scales between 2^-6 and 2^6 times their natural size: scores and values move with them."""
    w = _w("gqa_fp8_scales", 2, 16, 1, 900, 2, 41)
    inp = synth.make_inputs(w, "cuda")
    g = torch.Generator().manual_seed(9)
    k = torch.randint(-2, 3, inp.kv_scale.shape, generator=g).to(torch.float32)
    inp.kv_scale = (inp.kv_scale.cpu() * torch.exp2(k)).cuda()
    vmax = (inp.v.view(torch.float8_e4m3fn).float().abs().amax(dim=-1) * inp.kv_scale).max().item()
    run_f8(hx, oracle, w, inp, 2, value_bar=max(2e-3, 2.0 ** -11 * vmax))


def test_gqa_fp8_fused_cut_and_strided_views(hx, oracle):
    """helix_attn_decode_kvp on the unsharded fp8 cache, and a cache that is a strided view (token stride 160 bytes,
    scales with their own batch stride)."""
    from paper_2507_07120_amd import harness
    w = _w("gqa_fp8_kvp", 3, 16, 2, 2000, 4, 77)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor([2000, 1, 777], dtype=torch.int32)
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), inp.lens.numpy(), w.scale,
                                      kv_heads=2, kv_scale=inp.kv_scale.cpu().numpy())
    prob = harness.problem_for(w)
    kbig = torch.zeros((3, 2, 2000, 160), dtype=torch.uint8, device="cuda")
    vbig = torch.zeros((3, 2, 2000, 160), dtype=torch.uint8, device="cuda")
    kbig[..., :128] = inp.k
    vbig[..., 16:144] = inp.v
    sbig = torch.zeros((3, 4, 2000), device="cuda")
    sbig[:, ::2] = inp.kv_scale
    for k, v, s in ((inp.k, inp.v, inp.kv_scale), (kbig[..., :128], vbig[..., 16:144], sbig[:, ::2])):
        cache = hx.KVShard.from_padded(k, v, inp.lens.cuda(), 2000, kv_scale=s)
        ws = harness.workspace_for(prob, 4, 2000, "cuda")
        o = torch.full((3, 16, 128), float("nan"), device="cuda")
        lse = torch.full((3, 16), float("nan"), device="cuda")
        off = torch.empty((4, 3), dtype=torch.int64, device="cuda")
        ln = torch.empty((4, 3), dtype=torch.int32, device="cuda")
        hx.helix_attn_decode_kvp(prob, inp.q, cache, 4, o, ws, lse_out=lse, shard_off=off, shard_len=ln)
        torch.cuda.synchronize()
        off_ref, len_ref = oracle.shard_layout(inp.lens.numpy(), 4)
        assert np.array_equal(off.cpu().numpy(), off_ref) and np.array_equal(ln.cpu().numpy(), len_ref)
        check_o(o.cpu().numpy(), o_ref, "fp8 kvp O")
        check_lse(lse.cpu().numpy(), lse_ref, "fp8 kvp LSE")
