"""Pins of the CPU oracle against things other than itself: a high-precision brute-force evaluator,
closed forms, invariants of softmax attention, library routines and format definitions.
None of these tests touches the GPU or the HIP library."""
import math
import os

import mpmath
import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_bits(x):
    """float array -> (uint16 bf16 bits, float64 values after rounding), via torch's converter."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy(), t.to(torch.float64).numpy()


def rand_problem(rng, B, Q, K, dk, dv, S, mla=False):
    q, qf = bf16_bits(rng.standard_normal((B, Q, dk)))
    k, kf = bf16_bits(rng.standard_normal((B, K, S, dk)))
    if mla:
        return q, qf, k, kf, None, kf[..., :dv]
    v, vf = bf16_bits(rng.standard_normal((B, K, S, dv)))
    return q, qf, k, kf, v, vf


def brute_force(qf, kf, vf, lens, scale, prec=60):
    """Explicit softmax-matrix evaluation in 60-digit arithmetic, structured unlike the oracle:
    builds all weights first, normalises them, then takes the weighted sum."""
    mpmath.mp.dps = prec
    B, Q, dk = qf.shape
    K = kf.shape[1]
    dv = vf.shape[-1]
    g = Q // K
    o = np.zeros((B, Q, dv))
    lse = np.zeros((B, Q))
    for b in range(B):
        for h in range(Q):
            kh = h // g
            L = int(lens[b])
            e = []
            for t in range(L):
                dot = mpmath.mpf(0)
                for d in range(dk):
                    dot += mpmath.mpf(float(qf[b, h, d])) * mpmath.mpf(float(kf[b, kh, t, d]))
                e.append(mpmath.e ** (mpmath.mpf(scale) * dot))
            z = mpmath.fsum(e)
            w = [x / z for x in e]
            for j in range(dv):
                o[b, h, j] = float(mpmath.fsum(w[t] * mpmath.mpf(float(vf[b, kh, t, j])) for t in range(L)))
            lse[b, h] = float(mpmath.log(z))
    return o, lse


# ---------------------------------------------------------------- P1 brute force, tiny
@pytest.mark.parametrize("B,Q,K,dk,dv,S", [(1, 1, 1, 1, 1, 1), (2, 4, 2, 4, 3, 8), (1, 6, 3, 5, 2, 7), (2, 2, 1, 3, 3, 5)])
def test_brute_force_tiny(oracle, B, Q, K, dk, dv, S):
    rng = np.random.default_rng(100 + S)
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    lens = np.array([S - (b % 2) * min(2, S - 1) for b in range(B)], dtype=np.int32)
    scale = 0.37
    o, lse = oracle.attention(q, k, v, lens, scale, kv_heads=K)
    o_ref, lse_ref = brute_force(qf, kf, vf, lens, scale)
    assert np.abs(o - o_ref).max() <= 1e-13
    assert np.abs(lse - lse_ref).max() <= 1e-13


def test_brute_force_large_scores(oracle):
    """Scores of several hundred: a missing max-subtraction overflows exp in fp64."""
    rng = np.random.default_rng(5)
    q, qf, k, kf, v, vf = rand_problem(rng, 1, 2, 1, 4, 3, 6)
    lens = np.array([6], dtype=np.int32)
    scale = 300.0
    o, lse = oracle.attention(q, k, v, lens, scale, kv_heads=1)
    o_ref, lse_ref = brute_force(qf, kf, vf, lens, scale)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    assert np.abs(o - o_ref).max() <= 1e-12
    assert np.abs(lse - lse_ref).max() <= 1e-10 * max(1.0, np.abs(lse_ref).max())


# ---------------------------------------------------------------- P14 library routine
def test_against_torch_float64_softmax(oracle):
    rng = np.random.default_rng(11)
    B, Q, K, dk, dv, S = 2, 8, 2, 64, 32, 300
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    lens = np.array([S, S - 77], dtype=np.int32)
    scale = 1 / math.sqrt(dk)
    o, lse = oracle.attention(q, k, v, lens, scale, kv_heads=K)
    for b in range(B):
        L = lens[b]
        kk = torch.as_tensor(kf[b, :, :L]).repeat_interleave(Q // K, dim=0)      # [Q,L,dk]
        vv = torch.as_tensor(vf[b, :, :L]).repeat_interleave(Q // K, dim=0)
        s = torch.einsum("hd,htd->ht", torch.as_tensor(qf[b]), kk) * scale
        ref = torch.einsum("ht,htj->hj", torch.softmax(s, dim=-1), vv).numpy()
        assert np.abs(o[b] - ref).max() <= 1e-12
        assert np.abs(lse[b] - torch.logsumexp(s, dim=-1).numpy()).max() <= 1e-12


# ---------------------------------------------------------------- P2 shard-split identity
@pytest.mark.parametrize("n_shards", [1, 2, 5, 40])
def test_shard_split_identity(oracle, n_shards):
    """Attention per shard + LSE combine == attention over the unsharded cache (Sec. 2.1.1),
    for arbitrary cut points including empty shards and one token per shard."""
    rng = np.random.default_rng(20 + n_shards)
    B, Q, K, dk, dv, S = 2, 4, 2, 16, 8, 40
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    lens = np.array([S, S - 9], dtype=np.int32)
    scale = 0.5
    o_full, lse_full = oracle.attention(q, k, v, lens, scale, kv_heads=K)
    cuts = np.zeros((n_shards + 1, B), dtype=np.int64)
    for b in range(B):
        if n_shards == 40:
            inner = np.arange(1, n_shards)                         # one token per shard, then empties
        else:
            inner = np.sort(rng.integers(0, lens[b] + 1, size=n_shards - 1))
        cuts[1:n_shards, b] = np.minimum(inner, lens[b])
        cuts[n_shards, b] = lens[b]
    o_parts, lse_parts = [], []
    for i in range(n_shards):
        o_i, lse_i = oracle.attention(q, k, v, lens, scale, kv_heads=K, t_lo=cuts[i], t_hi=cuts[i + 1])
        o_parts.append(o_i)
        lse_parts.append(lse_i)
    o_c, lse_c = oracle.combine(np.stack(o_parts), np.stack(lse_parts))
    assert np.abs(o_c - o_full).max() <= 1e-12 * max(1.0, np.abs(o_full).max())
    assert np.abs(lse_c - lse_full).max() <= 1e-12 * max(1.0, np.abs(lse_full).max())
    # an empty shard reports lse = -inf and a zero partial
    for i in range(n_shards):
        for b in range(B):
            if cuts[i + 1, b] == cuts[i, b]:
                assert np.all(lse_parts[i][b] == -np.inf) and np.all(o_parts[i][b] == 0)


def test_partial_is_attention_of_the_slice(oracle):
    """A shard's partial equals plain attention over a cache that holds only the shard's tokens."""
    rng = np.random.default_rng(31)
    B, Q, K, dk, dv, S = 1, 4, 2, 8, 8, 24
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    lens = np.array([S], dtype=np.int32)
    lo, hi = 5, 17
    o_p, lse_p = oracle.attention(q, k, v, lens, 0.3, kv_heads=K, t_lo=np.array([lo]), t_hi=np.array([hi]))
    k2 = np.ascontiguousarray(k[:, :, lo:hi])
    v2 = np.ascontiguousarray(v[:, :, lo:hi])
    o_s, lse_s = oracle.attention(q, k2, v2, np.array([hi - lo], dtype=np.int32), 0.3, kv_heads=K)
    assert np.array_equal(o_p, o_s) and np.array_equal(lse_p, lse_s)


# ---------------------------------------------------------------- P3..P9 closed forms and invariants
def test_constant_v_gives_v(oracle):
    rng = np.random.default_rng(3)
    B, Q, K, dk, dv, S = 2, 4, 2, 8, 5, 33
    q, qf, k, kf, _, _ = rand_problem(rng, B, Q, K, dk, dv, S)
    c, cf = bf16_bits(rng.standard_normal((B, K, 1, dv)))
    v = np.ascontiguousarray(np.broadcast_to(c, (B, K, S, dv)))
    o, _ = oracle.attention(q, k, v, np.full(B, S, np.int32), 0.7, kv_heads=K)
    g = Q // K
    for h in range(Q):
        assert np.abs(o[:, h] - cf[:, h // g, 0]).max() <= 1e-14


def test_equal_keys_give_mean_v(oracle):
    rng = np.random.default_rng(4)
    B, Q, K, dk, dv, S = 1, 4, 2, 8, 6, 19
    q, qf, _, _, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    k1, k1f = bf16_bits(rng.standard_normal((B, K, 1, dk)))
    k = np.ascontiguousarray(np.broadcast_to(k1, (B, K, S, dk)))
    scale = 0.25
    o, lse = oracle.attention(q, k, v, np.full(B, S, np.int32), scale, kv_heads=K)
    g = Q // K
    for h in range(Q):
        assert np.abs(o[0, h] - vf[0, h // g].mean(axis=0)).max() <= 1e-13
        expect = scale * float(np.dot(qf[0, h], k1f[0, h // g, 0])) + math.log(S)
        assert abs(lse[0, h] - expect) <= 1e-13


def test_single_token(oracle):
    rng = np.random.default_rng(6)
    q, qf, k, kf, v, vf = rand_problem(rng, 2, 2, 1, 8, 4, 3)
    lens = np.array([1, 1], dtype=np.int32)
    o, lse = oracle.attention(q, k, v, lens, 0.9, kv_heads=1)
    for b in range(2):
        for h in range(2):
            assert np.array_equal(o[b, h], vf[b, 0, 0])
            assert abs(lse[b, h] - 0.9 * float(np.dot(qf[b, h], kf[b, 0, 0]))) <= 1e-15


def test_zero_query_gives_mean_v(oracle):
    rng = np.random.default_rng(7)
    _, _, k, kf, v, vf = rand_problem(rng, 1, 2, 1, 8, 4, 21)
    q = np.zeros((1, 2, 8), dtype=np.uint16)
    o, lse = oracle.attention(q, k, v, np.array([21], np.int32), 1.3, kv_heads=1)
    assert np.abs(o[0] - vf[0, 0].mean(axis=0)).max() <= 1e-14
    assert np.abs(lse - math.log(21)).max() <= 1e-14


def test_duplicate_and_permute(oracle):
    rng = np.random.default_rng(8)
    B, Q, K, dk, dv, S = 1, 4, 2, 8, 4, 13
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    o, lse = oracle.attention(q, k, v, np.array([S], np.int32), 0.4, kv_heads=K)
    k2 = np.ascontiguousarray(np.concatenate([k, k], axis=2))
    v2 = np.ascontiguousarray(np.concatenate([v, v], axis=2))
    o2, lse2 = oracle.attention(q, k2, v2, np.array([2 * S], np.int32), 0.4, kv_heads=K)
    assert np.abs(o2 - o).max() <= 1e-13 and np.abs(lse2 - lse - math.log(2)).max() <= 1e-13
    perm = rng.permutation(S)
    o3, lse3 = oracle.attention(q, np.ascontiguousarray(k[:, :, perm]), np.ascontiguousarray(v[:, :, perm]),
                                np.array([S], np.int32), 0.4, kv_heads=K)
    assert np.abs(o3 - o).max() <= 1e-13 and np.abs(lse3 - lse).max() <= 1e-13


def test_key_shift(oracle):
    """k_t <- k_t + c leaves O unchanged and adds scale*q.c to the LSE.  Small integers keep the
    shifted keys exact in bf16."""
    rng = np.random.default_rng(9)
    B, Q, K, dk, dv, S = 1, 2, 1, 6, 4, 11
    qi = rng.integers(-3, 4, size=(B, Q, dk)).astype(np.float32)
    ki = rng.integers(-4, 5, size=(B, K, S, dk)).astype(np.float32)
    ci = rng.integers(-4, 5, size=(dk,)).astype(np.float32)
    q, qf = bf16_bits(qi)
    k, _ = bf16_bits(ki)
    ks, _ = bf16_bits(ki + ci)
    v, _ = bf16_bits(rng.standard_normal((B, K, S, dv)))
    lens = np.array([S], np.int32)
    scale = 0.125
    o, lse = oracle.attention(q, k, v, lens, scale, kv_heads=K)
    o2, lse2 = oracle.attention(q, ks, v, lens, scale, kv_heads=K)
    assert np.abs(o2 - o).max() <= 1e-12
    for h in range(Q):
        assert abs(lse2[0, h] - lse[0, h] - scale * float(np.dot(qf[0, h], ci))) <= 1e-12


def test_peaked_limit(oracle):
    """Scaling one key's alignment with the query up drives O to that key's value, monotonically,
    with no inf/NaN."""
    rng = np.random.default_rng(10)
    B, Q, K, dk, dv, S = 1, 1, 1, 8, 4, 16
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    star = 5
    prev = None
    for lam in [1.0, 4.0, 16.0, 64.0, 256.0]:
        kk = kf.copy()
        kk[0, 0, star] = qf[0, 0] * lam            # aligned with q, so its score grows with lam
        kb, _ = bf16_bits(kk)
        o, lse = oracle.attention(q, kb, v, np.array([S], np.int32), 1.0, kv_heads=K)
        assert np.isfinite(o).all() and np.isfinite(lse).all()
        dist = np.abs(o[0, 0] - vf[0, 0, star]).max()
        if prev is not None:
            assert dist <= prev + 1e-15
        prev = dist
    assert prev <= 1e-12


# ---------------------------------------------------------------- P10, P11 structure
def test_gqa_grouping(oracle):
    rng = np.random.default_rng(12)
    B, Q, K, dk, dv, S = 1, 6, 3, 8, 4, 9
    q, qf, k, kf, v, vf = rand_problem(rng, B, Q, K, dk, dv, S)
    q[:, 1] = q[:, 0]          # heads 0,1 share KV head 0; give them the same query
    q[:, 2] = q[:, 0]          # head 2 is in the NEXT group: same query, different KV head
    lens = np.array([S], np.int32)
    o, lse = oracle.attention(q, k, v, lens, 0.6, kv_heads=K)
    assert np.array_equal(o[0, 0], o[0, 1]) and lse[0, 0] == lse[0, 1]
    assert not np.array_equal(o[0, 0], o[0, 2])
    # swapping KV heads 0 and 1 swaps the outputs of groups {0,1} and {2,3} when their queries swap too
    sw = [1, 0, 2]
    qs = q[:, [2, 3, 0, 1, 4, 5]]
    o2, lse2 = oracle.attention(np.ascontiguousarray(qs), np.ascontiguousarray(k[:, sw]),
                                np.ascontiguousarray(v[:, sw]), lens, 0.6, kv_heads=K)
    assert np.array_equal(o2[0, [2, 3, 0, 1, 4, 5]], o[0]) and np.array_equal(lse2[0, [2, 3, 0, 1, 4, 5]], lse[0])


def test_mla_alias_equals_explicit_v(oracle):
    rng = np.random.default_rng(13)
    B, Q, dk, dv, S = 2, 5, 12, 8, 17
    q, qf, k, kf, _, _ = rand_problem(rng, B, Q, 1, dk, dv, S, mla=True)
    lens = np.array([S, S - 4], np.int32)
    o_a, lse_a = oracle.attention(q, k, None, lens, 0.2, kv_heads=1, dv=dv)
    v = np.ascontiguousarray(k[..., :dv])
    o_e, lse_e = oracle.attention(q, k, v, lens, 0.2, kv_heads=1)
    assert np.array_equal(o_a, o_e) and np.array_equal(lse_a, lse_e)


def test_row_selection_and_ragged_packed(oracle):
    """The (b,h) subset interface and packed ragged storage address the same tokens."""
    rng = np.random.default_rng(14)
    B, Q, dk, dv = 3, 4, 8, 6
    lens = np.array([5, 9, 2], np.int32)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    q, qf = bf16_bits(rng.standard_normal((B, Q, dk)))
    kp, kpf = bf16_bits(rng.standard_normal((int(off[-1]), dk)))
    o_all, lse_all = oracle.attention(q, kp, None, lens, 0.5, kv_heads=1, dv=dv, tok_off=off[:B])
    # padded copy of the same tokens
    S = int(lens.max())
    kpad = np.zeros((B, 1, S, dk), np.uint16)
    for b in range(B):
        kpad[b, 0, :lens[b]] = kp[off[b]:off[b + 1]]
    o_pad, lse_pad = oracle.attention(q, kpad, None, lens, 0.5, kv_heads=1, dv=dv)
    assert np.array_equal(o_all, o_pad) and np.array_equal(lse_all, lse_pad)
    rows = [(2, 1), (0, 3), (1, 0)]
    o_r, lse_r = oracle.attention(q, kp, None, lens, 0.5, kv_heads=1, dv=dv, tok_off=off[:B], rows=rows)
    for i, (b, h) in enumerate(rows):
        assert np.array_equal(o_r[i], o_all[b, h]) and lse_r[i] == lse_all[b, h]


# ---------------------------------------------------------------- P12 storage formats
def test_e4m3_table_against_format_definition(oracle):
    with open(os.path.join(GOLDEN, "e4m3_values.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            code, val = line.split()
            got = oracle.e4m3_value(int(code, 16))
            if val == "nan":
                assert math.isnan(got)
            else:
                assert got == float(val) and math.copysign(1, got) == math.copysign(1, float(val))


def test_e4m3_all_codes_against_library_decoder(oracle):
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for c in range(256):
        got = oracle.e4m3_value(c)
        assert (math.isnan(got) and math.isnan(ref[c])) or got == ref[c]
    # monotone in the code within each sign (excluding NaN): a structural check of the exponent field
    vals = [oracle.e4m3_value(c) for c in range(0x7F)]
    assert all(a < b for a, b in zip(vals, vals[1:]))


def test_bf16_decoding_against_library(oracle):
    """Every bf16 bit pattern class: the oracle's decode (via S=1 attention returning v) equals torch's."""
    pats = np.array([0x0000, 0x8000, 0x3F80, 0xBF80, 0x0001, 0x007F, 0x0080, 0x7F7F, 0xFF7F, 0x3EAB, 0x4049],
                    dtype=np.uint16)
    ref = torch.as_tensor(pats.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    q = np.zeros((1, 1, len(pats)), np.uint16)
    k = pats.reshape(1, 1, 1, -1).copy()
    o, _ = oracle.attention(q, k, None, np.array([1], np.int32), 1.0, kv_heads=1, dv=len(pats))
    assert np.array_equal(o[0, 0], ref)


def test_fp8_attention_against_dequantised_bf16_free_reference(oracle):
    """fp8 codes * per-token scale: compare with torch float64 softmax on library-dequantised values."""
    rng = np.random.default_rng(15)
    B, Q, dk, dv, S = 2, 3, 16, 8, 29
    q, qf = bf16_bits(rng.standard_normal((B, Q, dk)))
    codes = rng.integers(0, 256, size=(B, 1, S, dk)).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x3A                                   # no NaN codes
    sc = rng.uniform(0.001, 0.02, size=(B, 1, S)).astype(np.float32)
    lens = np.array([S, S - 6], np.int32)
    scale = 1.7
    o, lse = oracle.attention(q, codes, None, lens, scale, kv_heads=1, dv=dv, kv_scale=sc)
    deq = torch.as_tensor(codes).view(torch.float8_e4m3fn).to(torch.float64) * torch.as_tensor(sc).to(torch.float64)[..., None]
    for b in range(B):
        L = lens[b]
        s = torch.as_tensor(qf[b]) @ deq[b, 0, :L].T * scale
        ref = torch.softmax(s, -1) @ deq[b, 0, :L, :dv]
        assert np.abs(o[b] - ref.numpy()).max() <= 1e-12
        assert np.abs(lse[b] - torch.logsumexp(s, -1).numpy()).max() <= 1e-12


def test_fp8_attention_with_separate_value_rows_and_kv_heads(oracle):
    """The GQA fp8 cache: separate key and value code rows per kv head, ONE scale per (sequence, kv head, token)
    that both rows share; query head h reads kv head h // (Q / K).  Against torch float64 softmax on
    library-dequantised values."""
    rng = np.random.default_rng(151)
    B, Q, K, dk, dv, S = 2, 6, 3, 16, 8, 23
    q, qf = bf16_bits(rng.standard_normal((B, Q, dk)))
    kc = rng.integers(0, 256, size=(B, K, S, dk)).astype(np.uint8)
    vc = rng.integers(0, 256, size=(B, K, S, dv)).astype(np.uint8)
    kc[(kc & 0x7F) == 0x7F] = 0x3A                                         # no NaN codes
    vc[(vc & 0x7F) == 0x7F] = 0x41
    sc = rng.uniform(0.001, 0.02, size=(B, K, S)).astype(np.float32)
    lens = np.array([S, S - 9], np.int32)
    scale = 0.9
    o, lse = oracle.attention(q, kc, vc, lens, scale, kv_heads=K, kv_scale=sc)
    f = torch.as_tensor(sc).to(torch.float64)[..., None]
    kd = torch.as_tensor(kc).view(torch.float8_e4m3fn).to(torch.float64) * f
    vd = torch.as_tensor(vc).view(torch.float8_e4m3fn).to(torch.float64) * f
    for b in range(B):
        L = lens[b]
        for h in range(Q):
            kh = h // (Q // K)
            s = torch.as_tensor(qf[b, h]) @ kd[b, kh, :L].T * scale
            ref = torch.softmax(s, -1) @ vd[b, kh, :L]
            assert np.abs(o[b, h] - ref.numpy()).max() <= 1e-12
            assert abs(lse[b, h] - torch.logsumexp(s, -1).item()) <= 1e-12
    # the value rows really are their own array: swapping them for the key rows' first dv entries changes O
    o2, _ = oracle.attention(q, kc, np.ascontiguousarray(kc[..., :dv]), lens, scale, kv_heads=K, kv_scale=sc)
    assert np.abs(o2 - o).max() > 1e-3


# ---------------------------------------------------------------- P13 combine alone
def test_combine_closed_forms(oracle):
    rng = np.random.default_rng(16)
    o_p = rng.standard_normal((3, 2, 4, 5))
    lse_p = rng.standard_normal((3, 2, 4))
    # N = 1 is the identity
    o1, l1 = oracle.combine(o_p[:1], lse_p[:1])
    assert np.array_equal(o1, o_p[0]) and np.array_equal(l1, lse_p[0])
    # equal LSEs: plain mean, LSE + ln N
    eq = np.broadcast_to(lse_p[:1], lse_p.shape)
    o2, l2 = oracle.combine(o_p, eq)
    assert np.abs(o2 - o_p.mean(axis=0)).max() <= 1e-15
    assert np.abs(l2 - (lse_p[0] + math.log(3))).max() <= 1e-15
    # a shard with lse = -inf is ignored, whatever its partial holds
    lse_inf = lse_p.copy()
    lse_inf[1] = -np.inf
    o_bad = o_p.copy()
    o_bad[1] = 1e300
    o3, l3 = oracle.combine(o_bad, lse_inf)
    o3_ref, l3_ref = oracle.combine(o_p[[0, 2]], lse_p[[0, 2]])
    assert np.array_equal(o3, o3_ref) and np.array_equal(l3, l3_ref)
    # all empty
    o4, l4 = oracle.combine(o_p, np.full_like(lse_p, -np.inf))
    assert np.all(o4 == 0) and np.all(l4 == -np.inf)
    # two shards, hand formula: weights sigmoid(a-b), sigmoid(b-a)
    a, b = 0.3, -1.1
    oa, ob = np.array([[1.0, 2.0]]), np.array([[-3.0, 0.5]])
    o5, l5 = oracle.combine(np.stack([oa, ob]), np.array([[a], [b]]))
    wa = 1 / (1 + math.exp(b - a))
    assert np.abs(o5 - (wa * oa + (1 - wa) * ob)).max() <= 1e-15
    assert abs(l5[0] - math.log(math.exp(a) + math.exp(b))) <= 1e-15
    # permuting the shards changes nothing
    o6, l6 = oracle.combine(o_p[[2, 0, 1]], lse_p[[2, 0, 1]])
    o7, l7 = oracle.combine(o_p, lse_p)
    assert np.abs(o6 - o7).max() <= 1e-15 and np.abs(l6 - l7).max() <= 1e-15


def test_argmax_bookkeeping(oracle):
    lse = np.array([[1.0, -np.inf, 3.0, 2.0], [1.0, -np.inf, 3.0, 5.0], [0.5, -np.inf, 7.0, 5.0]], dtype=np.float32)
    assert oracle.argmax_f32(lse).tolist() == [0, 0, 2, 1]
    rng = np.random.default_rng(17)
    x = rng.standard_normal((7, 50)).astype(np.float32)
    assert np.array_equal(oracle.argmax_f32(x), np.argmax(x, axis=0).astype(np.int32))


# ---------------------------------------------------------------- integer metadata
def test_shard_layout_properties(oracle):
    rng = np.random.default_rng(18)
    lens = np.concatenate([[0, 1, 15, 16, 17, 127, 128, 129, 4096, 262144], rng.integers(1, 300000, size=50)])
    for N in [1, 2, 3, 4, 8, 16, 64]:
        off, ln = oracle.shard_layout(lens, N)
        assert off.dtype == np.int64 and ln.dtype == np.int32 and off.shape == (N, len(lens))
        assert np.array_equal(ln.sum(axis=0), lens)                       # a partition ...
        assert np.array_equal(off[0], np.zeros(len(lens)))                # ... starting at 0 ...
        assert np.array_equal(off[1:], (off + ln)[:-1])                   # ... contiguous, in order
        width = ln.max(axis=0)
        assert np.all(width % 16 == 0) or np.all((width % 16 == 0) | (ln[0] == lens))   # whole 16-token blocks
        assert np.all(width <= -(-lens // N) + 15)                        # within a block of equal slices
        # only the last non-empty shard may be short
        for b in range(len(lens)):
            nz = ln[:, b][ln[:, b] > 0]
            assert np.all(nz[:-1] == nz[0]) if len(nz) > 1 else True
    off, ln = oracle.shard_layout([4096], 4)                              # equal slices S/KVP when N*16 | S
    assert ln[:, 0].tolist() == [1024] * 4 and off[:, 0].tolist() == [0, 1024, 2048, 3072]
    off, ln = oracle.shard_layout([100], 8)                               # 100 tokens: 16-token slices, tails empty
    assert ln[:, 0].tolist() == [16, 16, 16, 16, 16, 16, 4, 0]


def test_round_robin_append_owner(oracle):
    """Sec. 2.3: 16 decode steps append to rank 0, the next 16 to rank 1, cycling over the ranks."""
    N = 4
    owners = [oracle.round_robin_owner(t, N) for t in range(16 * N * 2)]
    assert owners[:16] == [0] * 16 and owners[16:32] == [1] * 16 and owners[48:64] == [3] * 16
    assert owners[64:80] == [0] * 16
    counts = np.bincount(owners, minlength=N)
    assert np.all(counts == 32)


def test_appendix_a_kv_read_time(oracle):
    with open(os.path.join(GOLDEN, "appendix_a_kv_read.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            B, K, Hsz, S, bp, bw, TPA, KVP, sec = line.split()
            got = oracle.kv_read_seconds(int(B), int(K), int(Hsz), int(S), float(bp), float(bw), int(TPA), int(KVP))
            assert abs(got - float(sec)) <= 1e-15


def test_appendix_a_weight_read_time(oracle):
    with open(os.path.join(GOLDEN, "appendix_a_weight_read.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            H, Q, K, Hsz, F, bp, bw, TPA, TPF, sec = line.split()
            got = oracle.weight_read_seconds(int(H), int(Q), int(K), int(Hsz), int(F), float(bp), float(bw), int(TPA), int(TPF))
            assert abs(got - float(sec)) <= 1e-15


def test_appendix_a_trends_of_fig_1(oracle):
    """The three trends Fig. 1 shows for KV reads: flat in TP width beyond TP = K, linear in S, 1/KVP."""
    kv = lambda **kw: oracle.kv_read_seconds(8, 8, 128, kw.get("S", 1 << 20), 0.5, 8.0e12, kw.get("TPA", 1), kw.get("KVP", 1))
    assert kv(TPA=8) == kv(TPA=16) == kv(TPA=64) and kv(TPA=4) == 2 * kv(TPA=8)
    assert kv(S=1 << 22) == 4 * kv(S=1 << 20)
    assert kv(KVP=32) == kv() / 32


def test_hopb_timeline_of_fig_3(oracle):
    with open(os.path.join(GOLDEN, "fig3_hopb_timeline.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            n, ta, tc, pipe, span, tol = line.split()
            assert abs(oracle.hopb_span(int(n), float(ta), float(tc), int(pipe)) - float(span)) <= float(tol)
    # structure: one request cannot overlap with anything; a slow exchange becomes the bottleneck stage;
    # the pipelined span never exceeds the sequential one and never undercuts either stage's total
    assert oracle.hopb_span(1, 2.0, 1.2, 1) == oracle.hopb_span(1, 2.0, 1.2, 0) == 3.2
    assert oracle.hopb_span(8, 2.0, 1.2, 1) == 8 * 2.0 + 1.2
    assert oracle.hopb_span(8, 1.0, 3.0, 1) == 1.0 + 8 * 3.0
    for n, ta, tc in [(2, 1.0, 1.0), (5, 0.3, 2.0), (7, 2.0, 0.1)]:
        p_, s_ = oracle.hopb_span(n, ta, tc, 1), oracle.hopb_span(n, ta, tc, 0)
        assert max(n * ta, n * tc) <= p_ <= s_
    # brute force: simulate the two resources event by event
    def simulate(n, ta, tc):
        attn_free = comm_free = 0.0
        for _ in range(n):
            attn_free += ta                       # attention unit is busy back to back
            comm_free = max(comm_free, attn_free) + tc
        return comm_free
    for n, ta, tc in [(8, 2.0, 1.2), (3, 1.0, 4.0), (6, 0.5, 0.5)]:
        assert abs(simulate(n, ta, tc) - oracle.hopb_span(n, ta, tc, 1)) <= 1e-12


# ---------------------------------------------------------------- P13 MXFP4 storage (FP4 of the paper's evaluation, Sec. 3)
def test_mxfp4_tables_against_format_definition(oracle):
    with open(os.path.join(GOLDEN, "mxfp4_values.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            kind, code, val = line.split()
            got = (oracle.e2m1_value if kind == "e2m1" else oracle.e8m0_value)(int(code, 16))
            if val == "nan":
                assert math.isnan(got)
            else:
                assert got == float(val) and math.copysign(1, got) == math.copysign(1, float(val)), (kind, code)
    # closed form of the scale: successive codes double
    for c in range(0, 254):
        assert oracle.e8m0_value(c + 1) == 2.0 * oracle.e8m0_value(c)


def _mxfp4_random(rng, shape_rows, D):
    """Random MXFP4 codes / scales and their values: every product 2^(s-127) * e2m1 with s near 127 is
    exactly representable in bf16, so the same tensor can be handed over as bf16 bits."""
    grid = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
    nib = rng.integers(0, 16, size=shape_rows + (D,)).astype(np.uint8)
    sc = rng.integers(120, 134, size=shape_rows + (D // 32,)).astype(np.uint8)
    vals = np.where(nib & 8, -1.0, 1.0) * grid[nib & 7] * np.exp2(np.repeat(sc.astype(np.float64), 32, axis=-1) - 127.0)
    packed = (nib[..., 0::2] | (nib[..., 1::2] << 4)).astype(np.uint8)
    return packed, sc, vals


def test_mxfp4_attention_equals_the_same_values_given_as_bf16(oracle):
    """Ties the MXFP4 read path (nibble order, scale index, strides) to the pinned bf16 path: identical
    element values must give identical results, bit for bit."""
    rng = np.random.default_rng(16)
    B, Q, K, D, S = 2, 4, 2, 64, 37
    q, _ = bf16_bits(rng.standard_normal((B, Q, D)))
    kc, ks, kv = _mxfp4_random(rng, (B, K, S), D)
    vc, vs, vv = _mxfp4_random(rng, (B, K, S), D)
    kb, kf = bf16_bits(kv)
    vb, vf = bf16_bits(vv)
    assert np.array_equal(kf, kv) and np.array_equal(vf, vv)               # exactly representable
    lens = np.array([S, S - 9], np.int32)
    o4, l4 = oracle.attention(q, kc, vc, lens, 0.3, kv_heads=K, mx=(ks, vs))
    o16, l16 = oracle.attention(q, kb, vb, lens, 0.3, kv_heads=K)
    assert np.array_equal(o4, o16) and np.array_equal(l4, l16)
    # a shard of it as well
    t_lo, t_hi = np.array([5, 0], np.int64), np.array([30, 11], np.int64)
    o4s, l4s = oracle.attention(q, kc, vc, lens, 0.3, kv_heads=K, mx=(ks, vs), t_lo=t_lo, t_hi=t_hi)
    o16s, l16s = oracle.attention(q, kb, vb, lens, 0.3, kv_heads=K, t_lo=t_lo, t_hi=t_hi)
    assert np.array_equal(o4s, o16s) and np.array_equal(l4s, l16s)


def test_mxfp4_latent_equals_the_same_values_given_as_bf16(oracle):
    """The MLA case of the MXFP4 read path: the value is the first dv entries of the key row, block scales
    included.  Identical element values given as a bf16 latent must give identical results, bit for bit --
    and a value that took its scales from anywhere else would not."""
    rng = np.random.default_rng(18)
    B, Q, D, DV, S = 2, 5, 96, 64, 29
    q, _ = bf16_bits(rng.standard_normal((B, Q, D)))
    kc, ks, kv = _mxfp4_random(rng, (B, 1, S), D)
    kb, kf = bf16_bits(kv)
    assert np.array_equal(kf, kv)
    lens = np.array([S, S - 6], np.int32)
    o4, l4 = oracle.attention(q, kc, None, lens, 0.2, kv_heads=1, dv=DV, mx=(ks, None))
    o16, l16 = oracle.attention(q, kb, None, lens, 0.2, kv_heads=1, dv=DV)
    assert o4.shape == (B, Q, DV) and np.array_equal(o4, o16) and np.array_equal(l4, l16)
    t_lo, t_hi = np.array([3, 0], np.int64), np.array([20, 7], np.int64)
    o4s, l4s = oracle.attention(q, kc, None, lens, 0.2, kv_heads=1, dv=DV, mx=(ks, None), t_lo=t_lo, t_hi=t_hi)
    o16s, l16s = oracle.attention(q, kb, None, lens, 0.2, kv_heads=1, dv=DV, t_lo=t_lo, t_hi=t_hi)
    assert np.array_equal(o4s, o16s) and np.array_equal(l4s, l16s)
    # one token: O is that token's decoded row, cut to dv
    o1, _ = oracle.attention(q, kc, None, np.array([1, 1], np.int32), 0.2, kv_heads=1, dv=DV, mx=(ks, None))
    assert np.array_equal(o1, np.broadcast_to(kv[:, 0, 0:1, :DV], (B, Q, DV)))


def test_mxfp4_latent_packed_rows_equal_padded(oracle):
    """Ragged packed storage of an MXFP4 latent (rows of all sequences back to back, odd first rows
    included) addresses the same codes and block scales as the padded layout."""
    rng = np.random.default_rng(19)
    B, Q, D, DV = 3, 4, 64, 32
    lens = np.array([7, 12, 5], np.int32)
    q, _ = bf16_bits(rng.standard_normal((B, Q, D)))
    kc, ks, _ = _mxfp4_random(rng, (int(lens.sum()),), D)
    off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64)
    S = int(lens.max())
    pc = np.zeros((B, 1, S, D // 2), np.uint8)
    ps = np.full((B, 1, S, D // 32), 127, np.uint8)
    for b in range(B):
        pc[b, 0, :lens[b]] = kc[off[b]:off[b] + lens[b]]
        ps[b, 0, :lens[b]] = ks[off[b]:off[b] + lens[b]]
    o_p, l_p = oracle.attention(q, kc, None, lens, 0.25, kv_heads=1, dv=DV, mx=(ks, None), tok_off=off)
    o_d, l_d = oracle.attention(q, pc, None, lens, 0.25, kv_heads=1, dv=DV, mx=(ps, None))
    assert np.array_equal(o_p, o_d) and np.array_equal(l_p, l_d)
    t_lo, t_hi = np.array([2, 0, 1], np.int64), np.array([7, 5, 1], np.int64)
    o_p, l_p = oracle.attention(q, kc, None, lens, 0.25, kv_heads=1, dv=DV, mx=(ks, None), tok_off=off, t_lo=t_lo, t_hi=t_hi)
    o_d, l_d = oracle.attention(q, pc, None, lens, 0.25, kv_heads=1, dv=DV, mx=(ps, None), t_lo=t_lo, t_hi=t_hi)
    assert np.array_equal(o_p, o_d) and np.array_equal(l_p, l_d)


def test_mxfp4_single_token_returns_the_decoded_value_row(oracle):
    """S = 1: the output is the value row itself -- element j of the row must come from nibble j%2 of
    byte j/2 and scale j/32 (a transposed nibble or a shifted scale index fails here)."""
    D = 64
    nib = (np.arange(D) * 7 + 3) % 16
    packed = (nib[0::2] | (nib[1::2] << 4)).astype(np.uint8).reshape(1, 1, 1, D // 2)
    sc = np.array([126, 129], np.uint8).reshape(1, 1, 1, 2)
    q = np.zeros((1, 1, D), np.uint16)
    o, lse = oracle.attention(q, packed, packed, np.array([1], np.int32), 1.0, kv_heads=1, mx=(sc, sc))
    grid = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    want = [(-1.0 if n & 8 else 1.0) * grid[n & 7] * (0.5 if j < 32 else 4.0) for j, n in enumerate(nib)]
    assert np.array_equal(o[0, 0], np.array(want)) and lse[0, 0] == 0.0


def test_mxfp4_quantiser_round_trip_properties(oracle):
    """The input generator's quantiser against the format: decoded values are within half a grid step
    of the source (a quarter of the block scale times the local spacing), and the largest entry of a
    block lands on 4 or 6 times the scale."""
    import synth
    x = synth.normal_f32(3, 9, 0, 64 * 128, "cpu").view(64, 128)
    codes, scales = synth.quantize_mxfp4(x)
    codes, scales = codes.numpy(), scales.numpy()
    dec = np.empty((64, 128))
    for r in range(64):
        for j in range(128):
            dec[r, j] = oracle.e8m0_value(scales[r, j // 32]) * oracle.e2m1_value(int(codes[r, j // 2]) >> (4 * (j & 1)))
    xs = x.numpy().astype(np.float64)
    X = np.repeat(np.array([[oracle.e8m0_value(s) for s in row] for row in scales]), 32, axis=1)
    a = np.abs(xs) / X
    step = np.where(a < 2, 0.5, np.where(a < 4, 1.0, 2.0))
    assert np.all(np.abs(dec - xs) <= np.where(a > 6, a - 6 + 1e-12, step / 2 + 1e-12) * X)
    top = np.abs(dec).reshape(64, 4, 32).max(-1) / np.array([[oracle.e8m0_value(s) for s in row] for row in scales])
    assert np.all((top == 4.0) | (top == 6.0))
