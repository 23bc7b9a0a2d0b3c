"""Multi-step decode with the staggered round-robin KV append (Sec. 2.3): 16 decode tokens go to
KVP rank 0, the next 16 to rank 1, ...  After every step the sharded attention over the unevenly
grown shards must still equal attention over the logical (unsharded) sequence, the integer
bookkeeping (owner, shard lengths) must be bit-exact, and the appended rows must be exact copies."""
import math

import numpy as np
import pytest
import torch

import synth
from test_gpu_parity_gqa import check_lse, check_o

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    hx_.load_library()
    assert torch.cuda.is_available()
    return hx_


def run_loop(hx, oracle, w, prefill_lens, n_steps, cap):
    from paper_2507_07120_amd import harness
    dev = "cuda"
    N, B = w.n_shards, w.B
    prob = harness.problem_for(w)
    S0 = max(prefill_lens)
    base = synth.make_inputs(synth.scaled(w, seq_len=S0, len_range=None), dev)        # prefill cache, padded layout
    lens0 = torch.tensor(prefill_lens, dtype=torch.int32)
    # KVP cut of the prefill by the library's layout kernel
    off = torch.empty((N, B), dtype=torch.int64, device=dev)
    ln = torch.empty((N, B), dtype=torch.int32, device=dev)
    hx.helix_shard_layout(lens0.to(dev), N, off, ln)
    off_h, ln_h = off.cpu().numpy(), ln.cpu().numpy()
    off_ref, ln_ref = oracle.shard_layout(prefill_lens, N)
    assert np.array_equal(off_h, off_ref) and np.array_equal(ln_h, ln_ref)
    # every rank owns its own storage with room to grow
    kdt = base.k.dtype
    ks = [torch.zeros((B, w.K, cap, w.dk), dtype=kdt, device=dev) for _ in range(N)]
    vs = [None if w.mla else torch.zeros((B, w.K, cap, w.dv), dtype=kdt, device=dev) for _ in range(N)]
    ss = [torch.zeros((B, w.K, cap), dtype=torch.float32, device=dev) if w.fp8 else None for _ in range(N)]
    for i in range(N):
        for b in range(B):
            lo, n = int(off_h[i, b]), int(ln_h[i, b])
            ks[i][b, :, :n] = base.k[b, :, lo:lo + n]
            if not w.mla:
                vs[i][b, :, :n] = base.v[b, :, lo:lo + n]
            if w.fp8:
                ss[i][b, :, :n] = base.kv_scale[b, :, lo:lo + n]
    shards = [hx.KVShard.from_padded(ks[i], vs[i], ln[i], int(ln_h[i].max()), kv_scale=ss[i]) for i in range(N)]
    ws = harness.workspace_for(prob, N, cap, dev)
    overflow = torch.zeros(1, dtype=torch.int32, device=dev)
    # the logical, unsharded sequence on the host (what the oracle sees)
    log_k = [synth.bits(base.k[b, :, :prefill_lens[b]]) for b in range(B)]          # [K, L, dk] each
    log_v = [None if w.mla else synth.bits(base.v[b, :, :prefill_lens[b]]) for b in range(B)]
    log_s = [base.kv_scale[b, :, :prefill_lens[b]].cpu().numpy() if w.fp8 else None for b in range(B)]
    model_len = ln_h.copy()
    o = torch.empty((B, w.Q, w.dv), device=dev)
    lse = torch.empty((B, w.Q), device=dev)
    for t in range(n_steps):
        q = synth.normal_bf16(w.seed, 1000 + t, (B, w.Q, w.dk), dev)
        if w.fp8 and not w.mla:
            kc, vc, sc = synth.normal_e4m3_kv_rows(w.seed, 2000 + t, 3000 + t, B * w.K, w.dk, w.dv, dev)
            k_new, v_new, s_new = kc.view(B, w.K, w.dk), vc.view(B, w.K, w.dv), sc.view(B, w.K)
        elif w.fp8:
            codes, sc = synth.normal_e4m3_rows(w.seed, 2000 + t, B * w.K, w.dk, dev)
            k_new, s_new, v_new = codes.view(B, w.K, w.dk), sc.view(B, w.K), None
        else:
            k_new = synth.normal_bf16(w.seed, 2000 + t, (B, w.K, w.dk), dev)
            v_new = None if w.mla else synth.normal_bf16(w.seed, 3000 + t, (B, w.K, w.dv), dev)
            s_new = None
        owner = oracle.round_robin_owner(t, N)
        assert hx.helix_kv_append_owner(t, N) == owner
        hx.helix_kv_append(prob, shards, t, k_new, v_new, cap, scale_new=s_new, overflow=overflow)
        model_len[owner] += 1
        shards[owner].max_len += 1
        for b in range(B):
            log_k[b] = np.concatenate([log_k[b], synth.bits(k_new[b])[:, None, :]], axis=1)
            if not w.mla:
                log_v[b] = np.concatenate([log_v[b], synth.bits(v_new[b])[:, None, :]], axis=1)
            if w.fp8:
                log_s[b] = np.concatenate([log_s[b], s_new[b].cpu().numpy()[:, None]], axis=1)
        hx.helix_attn_decode(prob, q, shards, o, ws, lse_out=lse)
        torch.cuda.synchronize()
        check = t < 3 or t % 7 == 0 or t == n_steps - 1 or t % 16 in (0, 15)
        if check:
            assert np.array_equal(ln.cpu().numpy(), model_len), f"step {t}: shard lengths"
            # the row just appended is an exact copy
            for b in range(B):
                pos = int(model_len[owner, b]) - 1
                assert torch.equal(ks[owner][b, :, pos].view(torch.uint8), k_new[b].view(torch.uint8))
            L = [prefill_lens[b] + t + 1 for b in range(B)]
            for b in range(B):
                ob, lb = oracle.attention(synth.bits(q[b:b + 1]), np.ascontiguousarray(log_k[b][None]),
                                          None if w.mla else np.ascontiguousarray(log_v[b][None]),
                                          np.array([L[b]], np.int32), w.scale, kv_heads=w.K, dv=w.dv,
                                          kv_scale=None if not w.fp8 else np.ascontiguousarray(log_s[b][None]))
                check_o(o[b:b + 1].cpu().numpy(), ob, f"step {t} seq {b} O")
                check_lse(lse[b:b + 1].cpu().numpy(), lb, f"step {t} seq {b} LSE")
    assert overflow.item() == 0
    # growth is balanced: after whole cycles every rank received the same number of decode tokens
    grown = model_len - ln_h
    whole = (n_steps // (16 * N)) * 16
    assert np.all(grown >= whole) and np.all(grown <= whole + 16)
    return shards, overflow, prob, ks


def test_gqa_decode_loop_round_robin(hx, oracle):
    w = synth.Workload("loop_gqa", B=2, Q=8, K=2, dk=128, dv=128, n_shards=3, scale=1 / math.sqrt(128), seed=61, seq_len=1)
    shards, overflow, prob, ks = run_loop(hx, oracle, w, prefill_lens=[100, 37], n_steps=16 * 3 * 2 + 5, cap=128)
    # a full shard refuses the token and raises the flag instead of writing out of bounds
    k_new = synth.normal_bf16(1, 1, (2, 2, 128), "cuda")
    before = shards[0].len.clone()
    t = 0
    while True:                      # fill rank 0 of the shorter sequence up to its capacity
        if hx.helix_kv_append_owner(t, 3) == 0:
            hx.helix_kv_append(prob, shards, t, k_new, k_new, 128, overflow=overflow)
            torch.cuda.synchronize()
            if overflow.item():
                break
        t += 1
        assert t < 10000
    assert shards[0].len.max().item() == 128 and (shards[0].len >= before).all()


def test_mla_fp8_decode_loop_round_robin(hx, oracle):
    w = synth.Workload("loop_mla", B=2, Q=128, K=1, dk=576, dv=512, n_shards=2, scale=1 / math.sqrt(192), seed=62,
                       seq_len=1, mla=True, fp8=True)
    run_loop(hx, oracle, w, prefill_lens=[70, 33], n_steps=40, cap=96)


def test_gqa_fp8_decode_loop_round_robin(hx, oracle):
    """The e4m3 GQA cache grows by one key row, one value row and their shared scale per step."""
    w = synth.Workload("loop_gqa_fp8", B=2, Q=16, K=2, dk=128, dv=128, n_shards=3, scale=1 / math.sqrt(128), seed=63,
                       seq_len=1, fp8=True)
    run_loop(hx, oracle, w, prefill_lens=[90, 41], n_steps=16 * 3 + 9, cap=128)
