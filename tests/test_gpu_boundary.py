"""Behaviour of the C ABI on the GPU beyond plain parity: the device status word (a sequence longer than
the host said), calls from two threads on their own streams, the timed entry point, the ceiling probes,
and MXFP4 inputs at the edge of the format (scale code 0, rows far below the others)."""
import math
import threading

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


def _gqa(seed, B=3, Q=16, K=2, D=128, S=3000, fp4=False):
    w = synth.Workload("edge", B=B, Q=Q, K=K, dk=D, dv=D, n_shards=1, scale=1 / math.sqrt(D), seed=seed, seq_len=S, fp4=fp4)
    return w, synth.make_inputs(w, "cuda")


def _mla(seed, B=2, Q=128, S=700, fp8=False, fp4=False):
    w = synth.Workload("edge_mla", B=B, Q=Q, K=1, dk=576, dv=512, n_shards=1, scale=1 / math.sqrt(192), seed=seed,
                       seq_len=S, mla=True, fp8=fp8, fp4=fp4)
    return w, synth.make_inputs(w, "cuda")


@pytest.mark.parametrize("kind", ["gqa", "gqa_mxfp4", "mla", "mla_e4m3", "mla_two_head_tiles"])
def test_a_sequence_longer_than_max_len(hx, oracle, kind):
    """max_len is an upper bound the host states.  The launches are cut on the device over the tokens the sequences
    really have, so a device-side length beyond it loses nothing and the status word stays clear -- except on the
    one path whose runs are fixed by the host (MLA with more than 128 heads: runs by workgroup id), where the
    surplus tokens are left out and the status word says so.  Every kernel exits normally either way."""
    from paper_2507_07120_amd import harness
    if kind.startswith("gqa"):
        w, inp = _gqa(71, fp4=kind == "gqa_mxfp4")
    else:
        w, inp = _mla(72, Q=160 if kind == "mla_two_head_tiles" else 128, S=9000, fp8=kind == "mla_e4m3")
    prob = harness.problem_for(w)
    S = w.seq_len
    lens = torch.full((w.B,), S, dtype=torch.int32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    o = torch.empty((w.B, w.Q, w.dv), device="cuda")
    lse = torch.empty((w.B, w.Q), device="cuda")

    def shard(max_len):
        if inp.k_mx is not None:
            s = hx.KVShard.from_mxfp4(inp.k, inp.v, inp.k_mx, inp.v_mx, lens, max_len)
        else:
            s = hx.KVShard.from_padded(inp.k, inp.v, lens, max_len, kv_scale=inp.kv_scale)
        s.status = status
        return s
    ws = harness.workspace_for(prob, 2, S, "cuda")
    hx.helix_attn_decode(prob, inp.q, [shard(S)], o, ws, lse_out=lse)
    torch.cuda.synchronize()
    assert status.item() == 0
    o_full = o.clone()
    # the host claims far fewer tokens than the device lengths say
    short = S // 3 if kind.startswith("gqa") else 4096
    hx.helix_attn_decode(prob, inp.q, [shard(short)], o, ws, lse_out=lse)
    torch.cuda.synchronize()
    assert torch.isfinite(o).all()
    if kind != "mla_two_head_tiles":
        assert status.item() == 0
        assert (o - o_full).abs().max().item() <= 1e-5
        hx.helix_attn_decode_kvp(prob, inp.q, shard(short), 2, o, ws, lse_out=lse)     # the fused cut likewise
        torch.cuda.synchronize()
        assert status.item() == 0
        assert (o - o_full).abs().max().item() <= 1e-5
        return
    assert status.item() & 1 == 1
    status.zero_()
    hx.helix_attn_decode_kvp(prob, inp.q, shard(short), 2, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    assert status.item() & 1 == 1
    status.zero_()
    hx.helix_attn_decode_kvp(prob, inp.q, shard(S), 2, o, ws, lse_out=lse)
    torch.cuda.synchronize()
    assert status.item() == 0


def test_two_threads_on_their_own_streams(hx, oracle):
    """No call leaves state behind: two host threads, each with its own stream, buffers and problem (one of them
    the MLA path, whose first call on a device also sets a kernel attribute), get the results of serial calls."""
    from paper_2507_07120_amd import harness
    jobs = []
    for w, inp in (_gqa(81, S=6000), _mla(82, S=2500)):
        prob = harness.problem_for(w)
        lens = inp.lens.cuda()
        sh = hx.KVShard.from_padded(inp.k, inp.v, lens, w.seq_len)
        ws = harness.workspace_for(prob, 1, w.seq_len, "cuda")
        ref_o = torch.empty((w.B, w.Q, w.dv), device="cuda")
        ref_l = torch.empty((w.B, w.Q), device="cuda")
        jobs.append(dict(w=w, inp=inp, prob=prob, sh=sh, ws=ws, ref_o=ref_o, ref_l=ref_l,
                         o=torch.zeros_like(ref_o), lse=torch.zeros_like(ref_l), stream=torch.cuda.Stream()))
    torch.cuda.synchronize()
    errors = []

    def work(j):
        try:
            for _ in range(20):
                hx.helix_attn_decode(j["prob"], j["inp"].q, [j["sh"]], j["o"], j["ws"], lse_out=j["lse"], stream=j["stream"])
            j["stream"].synchronize()
        except Exception as e:      # noqa: BLE001 -- reported in the main thread
            errors.append(e)
    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for j in jobs:                  # the serial reference comes afterwards: the threads may hold the process's first MLA call
        hx.helix_attn_decode(j["prob"], j["inp"].q, [j["sh"]], j["ref_o"], j["ws"], lse_out=j["ref_l"])
    torch.cuda.synchronize()
    for j in jobs:
        assert torch.equal(j["o"], j["ref_o"]) and torch.equal(j["lse"], j["ref_l"])


def test_timed_entry_point_gives_the_same_result_and_a_duration(hx):
    """helix_attn_decode_kvp_timed = helix_attn_decode_kvp + an event pair around the streaming kernel."""
    import ctypes
    import os
    from paper_2507_07120_amd import harness
    w, inp = _gqa(91, B=4, S=20000)
    prob = harness.problem_for(w)
    cache = hx.KVShard.from_padded(inp.k, inp.v, inp.lens.cuda(), w.seq_len)
    ws = harness.workspace_for(prob, 4, w.seq_len, "cuda")
    o1 = torch.empty((w.B, w.Q, w.dv), device="cuda")
    o2 = torch.empty_like(o1)
    hx.helix_attn_decode_kvp(prob, inp.q, cache, 4, o1, ws)
    hip = ctypes.CDLL(os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so"))
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
    hx.helix_attn_decode_kvp(prob, inp.q, cache, 4, o2, ws, events=(e0, e1))
    torch.cuda.synchronize()
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
    assert 0.0 < ms.value < 50.0
    assert torch.equal(o1, o2)
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)


def test_ceiling_probes_run_and_reject_bad_arguments(hx):
    buf = synth.normal_bf16(5, 1, (1 << 24,), "cuda")               # 32 MiB
    assert hx.helix_probe_stream_read(buf, 256, True) == 32 << 20
    assert hx.helix_probe_stream_read(buf, 64, False) == 32 << 20
    flops, nbytes = hx.helix_probe_mfma_lds(buf, 64)
    assert flops == 256 * 8 * 64 * 8 * 16384 and nbytes == 0
    flops, nbytes = hx.helix_probe_mfma_lds(buf, 64, buf)
    assert nbytes == 256 * 8 * 1024 * (64 // 2 + 4)
    torch.cuda.synchronize()
    import ctypes
    lib = hx.load_library()
    assert lib.helix_probe_stream_read(None, 1 << 20, 256, 1, None) == 1
    assert lib.helix_probe_stream_read(buf.data_ptr(), 1000, 256, 1, None) == 2
    assert lib.helix_probe_mfma_lds(buf.data_ptr(), 7, None, 0, None, None, None) == 2
    assert lib.helix_probe_mfma_lds(buf.data_ptr(), 8, buf.data_ptr(), 3 << 20, None, None, None) == 2   # not a power of two


def test_mxfp4_scale_code_zero_and_rows_far_below_the_rest(hx, oracle):
    """E8M0 code 0 is 2^-127: the kernels treat such a block as zero, which is the oracle's value to within
    2^-124 -- far inside the bars when anything else in the cache is of ordinary size.  Likewise an MLA row whose
    largest scale code is below 10 (entries below 2^-115)."""
    from paper_2507_07120_amd import harness
    # GQA: some K and V blocks with scale code 0
    w, inp = _gqa(101, B=2, Q=16, K=1, S=1500, fp4=True)
    g = torch.Generator(device="cpu").manual_seed(7)
    hit = (torch.rand(inp.k_mx.shape, generator=g) < 0.05).cuda()
    inp.k_mx[hit] = 0
    hit = (torch.rand(inp.v_mx.shape, generator=g) < 0.05).cuda()
    inp.v_mx[hit] = 0
    prob = harness.problem_for(w)
    sh = hx.KVShard.from_mxfp4(inp.k, inp.v, inp.k_mx, inp.v_mx, inp.lens.cuda(), w.seq_len)
    ws = harness.workspace_for(prob, 1, w.seq_len, "cuda")
    o = torch.empty((w.B, w.Q, w.dv), device="cuda")
    lse = torch.empty((w.B, w.Q), device="cuda")
    hx.helix_attn_decode(prob, inp.q, [sh], o, ws, lse_out=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), inp.v.cpu().numpy(), inp.lens.numpy(), w.scale,
                                      kv_heads=w.K, mx=(inp.k_mx.cpu().numpy(), inp.v_mx.cpu().numpy()))
    check_o(o.cpu().numpy(), o_ref, "gqa mxfp4 with scale code 0")
    check_lse(lse.cpu().numpy(), lse_ref, "gqa mxfp4 with scale code 0")
    # MLA: whole rows whose scale codes are all below 10, and blocks with code 0 inside ordinary rows
    w, inp = _mla(102, B=2, Q=128, S=900, fp4=True)
    rows = (torch.rand(inp.k_mx.shape[:-1], generator=g) < 0.04).cuda()
    inp.k_mx[rows] = torch.randint(0, 10, (int(rows.sum()), 18), generator=g, dtype=torch.uint8).cuda()
    blocks = (torch.rand(inp.k_mx.shape, generator=g) < 0.03).cuda()
    inp.k_mx[blocks] = 0
    prob = harness.problem_for(w)
    sh = hx.KVShard.from_mxfp4(inp.k, None, inp.k_mx, None, inp.lens.cuda(), w.seq_len)
    ws = harness.workspace_for(prob, 1, w.seq_len, "cuda")
    o = torch.empty((w.B, w.Q, w.dv), device="cuda")
    lse = torch.empty((w.B, w.Q), device="cuda")
    hx.helix_attn_decode(prob, inp.q, [sh], o, ws, lse_out=lse)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attention(synth.bits(inp.q), inp.k.cpu().numpy(), None, inp.lens.numpy(), w.scale,
                                      kv_heads=1, dv=w.dv, mx=(inp.k_mx.cpu().numpy(), None))
    check_o(o.cpu().numpy(), o_ref, "mla mxfp4 with tiny rows")
    check_lse(lse.cpu().numpy(), lse_ref, "mla mxfp4 with tiny rows")
