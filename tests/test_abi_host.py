"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad arguments before launching anything (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    if not os.path.exists(hx_.library_path()):
        from paper_2507_07120_amd import build
        build.build()
    hx_.load_library()
    return hx_


def test_every_declared_symbol_is_exported(hx):
    header = open(os.path.join(ROOT, "include", "helix_attn.h")).read()
    names = set(re.findall(r"\b(helix_[a-z_]+)\s*\(", header))
    assert {"helix_attn_partial", "helix_attn_combine", "helix_attn_decode"} <= names
    lib = ctypes.CDLL(hx.library_path())
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def test_status_strings(hx):
    assert hx.helix_status_string(0) == "ok"
    assert all(hx.helix_status_string(s) for s in range(0, 7))


def test_problem_validation_without_gpu(hx):
    ok = hx.Problem(16, 16, 1, 128, 128, 0.088)
    assert hx.helix_attn_workspace_bytes(ok, 1, 131072) > 0
    split, wgs = hx.helix_attn_plan(ok, [131072])
    assert split % 128 == 0 and wgs >= 256
    # Q not a multiple of K, zero batch, bad scale, unsupported widths
    for bad in [hx.Problem(1, 7, 2, 128, 128, 0.1), hx.Problem(0, 8, 2, 128, 128, 0.1),
                hx.Problem(1, 8, 2, 128, 128, float("nan")), hx.Problem(1, 8, 2, 128, 128, -1.0),
                hx.Problem(1, 8, 2, 96, 96, 0.1), hx.Problem(1, 8, 2, 128, 64, 0.1)]:
        assert hx.helix_attn_workspace_bytes(bad, 1, 1024) == 0
        with pytest.raises(hx.HelixError):
            hx.helix_attn_plan(bad, [1024])
    mla = hx.Problem(32, 128, 1, 576, 512, 0.07, v_aliases_k=True)
    assert hx.helix_attn_workspace_bytes(mla, 1, 131072) > 0
    assert hx.helix_attn_workspace_bytes(hx.Problem(32, 128, 1, 576, 512, 0.07, v_aliases_k=True, kv_dtype=hx.KV_FP8_E4M3), 8, 32768) > 0
    assert hx.helix_attn_workspace_bytes(hx.Problem(32, 128, 2, 576, 512, 0.07, v_aliases_k=True), 1, 1024) == 0   # one latent only
    assert hx.helix_attn_workspace_bytes(hx.Problem(1, 8, 2, 128, 128, 0.1, kv_dtype=hx.KV_FP8_E4M3), 1, 1024) > 0   # e4m3 K/V, head width 128
    assert hx.helix_attn_workspace_bytes(hx.Problem(1, 8, 2, 64, 64, 0.1, kv_dtype=hx.KV_FP8_E4M3), 1, 1024) == 0     # ... and no other
    assert hx.helix_attn_workspace_bytes(ok, 0, 1024) == 0
    assert hx.helix_attn_workspace_bytes(ok, 1, -5) == 0


def test_workspace_bound_covers_shorter_shards(hx):
    """The sizing call must cover any set of shards no longer than max_len."""
    lib = hx.load_library()
    for prob in [hx.Problem(16, 16, 1, 128, 128, 0.088), hx.Problem(4, 64, 8, 128, 128, 0.088),
                 hx.Problem(1, 8, 2, 64, 64, 0.125), hx.Problem(2, 40, 2, 64, 64, 0.125, split_tokens=256),
                 hx.Problem(16, 16, 1, 128, 128, 0.088, kv_dtype=hx.KV_MXFP4), hx.Problem(2, 32, 2, 128, 128, 0.088, kv_dtype=hx.KV_MXFP4),
                 hx.Problem(4, 128, 1, 576, 512, 0.07, v_aliases_k=True), hx.Problem(2, 160, 1, 576, 512, 0.07, v_aliases_k=True),
                 hx.Problem(4, 128, 1, 576, 512, 0.07, v_aliases_k=True, kv_dtype=hx.KV_MXFP4)]:
        for n, max_len in [(1, 131072), (16, 65536), (4, 1024), (8, 100)]:
            bound = hx.helix_attn_workspace_bytes(prob, n, max_len)
            for lens in [[max_len] * n, [max_len // 3] * n, [1] * n, [0] * n, [max_len] + [7] * (n - 1)]:
                split, wgs = hx.helix_attn_plan(prob, lens)
                g = prob.q_heads // prob.kv_heads
                hpw = 128 if prob.v_aliases_k else 16           # query heads one workgroup serves
                tiles = (g + hpw - 1) // hpw
                if prob.v_aliases_k and tiles > 1:
                    # MLA with several head tiles: fixed runs by workgroup id, records of batch * q_heads rows
                    splits = wgs // (prob.batch * tiles)
                    need = splits * prob.batch * prob.q_heads * (prob.dv + 2) * 4
                else:
                    # evenly cut launches: one record per workgroup and per row; a record holds the heads of one
                    # workgroup (all of them for MLA, a tile of 16 for GQA)
                    rows = n * prob.batch * (1 if prob.v_aliases_k else prob.kv_heads * tiles)
                    need = (wgs + rows) * (prob.q_heads if prob.v_aliases_k else 16) * (prob.dv + 2) * 4
                assert need <= bound, (prob, n, max_len, lens)
    del lib


def test_null_and_shape_errors_return_codes(hx):
    lib = hx.load_library()
    p = hx.Problem(1, 8, 2, 64, 64, 0.125).c()
    # NULL q / outputs: status 1, nothing launched
    assert lib.helix_attn_partial(ctypes.byref(p), None, None, None, None, None, 0, None) == 1
    assert lib.helix_attn_combine(ctypes.byref(p), 4, None, None, None, None, None, None) == 1
    assert lib.helix_attn_decode(ctypes.byref(p), None, None, 4, None, None, None, None, None, 0, None) == 1
    assert lib.helix_shard_layout(None, None, 4, 4, None, None, None) == 1
    assert lib.helix_attn_partial(None, 16, None, 16, 16, None, 0, None) == 1
    # a shard with a NULL key pointer, a misaligned one, a bad stride, a missing workspace
    from paper_2507_07120_amd.binding import _CShard
    fake = 0x100000
    def shard(**kw):
        d = dict(k=fake, v=fake, kv_scale=None, k_stride_b=0, k_stride_h=64 * 1024, k_stride_t=64,
                 v_stride_b=0, v_stride_h=64 * 1024, v_stride_t=64, s_stride_b=0, s_stride_h=0,
                 tok_off=None, len=fake, max_len=1024)
        d.update(kw)
        return _CShard(**d)
    def partial(s, ws=fake, ws_bytes=1 << 30):
        return lib.helix_attn_partial(ctypes.byref(p), fake, ctypes.byref(s), fake, fake, ws, ws_bytes, None)
    assert partial(shard(k=None)) == 1
    assert partial(shard(k=fake + 2)) == 2
    assert partial(shard(k_stride_t=60)) == 2
    assert partial(shard(v_stride_t=65)) == 2
    assert partial(shard(max_len=-1)) == 2
    assert partial(shard(), ws=None) == 4
    assert partial(shard(), ws_bytes=16) == 4
    assert partial(shard(), ws=fake + 8) == 4
    arr = (_CShard * 1)(shard())
    assert lib.helix_attn_decode(ctypes.byref(p), fake, arr, 0, fake, None, None, None, fake, 1 << 30, None) == 2
    assert lib.helix_attn_decode(ctypes.byref(p), fake, arr, 1, fake, None, fake, None, fake, 1 << 30, None) == 1


def test_append_owner_matches_the_oracle_rule(hx, oracle):
    """Sec. 2.3: 16 decode tokens per rank, round robin -- host integer arithmetic, bit-exact."""
    for n in [1, 2, 3, 8, 16, 64]:
        for t in list(range(0, 300)) + [10 ** 6, 2 ** 40 + 17]:
            assert hx.helix_kv_append_owner(t, n) == oracle.round_robin_owner(t, n)
    assert hx.helix_kv_append_owner(-1, 4) == -1 and hx.helix_kv_append_owner(3, 0) == -1


def test_appendix_a_calculator_matches_the_oracle(hx, oracle):
    """Host arithmetic of the library against the oracle's closed forms (Appendix A), over the Fig. 1
    parameter set and MI355X parameters, plus the plateau beyond TP = K."""
    for TPA in (1, 2, 4, 8, 16, 64):
        for KVP in (1, 2, 8, 32):
            for S in (4096, 1 << 20, 3.5e6):
                for bp, bw in ((0.5, 8.0e12), (2.0, 8.0e12), (0.53125, 8.0e12)):
                    a = hx.helix_kv_read_seconds(8, 8, 128, S, bp, bw, TPA, KVP)
                    b = oracle.kv_read_seconds(8, 8, 128, S, bp, bw, TPA, KVP)
                    assert abs(a - b) <= 1e-15 * max(1.0, abs(b))
    for TPA, TPF in ((1, 1), (8, 8), (16, 16), (8, 64)):
        a = hx.helix_weight_read_seconds(16384, 128, 8, 128, 65536, 0.5, 8.0e12, TPA, TPF)
        b = oracle.weight_read_seconds(16384, 128, 8, 128, 65536, 0.5, 8.0e12, TPA, TPF)
        assert abs(a - b) <= 1e-18 + 1e-15 * abs(b)
    assert hx.helix_kv_read_seconds(8, 8, 128, 1 << 20, 0.5, 8.0e12, 8, 1) == hx.helix_kv_read_seconds(8, 8, 128, 1 << 20, 0.5, 8.0e12, 64, 1)
    import math
    assert math.isnan(hx.helix_kv_read_seconds(0, 8, 128, 1.0, 0.5, 8.0e12, 1, 1))
    assert math.isnan(hx.helix_weight_read_seconds(1, 1, 1, 1, 1, 0.5, 0.0, 1, 1))


def test_hopb_timeline_model_matches_the_oracle(hx, oracle):
    """Fig. 3 as arithmetic, library against oracle; 8 requests of 2 + 1.2 units: 25.6 without overlap."""
    import math
    assert hx.helix_hopb_span(8, 2.0, 1.2, False) == 25.6
    for n in (1, 2, 8, 33):
        for ta, tc in ((2.0, 1.2), (0.5, 3.0), (1.0, 1.0), (0.0, 1.0)):
            for pipe in (False, True):
                assert hx.helix_hopb_span(n, ta, tc, pipe) == oracle.hopb_span(n, ta, tc, pipe)
    assert math.isnan(hx.helix_hopb_span(0, 1.0, 1.0, True)) and math.isnan(hx.helix_hopb_span(3, -1.0, 1.0, True))


def test_plans_follow_from_the_upper_bounds(hx):
    """Every launch is cut on the device, evenly over the tokens the sequences really have, so the host plan follows
    from the upper bounds alone: one workgroup per CU (three for MXFP4 K/V), fewer for a launch with little work, as
    many as an explicit run length asks for."""
    gqa = hx.Problem(16, 16, 1, 128, 128, 0.088)
    assert hx.helix_attn_plan(gqa, [131072]) == (8192, 256)
    with pytest.raises(hx.HelixError):
        hx.helix_attn_plan(gqa, [-1])
    assert hx.helix_attn_plan(hx.Problem(16, 16, 1, 128, 128, 0.088, kv_dtype=hx.KV_MXFP4), [524288])[1] == 768
    assert hx.helix_attn_plan(hx.Problem(4, 64, 8, 128, 128, 0.088), [65536] * 16)[1] == 256
    assert hx.helix_attn_plan(hx.Problem(1, 8, 2, 64, 64, 0.125), [1024] * 4) == (128, 64)      # 4 x 2 rows x 8 tiles
    assert hx.helix_attn_plan(hx.Problem(2, 16, 1, 128, 128, 0.088, split_tokens=1000), [10000])[1] == 20   # runs of 1024
    mla = hx.Problem(64, 128, 1, 576, 512, 0.07, v_aliases_k=True, kv_dtype=hx.KV_FP8_E4M3)
    assert hx.helix_attn_plan(mla, [32768] * 8)[1] == 256
    assert hx.helix_attn_plan(hx.Problem(1, 128, 1, 576, 512, 0.07, v_aliases_k=True), [1000])[1] == 3
    assert hx.helix_attn_plan(hx.Problem(2, 128, 1, 576, 512, 0.07, v_aliases_k=True, split_tokens=64), [1000, 24])[1] == 32
    # more shards than one launch carries: a plan per launch
    assert hx.helix_attn_plan(gqa, [131072] * 20)[1] == 512
    # more than 16 query heads per KV head: one set of workgroups per head tile, a multiple of 8 each where the launch
    # is large enough (the workgroups that read the same tokens then share an XCD), the sets cut alike
    assert hx.helix_attn_plan(hx.Problem(2, 32, 1, 128, 128, 0.088), [524288]) == (8192, 256)          # 2 x 128
    assert hx.helix_attn_plan(hx.Problem(2, 80, 2, 128, 128, 0.088), [524288])[1] == 240               # 3 x 80
    assert hx.helix_attn_plan(hx.Problem(1, 128, 1, 128, 128, 0.088), [1 << 20])[1] == 256             # 8 x 32
    assert hx.helix_attn_plan(hx.Problem(1, 40, 1, 64, 64, 0.125), [600])[1] == 15                     # 3 x 5 tiles
    assert hx.helix_attn_plan(hx.Problem(2, 32, 1, 128, 128, 0.088, split_tokens=1000), [10000])[1] == 40


def test_mxfp4_and_hopb_argument_errors_without_gpu(hx):
    """The newer entry points validate on the host as well: status codes, nothing launched."""
    lib = hx.load_library()
    mx = hx.Problem(2, 16, 1, 128, 128, 0.088, kv_dtype=hx.KV_MXFP4)
    assert hx.helix_attn_workspace_bytes(mx, 1, 4096) > 0
    assert hx.helix_attn_workspace_bytes(hx.Problem(2, 16, 1, 64, 64, 0.125, kv_dtype=hx.KV_MXFP4), 1, 4096) == 0
    mla_mx = hx.Problem(2, 128, 1, 576, 512, 0.07, v_aliases_k=True, kv_dtype=hx.KV_MXFP4)
    assert hx.helix_attn_workspace_bytes(mla_mx, 1, 4096) > 0                 # an MXFP4 latent is served by the MLA path
    assert hx.helix_attn_workspace_bytes(hx.Problem(2, 128, 1, 576, 512, 0.07, kv_dtype=hx.KV_MXFP4), 1, 4096) == 0
    # ... and appended to without value rows: value codes or scales given for a latent are a shape error
    pm = mla_mx.c()
    from paper_2507_07120_amd import binding
    dummy, no_shard = ctypes.c_void_p(64), (binding._CShard * 1)()            # never dereferenced: both calls fail first
    assert lib.helix_kv_append_mxfp4(ctypes.byref(pm), no_shard, 1, 0, dummy, dummy, dummy, None, 16, None, None) == 2
    assert lib.helix_kv_append_mxfp4(ctypes.byref(pm), no_shard, 1, 0, dummy, None, None, None, 16, None, None) == 1
    p = mx.c()
    # helix_kv_append refuses an MXFP4 cache (3 = unsupported); the MXFP4 variant refuses a bf16 one and NULLs
    assert lib.helix_kv_append(ctypes.byref(p), None, 1, 0, None, None, None, 16, None, None) == 3
    pb = hx.Problem(2, 16, 1, 128, 128, 0.088).c()
    assert lib.helix_kv_append_mxfp4(ctypes.byref(pb), None, 1, 0, None, None, None, None, 16, None, None) == 3
    assert lib.helix_kv_append_mxfp4(ctypes.byref(p), None, 1, 0, None, None, None, None, 16, None, None) == 1
    # pipelined decode: NULL buffers, more groups than sequences
    assert lib.helix_attn_decode_hopb(ctypes.byref(pb), None, None, 1, 2, None, None, None, None, None, None,
                                      None, 0, None, None, None) == 1
    # decode with the cut inside the kernel: NULL buffers, a shard count out of range
    assert lib.helix_attn_decode_kvp(ctypes.byref(pb), None, None, 2, None, None, None, None, None, None, None, 0, None) == 1
    assert hx.helix_attn_hopb_workspace_bytes(hx.Problem(2, 16, 1, 128, 128, 0.088), 1, 4096, 2) > 0
    assert hx.helix_attn_hopb_workspace_bytes(hx.Problem(2, 16, 1, 128, 128, 0.088), 1, 4096, 3) == 0


def test_decode_kvp_rejects_a_null_problem_before_reading_it(hx):
    """helix_attn_decode_kvp derives slice bounds from the problem: a NULL problem is a status, not a crash."""
    lib = hx.load_library()
    from paper_2507_07120_amd.binding import _CShard
    fake = 0x100000
    cache = _CShard(k=fake, v=fake, len=fake, max_len=1024, k_stride_h=128 * 1024, k_stride_t=128,
                    v_stride_h=128 * 1024, v_stride_t=128)
    assert lib.helix_attn_decode_kvp(None, fake, ctypes.byref(cache), 2, fake, None, None, None, None, None,
                                     fake, 1 << 30, None) == 1
    assert lib.helix_attn_decode_kvp_timed(None, fake, ctypes.byref(cache), 2, fake, None, None, None, None, None,
                                           fake, 1 << 30, None, fake, fake) == 1
    # the timed form needs both events
    p = hx.Problem(2, 16, 1, 128, 128, 0.088).c()
    assert lib.helix_attn_decode_kvp_timed(ctypes.byref(p), fake, ctypes.byref(cache), 2, fake, None, None, None, None, None,
                                           fake, 1 << 30, None, None, fake) == 1
    # a status word must be a 4-byte aligned device address
    bad = _CShard(k=fake, v=fake, len=fake, max_len=1024, k_stride_h=128 * 1024, k_stride_t=128,
                  v_stride_h=128 * 1024, v_stride_t=128, status=fake + 2)
    assert lib.helix_attn_partial(ctypes.byref(p), fake, ctypes.byref(bad), fake, fake, fake, 1 << 30, None) == 2


def test_plan_of_many_long_shards_does_not_wrap(hx):
    """rows * total tokens beyond 2^39: the run length stays a positive multiple of the granule that fits
    32 bits, and the workgroup count follows from that same value (or the call is refused as a shape error)."""
    n = 1024
    for prob, granule in [(hx.Problem(64, 128, 1, 576, 512, 0.07, v_aliases_k=True), 32),
                          (hx.Problem(4096, 16, 1, 128, 128, 0.088), 128),
                          (hx.Problem(4096, 16, 1, 128, 128, 0.088, kv_dtype=hx.KV_MXFP4), 128)]:
        lens = [2 ** 31 - 1] * n
        try:
            split, wgs = hx.helix_attn_plan(prob, lens)
        except hx.HelixError as e:
            assert e.status == 2
            continue
        assert 0 < split <= 2 ** 31 - 1 and split % granule == 0
        rows = prob.batch * prob.kv_heads
        # one launch per 16 shards, each cut evenly over one workgroup per CU (three for MXFP4 K/V, and as many more as
        # keep a run's byte offsets within 32 bits)
        assert wgs >= 256 * (n // 16) and wgs % (n // 16) == 0
        assert rows > 0
        assert hx.helix_attn_workspace_bytes(prob, n, 2 ** 31 - 1) > 0
    # an explicit run length near the top of the range is rounded down to the granule, not up past 2^31
    prob = hx.Problem(2, 16, 1, 128, 128, 0.088, split_tokens=2 ** 31 - 1)
    split, _ = hx.helix_attn_plan(prob, [1000])
    assert 0 < split <= 2 ** 31 - 1 and split % 128 == 0


def test_host_entry_points_from_several_threads(hx):
    """The library keeps no per-call state: planning, sizing and argument checks run concurrently from several
    threads and give each thread the answers a single thread gets."""
    import threading
    lib = hx.load_library()
    probs = [hx.Problem(16, 16, 1, 128, 128, 0.088), hx.Problem(4, 64, 8, 128, 128, 0.088),
             hx.Problem(32, 128, 1, 576, 512, 0.07, v_aliases_k=True),
             hx.Problem(64, 128, 1, 576, 512, 0.07, v_aliases_k=True, kv_dtype=hx.KV_FP8_E4M3)]
    want = [(hx.helix_attn_plan(p, [131072, 777]), hx.helix_attn_workspace_bytes(p, 2, 131072)) for p in probs]
    errors = []

    def work(i):
        try:
            for _ in range(200):
                p = probs[i % len(probs)]
                got = (hx.helix_attn_plan(p, [131072, 777]), hx.helix_attn_workspace_bytes(p, 2, 131072))
                assert got == want[i % len(probs)]
                c = p.c()
                assert lib.helix_attn_partial(ctypes.byref(c), None, None, None, None, None, 0, None) == 1
                assert lib.helix_attn_decode_kvp(ctypes.byref(c), None, None, 2, None, None, None, None, None, None, None, 0, None) == 1
        except Exception as e:      # noqa: BLE001 -- reported below, in the main thread
            errors.append(e)
    threads = [threading.Thread(target=work, args=(i,)) for i in range(8)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
