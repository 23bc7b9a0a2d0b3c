"""Seeded random shapes through the C ABI against the CPU oracle: batch, head grouping, head width, shard count,
forced run lengths and ragged lengths (empty and one-token sequences included) drawn per case, for the bf16, e4m3 and
MXFP4 GQA kernels and the three MLA latent formats.  The fixed cases of the other test files aim at known edges;
these look for the ones nobody thought of.  Usual bars: O max-abs 2e-3 / relative L2 1e-3, LSE 1e-4, per-shard
fragments and the argmax bookkeeping included (the helpers of the parity tests do the checking)."""
import math
import random

import pytest
import torch

import synth
from test_gpu_parity_gqa import run_sharded
from test_gpu_parity_mla import O_MAX_ABS, run_mla
from test_gpu_parity_mla_mxfp4 import run as run_mla_mx
from test_gpu_parity_mxfp4 import run_mx
from test_gpu_parity_gqa_fp8 import run_f8

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hx():
    import paper_2507_07120_amd as hx_
    hx_.load_library()
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return hx_


def _lens(rng, B, S):
    out = []
    for _ in range(B):
        kind = rng.random()
        out.append(0 if kind < 0.1 else 1 if kind < 0.15 else S if kind < 0.3 else rng.randint(1, S))
    if all(x == 0 for x in out):
        out[0] = S
    return out


def _split(rng, granule):
    return 0 if rng.random() < 0.5 else granule * rng.randint(1, 6) - rng.randint(0, granule - 1)


@pytest.mark.parametrize("case", range(24))
def test_random_gqa_bf16(hx, oracle, case):
    rng = random.Random(1000 + case)
    D = rng.choice([64, 128])
    K = rng.choice([1, 1, 2, 3, 8])
    g = rng.choice([1, 2, 5, 8, 16, 16, 20, 33])
    B = rng.randint(1, 9)
    S = rng.choice([1, 31, 128, 129, 700, 2500, 6000])
    N = rng.choice([1, 1, 2, 3, 5, 8, 17, 20])
    w = synth.Workload(f"rand_gqa_{case}", B=B, Q=K * g, K=K, dk=D, dv=D, n_shards=N, scale=1 / math.sqrt(D), seed=5000 + case, seq_len=S)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(_lens(rng, B, S), dtype=torch.int32)
    run_sharded(hx, oracle, w, inp, N, split_tokens=_split(rng, 128))


@pytest.mark.parametrize("case", range(10))
def test_random_gqa_mxfp4(hx, oracle, case):
    rng = random.Random(2000 + case)
    K = rng.choice([1, 2, 4])
    g = rng.choice([1, 4, 16, 16, 24])
    B = rng.randint(1, 7)
    S = rng.choice([1, 33, 128, 500, 3000])
    N = rng.choice([1, 2, 3, 6, 18])
    w = synth.Workload(f"rand_mx_{case}", B=B, Q=K * g, K=K, dk=128, dv=128, n_shards=N, scale=1 / math.sqrt(128), seed=6000 + case,
                       seq_len=S, fp4=True)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(_lens(rng, B, S), dtype=torch.int32)
    run_mx(hx, oracle, w, inp, N, split_tokens=_split(rng, 128))


@pytest.mark.parametrize("case", range(12))
def test_random_gqa_fp8(hx, oracle, case):
    rng = random.Random(4000 + case)
    K = rng.choice([1, 2, 4])
    g = rng.choice([1, 4, 16, 16, 24])
    B = rng.randint(1, 7)
    S = rng.choice([1, 33, 128, 500, 3000])
    N = rng.choice([1, 2, 3, 6, 18])
    w = synth.Workload(f"rand_f8_{case}", B=B, Q=K * g, K=K, dk=128, dv=128, n_shards=N, scale=1 / math.sqrt(128), seed=8000 + case,
                       seq_len=S, fp8=True)
    inp = synth.make_inputs(w, "cuda")
    inp.lens = torch.tensor(_lens(rng, B, S), dtype=torch.int32)
    run_f8(hx, oracle, w, inp, N, split_tokens=_split(rng, 128))


@pytest.mark.parametrize("case", range(18))
def test_random_mla(hx, oracle, case):
    rng = random.Random(3000 + case)
    fmt = ["bf16", "e4m3", "mxfp4"][case % 3]
    Q = rng.choice([1, 16, 40, 64, 128, 128, 200])
    B = rng.randint(1, 6)
    S = rng.choice([1, 31, 32, 33, 400, 1500])
    N = rng.choice([1, 2, 3, 8, 19])
    if fmt == "mxfp4":
        S += S & 1                              # an MXFP4 cache needs batch strides that are multiples of 128 elements
    w = synth.Workload(f"rand_mla_{case}", B=B, Q=Q, K=1, dk=576, dv=512, n_shards=N, scale=1 / math.sqrt(192), seed=7000 + case,
                       seq_len=S, mla=True, fp8=fmt == "e4m3", fp4=fmt == "mxfp4")
    inp = synth.make_inputs(w, "cuda")
    lens = _lens(rng, B, S)
    if fmt != "mxfp4":
        lens = [max(x, 1) for x in lens]        # that helper compares every row (no empty sequences)
    inp.lens = torch.tensor(lens, dtype=torch.int32)
    if fmt == "mxfp4":
        run_mla_mx(hx, oracle, w, inp, N, split_tokens=_split(rng, 32))
        return
    # one fp16 weight per token on the e4m3 latent: 2^-12 of the largest value on a one-hot softmax
    bar = O_MAX_ABS if fmt == "bf16" else max(O_MAX_ABS, 2.0 ** -11 * 6.0)
    run_mla(hx, oracle, w, inp, N, split_tokens=_split(rng, 32), max_abs=bar)
