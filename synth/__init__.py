"""Seeded synthetic inputs for the Helix decode-attention tests and bench.

Serves both the CPU oracle and the HIP library and contains none of the method's arithmetic: only
random draws, rounding to the storage formats (bf16, e4m3 + per-token scale, MXFP4) and the shapes of
the workloads.  Every value is a pure function of (seed, tag, flat index) through a counter-based
hash, so tensors can be produced chunk by chunk on any torch device.  Transcendentals differ by an
ulp between devices, so a tensor is generated ONCE and its *bits* are handed to both sides.

The paper evaluates Llama-405B (128 query / 8 KV heads, GQA) and DeepSeek-R1 (MLA, 128 query
heads on one latent) at >=1M-token KV lengths in a simulator (Sec. 3): attention cost depends on
shapes only, so i.i.d. N(0,1) tensors of those shapes stand in for real caches.
"""
import math
import os
import sys
from dataclasses import dataclass, field
from typing import Optional

import torch

_M64 = (1 << 64) - 1


def _s64(x: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 tensors (wrapping arithmetic)."""
    x = (x ^ _lsr(x, 30)) * _s64(0xBF58476D1CE4E5B9)
    x = (x ^ _lsr(x, 27)) * _s64(0x94D049BB133111EB)
    return x ^ _lsr(x, 31)


def _key(seed: int, tag: int) -> int:
    return _s64((seed * 0x9E3779B97F4A7C15) ^ (tag * 0xD1B54A32D192ED03) ^ 0x2545F4914F6CDD1D)


def hash_u64(seed: int, tag: int, start: int, count: int, device) -> torch.Tensor:
    """64 random bits for flat indices start..start+count-1 (as int64)."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(_mix(idx * _s64(0x9E3779B97F4A7C15) + _key(seed, tag)))


def normal_f32(seed: int, tag: int, start: int, count: int, device) -> torch.Tensor:
    """N(0,1) draws (Box-Muller on two 24-bit uniforms from one 64-bit hash) as float32."""
    h = hash_u64(seed, tag, start, count, device)
    u1 = ((_lsr(h, 40)).to(torch.float32) + 1.0) * (1.0 / 16777216.0)          # (0,1]
    u2 = ((_lsr(h, 16) & 0xFFFFFF).to(torch.float32)) * (1.0 / 16777216.0)      # [0,1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def uniform_f32(seed: int, tag: int, start: int, count: int, device) -> torch.Tensor:
    h = hash_u64(seed, tag, start, count, device)
    return (_lsr(h, 40)).to(torch.float32) * (1.0 / 16777216.0)                  # [0,1)


_CHUNK = 1 << 26


def _progress(what: str, done: int, total: int) -> None:
    """With HELIX_SYNTH_PROGRESS set, one line per generated chunk on stderr: under a counter-collecting
    profiler the generation of a multi-GB workload takes minutes, and a run that shows no sign of life
    for that long is taken for hung."""
    if os.environ.get("HELIX_SYNTH_PROGRESS"):
        print(f"synth: {what} {done}/{total}", file=sys.stderr, flush=True)


def normal_bf16(seed: int, tag: int, shape, device="cpu") -> torch.Tensor:
    """N(0,1) rounded to nearest-even bf16, shape ``shape``."""
    n = math.prod(shape)
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        out[s:s + c] = normal_f32(seed, tag, s, c, device).to(torch.bfloat16)
        _progress("bf16 elements", s + c, n)
    return out.view(*shape)


def scale_rows_(x: torch.Tensor, seed: int, tag: int, prob: float, factor: float) -> torch.Tensor:
    """In place: each row x[..., :] is multiplied by ``factor`` with probability ``prob``
    (independent per row).  factor a power of two keeps bf16 values exact."""
    rows = x.numel() // x.shape[-1]
    flat = x.view(rows, x.shape[-1])
    for s in range(0, rows, _CHUNK):
        c = min(_CHUNK, rows - s)
        hit = uniform_f32(seed, tag, s, c, x.device) < prob
        flat[s:s + c] = torch.where(hit[:, None], flat[s:s + c] * factor, flat[s:s + c])
    return x


def uniform_lengths(seed: int, tag: int, count: int, lo: int, hi: int) -> torch.Tensor:
    """``count`` integers uniform on [lo, hi] inclusive, int32, on the CPU."""
    h = hash_u64(seed, tag, 0, count, "cpu")
    span = hi - lo + 1
    return (lo + (_lsr(h, 11) % span)).to(torch.int32)


E4M3_MAX = 448.0


def quantize_e4m3_per_token(x: torch.Tensor):
    """Per-row (= per token) symmetric quantisation to OCP e4m3 with one fp32 scale per row:
    scale = max|x| / 448 (1 for an all-zero row), code = round-to-nearest-even(x / scale),
    saturating.  Returns (codes uint8 [..., D], scale float32 [...]).  This is input preparation:
    both the oracle and the GPU consume the codes and scales, never ``x``."""
    xf = x.to(torch.float32)
    amax = xf.abs().amax(dim=-1)
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax))
    y = (xf / scale[..., None]).clamp_(-E4M3_MAX, E4M3_MAX)
    codes = y.to(torch.float8_e4m3fn).view(torch.uint8)
    return codes, scale


def _peaked(x: torch.Tensor, seed: int, first_row: int, prob: float, factor: float) -> torch.Tensor:
    """Rows first_row .. of a chunk, each multiplied by ``factor`` with probability ``prob`` (the draw of row r
    depends on (seed, r) only, as in scale_rows_)."""
    if prob <= 0:
        return x
    hit = uniform_f32(seed, TAG_PEAK, first_row, x.shape[0], x.device) < prob
    return torch.where(hit[:, None], x * factor, x)


def normal_e4m3_rows(seed: int, tag: int, rows: int, dim: int, device="cpu", row_chunk: int = 1 << 17,
                     peak_prob: float = 0.0, peak_factor: float = 1.0):
    """rows x dim N(0,1) values (a fraction peak_prob of the rows times peak_factor) quantised per row to e4m3;
    returns (codes uint8, scale fp32)."""
    codes = torch.empty((rows, dim), dtype=torch.uint8, device=device)
    scale = torch.empty((rows,), dtype=torch.float32, device=device)
    for r in range(0, rows, row_chunk):
        c = min(row_chunk, rows - r)
        x = _peaked(normal_f32(seed, tag, r * dim, c * dim, device).view(c, dim), seed, r, peak_prob, peak_factor)
        codes[r:r + c], scale[r:r + c] = quantize_e4m3_per_token(x)
        _progress("e4m3 rows", r + c, rows)
    return codes, scale


def normal_e4m3_kv_rows(seed: int, tag_k: int, tag_v: int, rows: int, dk: int, dv: int, device="cpu", row_chunk: int = 1 << 17,
                        peak_prob: float = 0.0, peak_factor: float = 1.0):
    """rows x dk key rows and rows x dv value rows of N(0,1) values (a fraction peak_prob of the key rows times
    peak_factor), quantised to e4m3 with ONE scale per row pair -- a token's key row and value row share it, as the
    GQA fp8 cache does; returns (k codes uint8, v codes uint8, scale fp32)."""
    kc = torch.empty((rows, dk), dtype=torch.uint8, device=device)
    vc = torch.empty((rows, dv), dtype=torch.uint8, device=device)
    scale = torch.empty((rows,), dtype=torch.float32, device=device)
    for r in range(0, rows, row_chunk):
        c = min(row_chunk, rows - r)
        xk = _peaked(normal_f32(seed, tag_k, r * dk, c * dk, device).view(c, dk), seed, r, peak_prob, peak_factor)
        xv = normal_f32(seed, tag_v, r * dv, c * dv, device).view(c, dv)
        codes, scale[r:r + c] = quantize_e4m3_per_token(torch.cat([xk, xv], dim=1))
        kc[r:r + c], vc[r:r + c] = codes[:, :dk], codes[:, dk:]
        _progress("e4m3 kv rows", r + c, rows)
    return kc, vc, scale


def quantize_mxfp4(x: torch.Tensor):
    """Rounds rows to the OCP microscaling FP4 format: blocks of 32 consecutive entries of the last
    axis share one E8M0 scale 2^(floor(log2 max|x|) - 2) (2 = exponent of the largest E2M1 value, 6),
    entries become round-to-nearest-even(x / scale) on the E2M1 grid {0, .5, 1, 1.5, 2, 3, 4, 6},
    saturating.  An all-zero block gets scale code 127.  Returns (codes uint8 [..., D/2], two
    entries per byte with the even one in the low nibble; scales uint8 [..., D/32]).  This is input
    preparation: both the oracle and the GPU consume codes and scales, never ``x``."""
    D = x.shape[-1]
    assert D % 32 == 0
    xf = x.to(torch.float32).reshape(*x.shape[:-1], D // 32, 32)
    amax = xf.abs().amax(dim=-1)
    _, e = torch.frexp(amax)                               # amax = m * 2^e, m in [0.5, 1)
    shared = torch.where(amax > 0, e - 1 - 2, torch.zeros_like(e)).clamp_(-127, 127)
    y = torch.ldexp(xf, -shared[..., None])
    a = y.abs()
    q = torch.where(a < 2, torch.round(a * 2) * 0.5, torch.where(a < 4, torch.round(a), torch.round(a * 0.5) * 2))
    q = q.clamp_(max=6.0)
    # magnitude -> code: 0, .5, 1, 1.5 are code = 2*value; 2, 3 -> 4, 5; 4, 6 -> 6, 7
    code = torch.where(q < 2, q * 2, torch.where(q < 4, q + 2, q * 0.5 + 4)).to(torch.uint8)
    code = code | ((y < 0) | ((y == 0) & torch.signbit(y))).to(torch.uint8) * 8
    code = code.reshape(*x.shape[:-1], D // 2, 2)
    packed = code[..., 0] | (code[..., 1] << 4)
    return packed, (shared + 127).to(torch.uint8)


def normal_mxfp4_rows(seed: int, tag: int, rows: int, dim: int, device="cpu", row_chunk: int = 1 << 17,
                      peak_prob: float = 0.0, peak_factor: float = 1.0):
    """rows x dim N(0,1) values (a fraction peak_prob of the rows times peak_factor) in MXFP4; returns (codes uint8
    [rows, dim/2], scales uint8 [rows, dim/32])."""
    codes = torch.empty((rows, dim // 2), dtype=torch.uint8, device=device)
    scales = torch.empty((rows, dim // 32), dtype=torch.uint8, device=device)
    for r in range(0, rows, row_chunk):
        c = min(row_chunk, rows - r)
        x = _peaked(normal_f32(seed, tag, r * dim, c * dim, device).view(c, dim), seed, r, peak_prob, peak_factor)
        codes[r:r + c], scales[r:r + c] = quantize_mxfp4(x)
        _progress("MXFP4 rows", r + c, rows)
    return codes, scales


TAG_Q, TAG_K, TAG_V, TAG_PEAK, TAG_LEN = 1, 2, 3, 4, 5


@dataclass
class Workload:
    """One of the benchmark configurations: shapes, storage format and seed."""
    name: str
    B: int
    Q: int
    K: int
    dk: int
    dv: int
    n_shards: int
    scale: float
    seed: int
    seq_len: Optional[int] = None          # fixed context per sequence (None: ragged)
    len_range: Optional[tuple] = None      # (lo, hi) inclusive for ragged lengths
    mla: bool = False                      # value = first dv entries of the key row
    fp8: bool = False                      # e4m3 codes + per-token fp32 scale
    fp4: bool = False                      # MXFP4: e2m1 codes, one e8m0 scale per 32 entries of a row
    peak_prob: float = 0.0                 # fraction of key rows multiplied by peak_factor
    peak_factor: float = 1.0
    note: str = ""
    extra: dict = field(default_factory=dict)


WORKLOADS = {
    # B=1, 8 query / 2 KV heads, d=64, S=4096 in 4 equal shards
    "tiny_gqa": Workload("tiny_gqa", B=1, Q=8, K=2, dk=64, dv=64, n_shards=4, scale=1 / math.sqrt(64),
                         seed=1001, seq_len=4096),
    # one GPU's share of a Llama-405B-like layer at TPA=8, KVP=8 of a 1M-token context
    "gqa_share": Workload("gqa_share", B=16, Q=16, K=1, dk=128, dv=128, n_shards=1,
                          scale=1 / math.sqrt(128), seed=1002, seq_len=131072),
    # one GPU's share of a DeepSeek-R1-like MLA layer at KVP=8 of a 1M-token context
    "mla_share": Workload("mla_share", B=32, Q=128, K=1, dk=576, dv=512, n_shards=1,
                          scale=1 / math.sqrt(192), seed=1003, seq_len=131072, mla=True),
    # all 16 shards of a 1M-token GQA context on one GPU, with sharp softmax peaks
    "gqa_full": Workload("gqa_full", B=4, Q=64, K=8, dk=128, dv=128, n_shards=16,
                         scale=1 / math.sqrt(128), seed=1004, seq_len=1048576,
                         peak_prob=0.01, peak_factor=8.0),
    # ragged MLA with e4m3 latent + per-token scale, 8 shards with uneven tails
    "mla_fp8_ragged": Workload("mla_fp8_ragged", B=64, Q=128, K=1, dk=576, dv=512, n_shards=8,
                               scale=1 / math.sqrt(192), seed=1005, len_range=(16384, 262144),
                               mla=True, fp8=True),
    # the GQA share with the KV cache in MXFP4 (the precision of the paper's evaluation, Sec. 3) and a
    # 4x longer context, which keeps the cache near 1 GiB: KVP=8 of a 4M-token context
    "gqa_share_mxfp4": Workload("gqa_share_mxfp4", B=16, Q=16, K=1, dk=128, dv=128, n_shards=1,
                                scale=1 / math.sqrt(128), seed=1006, seq_len=524288, fp4=True),
    # the GQA share with the KV cache in e4m3 (one fp32 scale per token for its key and value row) and twice the
    # context, which keeps the cache near 1 GiB: KVP=8 of a 2M-token context
    "gqa_share_fp8": Workload("gqa_share_fp8", B=16, Q=16, K=1, dk=128, dv=128, n_shards=1,
                              scale=1 / math.sqrt(128), seed=1009, seq_len=262144, fp8=True),
    # the MLA share with the latent in MXFP4 (DeepSeek-R1 with FP4 KV states is the paper's second model, Sec. 3)
    "mla_share_mxfp4": Workload("mla_share_mxfp4", B=32, Q=128, K=1, dk=576, dv=512, n_shards=1,
                                scale=1 / math.sqrt(192), seed=1007, seq_len=131072, mla=True, fp4=True),
    # the ragged MLA configuration (same seed: same lengths, same rows before quantisation) with the latent in MXFP4
    "mla_mxfp4_ragged": Workload("mla_mxfp4_ragged", B=64, Q=128, K=1, dk=576, dv=512, n_shards=8,
                                 scale=1 / math.sqrt(192), seed=1005, len_range=(16384, 262144),
                                 mla=True, fp4=True),
    # the MLA configurations with the sharp softmax peaks of the full GQA configuration (1 % of the latent rows
    # times 8 before quantisation): the scores of those rows stand 60 octaves and more above the rest
    "mla_share_peaked": Workload("mla_share_peaked", B=32, Q=128, K=1, dk=576, dv=512, n_shards=1,
                                 scale=1 / math.sqrt(192), seed=1003, seq_len=131072, mla=True,
                                 peak_prob=0.01, peak_factor=8.0),
    "mla_fp8_peaked": Workload("mla_fp8_peaked", B=64, Q=128, K=1, dk=576, dv=512, n_shards=8,
                               scale=1 / math.sqrt(192), seed=1005, len_range=(16384, 262144),
                               mla=True, fp8=True, peak_prob=0.01, peak_factor=8.0),
    "mla_mxfp4_peaked": Workload("mla_mxfp4_peaked", B=64, Q=128, K=1, dk=576, dv=512, n_shards=8,
                                 scale=1 / math.sqrt(192), seed=1005, len_range=(16384, 262144),
                                 mla=True, fp4=True, peak_prob=0.01, peak_factor=8.0),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of ``w`` with some fields replaced (reduced sizes for element-wise parity)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


@dataclass
class Inputs:
    """Tensors of one workload.  Padded layout: k [B,K,S,dk], v [B,K,S,dv] (None for MLA).
    Ragged layout (len_range): k [sum L_b, dk] packed, seq_off int64 [B+1]; kv_scale [sum L_b]
    (MXFP4: k [sum L_b, dk/2] codes, k_mx [sum L_b, dk/32])."""
    w: Workload
    q: torch.Tensor
    k: torch.Tensor
    v: Optional[torch.Tensor]
    kv_scale: Optional[torch.Tensor]
    lens: torch.Tensor                      # int32 [B], CPU
    seq_off: Optional[torch.Tensor]         # int64 [B+1], CPU (ragged only)
    k_mx: Optional[torch.Tensor] = None     # MXFP4 only: uint8 [B,K,S,dk/32] block scales (k, v are uint8 codes)
    v_mx: Optional[torch.Tensor] = None


def make_inputs(w: Workload, device="cpu") -> Inputs:
    q = normal_bf16(w.seed, TAG_Q, (w.B, w.Q, w.dk), device)
    if w.len_range is not None:
        lens = uniform_lengths(w.seed, TAG_LEN, w.B, w.len_range[0], w.len_range[1])
        seq_off = torch.zeros(w.B + 1, dtype=torch.int64)
        seq_off[1:] = torch.cumsum(lens.to(torch.int64), 0)
        rows = int(seq_off[-1])
        assert w.K == 1 and w.mla, "ragged packed storage is defined for the single-latent case"
        if w.fp4:
            assert not w.fp8
            kc, ks = normal_mxfp4_rows(w.seed, TAG_K, rows, w.dk, device, peak_prob=w.peak_prob, peak_factor=w.peak_factor)
            return Inputs(w, q, kc, None, None, lens, seq_off, ks, None)
        if w.fp8:
            k, kv_scale = normal_e4m3_rows(w.seed, TAG_K, rows, w.dk, device, peak_prob=w.peak_prob, peak_factor=w.peak_factor)
        else:
            k, kv_scale = normal_bf16(w.seed, TAG_K, (rows, w.dk), device), None
            if w.peak_prob > 0:
                scale_rows_(k, w.seed, TAG_PEAK, w.peak_prob, w.peak_factor)
        return Inputs(w, q, k, None, kv_scale, lens, seq_off)
    S = w.seq_len
    lens = torch.full((w.B,), S, dtype=torch.int32)
    kv_scale = None
    if w.fp4 and w.mla:
        # one MXFP4 latent per token: 576 codes (288 bytes) + 18 block scales; the value aliases its first 512 entries
        assert not w.fp8 and w.K == 1
        kc, ks = normal_mxfp4_rows(w.seed, TAG_K, w.B * S, w.dk, device, peak_prob=w.peak_prob, peak_factor=w.peak_factor)
        return Inputs(w, q, kc.view(w.B, 1, S, w.dk // 2), None, None, lens, None, ks.view(w.B, 1, S, w.dk // 32), None)
    if w.fp4:
        assert not w.fp8
        kc, ks = normal_mxfp4_rows(w.seed, TAG_K, w.B * w.K * S, w.dk, device)
        vc, vs = normal_mxfp4_rows(w.seed, TAG_V, w.B * w.K * S, w.dv, device)
        return Inputs(w, q, kc.view(w.B, w.K, S, w.dk // 2), vc.view(w.B, w.K, S, w.dv // 2), None, lens, None,
                      ks.view(w.B, w.K, S, w.dk // 32), vs.view(w.B, w.K, S, w.dv // 32))
    if w.fp8 and not w.mla:
        # GQA fp8 cache: separate key and value rows, one scale per (sequence, kv head, token) for both
        kc, vc, sc = normal_e4m3_kv_rows(w.seed, TAG_K, TAG_V, w.B * w.K * S, w.dk, w.dv, device, peak_prob=w.peak_prob, peak_factor=w.peak_factor)
        return Inputs(w, q, kc.view(w.B, w.K, S, w.dk), vc.view(w.B, w.K, S, w.dv), sc.view(w.B, w.K, S), lens, None)
    if w.fp8:
        codes, sc = normal_e4m3_rows(w.seed, TAG_K, w.B * w.K * S, w.dk, device, peak_prob=w.peak_prob, peak_factor=w.peak_factor)
        k, kv_scale = codes.view(w.B, w.K, S, w.dk), sc.view(w.B, w.K, S)
    else:
        k = normal_bf16(w.seed, TAG_K, (w.B, w.K, S, w.dk), device)
        if w.peak_prob > 0:
            scale_rows_(k, w.seed, TAG_PEAK, w.peak_prob, w.peak_factor)
    v = None
    if not w.mla:
        v = normal_bf16(w.seed, TAG_V, (w.B, w.K, S, w.dv), device)
    return Inputs(w, q, k, v, kv_scale, lens, None)


def bits(t: Optional[torch.Tensor]):
    """The stored bits of a tensor as a numpy array on the host (bf16 -> uint16, e4m3 -> uint8)."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    return t.numpy()
