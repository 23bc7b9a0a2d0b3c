"""CPU fp64 oracle for the attention phase of Helix Parallelism (Sec. 2.1.1, Fig. 4 top, Sec. 2.2).

TEST INFRASTRUCTURE ONLY: tests/, ``__graft_entry__.smoke()`` and bench.py's ``cpu_baseline`` leg
may import this package; the product (``paper_2507_07120_amd``) never does, and this package never
imports the product.  It shares no arithmetic with the HIP library.

Functions
---------
attention        softmax attention of the decode query over the unsharded cache, or over a token
                 range of it (one KVP rank's shard); the textbook definition in fp64, in C.
combine          the rescale-and-sum of N shard partials by their log-sum-exp (Sec. 2.1.1).
argmax_f32       which shard holds the largest stored fp32 LSE (integer bookkeeping).
shard_layout     how a sequence of L tokens is cut into N contiguous KVP shards.
round_robin_owner  which KVP rank stores decode token t under staggered appends (Sec. 2.3).
kv_read_seconds  Appendix A's KV-cache read-time formula.
e4m3_value       OCP E4M3 code -> value, from the format definition.
e2m1_value, e8m0_value   OCP microscaling FP4 element and shared scale codes -> values.

Inputs are the exact stored bits: bf16 as uint16 arrays, e4m3 as uint8 arrays plus fp32 scales.
"""
import ctypes
import math
import os

import numpy as np

from . import build as _build

KV_BF16 = 0
KV_FP8_E4M3 = 1
KV_MXFP4 = 2

_lib = None


class _Problem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Q", ctypes.c_int32), ("K", ctypes.c_int32),
        ("dk", ctypes.c_int32), ("dv", ctypes.c_int32),
        ("v_aliases_k", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
        ("scale", ctypes.c_double),
        ("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
        ("k_sb", ctypes.c_int64), ("k_sh", ctypes.c_int64), ("k_st", ctypes.c_int64),
        ("v_sb", ctypes.c_int64), ("v_sh", ctypes.c_int64), ("v_st", ctypes.c_int64),
        ("kv_scale", ctypes.c_void_p),
        ("s_sb", ctypes.c_int64), ("s_sh", ctypes.c_int64),
        ("tok_off", ctypes.c_void_p), ("len", ctypes.c_void_p),
        ("k_mx", ctypes.c_void_p), ("v_mx", ctypes.c_void_p),
    ]


def lib():
    global _lib
    if _lib is None:
        # HELIX_ORACLE_LIB: another build of the same source (the sanitizer job loads an instrumented one)
        _lib = ctypes.CDLL(os.environ.get("HELIX_ORACLE_LIB") or _build.build())
        _lib.helix_oracle_e4m3_value.restype = ctypes.c_double
        _lib.helix_oracle_e4m3_value.argtypes = [ctypes.c_uint8]
        for name in ("helix_oracle_e2m1_value", "helix_oracle_e8m0_value"):
            getattr(_lib, name).restype = ctypes.c_double
            getattr(_lib, name).argtypes = [ctypes.c_uint8]
        _lib.helix_oracle_attention.restype = ctypes.c_int
        _lib.helix_oracle_combine.restype = ctypes.c_int
        _lib.helix_oracle_argmax_f32.restype = ctypes.c_int
        _lib.helix_oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    """Threads the C oracle will use (OpenMP)."""
    return lib().helix_oracle_threads()


def e4m3_value(code: int) -> float:
    return lib().helix_oracle_e4m3_value(int(code) & 0xFF)


def e2m1_value(code: int) -> float:
    """OCP microscaling FP4 element (E2M1) code 0..15 -> value."""
    return lib().helix_oracle_e2m1_value(int(code) & 0xF)


def e8m0_value(code: int) -> float:
    """OCP microscaling shared scale (E8M0) code -> 2^(code-127), NaN for 255."""
    return lib().helix_oracle_e8m0_value(int(code) & 0xFF)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def attention(q, k, v, lens, scale, *, kv_heads, dv=None, kv_scale=None, tok_off=None,
              t_lo=None, t_hi=None, rows=None, mx=None):
    """Exact softmax attention of one decode query per sequence.

    q         uint16 [B,Q,dk]   bf16 bits
    k         uint16/uint8 [B,K,T,dk] (or [T,dk] rows addressed through tok_off with B-stride 0; MXFP4
              codes: half as many bytes in the last axis)
    v         same layout with dv columns, or None: the value is the first ``dv`` entries of the
              key row (MLA latent)
    lens      int32 [B]  tokens of sequence b
    kv_scale  float32 [B,K,T] (or [T]) per-token dequantisation factor (uint8 = e4m3 input only)
    tok_off   int64 [B] row of sequence b's first token (ragged packed storage), or None
    t_lo,t_hi int64 [B] restrict to tokens [t_lo,t_hi) -- one shard; None = whole sequence
    rows      optional list of (b,h) pairs to evaluate instead of all B*Q rows
    mx        (k_mx, v_mx) uint8 E8M0 scales [B,K,T,dk/32], [B,K,T,dv/32]: k, v are then MXFP4 codes,
              uint8 [B,K,T,dk/2] and [B,K,T,dv/2], two E2M1 elements per byte (even element low nibble)

    Returns (o float64 [B,Q,dv] or [n_rows,dv], lse float64 [B,Q] or [n_rows]).
    """
    q = np.ascontiguousarray(q)
    assert q.dtype == np.uint16 and q.ndim == 3
    B, Q, dk = q.shape
    K = int(kv_heads)
    fp4 = mx is not None
    fp8 = k.dtype == np.uint8 and not fp4
    assert k.dtype in (np.uint16, np.uint8)
    assert k.flags.c_contiguous
    packed = k.ndim == 2
    epb = 2 if fp4 else 1                                  # elements per stored unit
    if packed:
        assert tok_off is not None and K == 1 and k.shape[1] * epb == dk
        k_sb, k_sh, k_st = 0, 0, dk
    else:
        assert k.ndim == 4 and k.shape[0] == B and k.shape[1] == K and k.shape[3] * epb == dk
        k_sb, k_sh, k_st = K * k.shape[2] * dk, k.shape[2] * dk, dk
    alias = v is None
    if alias:
        assert dv is not None and dv <= dk
        v_sb = v_sh = v_st = 0
    else:
        assert v.dtype == k.dtype and v.flags.c_contiguous and v.ndim == k.ndim
        dv = v.shape[-1] * epb
        if packed:
            v_sb, v_sh, v_st = 0, 0, dv
        else:
            v_sb, v_sh, v_st = K * v.shape[2] * dv, v.shape[2] * dv, dv
    s_sb = s_sh = 0
    if fp8:
        assert kv_scale is not None and kv_scale.dtype == np.float32 and kv_scale.flags.c_contiguous
        if not packed:
            assert kv_scale.shape == (B, K, k.shape[2])
            s_sb, s_sh = K * k.shape[2], k.shape[2]
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    assert lens.shape == (B,)
    tok_off_a = None if tok_off is None else np.ascontiguousarray(tok_off, dtype=np.int64)
    t_lo_a = None if t_lo is None else np.ascontiguousarray(t_lo, dtype=np.int64)
    t_hi_a = None if t_hi is None else np.ascontiguousarray(t_hi, dtype=np.int64)

    k_mx = v_mx = None
    if fp4:
        assert k.dtype == np.uint8 and dk % 32 == 0 and dv % 32 == 0
        k_mx, v_mx = mx
        assert k_mx.dtype == np.uint8 and k_mx.flags.c_contiguous and k_mx.shape == k.shape[:-1] + (dk // 32,)
        if not alias:
            assert v_mx.dtype == np.uint8 and v_mx.flags.c_contiguous and v_mx.shape == v.shape[:-1] + (dv // 32,)

    p = _Problem(B, Q, K, dk, dv, int(alias), KV_MXFP4 if fp4 else KV_FP8_E4M3 if fp8 else KV_BF16, float(scale),
                 _ptr(q), _ptr(k), _ptr(v), k_sb, k_sh, k_st, v_sb, v_sh, v_st,
                 _ptr(kv_scale) if fp8 else None, s_sb, s_sh, _ptr(tok_off_a), _ptr(lens),
                 _ptr(k_mx), _ptr(v_mx))
    if rows is None:
        n_rows, rb, rh = 0, None, None
        o = np.empty((B, Q, dv), dtype=np.float64)
        lse = np.empty((B, Q), dtype=np.float64)
    else:
        rb = np.ascontiguousarray([r[0] for r in rows], dtype=np.int32)
        rh = np.ascontiguousarray([r[1] for r in rows], dtype=np.int32)
        n_rows = len(rows)
        o = np.empty((n_rows, dv), dtype=np.float64)
        lse = np.empty((n_rows,), dtype=np.float64)
    rc = lib().helix_oracle_attention(ctypes.byref(p), _ptr(t_lo_a), _ptr(t_hi_a),
                                      ctypes.c_int32(n_rows), _ptr(rb), _ptr(rh), _ptr(o), _ptr(lse))
    if rc != 0:
        raise ValueError("helix_oracle_attention rejected its arguments")
    return o, lse


def combine(o_parts, lse_parts):
    """LSE rescale-and-sum of N shard partials.  o_parts float64 [N,...,dv], lse_parts [N,...].

    Returns (o [...,dv], lse [...])."""
    o_parts = np.ascontiguousarray(o_parts, dtype=np.float64)
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    N = o_parts.shape[0]
    dv = o_parts.shape[-1]
    lead = o_parts.shape[1:-1]
    assert lse_parts.shape == (N,) + lead
    R = int(np.prod(lead, dtype=np.int64)) if lead else 1
    o = np.empty(lead + (dv,), dtype=np.float64)
    lse = np.empty(lead, dtype=np.float64)
    rc = lib().helix_oracle_combine(ctypes.c_int32(N), ctypes.c_int64(R), ctypes.c_int32(dv),
                                    _ptr(o_parts), _ptr(lse_parts), _ptr(o), _ptr(lse))
    if rc != 0:
        raise ValueError("helix_oracle_combine rejected its arguments")
    return o, lse


def argmax_f32(lse_parts):
    """Lowest shard index holding the largest stored fp32 LSE; lse_parts float32 [N,...]."""
    lse_parts = np.ascontiguousarray(lse_parts)
    assert lse_parts.dtype == np.float32
    N = lse_parts.shape[0]
    lead = lse_parts.shape[1:]
    R = int(np.prod(lead, dtype=np.int64)) if lead else 1
    out = np.empty(lead, dtype=np.int32)
    rc = lib().helix_oracle_argmax_f32(ctypes.c_int32(N), ctypes.c_int64(R), _ptr(lse_parts), _ptr(out))
    if rc != 0:
        raise ValueError("helix_oracle_argmax_f32 rejected its arguments")
    return out


SHARD_GRANULE = 16  # tokens; the block size of the staggered appends in Sec. 2.3


def shard_layout(lens, n_shards):
    """Contiguous KVP sharding of each sequence (Sec. 2.1.1: every rank holds an S/KVP slice).

    The paper cuts S into equal slices and is silent on lengths N does not divide.  Reading used
    here: slice width c_b = 16 * ceil(ceil(L_b / N) / 16) (whole 16-token blocks, the granule of
    Sec. 2.3), shard i = [min(i*c_b, L_b), min((i+1)*c_b, L_b)), so tail shards may be short or
    empty.  Returns (off int64 [N,B], length int32 [N,B]).
    """
    lens = [int(x) for x in np.asarray(lens).reshape(-1)]
    N = int(n_shards)
    off = np.zeros((N, len(lens)), dtype=np.int64)
    ln = np.zeros((N, len(lens)), dtype=np.int32)
    for b, L in enumerate(lens):
        per = -(-L // N)
        c = SHARD_GRANULE * (-(-per // SHARD_GRANULE))
        for i in range(N):
            lo = min(i * c, L)
            hi = min((i + 1) * c, L)
            off[i, b] = lo
            ln[i, b] = hi - lo
    return off, ln


def round_robin_owner(t, n_ranks, block=SHARD_GRANULE):
    """KVP rank that stores the t-th decode token (t = 0 is the first token after prefill):
    ``block`` consecutive tokens go to rank 0, the next ``block`` to rank 1, ... (Sec. 2.3)."""
    return (int(t) // int(block)) % int(n_ranks)


def kv_read_seconds(B, K, Hsz, S, bytes_param, mem_bw, TPA=1, KVP=1):
    """Appendix A, first formula: time to read one layer's KV cache,
    B * 2 * ceil(K/TPA) * Hsz * (S/KVP) * bytes_param / MemBW."""
    return B * 2 * math.ceil(K / TPA) * Hsz * (S / KVP) * bytes_param / mem_bw


def hopb_span(n_requests, t_attn, t_comm, pipelined):
    """Fig. 3's timeline.  Without HOP-B all requests finish attention, then all exchange:
    n*t_attn + n*t_comm.  With HOP-B request i's exchange runs under request i+1's attention, a
    two-stage pipeline: the first attention, then n-1 steps bounded by the slower stage, then the
    last exchange."""
    if not pipelined:
        return n_requests * t_attn + n_requests * t_comm
    return t_attn + (n_requests - 1) * max(t_attn, t_comm) + t_comm


def weight_read_seconds(H, Q, K, Hsz, F, bytes_param, mem_bw, TPA=1, TPF=1):
    """Appendix A, second formula: time to read one layer's weights (SwiGLU FFN),
    (2*H*(Q/TPA)*Hsz + 2*H*ceil(K/TPA)*Hsz + 3*H*F/TPF) * bytes_param / MemBW."""
    return (2 * H * (Q / TPA) * Hsz + 2 * H * math.ceil(K / TPA) * Hsz + 3 * (H * F / TPF)) * bytes_param / mem_bw
