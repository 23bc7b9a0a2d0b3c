"""ctypes binding of include/helix_attn.h: same names, argument marshalling only.

Tensors are torch tensors on the GPU (torch provides device memory and the current stream); every
step of the path runs inside the library's kernels.
"""
import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

KV_BF16 = 0
KV_FP8_E4M3 = 1
KV_MXFP4 = 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhelix_attn.so")
_lib = None


class HelixError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({helix_status_string(status)})")


class _CProblem(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("q_heads", ctypes.c_int32), ("kv_heads", ctypes.c_int32),
                ("dk", ctypes.c_int32), ("dv", ctypes.c_int32), ("v_aliases_k", ctypes.c_int32),
                ("kv_dtype", ctypes.c_int32), ("scale", ctypes.c_float), ("split_tokens", ctypes.c_int32)]


class _CShard(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("kv_scale", ctypes.c_void_p),
                ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_t", ctypes.c_int64),
                ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_t", ctypes.c_int64),
                ("s_stride_b", ctypes.c_int64), ("s_stride_h", ctypes.c_int64),
                ("tok_off", ctypes.c_void_p), ("len", ctypes.c_void_p), ("max_len", ctypes.c_int32),
                ("k_scale_mx", ctypes.c_void_p), ("v_scale_mx", ctypes.c_void_p),
                ("status", ctypes.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libhelix_attn.so (built by ``paper_2507_07120_amd.build``); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is not built: run `python -m paper_2507_07120_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    # torch (imported above) has already loaded its bundled HIP runtime under the soname this
    # library needs, so both share ONE runtime: torch's stream handles are valid here and
    # torch.cuda.synchronize() covers the library's kernels.  A second copy would break both.
    with open("/proc/self/maps") as f:
        runtimes = {line.split()[-1] for line in f if "libamdhip64" in line}
    if len(runtimes) != 1:
        raise RuntimeError(f"expected exactly one HIP runtime in the process, found {sorted(runtimes)}")
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.helix_status_string.restype = ctypes.c_char_p
    lib.helix_status_string.argtypes = [ctypes.c_int]
    lib.helix_attn_workspace_bytes.restype = ctypes.c_size_t
    lib.helix_attn_workspace_bytes.argtypes = [ctypes.POINTER(_CProblem), i32, i32]
    lib.helix_attn_plan.restype = ctypes.c_int
    lib.helix_attn_plan.argtypes = [ctypes.POINTER(_CProblem), ctypes.POINTER(i32), i32,
                                    ctypes.POINTER(i32), ctypes.POINTER(i64)]
    lib.helix_attn_partial.restype = ctypes.c_int
    lib.helix_attn_partial.argtypes = [ctypes.POINTER(_CProblem), vp, ctypes.POINTER(_CShard), vp, vp,
                                       vp, ctypes.c_size_t, vp]
    lib.helix_attn_combine.restype = ctypes.c_int
    lib.helix_attn_combine.argtypes = [ctypes.POINTER(_CProblem), i32, vp, vp, vp, vp, vp, vp]
    lib.helix_attn_decode.restype = ctypes.c_int
    lib.helix_attn_decode.argtypes = [ctypes.POINTER(_CProblem), vp, ctypes.POINTER(_CShard), i32,
                                      vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.helix_attn_decode_static.restype = ctypes.c_int
    lib.helix_attn_decode_static.argtypes = [ctypes.POINTER(_CProblem), vp, ctypes.POINTER(_CShard), i32, vp, vp, vp]
    lib.helix_attn_decode_kvp.restype = ctypes.c_int
    lib.helix_attn_decode_kvp.argtypes = [ctypes.POINTER(_CProblem), vp, ctypes.POINTER(_CShard), i32,
                                          vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.helix_shard_layout.restype = ctypes.c_int
    lib.helix_shard_layout.argtypes = [vp, vp, i32, i32, vp, vp, vp]
    lib.helix_kv_append_owner.restype = ctypes.c_int32
    lib.helix_kv_append_owner.argtypes = [i64, i32]
    lib.helix_kv_append.restype = ctypes.c_int
    lib.helix_kv_append.argtypes = [ctypes.POINTER(_CProblem), ctypes.POINTER(_CShard), i32, i64, vp, vp, vp, i32, vp, vp]
    lib.helix_kv_append_mxfp4.restype = ctypes.c_int
    lib.helix_kv_append_mxfp4.argtypes = [ctypes.POINTER(_CProblem), ctypes.POINTER(_CShard), i32, i64, vp, vp, vp, vp, i32, vp, vp]
    f64 = ctypes.c_double
    lib.helix_attn_decode_hopb.restype = ctypes.c_int
    lib.helix_attn_decode_hopb.argtypes = [ctypes.POINTER(_CProblem), vp, ctypes.POINTER(_CShard), i32, i32, vp, vp,
                                           vp, vp, vp, vp, vp, ctypes.c_size_t, vp, vp, ctypes.POINTER(vp)]
    lib.helix_attn_hopb_workspace_bytes.restype = ctypes.c_size_t
    lib.helix_attn_hopb_workspace_bytes.argtypes = [ctypes.POINTER(_CProblem), i32, i32, i32]
    lib.helix_hopb_span.restype = f64
    lib.helix_hopb_span.argtypes = [i32, f64, f64, i32]
    lib.helix_kv_read_seconds.restype = f64
    lib.helix_kv_read_seconds.argtypes = [i64, i64, i64, f64, f64, f64, i64, i64]
    lib.helix_weight_read_seconds.restype = f64
    lib.helix_weight_read_seconds.argtypes = [i64, i64, i64, i64, i64, f64, f64, i64, i64]
    lib.helix_attn_decode_kvp_timed.restype = ctypes.c_int
    lib.helix_attn_decode_kvp_timed.argtypes = lib.helix_attn_decode_kvp.argtypes + [vp, vp]
    lib.helix_probe_stream_read.restype = ctypes.c_int
    lib.helix_probe_stream_read.argtypes = [vp, ctypes.c_size_t, i32, i32, vp]
    lib.helix_probe_mfma_lds.restype = ctypes.c_int
    lib.helix_probe_mfma_lds.argtypes = [vp, i32, vp, ctypes.c_size_t, ctypes.POINTER(f64), ctypes.POINTER(f64), vp]
    _lib = lib
    return lib


def helix_status_string(status: int) -> str:
    return load_library().helix_status_string(int(status)).decode()


@dataclass
class Problem:
    """helix_problem: B sequences, Q query heads sharing K KV heads (or one MLA latent)."""
    batch: int
    q_heads: int
    kv_heads: int
    dk: int
    dv: int
    scale: float
    v_aliases_k: bool = False
    kv_dtype: int = KV_BF16
    split_tokens: int = 0

    def c(self) -> _CProblem:
        return _CProblem(self.batch, self.q_heads, self.kv_heads, self.dk, self.dv, int(self.v_aliases_k),
                         self.kv_dtype, self.scale, self.split_tokens)


@dataclass
class KVShard:
    """helix_kv_shard.  ``k``/``v`` are device tensors whose element (b,kh,t,d) sits at
    data_ptr + (b*stride_b + kh*stride_h + (tok_off[b]+t)*stride_t + d) elements."""
    k: torch.Tensor
    v: Optional[torch.Tensor]
    len: torch.Tensor                      # int32 [B] on the device
    max_len: int
    k_strides: Sequence[int]               # (b, h, t) in elements
    v_strides: Sequence[int] = (0, 0, 0)
    kv_scale: Optional[torch.Tensor] = None
    s_strides: Sequence[int] = (0, 0)
    tok_off: Optional[torch.Tensor] = None  # int64 [B] on the device
    k_scale_mx: Optional[torch.Tensor] = None   # MXFP4: uint8 block scales, k / v are uint8 codes and
    v_scale_mx: Optional[torch.Tensor] = None   # the strides count elements (two per byte)
    status: Optional[torch.Tensor] = None       # int32 [1] on the device: HELIX_STATUS_* bits the kernels raise

    @staticmethod
    def from_padded(k: torch.Tensor, v: Optional[torch.Tensor], lens: torch.Tensor, max_len: int,
                    tok_off: Optional[torch.Tensor] = None, kv_scale: Optional[torch.Tensor] = None) -> "KVShard":
        """k [B,K,S,dk] (v [B,K,S,dv] or None for MLA, kv_scale [B,K,S]) possibly strided views."""
        assert k.dim() == 4 and k.stride(3) == 1
        vs = (0, 0, 0)
        if v is not None:
            assert v.dim() == 4 and v.stride(3) == 1
            vs = (v.stride(0), v.stride(1), v.stride(2))
        ss = (0, 0)
        if kv_scale is not None:
            assert kv_scale.dim() == 3 and kv_scale.stride(2) == 1
            ss = (kv_scale.stride(0), kv_scale.stride(1))
        return KVShard(k, v, lens, int(max_len), (k.stride(0), k.stride(1), k.stride(2)), vs, kv_scale, ss, tok_off)

    @staticmethod
    def from_mxfp4(k: torch.Tensor, v: Optional[torch.Tensor], k_mx: torch.Tensor, v_mx: Optional[torch.Tensor], lens: torch.Tensor,
                   max_len: int, tok_off: Optional[torch.Tensor] = None) -> "KVShard":
        """k [B,K,S,dk/2], v [B,K,S,dv/2] uint8 codes, k_mx [B,K,S,dk/32], v_mx [B,K,S,dv/32] uint8 scales,
        all contiguous in their last two axes; strides are handed over in elements.  v and v_mx are None
        for an MLA latent (the value is the first dv entries of the key row), which may also be packed:
        k [rows, dk/2], k_mx [rows, dk/32], sequence b starting at row tok_off[b]."""
        assert (v is None) == (v_mx is None)
        for t, m in ((k, k_mx), (v, v_mx)):
            if t is None:
                continue
            assert t.dtype == torch.uint8 and m.dtype == torch.uint8 and t.dim() == m.dim()
            assert m.is_contiguous() and t.is_contiguous()
            assert m.shape[:-1] == t.shape[:-1] and m.shape[-1] * 16 == t.shape[-1]
        if k.dim() == 2:
            assert v is None and tok_off is not None
            return KVShard(k, None, lens, int(max_len), (0, 0, 2 * k.stride(0)), (0, 0, 0), None, (0, 0), tok_off, k_mx, None)
        assert k.dim() == 4
        v_strides = (0, 0, 0) if v is None else tuple(2 * x for x in (v.stride(0), v.stride(1), v.stride(2)))
        return KVShard(k, v, lens, int(max_len), tuple(2 * x for x in (k.stride(0), k.stride(1), k.stride(2))),
                       v_strides, None, (0, 0), tok_off, k_mx, v_mx)

    @staticmethod
    def from_packed(k: torch.Tensor, lens: torch.Tensor, max_len: int, tok_off: torch.Tensor,
                    kv_scale: Optional[torch.Tensor] = None) -> "KVShard":
        """k [rows, dk] packed token rows of all sequences (single latent head); the value aliases the key."""
        assert k.dim() == 2 and k.stride(1) == 1
        return KVShard(k, None, lens, int(max_len), (0, 0, k.stride(0)), (0, 0, 0), kv_scale, (0, 0), tok_off)

    def c(self) -> _CShard:
        def ptr(t):
            return None if t is None else t.data_ptr()
        assert self.len.dtype == torch.int32 and self.len.is_contiguous()
        if self.tok_off is not None:
            assert self.tok_off.dtype == torch.int64 and self.tok_off.is_contiguous()
        if self.kv_scale is not None:
            assert self.kv_scale.dtype == torch.float32
        if self.status is not None:
            assert self.status.dtype == torch.int32 and self.status.numel() == 1
        return _CShard(ptr(self.k), ptr(self.v), ptr(self.kv_scale), *[int(x) for x in self.k_strides],
                       *[int(x) for x in self.v_strides], *[int(x) for x in self.s_strides],
                       ptr(self.tok_off), ptr(self.len), int(self.max_len), ptr(self.k_scale_mx), ptr(self.v_scale_mx),
                       ptr(self.status))


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _check(status: int, where: str):
    if status != 0:
        raise HelixError(status, where)


def _f32(t: torch.Tensor, shape, name: str):
    assert t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == tuple(shape), \
        f"{name}: expected contiguous float32 {tuple(shape)}, got {t.dtype} {tuple(t.shape)}"


def helix_attn_workspace_bytes(problem: Problem, n_shards: int, max_len: int) -> int:
    p = problem.c()
    return int(load_library().helix_attn_workspace_bytes(ctypes.byref(p), n_shards, max_len))


def helix_attn_plan(problem: Problem, max_lens: Sequence[int]):
    """(split_tokens, workgroups) the library would use; launches nothing."""
    p = problem.c()
    arr = (ctypes.c_int32 * len(max_lens))(*[int(x) for x in max_lens])
    st, wg = ctypes.c_int32(0), ctypes.c_int64(0)
    _check(load_library().helix_attn_plan(ctypes.byref(p), arr, len(max_lens), ctypes.byref(st), ctypes.byref(wg)),
           "helix_attn_plan")
    return st.value, wg.value


def helix_attn_partial(problem: Problem, q: torch.Tensor, shard: KVShard, o_partial: torch.Tensor,
                       lse: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    assert q.dtype == torch.bfloat16 and q.is_contiguous()
    assert tuple(q.shape) == (problem.batch, problem.q_heads, problem.dk)
    _f32(o_partial, (problem.batch, problem.q_heads, problem.dv), "o_partial")
    _f32(lse, (problem.batch, problem.q_heads), "lse")
    p, s = problem.c(), shard.c()
    _check(load_library().helix_attn_partial(ctypes.byref(p), q.data_ptr(), ctypes.byref(s), o_partial.data_ptr(),
                                             lse.data_ptr(), workspace.data_ptr(),
                                             workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "helix_attn_partial")


def helix_attn_combine(problem: Problem, o_partials: torch.Tensor, lses: torch.Tensor, o: torch.Tensor,
                       lse_out: Optional[torch.Tensor] = None, argmax_shard: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    n = o_partials.shape[0]
    _f32(o_partials, (n, problem.batch, problem.q_heads, problem.dv), "o_partials")
    _f32(lses, (n, problem.batch, problem.q_heads), "lses")
    _f32(o, (problem.batch, problem.q_heads, problem.dv), "o")
    if lse_out is not None:
        _f32(lse_out, (problem.batch, problem.q_heads), "lse_out")
    if argmax_shard is not None:
        assert argmax_shard.dtype == torch.int32 and argmax_shard.is_contiguous()
        assert tuple(argmax_shard.shape) == (problem.batch, problem.q_heads)
    p = problem.c()
    _check(load_library().helix_attn_combine(ctypes.byref(p), n, o_partials.data_ptr(), lses.data_ptr(), o.data_ptr(),
                                             None if lse_out is None else lse_out.data_ptr(),
                                             None if argmax_shard is None else argmax_shard.data_ptr(),
                                             _stream_ptr(stream)),
           "helix_attn_combine")


def helix_attn_decode(problem: Problem, q: torch.Tensor, shards: Sequence[KVShard], o: torch.Tensor,
                      workspace: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                      o_partials: Optional[torch.Tensor] = None, lses: Optional[torch.Tensor] = None,
                      stream=None) -> None:
    n = len(shards)
    assert q.dtype == torch.bfloat16 and q.is_contiguous()
    assert tuple(q.shape) == (problem.batch, problem.q_heads, problem.dk)
    _f32(o, (problem.batch, problem.q_heads, problem.dv), "o")
    if lse_out is not None:
        _f32(lse_out, (problem.batch, problem.q_heads), "lse_out")
    if o_partials is not None:
        _f32(o_partials, (n, problem.batch, problem.q_heads, problem.dv), "o_partials")
    if lses is not None:
        _f32(lses, (n, problem.batch, problem.q_heads), "lses")
    p = problem.c()
    arr = (_CShard * n)(*[s.c() for s in shards])
    _check(load_library().helix_attn_decode(ctypes.byref(p), q.data_ptr(), arr, n, o.data_ptr(),
                                            None if lse_out is None else lse_out.data_ptr(),
                                            None if o_partials is None else o_partials.data_ptr(),
                                            None if lses is None else lses.data_ptr(),
                                            workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                            _stream_ptr(stream)),
           "helix_attn_decode")


STATIC_SCRATCH_BYTES = 16 << 20


def helix_attn_decode_static(problem: Problem, q: torch.Tensor, shards: Sequence[KVShard], o: torch.Tensor,
                             lse_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """helix_attn_decode without a workspace argument: the library's static device scratch serves (no allocation)."""
    n = len(shards)
    assert q.dtype == torch.bfloat16 and q.is_contiguous()
    assert tuple(q.shape) == (problem.batch, problem.q_heads, problem.dk)
    _f32(o, (problem.batch, problem.q_heads, problem.dv), "o")
    if lse_out is not None:
        _f32(lse_out, (problem.batch, problem.q_heads), "lse_out")
    p = problem.c()
    arr = (_CShard * n)(*[s.c() for s in shards])
    _check(load_library().helix_attn_decode_static(ctypes.byref(p), q.data_ptr(), arr, n, o.data_ptr(),
                                                   None if lse_out is None else lse_out.data_ptr(),
                                                   _stream_ptr(stream)),
           "helix_attn_decode_static")


def helix_shard_layout(seq_len: torch.Tensor, n_shards: int, shard_off: torch.Tensor, shard_len: torch.Tensor,
                       seq_base: Optional[torch.Tensor] = None, stream=None) -> None:
    B = seq_len.numel()
    assert seq_len.dtype == torch.int32 and seq_len.is_contiguous()
    assert shard_off.dtype == torch.int64 and shard_off.is_contiguous() and tuple(shard_off.shape) == (n_shards, B)
    assert shard_len.dtype == torch.int32 and shard_len.is_contiguous() and tuple(shard_len.shape) == (n_shards, B)
    if seq_base is not None:
        assert seq_base.dtype == torch.int64 and seq_base.is_contiguous() and seq_base.numel() == B
    _check(load_library().helix_shard_layout(seq_len.data_ptr(), None if seq_base is None else seq_base.data_ptr(),
                                             B, n_shards, shard_off.data_ptr(), shard_len.data_ptr(),
                                             _stream_ptr(stream)),
           "helix_shard_layout")


def helix_kv_append_owner(decode_index: int, n_shards: int) -> int:
    return int(load_library().helix_kv_append_owner(int(decode_index), int(n_shards)))


def helix_kv_append(problem: Problem, shards: Sequence[KVShard], decode_index: int, k_new: torch.Tensor,
                    v_new: Optional[torch.Tensor], capacity: int, scale_new: Optional[torch.Tensor] = None,
                    overflow: Optional[torch.Tensor] = None, stream=None) -> None:
    """Appends one decode token per sequence to the round-robin owner shard (its storage and len are written)."""
    n = len(shards)
    assert k_new.is_contiguous() and tuple(k_new.shape) == (problem.batch, problem.kv_heads, problem.dk)
    if v_new is not None:
        assert v_new.is_contiguous() and tuple(v_new.shape) == (problem.batch, problem.kv_heads, problem.dv)
    if scale_new is not None:
        assert scale_new.dtype == torch.float32 and scale_new.is_contiguous()
    if overflow is not None:
        assert overflow.dtype == torch.int32 and overflow.numel() == 1
    p = problem.c()
    arr = (_CShard * n)(*[s.c() for s in shards])
    _check(load_library().helix_kv_append(ctypes.byref(p), arr, n, int(decode_index), k_new.data_ptr(),
                                          None if v_new is None else v_new.data_ptr(),
                                          None if scale_new is None else scale_new.data_ptr(),
                                          int(capacity), None if overflow is None else overflow.data_ptr(),
                                          _stream_ptr(stream)),
           "helix_kv_append")


def helix_kv_append_mxfp4(problem: Problem, shards: Sequence[KVShard], decode_index: int, k_codes: torch.Tensor,
                          v_codes: Optional[torch.Tensor], k_scales: torch.Tensor, v_scales: Optional[torch.Tensor], capacity: int,
                          overflow: Optional[torch.Tensor] = None, stream=None) -> None:
    """helix_kv_append for an MXFP4 cache: code rows [B,K,d/2] and their block scales [B,K,d/32] (uint8);
    v_codes and v_scales are None for an MLA latent."""
    n = len(shards)
    B, K = problem.batch, problem.kv_heads
    for t, shape in ((k_codes, (B, K, problem.dk // 2)), (v_codes, (B, K, problem.dv // 2)),
                     (k_scales, (B, K, problem.dk // 32)), (v_scales, (B, K, problem.dv // 32))):
        assert t is None or (t.dtype == torch.uint8 and t.is_contiguous() and tuple(t.shape) == shape)
    if overflow is not None:
        assert overflow.dtype == torch.int32 and overflow.numel() == 1
    p = problem.c()
    arr = (_CShard * n)(*[s.c() for s in shards])

    def ptr(t):
        return None if t is None else t.data_ptr()
    _check(load_library().helix_kv_append_mxfp4(ctypes.byref(p), arr, n, int(decode_index), ptr(k_codes),
                                                ptr(v_codes), ptr(k_scales), ptr(v_scales),
                                                int(capacity), ptr(overflow), _stream_ptr(stream)),
           "helix_kv_append_mxfp4")


def helix_kv_read_seconds(B: int, K: int, Hsz: int, S: float, bytes_per_param: float, mem_bw: float,
                          TPA: int = 1, KVP: int = 1) -> float:
    """Appendix A: DRAM-read time of one layer's KV cache (host arithmetic in the library)."""
    return float(load_library().helix_kv_read_seconds(B, K, Hsz, float(S), float(bytes_per_param), float(mem_bw), TPA, KVP))


def helix_weight_read_seconds(H: int, Q: int, K: int, Hsz: int, F: int, bytes_per_param: float, mem_bw: float,
                              TPA: int = 1, TPF: int = 1) -> float:
    """Appendix A: DRAM-read time of one layer's weights (host arithmetic in the library)."""
    return float(load_library().helix_weight_read_seconds(H, Q, K, Hsz, F, float(bytes_per_param), float(mem_bw), TPA, TPF))


def helix_hopb_span(n_requests: int, t_attn: float, t_comm: float, pipelined: bool) -> float:
    """Fig. 3's timeline model (host arithmetic in the library)."""
    return float(load_library().helix_hopb_span(int(n_requests), float(t_attn), float(t_comm), int(bool(pipelined))))


def helix_probe_stream_read(buf: torch.Tensor, workgroups: int, nontemporal: bool = True, stream=None) -> int:
    """Enqueues the bare streaming-read probe over ``buf`` (whole 16 KB blocks); returns the bytes it reads."""
    assert buf.is_contiguous()
    nbytes = buf.numel() * buf.element_size() // 16384 * 16384
    _check(load_library().helix_probe_stream_read(buf.data_ptr(), nbytes, int(workgroups), int(bool(nontemporal)),
                                                  _stream_ptr(stream)), "helix_probe_stream_read")
    return nbytes


def helix_probe_mfma_lds(operands: torch.Tensor, iters: int, stream_buf: Optional[torch.Tensor] = None, stream=None):
    """Enqueues the LDS-fed MFMA probe; returns (flops, bytes_read) of the launch."""
    assert operands.is_contiguous() and operands.numel() * operands.element_size() >= 65536
    fl, by = ctypes.c_double(0), ctypes.c_double(0)
    sb, sbytes = (None, 0) if stream_buf is None else (stream_buf.data_ptr(), stream_buf.numel() * stream_buf.element_size())
    _check(load_library().helix_probe_mfma_lds(operands.data_ptr(), int(iters), sb, sbytes, ctypes.byref(fl), ctypes.byref(by),
                                               _stream_ptr(stream)), "helix_probe_mfma_lds")
    return fl.value, by.value


def helix_attn_hopb_workspace_bytes(problem: Problem, n_shards: int, max_len: int, n_groups: int) -> int:
    p = problem.c()
    return int(load_library().helix_attn_hopb_workspace_bytes(ctypes.byref(p), n_shards, max_len, n_groups))


class HopbBuffers:
    """Send / receive fragment buffers and the events of helix_attn_decode_hopb, owned by the caller."""

    def __init__(self, problem: Problem, n_shards: int, n_groups: int, device="cuda"):
        n_o = n_shards * problem.batch * problem.q_heads * problem.dv
        n_l = n_shards * problem.batch * problem.q_heads
        self.send_o, self.recv_o = (torch.empty(n_o, dtype=torch.float32, device=device) for _ in range(2))
        self.send_lse, self.recv_lse = (torch.empty(n_l, dtype=torch.float32, device=device) for _ in range(2))
        self.events = [torch.cuda.Event() for _ in range(n_groups + 1)]
        for e in self.events:                   # torch creates the hipEvent_t lazily, on the first record
            e.record()
        self.n_groups = n_groups


def helix_attn_decode_hopb(problem: Problem, q: torch.Tensor, shards: Sequence[KVShard], o: torch.Tensor,
                           workspace: torch.Tensor, buffers: HopbBuffers, compute_stream, exchange_stream,
                           lse_out: Optional[torch.Tensor] = None) -> None:
    """Sec. 2.1.3 on one GPU: group g's fragments are exchanged and combined on ``exchange_stream`` while
    group g+1's attention runs on ``compute_stream``."""
    n = len(shards)
    assert q.dtype == torch.bfloat16 and q.is_contiguous()
    _f32(o, (problem.batch, problem.q_heads, problem.dv), "o")
    if lse_out is not None:
        _f32(lse_out, (problem.batch, problem.q_heads), "lse_out")
    p = problem.c()
    arr = (_CShard * n)(*[s.c() for s in shards])
    ev = (ctypes.c_void_p * (buffers.n_groups + 1))(*[e.cuda_event for e in buffers.events])
    _check(load_library().helix_attn_decode_hopb(
        ctypes.byref(p), q.data_ptr(), arr, n, buffers.n_groups, o.data_ptr(),
        None if lse_out is None else lse_out.data_ptr(),
        buffers.send_o.data_ptr(), buffers.send_lse.data_ptr(), buffers.recv_o.data_ptr(), buffers.recv_lse.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(),
        _stream_ptr(compute_stream), _stream_ptr(exchange_stream), ev), "helix_attn_decode_hopb")


def helix_attn_decode_kvp(problem: Problem, q: torch.Tensor, cache: KVShard, n_shards: int, o: torch.Tensor,
                          workspace: torch.Tensor, lse_out: Optional[torch.Tensor] = None,
                          o_partials: Optional[torch.Tensor] = None, lses: Optional[torch.Tensor] = None,
                          shard_off: Optional[torch.Tensor] = None, shard_len: Optional[torch.Tensor] = None,
                          stream=None, events=None) -> None:
    """Layout + decode in one call: ``cache`` describes the unsharded cache, the KVP cut happens in the kernel.
    ``events`` = (start, stop) raw hipEvent_t handles: helix_attn_decode_kvp_timed, which records them around
    the streaming attention kernel."""
    assert q.dtype == torch.bfloat16 and q.is_contiguous()
    _f32(o, (problem.batch, problem.q_heads, problem.dv), "o")
    if lse_out is not None:
        _f32(lse_out, (problem.batch, problem.q_heads), "lse_out")
    if o_partials is not None:
        _f32(o_partials, (n_shards, problem.batch, problem.q_heads, problem.dv), "o_partials")
        _f32(lses, (n_shards, problem.batch, problem.q_heads), "lses")
    if shard_off is not None:
        assert shard_off.dtype == torch.int64 and shard_off.is_contiguous() and tuple(shard_off.shape) == (n_shards, problem.batch)
        assert shard_len.dtype == torch.int32 and shard_len.is_contiguous() and tuple(shard_len.shape) == (n_shards, problem.batch)
    p, c = problem.c(), cache.c()

    def ptr(t):
        return None if t is None else t.data_ptr()
    args = (ctypes.byref(p), q.data_ptr(), ctypes.byref(c), int(n_shards), o.data_ptr(),
            ptr(lse_out), ptr(o_partials), ptr(lses), ptr(shard_off), ptr(shard_len),
            workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if events is not None:
        _check(load_library().helix_attn_decode_kvp_timed(*args, events[0], events[1]), "helix_attn_decode_kvp_timed")
    else:
        _check(load_library().helix_attn_decode_kvp(*args), "helix_attn_decode_kvp")
