"""Glue for tests, the smoke check and the bench: turns tensors of one workload into the
library's shard descriptors.  Holds no arithmetic of the method: the KVP cut itself comes from
``helix_shard_layout`` (a device kernel of the library)."""
from typing import List, Optional

import torch

from . import binding as hx


def problem_for(w, split_tokens: int = 0) -> hx.Problem:
    """helix_problem of a synth.Workload-like object (B, Q, K, dk, dv, scale, mla, fp8)."""
    return hx.Problem(batch=w.B, q_heads=w.Q, kv_heads=w.K, dk=w.dk, dv=w.dv, scale=float(w.scale),
                      v_aliases_k=bool(w.mla),
                      kv_dtype=hx.KV_MXFP4 if getattr(w, "fp4", False) else hx.KV_FP8_E4M3 if w.fp8 else hx.KV_BF16,
                      split_tokens=split_tokens)


class ShardSet:
    """N shard descriptors over one cache, plus the device integer metadata they point into."""

    def __init__(self, shards: List[hx.KVShard], shard_off: torch.Tensor, shard_len: torch.Tensor, max_lens: List[int]):
        self.shards = shards
        self.shard_off = shard_off      # int64 [N,B] device (includes seq_base for packed storage)
        self.shard_len = shard_len      # int32 [N,B] device
        self.max_lens = max_lens


def make_shards(k: torch.Tensor, v: Optional[torch.Tensor], lens_dev: torch.Tensor, n_shards: int,
                kv_scale: Optional[torch.Tensor] = None, seq_base: Optional[torch.Tensor] = None,
                mx=None) -> ShardSet:
    """Cuts every sequence into ``n_shards`` KVP slices with the library's layout kernel and wraps
    each slice as a view (tok_off) into the unsharded tensors.

    Padded storage: k [B,K,S,dk], v [B,K,S,dv] or None (MLA), kv_scale [B,K,S].
    Packed storage: k [rows,dk], seq_base int64 [B] = first row of each sequence, kv_scale [rows].
    MXFP4: k, v uint8 codes [B,K,S,d/2] and mx = (k_mx, v_mx) uint8 block scales [B,K,S,d/32].
    """
    B = lens_dev.numel()
    dev = lens_dev.device
    shard_off = torch.empty((n_shards, B), dtype=torch.int64, device=dev)
    shard_len = torch.empty((n_shards, B), dtype=torch.int32, device=dev)
    hx.helix_shard_layout(lens_dev, n_shards, shard_off, shard_len, seq_base=seq_base)
    max_lens = shard_len.max(dim=1).values.cpu().tolist()      # harness-side sync, not in the library
    shards = []
    for i in range(n_shards):
        if mx is not None:
            s = hx.KVShard.from_mxfp4(k, v, mx[0], mx[1], shard_len[i], max_lens[i], tok_off=shard_off[i])
        elif k.dim() == 2:
            s = hx.KVShard.from_packed(k, shard_len[i], max_lens[i], shard_off[i], kv_scale=kv_scale)
        else:
            s = hx.KVShard.from_padded(k, v, shard_len[i], max_lens[i], tok_off=shard_off[i], kv_scale=kv_scale)
        shards.append(s)
    return ShardSet(shards, shard_off, shard_len, max_lens)


def workspace_for(problem: hx.Problem, n_shards: int, max_len: int, device) -> torch.Tensor:
    nbytes = hx.helix_attn_workspace_bytes(problem, n_shards, max_len)
    if nbytes == 0:
        raise hx.HelixError(3, "helix_attn_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)
