"""Appendix A as a command-line calculator: DRAM-read time of one layer's KV cache and weights against
TP width, KVP width and context length -- the three panels of Fig. 1 -- for MI355X parameters
(8 TB/s HBM) and a choice of KV precision.  The arithmetic is the library's (helix_kv_read_seconds,
helix_weight_read_seconds); this module only loops and prints.

    python -m paper_2507_07120_amd.roofline --kv-bytes 0.53125        # MXFP4: 0.5 + 1/32 byte per element
"""
import argparse

from . import binding as hx


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--q-heads", type=int, default=128)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--head-size", type=int, default=128)
    ap.add_argument("--ffn", type=int, default=65536)
    ap.add_argument("--seq", type=float, default=float(1 << 20))
    ap.add_argument("--kv-bytes", type=float, default=0.5, help="bytes per KV element (0.5 FP4, 0.53125 MXFP4 with scales, 2 bf16)")
    ap.add_argument("--weight-bytes", type=float, default=0.5)
    ap.add_argument("--mem-bw", type=float, default=8.0e12, help="bytes per second (MI355X: 8.0e12)")
    a = ap.parse_args(argv)
    H = a.q_heads * a.head_size
    kv = lambda S, tpa, kvp: hx.helix_kv_read_seconds(a.batch, a.kv_heads, a.head_size, S, a.kv_bytes, a.mem_bw, tpa, kvp)
    wt = lambda tpa, tpf: hx.helix_weight_read_seconds(H, a.q_heads, a.kv_heads, a.head_size, a.ffn, a.weight_bytes, a.mem_bw, tpa, tpf)
    print(f"B={a.batch} Q={a.q_heads} K={a.kv_heads} Hsz={a.head_size} F={a.ffn} S={a.seq:.0f} MemBW={a.mem_bw / 1e12:.1f} TB/s")
    print("\nread time per layer vs TP width (KVP=1): KV reads stop shrinking at TP = K")
    print(f"{'TP':>4} {'KV us':>10} {'weights us':>11}")
    for tp in (1, 2, 4, 8, 16, 32, 64):
        print(f"{tp:>4} {kv(a.seq, tp, 1) * 1e6:>10.2f} {wt(tp, tp) * 1e6:>11.2f}")
    print("\nKV read time per layer vs context length (TP = K, KVP=1): linear in S")
    print(f"{'S':>10} {'KV us':>10}")
    for s in (1 << 16, 1 << 18, 1 << 20, 1 << 22):
        print(f"{s:>10} {kv(float(s), a.kv_heads, 1) * 1e6:>10.2f}")
    print("\nKV read time per layer vs KVP width (TP = K): 1/KVP")
    print(f"{'KVP':>4} {'KV us':>10}")
    for kvp in (1, 2, 4, 8, 16, 32):
        print(f"{kvp:>4} {kv(a.seq, a.kv_heads, kvp) * 1e6:>10.2f}")


if __name__ == "__main__":
    main()
