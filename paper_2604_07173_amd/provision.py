"""Command-line front end of the cache-provisioning calls (Sec. 4.2, Algorithm 1).

    python -m paper_2604_07173_amd.provision --adapters 512 --zipf 1.2 --instances 4 --batch 64

prints the smallest cache capacity M* whose Immediate Admissibility Rate reaches the target,
the rate at a few capacities around it, and the pool memory M* adapters take.  The numbers
come from liblora.so (lora_provision_*); this file only parses arguments and prints.
"""
from __future__ import annotations

import argparse
import json
import sys

from . import binding as L


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--adapters", type=int, default=512, help="N, number of adapters")
    ap.add_argument("--zipf", type=float, default=1.2, help="popularity p_i ~ i^-s (Sec. 6.1 uses s = 1.2)")
    ap.add_argument("--probabilities", help="JSON file with a list of invocation probabilities (overrides --zipf)")
    ap.add_argument("--instances", type=int, default=4, help="L, number of LLM instances")
    ap.add_argument("--batch", type=float, default=64, help="B, batch size per LLM instance")
    ap.add_argument("--alpha", type=float, default=0.95, help="target rate (0.95 for a P95 TTFT target)")
    ap.add_argument("--adapter-bytes", type=int, default=1811939328,
                    help="footprint of one adapter (default: Mixtral-8x7B rank 64, Sec. 2.3)")
    args = ap.parse_args(argv)
    if args.probabilities:
        p = [float(v) for v in json.load(open(args.probabilities))]
    else:
        w = [(i + 1) ** (-args.zipf) for i in range(args.adapters)]
        total = sum(w)
        p = [v / total for v in w]
    LB = args.instances * args.batch
    m_star, rate = L.lora_provision_min_cache(p, LB, args.alpha)
    print(f"N = {len(p)}, LB = {LB:g}, target IAR = {args.alpha:g}")
    print(f"M* = {m_star}  (IAR = {rate:.4f}),  pool memory = "
          f"{L.lora_provision_memory_bytes(m_star, args.adapter_bytes) / 2 ** 30:.1f} GiB")
    for M in sorted({max(1, m_star // 2), max(1, m_star - 1), m_star, min(len(p), 2 * m_star), len(p)}):
        print(f"  IAR({M}) = {L.lora_provision_iar(p, LB, M)[0]:.4f}")
    return 0


if __name__ == "__main__":
    sys.exit(main())
