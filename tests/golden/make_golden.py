"""Writes tests/golden/tiny_oracle.txt: the fp64 oracle's result on the 'tiny' workload
(batch 4, 8 query / 2 KV heads, head_dim 128, KV lengths 17/64/100/256, seed 0).

The paper prints no worked numeric example of attention, so this fixture is not a paper value:
it is written by this script, which calls only the CPU oracle and the seeded input generator,
and guards both against silent drift.  Run:  python tests/golden/make_golden.py
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))

import oracle  # noqa: E402
import workloads  # noqa: E402


def main():
    w = workloads.CONFIGS["tiny"]
    q = w.make_q()
    ks, vs = w.make_kv()
    out, lse = oracle.attn(q, ks, vs, w.kv_lens(), w.scale)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.txt")
    with open(path, "w") as f:
        f.write("# fp64 oracle on workload 'tiny' (seed 0); written by tests/golden/make_golden.py\n")
        f.write("# lse b t h value\n")
        for b in range(w.batch):
            for h in range(w.n_q_heads):
                f.write("lse %d 0 %d %.17g\n" % (b, h, lse[b, 0, h]))
        f.write("# out b t h d value   (every 16th element)\n")
        for b in range(w.batch):
            for h in range(w.n_q_heads):
                for d in range(0, w.head_dim, 16):
                    f.write("out %d 0 %d %d %.17g\n" % (b, h, d, out[b, 0, h, d]))
    print("wrote", path)


if __name__ == "__main__":
    main()
