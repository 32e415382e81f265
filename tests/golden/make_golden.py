"""Writes the stored expected values under tests/golden/ from the CPU oracle alone.

The paper prints no worked values for this path (no attention output, no swap sizes, no waste figures for a
stated input), so nothing here is "the paper's number": these files freeze what the pinned oracle gives on the
seeded tiny inputs, so that a later edit of the oracle's arithmetic shows up as a diff.  Run from the repo root:

    python tests/golden/make_golden.py

Only oracle/ and the seeded input generators are used; nothing here touches the HIP library.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2402_01869_amd import workloads as W  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def hex64(a):
    return [float(x).hex() for x in np.asarray(a, dtype=np.float64).ravel()]


def tiny_attention():
    """Tiny config (Sections 3.1, 4.2): first and last row of every sequence, all heads, dims 0..7, exact fp64 hex."""
    batch = W.make_batch(W.TINY)
    pool, q = W.make_host_inputs(batch, W.TINY.seed, poison_unused=True)
    out = oracle.attn_batch(batch, pool, q)
    lines = ["# oracle.attn_batch on workloads.TINY (seed %d); per line: sequence, row in span, head, then dims 0..7" % W.TINY.seed]
    for s in range(batch.num_seqs):
        for i in sorted({0, int(batch.q_len[s]) - 1}):
            for h in range(batch.num_heads):
                lines.append("%d %d %d " % (s, i, h) + " ".join(hex64(out[batch.q_start[s] + i, h, :8])))
    return "\n".join(lines) + "\n"


def model_values():
    """Section 4.1 swap limit, Eq. 1-5 and the saturation point on fixed inputs."""
    t = oracle.TfwdTable([256, 512, 1024, 2048, 4096], [0.010, 0.022, 0.050, 0.120, 0.300])
    M, C, Co = 819200.0, 1536.0, 90000.0
    rows = [
        ("swap_limit_tokens(0.030 s, 32e9 B/s, 819200 B)", oracle.swap_limit_tokens(0.030, 32e9, 819200)),
        ("swap_limit_tokens(0.001097 s, 55.4e9 B/s, 20480 B)", oracle.swap_limit_tokens(0.001097, 55.4e9, 20480)),
        ("tfwd(1536)", oracle.tfwd(t, C).hex()),
        ("waste_discard", oracle.waste_discard(t, C, Co, M).hex()),
        ("waste_chunked_discard n=3", oracle.waste_chunked_discard(t, C, Co, M, 3).hex()),
        ("waste_preserve T_int=2.5", oracle.waste_preserve(2.5, C, M).hex()),
        ("waste_swap T_swap=0.04", oracle.waste_swap(0.04, C + Co, M).hex()),
        ("chunk_tokens(S=640, running=128)", oracle.chunk_tokens(640, 128)),
        ("chunk_count(1536, 512)", oracle.chunk_count(1536, 512)),
        ("saturation_point", oracle.saturation_point([64, 128, 256, 384, 480, 512, 768, 1024], np.maximum(1e-3, 2e-6 * np.array([64, 128, 256, 384, 480, 512, 768, 1024.0])))),
        ("swap_schedule(10 blocks, 16, [40,16,15,100,100])", list(map(int, oracle.swap_schedule(10, 16, [40, 16, 15, 100, 100])[1]))),
    ]
    return "\n".join("%s = %s" % r for r in rows) + "\n"


FILES = {"tiny_attention_oracle.txt": tiny_attention, "scheduler_model_oracle.txt": model_values}

if __name__ == "__main__":
    for name, fn in FILES.items():
        with open(os.path.join(HERE, name), "w") as f:
            f.write(fn())
        print("wrote", name)
