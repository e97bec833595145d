"""Writes tests/golden/lengths_seeded.txt from the seeded input generators."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from paper_2603_10342_amd import inputs as I  # noqa: E402


def lines():
    rng = I.rng_for(I.config_seed(2), 0)
    ctx = I.uniform_lens(rng, 1024, 4096, 64)
    bt = I.deal_block_tables(rng, ctx, 16, 32768)
    yield "config2 ctx_lens " + " ".join(map(str, ctx))
    yield "config2 bt_row0_first8 " + " ".join(map(str, bt[0, :8]))
    rng = I.rng_for(I.config_seed(4), 0)
    p = I.uniform_lens(rng, 2048, 8192, 32)
    n = I.uniform_lens(rng, 128, 1024, 32)
    yield "config4 prefix_lens " + " ".join(map(str, p))
    yield "config4 new_lens " + " ".join(map(str, n))
    rng = I.rng_for(I.config_seed(5), 0)
    yield "config5 decode_ctx_lens " + " ".join(map(str, I.uniform_lens(rng, 1024, 8192, 64)))


if __name__ == "__main__":
    with open(os.path.join(HERE, "lengths_seeded.txt"), "w") as f:
        f.write("\n".join(lines()) + "\n")
