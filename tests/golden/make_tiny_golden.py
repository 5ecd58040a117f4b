"""Writes tests/golden/tiny_seed0.txt: sampled oracle outputs of the tiny configuration.

Calls only the input generator and the CPU oracle.  The file is a regression pin for the
oracle (the paper prints no worked numeric example of a layer); it is never produced from, or
compared by construction with, the HIP library.

    python tests/golden/make_tiny_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2504_14775_amd import synth  # noqa: E402


def main():
    shape = synth.SHAPES["tiny"]
    w = [{k: synth.bf16_bits(v) for k, v in synth.make_layer_weights(shape, 0, l).items()}
         for l in range(shape.num_layers)]
    batch = synth.make_batch("tiny", seed=0)
    x = synth.bf16_bits(synth.make_hidden(shape, 0, batch.num_tokens))
    k, v = synth.make_pool(shape, 0, batch.num_blocks)
    kp, vp = synth.bf16_bits(k).copy(), synth.bf16_bits(v).copy()
    out, _ = oracle.stage_forward(shape, w, batch.new_tokens, batch.cached_len, batch.block_tables,
                                  batch.num_blocks, kp, vp, x)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_seed0.txt")
    with open(path, "w") as f:
        f.write("# tiny configuration, seed 0: row, column, oracle residual-stream output (float64)\n")
        f.write("# written by tests/golden/make_tiny_golden.py from oracle/ only\n")
        for t in (0, 17, 31, 32, 47, 48, 49, 50, 51):
            for j in (0, 1, 127, 255):
                f.write(f"{t} {j} {out[t, j]:.17g}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
