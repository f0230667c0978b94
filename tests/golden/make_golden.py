"""Writes the stored expected values under tests/golden/ from the fp64 oracle alone.

The paper prints no worked numerical example of the decoder, so nothing here is a value of the paper's: the
fixture freezes what the pinned oracle computes today on seeded inputs, so that a later change to the
oracle's arithmetic shows up as a diff of this file (and has to be justified).  Run from the repository root:
    python tests/golden/make_golden.py
Calls only oracle/ and the shared input generators.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import ref                      # noqa: E402
from paper_2602_00608_amd import synth      # noqa: E402

CHANS = (512, 128, 64, 32)


def reduced_decoder_samples():
    """A narrower, shallower decoder (the topology of Sec. IV-B-1's fused chain, reduced) on a 7x9 latent."""
    spec = synth.decoder_weight_spec(level_channels=CHANS, resblocks_per_level=2)
    weights = synth.draw_params(spec, synth.weight_seed(9), random_affine=True)
    z = synth.latent_sequence(workload=9, frames=1, h=7, w=9)
    out = ref.decoder(z, weights, level_channels=CHANS, resblocks_per_level=2, groups=32, eps=1e-6)
    flat = out.reshape(-1)
    idx = np.linspace(0, flat.size - 1, 48).astype(np.int64)
    return out.shape, idx, flat[idx], float(np.sqrt(np.mean(flat ** 2)))


def main():
    shape, idx, vals, rms = reduced_decoder_samples()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "reduced_decoder_f64.txt")
    with open(path, "w") as f:
        f.write("# fp64 oracle, reduced decoder (channels 512/128/64/32, 2 ResBlocks per level, latent 7x9, seed workload 9)\n")
        f.write("# written by tests/golden/make_golden.py; shape %s; rms %.17g\n" % ("x".join(map(str, shape)), rms))
        f.write("# flat_index value\n")
        for i, v in zip(idx, vals):
            f.write("%d %.17g\n" % (i, v))
    print("wrote", path)


if __name__ == "__main__":
    main()
