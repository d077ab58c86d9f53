"""Writes tests/golden/tiny_oracle.txt: sampled values of the oracle's output on the tiny
benchmark configuration (2 joint blocks, hidden 256, 64 image + 16 text tokens, 4 Euler
steps).  Calls only `oracle/` and the seeded generators; nothing here comes from the GPU
library.  The paper prints no numbers for the Diffuse stage, so this file is a regression
guard for the oracle itself, not a paper value.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth  # noqa: E402
from oracle import dit_oracle as O  # noqa: E402


def compute():
    cfg = synth.CONFIGS["tiny"]
    arch = cfg["arch"]
    params = synth.make_params(O.param_shapes(arch), seed=1, std=0.02)
    reqs = synth.make_requests("tiny")
    lat, cond, sig = synth.make_inputs(reqs, arch["latent_ch"], arch["cond_dim"], cfg["steps"])
    m = O.DiTOracle(arch, params)
    v0 = m.velocity(lat[0], cond[0], sig[0][0])
    xT = m.sample(lat[0], cond[0], sig[0])
    idx = np.arange(0, v0.size, 97)
    return idx, v0.ravel()[idx], xT.ravel()[idx]


if __name__ == "__main__":
    idx, v0, x0 = compute()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_oracle.txt")
    with open(path, "w") as f:
        f.write("# flat_index  velocity_at_step0  final_latent_after_4_euler_steps\n")
        f.write("# source: oracle/dit_oracle.py on synth config 'tiny' (weights seed 1, std 0.02;\n")
        f.write("# noise seed 2, condition seed 100); written by tests/golden/make_golden.py\n")
        for i, a, b in zip(idx, v0, x0):
            f.write(f"{i} {a:.15e} {b:.15e}\n")
    print("wrote", path)
