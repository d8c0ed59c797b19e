"""Writes tests/golden/tiny_o64.txt: values of the fp64 CPU oracle on the tiny
configuration (Algorithm 1 with the Nesterov base of Table C.1; m = 4,
d = 65536, tau = 12, 10 outer iterations, seeded synthetic gradients).

The stored values come from the oracle only -- this script imports nothing of
the HIP path -- and serve as a regression guard on the oracle and as a second
route from the GPU tests to the same expected values.

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import slowmo_oracle as O            # noqa: E402
from slowmo_inputs import generator as G         # noqa: E402
from slowmo_inputs import workloads as W         # noqa: E402

SAMPLE = [0, 1, 2, 3, 63, 64, 255, 256, 1023, 4095, 4096, 4097, 8191, 16384,
          32767, 32768, 50000, 65532, 65533, 65534, 65535]


def run():
    w = W.tiny()
    idx = np.arange(w.d, dtype=np.int64)
    o = O.SlowMoOracle(G.initial_params(w.seed, idx), m=w.m, tau=w.tau,
                       alpha=w.f32("alpha"), beta=w.f32("beta"), base=w.base,
                       policy=w.policy, momentum=w.f32("momentum"),
                       weight_decay=w.f32("weight_decay"), prec="f64")
    o.run(lambda t, k: np.stack([G.gradient(w.seed, i, t * w.tau + k, idx, w.sigma)
                                 for i in range(w.m)]), w.f32("lr"), w.rounds)
    return o


def main():
    o = run()
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_o64.txt")
    with open(path, "w") as f:
        f.write("# fp64 oracle, tiny configuration, after 10 outer iterations\n")
        f.write("# Algorithm 1 + Table C.1 (SGD row); written by make_golden.py\n")
        f.write("# index x0 u\n")
        for j in SAMPLE:
            f.write(f"{j} {float(o.x0[j]).hex()} {float(o.u[j]).hex()}\n")
        f.write(f"# sum_x0 {float(o.x0.sum()).hex()}\n# sum_u {float(o.u.sum()).hex()}\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
