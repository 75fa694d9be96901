"""Writes tests/golden/datagen_first8.json: the first eight fp32 values (as hex
bit patterns) of every input tensor of the workloads at full size.  Calls
only the input generator.  Re-run after a deliberate change of the generator."""
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from paper_2506_10401_amd import datagen  # noqa: E402


def main():
    out = {}
    for cfg, specs_fn in datagen.CONFIGS.items():
        for name, (ti, shape, kind, p0, p1) in specs_fn().items():
            seed = datagen.tensor_seed(cfg, ti)
            gen = datagen.gen_uniform if kind == "u" else datagen.gen_normal
            first = gen(seed, (8,), p0, p1)
            out["%d/%s" % (cfg, name)] = {"seed": hex(seed), "kind": kind, "p0": p0, "p1": p1,
                                          "bits": ["%08x" % int(b) for b in first.view(np.uint32)]}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "datagen_first8.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
    print("wrote", path)


if __name__ == "__main__":
    main()
