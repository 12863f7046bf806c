"""Writes tests/golden/*.txt from the CPU oracle only (never from the GPU path).

Run from the repository root:  python tests/golden/make_golden.py
Each file holds the int32 logits of the first images of one seeded benchmark model
(workloads.model_by_name; images drawn from stream (config, layer 0, tensor 0)), one
image per line.  The paper prints no worked numeric example, so these are regression
values of the pinned oracle, not the paper's.
"""
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import workloads as W  # noqa: E402

N_IMAGES = {"mlp": 8, "small_cnn": 8, "vgg_small": 4}


def main():
    for name, n in N_IMAGES.items():
        cid, layers, (ih, iw, ic) = W.model_by_name(name)
        imgs = W.draw_images(W.rng_for(cid, 0, 0), n, ih, iw, ic)
        logits, _ = oracle.run_model(layers, imgs)
        path = os.path.join(HERE, f"{name}_logits.txt")
        with open(path, "w") as f:
            f.write(f"# oracle logits, model={name}, images={n}, seed stream=({cid},0,0), "
                    f"first-layer pad value -1, order step->pool\n")
            for row in logits:
                f.write(" ".join(str(int(v)) for v in row) + "\n")
        print("wrote", path)


if __name__ == "__main__":
    main()
