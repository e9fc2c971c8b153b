"""Writes tests/golden/bf16_floor_c2_small.json: the error floor of ideal bf16-operand arithmetic
(tests/bf16_model.py against the float64 oracle) for the T5.1.1-Small block shape at batch 1, for the two
readings of the logit scale and for the two split-operand variants of the score path.

Calls only the oracle, the floor model built from the oracle's pieces and the seeded input generators;
nothing here touches the HIP path.      python tests/golden/make_bf16_floor.py
"""
import json
import os
import sys
from dataclasses import replace

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import bf16_model as M  # noqa: E402
import synth_inputs as SI  # noqa: E402
from oracle import t5_oracle as O  # noqa: E402


def floors():
    out = {}
    base = SI.CONFIGS["c2_small"].with_batch(1)
    for reading, cfg in (("scaled", replace(base, attn_scale=base.d_kv ** -0.5)), ("literal", base)):
        w = SI.make_weights(cfg)
        w.update(SI.make_random_scales(cfg))
        x, dy = SI.make_activations(cfg)
        y, saved = O.block_fwd(cfg, x, w)
        dx, g = O.block_bwd(cfg, dy, w, saved)
        for variant, kw in (("plain", {}), ("split_qk", {"split_qk": True}),
                            ("split_qk_n1", {"split_qk": True, "split_n1": True})):
            f = M.block_floor(cfg, x, w, dy, ref=(y, dx, g), **kw)
            out[f"{reading}/{variant}"] = {k: [float(f"{v[0]:.4g}"), float(f"{v[1]:.4g}")] for k, v in f.items()}
    return out


if __name__ == "__main__":
    path = os.path.join(HERE, "bf16_floor_c2_small.json")
    with open(path, "w") as fh:
        json.dump(floors(), fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("wrote", path)
