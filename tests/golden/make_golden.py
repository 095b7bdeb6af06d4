"""Writes tests/golden/tiny_f32_trace.json from the CPU oracle ALONE (never from the HIP path).

The paper prints no worked numeric example of Algorithm 1 (no table, mask or score), so these stored values are
not the paper's: they freeze the pinned oracle's output on the tiny fp32 configuration (8 layers, d=256,
64-token random context, M=3, draft length 4, 32 generated tokens) so that an unintended change of the oracle's
arithmetic shows up. Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402
from oracle import clasp_oracle as oc  # noqa: E402


def main():
    out = {}
    for tag, resid_scale in (("plain_init", 1.0), ("slow_drift", 0.05)):
        shape = si.TINY_F32
        om = oc.OracleModel(shape, si.model_to_numpy(si.gen_model(shape, 1, "cpu", resid_scale)))
        prompt = [int(t) for t in si.gen_tokens(2, 64, shape.vocab)]
        plain, _ = om.greedy_decode(prompt, 32)
        spec = om.spec_decode(prompt, 32, 3, 4)
        first = spec["rounds"][0]["dp"]
        out[tag] = {
            "prompt_head": prompt[:8],
            "greedy_tokens": plain,
            "spec_tokens": spec["tokens"],
            "accepted": [r["accepted"] for r in spec["rounds"]],
            "masks": [r["mask"].tolist() for r in spec["rounds"]],
            "first_dp_sigma_c": np.where(np.isnan(first["sigma_c"]), None, np.round(first["sigma_c"], 9)).tolist(),
            "first_dp_sigma_s": np.where(np.isnan(first["sigma_s"]), None, np.round(first["sigma_s"], 9)).tolist(),
            "first_dp_choice": first["choice"].tolist(),
        }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_f32_trace.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
