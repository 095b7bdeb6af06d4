"""The oracle still produces the frozen tiny-config trace (tests/golden/tiny_f32_trace.json, written by
tests/golden/make_golden.py from the oracle alone; the paper itself prints no numeric example of Algorithm 1)."""
import json
import os

import numpy as np
import pytest

import synth_inputs as si
from tests.helpers import oracle_model

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_f32_trace.json")


@pytest.mark.parametrize("tag,resid_scale", [("plain_init", 1.0), ("slow_drift", 0.05)])
def test_tiny_trace(tag, resid_scale):
    want = json.load(open(GOLDEN))[tag]
    shape = si.TINY_F32
    om = oracle_model("tiny-f32", 1, resid_scale)
    prompt = [int(t) for t in si.gen_tokens(2, 64, shape.vocab)]
    assert prompt[:8] == want["prompt_head"]
    plain, _ = om.greedy_decode(prompt, 32)
    spec = om.spec_decode(prompt, 32, 3, 4)
    assert plain == want["greedy_tokens"] and spec["tokens"] == want["spec_tokens"]
    assert [r["accepted"] for r in spec["rounds"]] == want["accepted"]
    assert [r["mask"].tolist() for r in spec["rounds"]] == want["masks"]
    first = spec["rounds"][0]["dp"]
    assert first["choice"].tolist() == want["first_dp_choice"]
    for key in ("sigma_c", "sigma_s"):
        ref = np.array([[np.nan if v is None else v for v in row] for row in want["first_dp_" + key]])
        np.testing.assert_allclose(first[key], ref, atol=2e-9, equal_nan=True)
