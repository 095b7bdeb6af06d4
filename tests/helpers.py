"""Shared test plumbing: builds oracle models from the seeded generators. No method arithmetic here."""
import functools

import numpy as np

import synth_inputs as si
from oracle import clasp_oracle as oc


@functools.lru_cache(maxsize=8)
def torch_model(shape_name: str, seed: int = 1, resid_scale: float = 1.0):
    return si.gen_model(si.SHAPES[shape_name], seed, "cpu", resid_scale)


@functools.lru_cache(maxsize=8)
def oracle_model(shape_name: str, seed: int = 1, resid_scale: float = 1.0):
    shape = si.SHAPES[shape_name]
    return oc.OracleModel(shape, si.model_to_numpy(torch_model(shape_name, seed, resid_scale)))


def prompt(shape, n: int, seed: int = 2):
    return [int(t) for t in si.gen_tokens(seed, n, shape.vocab)]
