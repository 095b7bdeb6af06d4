"""clasp_prefill_static (the prompt pass on the library's static scratch array, for callers that cannot allocate)
against clasp_prefill with a caller workspace: the same kernels on the same passes, so the caches they leave are equal
bit for bit. Two calls in a row, the second on a shorter prompt (the array then still holds the first call's buffers);
sizes beyond the array are rejected; the call itself allocates nothing torch can see."""
import ctypes as C

import pytest
import torch

import synth_inputs as si
from paper_2505_24196_amd import binding
from paper_2505_24196_amd.binding import ClaspError
from tests.helpers import prompt
from tests.test_gpu_parity import dev, engine

pytestmark = pytest.mark.gpu


def cache_of(eng, T):
    return [tuple(t.clone() for t in eng.clasp_kv_read(l, 0, T)) for l in range(eng.shape.n_layers)]


def test_static_prefill_equals_workspace_prefill_on_two_calls_in_a_row():
    name = "small-bf16"
    shape = si.SHAPES[name]
    eng = engine(name, max_seq=320)
    for T, chunk in ((300, 128), (141, 128)):  # ragged lengths, three passes then two; the second call is the shorter
        tt = dev(prompt(shape, T, seed=2 + T), torch.int32)
        before = torch.cuda.memory_allocated()
        eng.clasp_prefill_static(tt, 0, chunk)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        got = cache_of(eng, T)
        eng.k_cache.zero_()
        eng.v_cache.zero_()
        eng.clasp_prefill(tt, 0, chunk)
        want = cache_of(eng, T)
        for l in range(shape.n_layers):
            assert torch.equal(got[l][0], want[l][0]) and torch.equal(got[l][1], want[l][1]), f"T={T} layer {l}"
            assert got[l][0].abs().max() > 0


def test_static_prefill_continues_a_prefix_and_rejects_what_does_not_fit():
    name = "small-bf16-hd128"
    shape = si.SHAPES[name]
    eng = engine(name, max_seq=320)
    T0, T = 77, 77 + 150
    tt = dev(prompt(shape, T), torch.int32)
    eng.clasp_prefill(tt, 0, 128)
    want = cache_of(eng, T)
    eng.k_cache.zero_()
    eng.v_cache.zero_()
    eng.clasp_prefill_static(tt[:T0], 0, 128)
    eng.clasp_prefill_static(tt[T0:], T0, 256)
    got = cache_of(eng, T)
    # reference for the split call: the same two calls through the workspace path
    eng.k_cache.zero_()
    eng.v_cache.zero_()
    eng.clasp_prefill(tt[:T0], 0, 128)
    eng.clasp_prefill(tt[T0:], T0, 256)
    ref = cache_of(eng, T)
    for l in range(shape.n_layers):
        assert torch.equal(got[l][0], ref[l][0]) and torch.equal(got[l][1], ref[l][1]), f"layer {l}"
        assert (got[l][0] - want[l][0]).abs().max() <= 2e-2 * want[l][0].abs().max()
    lib = binding.lib()
    limit = lib.clasp_static_scratch_bytes()
    assert limit == 32 << 20
    big = 8192
    assert lib.clasp_prefill_workspace_bytes(C.byref(eng.cfg), big) > limit
    with pytest.raises(ClaspError, match="workspace"):
        eng.clasp_prefill_static(tt, 0, big)
    with pytest.raises(ClaspError):
        eng.clasp_prefill_static(tt, 0, 100)  # not a multiple of 128
