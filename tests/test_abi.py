"""CPU-side checks of the boundary: the built library loads and exports every function include/clasp.h declares,
and the size / validation entry points that need no GPU behave."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "clasp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(clasp_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_hot_path_calls():
    names = declared_functions()
    for n in ("clasp_verify_forward", "clasp_dp_select", "clasp_draft_step"):
        assert n in names


def test_library_exports_every_declared_function():
    from paper_2505_24196_amd import binding
    lib = binding.lib()
    for name in declared_functions():
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(declared_functions())


def test_sizes_and_validation_without_a_gpu():
    from paper_2505_24196_amd import binding
    import synth_inputs as si
    lib = binding.lib()
    assert lib.clasp_strerror(0) == b"ok" and lib.clasp_strerror(-2) == b"unsupported shape"
    assert lib.clasp_packed_bytes(4096, 14336, binding.CLASP_BF16) == 4096 * 14336 * 2
    assert lib.clasp_packed_bytes(100, 128, binding.CLASP_BF16) == 0  # rows not a multiple of 16
    assert lib.clasp_packed_bytes(128, 100, binding.CLASP_BF16) == 0  # cols not a multiple of 32
    assert lib.clasp_packed_bytes(688, 256, binding.CLASP_F32) == 688 * 256 * 4
    s = si.LLAMA3_8B
    cfg = binding.Config(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 1024, 16, 1,
                         s.rms_eps, s.rope_base)
    assert lib.clasp_kv_cache_bytes(C.byref(cfg)) == 32 * 8 * 1024 * 128 * 2
    assert lib.clasp_workspace_bytes(C.byref(cfg)) > 0
    cfg.max_rows = 33
    assert lib.clasp_workspace_bytes(C.byref(cfg)) == 0
    cfg.max_rows, cfg.max_seq = 16, 1000  # not a multiple of 32
    assert lib.clasp_workspace_bytes(C.byref(cfg)) == 0
    out = C.c_void_p()
    cfg.max_seq = 1024
    assert lib.clasp_create(C.byref(cfg), None, None, 0, None, None, C.byref(out)) == -1
    assert lib.clasp_destroy(None) == -1


def test_create_rejects_null_and_misaligned_weight_pointers_before_touching_the_gpu():
    """clasp_create validates every pointer on the host first: a missing or not 16-byte aligned matrix / gain pointer is
    CLASP_E_INVALID_ARG (the addresses below are made up and never dereferenced)."""
    from paper_2505_24196_amd import binding
    import synth_inputs as si
    lib = binding.lib()
    s = si.SMALL_BF16
    cfg = binding.Config(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 64, 16, 1,
                         s.rms_eps, s.rope_base)
    L = s.n_layers
    arr = lambda bad_layer=None, bad=0: (C.c_void_p * L)(*[(bad if l == bad_layer else 0x10000000 + 0x1000 * l) for l in range(L)])
    big = C.c_size_t(1 << 40)
    out = C.c_void_p()

    def create(**over):
        w = binding.Weights()
        w.embed, w.lm_head, w.final_norm = 0x20000000, 0x30000000, 0x40000000
        fields = dict(attn_norm=arr(), mlp_norm=arr(), wq=arr(), wk=arr(), wv=arr(), wo=arr(), w_gate_up=arr(), w_down=arr())
        fields.update(over)
        for k, v in fields.items():
            if k in ("embed", "lm_head", "final_norm"):
                setattr(w, k, v)
            else:
                setattr(w, k, C.cast(v, C.POINTER(C.c_void_p)))
        return lib.clasp_create(C.byref(cfg), C.byref(w), C.c_void_p(0x50000000), big, C.c_void_p(0x60000000),
                                C.c_void_p(0x70000000), C.byref(out))

    assert create(mlp_norm=arr(3, 0x10000004)) == -1   # gains not 16-byte aligned
    assert create(w_down=arr(L - 1, None)) == -1       # a missing matrix
    assert create(wq=arr(0, 0x10000008)) == -1
    assert create(final_norm=0x40000002) == -1


def test_prefill_workspace_sizes_without_a_gpu():
    """The prompt pass's workspace: refused chunk sizes give 0; it grows with the chunk; from 640 rows on it also holds
    the fp16 copy of one layer's matrices."""
    from paper_2505_24196_amd import binding
    import synth_inputs as si
    lib = binding.lib()
    s = si.LLAMA3_8B
    cfg = binding.Config(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.head_dim, s.d_ffn, s.vocab, 8192, 16, 1,
                         s.rms_eps, s.rope_base)
    size = lambda rows: lib.clasp_prefill_workspace_bytes(C.byref(cfg), rows)
    for bad in (0, 100, 64, 8192 + 128, -128):
        assert size(bad) == 0
    assert 0 < size(128) < size(256) < size(512)
    per_128_rows = size(512) - size(384)
    assert size(384) - size(256) == per_128_rows
    assert size(640) - size(512) >= per_128_rows + s.layer_weight_elems() * 2  # the fp16 copy of a layer's matrices
    assert size(768) - size(640) == per_128_rows
    f32 = si.TINY_F32
    cfg32 = binding.Config(f32.n_layers, f32.d_model, f32.n_heads, f32.n_kv_heads, f32.head_dim, f32.d_ffn, f32.vocab,
                           64, 16, 0, f32.rms_eps, f32.rope_base)
    assert lib.clasp_prefill_workspace_bytes(C.byref(cfg32), 128) == 0  # fp32 models take the row-limited path


def test_engine_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    import paper_2505_24196_amd as clasp
    import synth_inputs as si
    with pytest.raises(clasp.ClaspError):
        clasp.Engine(si.TINY_F32, max_seq=64)


def test_skip_set_jaccard_curve_by_hand():
    """Sparse persistence statistic (Sec. 3.7): Jaccard similarity of skip sets `gap` optimisations apart."""
    from paper_2505_24196_amd import skip_set_jaccard
    masks = [[1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 1, 0], [0, 0, 0, 1]]
    # gap 1: {0,1}~{0,2} = 1/3, {0,2}~{0,2} = 1, {0,2}~{3} = 0; gap 2: {0,1}~{0,2} = 1/3, {0,2}~{3} = 0; gap 3: 0
    curve = skip_set_jaccard(masks, max_gap=8)
    assert curve == pytest.approx([(1 / 3 + 1 + 0) / 3, (1 / 3 + 0) / 2, 0.0])
    assert skip_set_jaccard([[0, 0], [0, 0]]) == [1.0]  # two empty sets are identical
    assert skip_set_jaccard([[1, 0]]) == []


def test_algorithmic_bytes_of_the_benchmark_configurations():
    """bench.py prices every call against the bytes the method itself has to move: the weights of each evaluated layer
    once plus the shared KV prefix once per layer (the DP never evaluates layer 0; a draft step runs L - M layers and
    the head). The figures for the LLaMA-3-8B and -70B shapes, worked out by hand from the shapes."""
    import bench
    import synth_inputs as si
    s = si.LLAMA3_8B
    w_layer = (4096 * (4096 + 2 * 1024) + 4096 * 4096 + 3 * 4096 * 14336) * 2
    assert s.layer_weight_elems() * s.elem_bytes() == w_layer == 436_207_616
    ab = bench.algorithmic_bytes(s, 512, 12)
    kv = 2 * 1024 * 2 * 512
    assert ab["dp_select"] == 31 * (w_layer + kv) and abs(ab["dp_select"] / 1e9 - 13.59) < 0.01
    assert ab["draft_step"] == 20 * (w_layer + kv) + 128256 * 4096 * 2 and abs(ab["draft_step"] / 1e9 - 9.82) < 0.01
    assert ab["verify_forward"] == 32 * (w_layer + kv) + 128256 * 4096 * 2
    assert ab["gate_up_kernel"] == 234_881_024
    assert abs(bench.algorithmic_bytes(s, 32768, 12)["dp_select"] / 1e9 - 17.68) < 0.01
    assert abs(bench.algorithmic_bytes(s, 32768, 12)["kv_share_per_layer"] - 0.2353) < 1e-3
    b70 = bench.algorithmic_bytes(si.LLAMA3_70B, 1024, 32)
    assert abs(b70["dp_select"] / 1e9 - 135.5) < 0.1 and abs(b70["draft_step"] / 1e9 - 84.4) < 0.1
