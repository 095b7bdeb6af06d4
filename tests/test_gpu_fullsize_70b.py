"""GPU parity at the LLaMA-3-70B shape (benchmark configuration 4: T = 1024, M = 32, K = 4).

The fp64 oracle needs ~0.5 s per row and layer at this width, so the comparison is split:
  * against the oracle, element by element: a model of the FIRST FOUR layers of the 70B-shape model (same seeds, same
    layer shapes: d_model 8192, 64 / 8 heads, d_ffn 28672, vocab 128256) over a 1024-token synthetic prefix: verify
    rows, the search with and without tables (M = 3), a draft step, and a verify pass of 18 rows (two 16-row groups, the
    second ragged: the launch shape the search takes at M = 32);
  * against the oracle, element by element: the FIRST 24 layers of the same model with a prefix of 40 tokens that each
    side produces itself (the device in verify passes of 32 and 8 rows), then two verify rows, the search with M = 20
    on the device's own states (two 16-row groups from level 18 on: four column tiles per wavefront in the projections,
    the two-group K-split down projection and select step), the search without tables, and a draft step;
  * on the whole 80-layer model with M = 32, where the oracle cannot follow: what holds for any correct search
    (Algorithm 1's structure; the skip set replayed layer by layer reproduces the score the table ends on).
"""
import dataclasses

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import clasp_oracle as oc
from tests.test_gpu_fullsize import load_prefix, verify_dp_draft
from tests.test_gpu_parity import COS_TOL, HID_TOL, dev, relerr

pytestmark = pytest.mark.gpu

T = 1024


def test_70b_layer_shapes_against_the_oracle():
    import bench
    shape = dataclasses.replace(si.LLAMA3_70B, name="llama3-70b-shape-first-4-layers", n_layers=4)
    eng, host = bench.build_engine(shape, 1, T + 64, 32, keep_host=True)
    try:
        om = oc.OracleModel(shape, host)
        cache = oc.KVCache(shape, T + 40)
        load_prefix(shape, eng, cache, T, shape.n_layers)
        verify_dp_draft(shape, T, eng, om, cache, M=3)
        # 18 rows in one verify pass on top of the same prefix (their keys / values overwrite rows T.. of both caches)
        toks = [int(t) for t in si.gen_tokens(2, 18, shape.vocab, stream=21)]
        st = []
        for r, tk in enumerate(toks):
            print(f"oracle verify row {r} of 18", flush=True)
            s, _ = om.token(tk, T + r, cache, want_states=True, want_logits=False)
            st.append(s)
        ost = np.stack(st, 1)
        out = eng.clasp_verify_forward(dev(toks, torch.int32), T, want_hidden=True)
        for l in range(shape.n_layers + 1):
            assert relerr(out["hidden"][l].cpu().numpy(), ost[l]) <= HID_TOL["bf16"], f"layer {l}"
    finally:
        eng.close()


def test_70b_24_layers_two_row_groups_against_the_oracle():
    import bench
    shape = dataclasses.replace(si.LLAMA3_70B, name="llama3-70b-shape-first-24-layers", n_layers=24)
    n_prompt, M = 40, 20
    eng, host = bench.build_engine(shape, 1, 128, 32, keep_host=True)
    try:
        om = oc.OracleModel(shape, host)
        toks = [int(t) for t in si.gen_tokens(2, n_prompt, shape.vocab, stream=31)]
        cache = oc.KVCache(shape, n_prompt + 8)
        for t, tk in enumerate(toks):
            if t % 8 == 0:
                print(f"oracle prompt token {t} of {n_prompt}", flush=True)
            om.token(tk, t, cache, want_logits=False)
        tt = dev(toks, torch.int32)
        eng.clasp_verify_forward(tt[:32], 0)
        eng.clasp_verify_forward(tt[32:], 32)
        worst = 0.0
        for l in range(shape.n_layers):
            K, V = (x.cpu().numpy() for x in eng.clasp_kv_read(l, 0, n_prompt))
            ek, ev = relerr(K, cache.K[l, :n_prompt]), relerr(V, cache.V[l, :n_prompt])
            assert ek <= HID_TOL["bf16"] and ev <= HID_TOL["bf16"], f"cache layer {l}: K {ek:.3e} V {ev:.3e}"
            worst = max(worst, ek, ev)
        print(f"largest cache error over 24 layers: {worst:.3e}", flush=True)
        stats = verify_dp_draft(shape, n_prompt, eng, om, cache, M=M)
        print(f"dp cells compared: {stats}", flush=True)
    finally:
        eng.close()


def test_70b_whole_model_search_properties():
    import bench
    shape, M = si.LLAMA3_70B, 32
    L = shape.n_layers
    eng, _ = bench.build_engine(shape, 1, T + 64, 32)
    try:
        for l in range(L):
            K, V = si.gen_kv(shape, 1000 + l, 1, T, "cuda")
            eng.clasp_kv_load(l, K[0], V[0])
        tok = dev([int(t) for t in si.gen_tokens(2, 2, shape.vocab, stream=9)], torch.int32)
        ver = eng.clasp_verify_forward(tok, T, want_hidden=True)
        X = ver["hidden"][:, 1, :].contiguous()  # states of the row at position T + 1
        out = eng.clasp_dp_select(X, T + 1, M, want_tables=True)
        mask = out["mask"].cpu().numpy()
        choice = out["choice"].cpu().numpy()
        sc = out["scores"].cpu().numpy().astype(np.float64)
        assert int(mask.sum()) == M
        # structure of Algorithm 1: layer 0 is never evaluated (cell (1, 1) keeps the skip candidate), the diagonal
        # i = j <= M has no computed candidate, cells beyond min(i, M) do not exist, scores are cosines
        assert choice[1, 1] == 1
        for i in range(1, L + 1):
            for j in range(1, M + 1):
                if j > i:
                    assert choice[i, j] == 255
                elif j == i:
                    assert choice[i, j] == 1 and np.isnan(sc[i, j, 0])
                else:
                    assert choice[i, j] in (0, 1)
                    assert choice[i, j] == (0 if sc[i, j, 0] > sc[i, j, 1] else 1)
        assert np.nanmax(np.abs(sc)) <= 1.0 + 1e-5
        # backtracking by hand from (L, M) gives the mask
        want = np.zeros(L, dtype=np.uint8)
        i, j = L, M
        while i > 0 and j > 0:
            if choice[i, j] == 1:
                want[i - 1] = 1
                j -= 1
            i -= 1
        assert mask.tolist() == want.tolist()
        # the table ends on D(L, M); replaying the skip set layer by layer (one row, the single-row kernels) from the
        # token's embedding reaches the same cosine with x_L, and the same state
        d_lm = np.nanmax(sc[L, M])
        replay = eng.clasp_skip_cosine([mask], tok[1:2], T + 1, X[L])
        assert abs(float(replay[0]) - d_lm) <= 2 * COS_TOL
        g = out["g_final"]
        cos_g = float(torch.dot(g, X[L]) / (g.norm() * X[L].norm()))
        assert abs(cos_g - d_lm) <= COS_TOL
        # the search without tables (cells that cannot reach (L, M) left out) selects the same set
        lean = eng.clasp_dp_select(X, T + 1, M)
        assert torch.equal(lean["mask"], out["mask"])
        # a draft step with 32 of the 80 layers skipped runs and returns a token of the vocabulary
        nxt = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        eng.clasp_draft_step(mask.tolist(), tok[1:2], T + 1, nxt)
        assert 0 <= int(nxt) < shape.vocab
    finally:
        eng.close()
