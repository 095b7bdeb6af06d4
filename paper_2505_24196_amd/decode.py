"""Host side of the Draft -> Verify -> Layer-Optimisation loop (Sec. 3.1 of the paper) on top of the C ABI.

Only integer control flow lives here (greedy acceptance: the longest prefix of the draft that matches the full model's
argmax, plus the full model's own next token); every forward, the DP and the argmax run in the HIP library.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import torch

from .binding import Engine


PREFILL_MIN_ROWS = 64  # prompts at least this long go through the many-row kernels (bf16 models)


def prefill(engine: Engine, prompt: Sequence[int], pos0: int = 0, chunk_rows: Optional[int] = None):
    """Full model over the prompt. Returns (states [L+1][d] of the last token, its argmax, its margin). All tokens
    but the last go through clasp_prefill (compute-bound kernels, `chunk_rows` rows per pass; default: the prompt
    length rounded up to 128, at most 8192) when the model is bf16 and the prompt is long enough, else through
    clasp_verify_forward in chunks of max_rows; the last token always takes clasp_verify_forward, which yields its
    per-layer states. chunk_rows = 0 forces the clasp_verify_forward path."""
    toks = torch.as_tensor(list(prompt), dtype=torch.int32, device=engine.device)
    n, step = toks.numel(), engine.max_rows
    out = None
    start = 0
    if engine.shape.dtype == "bf16" and chunk_rows != 0 and n - 1 >= PREFILL_MIN_ROWS:
        if chunk_rows is None:
            chunk_rows = min(8192, (n - 1 + 127) // 128 * 128)
        engine.clasp_prefill(toks[:n - 1], pos0, chunk_rows)
        start = n - 1
    for s in range(start, n, step):
        chunk = toks[s:s + step]
        out = engine.clasp_verify_forward(chunk, pos0 + s, want_hidden=(s + step >= n), want_margin=True)
    last = out["argmax"].numel() - 1
    return out["hidden"][:, last, :], out["argmax"][last:last + 1], out["margin"][last:last + 1]


def greedy_generate(engine: Engine, prompt: Sequence[int], n_gen: int):
    """Plain greedy decoding with the full model (one row per step). Returns (tokens, top-1 minus top-2 margins)."""
    _, nxt, mg = prefill(engine, prompt)
    buf = torch.empty(n_gen, dtype=torch.int32, device=engine.device)
    margins = torch.empty(n_gen, dtype=torch.float32, device=engine.device)
    buf[0:1].copy_(nxt)
    margins[0:1].copy_(mg)
    pos = len(prompt)
    for t in range(1, n_gen):
        out = engine.clasp_verify_forward(buf[t - 1:t], pos, want_margin=True)
        buf[t:t + 1].copy_(out["argmax"])
        margins[t:t + 1].copy_(out["margin"])
        pos += 1
    return buf.cpu().tolist(), margins.cpu().tolist()


def clasp_generate(engine: Engine, prompt: Sequence[int], n_gen: int, M: int, K: int, dp_interval: int = 1,
                   trace: bool = False, det_threshold: Optional[float] = None) -> Dict[str, object]:
    """Greedy self-speculative decoding with the DP-selected skip set re-optimised every `dp_interval` verify steps
    (1 = after every verification, the paper's default; larger values are its lower optimisation frequency).
    det_threshold (Sec. 5.3.3, draft-exiting threshold): drafting stops after the first draft token whose top-1
    probability under the draft model is below the threshold; that token is still proposed, so a round verifies
    2..K+1 rows. Reading the probability costs one 4-byte device-to-host copy per draft step."""
    dev = engine.device
    states, nxt, _ = prefill(engine, prompt)
    pos = len(prompt)
    dp = engine.clasp_dp_select(states, pos - 1, M, want_tables=trace)  # prefill counts as verification 0
    mask = dp["mask"].cpu().tolist()
    out: List[int] = [int(nxt.item())]
    tok = torch.empty(K + 1, dtype=torch.int32, device=dev)
    tok[0:1].copy_(nxt)
    conf = torch.zeros(K, dtype=torch.float32, device=dev) if (det_threshold is not None or trace) else None
    rounds = []
    n_verify = 0
    while len(out) < n_gen:
        n_draft = 0
        for k in range(K):
            engine.clasp_draft_step(mask, tok[k:k + 1], pos + k, tok[k + 1:k + 2],
                                    None if conf is None else conf[k:k + 1])
            n_draft += 1
            if det_threshold is not None and float(conf[k].item()) < det_threshold:
                break
        ver = engine.clasp_verify_forward(tok[:n_draft + 1], pos, want_hidden=True, want_margin=trace)
        rows = tok[:n_draft + 1].cpu().tolist()
        v = ver["argmax"].cpu().tolist()
        a = 0
        while a < n_draft and rows[a + 1] == v[a]:
            a += 1
        out.extend(rows[1:a + 1] + [v[a]])
        n_verify += 1
        if trace:
            rounds.append({"pos": pos, "mask": list(mask), "drafts": rows[1:], "verify": v, "accepted": a,
                           "verify_margin": ver["margin"].cpu().tolist(), "dp": {k: t.cpu() for k, t in dp.items()},
                           "draft_conf": conf[:n_draft].cpu().tolist(),
                           "states": ver["hidden"][:, a, :].cpu()})
        else:
            rounds.append({"pos": pos, "accepted": a, "mask": list(mask)})
        if n_verify % dp_interval == 0 and len(out) < n_gen:
            dp = engine.clasp_dp_select(ver["hidden"][:, a, :], pos + a, M, want_tables=trace)
            mask = dp["mask"].cpu().tolist()
        tok[0:1].copy_(ver["argmax"][a:a + 1])
        pos += a + 1
    return {"tokens": out[:n_gen], "rounds": rounds}


def clasp_sample_generate(engine: Engine, prompt: Sequence[int], n_gen: int, M: int, K: int,
                          uniforms: Dict[str, torch.Tensor], temperature: float = 1.0,
                          trace: bool = False) -> Dict[str, object]:
    """Stochastic self-speculative decoding (the Temperature = 1 setting of Sec. 4): drafts are drawn from the
    layer-skipped model's distribution, one verify pass gives the full model's logits for all of them, and the
    speculative-sampling rule keeps a prefix of the drafts and draws the next token, so the output is distributed as
    the full model's own sampling. The layer optimisation runs on the last accepted row as in the greedy loop.

    uniforms: device fp32 tensors "first" [1], "draft" [rounds*K], "accept" [rounds*K], "final" [rounds] in [0, 1);
    round r consumes draft/accept indices r*K .. r*K+K-1 and final index r. Per round one 8-byte device-to-host copy
    (accepted count, next token) plus the mask bytes."""
    dev = engine.device
    V = engine.shape.vocab
    toks = torch.as_tensor(list(prompt), dtype=torch.int32, device=dev)
    n, step = toks.numel(), engine.max_rows
    for s in range(0, n, step):
        last = engine.clasp_verify_forward(toks[s:s + step], s, want_hidden=(s + step >= n), want_logits=(s + step >= n))
    rows_last = last["argmax"].numel() - 1
    tok = torch.empty(K + 1, dtype=torch.int32, device=dev)
    engine.clasp_sample_token(last["logits"][rows_last], temperature, uniforms["first"][0:1], tok[0:1])
    pos = len(prompt)
    dp = engine.clasp_dp_select(last["hidden"][:, rows_last, :], pos - 1, M)
    mask = dp["mask"].cpu().tolist()
    out: List[int] = [int(tok[0].item())]
    q_logits = torch.empty(K, V, dtype=torch.float32, device=dev)
    res = torch.empty(2, dtype=torch.int32, device=dev)
    rounds = []
    r = 0
    while len(out) < n_gen:
        for k in range(K):
            engine.clasp_draft_sample(mask, tok[k:k + 1], pos + k, temperature, uniforms["draft"][r * K + k:r * K + k + 1],
                                      q_logits[k], tok[k + 1:k + 2])
        ver = engine.clasp_verify_forward(tok, pos, want_hidden=True, want_logits=True)
        engine.clasp_spec_accept(ver["logits"], q_logits, tok, K, temperature, uniforms["accept"][r * K:(r + 1) * K],
                                 uniforms["final"][r:r + 1], res[0:1], res[1:2])
        a, nxt = res.cpu().tolist()
        drafts = tok[1:].cpu().tolist()
        out.extend(drafts[:a] + [nxt])
        rec = {"pos": pos, "accepted": a, "next": nxt, "drafts": drafts, "mask": list(mask)}
        if trace:
            rec["p_logits"], rec["q_logits"] = ver["logits"].cpu(), q_logits.cpu()
        rounds.append(rec)
        if len(out) < n_gen:
            dp = engine.clasp_dp_select(ver["hidden"][:, a, :], pos + a, M)
            mask = dp["mask"].cpu().tolist()
        tok[0:1].copy_(res[1:2])
        pos += a + 1
        r += 1
    return {"tokens": out[:n_gen], "rounds": rounds}


def skip_set_jaccard(masks: Sequence[Sequence[int]], max_gap: int = 8) -> List[float]:
    """Sparse persistence (Sec. 3.7, Fig. 3a): mean Jaccard similarity |A & B| / |A | B| between the skip sets chosen
    `gap` optimisations apart, for gap = 1..max_gap (two empty sets count as identical). masks: one 0/1 sequence of
    length L per optimisation, in order. Gaps with no pair are left out."""
    sets = [frozenset(i for i, m in enumerate(mask) if m) for mask in masks]
    curve = []
    for gap in range(1, max_gap + 1):
        pairs = [(a, b) for a, b in zip(sets, sets[gap:])]
        if not pairs:
            break
        curve.append(sum(1.0 if not (a | b) else len(a & b) / len(a | b) for a, b in pairs) / len(pairs))
    return curve


def markov_study(engine: Engine, states: torch.Tensor, token: torch.Tensor, pos: int, layer_lo: int, layer_hi: int,
                 budgets: Sequence[int], n_random: int = 32, seed: int = 0) -> List[Dict[str, object]]:
    """The comparison of Sec. 3.5 (approximate Markov property): with the layers outside layer_lo..layer_hi-1 fixed,
    the cosine between the full model's last hidden state (states[L]) and the one a skip set of size M produces, for
    the set the dynamic program selects, for the best of all C(window, M) sets (brute force) and for random sets.
    states: device fp32 [L+1][d] of the token (device int32 [1]) at position pos. Host side: enumeration only."""
    import itertools
    import random
    L = engine.shape.n_layers
    target = states[L].contiguous()
    rng = random.Random(seed)
    rows = []
    for M in budgets:
        combos = list(itertools.combinations(range(layer_lo, layer_hi), M))
        masks = [[1 if l in c else 0 for l in range(L)] for c in map(set, combos)]
        cos = engine.clasp_skip_cosine(masks, token, pos, target).cpu()
        best = int(torch.argmax(cos))
        dp_mask = engine.clasp_dp_select_window(states, pos, M, layer_lo, layer_hi)["mask"].cpu().tolist()
        dp_cos = float(engine.clasp_skip_cosine([dp_mask], token, pos, target).cpu()[0])
        picks = [rng.randrange(len(combos)) for _ in range(n_random)]
        rnd = cos[picks]
        rows.append({"M": M, "sets": len(combos), "brute_force_cos": float(cos[best]), "brute_force_set": list(combos[best]),
                     "dp_cos": dp_cos, "dp_set": [l for l in range(L) if dp_mask[l]],
                     "dp_rank": int((cos > dp_cos + 1e-7).sum()) + 1,
                     "random_mean_cos": float(rnd.mean()), "random_min_cos": float(rnd.min())})
    return rows
