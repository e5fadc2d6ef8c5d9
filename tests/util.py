"""Glue shared by the GPU parity tests: oracle-side batch state built from the same synthetic
inputs the device gets.  No arithmetic of the method lives here."""
from __future__ import annotations

import copy
from typing import Dict, List, Sequence, Tuple

import numpy as np

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth

TOL = {synth.DT_F32: 1e-4, synth.DT_BF16: 3e-2}


def logit_tol_at_depth(n_layers: int) -> float:
    """Bound on max |logit - oracle| of the bf16-storage path after n_layers layers at the Llama-2-70B width.
    Every layer adds rounding noise of the fp16 activation stages (norm output, queries, probabilities, attention
    output, FFN activation) that is independent of the other layers', so the error grows like a random walk:
    measured 1.7e-2, 2.2e-2, 2.9e-2, 3.4e-2 at 1, 2, 4, 8 layers (exponent 0.43; 80 layers at a reduced width
    follow the same curve).  The 3e-2 of the bf16 path holds up to 4 layers; beyond, the bound follows sqrt(L)."""
    return TOL[synth.DT_BF16] * max(1.0, float(np.sqrt(n_layers / 4.0)))



def weights_f64(W: Dict[str, object]) -> Dict[str, object]:
    """The same parameters held as fp64 so the oracle does not convert them at every use."""
    out = {k: np.asarray(v, np.float64) for k, v in W.items() if k != "layers"}
    out["layers"] = [{k: np.asarray(v, np.float64) for k, v in L.items()} for L in W["layers"]]
    return out


def oracle_caches(desc, kv: synth.PagedKV) -> List[orc.SeqCache]:
    caches = []
    for b in range(len(kv.ctx_lens)):
        n = int(kv.ctx_lens[b])
        Ks, Vs = [], []
        for l in range(desc.n_layers):
            K, V = synth.gather_sequence_kv(kv, l, b, n)
            Ks.append(K)
            Vs.append(V)
        caches.append(orc.SeqCache(desc.n_layers, desc.n_kv_heads, desc.head_dim, Ks, Vs))
    return caches


def clone_cache(c: orc.SeqCache) -> orc.SeqCache:
    n = orc.SeqCache(len(c.K), c.K[0].shape[1], c.K[0].shape[2])
    n.K = [a for a in c.K]     # arrays are never modified in place by the oracle (concatenate copies)
    n.V = [a for a in c.V]
    return n


def greedy_continuations(desc, W, caches: Sequence[orc.SeqCache], last_toks: Sequence[int], ks: Sequence[int]):
    """Oracle greedy continuation of every sequence for ks[b] steps (plus the token after), by sequential
    single-token decodes on cloned caches.  Returns per sequence the list of k_b + 1 greedy tokens
    g[0..k_b] (g[j] follows input j) and the minimum top-1 margin met on the way."""
    B = len(caches)
    cl = [clone_cache(c) for c in caches]
    cur = [int(t) for t in last_toks]
    out = [[] for _ in range(B)]
    margin = [np.inf] * B
    for step in range(max(ks) + 1):
        toks = [[cur[b]] if step <= ks[b] else [] for b in range(B)]
        logits = orc.decoder_step(desc, W, toks, cl)
        for b in range(B):
            if step <= ks[b]:
                g = int(orc.greedy_tokens(logits[b])[0])
                margin[b] = min(margin[b], float(orc.top1_margin(logits[b])[0]))
                out[b].append(g)
                cur[b] = g
    return out, margin


def pick_decisive_last_tokens(desc, W, caches, ks, vocab, gen, tol, n_cand=4):
    """For every sequence try n_cand pending tokens and keep one whose whole greedy continuation has a
    top-1 margin of at least 2*tol at every position (so a logit error below tol cannot change any
    argmax).  Sequences where no candidate qualifies keep the best candidate; the caller treats them
    with the near-tie rule.  Returns last_tok[B], greedy[B] lists, margin[B]."""
    B = len(caches)
    cand_caches, cand_tok, cand_k = [], [], []
    for b in range(B):
        toks = gen.choice(vocab, size=n_cand, replace=False)
        for t in toks:
            cand_caches.append(caches[b])
            cand_tok.append(int(t))
            cand_k.append(int(ks[b]))
    g, m = greedy_continuations(desc, W, cand_caches, cand_tok, cand_k)
    last, greedy, margin = [], [], []
    for b in range(B):
        idx = range(b * n_cand, (b + 1) * n_cand)
        good = [i for i in idx if m[i] >= 2 * tol]
        pick = good[0] if good else max(idx, key=lambda i: m[i])
        last.append(cand_tok[pick])
        greedy.append(g[pick])
        margin.append(m[pick])
    return last, greedy, margin


def near_tie_ok(logits_row: np.ndarray, tok: int, tol: float) -> bool:
    return logits_row[tok] >= logits_row.max() - 2 * tol
