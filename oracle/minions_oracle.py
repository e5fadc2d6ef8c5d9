"""CPU oracle for the LLM verification step of aggregated speculative execution (Minions).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
path is checked against.  It may be imported by tests/, by the smoke check and
by the benchmark's cpu_baseline leg; the product path never calls it.  It shares
no code with the HIP path and imports nothing from it; it depends on numpy alone.

What it computes, with the passage of the paper each part follows:

* ``vote_tree``      tree-based weighted majority decision (section 3.2, "Tree-based
                     Weighted Majority Decision", the rule v_{i+1} = argmax_{u in c(v_i)} w_u).
* ``vote_column``    the literal per-position vote (no prefix filter); a second reading kept
                     beside the paper's tree walk.
* ``decoder_step``   the LLM forward that scores the speculated positions in parallel against
                     an existing KV cache (section 2.1; section 4 on multi-token input with an
                     existing cache).  The paper only names the model families (section 5.1):
                     the body is the textbook pre-norm decoder, OPT style (LayerNorm, biases,
                     ReLU, learned positions) or Llama style (RMSNorm, rotary positions,
                     grouped-query attention, SwiGLU).
* ``decoder_full``   the same model, cache-less, over a whole token sequence with a causal mask.
* ``greedy_tokens``  argmax per scored position (lowest id on ties).
* ``accept``         longest-prefix acceptance: the greedy (temperature -> 0) case of the
                     verification rule of section 2.1: a draft token is kept iff it equals the
                     LLM's argmax, the first mismatch discards the rest, and one more token
                     comes from the LLM's own distribution (correction or bonus token).
* ``accept_stochastic``  the general verification rule of section 2.1 (keep a token outright when the
                     SSM's probability does not exceed the LLM's, otherwise reject it with probability
                     1 - o/q and draw a replacement from the renormalised positive part of o - q), with
                     its random numbers from a counter-based generator (``philox4x32``).
* ``draft_sample``   the drafting side of that rule: an SSM's token drawn from its own distribution.
* ``commit``         drop the cache entries of the rejected tokens (section 4): the context
                     grows by the accepted prefix plus the pending token.
* ``acr_update``     speculation quality metric (equation ACR) and the multiplicative weight
                     update of section 3.2.
* ``fit_slope`` / ``Selector``  the adaptive speculation length selector of section 3.3: a
                     least-squares line through the monitored t_LLM / vl samples decides whether the
                     speculation length goes down (rising trend) or up.

Arithmetic: parameters are taken as stored (bf16 values arrive widened exactly);
every intermediate is fp64; nothing is rounded on the way.  Vote weights are summed
in fp32, sequentially in ascending draft order, because the paper's weights are reals
updated multiplicatively and the order of the sum is part of the contract.

Pins: tests/test_oracle_*.py (worked example of the paper's figure "majority", brute
force over an explicit token tree, a PyTorch-CPU fp64 model assembled from library
routines, closed forms for the norms and the rotary embedding, cached vs cache-less,
multi-position vs sequential single-position, losslessness vs plain greedy decoding; for the stochastic
rule: the generator's published known answers, the temperature softmax against distributions it must
return unchanged (scores T log p), the emitted-token distribution against the LLM's, the greedy limit,
the rejection probability; for the quality metric and the selector: hand-computed cases and
a library least-squares fit).  No function here is unpinned.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

ARCH_OPT = 0
ARCH_LLAMA = 1


# ---------------------------------------------------------------------------
# majority vote (section 3.2)
# ---------------------------------------------------------------------------

def vote_tree(drafts: Sequence[Sequence[int]], k: int, w: Sequence[float]) -> Tuple[List[int], int]:
    """Walk the token tree formed by the n drafts from the root, level by level.

    The children of the current node are the distinct tokens emitted at level t by the
    drafts that still follow the chosen path; a child's weight is the sum of the weights
    of those drafts.  The heaviest child is taken (ties: the child first reached by the
    lowest draft index).  The result is one draft's whole output; ``voted_ssm`` is the
    lowest-index draft on the final path.
    """
    n = len(drafts)
    alive = list(range(n))
    voted: List[int] = []
    for t in range(k):
        best_tok, best_w = None, None
        seen = []
        for j in alive:
            tok = int(drafts[j][t])
            if tok in seen:
                continue
            seen.append(tok)
            W = np.float32(0.0)
            for j2 in alive:
                if int(drafts[j2][t]) == tok:
                    W = np.float32(W + np.float32(w[j2]))
            if best_w is None or W > best_w:
                best_tok, best_w = tok, W
        voted.append(best_tok)
        alive = [j for j in alive if int(drafts[j][t]) == best_tok]
    return voted, (alive[0] if n > 0 else -1)


def vote_column(drafts: Sequence[Sequence[int]], k: int, w: Sequence[float]) -> Tuple[List[int], int]:
    """Per-position weighted vote over all n drafts, ignoring prefixes.  ``voted_ssm`` is the
    lowest-index draft whose whole output equals the result, or -1 when the vote spliced drafts."""
    n = len(drafts)
    voted: List[int] = []
    for t in range(k):
        best_tok, best_w = None, None
        seen = []
        for j in range(n):
            tok = int(drafts[j][t])
            if tok in seen:
                continue
            seen.append(tok)
            W = np.float32(0.0)
            for j2 in range(n):
                if int(drafts[j2][t]) == tok:
                    W = np.float32(W + np.float32(w[j2]))
            if best_w is None or W > best_w:
                best_tok, best_w = tok, W
        voted.append(best_tok)
    ssm = -1
    for j in range(n):
        if all(int(drafts[j][t]) == voted[t] for t in range(k)):
            ssm = j
            break
    return voted, ssm


def vote_batch(drafts: np.ndarray, spec_len: Sequence[int], w: Sequence[float], mode: int = 0,
               pad: int = -1) -> Tuple[np.ndarray, np.ndarray]:
    """drafts [B][n][k_max] -> voted [B][k_max] (padded with ``pad`` past k_b), voted_ssm [B]."""
    B, n, k_max = drafts.shape
    voted = np.full((B, k_max), pad, np.int32)
    ssm = np.zeros((B,), np.int32)
    fn = vote_tree if mode == 0 else vote_column
    for b in range(B):
        v, s = fn(drafts[b], int(spec_len[b]), w)
        voted[b, :len(v)] = v
        ssm[b] = s
    return voted, ssm


# ---------------------------------------------------------------------------
# decoder pieces (textbook definitions, fp64)
# ---------------------------------------------------------------------------

def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float) -> np.ndarray:
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * _f64(g) + _f64(b)


def rms_norm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(g)


def rope(v: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary position embedding on v[T][heads][hd]: element i (< hd/2) is paired with i + hd/2
    and the pair is rotated by the angle pos * base^(-2i/hd)."""
    hd = v.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=np.float64)
    inv = base ** (-2.0 * i / hd)
    ang = _f64(pos)[:, None] * inv[None, :]            # [T][half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def _linear(x: np.ndarray, W, b=None) -> np.ndarray:
    """x[M][in] times W[out][in]^T (+ b), in fp64."""
    y = x @ _f64(W).T
    if b is not None:
        y = y + _f64(b)
    return y


def _ffn(desc, L: Dict[str, np.ndarray], h: np.ndarray) -> np.ndarray:
    if desc.arch == ARCH_OPT:
        u = np.maximum(_linear(h, L["w1"], L["b1"]), 0.0)
        return _linear(u, L["w2"], L["b2"])
    F = desc.d_ffn
    gu = _linear(h, L["w1"])                            # rows [0,F) gate, [F,2F) up
    gate, up = gu[:, :F], gu[:, F:]
    silu = gate / (1.0 + np.exp(-gate))
    return _linear(silu * up, L["w2"])


def _norm(desc, x, g, b):
    if desc.arch == ARCH_OPT:
        return layer_norm(x, g, b, desc.norm_eps)
    return rms_norm(x, g, desc.norm_eps)


def _embed(desc, W, tokens: np.ndarray, pos: np.ndarray) -> np.ndarray:
    x = _f64(W["tok_emb"][tokens])
    if desc.arch == ARCH_OPT:
        x = x + _f64(W["pos_emb"][pos])
    return x


def _split_qkv(desc, L, h: np.ndarray, pos: np.ndarray):
    H, Hk, hd = desc.n_heads, desc.n_kv_heads, desc.head_dim
    qkv = _linear(h, L["wqkv"], L.get("bqkv"))
    T = h.shape[0]
    q = qkv[:, :H * hd].reshape(T, H, hd)
    k = qkv[:, H * hd:(H + Hk) * hd].reshape(T, Hk, hd)
    v = qkv[:, (H + Hk) * hd:].reshape(T, Hk, hd)
    if desc.arch == ARCH_LLAMA:
        q = rope(q, pos, desc.rope_base)
        k = rope(k, pos, desc.rope_base)
    return q, k, v


class SeqCache:
    """Contiguous (unpaged) per-sequence KV cache: K[l], V[l] are [ctx][Hkv][hd] fp64."""

    def __init__(self, n_layers: int, n_kv_heads: int, head_dim: int,
                 K: Optional[List[np.ndarray]] = None, V: Optional[List[np.ndarray]] = None):
        z = lambda: np.zeros((0, n_kv_heads, head_dim), np.float64)
        self.K = [_f64(a) for a in K] if K is not None else [z() for _ in range(n_layers)]
        self.V = [_f64(a) for a in V] if V is not None else [z() for _ in range(n_layers)]

    @property
    def ctx(self) -> int:
        return self.K[0].shape[0]

    def truncate(self, n: int) -> None:
        self.K = [a[:n] for a in self.K]
        self.V = [a[:n] for a in self.V]


def attention_cached(desc, q: np.ndarray, Kall: np.ndarray, Vall: np.ndarray, ctx: int) -> np.ndarray:
    """Multi-token attention against an existing cache.  q[T][H][hd] are the T new tokens at
    positions ctx..ctx+T-1; Kall/Vall [ctx+T][Hkv][hd] already include the new tokens' rows.
    New token j sees cache rows [0, ctx) and new rows 0..j (causal among the speculated tokens).
    Query head h reads KV head h // (H / Hkv)."""
    T, H, hd = q.shape
    G = H // desc.n_kv_heads
    out = np.zeros((T, H, hd), np.float64)
    scale = 1.0 / math.sqrt(hd)
    # visible[j][i]: key i is visible to new token j  <=>  i <= ctx + j
    visible = np.arange(ctx + T)[None, :] <= (ctx + np.arange(T))[:, None]
    for h in range(H):
        kh = h // G
        s = (q[:, h, :] @ Kall[:, kh, :].T) * scale      # [T][ctx+T]
        s = np.where(visible, s, -np.inf)
        out[:, h, :] = softmax_rows(s) @ Vall[:, kh, :]
    return out


def decoder_step(desc, W, seq_tokens: Sequence[Sequence[int]], caches: Sequence[SeqCache]) -> List[np.ndarray]:
    """Score, for every sequence b, its new tokens ``seq_tokens[b]`` (placed at positions
    ctx_b, ctx_b+1, ...) in one pass.  Appends their K/V rows to ``caches[b]`` and returns the
    logits [len(seq_tokens[b])][vocab] per sequence.  Row-wise operations run on all rows
    packed together (they are independent per row); attention runs per sequence."""
    lens = [len(t) for t in seq_tokens]
    if sum(lens) == 0:
        return [np.zeros((0, desc.vocab), np.float64) for _ in lens]
    tok = np.concatenate([np.asarray(t, np.int64) for t in seq_tokens])
    ctx0 = [c.ctx for c in caches]
    pos = np.concatenate([np.arange(c0, c0 + n, dtype=np.int64) for c0, n in zip(ctx0, lens)])
    offs = np.concatenate([[0], np.cumsum(lens)])
    x = _embed(desc, W, tok, pos)
    H, hd = desc.n_heads, desc.head_dim
    for l, L in enumerate(W["layers"]):
        h = _norm(desc, x, L["ln1_g"], L.get("ln1_b"))
        q, k, v = _split_qkv(desc, L, h, pos)
        att = np.zeros((x.shape[0], H, hd), np.float64)
        for b, c in enumerate(caches):
            lo, hi = offs[b], offs[b + 1]
            if hi == lo:
                continue
            c.K[l] = np.concatenate([c.K[l], k[lo:hi]], axis=0)
            c.V[l] = np.concatenate([c.V[l], v[lo:hi]], axis=0)
            att[lo:hi] = attention_cached(desc, q[lo:hi], c.K[l], c.V[l], ctx0[b])
        x = x + _linear(att.reshape(-1, H * hd), L["wo"], L.get("bo"))
        h = _norm(desc, x, L["ln2_g"], L.get("ln2_b"))
        x = x + _ffn(desc, L, h)
    h = _norm(desc, x, W["final_norm_g"], W.get("final_norm_b"))
    logits = _linear(h, W["lm_head"])
    return [logits[offs[b]:offs[b + 1]] for b in range(len(lens))]


def decoder_full(desc, W, tokens: Sequence[int]) -> np.ndarray:
    """Cache-less form: the whole sequence at positions 0..T-1 with a lower-triangular mask.
    Returns logits [T][vocab]."""
    tok = np.asarray(tokens, np.int64)
    T = tok.shape[0]
    pos = np.arange(T, dtype=np.int64)
    x = _embed(desc, W, tok, pos)
    H, Hk, hd = desc.n_heads, desc.n_kv_heads, desc.head_dim
    G = H // Hk
    mask = np.tril(np.ones((T, T), bool))
    for L in W["layers"]:
        h = _norm(desc, x, L["ln1_g"], L.get("ln1_b"))
        q, k, v = _split_qkv(desc, L, h, pos)
        att = np.zeros((T, H, hd), np.float64)
        for hh in range(H):
            s = (q[:, hh, :] @ k[:, hh // G, :].T) / math.sqrt(hd)
            s = np.where(mask, s, -np.inf)
            att[:, hh, :] = softmax_rows(s) @ v[:, hh // G, :]
        x = x + _linear(att.reshape(T, H * hd), L["wo"], L.get("bo"))
        h = _norm(desc, x, L["ln2_g"], L.get("ln2_b"))
        x = x + _ffn(desc, L, h)
    h = _norm(desc, x, W["final_norm_g"], W.get("final_norm_b"))
    return _linear(h, W["lm_head"])


# ---------------------------------------------------------------------------
# greedy verification, acceptance, commit (section 2.1 in its greedy case; section 4)
# ---------------------------------------------------------------------------

def greedy_tokens(logits: np.ndarray) -> np.ndarray:
    """Lowest token id attaining the row maximum."""
    return np.argmax(logits, axis=-1).astype(np.int32)


def top1_margin(logits: np.ndarray) -> np.ndarray:
    """Gap between the largest and second-largest logit of each row."""
    part = np.partition(logits, -2, axis=-1)
    return part[..., -1] - part[..., -2]


def accept(voted: Sequence[int], g: Sequence[int], k: int) -> Tuple[int, List[int]]:
    """Longest prefix of the voted draft that equals the LLM's greedy tokens.  Returns the accepted
    length a and the a+1 emitted tokens g[0..a] (the last one is the correction token when a < k,
    the bonus token when a == k)."""
    a = 0
    while a < k and int(voted[a]) == int(g[a]):
        a += 1
    return a, [int(t) for t in g[:a + 1]]


def commit(ctx: int, a: int, block_size: int) -> Tuple[int, int]:
    """Keep the cache rows of the pending token and of the a accepted drafts; everything after is
    dropped.  Returns the new context length and the number of blocks still in use."""
    new_ctx = ctx + a + 1
    return new_ctx, (new_ctx + block_size - 1) // block_size


def accept_batch(voted: np.ndarray, greedy: np.ndarray, spec_len: Sequence[int], ctx_lens: Sequence[int],
                 block_size: int, pad: int = -1):
    """Batched form of accept + commit.  voted [B][k_max], greedy [B][k_max+1]."""
    B, k_max = voted.shape
    acc = np.zeros((B,), np.int32)
    out = np.full((B, k_max + 1), pad, np.int32)
    n_out = np.zeros((B,), np.int32)
    nxt = np.zeros((B,), np.int32)
    new_ctx = np.zeros((B,), np.int32)
    blocks = np.zeros((B,), np.int32)
    for b in range(B):
        a, toks = accept(voted[b], greedy[b], int(spec_len[b]))
        acc[b] = a
        out[b, :len(toks)] = toks
        n_out[b] = len(toks)
        nxt[b] = toks[-1]
        new_ctx[b], blocks[b] = commit(int(ctx_lens[b]), a, block_size)
    return acc, out, n_out, nxt, new_ctx, blocks


def verify_step(desc, W, caches: Sequence[SeqCache], last_tok: Sequence[int], drafts: np.ndarray,
                spec_len: Sequence[int], ssm_w: Sequence[float], mode: int = 0, block_size: int = 16):
    """One whole verification step on the oracle: vote, score k_b+1 positions per sequence,
    argmax, accept, commit (the caches are truncated to the committed length)."""
    B = len(caches)
    voted, ssm = vote_batch(drafts, spec_len, ssm_w, mode)
    ctx0 = [c.ctx for c in caches]
    toks = [[int(last_tok[b])] + [int(t) for t in voted[b, :int(spec_len[b])]] for b in range(B)]
    logits = decoder_step(desc, W, toks, caches)
    k_max = drafts.shape[2]
    greedy = np.full((B, k_max + 1), -1, np.int32)
    for b in range(B):
        greedy[b, :len(toks[b])] = greedy_tokens(logits[b])
    acc, out, n_out, nxt, new_ctx, blocks = accept_batch(voted, greedy, spec_len, ctx0, block_size)
    for b, c in enumerate(caches):
        c.truncate(int(new_ctx[b]))
    return {"voted": voted, "voted_ssm": ssm, "logits": logits, "greedy": greedy, "accepted_len": acc,
            "out_tokens": out, "n_out": n_out, "next_last_tok": nxt, "ctx_lens": new_ctx,
            "blocks_in_use": blocks}


# ---------------------------------------------------------------------------
# stochastic verification (section 2.1, the general rule of which `accept` is the greedy case)
# ---------------------------------------------------------------------------

_M32 = 0xFFFFFFFF


def philox4x32(counter: Sequence[int], key: Sequence[int], rounds: int = 10) -> Tuple[int, int, int, int]:
    """Philox-4x32 counter-based generator (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as
    easy as 1, 2, 3", SC 2011): a 128-bit counter and a 64-bit key give four 32-bit words.  Each round
    multiplies words 0 and 2 by two fixed odd constants, swaps the halves of the products into the
    other lanes and mixes in the key, which advances by the golden-ratio / sqrt(3) constants."""
    c0, c1, c2, c3 = (int(c) & _M32 for c in counter)
    k0, k1 = (int(k) & _M32 for k in key)
    for _ in range(rounds):
        p0 = 0xD2511F53 * c0
        p1 = 0xCD9E8D57 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & _M32, p1 & _M32, ((p0 >> 32) ^ c3 ^ k1) & _M32, p0 & _M32
        k0 = (k0 + 0x9E3779B9) & _M32
        k1 = (k1 + 0xBB67AE85) & _M32
    return c0, c1, c2, c3


def unit_double(hi: int, lo: int) -> float:
    """53 random bits -> a double in [0, 1): the top 27 bits of `hi` and the top 26 bits of `lo`."""
    return float(((int(hi) >> 5) << 26) + (int(lo) >> 6)) / float(1 << 53)


def verify_uniforms(seed: int, step: int, b: int, j: int, consumer: int = 0) -> Tuple[float, float]:
    """The two uniform numbers position j of sequence b consumes in step `step`: the first decides
    acceptance, the second picks the replacement (or bonus) token.  Key = seed, counter = (b, j, step);
    the top byte of the counter's last word names the consumer (0 = the verifier, 1 + i = drafting SSM i),
    so that under one seed no two of them see the same numbers; steps stay below 2^56."""
    assert 0 <= step < (1 << 56) and 0 <= consumer < 256
    w = philox4x32((b, j, step & _M32, ((step >> 32) & 0xFFFFFF) | (consumer << 24)), (seed & _M32, (seed >> 32) & _M32))
    return unit_double(w[0], w[1]), unit_double(w[2], w[3])


def llm_probs(logits_row: np.ndarray, temperature: float) -> np.ndarray:
    """o(x): softmax of the LLM's scores at one position, at the given temperature, in fp64."""
    z = (_f64(logits_row) - float(np.max(logits_row))) / float(temperature)
    e = np.exp(z)
    return e / e.sum()


def sample_cdf(mass: np.ndarray, u: float) -> Tuple[int, float]:
    """Inverse-CDF sample in token order: the first token whose running sum of `mass` exceeds u times the
    total.  Also returns how far (relative to the total) the target is from the nearest running sum on
    either side of the chosen token, so that a test can tell a decision that hangs on the last bits."""
    cum = np.cumsum(_f64(mass))
    total = float(cum[-1])
    target = u * total
    v = int(np.searchsorted(cum, target, side="right"))
    if v >= len(cum):                       # rounding pushed the target to the total: last token with mass
        v = int(np.nonzero(mass > 0)[0][-1])
    below = float(cum[v - 1]) if v > 0 else -np.inf
    gap = min(abs(float(cum[v]) - target), abs(target - below)) / total
    return v, gap


def draft_sample(logits_row: np.ndarray, temperature: float, seed: int, step: int, ssm: int, b: int, t: int):
    """A drafting SSM's next token (section 2.1: the SSM predicts its tokens from its own distribution q):
    q = softmax(scores / T) rounded to fp32, which is what the verifier will be handed, and a token drawn
    from exactly those values by the inverse CDF in token order.  Returns (token, q as fp32, relative
    distance of the draw from the nearest boundary)."""
    q32 = llm_probs(logits_row, temperature).astype(np.float32)
    _, u = verify_uniforms(seed, step, b, t, consumer=1 + ssm)
    tok, gap = sample_cdf(q32.astype(np.float64), u)
    return tok, q32, gap


def accept_stochastic(voted: Sequence[int], logits: np.ndarray, draft_probs: np.ndarray, k: int,
                      temperature: float, seed: int, step: int, b: int):
    """Verification of one sequence's k speculated tokens (section 2.1).  logits [k+1][V] are the LLM's
    scores of the k+1 positions, draft_probs [k][V] the drafting SSM's distributions q_i.  Token x_i is
    kept when q_i(x_i) <= o_i(x_i); otherwise it is rejected with probability 1 - o_i(x_i)/q_i(x_i), and
    then a replacement is drawn from max(0, o_i - q_i) renormalised and everything after it is dropped.
    When all k survive, one more token is drawn from o_{k+1}.
    Returns (accepted length a, the a+1 emitted tokens, smallest relative distance of any decision taken
    from its threshold)."""
    out: List[int] = []
    margin = np.inf
    for i in range(k):
        x = int(voted[i])
        o = llm_probs(logits[i], temperature)
        q = _f64(draft_probs[i])
        u_acc, u_res = verify_uniforms(seed, step, b, i)
        if q[x] <= o[x]:
            out.append(x)
            continue
        ratio = o[x] / q[x]
        margin = min(margin, abs(u_acc - ratio))
        if u_acc < ratio:                   # rejected with probability 1 - o/q
            out.append(x)
            continue
        residual = np.maximum(0.0, o - q)
        if not residual.sum() > 0.0:        # q covers o everywhere (possible only for a q that sums above 1):
            residual = o.copy()             # the LLM's distribution without the rejected token, so that the
            residual[x] = 0.0               # replacement still differs from what it replaces
        if not residual.sum() > 0.0:        # ... and all of o sits on x: there is nothing else to emit, x stays
            out.append(x)
            continue
        tok, gap = sample_cdf(residual, u_res)
        margin = min(margin, gap)
        out.append(tok)
        return i, out, margin
    _, u_res = verify_uniforms(seed, step, b, k)
    tok, gap = sample_cdf(llm_probs(logits[k], temperature), u_res)
    out.append(tok)
    return k, out, min(margin, gap)


# ---------------------------------------------------------------------------
# speculation quality metric and weight update (section 3.2, equation ACR)
# ---------------------------------------------------------------------------

def acr_update(ssm_w: Sequence[float], voted_ssm: Sequence[int], accepted_len: Sequence[int],
               spec_len: Sequence[int], reward_threshold: float, punish_threshold: float,
               reward_factor: float, punish_factor: float,
               verified: Optional[Sequence[bool]] = None) -> Tuple[np.ndarray, np.ndarray]:
    """ACR_i = mean over the outputs whose voted SSM is i of (accepted length / speculation length);
    w_i is multiplied by the reward factor when ACR_i exceeds the reward threshold and by the punish
    factor when it falls below the punish threshold.  SSMs that won no vote keep their weight
    (their ACR is reported as NaN).  The set o_SSM_i holds verified outputs only: ``verified`` marks the
    outputs the LLM actually scored (all of them when omitted).  Returns (new weights fp32, ACR fp64)."""
    n = len(ssm_w)
    acr = np.full((n,), np.nan, np.float64)
    w = np.asarray(ssm_w, np.float32).copy()
    for i in range(n):
        rates = [float(accepted_len[b]) / float(spec_len[b]) for b in range(len(voted_ssm))
                 if int(voted_ssm[b]) == i and int(spec_len[b]) > 0 and (verified is None or bool(verified[b]))]
        if not rates:
            continue
        acr[i] = sum(rates) / len(rates)
        if acr[i] > reward_threshold:
            w[i] = np.float32(w[i] * np.float32(reward_factor))
        elif acr[i] < punish_threshold:
            w[i] = np.float32(w[i] * np.float32(punish_factor))
    return w, acr


# ---------------------------------------------------------------------------
# adaptive speculation length selector (section 3.3)
# ---------------------------------------------------------------------------

def fit_slope(y: Sequence[float]) -> float:
    """Slope of the least-squares line through (0, y_0) .. (m-1, y_{m-1}): the textbook
    sum((x - mean x)(y - mean y)) / sum((x - mean x)^2), in fp64."""
    m = len(y)
    xm = sum(float(i) for i in range(m)) / m
    ym = sum(float(v) for v in y) / m
    sxy = sum((i - xm) * (float(y[i]) - ym) for i in range(m))
    sxx = sum((i - xm) ** 2 for i in range(m))
    return sxy / sxx


class Selector:
    """Section 3.3.  ``observe(t_llm, vl)`` records t_llm / vl; once ``decision_threshold`` samples have
    been collected since the last change (reading: the text's "greater than or equal"), the fitted
    slope decides: positive -> s - s_penalty, otherwise -> s + s_reward (the listing's else branch);
    s stays inside [s_min, s_max]; the samples are dropped.  Returns the s to use next."""

    def __init__(self, s_init: int, s_min: int, s_max: int, decision_threshold: int, s_penalty: int, s_reward: int):
        self.s, self.s_min, self.s_max = s_init, s_min, s_max
        self.decision_threshold, self.s_penalty, self.s_reward = decision_threshold, s_penalty, s_reward
        self.samples: List[float] = []
        self.adjustments = 0
        self.last_slope = math.nan

    def observe(self, t_llm: float, vl: float) -> int:
        self.last_slope = math.nan
        self.samples.append(float(t_llm) / float(vl))
        if len(self.samples) >= self.decision_threshold:
            slope = fit_slope(self.samples)
            self.last_slope = slope
            self.s = self.s - self.s_penalty if slope > 0.0 else self.s + self.s_reward
            self.s = max(self.s_min, min(self.s_max, self.s))
            self.samples = []
            self.adjustments += 1
        return self.s
