"""Pins for the oracle's decoder forward (no GPU): a PyTorch-CPU fp64 model assembled from
library routines, closed forms, cached vs cache-less, one multi-position pass vs sequential
single-position passes."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth

TINY_OPT = synth.ModelDesc(synth.ARCH_OPT, synth.DT_F32, 2, 64, 4, 4, 16, 128, 97, 64)
TINY_LLAMA = synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_F32, 2, 64, 8, 2, 8, 96, 101, 64)
TINY_LLAMA_BF16 = synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 1, 64, 4, 2, 16, 96, 53, 64)


def _torch_model(desc, W, tokens):
    """The same network from torch.nn.functional pieces in fp64 (library layer_norm / rms_norm /
    linear / scaled_dot_product_attention / silu / relu; rotary embedding as a complex product)."""
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    tok = torch.tensor(tokens, dtype=torch.long)
    T = len(tokens)
    H, Hk, hd, d = desc.n_heads, desc.n_kv_heads, desc.head_dim, desc.d_model
    x = F.embedding(tok, t(W["tok_emb"]))
    if desc.arch == synth.ARCH_OPT:
        x = x + t(W["pos_emb"])[:T]
    def norm(x, g, b):
        if desc.arch == synth.ARCH_OPT:
            return F.layer_norm(x, (d,), t(g), t(b), desc.norm_eps)
        return F.rms_norm(x, (d,), t(g), desc.norm_eps)
    def rot(v):   # v [T][h][hd]: (v_i + i v_{i+hd/2}) * exp(i * pos * base^(-2i/hd))
        half = hd // 2
        z = torch.complex(v[..., :half], v[..., half:])
        inv = torch.tensor([desc.rope_base ** (-2.0 * i / hd) for i in range(half)], dtype=torch.float64)
        ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
        z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)
    for L in W["layers"]:
        h = norm(x, L["ln1_g"], L.get("ln1_b"))
        qkv = F.linear(h, t(L["wqkv"]), t(L["bqkv"]) if "bqkv" in L else None)
        q, k, v = torch.split(qkv, [H * hd, Hk * hd, Hk * hd], dim=-1)
        q, k, v = q.view(T, H, hd), k.view(T, Hk, hd), v.view(T, Hk, hd)
        if desc.arch == synth.ARCH_LLAMA:
            q, k = rot(q), rot(k)
        k = k.repeat_interleave(H // Hk, dim=1)
        v = v.repeat_interleave(H // Hk, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        a = a.transpose(0, 1).reshape(T, H * hd)
        x = x + F.linear(a, t(L["wo"]), t(L["bo"]) if "bo" in L else None)
        h = norm(x, L["ln2_g"], L.get("ln2_b"))
        if desc.arch == synth.ARCH_OPT:
            x = x + F.linear(F.relu(F.linear(h, t(L["w1"]), t(L["b1"]))), t(L["w2"]), t(L["b2"]))
        else:
            gu = F.linear(h, t(L["w1"]))
            x = x + F.linear(F.silu(gu[:, :desc.d_ffn]) * gu[:, desc.d_ffn:], t(L["w2"]))
    h = norm(x, W["final_norm_g"], W.get("final_norm_b"))
    return F.linear(h, t(W["lm_head"])).numpy()


@pytest.mark.parametrize("desc", [TINY_OPT, TINY_LLAMA, TINY_LLAMA_BF16], ids=["opt", "llama-gqa", "llama-bf16w"])
def test_full_forward_matches_torch_library_model(desc):
    W = synth.make_weights(desc, seed=5, std=0.2)      # large std: every term matters
    tokens = synth.stream(5, 1).integers(0, desc.vocab, size=23).tolist()
    want = _torch_model(desc, W, tokens)
    got = orc.decoder_full(desc, W, tokens)
    assert np.abs(got - want).max() < 1e-9 * max(1.0, np.abs(want).max())
    # and the cached path, fed in uneven pieces (prefill 7, then 5 at once, then 1, then 10)
    cache = orc.SeqCache(desc.n_layers, desc.n_kv_heads, desc.head_dim)
    rows = []
    at = 0
    for n in (7, 5, 1, 10):
        rows.append(orc.decoder_step(desc, W, [tokens[at:at + n]], [cache])[0])
        at += n
    got2 = np.concatenate(rows)
    assert cache.ctx == 23
    assert np.abs(got2 - want).max() < 1e-9 * max(1.0, np.abs(want).max())


@pytest.mark.parametrize("desc", [TINY_OPT, TINY_LLAMA], ids=["opt", "llama-gqa"])
def test_one_pass_equals_sequential_single_token_decodes(desc):
    # verifying k+1 positions in one pass == k+1 sequential single-token decodes
    W = synth.make_weights(desc, seed=9, std=0.1)
    g = synth.stream(9, 2)
    prompts = [g.integers(0, desc.vocab, size=n).tolist() for n in (11, 4, 19)]
    news = [g.integers(0, desc.vocab, size=n).tolist() for n in (5, 1, 8)]
    def prefill():
        cs = [orc.SeqCache(desc.n_layers, desc.n_kv_heads, desc.head_dim) for _ in prompts]
        orc.decoder_step(desc, W, prompts, cs)
        return cs
    cs = prefill()
    one = orc.decoder_step(desc, W, news, cs)
    cs2 = prefill()
    for b in range(3):
        for j, tok in enumerate(news[b]):
            toks = [[] for _ in range(3)]
            toks[b] = [tok]
            row = orc.decoder_step(desc, W, toks, cs2)[b]
            assert np.abs(row[0] - one[b][j]).max() < 1e-10
    for b in range(3):
        for l in range(desc.n_layers):
            assert np.abs(cs[b].K[l] - cs2[b].K[l]).max() < 1e-12
            assert np.abs(cs[b].V[l] - cs2[b].V[l]).max() < 1e-12


def test_batched_rows_do_not_interact():
    desc = TINY_LLAMA
    W = synth.make_weights(desc, seed=2, std=0.1)
    g = synth.stream(2, 3)
    seqs = [g.integers(0, desc.vocab, size=n).tolist() for n in (6, 9, 3)]
    together = orc.decoder_step(desc, W, seqs, [orc.SeqCache(2, 2, 8) for _ in seqs])
    for b, s in enumerate(seqs):
        alone = orc.decoder_full(desc, W, s)
        assert np.abs(alone - together[b]).max() < 1e-10


def test_attention_bruteforce_scalar_loops():
    # scalar-loop definition: o_j = sum_i softmax_i(q_j.k_i/sqrt(hd)) v_i over i <= ctx + j, GQA head map
    desc = TINY_LLAMA
    g = np.random.default_rng(0)
    ctx, T, H, Hk, hd = 5, 3, desc.n_heads, desc.n_kv_heads, desc.head_dim
    q = g.standard_normal((T, H, hd))
    K = g.standard_normal((ctx + T, Hk, hd))
    V = g.standard_normal((ctx + T, Hk, hd))
    got = orc.attention_cached(desc, q, K, V, ctx)
    for h in range(H):
        kh = h // (H // Hk)
        for j in range(T):
            n = ctx + j + 1
            s = [sum(q[j, h, e] * K[i, kh, e] for e in range(hd)) / math.sqrt(hd) for i in range(n)]
            m = max(s)
            p = [math.exp(v - m) for v in s]
            z = sum(p)
            for e in range(hd):
                want = sum(p[i] / z * V[i, kh, e] for i in range(n))
                assert abs(got[j, h, e] - want) < 1e-12


def test_norm_closed_forms():
    x = np.full((1, 8), 3.0)
    g = np.arange(1, 9, dtype=np.float64)
    # RMSNorm of a constant vector c: c / sqrt(c^2 + eps) * g
    assert np.allclose(orc.rms_norm(x, g, 1e-5), 3.0 / math.sqrt(9.0 + 1e-5) * g, rtol=0, atol=1e-15)
    # LayerNorm of a constant vector: the shift alone
    b = np.linspace(-1, 1, 8)
    assert np.allclose(orc.layer_norm(x, g, b, 1e-5), b, atol=1e-15)
    # LayerNorm of (+a, -a, ...): mean 0, var a^2
    y = np.array([[2.0, -2.0] * 4])
    assert np.allclose(orc.layer_norm(y, np.ones(8), np.zeros(8), 0.0), y / 2.0, atol=1e-15)
    # eps sits inside the square root
    assert np.allclose(orc.rms_norm(np.zeros((1, 8)) + 1e-3, np.ones(8), 1.0), 1e-3 / math.sqrt(1e-6 + 1.0))


def test_rope_closed_forms():
    g = np.random.default_rng(1)
    hd = 16
    v = g.standard_normal((4, 3, hd))
    # position 0 is the identity
    assert np.array_equal(orc.rope(v, np.zeros(4), 10000.0), v)
    # pair (i, i+hd/2) turns by pos * base^(-2i/hd): check one element by hand
    pos = np.array([3, 7, 11, 2])
    r = orc.rope(v, pos, 10000.0)
    i = 5
    th = 7 * 10000.0 ** (-2.0 * i / hd)
    assert abs(r[1, 2, i] - (v[1, 2, i] * math.cos(th) - v[1, 2, i + 8] * math.sin(th))) < 1e-14
    assert abs(r[1, 2, i + 8] - (v[1, 2, i + 8] * math.cos(th) + v[1, 2, i] * math.sin(th))) < 1e-14
    # a rotation: norms are kept, and <rope(q,m), rope(k,n)> depends on m - n only
    assert np.allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(v, axis=-1))
    q, k = g.standard_normal((1, 1, hd)), g.standard_normal((1, 1, hd))
    d1 = (orc.rope(q, np.array([9]), 10000.0) * orc.rope(k, np.array([4]), 10000.0)).sum()
    d2 = (orc.rope(q, np.array([25]), 10000.0) * orc.rope(k, np.array([20]), 10000.0)).sum()
    assert abs(d1 - d2) < 1e-12


def test_zero_weights_give_bias_only_logits():
    desc = TINY_OPT
    W = synth.make_weights(desc, seed=1)
    for L in W["layers"]:
        for key in ("wqkv", "wo", "w1", "w2"):
            L[key] = np.zeros_like(L[key])
    W["lm_head"] = np.zeros_like(W["lm_head"])
    assert np.array_equal(orc.decoder_full(desc, W, [1, 2, 3]), np.zeros((3, desc.vocab)))


def test_one_hot_attention_copies_the_value_row():
    # one head, huge score on one key: the output is that key's value row
    class D: n_kv_heads = 1
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 1.0
    K = np.zeros((6, 1, 4)); K[2, 0, 0] = 1e4
    V = np.arange(24, dtype=np.float64).reshape(6, 1, 4)
    out = orc.attention_cached(D, q, K, V, 5)
    assert np.allclose(out[0, 0], V[2, 0])
    # causal among the new tokens: with ctx=3, new token 0 must not see key 4
    K2 = np.zeros((6, 1, 4)); K2[4, 0, 0] = 1e4
    q2 = np.zeros((3, 1, 4)); q2[:, 0, 0] = 1.0
    out2 = orc.attention_cached(D, q2, K2, V, 3)
    assert np.allclose(out2[0, 0], V[:4, 0].mean(axis=0))       # sees keys 0..3, all scores 0
    assert np.allclose(out2[1, 0], V[4, 0])                     # sees key 4
    assert np.allclose(out2[2, 0], V[4, 0])
