"""Seeded synthetic inputs for the verification path (shapes, weights, KV pages, drafts).

This module serves both the HIP path and the CPU oracle with *inputs only*: it
holds none of the method's arithmetic (no vote, no decoder math, no argmax, no
acceptance).  Everything is driven by numpy's counter-based Philox generator
keyed by (seed, stream ids), so any tensor is reproducible on its own.

Conventions
-----------
* A tensor that both sides consume is generated once, here, and handed over
  bit for bit.  In bf16 models the matrices and embeddings are rounded to
  bf16 (round-to-nearest-even) here; the oracle receives the rounded values
  widened to fp32/fp64, the device receives the 16-bit patterns.
* Matrices are ``[out][in]`` row-major (the contraction index is contiguous).
* Paged KV cache, per layer (block = 16 tokens by default):
    K pages: ``[num_blocks][n_kv_heads][head_dim/8][block_size][8]``
    V pages: ``[num_blocks][n_kv_heads][head_dim][block_size]``
  Token ``p`` of a sequence lives in block ``block_table[p // block_size]`` at
  offset ``p % block_size`` (the logical block id + offset per token of the
  paper's section 4).
"""
from __future__ import annotations

import concurrent.futures
import dataclasses
from dataclasses import dataclass
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

ARCH_OPT = 0
ARCH_LLAMA = 1
DT_F32 = 0
DT_BF16 = 1


@dataclass(frozen=True)
class ModelDesc:
    arch: int          # ARCH_OPT | ARCH_LLAMA
    dtype: int         # DT_F32 | DT_BF16 (storage of matrices, embeddings, KV pages)
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    max_pos: int
    norm_eps: float = 1e-5
    rope_base: float = 10000.0

    @property
    def n_qkv(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def w1_rows(self) -> int:
        return self.d_ffn * (2 if self.arch == ARCH_LLAMA else 1)

    def with_layers(self, n_layers: int) -> "ModelDesc":
        return dataclasses.replace(self, n_layers=n_layers)

    def gemm_params(self) -> int:
        """Matrix parameters touched once per step (projections + LM head)."""
        per_layer = (self.n_qkv * self.d_model + self.d_model * self.n_heads * self.head_dim
                     + self.w1_rows * self.d_model + self.d_model * self.d_ffn)
        return per_layer * self.n_layers + self.vocab * self.d_model


@dataclass(frozen=True)
class Workload:
    name: str
    desc: ModelDesc
    batch: int
    ctx_lo: int        # context length range (inclusive); lo == hi for fixed contexts
    ctx_hi: int
    k_lo: int          # speculation length range (inclusive)
    k_hi: int
    n_drafts: int
    p_corrupt: float
    block_size: int = 16
    seed: int = 1234


OPT_TINY = ModelDesc(ARCH_OPT, DT_F32, 2, 256, 4, 4, 64, 1024, 4096, 2048)
OPT_13B = ModelDesc(ARCH_OPT, DT_BF16, 40, 5120, 40, 40, 128, 20480, 50272, 2048)
LLAMA2_70B = ModelDesc(ARCH_LLAMA, DT_BF16, 80, 8192, 64, 8, 128, 28672, 32000, 4096)
# attention-only workload: one layer of the 70B attention shape, long context
LLAMA2_70B_ATTN = dataclasses.replace(LLAMA2_70B, n_layers=1, max_pos=8192)
# the shape of the small speculative models the paper pairs with Llama-2-70B (section 5.1: Llama-160M)
LLAMA_160M = dataclasses.replace(LLAMA2_70B, n_layers=12, d_model=768, n_heads=12, n_kv_heads=12, head_dim=64, d_ffn=3072)

WORKLOADS: Tuple[Workload, ...] = (
    Workload("opt-tiny-fp32-b1-k4", OPT_TINY, 1, 64, 64, 4, 4, 3, 0.0, seed=1234),
    Workload("opt13b-bf16-b8-ctx512-k4", OPT_13B, 8, 512, 512, 4, 4, 4, 0.3, seed=1235),
    Workload("llama2-70b-bf16-b16-ctx1024-k8", LLAMA2_70B, 16, 1024, 1024, 8, 8, 4, 0.2, seed=1236),
    Workload("llama2-70b-bf16-b64-ragged-paged", LLAMA2_70B, 64, 256, 2048, 1, 16, 5, 0.25, seed=1237),
    Workload("llama2-70b-attn-b32-ctx8192-q16", LLAMA2_70B_ATTN, 32, 8176, 8176, 15, 15, 1, 0.0, seed=1238),
)


# --------------------------------------------------------------------------
# random streams and bf16 bit handling
# --------------------------------------------------------------------------

def stream(seed: int, *ids: int) -> np.random.Generator:
    """Independent Philox stream for (seed, ids...)."""
    ss = np.random.SeedSequence([int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF, *[int(i) for i in ids]])
    return np.random.Generator(np.random.Philox(ss))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 with round-to-nearest-even; returns the uint16 patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 patterns to fp32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def storage_round(x: np.ndarray, dtype: int) -> np.ndarray:
    """Values as the model stores them: identity in fp32 models, bf16-rounded (kept as fp32) otherwise."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == DT_BF16:
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    return x


_CHUNK = 1 << 22      # elements per independently seeded chunk (fixed: it is part of the recipe)
_THREADS = 8


def _normal(key: Sequence[int], shape, std: float, mean: float = 0.0, dtype: int = DT_F32) -> np.ndarray:
    """N(mean, std) tensor for the stream ``key`` = (seed, ids...), rounded to the storage type.  The
    tensor is cut into fixed-size chunks, each drawn from its own Philox stream (key + chunk index), so
    the values do not depend on how many threads fill it."""
    n = int(np.prod(shape))
    out = np.empty((n,), np.float32)

    def fill(c: int) -> None:
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        v = stream(*key, c).standard_normal(size=hi - lo, dtype=np.float32)
        v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[lo:hi] = storage_round(v, dtype)

    n_chunks = (n + _CHUNK - 1) // _CHUNK
    if n_chunks <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with concurrent.futures.ThreadPoolExecutor(_THREADS) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


# --------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------

MATRIX_KEYS = ("wqkv", "wo", "w1", "w2")
VECTOR_KEYS_OPT = ("ln1_g", "ln1_b", "bqkv", "bo", "ln2_g", "ln2_b", "b1", "b2")
VECTOR_KEYS_LLAMA = ("ln1_g", "ln2_g")


def make_weights(desc: ModelDesc, seed: int, std: float = 0.02) -> Dict[str, object]:
    """Random-init parameters: matrices, embeddings and biases N(0, std); norm gains 1+N(0, std);
    norm shifts N(0, std).  Matrices/embeddings are already rounded to the storage type and
    held as fp32; vectors (gains, shifts, biases) are fp32 in every model.

    Returns {"tok_emb", "pos_emb"(OPT), "final_norm_g", "final_norm_b"(OPT), "lm_head",
             "layers": [ {per-layer tensors} ]}.
    """
    d, hd = desc.d_model, desc.head_dim
    mat = lambda shape, *ids: _normal((seed, 100, *ids), shape, std, 0.0, desc.dtype)
    vec = lambda shape, mean, *ids: _normal((seed, 100, *ids), shape, std, mean, DT_F32)
    W: Dict[str, object] = {}
    W["tok_emb"] = mat((desc.vocab, d), 0)
    W["lm_head"] = mat((desc.vocab, d), 1)
    W["final_norm_g"] = vec((d,), 1.0, 2)
    if desc.arch == ARCH_OPT:
        W["pos_emb"] = mat((desc.max_pos, d), 3)
        W["final_norm_b"] = vec((d,), 0.0, 4)
    layers = []
    for l in range(desc.n_layers):
        L: Dict[str, np.ndarray] = {}
        L["wqkv"] = mat((desc.n_qkv, d), 10, l)
        L["wo"] = mat((d, desc.n_heads * hd), 11, l)
        L["w1"] = mat((desc.w1_rows, d), 12, l)
        L["w2"] = mat((d, desc.d_ffn), 13, l)
        L["ln1_g"] = vec((d,), 1.0, 14, l)
        L["ln2_g"] = vec((d,), 1.0, 15, l)
        if desc.arch == ARCH_OPT:
            L["ln1_b"] = vec((d,), 0.0, 16, l)
            L["ln2_b"] = vec((d,), 0.0, 17, l)
            L["bqkv"] = vec((desc.n_qkv,), 0.0, 18, l)
            L["bo"] = vec((d,), 0.0, 19, l)
            L["b1"] = vec((desc.d_ffn,), 0.0, 20, l)
            L["b2"] = vec((d,), 0.0, 21, l)
        layers.append(L)
    W["layers"] = layers
    return W


# --------------------------------------------------------------------------
# paged KV cache
# --------------------------------------------------------------------------

@dataclass
class PagedKV:
    """Host image of a paged KV cache.  k_pages[l]: [num_blocks][Hkv][hd/8][bs][8];
    v_pages[l]: [num_blocks][Hkv][hd][bs]; both fp32 holding storage-rounded values."""
    block_size: int
    num_blocks: int
    max_blocks_per_seq: int
    block_tables: np.ndarray          # int32 [B][max_blocks_per_seq], -1 = unmapped
    ctx_lens: np.ndarray              # int32 [B]
    k_pages: List[np.ndarray]
    v_pages: List[np.ndarray]


def blocks_needed(n_tokens: int, block_size: int) -> int:
    return (int(n_tokens) + block_size - 1) // block_size


def make_block_tables(ctx_lens: Sequence[int], spec_lens: Sequence[int], block_size: int, seed: int,
                      scatter: bool = True, spare_blocks: int = 0) -> Tuple[np.ndarray, int]:
    """Map enough blocks for ctx_b + k_b + 1 tokens of every sequence.  With ``scatter`` the physical
    block ids are a random permutation, so consecutive logical blocks are far apart in memory."""
    B = len(ctx_lens)
    need = [blocks_needed(int(c) + int(k) + 1, block_size) for c, k in zip(ctx_lens, spec_lens)]
    mb = max(need) if need else 1
    total = int(sum(need)) + int(spare_blocks)
    ids = np.arange(total, dtype=np.int32)
    if scatter:
        ids = stream(seed, 200).permutation(total).astype(np.int32)
    bt = np.full((B, mb), -1, dtype=np.int32)
    at = 0
    for b in range(B):
        bt[b, :need[b]] = ids[at:at + need[b]]
        at += need[b]
    return bt, total


def make_paged_kv(desc: ModelDesc, ctx_lens: Sequence[int], spec_lens: Sequence[int], seed: int,
                  block_size: int = 16, scatter: bool = True, fill: bool = True, std: float = 1.0) -> PagedKV:
    """Synthetic cache: every mapped slot (including the not-yet-valid ones past ctx_b) gets
    N(0, std) values rounded to the storage type, so stale data is never conveniently zero."""
    bt, nb = make_block_tables(ctx_lens, spec_lens, block_size, seed, scatter)
    hd, hk = desc.head_dim, desc.n_kv_heads
    ks, vs = [], []
    for l in range(desc.n_layers):
        if fill:
            k = _normal((seed, 201, l), (nb, hk, hd // 8, block_size, 8), std, 0.0, desc.dtype)
            v = _normal((seed, 202, l), (nb, hk, hd, block_size), std, 0.0, desc.dtype)
        else:
            k = np.zeros((nb, hk, hd // 8, block_size, 8), np.float32)
            v = np.zeros((nb, hk, hd, block_size), np.float32)
        ks.append(k)
        vs.append(v)
    return PagedKV(block_size, nb, bt.shape[1], bt, np.asarray(ctx_lens, np.int32).copy(), ks, vs)


def gather_sequence_kv(kv: PagedKV, layer: int, b: int, n_tokens: int) -> Tuple[np.ndarray, np.ndarray]:
    """Layout conversion only: the first n_tokens cached rows of sequence b as contiguous
    K[n_tokens][Hkv][hd], V[n_tokens][Hkv][hd]."""
    bs = kv.block_size
    kp, vp = kv.k_pages[layer], kv.v_pages[layer]
    hk = kp.shape[1]
    hd = vp.shape[2]
    K = np.empty((n_tokens, hk, hd), kp.dtype)
    V = np.empty((n_tokens, hk, hd), vp.dtype)
    for lb in range(blocks_needed(n_tokens, bs)):
        pb = int(kv.block_tables[b, lb])
        lo = lb * bs
        n = min(bs, n_tokens - lo)
        # K page [Hkv][hd/8][bs][8] -> [bs][Hkv][hd]
        K[lo:lo + n] = kp[pb].transpose(2, 0, 1, 3).reshape(bs, hk, hd)[:n]
        # V page [Hkv][hd][bs] -> [bs][Hkv][hd]
        V[lo:lo + n] = vp[pb].transpose(2, 0, 1)[:n]
    return K, V


def scatter_sequence_kv(kv: PagedKV, layer: int, b: int, start: int, K: np.ndarray, V: np.ndarray) -> None:
    """Layout conversion only: write contiguous rows K/V[t] to logical positions start+t of sequence b."""
    bs = kv.block_size
    for t in range(K.shape[0]):
        p = start + t
        pb = int(kv.block_tables[b, p // bs])
        off = p % bs
        hk, hd = K.shape[1], K.shape[2]
        kv.k_pages[layer][pb, :, :, off, :] = K[t].reshape(hk, hd // 8, 8)
        kv.v_pages[layer][pb, :, :, off] = V[t]


# --------------------------------------------------------------------------
# drafts, contexts, speculation lengths
# --------------------------------------------------------------------------

def draw_ctx_lens(w: Workload, gen: Optional[np.random.Generator] = None) -> np.ndarray:
    gen = gen or stream(w.seed, 300)
    if w.ctx_lo == w.ctx_hi:
        return np.full((w.batch,), w.ctx_lo, np.int32)
    return gen.integers(w.ctx_lo, w.ctx_hi + 1, size=w.batch).astype(np.int32)


def draw_spec_lens(w: Workload, gen: Optional[np.random.Generator] = None) -> np.ndarray:
    gen = gen or stream(w.seed, 301)
    if w.k_lo == w.k_hi:
        return np.full((w.batch,), w.k_lo, np.int32)
    return gen.integers(w.k_lo, w.k_hi + 1, size=w.batch).astype(np.int32)


def corrupt_token(tok: int, vocab: int, gen: np.random.Generator) -> int:
    """A token drawn uniformly from the vocabulary without ``tok``."""
    r = int(gen.integers(0, vocab - 1))
    return r + 1 if r >= tok else r


def drafts_config0(greedy: Sequence[int], vocab: int, gen: np.random.Generator) -> Tuple[np.ndarray, Dict[str, int]]:
    """Three drafts: the greedy continuation, that continuation with one uniformly drawn position
    replaced by a different token, and a uniform-random one; order shuffled.  Returns the drafts
    [3][k] and where each kind landed plus the corrupted position."""
    k = len(greedy)
    good = np.asarray(greedy, np.int32)
    bad = good.copy()
    pos = int(gen.integers(0, k))
    bad[pos] = corrupt_token(int(good[pos]), vocab, gen)
    rnd = gen.integers(0, vocab, size=k).astype(np.int32)
    order = gen.permutation(3)
    rows = [good, bad, rnd]
    drafts = np.stack([rows[i] for i in order]).astype(np.int32)
    info = {"greedy_at": int(np.where(order == 0)[0][0]), "corrupt_at": int(np.where(order == 1)[0][0]),
            "random_at": int(np.where(order == 2)[0][0]), "corrupt_pos": pos}
    return drafts, info


def drafts_corrupted(greedy: Sequence[int], n: int, p: float, vocab: int, gen: np.random.Generator) -> np.ndarray:
    """n drafts, each the greedy continuation with every position independently replaced, with
    probability p, by a uniformly drawn different token."""
    k = len(greedy)
    out = np.empty((n, k), np.int32)
    for j in range(n):
        for t in range(k):
            g = int(greedy[t])
            out[j, t] = corrupt_token(g, vocab, gen) if gen.random() < p else g
    return out


def pack_drafts(per_seq: Sequence[np.ndarray], k_max: int, pad: int = -1) -> np.ndarray:
    """[B] arrays of [n][k_b] -> one int32 [B][n][k_max] padded with ``pad``."""
    B = len(per_seq)
    n = per_seq[0].shape[0]
    out = np.full((B, n, k_max), pad, np.int32)
    for b, d in enumerate(per_seq):
        out[b, :, :d.shape[1]] = d
    return out
