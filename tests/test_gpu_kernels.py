"""GPU parity of the integer kernels and of the two hot kernels at their own shapes, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2402_15678_amd import binding, harness
    return harness, binding


def _dev(a, dt=torch.int32):
    return torch.tensor(np.asarray(a), dtype=dt, device="cuda:0")


# ---------------------------------------------------------------------------- vote
@pytest.mark.parametrize("B,n,k_max,V,mode", [(1, 3, 4, 4096, 0), (16, 4, 8, 5, 0), (64, 5, 16, 3, 0), (64, 5, 16, 3, 1),
                                              (257, 7, 3, 2, 0), (5, 64, 6, 4, 0), (3, 1, 9, 10, 1), (4, 2, 0, 10, 0)])
def test_vote_bit_exact(hb, B, n, k_max, V, mode):
    g = synth.stream(77, B, n, k_max, mode)
    w = (g.random(n) + 0.25).astype(np.float32)
    if B % 2 == 0:
        w = np.ones(n, np.float32)                                    # unit weights: plenty of exact ties
    _check_vote(hb, g, B, n, k_max, V, mode, w)


def test_vote_random_shapes_bit_exact(hb):
    """Forty drawn shapes (batch, drafts, length, alphabet, mode) with weights from a small set of exactly
    representable values, so that weighted ties between branches are common."""
    g = synth.stream(177)
    for _ in range(40):
        B, n, k_max = int(g.integers(1, 81)), int(g.integers(1, 9)), int(g.integers(0, 17))
        V, mode = int(g.integers(2, 7)), int(g.integers(0, 2))
        w = g.choice(np.asarray([0.5, 1.0, 1.5, 2.0], np.float32), size=n)
        _check_vote(hb, g, B, n, k_max, V, mode, w)


def _check_vote(hb, g, B, n, k_max, V, mode, w):
    harness, binding = hb
    drafts = g.integers(0, V, size=(B, n, max(1, k_max))).astype(np.int32)[:, :, :k_max]
    drafts = np.ascontiguousarray(drafts)
    spec = g.integers(0, k_max + 1, size=B).astype(np.int32)
    spec[0] = k_max
    want_v, want_s = orc.vote_batch(drafts.reshape(B, n, k_max), spec, w, mode)
    voted = torch.full((B, max(1, k_max)), -9, dtype=torch.int32, device="cuda:0")
    ssm = torch.full((B,), -9, dtype=torch.int32, device="cuda:0")
    st = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    d_dev = _dev(drafts.reshape(-1) if drafts.size else np.zeros(1))
    spec_d, w_d = _dev(spec), _dev(w, torch.float32)          # named: the buffers must outlive the call
    binding.mn_mv_vote(None, d_dev.data_ptr(), spec_d.data_ptr(), w_d.data_ptr(), B, n, k_max,
                       mode, voted.data_ptr(), ssm.data_ptr(), st.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    assert st.item() == 0
    if k_max:
        assert np.array_equal(voted.cpu().numpy().reshape(-1)[:B * k_max].reshape(B, k_max), want_v)
    assert np.array_equal(ssm.cpu().numpy(), want_s)


def test_vote_paper_example_and_bad_spec_len(hb):
    harness, binding = hb
    drafts = _dev([[[1, 3], [1, 4], [2, 5]]])
    voted = torch.zeros((1, 2), dtype=torch.int32, device="cuda:0")
    ssm = torch.zeros((1,), dtype=torch.int32, device="cuda:0")
    st = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    two, three = _dev([2]), _dev([3])
    for w, want, ws in [([3, 2, 4], [1, 3], 0), ([2, 3, 4], [1, 4], 1), ([1, 1, 3], [2, 5], 2)]:
        w_d = _dev(w, torch.float32)
        binding.mn_mv_vote(None, drafts.data_ptr(), two.data_ptr(), w_d.data_ptr(), 1, 3, 2, 0,
                           voted.data_ptr(), ssm.data_ptr(), st.data_ptr(), harness.stream_ptr())
        torch.cuda.synchronize()
        assert voted.cpu().tolist() == [want] and ssm.item() == ws
    w_d = _dev([1, 1, 1], torch.float32)
    binding.mn_mv_vote(None, drafts.data_ptr(), three.data_ptr(), w_d.data_ptr(), 1, 3, 2, 0,
                       voted.data_ptr(), ssm.data_ptr(), st.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    assert st.item() == binding.MN_DEV_DRAFTS and voted.cpu().tolist() == [[-1, -1]] and ssm.item() == -1


# ---------------------------------------------------------------------------- accept + commit
@pytest.mark.parametrize("B,k_max", [(1, 4), (16, 8), (64, 16), (300, 5), (7, 0)])
def test_accept_commit_bit_exact(hb, B, k_max):
    _check_accept(hb, synth.stream(78, B, k_max), B, k_max)


def test_accept_commit_drawn_shapes_bit_exact(hb):
    g = synth.stream(178)
    for _ in range(30):
        _check_accept(hb, g, int(g.integers(1, 130)), int(g.integers(0, 17)))


def _check_accept(hb, g, B, k_max):
    harness, binding = hb
    spec = g.integers(0, k_max + 1, size=B).astype(np.int32)
    spec[0] = k_max
    greedy = g.integers(0, 50, size=(B, k_max + 1)).astype(np.int32)
    voted = np.full((B, max(1, k_max)), -1, np.int32)
    for b in range(B):
        a = int(g.integers(0, spec[b] + 1))                          # planted accepted length
        voted[b, :spec[b]] = greedy[b, :spec[b]]
        if a < spec[b]:
            voted[b, a] = greedy[b, a] + 1
            voted[b, a + 1:spec[b]] = g.integers(0, 50, size=max(0, spec[b] - a - 1))
        greedy[b, spec[b] + 1:] = -1
    ctx = g.integers(0, 200, size=B).astype(np.int32)
    acc, out, n_out, nxt, new_ctx, blocks = orc.accept_batch(voted[:, :k_max], greedy, spec, ctx, 16)
    ctx_d = _dev(ctx)
    kv = binding.KV(None, None, 16, 64, 32, None, ctx_d.data_ptr())
    o = {k: torch.full(s, -9, dtype=torch.int32, device="cuda:0") for k, s in
         [("acc", (B,)), ("out", (B, k_max + 1)), ("n_out", (B,)), ("nxt", (B,)), ("blocks", (B,))]}
    st = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    voted_d, greedy_d, spec_d = _dev(voted), _dev(greedy), _dev(spec)
    binding.mn_accept_and_commit(None, voted_d.data_ptr(), greedy_d.data_ptr(), spec_d.data_ptr(), B, k_max, kv,
                                 o["acc"].data_ptr(), o["out"].data_ptr(), o["n_out"].data_ptr(), o["nxt"].data_ptr(),
                                 o["blocks"].data_ptr(), st.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    assert st.item() == 0
    for key, want in [("acc", acc), ("out", out), ("n_out", n_out), ("nxt", nxt), ("blocks", blocks)]:
        assert np.array_equal(o[key].cpu().numpy(), want), key
    assert np.array_equal(ctx_d.cpu().numpy(), new_ctx)


# ---------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M,N,K,split", [(5, 256, 256, 1), (40, 5120, 5120, 0), (144, 8192, 8192, 0), (144, 1000, 1024, 4),
                                         (17, 50272, 512, 1), (144, 10240, 8192, 2), (200, 3072, 2048, 0),
                                         (608, 2048, 8192, 0), (1, 64, 128, 1), (144, 8192, 28672, 0), (144, 640, 8192, 16),
                                         # the many-rows kernel: one row past the streaming kernel's limit, exact and
                                         # ragged row blocks, a column count short of a 256-column group, one k block,
                                         # forced splits, vocabulary-sized N
                                         (145, 384, 256, 0), (320, 10240, 512, 0), (321, 130, 128, 1), (700, 1000, 1024, 3),
                                         (631, 32000, 512, 2), (1024, 512, 2048, 4)])
def test_proj_gemm_matches_fp64(hb, M, N, K, split):
    harness, binding = hb
    g = synth.stream(79, M, N, K)
    a = g.standard_normal((M, K), dtype=np.float32).astype(np.float16).astype(np.float32)   # fp16 activations
    w = synth.storage_round(g.standard_normal((N, K), dtype=np.float32) * 0.05, synth.DT_BF16)
    bias = g.standard_normal(N).astype(np.float32)
    a_d, w_d = harness.to_device_act(a, synth.DT_BF16), harness.pack_matrix(harness.to_device(w, synth.DT_BF16))
    b_d = torch.from_numpy(bias).cuda()
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.empty((16 * M * N * 4 + 256,), dtype=torch.uint8, device="cuda:0")
    binding.mn_proj_gemm(None, a_d.data_ptr(), w_d.data_ptr(), b_d.data_ptr(), out.data_ptr(), M, N, K, split,
                         ws.data_ptr(), ws.numel(), harness.stream_ptr())
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # the oracle's linear step: x W^T + b in fp64, every output element (in column chunks: the fp64 copy of a
    # 8192 x 28672 matrix would take 2 GB at once)
    a64 = a.astype(np.float64)
    err = 0.0
    for c0 in range(0, N, 2048):
        want = orc._linear(a64, w[c0:c0 + 2048], bias[c0:c0 + 2048])
        err = max(err, float(np.abs(got[:, c0:c0 + 2048] - want).max()))
    # exact products, fp32 accumulation over K terms of magnitude ~0.05: far below 1e-3
    assert err < 2e-3 * max(1.0, np.sqrt(K / 1024.0)), err
    assert np.isfinite(got).all()


# ---------------------------------------------------------------------------- attention


@pytest.mark.parametrize("name,desc,ctx_lens,spec_lens", [
    ("gqa-cfg2-like", synth.LLAMA2_70B.with_layers(1), [1024, 1000, 37, 0], [8, 8, 8, 8]),
    ("gqa-ragged", synth.LLAMA2_70B.with_layers(1), [256, 2047, 513, 15, 16, 1, 300], [1, 16, 7, 0, 3, 16, 12]),
    ("mha-opt13b", synth.OPT_13B.with_layers(1), [512, 100, 31], [4, 4, 0]),
    ("fp32-generic", synth.OPT_TINY.with_layers(1), [64, 0, 300], [4, 63, 2]),
    # head_dim 64, few rows per KV head: the drafting models' decode shape and its neighbours
    ("fewrow-mha-decode", synth.LLAMA_160M.with_layers(1), [1024, 1000, 37, 0, 63, 64, 65, 2047], [0] * 8),
    ("fewrow-mha-k3", synth.LLAMA_160M.with_layers(1), [300, 17, 0, 640], [3, 1, 2, 0]),
    ("fewrow-gqa2", synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 1, 512, 8, 4, 64, 1024, 64, 4096), [129, 5, 0, 1500], [1, 0, 1, 1]),
    ("fewrow-gqa4", synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 1, 512, 8, 2, 64, 1024, 64, 4096), [200, 16, 1], [0, 0, 0]),
    ("hd64-many-rows-generic", synth.LLAMA_160M.with_layers(1), [100, 40], [7, 4]),
    # many sequences with long contexts: the device leaves every sequence in one KV split (the batch alone fills the
    # chip), so one workgroup walks all 151 key tiles of its sequence, many more than the most-splits bound the
    # host could assume
    ("one-split-long-context", synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 1, 1024, 8, 8, 128, 1024, 64, 8192),
     [4800] * 36 + [4700, 3000, 5000, 4800], [1] * 40),
])
def test_attention_matches_oracle(hb, name, desc, ctx_lens, spec_lens):
    _check_attention(hb, desc, ctx_lens, spec_lens)


@pytest.mark.parametrize("seed", list(range(10)))
def test_attention_drawn_batches(hb, seed):
    """Drawn batches for the MFMA kernel and its work list: 1-24 sequences, contexts 0-2500 (a few of them long, so
    that sequences of one batch get different numbers of KV splits), 0-16 speculated tokens (one or two row groups
    with grouped-query heads), grouped-query and plain multi-head shapes."""
    g = synth.stream(9191, seed)
    desc = (synth.LLAMA2_70B if seed % 3 else synth.OPT_13B).with_layers(1)
    B = int(g.integers(1, 25))
    ctx = g.integers(0, 400, size=B)
    longs = g.random(B) < 0.3
    ctx[longs] = g.integers(400, 2501, size=int(longs.sum()))
    ks = g.integers(0, 17, size=B)
    _check_attention(hb, desc, ctx.tolist(), ks.tolist())


def _check_attention(hb, desc, ctx_lens, spec_lens):
    harness, binding = hb
    B = len(ctx_lens)
    total = [int(c) + int(k) + 1 for c, k in zip(ctx_lens, spec_lens)]
    kvh = synth.make_paged_kv(desc, total, [-1] * B, 91, scatter=True)          # blocks for exactly `total` tokens
    kvh.ctx_lens = np.asarray(ctx_lens, np.int32)
    M = int(sum(k + 1 for k in spec_lens))
    g = synth.stream(91, 9)
    q = g.standard_normal((M, desc.n_heads, desc.head_dim), dtype=np.float32)
    if desc.dtype == synth.DT_BF16:
        q = q.astype(np.float16).astype(np.float32)                                   # fp16 activations
    tiny = synth.ModelDesc(desc.arch, desc.dtype, 1, 128, desc.n_heads, desc.n_kv_heads, desc.head_dim, 128, 8, 8192)
    model = harness.DeviceModel.from_host(tiny, synth.make_weights(tiny, 1))
    kvd = harness.DeviceKV.from_host(desc, kvh)
    kvd.ctx_lens.copy_(torch.from_numpy(kvh.ctx_lens))
    q_d = harness.to_device_act(q, desc.dtype)
    st_t = torch.float16 if desc.dtype == synth.DT_BF16 else torch.float32
    out = torch.full((M, desc.n_heads * desc.head_dim), float("nan"), dtype=st_t, device="cuda:0")
    max_ctx = max(total)
    wsb = binding.mn_workspace_bytes(model.ctx, B, M, max_ctx)
    ws = torch.empty((wsb,), dtype=torch.uint8, device="cuda:0")
    st = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    spec_d = _dev(spec_lens)
    binding.mn_attention(model.ctx, q_d.data_ptr(), spec_d.data_ptr(), binding.host_i32(spec_lens), B, max_ctx,
                         kvd.c, 0, out.data_ptr(), ws.data_ptr(), wsb, st.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    assert st.item() == 0
    got = out.float().cpu().numpy().reshape(M, desc.n_heads, desc.head_dim)
    row = 0
    worst = 0.0
    for b in range(B):
        T = spec_lens[b] + 1
        K, V = synth.gather_sequence_kv(kvh, 0, b, total[b])
        want = orc.attention_cached(desc, q[row:row + T].astype(np.float64), K.astype(np.float64), V.astype(np.float64),
                                    int(ctx_lens[b]))
        worst = max(worst, np.abs(got[row:row + T] - want).max())
        row += T
    # outputs are softmax averages of N(0,1) values (|o| up to ~1): fp16 rounding of the probabilities and
    # of the output is 2^-11 relative each; fp32 path: accumulation order only
    tol = 2e-3 if desc.dtype == synth.DT_BF16 else 1e-5
    assert worst < tol, worst


# ---------------------------------------------------------------------------- ACR + SSM weight update
@pytest.mark.parametrize("B,n,seed", [(1, 1, 0), (16, 4, 1), (64, 5, 2), (257, 7, 3), (4096, 64, 4), (0, 3, 5)])
def test_acr_update_bit_exact(hb, B, n, seed):
    harness, binding = hb
    g = synth.stream(31, B, n, seed)
    ssm = g.integers(-1, n, size=B).astype(np.int32)
    k = g.integers(0, 17, size=B).astype(np.int32)
    a = np.array([g.integers(0, kk + 1) for kk in k], np.int32).reshape(B)
    n_out = np.where(g.random(B) < 0.9, a + 1, 0).astype(np.int32)
    w0 = (g.random(n) + 0.5).astype(np.float32)
    want_w, want_acr = orc.acr_update(w0, ssm, a, k, 0.625, 0.375, 1.25, 0.75, verified=(n_out > 0))
    ssm_d, a_d, k_d, no_d = _dev(ssm if B else [0]), _dev(a if B else [0]), _dev(k if B else [0]), _dev(n_out if B else [0])
    w_d = _dev(w0, torch.float32)
    acr_d = torch.zeros(n, dtype=torch.float64, device="cuda:0")
    binding.mn_acr_update(None, ssm_d.data_ptr(), a_d.data_ptr(), k_d.data_ptr(), no_d.data_ptr(), B, n, 0.625, 0.375,
                          1.25, 0.75, w_d.data_ptr(), acr_d.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    got_acr, got_w = acr_d.cpu().numpy(), w_d.cpu().numpy()
    assert np.array_equal(np.isnan(got_acr), np.isnan(want_acr))
    assert np.array_equal(got_acr[~np.isnan(want_acr)], want_acr[~np.isnan(want_acr)])   # same sums in the same order
    assert np.array_equal(got_w, want_w)
    # without n_out every output with a speculation counts
    want_w2, want_acr2 = orc.acr_update(want_w, ssm, a, k, 0.625, 0.375, 1.25, 0.75)
    binding.mn_acr_update(None, ssm_d.data_ptr(), a_d.data_ptr(), k_d.data_ptr(), None, B, n, 0.625, 0.375, 1.25, 0.75,
                          w_d.data_ptr(), acr_d.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    assert np.array_equal(w_d.cpu().numpy(), want_w2)
    m = ~np.isnan(want_acr2)
    assert np.array_equal(acr_d.cpu().numpy()[m], want_acr2[m])
