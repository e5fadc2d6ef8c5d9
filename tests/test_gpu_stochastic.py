"""GPU parity of the stochastic verification rule (section 2.1) through the C ABI: mn_verify_sample followed by
mn_accept_and_commit against the oracle's accept_stochastic + commit on the same seeded inputs.

The decisions are integers taken from fp64 comparisons on both sides; the two evaluations of exp and the two
summation orders agree to ~1e-14 relative, so a sequence is compared bit for bit unless the oracle reports that
one of its decisions sat within 1e-9 of its threshold (none is expected: the uniform numbers have 53 bits)."""
import numpy as np
import pytest
import torch

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth

pytestmark = pytest.mark.gpu

MARGIN = 1e-9


@pytest.fixture(scope="module")
def hb():
    from paper_2402_15678_amd import binding, harness
    return harness, binding


def _dev(a, dt=torch.int32):
    return torch.tensor(np.asarray(a), dtype=dt, device="cuda:0")


def _softmax64(z):
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def _case(seed, B, k_max, V, T, noise, spread=2.0, one_hot=False):
    """Seeded inputs: scores N(0, spread) per row; q = softmax((scores + noise * N(0,1)) / T) stored as fp32 (or
    one-hot on the speculated token); speculated tokens drawn from q; ragged k_b with both ends present."""
    g = synth.stream(4100, seed, B, k_max, V)
    spec = g.integers(0, k_max + 1, size=B).astype(np.int32)
    spec[0] = k_max
    if B > 1:
        spec[1] = 0
    M = int((spec + 1).sum())
    logits = g.normal(0.0, spread, (M, V)).astype(np.float32)
    q = np.zeros((B, max(1, k_max), V), np.float32)
    voted = np.full((B, max(1, k_max)), -1, np.int32)
    row = 0
    for b in range(B):
        for j in range(int(spec[b])):
            if one_hot:
                tok = int(np.argmax(logits[row + j])) if g.random() < 0.6 else int(g.integers(V))
                q[b, j, tok] = 1.0
            else:
                p = _softmax64((logits[row + j].astype(np.float64) + noise * g.normal(0.0, 1.0, V)) / T)
                q[b, j] = p.astype(np.float32)
                tok = int(g.choice(V, p=p))
            voted[b, j] = tok
        row += int(spec[b]) + 1
    return spec, M, logits, q, voted


def _run_gpu(hb, spec, M, logits, q, voted, k_max, V, T, seed, step, ctx0, greedy0=None, block_size=16, max_blocks=64):
    harness, binding = hb
    B = len(spec)
    spec_d, log_d, q_d, voted_d = _dev(spec), _dev(logits, torch.float32), _dev(q, torch.float32), _dev(voted)
    greedy = np.zeros((B, k_max + 1), np.int32) if greedy0 is None else greedy0
    greedy_d = _dev(greedy)
    sampled = torch.full((B, k_max + 1), -9, dtype=torch.int32, device="cuda:0")
    st = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    binding.mn_verify_sample(None, log_d.data_ptr(), voted_d.data_ptr(), q_d.data_ptr(), spec_d.data_ptr(),
                             greedy_d.data_ptr(), B, k_max, M, V, T, seed, step, sampled.data_ptr(), st.data_ptr(),
                             harness.stream_ptr())
    ctx_d = _dev(ctx0)
    kv = binding.KV(None, None, block_size, 64, max_blocks, None, ctx_d.data_ptr())
    outs = {n: torch.full((B,), -9, dtype=torch.int32, device="cuda:0") for n in ("acc", "n_out", "nxt", "blocks")}
    out_tokens = torch.full((B, k_max + 1), -9, dtype=torch.int32, device="cuda:0")
    binding.mn_accept_and_commit(None, voted_d.data_ptr(), sampled.data_ptr(), spec_d.data_ptr(), B, k_max, kv,
                                 outs["acc"].data_ptr(), out_tokens.data_ptr(), outs["n_out"].data_ptr(),
                                 outs["nxt"].data_ptr(), outs["blocks"].data_ptr(), st.data_ptr(), harness.stream_ptr())
    torch.cuda.synchronize()
    return (sampled.cpu().numpy(), outs["acc"].cpu().numpy(), out_tokens.cpu().numpy(), outs["n_out"].cpu().numpy(),
            outs["nxt"].cpu().numpy(), ctx_d.cpu().numpy(), outs["blocks"].cpu().numpy(), int(st.item()))


def _check_against_oracle(res, spec, logits, q, voted, k_max, T, seed, step, ctx0, block_size=16):
    sampled, acc, out, n_out, nxt, ctx1, blocks, status = res
    assert status == 0
    row, skipped = 0, 0
    for b in range(len(spec)):
        k = int(spec[b])
        a, toks, margin = orc.accept_stochastic(voted[b], logits[row:row + k + 1], q[b], k, T, seed, step, b)
        row += k + 1
        assert (sampled[b, k + 1:] == -1).all()
        if margin < MARGIN:
            skipped += 1
            continue
        assert acc[b] == a, (b, k, acc[b], a)
        assert out[b, :a + 1].tolist() == toks and (out[b, a + 1:] == -1).all()
        assert n_out[b] == a + 1 and nxt[b] == toks[-1]
        assert (ctx1[b], blocks[b]) == orc.commit(int(ctx0[b]), a, block_size)
        assert sampled[b, :a].tolist() == [int(t) for t in voted[b, :a]]
    assert skipped <= max(1, len(spec) // 100)


@pytest.mark.parametrize("B,k_max,V,T,noise", [
    (1, 4, 7, 1.0, 1.0),            # a vocabulary inside one lane group
    (16, 8, 1003, 0.7, 1.5),        # one ragged tile, odd vocabulary
    (24, 5, 4096, 1.0, 0.0),        # q == o up to fp32 rounding: nearly everything survives
    (16, 8, 32000, 1.0, 1.0),       # the benchmark shape's vocabulary and batch
    (6, 16, 50272, 1.3, 3.0),       # the other family's vocabulary (49 tiles + a tail), mostly rejections
    (64, 3, 2500, 0.5, 0.7),
])
def test_sample_then_accept_matches_oracle(hb, B, k_max, V, T, noise):
    spec, M, logits, q, voted = _case(1, B, k_max, V, T, noise)
    ctx0 = (np.arange(B) * 7 + 3).astype(np.int32)
    for step in (0, 5):
        res = _run_gpu(hb, spec, M, logits, q, voted, k_max, V, T, seed=2024, step=step, ctx0=ctx0)
        _check_against_oracle(res, spec, logits, q, voted, k_max, T, 2024, step, ctx0)


def test_masked_vocabulary_entries(hb):
    """Scores of minus infinity (a masked part of the vocabulary) carry no mass on either side: such a token is
    never drawn, and a speculated token that the LLM masks is always rejected."""
    B, k_max, V, T = 12, 4, 1500, 1.0
    spec, M, logits, q, voted = _case(5, B, k_max, V, T, 1.0)
    g = synth.stream(4105, 0)
    masked = g.random((M, V)) < 0.4
    masked[np.arange(M), np.argmax(logits, axis=1)] = False           # every row keeps a finite maximum
    logits[masked] = -np.inf
    ctx0 = np.full(B, 20, np.int32)
    res = _run_gpu(hb, spec, M, logits, q, voted, k_max, V, T, seed=11, step=3, ctx0=ctx0)
    _check_against_oracle(res, spec, logits, q, voted, k_max, T, 11, 3, ctx0)
    out, n_out = res[2], res[3]
    row = 0
    for b in range(B):
        a = int(res[1][b])
        assert not masked[row + a, out[b, a]]                          # the drawn token is not a masked one
        for j in range(a):
            assert not masked[row + j, voted[b, j]]                    # a survivor was not masked by the LLM
        row += int(spec[b]) + 1


def test_low_temperature_equals_greedy_acceptance(hb):
    """One-hot drafts and T -> 0: the output is the longest-prefix acceptance on the argmax tokens."""
    B, k_max, V, T = 32, 6, 777, 1e-3
    spec, M, logits, q, voted = _case(3, B, k_max, V, 1.0, 0.0, spread=3.0, one_hot=True)
    top = np.argmax(logits, axis=1)
    logits[np.arange(M), top] += 0.1
    ctx0 = np.full(B, 40, np.int32)
    sampled, acc, out, n_out, nxt, ctx1, blocks, status = _run_gpu(hb, spec, M, logits, q, voted, k_max, V, T, 1, 0, ctx0)
    row = 0
    for b in range(B):
        k = int(spec[b])
        g = orc.greedy_tokens(logits[row:row + k + 1].astype(np.float64))
        row += k + 1
        a, toks = orc.accept(voted[b], g, k)
        assert acc[b] == a and out[b, :a + 1].tolist() == toks and ctx1[b] == 40 + a + 1


def test_disabled_sequences_and_row_mismatch(hb):
    B, k_max, V, T = 5, 3, 300, 1.0
    spec, M, logits, q, voted = _case(9, B, k_max, V, T, 1.0)
    greedy = np.zeros((B, k_max + 1), np.int32)
    greedy[2, 0] = -1                                  # made a no-op by the forward
    ctx0 = np.full(B, 10, np.int32)
    sampled, acc, out, n_out, nxt, ctx1, blocks, status = _run_gpu(hb, spec, M, logits, q, voted, k_max, V, T, 1, 0, ctx0,
                                                                   greedy0=greedy)
    assert status == 0 and (sampled[2] == -1).all() and n_out[2] == 0 and ctx1[2] == 10 and nxt[2] == -1
    assert (n_out[[0, 1, 3, 4]] >= 1).all()
    # fewer rows than the speculation lengths add up to: the surplus positions are refused, nothing is read past M
    res = _run_gpu(hb, spec, M - 1, logits, q, voted, k_max, V, T, 1, 0, ctx0)
    assert res[-1] & 2 and res[0][B - 1, int(spec[B - 1])] == -1


def test_emitted_token_distribution(hb):
    """Losslessness on the GPU path: over many sequences and steps the first emitted token follows the LLM's
    distribution whatever the SSM's (a property that needs no oracle)."""
    harness, binding = hb
    B, V, T, steps = 2048, 11, 0.9, 12
    g = synth.stream(4101, 0)
    row_logits = g.normal(0.0, 1.5, V).astype(np.float32)
    qv = _softmax64(g.normal(0.0, 1.5, V)).astype(np.float32)
    o = orc.llm_probs(row_logits, T)
    spec = np.ones(B, np.int32)
    logits = np.tile(np.stack([row_logits, row_logits]), (B, 1))
    q = np.tile(qv, (B, 1, 1))
    counts = np.zeros(V)
    for step in range(steps):
        voted = g.choice(V, size=(B, 1), p=qv.astype(np.float64) / qv.astype(np.float64).sum()).astype(np.int32)
        res = _run_gpu(hb, spec, 2 * B, logits, q, voted, 1, V, T, seed=7, step=step, ctx0=np.zeros(B, np.int32))
        counts += np.bincount(res[2][:, 0], minlength=V)
    N = B * steps
    assert np.abs(counts / N - o).max() < 4.0 * np.sqrt(0.25 / N)


def test_tiny_model_forward_sample_accept_end_to_end(hb):
    """The whole stochastic step on the small fp32 model: prompts prefilled through the library, speculated
    tokens drawn from distributions near the LLM's, forward -> mn_verify_sample -> accept + commit against the
    oracle's own forward and rule.  The two forwards agree to 1e-4 on the scores; at the low temperature used
    here (the model's scores are nearly flat, so T = 0.03 is what makes its distribution peaked enough for a
    draw to have a clear answer) that is up to 2 * 1e-4 / T = 7e-3 relative on a probability, so a sequence is
    compared only when every decision the oracle took cleared its threshold by 1e-2 (the others are counted and
    must be few)."""
    harness, binding = hb
    wl = synth.WORKLOADS[0]
    desc = wl.desc
    W = synth.make_weights(desc, wl.seed)
    model = harness.DeviceModel.from_host(desc, W)
    g = synth.stream(4102, 0)
    B, k, T, noise = 16, 4, 0.03, 0.02
    lens = [int(x) for x in g.integers(5, 24, size=B)]
    prompts = [g.integers(0, desc.vocab, size=n).astype(np.int32) for n in lens]
    kvh = synth.make_paged_kv(desc, [0] * B, [max(lens) + k + 1] * B, wl.seed, scatter=True, fill=True)
    kvd = harness.DeviceKV.from_host(desc, kvh)
    # ---- prefill: ctx = 0, the prompt's tokens as one causal block ----
    pmax = max(lens) - 1
    pre = harness.VerifySession(model, kvd, B, pmax, 1, max(lens))
    pv = np.full((B, pmax), -1, np.int32)
    for b, p in enumerate(prompts):
        pv[b, :len(p) - 1] = p[1:]
    t_last, t_k, t_v = _dev([p[0] for p in prompts]), _dev([n - 1 for n in lens]), _dev(pv)
    pre.forward(t_last, t_k, [n - 1 for n in lens], voted=t_v)
    torch.cuda.synchronize()
    assert pre.dev_status.item() == 0
    kvd.ctx_lens.copy_(_dev(lens))
    caches = [orc.SeqCache(desc.n_layers, desc.n_kv_heads, desc.head_dim) for _ in range(B)]
    pre_logits = orc.decoder_step(desc, W, [p.tolist() for p in prompts], caches)
    last = [int(np.argmax(l[-1])) for l in pre_logits]
    # ---- speculation: token j drawn from q_j = softmax((LLM scores of the prefix + noise) / T) ----
    voted = np.zeros((B, k), np.int32)
    q = np.zeros((B, k, desc.vocab), np.float32)
    for b in range(B):
        toks = prompts[b].tolist() + [last[b]]
        for j in range(k):
            z = orc.decoder_full(desc, W, toks)[-1] + noise * g.normal(0.0, 1.0, desc.vocab)
            p = _softmax64(z / T)
            q[b, j] = p.astype(np.float32)
            voted[b, j] = int(g.choice(desc.vocab, p=p))
            toks.append(int(voted[b, j]))
    # ---- the step on the device ----
    ses = harness.VerifySession(model, kvd, B, k, 1, max(lens) + k + 1, want_logits=True)
    t_last, t_k, t_v, t_q = _dev(last), _dev([k] * B), _dev(voted), _dev(q, torch.float32)
    ses.forward(t_last, t_k, [k] * B, voted=t_v)
    sampled = ses.sample(t_k, B * (k + 1), t_q, T, seed=31, step=2, voted=t_v)
    ses.accept(t_k, voted=t_v, tokens=sampled)
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    # ---- the step on the oracle ----
    want_logits = orc.decoder_step(desc, W, [[last[b]] + voted[b].tolist() for b in range(B)], caches)
    got_logits = ses.logits.cpu().numpy().reshape(B, k + 1, desc.vocab)
    acc, out, ctx1 = ses.accepted_len.cpu().numpy(), ses.out_tokens.cpu().numpy(), kvd.ctx_lens.cpu().numpy()
    compared = 0
    for b in range(B):
        assert np.abs(got_logits[b] - want_logits[b]).max() < 1e-4
        a, toks, margin = orc.accept_stochastic(voted[b], want_logits[b], q[b], k, T, 31, 2, b)
        if margin < 1e-2:
            continue
        compared += 1
        assert acc[b] == a and out[b, :a + 1].tolist() == toks and ctx1[b] == lens[b] + a + 1
    assert compared >= B - 4


@pytest.mark.parametrize("B,V,T,spread", [(1, 7, 1.0, 1.0), (16, 1003, 0.7, 2.0), (16, 32000, 1.0, 2.0), (5, 50272, 0.3, 1.0),
                                          (300, 4096, 1.5, 3.0)])
def test_draft_sample_matches_oracle(hb, B, V, T, spread):
    """mn_draft_sample on seeded scores: q within an fp32 ulp of the oracle's, and the token equal wherever the
    oracle's draw cleared its boundaries by more than an fp32 rounding of q could move them."""
    harness, binding = hb
    g = synth.stream(4103, B, V)
    logits = g.normal(0.0, spread, (B, V)).astype(np.float32)
    n, k_max, ssm, t = 3, 5, 2, 4
    drafts = torch.full((B, n, k_max), -5, dtype=torch.int32, device="cuda:0")
    probs = torch.full((B, k_max, V), -1.0, dtype=torch.float32, device="cuda:0")
    log_d = _dev(logits, torch.float32)
    binding.mn_draft_sample(None, log_d.data_ptr(), B, V, T, 77, 12, ssm, t, drafts[0, ssm, t:].data_ptr(), n * k_max,
                            probs[0, t].data_ptr(), k_max * V, harness.stream_ptr())
    torch.cuda.synchronize()
    got_tok, got_q = drafts.cpu().numpy(), probs.cpu().numpy()
    assert (np.delete(got_tok.reshape(B, -1), ssm * k_max + t, axis=1) == -5).all()      # only its own slot is written
    assert (got_q[:, :t] == -1.0).all()
    skipped = 0
    for b in range(B):
        tok, q32, gap = orc.draft_sample(logits[b], T, 77, 12, ssm, b, t)
        assert np.allclose(got_q[b, t], q32, rtol=3e-7, atol=1e-45)
        assert abs(float(got_q[b, t].astype(np.float64).sum()) - 1.0) < 1e-5
        if gap < 1e-6:
            skipped += 1
            continue
        assert got_tok[b, ssm, t] == tok, (b, got_tok[b, ssm, t], tok)
    assert skipped <= max(1, B // 50)


def test_sampled_drafting_loop_on_the_device(hb):
    """SSMs that sample, the vote, the LLM's stochastic verification and the commit, end to end on the device.
    Checked as properties (the parity of every stage has its own test): the drafts come with the distributions
    they were drawn from, the SSM caches advance, the same (seed, step) reproduces the drafts and another step
    does not, and the outcome is a prefix of the voted draft plus one token."""
    harness, binding = hb
    V, B, k, n = 512, 6, 4, 3
    llm_desc = synth.ModelDesc(synth.ARCH_OPT, synth.DT_F32, 2, 128, 4, 4, 32, 256, V, 256)
    ssm_descs = [synth.ModelDesc(synth.ARCH_OPT, synth.DT_F32, 1, 64, 2, 2, 32, 128, V, 256),
                 synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_F32, 1, 64, 4, 2, 16, 128, V, 256),
                 synth.ModelDesc(synth.ARCH_OPT, synth.DT_F32, 2, 64, 2, 2, 32, 64, V, 256)]
    ctx = np.array([40, 17, 64, 1, 33, 90], np.int32)
    ks = np.full(B, k, np.int32)
    last = synth.stream(4104, 0).integers(0, V, size=B).astype(np.int32)
    max_ctx = int((ctx + k + 1).max())

    def build(desc, seed):
        kvh = synth.make_paged_kv(desc, ctx, ks, seed, scatter=True)
        return harness.DeviceModel.from_host(desc, synth.make_weights(desc, seed)), harness.DeviceKV.from_host(desc, kvh)

    llm_m, llm_kv = build(llm_desc, 910)
    ssm = [build(d, 911 + i) for i, d in enumerate(ssm_descs)]
    ds = harness.DraftSession([s[0] for s in ssm], [s[1] for s in ssm], B, k, max_ctx, sampling=True)
    t_last, t_k = _dev(last), _dev(ks)
    T = 0.05                                     # the small models' scores are nearly flat
    d1 = ds.draft_sampled(t_last, k, T, seed=5, step=1).clone()
    q1 = ds.draft_probs.clone()
    torch.cuda.synchronize()
    for s in ssm:
        assert s[1].ctx_lens.cpu().tolist() == (ctx + k).tolist()
        s[1].ctx_lens.copy_(_dev(ctx))
    d1h, q1h = d1.cpu().numpy(), q1.cpu().numpy()
    assert ((d1h >= 0) & (d1h < V)).all()
    assert np.allclose(q1h.sum(axis=-1), 1.0, atol=1e-5)
    for j in range(n):
        for b in range(B):
            assert (q1h[j, b, np.arange(k), d1h[b, j]] > 0).all()          # a drawn token has mass
    d2 = ds.draft_sampled(t_last, k, T, seed=5, step=1).clone()
    for s in ssm:
        s[1].ctx_lens.copy_(_dev(ctx))
    d3 = ds.draft_sampled(t_last, k, T, seed=5, step=2).clone()
    torch.cuda.synchronize()
    assert torch.equal(d1, d2) and not torch.equal(d1, d3)
    # ---- vote, verify, sample, accept on the LLM with the winners' distributions ----
    ses = harness.VerifySession(llm_m, llm_kv, B, k, n, max_ctx, want_logits=True)
    w = torch.ones(n, device="cuda:0")
    ses.vote(d1, t_k, w)
    ses.forward(t_last, t_k, ks.tolist())
    ds.draft_probs.copy_(q1)
    qv = ds.voted_probs(ses.voted_ssm)
    sampled = ses.sample(t_k, B * (k + 1), qv, T, seed=5, step=1)
    ses.accept(t_k, tokens=sampled)
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    voted, ssm_idx = ses.voted.cpu().numpy(), ses.voted_ssm.cpu().numpy()
    acc, out, n_out = ses.accepted_len.cpu().numpy(), ses.out_tokens.cpu().numpy(), ses.n_out.cpu().numpy()
    for b in range(B):
        assert np.array_equal(voted[b], d1h[b, ssm_idx[b]])               # the vote returns one SSM's whole draft
        a = int(acc[b])
        assert 0 <= a <= k and n_out[b] == a + 1 and out[b, :a].tolist() == voted[b, :a].tolist()
        assert 0 <= out[b, a] < V and (a == k or out[b, a] != voted[b, a])
    assert llm_kv.ctx_lens.cpu().tolist() == (ctx + acc + 1).tolist()


def test_draft_probs_that_cover_the_llm_distribution(hb):
    """A draft_probs row that sums above 1 can lie above o everywhere: max(0, o - q) is then empty, the
    replacement comes from o without the rejected token (never that token itself), and where o has no other mass
    the token stays.  Decision by decision against the oracle."""
    B, k_max, V, T = 12, 6, 301, 1.0
    spec, M, logits, q, voted = _case(7, B, k_max, V, T, 1.0)
    row = 0
    for b in range(B):
        for j in range(int(spec[b])):
            o = orc.llm_probs(logits[row + j], T)
            q[b, j] = (1.5 * o + 1e-6).astype(np.float32)             # above o everywhere
        row += int(spec[b]) + 1
    # one position where all of o sits on the speculated token (the other scores are masked)
    logits[0, :] = -np.inf
    logits[0, int(voted[0, 0])] = 0.0
    q[0, 0, :] = 0.0
    q[0, 0, int(voted[0, 0])] = 4.0
    ctx0 = (np.arange(B) * 5 + 1).astype(np.int32)
    rejections = 0
    for step in range(6):
        res = _run_gpu(hb, spec, M, logits, q, voted, k_max, V, T, seed=99, step=step, ctx0=ctx0)
        _check_against_oracle(res, spec, logits, q, voted, k_max, T, 99, step, ctx0)
        sampled, acc = res[0], res[1]
        for b in range(B):
            a, k = int(acc[b]), int(spec[b])
            if a < k:
                rejections += 1
                assert sampled[b, a] != voted[b, a] and sampled[b, a] >= 0
        assert sampled[0, 0] == voted[0, 0]                             # nothing else could be emitted there
    assert rejections >= 10                                             # survival probability is 2/3 per position
