"""Pins for greedy verification, acceptance and commit on the oracle (no GPU)."""
import numpy as np
import pytest

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth

DESC = synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_F32, 2, 64, 4, 2, 16, 96, 211, 256)


def _greedy_decode(desc, W, prompt, n_new):
    """Plain one-token-at-a-time greedy decoding with the cache-less forward."""
    toks = list(prompt)
    for _ in range(n_new):
        toks.append(int(np.argmax(orc.decoder_full(desc, W, toks)[-1])))
    return toks[len(prompt):]


def _prefilled(desc, W, prompt):
    c = orc.SeqCache(desc.n_layers, desc.n_kv_heads, desc.head_dim)
    logits = orc.decoder_step(desc, W, [prompt], [c])[0]
    return c, int(np.argmax(logits[-1]))


def test_accept_closed_cases():
    assert orc.accept([5, 6, 7], [5, 6, 7, 8], 3) == (3, [5, 6, 7, 8])        # all accepted: bonus token
    assert orc.accept([5, 6, 7], [5, 9, 7, 8], 3) == (1, [5, 9])              # first mismatch discards the rest
    assert orc.accept([5, 6, 7], [1, 6, 7, 8], 3) == (0, [1])
    assert orc.accept([5, 6, 7], [5, 6, 7, 8], 2) == (2, [5, 6, 7])           # k_b shorter than the row
    assert orc.accept([], [4], 0) == (0, [4])                                 # plain decode step
    assert orc.commit(10, 3, 16) == (14, 1) and orc.commit(15, 0, 16) == (16, 1) and orc.commit(16, 0, 16) == (17, 2)


def test_greedy_tokens_lowest_id_on_ties():
    z = np.zeros((2, 7)); z[0, 3] = z[0, 5] = 2.0; z[1, 6] = 1.0
    assert orc.greedy_tokens(z).tolist() == [3, 6]
    assert np.allclose(orc.top1_margin(z), [0.0, 1.0])


@pytest.mark.parametrize("k", [1, 4, 7])
def test_all_greedy_drafts_are_fully_accepted_and_corruption_cuts_at_i(k):
    W = synth.make_weights(DESC, seed=21, std=0.1)
    prompt = synth.stream(21, 1).integers(0, DESC.vocab, size=12).tolist()
    cont = _greedy_decode(DESC, W, prompt, k + 2)           # cont[0] is the pending token
    last, good = cont[0], cont[1:k + 1]
    for corrupt_at in [None] + list(range(k)):
        cache, last2 = _prefilled(DESC, W, prompt)
        assert last2 == last
        d = np.array([[good, good, good]], np.int32)
        if corrupt_at is not None:
            d[0, :, corrupt_at] = synth.corrupt_token(good[corrupt_at], DESC.vocab, synth.stream(21, 2, corrupt_at))
        r = orc.verify_step(DESC, W, [cache], [last], d, [k], [1.0, 1.0, 1.0])
        a = k if corrupt_at is None else corrupt_at
        assert r["accepted_len"][0] == a and r["n_out"][0] == a + 1
        assert r["out_tokens"][0, :a + 1].tolist() == cont[1:a + 2]      # accepted drafts + the true next token
        assert r["next_last_tok"][0] == cont[a + 1]
        assert cache.ctx == len(prompt) + a + 1 and r["ctx_lens"][0] == cache.ctx


def test_losslessness_multi_round_equals_plain_greedy():
    # rounds of vote -> verify -> accept with arbitrary drafts emit exactly the greedy stream
    W = synth.make_weights(DESC, seed=33, std=0.1)
    g = synth.stream(33, 1)
    prompts = [g.integers(0, DESC.vocab, size=n).tolist() for n in (9, 17)]
    want = [_greedy_decode(DESC, W, p, 40) for p in prompts]
    caches, last, emitted = [], [], []
    for p in prompts:
        c, t = _prefilled(DESC, W, p)
        caches.append(c); last.append(t); emitted.append([t])
    ssm_w = np.array([1.0, 0.7, 1.3], np.float32)
    while min(len(e) for e in emitted) < 36:
        ks = [int(g.integers(1, 6)) for _ in prompts]
        kmax = max(ks)
        per = []
        for b in range(2):
            truth = want[b][len(emitted[b]):len(emitted[b]) + ks[b]]
            truth = truth + [0] * (ks[b] - len(truth))
            per.append(synth.drafts_corrupted(truth, 3, 0.3, DESC.vocab, g))
        d = synth.pack_drafts(per, kmax)
        r = orc.verify_step(DESC, W, caches, last, d, ks, ssm_w)
        for b in range(2):
            emitted[b] += r["out_tokens"][b, :r["n_out"][b]].tolist()
            last[b] = int(r["next_last_tok"][b])
            assert caches[b].ctx == len(prompts[b]) + len(emitted[b]) - 1
    for b in range(2):
        n = min(len(emitted[b]), 40)
        assert emitted[b][:n] == want[b][:n]


def test_committed_cache_equals_sequential_decode_cache():
    W = synth.make_weights(DESC, seed=44, std=0.1)
    prompt = synth.stream(44, 1).integers(0, DESC.vocab, size=10).tolist()
    cont = _greedy_decode(DESC, W, prompt, 6)
    cache, last = _prefilled(DESC, W, prompt)
    d = np.array([[cont[1:3] + [cont[3] ^ 1] + cont[4:6]]], np.int32)          # corrupted at position 2
    r = orc.verify_step(DESC, W, [cache], [last], d, [5], [1.0])
    assert r["accepted_len"][0] == 2
    ref = orc.SeqCache(DESC.n_layers, DESC.n_kv_heads, DESC.head_dim)
    orc.decoder_step(DESC, W, [prompt + cont[:3]], [ref])
    for l in range(DESC.n_layers):
        assert cache.K[l].shape == ref.K[l].shape
        assert np.abs(cache.K[l] - ref.K[l]).max() < 1e-12 and np.abs(cache.V[l] - ref.V[l]).max() < 1e-12


def test_config0_recipe_on_the_oracle():
    # tiny OPT-style fp32 model, batch 1, 64-token prompt, three drafts of k=4 (greedy / corrupted / random)
    wl = synth.WORKLOADS[0]
    desc = wl.desc
    W = synth.make_weights(desc, wl.seed)
    prompt = synth.stream(wl.seed, 400).integers(0, desc.vocab, size=64).tolist()
    cache, last = _prefilled(desc, W, prompt)
    greedy = []
    c2, t = _prefilled(desc, W, prompt)
    for _ in range(4):
        t = int(np.argmax(orc.decoder_step(desc, W, [[t]], [c2])[0][-1]))
        greedy.append(t)
    drafts, info = synth.drafts_config0(greedy, desc.vocab, synth.stream(wl.seed, 401))
    r = orc.verify_step(desc, W, [cache], [last], drafts[None], [4], [1.0, 1.0, 1.0])
    # Unit weights.  Before the corrupted position the greedy and the corrupted draft agree (weight 2)
    # and outvote the random one; at the corrupted position they split 1:1 and the lower draft index
    # wins.  A corruption at position 0 makes level 0 a three-way tie: draft 0 wins whatever it is.
    pos = info["corrupt_pos"]
    winner = 0 if pos == 0 else min(info["greedy_at"], info["corrupt_at"])
    assert r["voted_ssm"][0] == winner
    assert r["voted"][0].tolist() == drafts[winner].tolist()
    if winner == info["greedy_at"]:
        expect_a = 4
    elif winner == info["corrupt_at"]:
        expect_a = pos
    else:
        expect_a = 0 if drafts[winner][0] != greedy[0] else None
    if expect_a is not None:
        assert r["accepted_len"][0] == expect_a
    a = int(r["accepted_len"][0])
    assert r["out_tokens"][0, :a].tolist() == greedy[:a]
    assert cache.ctx == 64 + a + 1


def test_acr_update_worked_sets():
    # section 3.2: o_SSM1 = {o_1, o_3, o_4}: ACR_1 is the mean over exactly those outputs
    voted_ssm = [0, 1, 0, 0, 2]
    acc = [4, 1, 2, 0, 3]
    k = [4, 4, 4, 4, 4]
    w, acr = orc.acr_update([1.0, 1.0, 1.0, 1.0], voted_ssm, acc, k, 0.7, 0.3, 1.5, 0.5)
    assert np.allclose(acr[:3], [(1.0 + 0.5 + 0.0) / 3, 0.25, 0.75]) and np.isnan(acr[3])
    assert w.tolist() == [1.0, 0.5, 1.5, 1.0]


def test_acr_update_thresholds_are_strict_and_unverified_outputs_do_not_count():
    # ACR exactly at a threshold neither rewards nor punishes ("exceeds" / "falls below")
    w, acr = orc.acr_update([2.0, 2.0], [0, 1], [3, 1], [4, 4], 0.75, 0.25, 1.5, 0.5)
    assert acr.tolist() == [0.75, 0.25] and w.tolist() == [2.0, 2.0]
    # an output that was not verified, or that speculated nothing, is not in the set
    w, acr = orc.acr_update([1.0, 1.0], [0, 0, 0, 1], [4, 0, 2, 0], [4, 4, 0, 4], 0.9, 0.1, 2.0, 0.25,
                            verified=[True, False, True, True])
    assert acr.tolist() == [1.0, 0.0] and w.tolist() == [2.0, 0.25]
    # brute force over the definition on random data: mean of the per-output rates of each SSM's set
    g = synth.stream(3, 1)
    B, n = 200, 5
    ssm = g.integers(-1, n, size=B)
    k = g.integers(0, 9, size=B)
    a = np.array([g.integers(0, kk + 1) for kk in k])
    ok = g.random(B) < 0.9
    w0 = (g.random(n) + 0.5).astype(np.float32)
    w, acr = orc.acr_update(w0, ssm, a, k, 0.6, 0.4, 1.25, 0.8, verified=ok)
    for i in range(n):
        sel = [b for b in range(B) if ssm[b] == i and k[b] > 0 and ok[b]]
        want = np.mean([a[b] / k[b] for b in sel]) if sel else np.nan
        assert (np.isnan(want) and np.isnan(acr[i])) or abs(acr[i] - want) < 1e-12
        f = np.float32(1.25) if want > 0.6 else np.float32(0.8) if want < 0.4 else np.float32(1.0)
        assert w[i] == np.float32(w0[i] * f)
