"""End-to-end GPU parity of the verification step (vote -> verify forward -> accept + commit) against
the CPU oracle, through the C ABI: the tiny fp32 configuration in full, and full-width, layer-reduced
versions of the bf16 configurations (the oracle cannot run 40/80 layers in test time)."""
import numpy as np
import pytest
import torch

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hb():
    from paper_2402_15678_amd import binding, harness
    return harness, binding


def _i32(a):
    return torch.tensor(np.asarray(a, np.int32), dtype=torch.int32, device="cuda:0")


def _compare_cache(desc, kvd, kvh_tables, block_size, caches, tol):
    """Committed cache rows [0, ctx_b) on the device against the oracle's cache."""
    worst = 0.0
    for l in range(desc.n_layers):
        kp, vp = kvd.download(l)
        img = synth.PagedKV(block_size, kp.shape[0], kvh_tables.shape[1], kvh_tables, None, {l: kp}, {l: vp})
        for b, c in enumerate(caches):
            K, V = synth.gather_sequence_kv(img, l, b, c.ctx)
            worst = max(worst, np.abs(K - c.K[l]).max(), np.abs(V - c.V[l]).max())
    assert worst < tol, worst
    return worst


def test_config0_tiny_opt_fp32_end_to_end(hb):
    harness, binding = hb
    wl = synth.WORKLOADS[0]
    desc = wl.desc
    W = synth.make_weights(desc, wl.seed)
    model = harness.DeviceModel.from_host(desc, W)
    prompt = synth.stream(wl.seed, 400).integers(0, desc.vocab, size=64).astype(np.int32)
    # empty cache with room for the prompt and the scored positions
    kvh = synth.make_paged_kv(desc, [0], [64 + 4 + 1], wl.seed, scatter=True, fill=True)
    kvd = harness.DeviceKV.from_host(desc, kvh)
    # ---- prefill through the library: ctx = 0, 64 rows, causal among them ----
    pre = harness.VerifySession(model, kvd, 1, 63, 1, 64, want_logits=True)
    t_last, t_k, t_voted = _i32(prompt[:1]), _i32([63]), _i32(prompt[None, 1:])   # named: must outlive the call
    pre.forward(t_last, t_k, [63], voted=t_voted)
    torch.cuda.synchronize()
    assert pre.dev_status.item() == 0
    cache = orc.SeqCache(desc.n_layers, desc.n_kv_heads, desc.head_dim)
    want_pre = orc.decoder_step(desc, W, [prompt.tolist()], [cache])[0]
    got_pre = pre.logits.cpu().numpy()
    assert np.abs(got_pre - want_pre).max() < 1e-4
    assert np.array_equal(pre.greedy.cpu().numpy()[0], orc.greedy_tokens(want_pre))
    kvd.ctx_lens.fill_(64)                                    # the caller commits the prompt
    last = int(orc.greedy_tokens(want_pre)[-1])
    # ---- drafts: greedy continuation / corrupted / random ----
    (greedy,), (margin,) = util.greedy_continuations(desc, W, [cache], [last], [4])
    assert margin > 2e-4
    drafts, info = synth.drafts_config0(greedy[:4], desc.vocab, synth.stream(wl.seed, 401))
    ssm_w = np.ones(3, np.float32)
    want = orc.verify_step(desc, W, [cache], [last], drafts[None], [4], ssm_w)
    ses = harness.VerifySession(model, kvd, 1, 4, 3, 64 + 5, want_logits=True)
    t_last, t_drafts, t_k, t_w = _i32([last]), _i32(drafts[None]), _i32([4]), torch.ones(3, device="cuda:0")
    ses.step(t_last, t_drafts, t_k, [4], t_w)
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    assert np.array_equal(ses.voted.cpu().numpy(), want["voted"])
    assert ses.voted_ssm.cpu().tolist() == want["voted_ssm"].tolist()
    assert np.abs(ses.logits.cpu().numpy() - want["logits"][0]).max() < 1e-4
    assert np.array_equal(ses.greedy.cpu().numpy(), want["greedy"])
    assert ses.accepted_len.cpu().tolist() == want["accepted_len"].tolist()
    assert np.array_equal(ses.out_tokens.cpu().numpy(), want["out_tokens"])
    assert ses.n_out.cpu().tolist() == want["n_out"].tolist()
    assert ses.next_last_tok.cpu().tolist() == want["next_last_tok"].tolist()
    assert kvd.ctx_lens.cpu().tolist() == want["ctx_lens"].tolist()
    assert ses.blocks_in_use.cpu().tolist() == want["blocks_in_use"].tolist()
    _compare_cache(desc, kvd, kvh.block_tables, 16, [cache], 1e-4)
    # closing the loop: the weights the next vote will use, updated on the device from this step's outcome
    _check_acr(ses, t_k, [4], 3)


def _check_acr(ses, t_k, ks, n):
    """mn_acr_update on the session's own outputs against the oracle on the same integers."""
    w0 = np.linspace(0.5, 1.5, n).astype(np.float32)
    t_w = torch.tensor(w0, device="cuda:0")
    t_acr = torch.zeros(n, dtype=torch.float64, device="cuda:0")
    ses.acr_update(t_k, t_w, 0.75, 0.5, 1.25, 0.5, acr=t_acr)
    torch.cuda.synchronize()
    want_w, want_acr = orc.acr_update(w0, ses.voted_ssm.cpu().numpy(), ses.accepted_len.cpu().numpy(), ks, 0.75, 0.5,
                                      1.25, 0.5, verified=ses.n_out.cpu().numpy() > 0)
    got_acr = t_acr.cpu().numpy()
    assert np.array_equal(np.isnan(got_acr), np.isnan(want_acr))
    assert np.array_equal(got_acr[~np.isnan(want_acr)], want_acr[~np.isnan(want_acr)])
    assert np.array_equal(t_w.cpu().numpy(), want_w)


def _reduced_case(hb, wl, n_layers, B, n_cand, ctx_override=None, k_override=None, min_decisive=None):
    harness, binding = hb
    desc = wl.desc.with_layers(n_layers)
    tol = util.TOL[desc.dtype]
    W = synth.make_weights(desc, wl.seed)
    W64 = util.weights_f64(W)
    model = harness.DeviceModel.from_host(desc, W)
    g = synth.stream(wl.seed, 500)
    wl_b = synth.Workload(wl.name, desc, B, wl.ctx_lo, wl.ctx_hi, wl.k_lo, wl.k_hi, wl.n_drafts, wl.p_corrupt, seed=wl.seed)
    ctx = np.asarray(ctx_override, np.int32) if ctx_override is not None else synth.draw_ctx_lens(wl_b)
    ks = np.asarray(k_override, np.int32) if k_override is not None else synth.draw_spec_lens(wl_b)
    k_max = int(ks.max())
    kvh = synth.make_paged_kv(desc, ctx, ks, wl.seed, scatter=True)
    kvd = harness.DeviceKV.from_host(desc, kvh)
    caches = util.oracle_caches(desc, kvh)
    last, greedy, margin = util.pick_decisive_last_tokens(desc, W64, caches, ks, desc.vocab, g, tol, n_cand)
    per = [synth.drafts_corrupted(greedy[b][:ks[b]], wl.n_drafts, wl.p_corrupt, desc.vocab, g) if ks[b] > 0
           else np.zeros((wl.n_drafts, 0), np.int32) for b in range(B)]
    drafts = synth.pack_drafts(per, k_max)
    ssm_w = np.ones(wl.n_drafts, np.float32)
    want = orc.verify_step(desc, W64, caches, last, drafts, ks, ssm_w)
    M = int((ks + 1).sum())
    ses = harness.VerifySession(model, kvd, B, k_max, wl.n_drafts, int((ctx + ks + 1).max()), max_rows=M, want_logits=True)
    t_last, t_drafts, t_k, t_w = _i32(last), _i32(drafts), _i32(ks), torch.ones(wl.n_drafts, device="cuda:0")
    ses.step(t_last, t_drafts, t_k, ks.tolist(), t_w)
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    # votes: bit-exact
    assert np.array_equal(ses.voted.cpu().numpy()[:, :k_max], want["voted"])
    assert ses.voted_ssm.cpu().tolist() == want["voted_ssm"].tolist()
    # logits within tolerance, element by element
    got_logits = ses.logits.cpu().numpy()
    want_logits = np.concatenate(want["logits"])
    err = np.abs(got_logits - want_logits).max()
    assert err < tol, err
    # tokens: bit-exact wherever the oracle's margin is decisive; near ties must stay inside the tie set
    got_g = ses.greedy.cpu().numpy()
    row = 0
    decisive_seqs = 0
    for b in range(B):
        mg = orc.top1_margin(want["logits"][b])
        a = int(want["accepted_len"][b])
        for j in range(ks[b] + 1):
            if mg[j] >= 2 * tol:
                assert got_g[b, j] == want["greedy"][b, j], (b, j)
            else:
                assert util.near_tie_ok(want["logits"][b][j], int(got_g[b, j]), tol), (b, j)
        assert (got_g[b, ks[b] + 1:] == -1).all()
        if (mg[:a + 1] >= 2 * tol).all():
            decisive_seqs += 1
            assert ses.accepted_len[b].item() == a
            assert ses.n_out[b].item() == a + 1
            assert np.array_equal(ses.out_tokens[b].cpu().numpy(), want["out_tokens"][b])
            assert ses.next_last_tok[b].item() == want["next_last_tok"][b]
            assert kvd.ctx_lens[b].item() == want["ctx_lens"][b]
            assert ses.blocks_in_use[b].item() == want["blocks_in_use"][b]
        row += ks[b] + 1
    assert decisive_seqs >= ((3 * B) // 4 if min_decisive is None else min_decisive), (decisive_seqs, B)
    # committed cache rows of the decisive sequences
    ok_caches = [c if (orc.top1_margin(want["logits"][b])[:int(want["accepted_len"][b]) + 1] >= 2 * tol).all() else
                 None for b, c in enumerate(caches)]
    for l in range(desc.n_layers):
        kp, vp = kvd.download(l)
        img = synth.PagedKV(16, kp.shape[0], kvh.block_tables.shape[1], kvh.block_tables, None, {l: kp}, {l: vp})
        for b, c in enumerate(ok_caches):
            if c is None:
                continue
            K, V = synth.gather_sequence_kv(img, l, b, c.ctx)
            # the pages hold fp16: at most half an ulp (2^-12 relative; 2^-10 allowed) of storage rounding, on top
            # of the absolute noise the fp16 activations upstream leave on O(1) values
            for got, ref in ((K, c.K[l]), (V, c.V[l])):
                assert (np.abs(got - ref) <= 2.0 ** -10 * np.abs(ref) + 1e-2).all()
    _check_acr(ses, t_k, ks, wl.n_drafts)
    return err, decisive_seqs


def test_opt13b_width_two_layers(hb):
    # full OPT-13B width and batch shape, 2 of 40 layers
    err, dec = _reduced_case(hb, synth.WORKLOADS[1], 2, 8, 4)
    print("opt13b-width L=2 max |dlogit| = %.2e, decisive %d/8" % (err, dec))


def test_llama70b_width_one_layer_b16_k8(hb):
    # full Llama-2-70B width, B=16, k=8, ctx=1024, 1 of 80 layers
    err, dec = _reduced_case(hb, synth.WORKLOADS[2], 1, 16, 4)
    print("llama70b-width L=1 max |dlogit| = %.2e, decisive %d/16" % (err, dec))


def test_llama70b_width_ragged_paged(hb):
    # ragged contexts and speculation lengths (the paged, adaptive-k configuration), reduced batch
    wl = synth.WORKLOADS[3]
    ctx = [256, 2048, 700, 1023, 257, 1500, 16, 333, 1024, 15, 640, 1999]
    ks = [1, 16, 5, 9, 16, 2, 7, 12, 3, 1, 10, 4]
    err, dec = _reduced_case(hb, wl, 1, 12, 3, ctx_override=ctx, k_override=ks)
    print("llama70b-width ragged max |dlogit| = %.2e, decisive %d/12" % (err, dec))


def test_llama70b_width_full_ragged_batch(hb):
    # the ragged workload as the bench runs it: all 64 sequences, contexts and speculation lengths from the
    # workload's own seed (M = 631 rows: the many-rows GEMM, the attention work list over 64 unequal sequences),
    # 1 of 80 layers
    wl = synth.WORKLOADS[3]
    # (up to 17 scored positions per sequence: fewer sequences have a decisive margin at every one of them than
    # in the short cases, so half of the batch is asked for; the others are still held to the near-tie rule)
    err, dec = _reduced_case(hb, wl, 1, wl.batch, 3, min_decisive=wl.batch // 2)
    print("llama70b-width full ragged batch max |dlogit| = %.2e, decisive %d/%d" % (err, dec, wl.batch))


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6])
def test_small_models_drawn_batches(hb, seed):
    """Small models of every kind the library runs (Llama-style bf16 with grouped-query heads of 128 and of 64, OPT-style
    bf16 and fp32), each on a drawn batch: 1-12 sequences, contexts 0-300 (0: prefill), 0-12 speculated tokens."""
    g = synth.stream(4242, seed)
    descs = [synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 2, 1024, 8, 2, 128, 2048, 1000, 4096),
             synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 2, 512, 8, 4, 64, 1024, 777, 4096),
             synth.ModelDesc(synth.ARCH_OPT, synth.DT_BF16, 2, 512, 4, 4, 128, 2048, 1000, 2048),
             synth.OPT_TINY]
    desc = descs[seed % len(descs)]
    B = int(g.integers(1, 13))
    ctx = g.integers(0, 301, size=B)
    ks = g.integers(0, 13, size=B)
    ks[int(g.integers(0, B))] = 12
    wl = synth.Workload("drawn-%d" % seed, desc, B, 0, 300, 0, 12, 3, 0.3, seed=9000 + seed)
    err, dec = _reduced_case(hb, wl, desc.n_layers, B, 2, ctx_override=ctx.tolist(), k_override=ks.tolist(), min_decisive=0)
    print("drawn batch %d: B=%d max |dlogit| = %.2e, decisive %d/%d" % (seed, B, err, dec, B))


def test_llama160m_width_few_rows(hb):
    # the drafting models' shape (head_dim 64, bf16 storage) with 1 to 4 scored positions per sequence: the
    # few-row attention kernel, this step's own keys read back from the pages like the cached ones; 2 of 12 layers
    wl = synth.Workload("llama160m-bf16-few-rows", synth.LLAMA_160M, 10, 0, 0, 0, 3, 3, 0.3, seed=1240)
    ctx = [512, 1, 63, 64, 65, 1000, 16, 129, 300, 47]
    ks = [0, 3, 1, 2, 0, 3, 3, 0, 1, 2]
    err, dec = _reduced_case(hb, wl, 2, 10, 4, ctx_override=ctx, k_override=ks)
    print("llama160m-width few rows max |dlogit| = %.2e, decisive %d/10" % (err, dec))


def test_one_pass_equals_sequential_decodes_two_layers(hb):
    """Scoring k + 1 positions in one pass against k + 1 single-position passes of the library itself (section 2.1:
    the speculated tokens are scored in parallel with the outcome of scoring them one by one), at the 70B width and
    two layers.  Both decodings multiply the same numbers (the scored rows' K/V are in the pages in fp16 for both);
    what is left is the order of the fp32 sums in launches of other shapes, an fp16 rounding tipped now and then:
    a third of the bf16-path tolerance."""
    harness, binding = hb
    wl = synth.WORKLOADS[2]
    desc = wl.desc.with_layers(2)
    B, k = 6, 5
    g = synth.stream(9876, 1)
    ctx = g.integers(40, 400, size=B).astype(np.int32)
    ks = np.full(B, k, np.int32)
    model = harness.DeviceModel.from_host(desc, synth.make_weights(desc, 77))
    kvd = harness.DeviceKV.from_host(desc, synth.make_paged_kv(desc, ctx, ks, 77))
    ctx0 = kvd.ctx_lens.clone()
    max_ctx = int((ctx + ks + 1).max())
    last = _i32(g.integers(0, desc.vocab, size=B))
    toks = _i32(g.integers(0, desc.vocab, size=(B, k)))                 # the tokens both decodings are fed
    ses = harness.VerifySession(model, kvd, B, k, 1, max_ctx, max_rows=B * (k + 1), want_logits=True)
    ses.forward(last, _i32(ks), ks.tolist(), voted=toks)
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    one_pass = ses.logits.cpu().numpy().reshape(B, k + 1, -1).copy()
    one = harness.VerifySession(model, kvd, B, 0, 1, max_ctx, max_rows=B, want_logits=True)
    zeros, dummy = _i32(np.zeros(B)), _i32(np.zeros((B, 1)))
    seq = []
    for j in range(k + 1):
        cur = last if j == 0 else toks[:, j - 1].contiguous()
        kvd.ctx_lens.copy_(ctx0 + j)                                    # the rows scored so far are committed
        one.forward(cur, zeros, [0] * B, voted=dummy)
        torch.cuda.synchronize()
        assert one.dev_status.item() == 0
        seq.append(one.logits.cpu().numpy().copy())
    kvd.ctx_lens.copy_(ctx0)
    seq = np.stack(seq, axis=1)
    worst = float(np.abs(one_pass - seq).max())
    print("one pass vs sequential, 2 layers at the 70B width: max |dlogit| = %.2e" % worst)
    assert worst < util.TOL[synth.DT_BF16] / 3, worst
