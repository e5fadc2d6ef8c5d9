"""GPU edge cases through the C ABI: degenerate batches, device-detected errors (the sequence becomes a
no-op and nothing of it reaches the cache), run-to-run bit reproducibility, plain decode (k = 0),
and the one-pass == sequential-decodes invariant on the device."""
import numpy as np
import pytest
import torch

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth
from tests import util

pytestmark = pytest.mark.gpu

DESC = synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 2, 256, 8, 2, 128, 512, 1000, 512)


@pytest.fixture(scope="module")
def env():
    from paper_2402_15678_amd import binding, harness
    W = synth.make_weights(DESC, 77)
    model = harness.DeviceModel.from_host(DESC, W)
    return harness, binding, W, model


def _i32(a):
    return torch.tensor(np.asarray(a, np.int32), dtype=torch.int32, device="cuda:0")


def _setup(harness, model, ctx, ks, seed=3, want_logits=True):
    kvh = synth.make_paged_kv(DESC, ctx, ks, seed)
    kvd = harness.DeviceKV.from_host(DESC, kvh)
    B = len(ctx)
    ses = harness.VerifySession(model, kvd, B, int(max(ks)), 3, int((np.asarray(ctx) + np.asarray(ks) + 1).max()),
                                max_rows=int((np.asarray(ks) + 1).sum()), want_logits=want_logits)
    return kvh, kvd, ses


def test_empty_batch_is_a_noop(env):
    harness, binding, W, model = env
    kv = binding.KV(None, None, 16, 1, 1, None, None)
    binding.mn_mv_vote(model.ctx, None, None, None, 0, 3, 4, 0, None, None)
    binding.mn_verify_forward(model.ctx, None, None, None, binding.host_i32([]), 0, 4, 0, kv, None, None, None, 0)
    binding.mn_accept_and_commit(model.ctx, None, None, None, 0, 4, kv, None, None, None, None, None)
    torch.cuda.synchronize()


def test_plain_decode_k0_and_mixed_lengths(env):
    harness, binding, W, model = env
    ctx, ks = np.array([17, 40, 16, 1], np.int32), np.array([0, 3, 0, 5], np.int32)
    kvh, kvd, ses = _setup(harness, model, ctx, ks)
    g = synth.stream(5, 1)
    last = g.integers(0, DESC.vocab, size=4).astype(np.int32)
    drafts = g.integers(0, DESC.vocab, size=(4, 3, 5)).astype(np.int32)
    caches = util.oracle_caches(DESC, kvh)
    want = orc.verify_step(DESC, W, caches, last, drafts, ks, np.ones(3, np.float32))
    t = [_i32(last), _i32(drafts), _i32(ks), torch.ones(3, device="cuda:0")]
    ses.step(t[0], t[1], t[2], ks.tolist(), t[3])
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    assert np.array_equal(ses.voted.cpu().numpy(), want["voted"])
    assert np.abs(ses.logits.cpu().numpy() - np.concatenate(want["logits"])).max() < 3e-2
    margins = [orc.top1_margin(l) for l in want["logits"]]
    for b in range(4):
        if margins[b].min() >= 6e-2:
            assert np.array_equal(ses.greedy[b].cpu().numpy(), want["greedy"][b])
            assert ses.accepted_len[b].item() == want["accepted_len"][b]
            assert kvd.ctx_lens[b].item() == want["ctx_lens"][b]
            assert ses.n_out[b].item() == want["n_out"][b]


def test_bit_reproducible_run_to_run(env):
    harness, binding, W, model = env
    ctx, ks = np.array([100, 33, 257], np.int32), np.array([4, 7, 2], np.int32)
    g = synth.stream(6, 1)
    last, drafts = _i32(g.integers(0, DESC.vocab, size=3)), _i32(g.integers(0, DESC.vocab, size=(3, 3, 7)))
    spec, w = _i32(ks), torch.ones(3, device="cuda:0")
    outs = []
    for _ in range(2):
        kvh, kvd, ses = _setup(harness, model, ctx, ks)
        ses.step(last, drafts, spec, ks.tolist(), w)
        torch.cuda.synchronize()
        outs.append((ses.logits.clone(), ses.greedy.clone(), kvd.k_pages[1].clone(), kvd.ctx_lens.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)                                              # no float atomics: identical bits


def test_step_replays_from_a_captured_graph(env):
    """The whole step (vote -> forward -> accept + commit) issues only kernel launches on the caller's stream, so
    a caller may capture it once and replay it.  Three replays, with eager work and synchronisations in between,
    each against the eager result bit for bit (logits, tokens, cache pages, committed contexts)."""
    harness, binding, W, model = env
    ctx, ks = np.array([100, 33, 257, 0], np.int32), np.array([4, 7, 2, 5], np.int32)
    g = synth.stream(6, 2)
    last, drafts = _i32(g.integers(0, DESC.vocab, size=4)), _i32(g.integers(0, DESC.vocab, size=(4, 3, 7)))
    spec, w = _i32(ks), torch.ones(3, device="cuda:0")
    ctx0 = _i32(ctx)
    kvh, kvd, ses = _setup(harness, model, ctx, ks)
    ses.step(last, drafts, spec, ks.tolist(), w)                             # eager: the reference, and the warm-up
    torch.cuda.synchronize()
    want = [t.clone() for t in (ses.logits, ses.greedy, ses.out_tokens, ses.accepted_len, kvd.k_pages[1], kvd.v_pages[0],
                                kvd.ctx_lens)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        kvd.ctx_lens.copy_(ctx0)
        with torch.cuda.graph(graph, stream=side):
            ses.step(last, drafts, spec, ks.tolist(), w)
    torch.cuda.current_stream().wait_stream(side)
    for r in range(3):
        kvd.ctx_lens.copy_(ctx0)
        for t in (ses.logits, ses.greedy, ses.out_tokens, ses.accepted_len):
            t.fill_(-3)
        graph.replay()
        torch.cuda.synchronize()
        got = (ses.logits, ses.greedy, ses.out_tokens, ses.accepted_len, kvd.k_pages[1], kvd.v_pages[0], kvd.ctx_lens)
        for a, b in zip(got, want):
            assert torch.equal(a, b), r
        assert ses.dev_status.item() == 0
        # eager work of the program between the replays
        kvd.ctx_lens.copy_(ctx0)
        ses.step(last, drafts, spec, ks.tolist(), w)
        torch.cuda.synchronize()


def test_one_pass_equals_sequential_decodes_on_the_device(env):
    harness, binding, W, model = env
    ctx, k = np.array([50, 16, 129], np.int32), 5
    ks = np.full(3, k, np.int32)
    g = synth.stream(7, 1)
    last = g.integers(0, DESC.vocab, size=3).astype(np.int32)
    toks = g.integers(0, DESC.vocab, size=(3, k)).astype(np.int32)
    kvh, kvd, ses = _setup(harness, model, ctx, ks)
    t_last, t_voted, t_spec = _i32(last), _i32(toks), _i32(ks)
    ses.forward(t_last, t_spec, ks.tolist(), voted=t_voted)
    torch.cuda.synchronize()
    one = ses.logits.cpu().numpy().reshape(3, k + 1, -1)
    # the same tokens one at a time, committing each (ctx_lens advances by one per step)
    kvh2, kvd2, seq = _setup(harness, model, ctx, np.zeros(3, np.int32) + k)  # blocks for all k+1 positions
    single = harness.VerifySession(model, kvd2, 3, 0, 1, int(ctx.max()) + k + 1, max_rows=3, want_logits=True)
    zeros = _i32(np.zeros(3)); dummy = _i32(np.zeros((3, 1)))
    for j in range(k + 1):
        cur = _i32(last if j == 0 else toks[:, j - 1])
        single.forward(cur, zeros, [0, 0, 0], voted=dummy)
        torch.cuda.synchronize()
        step_logits = single.logits.cpu().numpy()
        # fp16 activations both ways; the sequential path re-reads its own K/V rounded to bf16 from the cache
        assert np.abs(step_logits - one[:, j]).max() < 3e-2, j
        kvd2.ctx_lens.add_(1)


def test_device_detected_errors_disable_only_the_bad_sequence(env):
    harness, binding, W, model = env
    ctx, ks = np.array([30, 45, 60], np.int32), np.array([3, 3, 3], np.int32)
    g = synth.stream(8, 1)
    last = g.integers(0, DESC.vocab, size=3).astype(np.int32)
    voted = g.integers(0, DESC.vocab, size=(3, 3)).astype(np.int32)
    # reference run
    kvh, kvd, ses = _setup(harness, model, ctx, ks)
    t = [_i32(last), _i32(voted), _i32(ks)]
    ses.forward(t[0], t[2], ks.tolist(), voted=t[1])
    torch.cuda.synchronize()
    ref_greedy, ref_k = ses.greedy.cpu().numpy().copy(), kvd.k_pages[0].clone()
    # (a) sequence 1 gets a block id out of range
    kvh2, kvd2, ses2 = _setup(harness, model, ctx, ks)
    before = kvd2.k_pages[0].clone()
    bt = kvd2.block_tables.clone(); bt[1, 0] = 10 ** 6
    kvd2.block_tables.copy_(bt)
    ses2.forward(t[0], t[2], ks.tolist(), voted=t[1])
    ses2.accept(t[2], voted=t[1])
    torch.cuda.synchronize()
    assert ses2.dev_status.item() & binding.MN_DEV_BLOCK_TABLE
    got = ses2.greedy.cpu().numpy()
    assert (got[1] == -1).all() and np.array_equal(got[[0, 2]], ref_greedy[[0, 2]])
    assert ses2.n_out.cpu().tolist()[1] == 0 and ses2.next_last_tok.cpu().tolist()[1] == -1
    assert kvd2.ctx_lens.cpu().tolist()[1] == 45                               # untouched
    # nothing of sequence 1 reached the cache: pages differ from `before` only where sequences 0 and 2 wrote
    changed = (kvd2.k_pages[0] != before).flatten(1).any(dim=1).nonzero().flatten().cpu().tolist()
    own_blocks = set(kvh2.block_tables[1][kvh2.block_tables[1] >= 0].tolist())
    assert not (set(changed) & own_blocks)
    # (b) a token id outside the vocabulary
    kvh3, kvd3, ses3 = _setup(harness, model, ctx, ks)
    bad = voted.copy(); bad[2, 1] = DESC.vocab + 5
    tb = _i32(bad)
    ses3.forward(t[0], t[2], ks.tolist(), voted=tb)
    torch.cuda.synchronize()
    assert ses3.dev_status.item() & binding.MN_DEV_TOKEN
    assert (ses3.greedy[2].cpu().numpy() == -1).all() and np.array_equal(ses3.greedy[:2].cpu().numpy(), ref_greedy[:2])
    # (c) device spec_len disagrees with the host copy: the whole batch is disabled, nothing is written
    kvh4, kvd4, ses4 = _setup(harness, model, ctx, ks)
    before4 = kvd4.k_pages[0].clone()
    wrong = _i32([3, 2, 3])
    ses4.forward(t[0], wrong, ks.tolist(), voted=t[1])
    torch.cuda.synchronize()
    assert ses4.dev_status.item() & binding.MN_DEV_SPEC_LEN
    assert (ses4.greedy.cpu().numpy() == -1).all() and torch.equal(kvd4.k_pages[0], before4)


def test_context_beyond_the_hosts_max_ctx_disables_the_sequence(env):
    """max_ctx sizes the attention launch on the host; ctx_lens lives on the device and may have moved on.  A
    sequence whose ctx_b + k_b + 1 exceeds max_ctx sets MN_DEV_CTX and becomes a no-op, the others are unaffected."""
    harness, binding, W, model = env
    ctx, ks = np.array([30, 45, 60], np.int32), np.array([3, 3, 3], np.int32)
    g = synth.stream(8, 3)
    t = [_i32(g.integers(0, DESC.vocab, size=3)), _i32(g.integers(0, DESC.vocab, size=(3, 3))), _i32(ks)]
    kvh, kvd, ref = _setup(harness, model, ctx, ks)
    ref.forward(t[0], t[2], ks.tolist(), voted=t[1])
    torch.cuda.synchronize()
    assert ref.dev_status.item() == 0
    kvh2, kvd2 = synth.make_paged_kv(DESC, ctx, ks, 3), None
    kvd2 = harness.DeviceKV.from_host(DESC, kvh2)
    before = kvd2.k_pages[0].clone()
    short = harness.VerifySession(model, kvd2, 3, 3, 3, 55, max_rows=12, want_logits=True)   # sequence 2 needs 64
    short.forward(t[0], t[2], ks.tolist(), voted=t[1])
    short.accept(t[2], voted=t[1])
    torch.cuda.synchronize()
    assert short.dev_status.item() == binding.MN_DEV_CTX
    got = short.greedy.cpu().numpy()
    assert (got[2] == -1).all() and np.array_equal(got[:2], ref.greedy.cpu().numpy()[:2])
    assert torch.equal(short.logits[:8], ref.logits[:8])
    assert short.n_out.cpu().tolist()[2] == 0 and kvd2.ctx_lens.cpu().tolist()[2] == 60
    changed = (kvd2.k_pages[0] != before).flatten(1).any(dim=1).nonzero().flatten().cpu().tolist()
    own = set(kvh2.block_tables[2][kvh2.block_tables[2] >= 0].tolist())
    assert not (set(changed) & own)


def test_values_beyond_the_fp16_range_saturate_and_are_reported(env):
    """bf16 models multiply in fp16.  A weight beyond +-65504 is saturated when it is packed, an activation beyond
    it when it is stored; both set MN_DEV_RANGE, and no infinity or NaN reaches the logits."""
    harness, binding, W, model = env
    # (a) weight packing: one entry of 1e5 (a bf16 value) and one of -3e38
    g = synth.stream(8, 4)
    w = synth.storage_round(g.standard_normal((256, 256), dtype=np.float32) * 0.05, synth.DT_BF16)
    big_vals = synth.storage_round(np.array([1e5, -3e38], np.float32), synth.DT_BF16)
    w[7, 130], w[200, 3] = big_vals[0], big_vals[1]
    st = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    packed = harness.pack_matrix(harness.to_device(w, synth.DT_BF16), 0, st)
    clean = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    harness.pack_matrix(harness.to_device(np.clip(w, -1.0, 1.0), synth.DT_BF16), 0, clean)
    a = np.zeros((16, 256), np.float32); a[0, 130] = 1.0; a[1, 3] = 0.5; a[2, :] = 0.25
    out = torch.full((16, 256), float("nan"), dtype=torch.float32, device="cuda:0")
    a_d = harness.to_device_act(a, synth.DT_BF16)
    binding.mn_proj_gemm(None, a_d.data_ptr(), packed.data_ptr(), None, out.data_ptr(), 16, 256, 256, 1, None, 0,
                         harness.stream_ptr())
    torch.cuda.synchronize()
    assert st.item() == binding.MN_DEV_RANGE and clean.item() == 0
    got = out.cpu().numpy()
    assert np.isfinite(got).all()
    assert got[0, 7] == 65280.0 and got[1, 200] == -32640.0         # saturated to the largest bf16 value fp16 holds
    wc = np.clip(w.astype(np.float64), -65280.0, 65280.0)
    assert np.abs(got - a.astype(np.float64) @ wc.T).max() < 1e-2
    # (b) activations: first FFN matrix of layer 0 scaled up until silu(gate) * up leaves the range
    import copy
    W2 = copy.deepcopy(W)
    W2["layers"][0]["w1"] = synth.storage_round(W2["layers"][0]["w1"] * 4096.0, synth.DT_BF16)
    big = harness.DeviceModel.from_host(DESC, W2)
    ctx, ks = np.array([30, 45], np.int32), np.array([3, 2], np.int32)
    t = [_i32(g.integers(0, DESC.vocab, size=2)), _i32(g.integers(0, DESC.vocab, size=(2, 3))), _i32(ks)]
    kvh, kvd, ses = _setup(harness, big, ctx, ks)
    ses.forward(t[0], t[2], ks.tolist(), voted=t[1])
    torch.cuda.synchronize()
    assert ses.dev_status.item() == binding.MN_DEV_RANGE
    assert torch.isfinite(ses.logits).all()
    assert (ses.greedy.cpu().numpy()[0, :4] >= 0).all() and (ses.greedy.cpu().numpy()[1, :3] >= 0).all()
    # the same batch on the unscaled model reports nothing
    kvh, kvd, ses = _setup(harness, model, ctx, ks)
    ses.forward(t[0], t[2], ks.tolist(), voted=t[1])
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0


def test_few_row_attention_path_disables_only_the_bad_sequence():
    """The drafting models' shape (head_dim 64, one to four rows per sequence) takes its own attention kernel:
    a sequence with a damaged block table becomes a no-op there too, the others are unaffected, plain decode
    (k = 0) and short speculations mix in one batch."""
    from paper_2402_15678_amd import binding, harness
    desc = synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 2, 256, 4, 4, 64, 512, 1000, 512)
    model = harness.DeviceModel.from_host(desc, synth.make_weights(desc, 78))
    ctx, ks = np.array([30, 45, 60, 0, 129], np.int32), np.array([0, 3, 1, 2, 0], np.int32)
    g = synth.stream(8, 2)
    last = _i32(g.integers(0, desc.vocab, size=5))
    voted = _i32(g.integers(0, desc.vocab, size=(5, 3)))
    spec = _i32(ks)

    def run(damage):
        kvh = synth.make_paged_kv(desc, ctx, ks, 3)
        kvd = harness.DeviceKV.from_host(desc, kvh)
        if damage:
            bt = kvd.block_tables.clone(); bt[1, 1] = 10 ** 6
            kvd.block_tables.copy_(bt)
        ses = harness.VerifySession(model, kvd, 5, 3, 1, int((ctx + ks + 1).max()), max_rows=int((ks + 1).sum()),
                                    want_logits=True)
        ses.forward(last, spec, ks.tolist(), voted=voted)
        ses.accept(spec, voted=voted)
        torch.cuda.synchronize()
        return kvh, kvd, ses

    _, kvd0, ref = run(False)
    assert ref.dev_status.item() == 0 and (ref.greedy.cpu().numpy()[:, 0] >= 0).all()
    kvh1, kvd1, bad = run(True)
    assert bad.dev_status.item() & binding.MN_DEV_BLOCK_TABLE
    got, want = bad.greedy.cpu().numpy(), ref.greedy.cpu().numpy()
    assert (got[1] == -1).all() and np.array_equal(got[[0, 2, 3, 4]], want[[0, 2, 3, 4]])
    assert bad.n_out.cpu().tolist()[1] == 0 and kvd1.ctx_lens.cpu().tolist()[1] == 45
    ok_rows = [0, 5, 6, 7, 8, 9, 10]                       # rows of sequences 0, 2, 3, 4 (sequence 1 owns rows 1-4)
    assert torch.equal(bad.logits[ok_rows], ref.logits[ok_rows])
    assert [kvd1.ctx_lens.cpu().tolist()[b] for b in (0, 2, 3, 4)] == [kvd0.ctx_lens.cpu().tolist()[b] for b in (0, 2, 3, 4)]


def test_measuring_sticks_run_and_report_plausible_rates(env):
    """The probes behind the ABI: they launch, finish, and land in the range of a working MI355X
    (loose bounds: they are a ruler for the bench, not a performance test)."""
    harness, binding = env[0], env[1]
    buf = torch.empty((1 << 28,), dtype=torch.uint8, device="cuda:0").fill_(1)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.mn_probe_stream_read(buf.data_ptr(), buf.numel(), harness.stream_ptr())
    e0.record()
    for _ in range(5):
        binding.mn_probe_stream_read(buf.data_ptr(), buf.numel(), harness.stream_ptr())
    e1.record()
    torch.cuda.synchronize()
    gbps = 5.0 * buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
    assert 1000.0 < gbps < 8000.0, gbps
    binding.mn_probe_mfma(100, harness.stream_ptr())
    e0.record()
    flop = binding.mn_probe_mfma(4000, harness.stream_ptr())
    e1.record()
    torch.cuda.synchronize()
    tflops = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    assert 300.0 < tflops < 2600.0, tflops
    binding.mn_probe_mfma_data(100, harness.stream_ptr())
    e0.record()
    flop = binding.mn_probe_mfma_data(4000, harness.stream_ptr())
    e1.record()
    torch.cuda.synchronize()
    on_data = flop / (e0.elapsed_time(e1) * 1e-3) / 1e12
    assert 300.0 < on_data < 2600.0, on_data


def test_largest_batch_many_rows(env):
    """MN_MAX_BATCH sequences in one step (thousands of rows: the many-rows GEMM, attention over thousands of
    short sequences); a sample of sequences is checked against the oracle, which treats them one by one."""
    harness, binding, W, model = env
    B = 4096
    g = synth.stream(8, 1)
    ctx = g.integers(1, 41, size=B).astype(np.int32)
    ks = g.integers(0, 3, size=B).astype(np.int32)
    kvh = synth.make_paged_kv(DESC, ctx, ks, 11)
    kvd = harness.DeviceKV.from_host(DESC, kvh)
    M = int((ks + 1).sum())
    ses = harness.VerifySession(model, kvd, B, 2, 3, int((ctx + ks + 1).max()), max_rows=M, want_logits=True)
    last = g.integers(0, DESC.vocab, size=B).astype(np.int32)
    drafts = g.integers(0, DESC.vocab, size=(B, 3, 2)).astype(np.int32)
    t = [_i32(last), _i32(drafts), _i32(ks), torch.ones(3, device="cuda:0")]
    ses.step(t[0], t[1], t[2], ks.tolist(), t[3])
    torch.cuda.synchronize()
    assert ses.dev_status.item() == 0
    pick = np.unique(np.concatenate([[0, B - 1], g.integers(0, B, size=10)]))
    caches = util.oracle_caches(DESC, _subset_kv(kvh, pick))
    want = orc.verify_step(DESC, W, caches, last[pick], drafts[pick], ks[pick], np.ones(3, np.float32))
    row0 = np.concatenate([[0], np.cumsum(ks + 1)])
    logits = ses.logits.cpu().numpy()
    voted = ses.voted.cpu().numpy()
    for i, b in enumerate(pick):
        assert np.array_equal(voted[b, :ks[b]], want["voted"][i, :ks[b]])
        got = logits[row0[b]:row0[b + 1]]
        assert np.abs(got - want["logits"][i]).max() < 3e-2
        if orc.top1_margin(want["logits"][i]).min() >= 6e-2:
            assert ses.accepted_len[b].item() == want["accepted_len"][i]
            assert kvd.ctx_lens[b].item() == want["ctx_lens"][i]
    # every sequence advanced by its accepted length + 1
    adv = kvd.ctx_lens.cpu().numpy() - ctx
    assert np.array_equal(adv, ses.accepted_len.cpu().numpy() + 1)
    assert (ses.n_out.cpu().numpy() == adv).all()


def _subset_kv(kvh, seqs):
    """A PagedKV image restricted to some sequences (same pages, only their block-table rows)."""
    import dataclasses
    return dataclasses.replace(kvh, block_tables=kvh.block_tables[seqs], ctx_lens=np.asarray(kvh.ctx_lens)[seqs])
