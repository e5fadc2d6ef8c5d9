"""No GPU needed: the C-ABI library loads, exports every symbol the header declares, and reports
host-visible argument errors before anything would be launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "minions_verify.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2402_15678_amd import binding
    return binding


def _declared():
    src = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(mn_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(binding):
    names = _declared()
    assert len(names) >= 12
    for n in names:
        assert hasattr(binding.lib, n), n
    assert set(names) == set(binding.EXPORTS)


def _desc(binding, **kw):
    d = dict(arch=1, dtype=1, n_layers=1, d_model=256, n_heads=2, n_kv_heads=1, head_dim=128, d_ffn=256, vocab=64,
             max_pos=128, norm_eps=1e-5, rope_base=10000.0)
    d.update(kw)
    return binding.ModelDesc(*[d[k] for k, _ in binding.ModelDesc._fields_])


def _weights(binding, n_layers=1):
    w = binding.Weights()
    fake = 0x1000  # never dereferenced by mn_create
    w.tok_emb = w.pos_emb = w.final_norm_g = w.final_norm_b = w.lm_head = fake
    arr = binding.ptr_array([fake] * n_layers)
    for k in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"):
        setattr(w, k, C.cast(arr, C.POINTER(C.c_void_p)))
    return w, arr


def test_create_validates_the_description(binding):
    w, keep = _weights(binding)
    ctx = binding.mn_create(_desc(binding), w)
    assert ctx
    assert binding.mn_workspace_bytes(ctx, 4, 20, 100) > 0
    assert binding.mn_workspace_bytes(ctx, -1, 20, 100) == 0
    binding.mn_destroy(ctx)
    bad = [dict(arch=7), dict(dtype=3), dict(head_dim=48), dict(d_model=100), dict(n_heads=3, n_kv_heads=2),
           dict(arch=0, n_heads=2, n_kv_heads=1), dict(vocab=0), dict(d_model=192), dict(norm_eps=-1.0)]
    for kw in bad:
        with pytest.raises(binding.MinionsError):
            binding.mn_create(_desc(binding, **kw), w)
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_create(_desc(binding), binding.Weights())
    assert e.value.status == binding.MN_ENULL


def test_step_calls_reject_bad_arguments_before_launch(binding):
    w, keep = _weights(binding)
    ctx = binding.mn_create(_desc(binding), w)
    p = 0x1000
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_mv_vote(ctx, p, p, p, 4, 0, 3, 0, p, p)
    assert e.value.status == binding.MN_EINVAL and "n = 0" in str(e.value)
    with pytest.raises(binding.MinionsError):
        binding.mn_mv_vote(ctx, p, p, p, 4, 65, 3, 0, p, p)
    with pytest.raises(binding.MinionsError):
        binding.mn_mv_vote(ctx, p, p, p, 4, 3, 3, 2, p, p)
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_mv_vote(ctx, None, p, p, 4, 3, 3, 0, p, p)
    assert e.value.status == binding.MN_ENULL
    binding.mn_mv_vote(ctx, None, None, None, 0, 3, 3, 0, None, None)          # B = 0: no-op, no launch
    kv = binding.KV(None, None, 16, 8, 4, None, None)
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_verify_forward(ctx, p, p, p, binding.host_i32([1]), 1, 1, 10, kv, p, None, p, 1 << 20)
    assert e.value.status == binding.MN_ENULL                                   # kv members
    arr = binding.ptr_array([p])
    kv = binding.KV(C.cast(arr, C.POINTER(C.c_void_p)), C.cast(arr, C.POINTER(C.c_void_p)), 16, 8, 4, p, p)
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_verify_forward(ctx, p, p, p, binding.host_i32([1]), 1, 1, 100, kv, p, None, p, 1 << 20)
    assert e.value.status == binding.MN_ECAPACITY                               # 100 tokens > 4 blocks of 16
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_verify_forward(ctx, p, p, p, binding.host_i32([5]), 1, 1, 10, kv, p, None, p, 1 << 20)
    assert e.value.status == binding.MN_EINVAL                                  # h_spec_len > k_max
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_verify_forward(ctx, p, p, p, binding.host_i32([1]), 1, 1, 10, kv, p, None, 0x1000, 16)
    assert e.value.status == binding.MN_EWORKSPACE                              # too small
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_verify_forward(ctx, p, p, p, binding.host_i32([1]), 1, 1, 10, kv, p, None, 0x1010, 1 << 30)
    assert e.value.status == binding.MN_EWORKSPACE                              # misaligned
    with pytest.raises(binding.MinionsError):
        binding.mn_accept_and_commit(ctx, p, p, p, 2, 3, binding.KV(None, None, 16, 8, 4, None, None), p, p, p, p, p)
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_proj_gemm(ctx, p, p, None, p, 4, 8, 100)
    assert e.value.status == binding.MN_ESHAPE
    assert binding.mn_packed_weight_bytes(130, 256) == 256 * 256 * 2            # columns padded to 128
    assert binding.mn_packed_weight_bytes(130, 100) == 0
    with pytest.raises(binding.MinionsError):
        binding.mn_pack_weight(p, 0x2000, 64, 256, 48)                          # N != 2 * half
    # the rows after the step and the measuring sticks: argument checks come before any launch
    for bad in [dict(B=-1), dict(n=0), dict(n=65), dict(rf=0.0), dict(pt=0.9, rt=0.1), dict(w=None)]:
        a = dict(B=2, n=3, rt=0.8, pt=0.2, rf=1.5, pf=0.5, w=p)
        a.update(bad)
        with pytest.raises(binding.MinionsError):
            binding.mn_acr_update(ctx, p, p, p, None, a["B"], a["n"], a["rt"], a["pt"], a["rf"], a["pf"], a["w"])
    with pytest.raises(binding.MinionsError):
        binding.mn_acr_update(ctx, None, p, p, None, 2, 3, 0.8, 0.2, 1.5, 0.5, p)   # B > 0 needs the arrays
    for buf, nbytes in [(None, 1 << 24), (p, 1 << 10), (p + 8, 1 << 24)]:
        with pytest.raises(binding.MinionsError):
            binding.mn_probe_stream_read(buf, nbytes)
    for iters in (0, -3, 1 << 23):
        with pytest.raises(binding.MinionsError):
            binding.mn_probe_mfma(iters)
        with pytest.raises(binding.MinionsError):
            binding.mn_probe_mfma_data(iters)
    binding.mn_destroy(ctx)


def _model_shapes():
    """(kwargs of the model description, batch sizes) of the benchmark models and of a drafting-model shape."""
    from paper_2402_15678_amd import synth
    out = []
    for d, Bs in ((synth.OPT_13B, (8,)), (synth.LLAMA2_70B, (16, 64)), (synth.LLAMA_160M, (16,)),
                  (synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 2, 512, 8, 2, 64, 2048, 4096, 4096), (16,)),
                  (synth.OPT_TINY, (1,))):
        kw = dict(arch=d.arch, dtype=d.dtype, n_layers=2, d_model=d.d_model, n_heads=d.n_heads, n_kv_heads=d.n_kv_heads,
                  head_dim=d.head_dim, d_ffn=d.d_ffn, vocab=d.vocab, max_pos=d.max_pos)
        out.append((kw, Bs))
    return out


def test_workspace_for_max_rows_serves_every_smaller_step(binding):
    """mn_workspace_bytes(max_rows) is an upper bound for every step with at most max_rows rows: the k-split of
    a projection (and with it the room its partial sums need) is not monotone in the row count, the query is."""
    for kw, Bs in _model_shapes():
        w, keep = _weights(binding, 2)
        ctx = binding.mn_create(_desc(binding, **kw), w)
        for B in Bs:
            top = 17 * B if B < 64 else 1100
            sizes = [binding.mn_workspace_bytes(ctx, B, m, 2048) for m in range(0, top + 1)]
            assert all(s > 0 for s in sizes)
            worst = 0
            for m, s in enumerate(sizes):
                worst = max(worst, s)
                assert s == worst, (kw["d_model"], B, m, s, worst)     # non-decreasing in the row count
        binding.mn_destroy(ctx)


def test_stochastic_entries_reject_bad_arguments_before_launch(binding):
    p = 0x1000
    vs = lambda **kw: binding.mn_verify_sample(None, kw.get("logits", p), p, p, p, p, kw.get("B", 2), kw.get("k_max", 3),
                                               kw.get("M", 8), kw.get("vocab", 100), kw.get("T", 1.0), 1,
                                               kw.get("step", 0), kw.get("sampled", p))
    for kw, status in [(dict(B=-1), binding.MN_EINVAL), (dict(B=5000), binding.MN_EINVAL), (dict(k_max=-1), binding.MN_EINVAL),
                       (dict(M=9), binding.MN_EINVAL), (dict(vocab=0), binding.MN_EUNSUPPORTED),
                       (dict(vocab=(1 << 21) + 1), binding.MN_EUNSUPPORTED), (dict(T=0.0), binding.MN_EINVAL),
                       (dict(T=float("inf")), binding.MN_EINVAL), (dict(T=float("nan")), binding.MN_EINVAL),
                       (dict(step=1 << 56), binding.MN_EINVAL), (dict(logits=None), binding.MN_ENULL),
                       (dict(sampled=None), binding.MN_ENULL)]:
        with pytest.raises(binding.MinionsError) as e:
            vs(**kw)
        assert e.value.status == status, kw
    binding.mn_verify_sample(None, None, None, None, None, None, 0, 3, 0, 100, 1.0, 1, 0, None)     # B = 0: no launch
    ds = lambda **kw: binding.mn_draft_sample(None, kw.get("logits", p), kw.get("B", 2), kw.get("vocab", 100),
                                              kw.get("T", 1.0), 1, kw.get("step", 0), kw.get("ssm", 0), kw.get("t", 0),
                                              kw.get("tokens", p), kw.get("ts", 1), kw.get("probs", None), kw.get("ps", 0))
    for kw, status in [(dict(B=-1), binding.MN_EINVAL), (dict(vocab=0), binding.MN_EUNSUPPORTED), (dict(T=-1.0), binding.MN_EINVAL),
                       (dict(step=1 << 56), binding.MN_EINVAL), (dict(ssm=-1), binding.MN_EINVAL), (dict(ssm=64), binding.MN_EINVAL),
                       (dict(t=-1), binding.MN_EINVAL), (dict(ts=0), binding.MN_EINVAL), (dict(probs=p, ps=99), binding.MN_EINVAL),
                       (dict(logits=None), binding.MN_ENULL), (dict(tokens=None), binding.MN_ENULL)]:
        with pytest.raises(binding.MinionsError) as e:
            ds(**kw)
        assert e.value.status == status, kw
    binding.mn_draft_sample(None, None, 0, 100, 1.0, 1, 0, 0, 0, None, 1)                             # B = 0: no launch
