"""How the logit error of the bf16-storage path grows with the number of layers, element by element against
the CPU oracle: the Llama-2-70B width at 1, 2, 4 and 8 layers (the benchmark's batch: 16 sequences, 1024 cached
tokens, 8 speculated), and all 80 layers at a reduced width (d_model 1024, grouped-query heads 8/2 x 128, SwiGLU,
RMSNorm, rotary positions: the same code paths).  Prefixes of one model share its weights (layer l's parameters do
not depend on the depth), so the table is one model seen after 1, 2, 4, ... layers.  The measured table is
printed.  Bounds: the tolerance of the bf16 path (3e-2) at every depth of the reduced width and up to 4 layers of
the 70B width, beyond that its square-root growth (tests/util.py::logit_tol_at_depth)."""
import numpy as np
import pytest
import torch

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth
from tests import util

pytestmark = pytest.mark.gpu
TOL = util.TOL[synth.DT_BF16]


def _i32(a):
    return torch.tensor(np.asarray(a, np.int32), dtype=torch.int32, device="cuda:0")


def _prefix(W, n):
    out = {k: v for k, v in W.items() if k != "layers"}
    out["layers"] = W["layers"][:n]
    return out


def _depth_table(desc, seed, ctx, ks, depths):
    """max |logit - oracle| and the fraction of positions with the oracle's token, after each depth."""
    from paper_2402_15678_amd import harness
    W = synth.make_weights(desc, seed)
    full = harness.DeviceModel.from_host(desc, W)
    B = len(ctx)
    k_max = int(ks.max())
    kvh = synth.make_paged_kv(desc, ctx, ks, seed)
    kvd = harness.DeviceKV.from_host(desc, kvh)
    g = synth.stream(seed, 700)
    last = g.integers(0, desc.vocab, size=B).astype(np.int32)
    voted = g.integers(0, desc.vocab, size=(B, k_max)).astype(np.int32)
    toks = [[int(last[b])] + [int(t) for t in voted[b, :ks[b]]] for b in range(B)]
    M = int((ks + 1).sum())
    t_last, t_voted, t_spec = _i32(last), _i32(voted), _i32(ks)
    rows = []
    for n in depths:
        d_n = desc.with_layers(n)
        t_n = {k: v for k, v in full.t.items() if k != "layers"}
        t_n["layers"] = full.t["layers"][:n]
        model = harness.DeviceModel(d_n, t_n)                    # the first n layers of the same device tensors
        ses = harness.VerifySession(model, kvd, B, k_max, 1, int((ctx + ks + 1).max()), max_rows=M, want_logits=True)
        ses.forward(t_last, t_spec, ks.tolist(), voted=t_voted)  # (nothing is committed: the cache stays as drawn)
        torch.cuda.synchronize()
        assert ses.dev_status.item() == 0
        got = ses.logits.cpu().numpy()
        caches = []
        for b in range(B):
            kv = [synth.gather_sequence_kv(kvh, l, b, int(ctx[b])) for l in range(n)]
            caches.append(orc.SeqCache(n, desc.n_kv_heads, desc.head_dim, [k for k, _ in kv], [v for _, v in kv]))
        want = np.concatenate(orc.decoder_step(d_n, _prefix(W, n), toks, caches))
        err = np.abs(got - want)
        margin = orc.top1_margin(want)
        same = got.argmax(axis=1) == want.argmax(axis=1)
        assert same[margin >= 2 * TOL].all() or err.max() >= TOL   # decisive positions keep their token within tol
        rows.append((n, float(err.max()), float(np.sqrt((err ** 2).mean())), float(want.std()), float(same.mean()),
                     int((margin >= 2 * TOL).sum()), M))
        model.close()
    return rows


def _show(title, rows):
    print("\n" + title)
    print("layers  max|dlogit|  rms|dlogit|  logit std  same argmax  decisive/positions")
    for n, mx, rms, sd, same, dec, M in rows:
        print("%6d  %11.3e  %11.3e  %9.3f  %11.3f  %d/%d" % (n, mx, rms, sd, same, dec, M))


def test_logit_error_against_the_oracle_at_70b_width_1_to_8_layers():
    wl = synth.WORKLOADS[2]
    desc = wl.desc.with_layers(8)
    ctx, ks = synth.draw_ctx_lens(wl), synth.draw_spec_lens(wl)
    rows = _depth_table(desc, wl.seed, ctx, ks, (1, 2, 4, 8))
    _show("Llama-2-70B width, B=16, ctx=1024, k=8 (M=144)", rows)
    for n, mx, *_ in rows:
        assert mx < util.logit_tol_at_depth(n), (n, mx)


def test_logit_error_against_the_oracle_at_80_layers_reduced_width():
    desc = synth.ModelDesc(synth.ARCH_LLAMA, synth.DT_BF16, 80, 1024, 8, 2, 128, 3584, 32000, 4096)
    g = synth.stream(4321, 1)
    B = 8
    ctx = g.integers(64, 321, size=B).astype(np.int32)
    ks = np.array([8, 8, 8, 3, 8, 0, 8, 5], np.int32)
    rows = _depth_table(desc, 4321, ctx, ks, (1, 2, 4, 8, 16, 40, 80))
    _show("d_model 1024, 8/2 heads x 128, FFN 3584, 80 layers, B=8, ctx 64-320", rows)
    for n, mx, *_ in rows:
        assert mx < TOL, (n, mx)
