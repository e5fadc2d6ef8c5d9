"""The projection entry point that allocates nothing (mn_proj_gemm_noalloc: split-K partial sums in a buffer
built into the library) against mn_proj_gemm with a caller workspace: same kernels, so the same bits.  Two
calls in a row share the built-in buffer, the second on a smaller input; then a request beyond the buffer."""
import numpy as np
import pytest
import torch

from paper_2402_15678_amd import synth

pytestmark = pytest.mark.gpu


def _case(harness, binding, M, N, K, split, seed):
    g = synth.stream(81, seed)
    a = g.standard_normal((M, K), dtype=np.float32).astype(np.float16).astype(np.float32)
    w = synth.storage_round(g.standard_normal((N, K), dtype=np.float32) * 0.05, synth.DT_BF16)
    bias = g.standard_normal(N).astype(np.float32)
    return (harness.to_device_act(a, synth.DT_BF16), harness.pack_matrix(harness.to_device(w, synth.DT_BF16)),
            torch.from_numpy(bias).cuda(), a, w, bias)


def test_noalloc_projection_matches_the_workspace_entry_point_twice_in_a_row():
    from paper_2402_15678_amd import binding, harness
    st = harness.stream_ptr()
    # (rows, columns, contraction, forced split): the first fills 18.9 MB of the built-in buffer with 4 splits,
    # the second uses 0.5 MB of it right afterwards, the third lets the library choose, the fourth is one split
    # (no buffer at all)
    shapes = [(144, 8192, 8192, 4), (40, 1000, 1024, 3), (17, 5120, 5120, 0), (5, 256, 256, 1)]
    cases = [_case(harness, binding, M, N, K, s, i) for i, (M, N, K, s) in enumerate(shapes)]
    want = []
    for (M, N, K, s), (a_d, w_d, b_d, a, w, bias) in zip(shapes, cases):
        out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        ws = torch.empty((16 * M * N * 4 + 256,), dtype=torch.uint8, device="cuda:0")
        binding.mn_proj_gemm(None, a_d.data_ptr(), w_d.data_ptr(), b_d.data_ptr(), out.data_ptr(), M, N, K, s,
                             ws.data_ptr(), ws.numel(), st)
        torch.cuda.synchronize()
        # the workspace entry point itself against the plain fp64 product
        ref = a.astype(np.float64) @ w.astype(np.float64).T + bias
        assert np.abs(out.cpu().numpy() - ref).max() < 2e-3 * max(1.0, np.sqrt(K / 1024.0))
        want.append(out)
    outs = [torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0") for (M, N, K, s) in shapes]
    # set-up: the first call on a device looks the built-in buffer up (the runtime places the array then)
    (M, N, K, s), (a_d, w_d, b_d, *_) = shapes[1], cases[1]
    binding.mn_proj_gemm_noalloc(None, a_d.data_ptr(), w_d.data_ptr(), b_d.data_ptr(), outs[1].data_ptr(), M, N, K, s, st)
    torch.cuda.synchronize()
    outs[1].fill_(float("nan"))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    # back to back on one stream, no synchronisation in between: the second call reuses the buffer the first one
    # has just filled
    for (M, N, K, s), (a_d, w_d, b_d, *_), out in zip(shapes, cases, outs):
        binding.mn_proj_gemm_noalloc(None, a_d.data_ptr(), w_d.data_ptr(), b_d.data_ptr(), out.data_ptr(), M, N, K, s, st)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before                    # no device memory was taken or given back
    for out, ref in zip(outs, want):
        assert torch.equal(out, ref)
    # and once more in the opposite order (small before large)
    for out in outs:
        out.fill_(float("nan"))
    for (M, N, K, s), (a_d, w_d, b_d, *_), out in reversed(list(zip(shapes, cases, outs))):
        binding.mn_proj_gemm_noalloc(None, a_d.data_ptr(), w_d.data_ptr(), b_d.data_ptr(), out.data_ptr(), M, N, K, s, st)
    torch.cuda.synchronize()
    for out, ref in zip(outs, want):
        assert torch.equal(out, ref)


def test_noalloc_projection_rejects_what_the_buffer_cannot_hold():
    from paper_2402_15678_amd import binding, harness
    M, N, K = 144, 8192, 1024
    a_d = torch.zeros((M, K), dtype=torch.float16, device="cuda:0")
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda:0")
    need = 8 * M * N * 4
    assert need > binding.MN_NOALLOC_SCRATCH_BYTES
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_proj_gemm_noalloc(None, a_d.data_ptr(), a_d.data_ptr(), None, out.data_ptr(), M, N, K, 8,
                                     harness.stream_ptr())
    assert e.value.status == binding.MN_ECAPACITY and str(need) in str(e.value)
    with pytest.raises(binding.MinionsError) as e:
        binding.mn_proj_gemm_noalloc(None, a_d.data_ptr(), a_d.data_ptr(), None, out.data_ptr(), M, N, 100, 0,
                                     harness.stream_ptr())
    assert e.value.status == binding.MN_ESHAPE
    torch.cuda.synchronize()
