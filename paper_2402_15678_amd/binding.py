"""ctypes binding of libminions_verify.so: same names as the C ABI, argument marshalling only.

Pointers are passed as integers (e.g. ``tensor.data_ptr()``); nothing here computes anything.
Importing this module fails loudly if the library has not been built
(``python -m paper_2402_15678_amd.build``): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libminions_verify.so")

MN_OK, MN_EINVAL, MN_ENULL, MN_ESHAPE, MN_EUNSUPPORTED, MN_ECAPACITY, MN_EWORKSPACE, MN_EHIP = 0, -1, -2, -3, -4, -5, -6, -7
MN_ARCH_OPT, MN_ARCH_LLAMA = 0, 1
MN_DT_F32, MN_DT_BF16 = 0, 1
MN_VOTE_TREE, MN_VOTE_COLUMN = 0, 1
MN_DEV_BLOCK_TABLE, MN_DEV_SPEC_LEN, MN_DEV_TOKEN, MN_DEV_DRAFTS, MN_DEV_RANGE, MN_DEV_CTX = 1, 2, 4, 8, 16, 32
MN_MAX_DRAFTS, MN_MAX_BATCH, MN_MAX_SPLIT_K = 64, 4096, 16
MN_NOALLOC_SCRATCH_BYTES = 32 << 20


EXPORTS = ("mn_create", "mn_destroy", "mn_last_error", "mn_status_str", "mn_workspace_bytes", "mn_mv_vote",
           "mn_verify_forward", "mn_accept_and_commit", "mn_proj_gemm", "mn_proj_gemm_noalloc", "mn_attention", "mn_profile_enable",
           "mn_profile_collect", "mn_packed_weight_bytes", "mn_pack_weight", "mn_acr_update",
           "mn_verify_sample", "mn_draft_sample",
           "mn_selector_create", "mn_selector_destroy", "mn_selector_observe", "mn_selector_current",
           "mn_selector_adjustments", "mn_probe_stream_read", "mn_probe_mfma", "mn_probe_mfma_data")
PROF_KINDS = ("prepare", "norm", "gemm", "rope_append", "attention", "act", "argmax", "vote", "accept")


class ModelDesc(C.Structure):
    _fields_ = [("arch", C.c_int), ("dtype", C.c_int), ("n_layers", C.c_int), ("d_model", C.c_int),
                ("n_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int), ("d_ffn", C.c_int),
                ("vocab", C.c_int), ("max_pos", C.c_int), ("norm_eps", C.c_float), ("rope_base", C.c_float)]


_PP = C.POINTER(C.c_void_p)


class Weights(C.Structure):
    _fields_ = [("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p), ("final_norm_g", C.c_void_p),
                ("final_norm_b", C.c_void_p), ("lm_head", C.c_void_p),
                ("ln1_g", _PP), ("ln1_b", _PP), ("wqkv", _PP), ("bqkv", _PP), ("wo", _PP), ("bo", _PP),
                ("ln2_g", _PP), ("ln2_b", _PP), ("w1", _PP), ("b1", _PP), ("w2", _PP), ("b2", _PP)]


class KV(C.Structure):
    _fields_ = [("k_layers", _PP), ("v_layers", _PP), ("block_size", C.c_int), ("num_blocks", C.c_int),
                ("max_blocks_per_seq", C.c_int), ("block_tables", C.c_void_p), ("ctx_lens", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2402_15678_amd.build` "
                          "(there is no CPU fallback)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.mn_create.restype = i32
    lib.mn_create.argtypes = [C.POINTER(vp), C.POINTER(ModelDesc), C.POINTER(Weights)]
    lib.mn_destroy.restype = None
    lib.mn_destroy.argtypes = [vp]
    lib.mn_last_error.restype = C.c_char_p
    lib.mn_last_error.argtypes = [vp]
    lib.mn_status_str.restype = C.c_char_p
    lib.mn_status_str.argtypes = [i32]
    lib.mn_workspace_bytes.restype = sz
    lib.mn_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.mn_mv_vote.restype = i32
    lib.mn_mv_vote.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.mn_verify_forward.restype = i32
    lib.mn_verify_forward.argtypes = [vp, vp, vp, vp, C.POINTER(C.c_int32), i32, i32, i32, C.POINTER(KV), vp, vp, vp, sz, vp, vp]
    lib.mn_accept_and_commit.restype = i32
    lib.mn_accept_and_commit.argtypes = [vp, vp, vp, vp, i32, i32, C.POINTER(KV), vp, vp, vp, vp, vp, vp, vp]
    lib.mn_proj_gemm.restype = i32
    lib.mn_proj_gemm.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]
    lib.mn_proj_gemm_noalloc.restype = i32
    lib.mn_proj_gemm_noalloc.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp]
    lib.mn_attention.restype = i32
    lib.mn_attention.argtypes = [vp, vp, vp, C.POINTER(C.c_int32), i32, i32, C.POINTER(KV), i32, vp, vp, sz, vp, vp]
    lib.mn_packed_weight_bytes.restype = sz
    lib.mn_packed_weight_bytes.argtypes = [i32, i32]
    lib.mn_pack_weight.restype = i32
    lib.mn_pack_weight.argtypes = [vp, vp, i32, i32, i32, vp, vp]
    lib.mn_verify_sample.restype = i32
    lib.mn_verify_sample.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, C.c_double, C.c_uint64, C.c_uint64,
                                     vp, vp, vp]
    lib.mn_draft_sample.restype = i32
    lib.mn_draft_sample.argtypes = [vp, vp, i32, i32, C.c_double, C.c_uint64, C.c_uint64, i32, i32, vp, C.c_long, vp,
                                    C.c_long, vp]
    lib.mn_acr_update.restype = i32
    lib.mn_acr_update.argtypes = [vp, vp, vp, vp, vp, i32, i32, C.c_double, C.c_double, C.c_float, C.c_float, vp, vp, vp]
    lib.mn_selector_create.restype = i32
    lib.mn_selector_create.argtypes = [C.POINTER(vp), i32, i32, i32, i32, i32, i32]
    lib.mn_selector_destroy.restype = None
    lib.mn_selector_destroy.argtypes = [vp]
    lib.mn_selector_observe.restype = i32
    lib.mn_selector_observe.argtypes = [vp, C.c_double, C.c_double, C.POINTER(C.c_int), C.POINTER(C.c_double)]
    lib.mn_selector_current.restype = i32
    lib.mn_selector_current.argtypes = [vp]
    lib.mn_selector_adjustments.restype = C.c_long
    lib.mn_selector_adjustments.argtypes = [vp]
    lib.mn_probe_stream_read.restype = i32
    lib.mn_probe_stream_read.argtypes = [vp, sz, vp]
    lib.mn_probe_mfma.restype = i32
    lib.mn_probe_mfma.argtypes = [i32, C.POINTER(C.c_double), vp]
    lib.mn_probe_mfma_data.restype = i32
    lib.mn_probe_mfma_data.argtypes = [i32, C.POINTER(C.c_double), vp]
    lib.mn_profile_enable.restype = i32
    lib.mn_profile_enable.argtypes = [vp, i32]
    lib.mn_profile_collect.restype = i32
    lib.mn_profile_collect.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    return lib


lib = _load()


class MinionsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s: %s" % (lib.mn_status_str(status).decode(), message))
        self.status = status


def _check(status: int, ctx) -> None:
    if status != MN_OK:
        raise MinionsError(status, (lib.mn_last_error(ctx) or b"").decode())


def ptr_array(ptrs: Sequence[Optional[int]]):
    """Host array of device pointers (None -> NULL)."""
    arr = (C.c_void_p * max(1, len(ptrs)))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


def host_i32(values: Sequence[int]):
    return (C.c_int32 * max(1, len(values)))(*[int(v) for v in values])


def mn_create(desc: ModelDesc, weights: Weights) -> int:
    out = C.c_void_p()
    st = lib.mn_create(C.byref(out), C.byref(desc), C.byref(weights))
    _check(st, None)
    return out.value




def mn_destroy(ctx: Optional[int]) -> None:
    if ctx:
        lib.mn_destroy(ctx)


def mn_workspace_bytes(ctx: int, B: int, max_rows: int, max_ctx: int) -> int:
    return int(lib.mn_workspace_bytes(ctx, B, max_rows, max_ctx))


def mn_mv_vote(ctx, drafts, spec_len, ssm_w, B, n, k_max, mode, voted, voted_ssm, dev_status=None, stream=None) -> None:
    _check(lib.mn_mv_vote(ctx, drafts, spec_len, ssm_w, B, n, k_max, mode, voted, voted_ssm, dev_status, stream), ctx)


def mn_verify_forward(ctx, last_tok, voted, spec_len, h_spec_len, B, k_max, max_ctx, kv: KV, greedy, logits,
                      workspace, workspace_bytes, dev_status=None, stream=None) -> None:
    _check(lib.mn_verify_forward(ctx, last_tok, voted, spec_len, h_spec_len, B, k_max, max_ctx, C.byref(kv), greedy,
                                 logits, workspace, workspace_bytes, dev_status, stream), ctx)


def mn_accept_and_commit(ctx, voted, greedy, spec_len, B, k_max, kv: KV, accepted_len, out_tokens, n_out,
                         next_last_tok, blocks_in_use, dev_status=None, stream=None) -> None:
    _check(lib.mn_accept_and_commit(ctx, voted, greedy, spec_len, B, k_max, C.byref(kv), accepted_len, out_tokens,
                                    n_out, next_last_tok, blocks_in_use, dev_status, stream), ctx)


def mn_proj_gemm(ctx, a, w, bias, out, M, N, K, split_k=0, workspace=None, workspace_bytes=0, stream=None) -> None:
    _check(lib.mn_proj_gemm(ctx, a, w, bias, out, M, N, K, split_k, workspace, workspace_bytes, stream), ctx)


def mn_proj_gemm_noalloc(ctx, a, w, bias, out, M, N, K, split_k=0, stream=None) -> None:
    _check(lib.mn_proj_gemm_noalloc(ctx, a, w, bias, out, M, N, K, split_k, stream), ctx)


def mn_attention(ctx, q, spec_len, h_spec_len, B, max_ctx, kv: KV, layer, out, workspace, workspace_bytes,
                 dev_status=None, stream=None) -> None:
    _check(lib.mn_attention(ctx, q, spec_len, h_spec_len, B, max_ctx, C.byref(kv), layer, out, workspace,
                            workspace_bytes, dev_status, stream), ctx)


def mn_profile_enable(ctx, on: bool) -> None:
    _check(lib.mn_profile_enable(ctx, 1 if on else 0), ctx)


def mn_profile_collect(ctx):
    """{family: (summed ms, launches)} since the last collect; synchronise the stream first."""
    ms = (C.c_double * len(PROF_KINDS))()
    cnt = (C.c_int * len(PROF_KINDS))()
    _check(lib.mn_profile_collect(ctx, ms, cnt), ctx)
    return {k: (ms[i], cnt[i]) for i, k in enumerate(PROF_KINDS)}


def mn_packed_weight_bytes(N: int, K: int) -> int:
    return int(lib.mn_packed_weight_bytes(N, K))


def mn_pack_weight(src, dst, N, K, interleave_half=0, dev_status=None, stream=None) -> None:
    _check(lib.mn_pack_weight(src, dst, N, K, interleave_half, dev_status, stream), None)


def mn_verify_sample(ctx, logits, voted, draft_probs, spec_len, greedy, B, k_max, M, vocab, temperature, seed, step,
                     sampled, dev_status=None, stream=None) -> None:
    _check(lib.mn_verify_sample(ctx, logits, voted, draft_probs, spec_len, greedy, B, k_max, M, vocab, temperature,
                                seed, step, sampled, dev_status, stream), ctx)


def mn_draft_sample(ctx, logits, B, vocab, temperature, seed, step, ssm, t, tokens, token_stride, probs=None,
                    probs_stride=0, stream=None) -> None:
    _check(lib.mn_draft_sample(ctx, logits, B, vocab, temperature, seed, step, ssm, t, tokens, token_stride, probs,
                               probs_stride, stream), ctx)


def mn_acr_update(ctx, voted_ssm, accepted_len, spec_len, n_out, B, n, reward_threshold, punish_threshold,
                  reward_factor, punish_factor, ssm_w, acr=None, stream=None) -> None:
    _check(lib.mn_acr_update(ctx, voted_ssm, accepted_len, spec_len, n_out, B, n, reward_threshold, punish_threshold,
                             reward_factor, punish_factor, ssm_w, acr, stream), ctx)


def mn_selector_create(s_init: int, s_min: int, s_max: int, decision_threshold: int, s_penalty: int,
                       s_reward: int) -> int:
    out = C.c_void_p()
    _check(lib.mn_selector_create(C.byref(out), s_init, s_min, s_max, decision_threshold, s_penalty, s_reward), None)
    return out.value


def mn_selector_destroy(sel: Optional[int]) -> None:
    if sel:
        lib.mn_selector_destroy(sel)


def mn_selector_observe(sel: int, t_llm: float, vl: float):
    """Returns (speculation length to use next, fitted slope or NaN when no decision was taken)."""
    s, slope = C.c_int(), C.c_double()
    _check(lib.mn_selector_observe(sel, t_llm, vl, C.byref(s), C.byref(slope)), None)
    return s.value, slope.value


def mn_selector_current(sel: int) -> int:
    return int(lib.mn_selector_current(sel))


def mn_selector_adjustments(sel: int) -> int:
    return int(lib.mn_selector_adjustments(sel))


def mn_probe_stream_read(buf, nbytes: int, stream=None) -> None:
    _check(lib.mn_probe_stream_read(buf, nbytes, stream), None)


def mn_probe_mfma(iters: int, stream=None) -> float:
    """Launches the MFMA loop; returns the floating-point operations of the launch."""
    flop = C.c_double()
    _check(lib.mn_probe_mfma(iters, C.byref(flop), stream), None)
    return flop.value


def mn_probe_mfma_data(iters: int, stream=None) -> float:
    """The MFMA loop on operands of random sign and mantissa; returns the floating-point operations of the launch."""
    flop = C.c_double()
    _check(lib.mn_probe_mfma_data(iters, C.byref(flop), stream), None)
    return flop.value
