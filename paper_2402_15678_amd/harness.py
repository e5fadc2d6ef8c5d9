"""Device-side plumbing for tests and benchmarks: PyTorch tensors own the HBM buffers, the HIP
library (through ``binding``) does all the computing.  Nothing here implements any step of the
verification path: the classes hold buffers and pass their addresses on."""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B
from . import synth


def _dev() -> torch.device:
    if not torch.cuda.is_available():
        raise RuntimeError("a GPU is required: the verification path has no CPU fallback")
    return torch.device("cuda:0")


def to_device(a: np.ndarray, dtype: int) -> torch.Tensor:
    """Host values (fp32, already representable in the storage type) -> device tensor in the storage type."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == synth.DT_BF16:
        bits = synth.f32_to_bf16_bits(a).view(np.int16)
        return torch.from_numpy(bits).to(_dev()).view(torch.bfloat16)
    return torch.from_numpy(a).to(_dev())


def to_device_act(a: np.ndarray, dtype: int) -> torch.Tensor:
    """Host values -> device tensor in the activation type of the model (fp32, or fp16 in bf16 models), which is
    also the type of its KV pages."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == synth.DT_BF16:
        return torch.from_numpy(a.astype(np.float16)).to(_dev())
    return torch.from_numpy(a).to(_dev())


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def pack_matrix(w: torch.Tensor, interleave_half: int = 0, dev_status: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Row-major bf16 [N][K] on the device -> the library's packed streaming layout (a new tensor)."""
    N, K = w.shape
    nbytes = B.mn_packed_weight_bytes(N, K)
    if nbytes == 0:
        raise ValueError("cannot pack a %dx%d matrix" % (N, K))
    out = torch.empty((nbytes // 2,), dtype=torch.bfloat16, device=w.device)
    B.mn_pack_weight(w.data_ptr(), out.data_ptr(), N, K, interleave_half,
                     dev_status.data_ptr() if dev_status is not None else None, stream_ptr())
    return out


PACKED_KEYS = ("wqkv", "wo", "w1", "w2", "lm_head")


def pack_model_tensors(desc: synth.ModelDesc, t: Dict[str, object]) -> None:
    """In bf16 models replace the five projection matrices by their packed form, in place."""
    if desc.dtype != synth.DT_BF16:
        return
    half = desc.d_ffn if desc.arch == synth.ARCH_LLAMA else 0
    t["lm_head"] = pack_matrix(t["lm_head"])
    for Lw in t["layers"]:
        for k in ("wqkv", "wo", "w2"):
            Lw[k] = pack_matrix(Lw[k])
        Lw["w1"] = pack_matrix(Lw["w1"], half)
    torch.cuda.synchronize()


class DeviceModel:
    """Weights on the device + the library context."""

    def __init__(self, desc: synth.ModelDesc, tensors: Dict[str, object]):
        self.desc = desc
        self.t = tensors  # keeps the tensors alive
        L = desc.n_layers
        layers: List[Dict[str, torch.Tensor]] = tensors["layers"]
        self._arrays = {}
        w = B.Weights()
        p = lambda t: t.data_ptr() if t is not None else None
        w.tok_emb = p(tensors["tok_emb"])
        w.pos_emb = p(tensors.get("pos_emb"))
        w.final_norm_g = p(tensors["final_norm_g"])
        w.final_norm_b = p(tensors.get("final_norm_b"))
        w.lm_head = p(tensors["lm_head"])
        for key in ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"):
            arr = B.ptr_array([p(layers[l].get(key)) for l in range(L)])
            self._arrays[key] = arr
            setattr(w, key, C.cast(arr, C.POINTER(C.c_void_p)))
        self.cdesc = B.ModelDesc(desc.arch, desc.dtype, desc.n_layers, desc.d_model, desc.n_heads, desc.n_kv_heads,
                                 desc.head_dim, desc.d_ffn, desc.vocab, desc.max_pos, desc.norm_eps, desc.rope_base)
        self.ctx = B.mn_create(self.cdesc, w)

    def close(self) -> None:
        if self.ctx:
            B.mn_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @classmethod
    def from_host(cls, desc: synth.ModelDesc, W: Dict[str, object]) -> "DeviceModel":
        mats = ("tok_emb", "pos_emb", "lm_head", "wqkv", "wo", "w1", "w2")
        conv = lambda k, a: to_device(a, desc.dtype if k in mats else synth.DT_F32)
        t: Dict[str, object] = {k: conv(k, v) for k, v in W.items() if k != "layers"}
        t["layers"] = [{k: conv(k, v) for k, v in Lw.items()} for Lw in W["layers"]]
        pack_model_tensors(desc, t)
        return cls(desc, t)

    @classmethod
    def random_on_device(cls, desc: synth.ModelDesc, seed: int, std: float = 0.02) -> "DeviceModel":
        """Random-init weights generated directly in HBM (full-size models never visit the host)."""
        dev = _dev()
        gen = torch.Generator(device=dev)
        gen.manual_seed(int(seed))
        st = torch.bfloat16 if desc.dtype == synth.DT_BF16 else torch.float32

        def mat(rows, cols):
            out = torch.empty((rows, cols), dtype=st, device=dev)
            chunk = max(1, (1 << 28) // cols)  # fp32 staging of at most 1 GiB
            for r in range(0, rows, chunk):
                n = min(chunk, rows - r)
                out[r:r + n] = (torch.randn((n, cols), generator=gen, device=dev, dtype=torch.float32) * std).to(st)
            return out

        vec = lambda n, mean=0.0: torch.randn((n,), generator=gen, device=dev, dtype=torch.float32) * std + mean
        d, hd = desc.d_model, desc.head_dim
        t: Dict[str, object] = {"tok_emb": mat(desc.vocab, d), "lm_head": mat(desc.vocab, d), "final_norm_g": vec(d, 1.0)}
        opt = desc.arch == synth.ARCH_OPT
        if opt:
            t["pos_emb"] = mat(desc.max_pos, d)
            t["final_norm_b"] = vec(d)
        layers = []
        bf = desc.dtype == synth.DT_BF16
        half = desc.d_ffn if desc.arch == synth.ARCH_LLAMA else 0
        pk = (lambda w, h=0: pack_matrix(w, h)) if bf else (lambda w, h=0: w)
        t["lm_head"] = pk(t["lm_head"])
        for _ in range(desc.n_layers):
            Lw = {"wqkv": pk(mat(desc.n_qkv, d)), "wo": pk(mat(d, desc.n_heads * hd)), "w1": pk(mat(desc.w1_rows, d), half),
                  "w2": pk(mat(d, desc.d_ffn)), "ln1_g": vec(d, 1.0), "ln2_g": vec(d, 1.0)}
            if opt:
                Lw.update({"ln1_b": vec(d), "ln2_b": vec(d), "bqkv": vec(desc.n_qkv), "bo": vec(d),
                           "b1": vec(desc.d_ffn), "b2": vec(d)})
            layers.append(Lw)
        t["layers"] = layers
        return cls(desc, t)


class DeviceKV:
    """Paged KV cache on the device."""

    def __init__(self, desc: synth.ModelDesc, block_size: int, num_blocks: int, block_tables: np.ndarray,
                 ctx_lens: Sequence[int], k_pages: List[torch.Tensor], v_pages: List[torch.Tensor]):
        self.desc = desc
        self.block_size, self.num_blocks = block_size, num_blocks
        self.k_pages, self.v_pages = k_pages, v_pages
        self.block_tables = torch.from_numpy(np.ascontiguousarray(block_tables, np.int32)).to(_dev())
        self.ctx_lens = torch.tensor(np.asarray(ctx_lens, np.int32), device=_dev())
        self.max_blocks_per_seq = int(block_tables.shape[1])
        self._k = B.ptr_array([t.data_ptr() for t in k_pages])
        self._v = B.ptr_array([t.data_ptr() for t in v_pages])
        self.c = B.KV(C.cast(self._k, C.POINTER(C.c_void_p)), C.cast(self._v, C.POINTER(C.c_void_p)), block_size,
                      num_blocks, self.max_blocks_per_seq, self.block_tables.data_ptr(), self.ctx_lens.data_ptr())

    @classmethod
    def from_host(cls, desc: synth.ModelDesc, kv: synth.PagedKV) -> "DeviceKV":
        ks = [to_device_act(a, desc.dtype) for a in kv.k_pages]   # (bf16-valued draws: the same numbers in fp16)
        vs = [to_device_act(a, desc.dtype) for a in kv.v_pages]
        return cls(desc, kv.block_size, kv.num_blocks, kv.block_tables, kv.ctx_lens, ks, vs)

    @classmethod
    def random_on_device(cls, desc: synth.ModelDesc, ctx_lens: Sequence[int], spec_lens: Sequence[int], seed: int,
                         block_size: int = 16, scatter: bool = True, std: float = 1.0) -> "DeviceKV":
        bt, nb = synth.make_block_tables(ctx_lens, spec_lens, block_size, seed, scatter)
        dev = _dev()
        gen = torch.Generator(device=dev)
        gen.manual_seed(int(seed) + 77)
        # 16-bit models: draws rounded to bf16 (the values the host recipe gives), held as fp16 pages
        page = ((lambda t: t.to(torch.bfloat16).to(torch.float16)) if desc.dtype == synth.DT_BF16 else (lambda t: t))
        hk, hd = desc.n_kv_heads, desc.head_dim
        ks, vs = [], []
        for _ in range(desc.n_layers):
            ks.append(page(torch.randn((nb, hk, hd // 8, block_size, 8), generator=gen, device=dev) * std))
            vs.append(page(torch.randn((nb, hk, hd, block_size), generator=gen, device=dev) * std))
        return cls(desc, block_size, nb, bt, ctx_lens, ks, vs)

    def download(self, layer: int):
        """K and V pages of one layer as fp32 numpy arrays (layout unchanged)."""
        return (self.k_pages[layer].float().cpu().numpy(), self.v_pages[layer].float().cpu().numpy())


class VerifySession:
    """Output buffers + workspace for batches of up to B sequences / max_rows scored positions."""

    def __init__(self, model: DeviceModel, kv: DeviceKV, B_: int, k_max: int, n_drafts: int, max_ctx: int,
                 max_rows: Optional[int] = None, want_logits: bool = False):
        dev = _dev()
        self.model, self.kv = model, kv
        self.B, self.k_max, self.n, self.max_ctx = B_, k_max, n_drafts, max_ctx
        self.max_rows = max_rows if max_rows is not None else B_ * (k_max + 1)
        i32 = lambda *s: torch.full(s, -7, dtype=torch.int32, device=dev)
        self.voted = i32(B_, max(1, k_max))
        self.voted_ssm = i32(B_)
        self.greedy = i32(B_, k_max + 1)
        self.accepted_len, self.n_out, self.next_last_tok, self.blocks_in_use = i32(B_), i32(B_), i32(B_), i32(B_)
        self.out_tokens = i32(B_, k_max + 1)
        self.dev_status = torch.zeros((1,), dtype=torch.int32, device=dev)
        self.logits = (torch.empty((self.max_rows, model.desc.vocab), dtype=torch.float32, device=dev)
                       if want_logits else None)
        self.ws_bytes = B.mn_workspace_bytes(model.ctx, B_, self.max_rows, max_ctx)
        if self.ws_bytes == 0:
            raise RuntimeError("mn_workspace_bytes rejected the shape")
        self.workspace = torch.empty((self.ws_bytes,), dtype=torch.uint8, device=dev)

    def vote(self, drafts: torch.Tensor, spec_len: torch.Tensor, ssm_w: torch.Tensor, mode: int = 0) -> None:
        B.mn_mv_vote(self.model.ctx, drafts.data_ptr(), spec_len.data_ptr(), ssm_w.data_ptr(), self.B, self.n,
                     self.k_max, mode, self.voted.data_ptr(), self.voted_ssm.data_ptr(), self.dev_status.data_ptr(),
                     stream_ptr())

    def forward(self, last_tok: torch.Tensor, spec_len: torch.Tensor, h_spec_len: Sequence[int],
                voted: Optional[torch.Tensor] = None) -> None:
        v = self.voted if voted is None else voted
        B.mn_verify_forward(self.model.ctx, last_tok.data_ptr(), v.data_ptr(), spec_len.data_ptr(),
                            B.host_i32(h_spec_len), self.B, self.k_max, self.max_ctx, self.kv.c,
                            self.greedy.data_ptr(), self.logits.data_ptr() if self.logits is not None else None,
                            self.workspace.data_ptr(), self.ws_bytes, self.dev_status.data_ptr(), stream_ptr())

    def sample(self, spec_len: torch.Tensor, M: int, draft_probs: torch.Tensor, temperature: float, seed: int,
               step: int, voted: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Stochastic verification on the logits of the last forward: fills and returns `sampled`, which
        accept(..., tokens=sampled) takes in place of the greedy tokens."""
        assert self.logits is not None, "the session was built without a logits buffer"
        v = self.voted if voted is None else voted
        if not hasattr(self, "sampled"):
            self.sampled = torch.full_like(self.greedy, -7)
        B.mn_verify_sample(self.model.ctx, self.logits.data_ptr(), v.data_ptr(), draft_probs.data_ptr(),
                           spec_len.data_ptr(), self.greedy.data_ptr(), self.B, self.k_max, M, self.model.desc.vocab,
                           temperature, seed, step, self.sampled.data_ptr(), self.dev_status.data_ptr(), stream_ptr())
        return self.sampled

    def accept(self, spec_len: torch.Tensor, voted: Optional[torch.Tensor] = None,
               tokens: Optional[torch.Tensor] = None) -> None:
        v = self.voted if voted is None else voted
        g = self.greedy if tokens is None else tokens
        B.mn_accept_and_commit(self.model.ctx, v.data_ptr(), g.data_ptr(), spec_len.data_ptr(), self.B,
                               self.k_max, self.kv.c, self.accepted_len.data_ptr(), self.out_tokens.data_ptr(),
                               self.n_out.data_ptr(), self.next_last_tok.data_ptr(), self.blocks_in_use.data_ptr(),
                               self.dev_status.data_ptr(), stream_ptr())

    def acr_update(self, spec_len: torch.Tensor, ssm_w: torch.Tensor, reward_threshold: float, punish_threshold: float,
                   reward_factor: float, punish_factor: float, acr: Optional[torch.Tensor] = None) -> None:
        """Speculation quality metric + SSM weight update on this step's outcome (ssm_w changes in place)."""
        B.mn_acr_update(self.model.ctx, self.voted_ssm.data_ptr(), self.accepted_len.data_ptr(), spec_len.data_ptr(),
                        self.n_out.data_ptr(), self.B, self.n, reward_threshold, punish_threshold, reward_factor,
                        punish_factor, ssm_w.data_ptr(), acr.data_ptr() if acr is not None else None, stream_ptr())

    def step(self, last_tok, drafts, spec_len, h_spec_len, ssm_w, mode: int = 0) -> None:
        """vote -> verify forward -> accept + commit, back to back on the current stream."""
        self.vote(drafts, spec_len, ssm_w, mode)
        self.forward(last_tok, spec_len, h_spec_len)
        self.accept(spec_len)


class DraftSession:
    """The step before the verification path (paper section 3.1: several SSMs speculate on one request):
    every SSM is a small decoder of its own (own weights, own paged KV cache) driven through the same
    library calls as the LLM, one token per call, each SSM on a stream of its own; its greedy tokens fill
    drafts[b][j][t] on the device, which mn_mv_vote reads directly.  Copying a token column into the drafts
    array is the only thing done outside the library."""

    def __init__(self, models: Sequence[DeviceModel], kvs: Sequence[DeviceKV], B_: int, k_max: int, max_ctx: int,
                 sampling: bool = False):
        assert len(models) == len(kvs) and len(models) >= 1
        self.n, self.B, self.k_max = len(models), B_, k_max
        self.sessions = [VerifySession(m, kv, B_, 0, 1, max_ctx, max_rows=B_, want_logits=sampling)
                         for m, kv in zip(models, kvs)]
        dev = _dev()
        self.vocab = models[0].desc.vocab
        # q of every drafted token, per SSM: [n][B][k_max][vocab] fp32 (only when the SSMs sample)
        self.draft_probs = (torch.zeros((self.n, B_, max(1, k_max), self.vocab), dtype=torch.float32, device=dev)
                            if sampling else None)
        self.drafts = torch.full((B_, self.n, max(1, k_max)), -1, dtype=torch.int32, device=dev)
        self._zeros = torch.zeros((B_,), dtype=torch.int32, device=dev)
        self._dummy = torch.zeros((B_, 1), dtype=torch.int32, device=dev)

    def _fork(self):
        """One stream per SSM (default priority), each starting after the work already queued on the current one."""
        if not hasattr(self, "_streams"):
            self._streams = [torch.cuda.Stream() for _ in range(self.n)]
        main = torch.cuda.current_stream()
        for st in self._streams:
            st.wait_stream(main)
        return main, self._streams

    def draft(self, last_tok: torch.Tensor, k: int, concurrent: bool = True) -> torch.Tensor:
        """k greedy tokens per sequence from every SSM, starting from the pending token; each SSM's cache
        advances by k entries (the caller truncates it to the accepted prefix after the verification).
        The SSMs do not depend on one another: with `concurrent` each runs on a stream of its own (their small
        kernels are bound by launch latency, not by the GPU, so side by side they take about the time of one)."""
        assert 0 <= k <= self.k_max
        self.drafts.fill_(-1)
        zeros = [0] * self.B
        if not concurrent or self.n == 1:
            for j, ses in enumerate(self.sessions):
                cur = last_tok
                for t in range(k):
                    ses.forward(cur, self._zeros, zeros, voted=self._dummy)
                    ses.accept(self._zeros, voted=self._dummy)
                    cur = ses.next_last_tok.clone()
                    self.drafts[:, j, t] = cur
            return self.drafts
        main, streams = self._fork()
        cur = [last_tok] * self.n
        for t in range(k):                       # token by token across the SSMs: every queue stays fed
            for j, ses in enumerate(self.sessions):
                with torch.cuda.stream(streams[j]):
                    ses.forward(cur[j], self._zeros, zeros, voted=self._dummy)
                    ses.accept(self._zeros, voted=self._dummy)
                    cur[j] = ses.next_last_tok.clone()
                    self.drafts[:, j, t] = cur[j]
        for st in streams:
            main.wait_stream(st)
        return self.drafts

    def draft_sampled(self, last_tok: torch.Tensor, k: int, temperature: float, seed: int, step: int) -> torch.Tensor:
        """k tokens per sequence from every SSM, each drawn from the SSM's own q = softmax(scores / T)
        (mn_draft_sample writes the token straight into drafts[b][j][t] and q into draft_probs[j][b][t]);
        the SSM's cache advances as in draft()."""
        assert self.draft_probs is not None, "the session was built without sampling"
        assert 0 <= k <= self.k_max
        self.drafts.fill_(-1)
        zeros = [0] * self.B
        kk = max(1, self.k_max)
        main, streams = self._fork()
        cur = [last_tok] * self.n
        for t in range(k):
            for j, ses in enumerate(self.sessions):
                with torch.cuda.stream(streams[j]):
                    ses.forward(cur[j], self._zeros, zeros, voted=self._dummy)
                    ses.accept(self._zeros, voted=self._dummy)        # the cache keeps the token just scored
                    B.mn_draft_sample(ses.model.ctx, ses.logits.data_ptr(), self.B, self.vocab, temperature, seed, step,
                                      j, t, self.drafts[0, j, t:].data_ptr(), self.n * kk,
                                      self.draft_probs[j, 0, t].data_ptr(), kk * self.vocab, stream_ptr())
                    cur[j] = self.drafts[:, j, t].contiguous()
        for st in streams:
            main.wait_stream(st)
        return self.drafts

    def voted_probs(self, voted_ssm: torch.Tensor) -> torch.Tensor:
        """q of the SSM whose draft won the vote, per sequence: [B][k_max][vocab] (a gather, no arithmetic)."""
        idx = voted_ssm.long().clamp_(min=0)
        return self.draft_probs[idx, torch.arange(self.B, device=idx.device)].contiguous()
