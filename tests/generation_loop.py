"""Test driver for several rounds of the whole method on one GPU (drafting, vote, verification, commit, weight
update, and bringing every SSM's cache back in line with what was committed).  The index bookkeeping between the
rounds (prefix lengths, gathers of token ids) is torch integer arithmetic and lives here, with the tests, not in
the package: the package holds the library and the marshalling of its arguments only."""
from __future__ import annotations

from typing import Sequence

import torch

from paper_2402_15678_amd.harness import DeviceKV, DeviceModel, VerifySession, _dev


class GenerationLoop:
    """Round after round of the whole method on one GPU (paper sections 3.1-3.3): every SSM drafts k tokens,
    the drafts are voted on, the LLM verifies the winner, the accepted tokens are committed, the SSM weights
    follow the acceptance rates, and every SSM's cache is brought back in line with what was committed.

    Bringing an SSM back in line: after drafting, SSM j's cache holds the pending token and its own first
    k - 1 draft tokens.  Of those, the entries up to the first disagreement with the committed tokens stay
    valid; the cache is cut there (its ctx_lens is set) and the committed tokens it has not seen, followed by
    the new pending token, become the rows of its first forward of the next round, whose last row yields
    the first token of the next draft.  That forward is an ordinary multi-row call of the same library.

    Everything runs on the device through the C ABI; index bookkeeping (prefix lengths, gathers of token ids)
    is torch integer arithmetic here, and the host reads back one small array per round: the numbers of rows
    of the next first forwards, which size the launches."""

    def __init__(self, llm: DeviceModel, llm_kv: DeviceKV, ssms: Sequence[DeviceModel], ssm_kvs: Sequence[DeviceKV],
                 B_: int, k: int, max_ctx: int, last_tok: torch.Tensor, ssm_w: torch.Tensor):
        assert k >= 1 and len(ssms) == len(ssm_kvs) >= 1
        dev = _dev()
        self.B, self.k, self.n = B_, k, len(ssms)
        self.llm = VerifySession(llm, llm_kv, B_, k, self.n, max_ctx)
        self.first = [VerifySession(m, kv, B_, k, 1, max_ctx) for m, kv in zip(ssms, ssm_kvs)]      # ragged rows
        self.single = [VerifySession(m, kv, B_, 0, 1, max_ctx, max_rows=B_) for m, kv in zip(ssms, ssm_kvs)]
        self.ssm_kvs = list(ssm_kvs)
        self.ssm_w = ssm_w
        self.last = last_tok.clone()                                            # the LLM's pending token
        self.ssm_last = [last_tok.clone() for _ in ssms]                        # first token an SSM has not seen
        self.ssm_extra = [torch.zeros((B_, k), dtype=torch.int32, device=dev) for _ in ssms]   # the ones after it
        self.ssm_nextra = [torch.zeros((B_,), dtype=torch.int32, device=dev) for _ in ssms]
        self.h_nextra = [[0] * B_ for _ in ssms]
        self.drafts = torch.full((B_, self.n, k), -1, dtype=torch.int32, device=dev)
        self.spec = torch.full((B_,), k, dtype=torch.int32, device=dev)
        self._zeros = torch.zeros((B_,), dtype=torch.int32, device=dev)
        self._dummy = torch.zeros((B_, 1), dtype=torch.int32, device=dev)
        self._ar = torch.arange(B_, device=dev)
        self._cols = torch.arange(k, device=dev, dtype=torch.int64)

    def draft(self) -> torch.Tensor:
        """k greedy tokens from every SSM; the first forward also feeds the committed tokens the SSM missed."""
        k = self.k
        if not hasattr(self, "_streams"):
            self._streams = [torch.cuda.Stream() for _ in range(self.n)]      # one per SSM: they are independent
        main = torch.cuda.current_stream()
        for st in self._streams:
            st.wait_stream(main)
        cur = [None] * self.n
        for t in range(k):
            for j in range(self.n):
                f, s = self.first[j], self.single[j]
                with torch.cuda.stream(self._streams[j]):
                    if t == 0:
                        commit = torch.cat([self.ssm_extra[j], self._zeros[:, None]], dim=1).contiguous()
                        f.forward(self.ssm_last[j], self.ssm_nextra[j], self.h_nextra[j], voted=self.ssm_extra[j])
                        f.accept(self.ssm_nextra[j], voted=self.ssm_extra[j], tokens=commit)   # every fed row is kept
                        cur[j] = f.greedy[self._ar, self.ssm_nextra[j].long()].contiguous()    # output of the last row
                    else:
                        s.forward(cur[j], self._zeros, [0] * self.B, voted=self._dummy)
                        s.accept(self._zeros, voted=self._dummy)
                        cur[j] = s.next_last_tok.clone()
                    self.drafts[:, j, t] = cur[j]
        for st in self._streams:
            main.wait_stream(st)
        return self.drafts

    def round(self, acr_args=None):
        """One round; returns (emitted tokens per sequence, accepted lengths) on the host."""
        k = self.k
        self.draft()
        L = self.llm
        L.vote(self.drafts, self.spec, self.ssm_w, 0)
        L.forward(self.last, self.spec, [k] * self.B)
        L.accept(self.spec)
        if acr_args is not None:
            L.acr_update(self.spec, self.ssm_w, *acr_args)
        a = L.accepted_len.long()                                                 # [B]
        out = L.out_tokens.long()                                                 # [B][k+1], padded with -1
        ctx0 = L.kv.ctx_lens.long() - (a + 1)                                     # committed context before the round
        for j in range(self.n):
            same = (self.drafts[:, j, :].long() == L.voted.long()[:, :k]).long()
            c = torch.cumprod(same, dim=1).sum(dim=1)                             # tokens before the first disagreement
            m = torch.minimum(torch.minimum(c, a), torch.full_like(a, k - 1))     # valid draft entries of the cache
            self.ssm_kvs[j].ctx_lens.copy_((ctx0 + 1 + m).to(torch.int32))
            self.ssm_last[j] = out[self._ar, m].to(torch.int32).contiguous()
            idx = (m[:, None] + 1 + self._cols[None, :]).clamp_(max=k)
            extra = torch.gather(out, 1, idx)
            n_extra = a - m
            extra = torch.where(self._cols[None, :] < n_extra[:, None], extra, torch.zeros_like(extra))
            self.ssm_extra[j] = extra.to(torch.int32).contiguous()
            self.ssm_nextra[j] = n_extra.to(torch.int32).contiguous()
        self.last = L.next_last_tok.clone()
        nx = torch.stack(self.ssm_nextra).cpu()                                   # the round's one read-back
        self.h_nextra = [[int(v) for v in row] for row in nx]
        n_out = L.n_out.cpu().tolist()
        toks = L.out_tokens.cpu().tolist()
        return [toks[b][:n_out[b]] for b in range(self.B)], L.accepted_len.cpu().tolist()
