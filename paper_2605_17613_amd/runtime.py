"""The paper's execution loop (section 5.2) for the requests of one attention layer on one GPU.

Control only: every decision comes from the library's admission control (vc_sched_*, Algorithm 1
and the reserve rings of section 5.1) and every step of the data path is a library call -
vc_swap_in when a request's reload span starts, one batched vc_draft_attn per iteration,
vc_swap_wait + vc_verify_attn + vc_accept_len when a request's verify window is the current one,
then Admit again.  Nothing here computes attention or touches KV contents.

A request drafts one token per iteration; the tokens drafted since its last verify are its verify
window (at most 64 at a GQA ratio of 4, so the horizon W must not exceed 64).  Iterations are not
paced by a clock: when a reload has not landed by its verify window the compute stream waits for
the ticket, so a link-bound schedule throttles itself to the link - the max() of Eq. 3.
"""
from __future__ import annotations

import torch

from . import binding as B


class StaggeredLayer:
    def __init__(self, ctx: B.Context, lay, bits: int, host_k, host_v, *, windows: int, x: int, t_iter: float,
                 link_bw: float, hbm_bytes: float, model_bytes: float = 0.0, chunk_tokens: int = 8192):
        """lay: a layer description (the fields of the test harness's Layer record) with R sequences, block records of `bits` for every sequence, windows of
        at least `windows` rows and planted logits; host_k / host_v: pinned copies of lay.k_full /
        lay.v_full (the requests' full KV in CPU memory)."""
        if windows > min(lay.win):
            raise ValueError("the horizon must not exceed the shortest window of the layer")
        self.ctx, self.lay, self.bits, self.x = ctx, lay, bits, int(x)
        self.R = len(lay.ctx_len)
        self.dev = lay.k_full.device
        self.host_k, self.host_v = host_k, host_v
        self.stage_k = torch.empty_like(lay.k_full)      # destination of the reloads (the "in-flight KV")
        self.stage_v = torch.empty_like(lay.v_full)
        hkv = lay.n_kv_heads
        self.row_bytes = hkv * 128 * 2
        self.kv_bytes = [2.0 * n * self.row_bytes for n in lay.ctx_len]
        comp_bytes = float(lay.blocks[bits].numel())
        self.sched = B.Sched(windows, t_iter, link_bw, hbm_bytes, model_bytes, comp_bytes, capacity=max(self.R, 1))
        self.chunk_tokens = chunk_tokens
        cu = lay.cu_ctx.tolist()
        self.c0 = cu[:-1]
        self.w0 = lay.cu_win.tolist()[:-1]
        self.r0 = lay.cu_rows.tolist()[:-1]
        # per-request single-sequence prefix arrays, and [0, cnt] for every possible window length
        self.cu_ctx1 = [torch.tensor([0, n], dtype=torch.int32, device=self.dev) for n in lay.ctx_len]
        self.cu_cnt = [torch.tensor([0, c], dtype=torch.int32, device=self.dev) for c in range(windows + 1)]
        self.max_win = windows
        self.out = torch.empty_like(lay.q)
        self.vout = torch.zeros_like(lay.q_win)
        dkw = dict(blocks=lay.blocks[bits], cu_blk=lay.cu_blk[bits], max_blk=lay.max_blk[bits], bits=bits,
                   sum_blk=int(lay.cu_blk[bits][-1]))
        self.dkw = dkw
        need = B.vc_draft_workspace_bytes(lay.n_q_heads, hkv, self.R, **dkw)
        for r in range(self.R):
            need = max(need, B.vc_verify_workspace_bytes(lay.n_q_heads, hkv, 1, total_win=windows, **self._vargs(r)))
        self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        rows, vocab = lay.logits.shape
        self.aws = torch.empty(B.vc_accept_workspace_bytes(windows, vocab), dtype=torch.uint8, device=self.dev)
        self.acc = torch.full((self.R,), -1, dtype=torch.int32, device=self.dev)
        self.nxt = torch.full((self.R,), -1, dtype=torch.int32, device=self.dev)
        self.amax = torch.empty(windows, dtype=torch.int32, device=self.dev)
        self.drafted = [0] * self.R
        self.waiting = list(range(self.R))
        self.last_ticket = [None] * self.R
        self.verified = [None] * self.R     # mark behind each request's last verify
        self.log = []            # (iteration, request, window length) of every verify
        self.kicks = 0
        self.bytes_moved = 0.0

    def _vargs(self, r):
        lay = self.lay
        n = lay.ctx_len[r]
        lo = self.c0[r]
        return dict(k=self.stage_k[lo:lo + n], v=self.stage_v[lo:lo + n], cu_ctx=self.cu_ctx1[r], max_ctx=n,
                    max_win=self.max_win, sum_ctx=n)

    def _kick(self, r):
        """Start the reload of request r: chunks of K then V rows on the library's copy stream."""
        if self.verified[r] is not None:
            # its previous verify must no longer read the staging rows: the copy stream waits, on the device,
            # for the mark recorded right behind that verify (the host does not block)
            B.vc_swap_after(self.ctx, self.verified[r])
        lo, n = self.c0[r], self.lay.ctx_len[r]
        chunks = []
        for t in range(0, n, self.chunk_tokens):
            m = min(self.chunk_tokens, n - t)
            chunks.append(((lo + t) * self.row_bytes, (lo + t) * self.row_bytes, m * self.row_bytes))
        first_k = B.vc_swap_in(self.ctx, self.host_k, self.stage_k, chunks)
        first_v = B.vc_swap_in(self.ctx, self.host_v, self.stage_v, chunks)
        self.last_ticket[r] = first_v + len(chunks) - 1
        assert first_k < first_v
        self.kicks += 1
        self.bytes_moved += self.kv_bytes[r]

    def _verify(self, it, r):
        lay, cnt = self.lay, self.drafted[r]
        if cnt == 0:
            return
        cnt = min(cnt, self.max_win)
        B.vc_swap_wait(self.ctx, self.last_ticket[r])
        w0, r0 = self.w0[r], self.r0[r]
        B.vc_verify_attn(self.ctx, lay.q_win[w0:w0 + cnt], lay.k_win[w0:w0 + cnt], lay.v_win[w0:w0 + cnt],
                         self.cu_cnt[cnt], lay.scale, self.vout[w0:w0 + cnt], n_seqs=1, workspace=self.ws,
                         **self._vargs(r))
        B.vc_accept_len(self.ctx, lay.logits[r0:r0 + cnt], self.cu_cnt[cnt], lay.draft_ids[w0:w0 + cnt],
                        self.cu_cnt[cnt], self.acc[r:r + 1], self.nxt[r:r + 1], self.amax, workspace=self.aws)
        self.verified[r] = B.vc_mark(self.ctx)
        self.log.append((it, r, cnt))
        self.drafted[r] = 0

    def run(self, iterations: int):
        lay = self.lay
        for it in range(iterations):
            still = []
            for r in self.waiting:                                     # Admit (Algorithm 1)
                if self.sched.admit(r, self.kv_bytes[r], self.x) < 0:
                    still.append(r)
            self.waiting = still
            kick, ver = self.sched.step()                              # section 5.2, steps (i) - (iii)
            for r in kick:
                self._kick(r)
            B.vc_draft_attn(self.ctx, lay.q, lay.scale, self.out, n_kv_heads=lay.n_kv_heads, workspace=self.ws,
                            **self.dkw)
            for r in range(self.R):
                self.drafted[r] += 1
            for r in ver:
                self._verify(it, r)
                self.waiting.append(r)
        return self.log
