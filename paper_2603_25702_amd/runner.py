"""Device-side session around the C ABI: buffers, prefix prefill through the library, step loop.

Host logic only (allocation, state set-up, call order).  All arithmetic happens in libs2d2.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import dataclasses

from .binding import AcceptOut, BlockState, DraftOut, Engine, KvCache, Params, RouteOut, RouteParams, VerifyOut

PREFILL_BLOCK = 64  # window used to push prompt tokens through the causal rows of the verifier


class Session:
    def __init__(self, cfg, weights: Dict[str, torch.Tensor], N: int, B: int, max_seq: int, page_size: int = 16,
                 device: str = "cuda:0", page_table: Optional[np.ndarray] = None, max_block: Optional[int] = None,
                 act_planes: int = 0):
        self.cfg, self.N, self.B = cfg, N, B
        self.dev = torch.device(device)
        self.eng = Engine(cfg, weights, N, max_block or max(B, PREFILL_BLOCK), device, act_planes=act_planes)
        i32 = torch.int32
        max_pages = (max_seq + page_size - 1) // page_size
        if page_table is None:
            page_table = np.arange(N * max_pages, dtype=np.int32).reshape(N, max_pages)
        n_pages = int(page_table.max()) + 1
        shape = (cfg.n_layers, n_pages, cfg.n_kv_heads, page_size, cfg.head_dim)
        vshape = (cfg.n_layers, n_pages, cfg.n_kv_heads, cfg.head_dim, page_size)  # V is cached key-minor
        self.kv = KvCache(torch.zeros(shape, dtype=cfg.torch_dtype, device=self.dev),
                          torch.zeros(vshape, dtype=cfg.torch_dtype, device=self.dev),
                          torch.as_tensor(page_table, dtype=i32, device=self.dev),
                          torch.zeros(N, dtype=i32, device=self.dev), torch.zeros(N, dtype=i32, device=self.dev))
        mb = self.eng.max_block
        self._blk = torch.full((N, mb), cfg.mask_id, dtype=i32, device=self.dev)
        self._car = torch.zeros((N, mb), dtype=i32, device=self.dev)
        self.pos0 = torch.zeros(N, dtype=i32, device=self.dev)
        self.d = self.eng.alloc_draft_out(N, B)
        self.v = self.eng.alloc_verify_out(N, B)
        self.a = self.eng.alloc_accept_out(N, B)
        self.step_dev = torch.zeros(1, dtype=i32, device=self.dev)
        self.st = self._state(B)

    def _state(self, B: int) -> BlockState:
        # [N, B] views over the front of flat storage, so any B <= max_block is contiguous
        n = self.N * B
        return BlockState(self._blk.view(-1)[:n].view(self.N, B), self.pos0, self._car.view(-1)[:n].view(self.N, B))

    def prefill(self, ids: Sequence[np.ndarray]):
        """Fills the cache with the causal K/V of the prompts by pushing them through the verifier's
        causal rows (committed tokens left of a [MASK]) and appending with n_accept = 0."""
        N, mb, mask = self.N, self.eng.max_block, self.cfg.mask_id
        lens = [len(x) for x in ids]
        done = [0] * N
        zeros = torch.zeros(N, dtype=torch.int32, device=self.dev)
        prm = Params()
        pd, pv = self.eng.alloc_draft_out(N, mb), self.eng.alloc_verify_out(N, mb)  # released after the prefill
        while any(done[n] < lens[n] for n in range(N)):
            T = [min(mb - 1, lens[n] - done[n]) for n in range(N)]
            Bc = max(T) + 1
            st = self._state(Bc)
            blk = np.full((N, Bc), mask, dtype=np.int32)
            for n in range(N):
                blk[n, :T[n]] = ids[n][done[n]:done[n] + T[n]]
            st.block_tokens.copy_(torch.from_numpy(blk))
            st.block_pos0.copy_(torch.as_tensor(done, dtype=torch.int32))
            self.kv.seq_len.copy_(torch.as_tensor(done, dtype=torch.int32))
            pd.xhat.zero_()
            pd.span_len.zero_()
            self.eng.s2d2_verify(self.kv, st, N, Bc, prm, pd, pv)
            self.eng.s2d2_kv_append(self.kv, N, Bc, pd, pv, zeros)
            done = [done[n] + T[n] for n in range(N)]
        torch.cuda.synchronize(self.dev)
        self.reset_blocks(lens, [int(x[-1]) for x in ids])

    def reset_blocks(self, seq_lens: Sequence[int], last_tokens: Optional[Sequence[int]] = None):
        """Fresh [MASK]^B block right after the prefix of every sequence.  For a right-shifted model the last prefix
        token is carried in front of the block instead of being counted as cached (its row scores the block's
        first position), so `last_tokens` is required there."""
        self.st = self._state(self.B)
        self.st.block_tokens.fill_(self.cfg.mask_id)
        self.st.carry_tokens.zero_()
        t = torch.as_tensor(list(seq_lens), dtype=torch.int32)
        self.st.block_pos0.copy_(t)
        if getattr(self.cfg, "right_shifted", False):
            if last_tokens is None:
                raise ValueError("a right-shifted model needs the last prefix token of every sequence")
            self.st.carry_tokens[:, 0].copy_(torch.as_tensor(list(last_tokens), dtype=torch.int32))
            t = t - 1
        self.kv.seq_len.copy_(t)
        self.kv.status.zero_()
        self.step_dev.zero_()

    def step(self, prm: Params, n_accept: Optional[torch.Tensor] = None, n_commit: Optional[torch.Tensor] = None,
             advance: bool = True):
        """draft -> verify -> accept -> kv_append -> block_advance, enqueued without any sync."""
        N, B, e = self.N, self.B, self.eng
        if n_accept is not None:
            self.a.t["n_accept"], self.a.t["n_commit"] = n_accept, n_commit
        e.s2d2_draft(self.kv, self.st, N, B, prm, self.d)
        e.s2d2_verify(self.kv, self.st, N, B, prm, self.d, self.v)
        e.s2d2_accept(self.st, N, B, prm, self.d, self.v, self.a)
        e.s2d2_kv_append(self.kv, N, B, self.d, self.v, self.a.n_accept)
        if advance:
            e.s2d2_block_advance(self.kv, self.st, N, B, prm.step_dev)

    def step_routed(self, prm: Params, rp: RouteParams):
        """Alg. 3 with its routing: draft -> DoVerify -> (verify -> accept -> kv_append for the sequences routed to the
        verifier, threshold commit for the others) -> block_advance.  The hysteresis state lives on the device and
        persists across steps and blocks (initially ON)."""
        N, B, e = self.N, self.B, self.eng
        if not hasattr(self, "route"):
            self.route = RouteOut.alloc(N, self.dev)
            self.hysteresis = torch.ones(N, dtype=torch.int32, device=self.dev)
            self._d_fallback = DraftOut({**self.d.t, "unmask": self.route.unmask_fallback})
        e.s2d2_draft(self.kv, self.st, N, B, prm, self.d)
        e.s2d2_route(N, B, rp, self.d, self.hysteresis, self.route)
        prm_r = dataclasses.replace(prm, active=self.route.do_verify)
        e.s2d2_verify(self.kv, self.st, N, B, prm_r, self.d, self.v)
        e.s2d2_accept(self.st, N, B, prm_r, self.d, self.v, self.a)
        e.s2d2_kv_append(self.kv, N, B, self.d, self.v, self.a.n_accept)
        e.s2d2_commit_threshold(self.st, N, B, self._d_fallback)
        e.s2d2_block_advance(self.kv, self.st, N, B, prm.step_dev)

    def generate(self, prm: Params, rp: RouteParams, n_blocks: int, max_steps_per_block: int, caching: str = "causal"):
        """Alg. 1's outer loop around the routed block sampler, for n_blocks blocks per sequence.  Host-driven: after
        every step the block tokens are read back to see which blocks are finished (one small copy per step).
        caching = "causal": the accepted prefix is appended after every verified step; "block": nothing is appended
        inside a block, drafting is fully bidirectional, and a finished block is appended by s2d2_block_complete.
        A block that has used max_steps_per_block steps commits all remaining proposals on its next step.
        Returns the committed tokens per sequence and the (kind, n_accept, n_commit) record of every step."""
        assert caching in ("causal", "block")
        N, B, e, mask = self.N, self.B, self.eng, self.cfg.mask_id
        if not hasattr(self, "route"):
            self.route = RouteOut.alloc(N, self.dev)
            self.hysteresis = torch.ones(N, dtype=torch.int32, device=self.dev)
            self._d_fallback = DraftOut({**self.d.t, "unmask": self.route.unmask_fallback})
        steps_in_block, blocks_done = [0] * N, [0] * N
        out, log = [[] for _ in range(N)], [[] for _ in range(N)]
        step = prm.step
        while any(b < n_blocks for b in blocks_done):
            p = dataclasses.replace(prm, step=step, ar_mask=1 if caching == "causal" else 0)
            e.s2d2_draft(self.kv, self.st, N, B, p, self.d)
            e.s2d2_route(N, B, rp, self.d, self.hysteresis, self.route)
            blk = self.st.block_tokens.cpu().numpy()
            dv = self.route.do_verify.cpu().numpy().copy()
            fb = self.route.unmask_fallback.cpu().numpy().copy()
            forced = False
            for n in range(N):
                if blocks_done[n] >= n_blocks:                     # finished sequences idle
                    dv[n], fb[n], forced = 0, 0, True
                elif steps_in_block[n] >= max_steps_per_block:     # out of steps: commit every proposal
                    dv[n], fb[n], forced = 0, sum(1 << i for i in range(B) if blk[n, i] == mask), True
            if forced:
                self.route.do_verify.copy_(torch.from_numpy(dv))
                self.route.unmask_fallback.copy_(torch.from_numpy(fb))
            pr = dataclasses.replace(p, active=self.route.do_verify)
            e.s2d2_verify(self.kv, self.st, N, B, pr, self.d, self.v)
            e.s2d2_accept(self.st, N, B, pr, self.d, self.v, self.a)
            if caching == "causal":
                e.s2d2_kv_append(self.kv, N, B, self.d, self.v, self.a.n_accept)
            e.s2d2_commit_threshold(self.st, N, B, self._d_fallback)
            if caching == "block":
                e.s2d2_block_complete(self.kv, self.st, N, B, self.v)
            after = self.st.block_tokens.cpu().numpy()
            if caching == "causal":
                # a block finished without a verifier forward is carried in front of the next one; what the carry
                # list (capacity B) cannot take is cached now by one causal forward (Alg. 1's per-block cache update)
                S, P0 = self.kv.seq_len.cpu().numpy(), self.st.block_pos0.cpu().numpy()
                if any((after[n] != mask).all() and max(0, int(P0[n] - S[n])) + B - max(0, min(B, int(S[n] - P0[n]))) > B
                       for n in range(N)):
                    e.s2d2_block_complete(self.kv, self.st, N, B, self.v, causal=1)
            n_acc, n_com = self.a.n_accept.cpu().numpy(), self.a.n_commit.cpu().numpy()
            for n in range(N):
                if blocks_done[n] >= n_blocks:
                    continue
                if dv[n]:
                    log[n].append(("verify", int(n_acc[n]), int(n_com[n])))
                else:
                    log[n].append(("threshold", 0, int(bin(int(fb[n]) & ((1 << B) - 1)).count("1"))))
                if (after[n] != mask).all():
                    out[n].extend(int(x) for x in after[n])
                    blocks_done[n] += 1
                    steps_in_block[n] = 0
                else:
                    steps_in_block[n] += 1
            e.s2d2_block_advance(self.kv, self.st, N, B, None)
            if int(self.kv.status.abs().sum()):   # a block that could not roll over, or a cache without room
                raise RuntimeError(f"generate: device status {self.kv.status.cpu().tolist()} after step {step}")
            step += 1
        return out, log

    def capture_step(self, prm: Params, advance: bool = True):
        """Records one step (plus the on-device running totals of accepted and committed tokens) into a HIP graph
        and returns it; `graph.replay()` then enqueues the whole step with one host call.  The RNG step word advances
        on the device (prm.step_dev), so every replay is a new step of the same session.  advance=False leaves
        s2d2_block_advance (which also bumps the step word) out of the graph, for a caller that wants to look at the
        block before it rolls over."""
        assert prm.step_dev is not None, "a captured step needs the device-resident step counter"
        self.tot_accept = torch.zeros(self.N, dtype=torch.int32, device=self.dev)
        self.tot_commit = torch.zeros(self.N, dtype=torch.int32, device=self.dev)
        side = torch.cuda.Stream(self.dev)
        side.wait_stream(torch.cuda.current_stream(self.dev))
        graph = torch.cuda.CUDAGraph()
        self.eng.set_stream(side)
        try:
            with torch.cuda.graph(graph, stream=side):
                self.step(prm, advance=advance)
                self.tot_accept += self.a.n_accept
                self.tot_commit += self.a.n_commit
        finally:
            self.eng.set_stream(torch.cuda.current_stream(self.dev))
        return graph
