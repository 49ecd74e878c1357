"""Admission and compaction of sequences around the step entry points.

The outer loop of Alg. 1 ("while no EOS: speculative step") for more requests than
the engine has cache slots.  A request is admitted into a free slot (xsm_prefill of
its condition prefix, block = start token + K initial candidates, Alg. 1 line 1),
steps with the other admitted sequences as one batch, and leaves when it has
produced its token budget or an EOS token; the rows of the batch are then compacted
so that every step runs over live sequences only.  The library's batch rows name
their cache slot, so compaction moves a few integers, never cache contents.

Everything here is argument marshalling: the arithmetic of a step runs in the
library's kernels, row arrays are gathered with device-side indexing.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Request:
    first_block: list                  # start token, then K initial candidate tokens (1 token for plain steps)
    max_new_tokens: int
    prefix: np.ndarray | None = None   # [P][d] prefix embeddings, None = empty prefix
    cond: np.ndarray | None = None     # [n_cond][d] condition tokens (cross-attention models)
    eos: int = -1                      # token id that ends the sequence, -1 = none


@dataclass
class _Live:
    rid: int
    slot: int
    length: int                        # cached positions, mirrors the device's kv_len
    tokens: list = field(default_factory=list)


class Batcher:
    def __init__(self, engine, vp, spec: bool = True):
        self.eng, self.vp, self.spec = engine, vp, spec
        self.R = engine.c_cfg.n_draft + 1 if spec else 1
        self.pending: list = []
        self.requests: dict = {}
        self.free = list(range(engine.max_batch))
        self.live: list = []
        self.buf = None
        self.accepted_per_step: list = []    # one entry per (step, live sequence)
        self.steps = 0

    def submit(self, req: Request) -> int:
        P = 0 if req.prefix is None else int(req.prefix.shape[0])
        if req.max_new_tokens < 1:
            raise ValueError("max_new_tokens < 1")
        if P + req.max_new_tokens - 1 + self.R > self.eng.max_ctx:
            raise ValueError("prefix + token budget + block does not fit max_ctx")
        if len(req.first_block) < self.R:
            raise ValueError(f"first_block needs {self.R} tokens")
        rid = len(self.requests)
        self.requests[rid] = req
        self.pending.append(rid)
        return rid

    # -- admission: one prefill call per distinct prefix length ----------------------------
    def _admit(self):
        new = []
        while self.pending and self.free:
            rid = self.pending.pop(0)
            new.append(_Live(rid, self.free.pop(0), 0))
        by_len: dict = {}
        for lv in new:
            req = self.requests[lv.rid]
            lv.length = 0 if req.prefix is None else int(req.prefix.shape[0])
            by_len.setdefault(lv.length, []).append(lv)
        for P, group in by_len.items():
            pre = None if P == 0 else self.eng.to_device(np.stack([self.requests[lv.rid].prefix for lv in group]))
            cond = None
            if self.requests[group[0].rid].cond is not None:
                cond = self.eng.to_device(np.stack([self.requests[lv.rid].cond for lv in group]))
            if pre is not None or cond is not None:
                self.eng.xsm_prefill([lv.slot for lv in group], pre, cond)
        return new

    # -- the batch's row arrays after a change of the live set ------------------------------
    def _rebuild(self, keep_rows: list, new: list):
        torch = self.eng.torch
        live = [self.live[i] for i in keep_rows] + new
        nb = self.eng.buffers(len(live), spec=self.spec) if live else None
        if nb is not None:
            k = len(keep_rows)
            if k:
                idx = torch.tensor(keep_rows, dtype=torch.int64, device=self.eng.device)
                nb.kv_len[:k] = self.buf.kv_len[idx]
                nb.block[:k] = self.buf.block[idx]
            if new:
                nb.kv_len[k:] = torch.tensor([lv.length for lv in new], dtype=torch.int32)
                nb.block[k:] = torch.tensor([list(self.requests[lv.rid].first_block[:self.R]) for lv in new],
                                            dtype=torch.int32)
            nb.slot.copy_(torch.tensor([lv.slot for lv in live], dtype=torch.int32))
        self.live, self.buf = live, nb

    def run(self) -> dict:
        """Runs until every submitted request has finished; returns {request id: tokens}."""
        torch = self.eng.torch
        done: dict = {}
        while self.pending or self.live:
            new = self._admit()
            if new:
                self._rebuild(list(range(len(self.live))), new)
            bound = max(lv.length for lv in self.live)
            if self.spec:
                self.eng.xsm_spec_step(self.buf, self.vp, bound)
            else:
                self.eng.xsm_plain_step(self.buf, self.vp, bound)
            self.steps += 1
            n_acc = self.buf.n_accepted.cpu().numpy()          # (synchronises the stream)
            out = self.buf.out_tokens.cpu().numpy()
            flags = self.buf.flags.cpu().numpy()
            keep = []
            for i, lv in enumerate(self.live):
                if flags[i] & 16:           # XSM_FLAG_DEVICE_TIMEOUT: nothing was produced; say why
                    self.eng.xsm_check_device()
                    raise RuntimeError(f"request {lv.rid}: the step timed out on the device")
                if flags[i] & ~1 or n_acc[i] < 1:
                    raise RuntimeError(f"request {lv.rid}: device flagged input error {int(flags[i])}")
                req = self.requests[lv.rid]
                a = int(n_acc[i])
                self.accepted_per_step.append(a)
                lv.length += a
                finished = False
                for t in out[i, :a]:
                    lv.tokens.append(int(t))
                    if int(t) == req.eos or len(lv.tokens) >= req.max_new_tokens:
                        finished = True
                        break
                if finished:
                    done[lv.rid] = lv.tokens
                    self.free.append(lv.slot)
                else:
                    keep.append(i)
            if len(keep) != len(self.live):
                self._rebuild(keep, [])
        return done
