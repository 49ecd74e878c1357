"""Admission and compaction of sequences around the step entry points.

The outer loop of Alg. 1 ("while no EOS: speculative step") for more requests than
the engine has cache slots.  A request is admitted into a free slot (xsm_prefill of
its condition prefix, block = start token + K initial candidates, Alg. 1 line 1),
steps with the other admitted sequences as one batch, and leaves when it has
produced its token budget or an EOS token; the rows of the batch are then compacted
so that every step runs over live sequences only.  The library's batch rows name
their cache slot, so compaction moves a few integers, never cache contents.

The host does not wait for the device after every step: `sync_every` = n steps are
enqueued back to back, each followed by a device-side copy of its outputs (accepted
count, flags, tokens) into row j of a ring, and the ring comes back in one copy.  EOS
and token budgets are therefore seen up to n - 1 steps late; what a finished
sequence produced after its end is dropped (at most (n - 1)(K + 1) tokens, and that
much cache room is asked for at submission).

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
    def __init__(self, engine, vp, spec: bool = True, sync_every: int = 4):
        if sync_every < 1:
            raise ValueError("sync_every < 1")
        self.eng, self.vp, self.spec, self.n = engine, vp, spec, sync_every
        self.R = engine.c_cfg.n_draft + 1 if spec else 1
        self.ring = self.ring_host = None     # [n][rows][2 + R] int32: accepted, flags, tokens
        self.syncs = 0
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
        # a sequence may run on until its group of n steps ends: room for the blocks of all of them
        if P + req.max_new_tokens - 1 + self.n * self.R > self.eng.max_ctx:
            raise ValueError("prefix + token budget + the blocks of sync_every steps do not fit max_ctx")
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
            self.ring = torch.zeros((self.n, len(live), 2 + self.R), dtype=torch.int32, device=self.eng.device)
            self.ring_host = torch.zeros((self.n, len(live), 2 + self.R), dtype=torch.int32,
                                         pin_memory=self.eng.device.type == "cuda")
        self.live, self.buf = live, nb

    def run(self) -> dict:
        """Runs until every submitted request has finished; returns {request id: tokens}."""
        torch = self.eng.torch
        done: dict = {}
        step = self.eng.xsm_spec_step if self.spec else self.eng.xsm_plain_step
        while self.pending or self.live:
            new = self._admit()
            if new:
                self._rebuild(list(range(len(self.live))), new)
            # n steps without a host round trip; the lengths grow on the device, the host only
            # knows a bound for them (every step adds at most R positions)
            bound = max(lv.length for lv in self.live)
            for j in range(self.n):
                step(self.buf, self.vp, min(bound + j * self.R, self.eng.max_ctx - self.R))
                self.ring[j, :, 0] = self.buf.n_accepted
                self.ring[j, :, 1] = self.buf.flags
                self.ring[j, :, 2:] = self.buf.out_tokens
            self.steps += self.n
            self.ring_host.copy_(self.ring)                    # one copy back; synchronises the stream
            if self.eng.device.type == "cuda":
                torch.cuda.current_stream().synchronize()
            self.syncs += 1
            rec = self.ring_host.numpy()
            keep = []
            for i, lv in enumerate(self.live):
                req = self.requests[lv.rid]
                finished = False
                for j in range(self.n):
                    a, fl = int(rec[j, i, 0]), int(rec[j, i, 1])
                    if fl & 16:             # XSM_FLAG_DEVICE_TIMEOUT: nothing was produced; say why
                        self.eng.xsm_check_device()
                        raise RuntimeError(f"request {lv.rid}: the step timed out on the device")
                    if fl & ~1 or a < 1:
                        raise RuntimeError(f"request {lv.rid}: device flagged input error {fl}")
                    self.accepted_per_step.append(a)
                    lv.length += a
                    for t in rec[j, i, 2:2 + a]:
                        lv.tokens.append(int(t))
                        if int(t) == req.eos or len(lv.tokens) >= req.max_new_tokens:
                            finished = True
                            break
                    if finished:            # the group's later steps of this sequence are dropped
                        break
                if finished:
                    done[lv.rid] = lv.tokens
                    self.free.append(lv.slot)
                else:
                    keep.append(i)
            if len(keep) != len(self.live):
                self._rebuild(keep, [])
        return done
