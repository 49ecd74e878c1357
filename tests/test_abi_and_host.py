"""CPU-side checks: the built library exports every symbol the header declares,
argument validation works without a GPU, and the speed accounting reproduces
the paper's printed table rows."""
import ctypes as C
import os
import re

import pytest

from paper_2507_23777_amd import metrics, xsm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "xsm.h")).read()
    return sorted(set(re.findall(r"XSM_API\s+[\w\s\*]+?\b(xsm_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert len(names) >= 14 and set(names) == set(xsm.API)
    L = xsm.lib()
    for n in names:
        assert hasattr(L, n), n


def test_create_validates_configuration():
    L = xsm.lib()
    import synth_inputs as si
    h = C.c_void_p()
    good = xsm.make_config(si.get_config("c0"))
    assert L.xsm_create(C.byref(good), C.byref(h)) == 0
    assert L.xsm_weights_bytes(h) > 0 and L.xsm_kv_bytes(h) > 0 and L.xsm_workspace_bytes(h) > 0
    import numpy as np
    w = si.make_weights(si.get_config("c0"))
    assert L.xsm_canonical_weight_elems(h) == si.pack_canonical(si.get_config("c0"), w).size
    # unbound context refuses work, with a message
    vp, bt = xsm.xsm_verify_params(), xsm.xsm_batch()
    assert L.xsm_spec_step(h, C.byref(bt), C.byref(vp), None) == -3
    assert b"bound" in L.xsm_last_error(h)
    assert L.xsm_bind(h, None, None, None) == -1
    L.xsm_destroy(h)
    for field, val in [("head_dim", 48), ("n_draft", 16), ("d_model", 100), ("dtype", 3), ("max_batch", 0)]:
        bad = xsm.make_config(si.get_config("c0"))
        setattr(bad, field, val)
        assert L.xsm_create(C.byref(bad), C.byref(h)) == -1, field
        assert len(L.xsm_last_error(None)) > 0


def test_speedup_formula_reproduces_printed_tables(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "speedup_tables.txt"))
            if l.strip() and not l.startswith("#")]
    base = float(rows[0][2])
    assert rows[0][0] == "A"
    for name, scr, lat, printed in rows:
        s = metrics.speedup(float(scr), float(lat), base)
        # printed inputs are themselves rounded, so allow one unit of the last printed digit
        assert abs(s - float(printed)) < 0.0101, name
    assert metrics.step_compression_ratio([1, 2, 5, 1, 1]) == 2.0
    with pytest.raises(ValueError):
        metrics.step_compression_ratio([])


class _StubEngine:
    """Stands in for Engine in the batcher's host logic: the 'model' is a fixed integer rule of
    (cache length, last token), so every request's token stream is known without a GPU."""

    def __init__(self, torch, K, max_batch, max_ctx):
        self.torch, self.device = torch, torch.device("cpu")
        self.c_cfg = type("C", (), {"n_draft": K, "vocab": 1001})()
        self.max_batch, self.max_ctx = max_batch, max_ctx
        self.prefills, self.batch_sizes = [], []

    def to_device(self, x):
        return self.torch.from_numpy(x)

    def xsm_prefill(self, slots, prefix=None, cond=None):
        assert len(set(slots)) == len(slots) and all(0 <= s < self.max_batch for s in slots)
        self.prefills.append((list(slots), 0 if prefix is None else int(prefix.shape[1])))

    def buffers(self, n_seq, spec=True, debug=False):
        K = self.c_cfg.n_draft
        return xsm.StepBuffers(self.torch, self.device, n_seq, K + 1 if spec else 1, 1001, K, False)

    @staticmethod
    def rule(n, last, R):
        a = 1 + (last + n) % R
        return a, [(last * 31 + n + 7 * j) % 1000 + 1 for j in range(a)]

    def xsm_spec_step(self, buf, vp, bound):
        slots = buf.slot.tolist()
        assert len(set(slots)) == len(slots)
        self.batch_sizes.append(buf.n_seq)
        for i in range(buf.n_seq):
            n, last = int(buf.kv_len[i]), int(buf.block[i, 0])
            assert n <= bound and n + buf.R <= self.max_ctx
            a, toks = self.rule(n, last, buf.R)
            buf.n_accepted[i] = a
            buf.out_tokens[i, :a] = self.torch.tensor(toks, dtype=self.torch.int32)
            buf.block[i, 0] = toks[-1]
            buf.kv_len[i] = n + a
            buf.flags[i] = 0

    xsm_plain_step = xsm_spec_step


@pytest.mark.parametrize("sync_every", [1, 4])
@pytest.mark.parametrize("spec", [True, False])
def test_batcher_admission_compaction_budget_and_eos(spec, sync_every):
    """Also with the host looking at the outputs only every fourth step: EOS and budgets are then
    seen late, the tokens a finished sequence went on to produce are dropped, and every request's
    stream is the same as with a look after every step."""
    import numpy as np
    import torch
    from paper_2507_23777_amd.batcher import Batcher, Request
    K = 4
    R = K + 1 if spec else 1
    eng = _StubEngine(torch, K, max_batch=3, max_ctx=200)
    P = [10, 0, 10, 33, 5, 10, 0, 21]
    budget = [17, 5, 40, 1, 23, 9, 30, 12]
    eos = [-1, -1, -1, -1, -1, -1, 500, -1]
    expect = {}
    for i in range(len(P)):
        n, last, toks = P[i], 3 + i, []
        while len(toks) < budget[i]:
            a, t = _StubEngine.rule(n, last, R)
            toks += t
            n, last = n + a, t[-1]
        toks = toks[:budget[i]]
        if i == 6:                       # an EOS that the stream is known to reach
            eos[i] = toks[11]
            toks = toks[:toks.index(eos[i]) + 1]
        expect[i] = toks
    bt = Batcher(eng, None, spec=spec, sync_every=sync_every)
    for i in range(len(P)):
        rid = bt.submit(Request(first_block=[3 + i] + [0] * K, max_new_tokens=budget[i], eos=eos[i],
                                prefix=None if P[i] == 0 else np.zeros((P[i], 8), np.float32)))
        assert rid == i
    got = bt.run()
    assert got == expect
    assert sorted(bt.free) == [0, 1, 2] and not bt.live and not bt.pending
    assert bt.syncs * sync_every == bt.steps == len(eng.batch_sizes)
    assert max(eng.batch_sizes) == 3 and min(eng.batch_sizes) >= 1
    # every request was prefilled exactly once (empty prefixes need none), into a slot that was free
    assert sorted(s for slots, _ in eng.prefills for s in slots).count(0) >= 1
    assert sum(len(slots) for slots, _ in eng.prefills) == sum(1 for p in P if p > 0)
    assert all(p in P for _, p in eng.prefills)
    with pytest.raises(ValueError):
        bt.submit(Request(first_block=[1] * R, max_new_tokens=500))          # does not fit max_ctx
    with pytest.raises(ValueError):
        bt.submit(Request(first_block=[1], max_new_tokens=5) if spec else Request(first_block=[], max_new_tokens=5))


def test_algorithmic_bytes_of_the_workloads():
    """The roofline's numerator: weights once + cached keys/values once + new keys/values + logits.
    Hand-computed figures of three workloads: config 1 at context 257 (620.8 MB of weights, 25.3 MB
    of cache), config 4 at batch 128, K = 8, context 10000 (327.2 MB, 62.9 GB), config 3 at batch 8,
    context 16384 (1.63 GB, 19.3 GB of self-attention cache and 2.4 GB of condition keys/values)."""
    import bench
    import synth_inputs as si
    c1 = si.get_config("c1")
    assert abs(bench.algorithmic_bytes(c1, 1, 257) - (620.8e6 + 25.3e6 + 0.5e6 + 0.15e6)) < 0.5e6
    c4 = si.get_config("c4", batch=128, n_draft=8)
    assert abs(bench.algorithmic_bytes(c4, 128, 128 * 10000) - (0.3272e9 + 62.91e9 + 0.057e9 + 0.036e9)) < 0.02e9
    c3 = si.get_config("c3")
    assert abs(bench.algorithmic_bytes(c3, 8, 8 * 16384) - (1.63e9 + 19.33e9 + 2.42e9)) < 0.02e9
