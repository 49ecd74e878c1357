"""The step entry point that allocates nothing (xsm_spec_step_static): through the C ABI, its
outputs against xsm_spec_step's on the same inputs, bit for bit (same kernels, same order; the
bound workspace is filled with NaN bytes while it runs, so it cannot have been used), on two
calls in a row, the second with fewer sequences; then both paths against the oracle; and the
refusal of a configuration whose steps need more than the static array holds."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import VerifyParams

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def X():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the xsm hot path has no CPU fallback")
    import paper_2507_23777_amd as pkg
    from paper_2507_23777_amd import xsm
    import xsm_harness as H
    xsm.lib()
    return type("X", (), {"pkg": pkg, "xsm": xsm, "H": H, "torch": torch})


def _outputs(torch, buf):
    torch.cuda.synchronize()
    return {k: getattr(buf, k).cpu().clone() for k in ("n_accepted", "out_tokens", "block", "kv_len", "flags",
                                                       "logits", "head_logits")}


@pytest.mark.parametrize("shape", ["mid_bf16", "c1_shape_bf16", "tiny_fp32"])
def test_static_scratch_step_equals_the_workspace_step(X, shape):
    torch = X.torch
    if shape == "mid_bf16":
        cfg = si.tiny_config(n_layers=3, d_model=256, n_heads=4, head_dim=64, d_ffn=1024, vocab=1008,
                             n_draft=4, dtype="bf16", prefix=37, max_ctx=512, seed=71)
        lens = [37, 20, 9]
    elif shape == "c1_shape_bf16":
        cfg = si.get_config("c1", n_layers=2, max_ctx=512, prefix=70)
        lens = [70, 33, 5]
    else:
        cfg = si.tiny_config(n_layers=2, d_model=64, n_heads=2, head_dim=32, d_ffn=128, vocab=64, n_draft=3,
                             dtype="f32", max_ctx=160, seed=72)
        lens = [5, 17, 33]
    vp = VerifyParams(mode=1, top_ka=4, temperature=0.9, sample=1, seed=321)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=lens)
    # the reference is the same per-stage kernels with the bound workspace
    eng.xsm_set_option(X.xsm.XSM_OPT_SINGLE_LAUNCH, 0)
    vpg = X.H.to_vp_gpu(X.xsm, vp)
    first = torch.tensor(si.first_block(cfg, 3), dtype=torch.int32)
    cur_len = torch.tensor(lens, dtype=torch.int32)
    for n_seq in (3, 2):                               # two calls in a row, the second with a smaller input
        got = {}
        for which in ("workspace", "static"):
            buf = eng.buffers(n_seq, spec=True, debug=True)
            buf.kv_len.copy_(cur_len[:n_seq]); buf.block.copy_(first[:n_seq])
            buf.n_accepted.fill_(-5); buf.out_tokens.fill_(-5)
            if which == "workspace":
                eng.xsm_spec_step(buf, vpg, int(cur_len.max()))
            else:
                torch.cuda.synchronize()
                keep = eng.d_ws.clone()
                eng.d_ws.fill_(0xFF)                   # NaN bytes: the call must not touch the bound workspace
                eng.xsm_spec_step_static(buf, vpg, int(cur_len.max()))
                torch.cuda.synchronize()
                assert bool((eng.d_ws == 0xFF).all()), "xsm_spec_step_static wrote to the bound workspace"
                eng.d_ws.copy_(keep)
            got[which] = _outputs(torch, buf)
        a, b = got["workspace"], got["static"]
        for k in ("n_accepted", "block", "kv_len", "flags", "logits", "head_logits"):
            assert torch.equal(a[k], b[k]), (shape, n_seq, k)
        for r in range(n_seq):
            n = int(a["n_accepted"][r])
            assert 1 <= n <= cfg["n_draft"] + 1
            assert torch.equal(a["out_tokens"][r, :n], b["out_tokens"][r, :n]), (shape, n_seq, r)
        cur_len[:n_seq] = a["kv_len"]
        first[:n_seq] = a["block"]
    # and against the oracle, from the prefilled state (lock-step re-sets lengths and blocks itself)
    class StaticEngine:                                # the harness calls eng.xsm_spec_step
        def __init__(self, e): self.e = e
        def __getattr__(self, k): return getattr(self.e, k)
        def xsm_spec_step(self, buf, vpg, bound): return self.e.xsm_spec_step_static(buf, vpg, bound)
    tal = X.H.lockstep(cfg, orc, states, StaticEngine(eng), X.xsm, vp, 4, si.first_block(cfg, 3))
    X.H.report(tal, f"static-scratch step vs oracle ({shape})")
    eng.xsm_check_device()


def test_static_scratch_step_refuses_what_does_not_fit(X):
    cfg = si.get_config("c4", batch=32, n_draft=8, n_layers=1, max_ctx=256)
    eng = X.pkg.Engine(cfg, max_batch=32, max_ctx=256)
    eng.xsm_load_weights(si.pack_canonical(cfg, si.make_weights(cfg)))
    buf = eng.buffers(32, spec=True)
    buf.block.fill_(1)
    vpg = X.H.to_vp_gpu(X.xsm, VerifyParams())
    with pytest.raises(X.xsm.XsmError, match="static array holds"):
        eng.xsm_spec_step_static(buf, vpg, 0)
    eng.xsm_spec_step(buf, vpg, 0)                     # the workspace entry point takes it
    X.torch.cuda.synchronize()
    assert (buf.n_accepted >= 1).all()
