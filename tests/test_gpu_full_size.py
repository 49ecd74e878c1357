"""GPU parity at the workloads' full shapes (all layers, full batch, long context), on sampled
sequences: sequences are independent, so row b of a batched GPU step must equal the oracle run
on sequence b alone.  Long caches are synthetic (seeded N(0, 0.64), keys sharpened), imported
once and cloned to every slot; sequences differ by their draft blocks and (ragged) lengths."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import Oracle, VerifyParams

pytestmark = pytest.mark.gpu
GREEDY = VerifyParams(mode=0, sample=0)


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


def _run_sampled(X, cfg, B, n_pos, lens, sample_ids, vp, steps=2, single_launch=None, plain=False,
                 expect_kernel=None):
    """GPU: B sequences with lengths lens; oracle: only sample_ids.  plain: next-token steps
    (one row per sequence) instead of speculative ones.  expect_kernel: a kernel class that the
    steps must have launched (checked with the library's per-launch trace).  Returns the tally."""
    K = 0 if plain else cfg["n_draft"]
    max_ctx = ((n_pos + (K + 1) * (steps + 1) + 63) // 64) * 64
    w = si.make_weights(cfg)
    eng = X.pkg.Engine(cfg, max_batch=B, max_ctx=max_ctx)
    eng.xsm_load_weights(si.pack_canonical(cfg, w))
    if single_launch is not None:
        eng.xsm_set_option(X.xsm.XSM_OPT_SINGLE_LAUNCH, single_launch)
    orc = Oracle(cfg, w, kv_dtype=np.float32)
    del w
    cond = si.make_cond(cfg, 1)                      # same condition tokens for every sequence
    if cond is not None:
        eng.xsm_prefill([0], None, eng.to_device(cond))
    fill = si.make_kv_fill(cfg, 1, n_pos)
    fill[:, 0] = si.bf16_round(fill[:, 0] * 6.0)
    for l in range(cfg["n_layers"]):
        eng.xsm_debug_kv_import(l, 0, 0, 0, fill[l, 0, 0])
        eng.xsm_debug_kv_import(l, 1, 0, 0, fill[l, 1, 0])
    for b in range(1, B):
        eng.xsm_debug_kv_clone(0, b)
    first = si.first_block(cfg, B)[:, :K + 1]
    torch = X.torch
    buf = eng.buffers(B, spec=not plain, debug=True)
    cur_len = list(lens)
    blocks = first.copy()
    states = {}
    for b in sample_ids:
        st = orc.new_state(cap=max_ctx, seq_id=b)
        if cond is not None:
            orc.prefill(st, None, cond[0])
        for l in range(cfg["n_layers"]):
            st.k[l][:n_pos] = np.transpose(fill[l, 0, 0], (1, 0, 2))
            st.v[l][:n_pos] = np.transpose(fill[l, 1, 0], (1, 0, 2))
        st.n = lens[b]
        states[b] = st
    del fill
    tal = X.H.Tally()
    tol = X.H.logit_tol(cfg)
    vpg = X.H.to_vp_gpu(X.xsm, vp)
    own = X.H.own_draws(cfg)
    if expect_kernel:
        X.xsm.xsm_debug_trace_enable(True)
        X.xsm.xsm_debug_trace_report()
    for step in range(steps):
        buf.kv_len.copy_(torch.tensor(cur_len, dtype=torch.int32))
        buf.block.copy_(torch.tensor(blocks, dtype=torch.int32))
        (eng.xsm_plain_step if plain else eng.xsm_spec_step)(buf, vpg, max(cur_len))
        torch.cuda.synchronize()
        eng.xsm_check_device()
        g_acc = buf.n_accepted.cpu().numpy()
        g_blk = buf.block.cpu().numpy()
        g_out = buf.out_tokens.cpu().numpy()
        assert ((g_acc >= 1) & (g_acc <= K + 1)).all()
        assert (buf.flags.cpu().numpy() & ~1 == 0).all()
        assert (buf.kv_len.cpu().numpy() == np.array(cur_len) + g_acc).all()
        for b in sample_ids:
            st = states[b]
            n0 = st.n
            r = orc.plain_step(st, int(blocks[b][0]), vp) if plain else orc.spec_step(st, blocks[b], vp)
            zg = buf.logits[b].cpu().numpy()
            for j in range(K + 1):
                e = X.H.rel_err(zg[j], r["Z0"][j])
                tal.max_rel = max(tal.max_rel, e); tal.rows += 1
                assert e <= tol, f"step {step} seq {b} row {j}: rel err {e:.3e}"
            a = r["n_accepted"] - 1
            safe = all(X.H.accept_margin(r["Z0"][j - 1], int(blocks[b][j]), vp) > X.H.TIE
                       for j in range(1, min(a + 1, K) + 1))
            tal.decisions += 1
            if not safe:
                tal.flagged += 1
            elif int(g_acc[b]) != a + 1:
                tal.mismatches.append(f"step {step} seq {b}: n_accepted {g_acc[b]} vs {a + 1}")
            else:
                zh = buf.head_logits[b].cpu().numpy() if K > 0 else None
                X.H.check_draw(tal, f"step {step} seq {b}", "y0", r["diag"][0], int(g_out[b, a]),
                               r["out_tokens"][a], zg[a], vp, n0 + a + 1, 0, st.seq_id, own=own)
                for k in range(1, K + 1):
                    e = X.H.rel_err(zh[k - 1], r["Zh"][k - 1])
                    tal.max_rel = max(tal.max_rel, e); tal.rows += 1
                    assert e <= tol, f"step {step} seq {b} head {k}: rel err {e:.3e}"
                    X.H.check_draw(tal, f"step {step} seq {b}", f"head {k}", r["diag"][k], int(g_blk[b, k]),
                                   r["next_block"][k], zh[k - 1], vp, n0 + a + 1 + k, k, st.seq_id, own=own)
            # teacher forcing for the sampled sequences; the others free-run
            g_blk[b] = r["next_block"]
            g_acc[b] = r["n_accepted"]
        blocks = g_blk.copy()
        cur_len = [int(cur_len[b] + g_acc[b]) for b in range(B)]
    if expect_kernel:
        ran = X.xsm.xsm_debug_trace_report()
        X.xsm.xsm_debug_trace_enable(False)
        assert expect_kernel in ran and ran[expect_kernel][0] >= steps, (expect_kernel, sorted(ran))
    eng.close()
    X.H.report(tal, f"{cfg['name']} B{B} K{K}{' plain' if plain else ''} ctx {n_pos}"
                    f"{'' if single_launch is None else f' single_launch={single_launch}'}")
    return tal


@pytest.mark.parametrize("single_launch", [1, 0])
def test_config1_full_model_long_context(X, single_launch):
    """The benchmark's launch configuration: 24 layers, batch 1, K=4, context near its end."""
    cfg = si.get_config("c1")
    _run_sampled(X, cfg, 1, 4340, [4331], [0], GREEDY, steps=3, single_launch=single_launch)


def test_config2_full_batch_top8_sampling(X):
    cfg = si.get_config("c2")
    B = cfg["batch"]
    lens = [8100 - 37 * b for b in range(B)]
    vp = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=2024)
    _run_sampled(X, cfg, B, 8100, lens, [0, B - 1], vp, steps=2)


def test_config3_cross_attention_full_size(X):
    cfg = si.get_config("c3")
    B = cfg["batch"]
    lens = [16300 - 501 * b for b in range(B)]
    _run_sampled(X, cfg, B, 16300, lens, [B - 1], GREEDY, steps=2)


def test_config3_shape_with_cross_attention_heads(X):
    """Config 3's shape (d=1536, 2048 condition tokens, vocabulary 8192, batch 8, long context) with
    cross-attention decoding heads and per-head unembeddings; 6 layers keep the oracle within
    seconds."""
    cfg = si.get_config("c3", head_kind="ca", n_layers=6)
    B = cfg["batch"]
    lens = [16300 - 501 * b for b in range(B)]
    _run_sampled(X, cfg, B, 16300, lens, [0, B - 1], GREEDY, steps=2)


def test_config4_large_batch(X):
    cfg = si.get_config("c4", batch=128, n_draft=8)
    lens = [10000 - 7 * b for b in range(128)]
    _run_sampled(X, cfg, 128, 10000, lens, [0, 127], GREEDY, steps=2)


@pytest.mark.parametrize("B,K", [(1, 8), (8, 4), (32, 4), (64, 4), (64, 8)])
def test_config4_grid_points(X, B, K):
    """More points of the throughput sweep at context 10000, two sampled sequences each:
    batch 1 with K = 8 runs on the single-launch kernel (9 block rows: two read rounds per stage,
    16 key slices per head); M = 40 / 160 on the mid-batch kernels, M = 320 / 576 on the
    row-blocked ones."""
    cfg = si.get_config("c4", batch=B, n_draft=K)
    lens = [10000 - 7 * b for b in range(B)]
    _run_sampled(X, cfg, B, 10000, lens, sorted({0, B - 1}), GREEDY, steps=2,
                 expect_kernel="step_small" if B == 1 else "fattn")


@pytest.mark.parametrize("B", [8, 128])
def test_config4_plain_step(X, B):
    """The sweep's non-speculative comparison: next-token steps at the same shapes (batch 8 runs
    on the single-launch kernel, batch 128 on the mid-batch kernels)."""
    cfg = si.get_config("c4", batch=B)
    lens = [10000 - 7 * b for b in range(B)]
    _run_sampled(X, cfg, B, 10000, lens, [0, B - 1], GREEDY, steps=2, plain=True,
                 expect_kernel="step_small" if B == 8 else "fattn")
