"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Token decisions must agree wherever the oracle's margin
exceeds 1e-2 (flagged otherwise); logits within 2e-2 (bf16) / 1e-5 (fp32) max
relative error per row."""
import copy

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


def _mid_cfg(**kw):
    cfg = si.tiny_config(n_layers=3, d_model=256, n_heads=4, head_dim=64, d_ffn=1024, vocab=1008,
                         n_draft=4, dtype="bf16", prefix=37, max_ctx=512, seed=21)
    cfg.update(kw)
    return cfg


def _report(tal, name):
    import xsm_harness
    xsm_harness.report(tal, name)


def test_config0_fp32_lockstep_and_free_running(X):
    cfg = si.get_config("c0")
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, perturb=False)
    st0 = copy.deepcopy(states[0])
    first = si.first_block(cfg, 1)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 40, first)
    _report(tal, "c0 lockstep")
    assert tal.max_rel < 1e-5
    # free-running generation: 512 tokens, GPU alone, must equal the oracle's and plain decoding
    ref, _, _ = orc.generate_spec(copy.deepcopy(st0), first[0], 512, GREEDY)
    torch = X.torch
    buf = eng.buffers(1, spec=True)
    buf.kv_len.fill_(cfg["prefix"]); buf.block.copy_(torch.tensor(first))
    vpg = X.H.to_vp_gpu(X.xsm, GREEDY)
    toks, steps, flagged = [], 0, 0
    while len(toks) < 512:
        eng.xsm_spec_step(buf, vpg, cfg["prefix"] + len(toks))
        torch.cuda.synchronize()
        n = int(buf.n_accepted[0]); assert 1 <= n <= cfg["n_draft"] + 1
        toks += buf.out_tokens[0, :n].tolist(); steps += 1
        flagged += int(buf.flags[0]) & 1
    assert int(buf.kv_len[0]) == cfg["prefix"] + len(toks)
    pb = eng.buffers(1, spec=False)
    # plain decoding restarts from the prefix: the cache beyond it is simply overwritten
    pb.kv_len.fill_(cfg["prefix"]); pb.block.copy_(torch.tensor(first[:, :1]))
    ptoks = []
    for i in range(512):
        eng.xsm_plain_step(pb, vpg, cfg["prefix"] + i)
        ptoks.append(int(pb.out_tokens[0, 0]))
    print(f"[c0 free-run] steps {steps} device near-tie flags {flagged}", flush=True)
    assert toks[:512] == ref, "speculative GPU output differs from the oracle"
    assert ptoks == ref, "plain GPU decoding differs from greedy speculative decoding"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tiny_ragged_batch(X, dtype):
    cfg = si.tiny_config(n_layers=2, d_model=64, n_heads=2, head_dim=32, d_ffn=128, vocab=64, n_draft=3,
                         dtype=dtype, max_ctx=160, seed=11)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=[5, 17, 33])
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 12, si.first_block(cfg, 3))
    _report(tal, f"tiny ragged {dtype}")


def test_fp32_sampled_draws_equal_the_oracles_own_draws(X):
    """fp32 models: the GPU's logits agree with the oracle's to 1e-6, so its categorical and
    probability-tree draws are compared with the oracle's OWN draws (the Philox uniforms, the
    inverse CDF over ascending token index, the tree's depth-first order), not with the oracle's
    sampler re-run on the GPU's logits.  Top-K_a acceptance, the probability threshold, plain
    sampled steps; a ragged batch on the general-shape kernels, and config 0's shape."""
    cfg = si.tiny_config(n_layers=2, d_model=64, n_heads=2, head_dim=32, d_ffn=128, vocab=64, n_draft=3,
                         dtype="f32", max_ctx=224, seed=14)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=[5, 17, 33])
    assert X.H.own_draws(cfg)
    vp = VerifyParams(mode=1, top_ka=4, temperature=0.8, sample=1, seed=4242)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 16, si.first_block(cfg, 3))
    _report(tal, "fp32 own draws: top-4 categorical T=0.8")
    vp = VerifyParams(mode=2, delta=0.03, temperature=0.6, sample=1, seed=4243)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 10, si.first_block(cfg, 3))
    _report(tal, "fp32 own draws: threshold 0.03 categorical T=0.6")
    seen = set()
    for ks, T in ((2, 0.05), (3, 0.1), (2, 0.3), (4, 0.02)):
        vp = VerifyParams(mode=1, top_ka=4, temperature=T, sample=2, seed=4300 + ks, top_ks=ks, pts_prune=1e-5)
        tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 4, si.first_block(cfg, 3))
        _report(tal, f"fp32 own draws: tree K_s={ks} T={T} paths {sorted(set(tal.pts_paths))}")
        seen |= {"none" if n == 0 else "all" if n == ks ** cfg["n_draft"] else "some" for n in tal.pts_paths}
    assert "some" in seen or "all" in seen, seen
    vp = VerifyParams(mode=0, temperature=1.3, sample=1, seed=4244)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 10, [[3], [4], [5]], plain=True)
    _report(tal, "fp32 own draws: plain sampled steps T=1.3")
    cfg = si.get_config("c0")
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, perturb=False)
    vp = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=4245)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 12, si.first_block(cfg, 1))
    _report(tal, "c0 own draws: top-8 categorical T=0.8")
    assert tal.max_rel < 1e-5


def test_mid_bf16_forced_drafts_hit_every_accept_length(X):
    cfg = _mid_cfg()
    K = cfg["n_draft"]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2)

    def forced(step, b, st, blk):
        full = X.H.true_continuation(orc, st, blk[0], K, GREEDY)
        j = (step + b) % (K + 1)            # corrupt candidate j+1 (none when j == K)
        if j < K:
            full[j + 1] = (full[j + 1] + 1) % cfg["vocab"]
        return full

    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 2 * (K + 1), si.first_block(cfg, 2), forced=forced)
    _report(tal, "mid forced")
    assert set(tal.accept_hist) == set(range(1, K + 2))


def test_mid_bf16_topk_categorical(X):
    cfg = _mid_cfg(n_draft=6, seed=22)
    vp = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=0xABCDEF0123)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 4, prefix_lens=[37, 20, 37, 9])
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 10, si.first_block(cfg, 4))
    _report(tal, "mid top-8 T=0.8")
    # threshold criterion with argmax draws
    vp2 = VerifyParams(mode=2, delta=0.02, temperature=1.0, sample=0)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp2, 6, si.first_block(cfg, 4))
    _report(tal, "mid threshold")


def test_probability_tree_sampling(X):
    """Top-K_s probability-tree sampling of the head tokens (appendix): K_s = 2 and 3 with the
    paper's cut-off, K_s = 1 (always the most probable path), and a cut-off that removes paths."""
    cfg = _mid_cfg(seed=51)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=[37, 20, 9])
    K = cfg["n_draft"]
    seen = set()
    # random-init heads are nearly uniform over the vocabulary (every path weight ~1e-12), so the
    # temperature is what makes the tree non-trivial: sharp levels, partial cuts, no cuts, all cut
    for ks, prune, T in ((2, 1e-5, 0.02), (3, 1e-5, 0.05), (4, 1e-5, 0.03), (3, 0.0, 0.8), (1, 1e-5, 0.8),
                         (3, 1e-5, 0.8), (3, 1e-2, 0.03)):
        vp = VerifyParams(mode=1, top_ka=8, temperature=T, sample=2, seed=100 + ks, top_ks=ks, pts_prune=prune)
        tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 4, si.first_block(cfg, 3))
        _report(tal, f"PTS K_s={ks} prune={prune} T={T} paths {sorted(set(tal.pts_paths))}")
        for n in tal.pts_paths:
            seen.add("none" if n == 0 else "all" if n == ks ** K else "some")
    assert seen == {"none", "some", "all"}, seen
    buf = eng.buffers(3, spec=True)
    buf.kv_len.fill_(40); buf.block.fill_(1)
    bad = X.xsm.xsm_verify_params(1, 8, 0.5, 0.8, 2, 1, 5, 1e-5)
    with pytest.raises(X.xsm.XsmError, match="top_ks"):
        eng.xsm_spec_step(buf, bad, 40)


@pytest.mark.parametrize("V", [1024, 2048, 8192])
def test_sampling_rules_on_register_resident_rows(X, V):
    """Vocabularies of 1024, 2048 and 8192 (4096 is the latency model's): the accept checks, the
    categorical draw and the tree levels then hold a logits row in registers (thread t owns
    V / 256 consecutive tokens) instead of walking it in memory; every rule once at each size."""
    cfg = _mid_cfg(vocab=V, n_layers=2, seed=60 + V // 1024)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, prefix_lens=[37, 12])
    # (a draw is a near-tie when its uniform lies within 2e-5 of a CDF edge: with V nearly equal
    # weights that is 4e-5 V of all draws, so the larger vocabularies draw at a lower temperature)
    T = 0.8 if V <= 2048 else 0.1
    for name, vp in (("top-8 categorical", VerifyParams(mode=1, top_ka=8, temperature=T, sample=1, seed=V + 1)),
                     ("threshold", VerifyParams(mode=2, delta=1.5 / V, temperature=1.0 if V <= 2048 else 0.25, sample=1, seed=V + 2)),
                     ("tree K_s=3", VerifyParams(mode=1, top_ka=8, temperature=0.04, sample=2, seed=V + 3, top_ks=3))):
        tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 4, si.first_block(cfg, 2))
        _report(tal, f"V={V} {name}")


def test_plain_step_matches_oracle(X):
    cfg = _mid_cfg(seed=23, vocab=1000)        # vocabulary not a multiple of 16: general-shape kernels
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 8, si.first_block(cfg, 2), plain=True)
    _report(tal, "mid plain")


def test_cross_attention_backbone(X):
    cfg = _mid_cfg(n_cond=50, prefix=0, seed=24, n_layers=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 8, si.first_block(cfg, 2))
    _report(tal, "cross-attn")
    cfg = _mid_cfg(n_cond=19, prefix=21, seed=25, n_layers=2, dtype="f32", d_model=128, head_dim=32, d_ffn=256)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 6, si.first_block(cfg, 1))
    _report(tal, "cross-attn f32")
    assert tal.max_rel < 1e-5
    # a prefix as well: the prefill pass runs the 64-row attention kernel over the cached prefix rows
    # (causal) and over the condition tokens (all visible), here with a ragged last tile
    cfg = _mid_cfg(n_cond=70, prefix=85, seed=29, n_layers=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, prefix_lens=[85, 40])
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 2))
    _report(tal, "cross-attn with prefixes 85 / 40")
    # prefill passes of a few hundred and of several thousand rows: the self- and cross-attention
    # outputs reach their O-projections as operand planes (contraction in slices / whole)
    cfg = _c1_small(n_layers=2, n_cond=40, prefix=300, seed=30, max_ctx=384)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 2, si.first_block(cfg, 1))
    _report(tal, "cross-attn d1024, prefix 300")
    cfg = _mid_cfg(n_cond=70, prefix=2700, seed=31, n_layers=2, max_ctx=2752)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 2, si.first_block(cfg, 3))
    _report(tal, "cross-attn, one 8100-row prefill pass")


def test_cross_attention_decoding_heads(X):
    """Eq. 4 with cross-attention heads and per-head unembeddings (Table 3 rows D/E): fp32 general
    kernels, bf16 MFMA kernels at a small batch, and a batch large enough for the
    split-contraction GEMMs; condition length not a multiple of the 64-key chunk."""
    cfg = _mid_cfg(n_cond=19, prefix=9, seed=31, n_layers=2, dtype="f32", d_model=128, head_dim=32, d_ffn=256,
                   head_kind="ca", n_draft=3)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 6, si.first_block(cfg, 2))
    _report(tal, "CA heads f32")
    assert tal.max_rel < 1e-5
    cfg = _mid_cfg(n_cond=150, prefix=0, seed=32, n_layers=2, head_kind="ca")
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3)
    K = cfg["n_draft"]

    def forced(step, b, st, blk):
        full = X.H.true_continuation(orc, st, blk[0], K, GREEDY)
        j = (step + b) % (K + 1)
        if j < K:
            full[j + 1] = (full[j + 1] + 1) % cfg["vocab"]
        return full

    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, K + 2, si.first_block(cfg, 3), forced=forced)
    _report(tal, "CA heads bf16 B3")
    assert set(tal.accept_hist) == set(range(1, K + 2))
    top8 = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=77)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, top8, 4, si.first_block(cfg, 3))
    _report(tal, "CA heads bf16 top-8 categorical")
    cfg = _mid_cfg(n_cond=130, prefix=5, seed=33, n_layers=1, d_model=512, n_heads=8, d_ffn=1024, vocab=1024,
                   head_kind="ca", n_draft=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 20)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 3, si.first_block(cfg, 20))
    _report(tal, "CA heads bf16 B20")


def test_prefill_in_large_chunks(X):
    """Prefill on the MFMA path runs up to 8192 rows per pass (many 16-row query tiles per sequence,
    causal inside the chunk, the row-blocked GEMMs with a ragged last block): one sequence with a
    300-token prefix in one pass, a ragged batch, and three sequences of 900 tokens, in one pass of
    2700 rows and, with the pass size limited to 2048 rows, in two passes (672 + 228 rows each); the
    cache must match the oracle's and the steps after it too."""
    cfg = _mid_cfg(prefix=300, seed=41, n_layers=2, max_ctx=512)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1)
    for l in range(cfg["n_layers"]):
        for which, ref in ((0, states[0].k[l]), (1, states[0].v[l])):
            got = eng.xsm_debug_kv_export(l, which, 0, 0, 300)          # [H][pos][hd]
            want = np.transpose(np.asarray(ref[:300], np.float64), (1, 0, 2))
            err = np.abs(got - want).max() / np.abs(want).max()
            assert err < 1e-2, (l, which, err)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 1))
    _report(tal, "prefix 300 B1")
    cfg = _mid_cfg(prefix=150, seed=42, n_layers=2, max_ctx=512)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=[150, 97, 16])
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 3))
    _report(tal, "prefix 150/97/16 B3")
    cfg = _mid_cfg(prefix=900, seed=43, n_layers=2, max_ctx=1024)
    for pass_rows in (0, 2048):
        w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, options=[(X.xsm.XSM_OPT_PREFILL_ROWS, pass_rows)])
        for b in (0, 2):
            for which, ref in ((0, states[b].k[1]), (1, states[b].v[1])):
                got = eng.xsm_debug_kv_export(1, which, b, 0, 900)
                want = np.transpose(np.asarray(ref[:900], np.float64), (1, 0, 2))
                err = np.abs(got - want).max() / np.abs(want).max()
                assert err < 1e-2, (pass_rows, b, which, err)
        tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 3, si.first_block(cfg, 3))
        _report(tal, f"prefix 900 B3 (pass limit {pass_rows})")


def test_prefill_pass_with_operand_planes_end_to_end(X):
    """A 2048-row pass at d = 1024 (the same chain serves passes of up to 8192 rows): the residual-add projections have enough blocks for the
    row-blocked kernel, so attention and the FFN-up epilogue hand them bf16 hi/lo operand planes
    instead of fp32 rows.  Second-layer cache and the steps after it against the oracle."""
    cfg = _c1_small(n_layers=2, prefix=2048, max_ctx=2112)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1)
    for which, ref in ((0, states[0].k[1]), (1, states[0].v[1])):
        got = eng.xsm_debug_kv_export(1, which, 0, 0, 2048)
        want = np.transpose(np.asarray(ref[:2048], np.float64), (1, 0, 2))
        err = np.abs(got - want).max() / np.abs(want).max()
        assert err < 1e-2, (which, err)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 2, si.first_block(cfg, 1))
    _report(tal, "prefix 2048 B1 d1024 (operand planes)")


def test_rows_name_their_cache_slot(X):
    """A batch row carries the index of its cache slot: rows in an order that is not the slot
    order, with one slot left out, against the oracle states of those sequences; on the per-stage
    kernels and on the single-launch kernel.  The oracle's Philox counter carries the sequence id,
    the library's the slot, so the states keep seq_id = slot."""
    vp = VerifyParams(mode=1, top_ka=4, temperature=0.9, sample=1, seed=99)
    cfg = _mid_cfg(seed=51, n_layers=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 4, prefix_lens=[37, 20, 9, 30])
    order = [2, 0, 3]
    first = si.first_block(cfg, 4)
    tal = X.H.lockstep(cfg, orc, [states[b] for b in order], eng, X.xsm, vp, 5, [first[b] for b in order],
                       slots=order)
    _report(tal, "slots 2,0,3 of 4 (per-stage)")
    cfg = _c1_small(n_layers=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=[70, 33, 5])
    order = [2, 0]
    first = si.first_block(cfg, 3)
    tal = X.H.lockstep(cfg, orc, [states[b] for b in order], eng, X.xsm, GREEDY, 5, [first[b] for b in order],
                       slots=order)
    _report(tal, "slots 2,0 of 3 (single launch)")
    eng.xsm_check_device()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_batcher_admission_and_compaction(X, dtype):
    """Seven requests with different prefix lengths and token budgets through three cache slots:
    sequences are admitted as slots free up and the batch rows are compacted when one finishes.
    Greedy speculative decoding must give every request the tokens of plain greedy decoding of
    that request alone (Sec. 4.2; the oracle's plain loop); at a decision the oracle marks as a
    near-tie it continues from the GPU's token."""
    from paper_2507_23777_amd.batcher import Batcher, Request
    if dtype == "fp32":
        cfg = si.tiny_config(n_layers=2, d_model=64, n_heads=2, head_dim=32, d_ffn=128, vocab=64, n_draft=3,
                             dtype="fp32", max_ctx=160, seed=12)
    else:
        cfg = _mid_cfg(seed=52, n_layers=2, max_ctx=256)
    K = cfg["n_draft"]
    w = si.make_weights(cfg, perturb=True)
    orc = Oracle(cfg, w)
    eng = X.pkg.Engine(cfg, max_batch=3, max_ctx=cfg["max_ctx"])
    eng.xsm_load_weights(si.pack_canonical(cfg, w))
    P = [37, 20, 9, 37, 50, 0, 20]
    budget = [30, 12, 45, 7, 25, 18, 33]
    prefixes = si.make_prefix(cfg, len(P), P=max(P))
    firsts = si.first_block(cfg, len(P))
    # fp32: a look at the outputs after every step; bf16: every fourth step (late EOS / budget)
    bt = Batcher(eng, X.H.to_vp_gpu(X.xsm, GREEDY), spec=True, sync_every=1 if dtype == "fp32" else 4)
    for i in range(len(P)):
        bt.submit(Request(first_block=list(map(int, firsts[i])), max_new_tokens=budget[i],
                          prefix=None if P[i] == 0 else prefixes[i, :P[i]]))
    got = bt.run()
    assert sorted(got) == list(range(len(P)))
    assert sorted(bt.free) == [0, 1, 2] and not bt.live
    assert all(1 <= a <= K + 1 for a in bt.accepted_per_step)
    compared = total = 0
    tie = 1e-4 if dtype == "fp32" else X.H.TIE         # fp32 logits agree to 1e-5 of the row's largest
    for i in range(len(P)):
        assert len(got[i]) == budget[i]
        st = orc.new_state(cap=cfg["max_ctx"], seq_id=0)
        orc.prefill(st, None if P[i] == 0 else prefixes[i, :P[i]], None)
        tok = int(firsts[i][0])
        for j in range(budget[i]):
            r = orc.plain_step(st, tok, GREEDY)
            if r["diag"][0]["margin"] <= tie:          # flagged, not counted: the oracle follows the GPU's choice
                tok = got[i][j]
                continue
            tok = int(r["out_tokens"][0])
            assert got[i][j] == tok, f"request {i} token {j}: gpu {got[i][j]} oracle {tok}"
            compared += 1
        total += budget[i]
    print(f"[batcher {dtype}] {bt.steps} steps for {total} tokens, {compared} compared token for token", flush=True)
    assert compared >= total // 2


def test_cache_contents_and_rollback(X):
    cfg = _mid_cfg(seed=26, n_layers=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 5, si.first_block(cfg, 2))
    _report(tal, "rollback warm-up")
    for b, st in enumerate(states):
        for l in range(cfg["n_layers"]):
            for which, ref in ((0, st.k[l]), (1, st.v[l])):
                got = eng.xsm_debug_kv_export(l, which, b, 0, st.n)            # [H][n][hd]
                want = np.transpose(ref[:st.n], (1, 0, 2))
                err = np.abs(got - want).max() / np.abs(want).max()
                assert err < 1e-2, (b, l, which, err)
    # stale slots beyond the accepted length are garbage by contract: poison them with NaN
    for b, st in enumerate(states):
        for l in range(cfg["n_layers"]):
            nan = np.full((cfg["n_heads"], 8, cfg["head_dim"]), np.nan, np.float32)
            # rows n .. n+K are rewritten by the next step; poison the ones after them too
            eng.xsm_debug_kv_import(l, 0, b, st.n, nan)
            eng.xsm_debug_kv_import(l, 1, b, st.n, nan)
    blocks = [[1, 2, 3, 4, 5], [5, 4, 3, 2, 1]]
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 3, blocks)
    _report(tal, "after NaN poisoning")


def test_long_context_synthetic_cache(X):
    cfg = _mid_cfg(seed=27, n_layers=2, max_ctx=8192 + 64, prefix=0)
    n_pos = 8192
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, max_ctx=cfg["max_ctx"], kv_dtype=np.float32)
    fill = si.make_kv_fill(cfg, 2, n_pos)
    fill[:, 0] = si.bf16_round(fill[:, 0] * 6.0)        # sharper scores: a few hundred keys carry the weight
    lens = [n_pos, n_pos - 1237]
    for b, st in enumerate(states):
        for l in range(cfg["n_layers"]):
            st.k[l][:lens[b]] = np.transpose(fill[l, 0, b, :, :lens[b]], (1, 0, 2))
            st.v[l][:lens[b]] = np.transpose(fill[l, 1, b, :, :lens[b]], (1, 0, 2))
            eng.xsm_debug_kv_import(l, 0, b, 0, fill[l, 0, b, :, :lens[b]])
            eng.xsm_debug_kv_import(l, 1, b, 0, fill[l, 1, b, :, :lens[b]])
        st.n = lens[b]
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 3, si.first_block(cfg, 2))
    _report(tal, "ctx 8192")


def test_config1_shape_bf16(X):
    cfg = si.get_config("c1")
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, perturb=False, max_ctx=512)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 6, si.first_block(cfg, 1))
    _report(tal, "c1 lockstep")


def test_large_batch_row_blocked_gemm(X):
    """M = 200 block rows and 40 head rows: the row-blocked MFMA GEMM (all epilogues), ragged lengths."""
    cfg = _mid_cfg(seed=29, vocab=1024, n_layers=2)
    lens = [37 - (b % 9) * 3 for b in range(40)]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 40, prefix_lens=lens)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 3, si.first_block(cfg, 40))
    _report(tal, "B40 row-blocked")
    vp = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=77)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 2, si.first_block(cfg, 40))
    _report(tal, "B40 row-blocked top-8")


def _c1_small(**kw):
    """The latency model's shape (d=1024, FFN 4096, 16 heads, vocab 4096) with few layers: the
    shape the single-launch step kernel is built for."""
    cfg = si.get_config("c1", n_layers=3, max_ctx=1536, prefix=70)
    cfg.update(kw)
    return cfg


def test_mid_batch_few_rows_on_the_wide_model(X):
    """M = 35 block rows (7 sequences, K = 4) and 28 head rows at d = 1024: the mid-batch kernels'
    variant for up to 64 rows (QKV, GELU, unembedding and head epilogues), ragged lengths, and a
    46-row batch with top-8 acceptance and categorical draws."""
    cfg = _c1_small(n_layers=2)
    lens = [70, 33, 5, 64, 17, 48, 21]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 7, prefix_lens=lens)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 3, si.first_block(cfg, 7))
    _report(tal, "B7 d1024")
    cfg = _c1_small(n_layers=2, n_draft=1)
    lens = [5 + 3 * b for b in range(23)]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 23, prefix_lens=lens)
    vp = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=78)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 2, si.first_block(cfg, 23))
    _report(tal, "B23 K1 d1024 top-8")


@pytest.mark.parametrize("single_launch", [1, 0])
def test_single_launch_step_matches_oracle_and_per_stage_kernels(X, single_launch):
    cfg = _c1_small()
    K = cfg["n_draft"]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 3, prefix_lens=[70, 33, 5], perturb=True)
    eng.xsm_set_option(X.xsm.XSM_OPT_SINGLE_LAUNCH, single_launch)

    def forced(step, b, st, blk):
        if step < 2:
            return blk
        full = X.H.true_continuation(orc, st, blk[0], K, GREEDY)
        j = (step + b) % (K + 1)
        if j < K:
            full[j + 1] = (full[j + 1] + 1) % cfg["vocab"]
        return full

    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 2 + K + 1, si.first_block(cfg, 3), forced=forced)
    _report(tal, f"c1-shape B3 single_launch={single_launch}")
    assert set(tal.accept_hist) == set(range(1, K + 2))
    eng.xsm_check_device()
    # plain next-token steps through the same kernel
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 3), plain=True)
    _report(tal, f"c1-shape plain single_launch={single_launch}")
    eng.xsm_check_device()


@pytest.mark.parametrize("K,V", [(2, 4096), (4, 4096), (4, 2048)])
def test_single_launch_one_sequence_compile_time_shapes(X, K, V):
    """One sequence with K = 2 and K = 4 heads, and plain next-token steps of one sequence: the
    single-launch kernel has an instantiation of its own for each of these shapes (rows per
    sequence and batch as compile-time constants; K = 8 is covered by the eight-heads case), and
    for K = 4 one with the latency model's vocabulary as a constant and one without."""
    cfg = _c1_small(n_layers=2, n_draft=K, vocab=V)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, perturb=True)
    X.xsm.xsm_debug_trace_enable(True); X.xsm.xsm_debug_trace_report()
    vp = VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=77 + K)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 1))
    _report(tal, f"c1-shape B1 K{K} V{V} greedy")
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 4, si.first_block(cfg, 1))
    _report(tal, f"c1-shape B1 K{K} V{V} top-8 categorical")
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 1), plain=True)
    _report(tal, f"c1-shape B1 plain (model with K={K})")
    ran = X.xsm.xsm_debug_trace_report(); X.xsm.xsm_debug_trace_enable(False)
    assert ran["step_small"][0] == 12, sorted(ran)
    eng.xsm_check_device()


def test_single_launch_eight_draft_heads(X):
    """K = 8 at batch 1: 9 backbone rows + 72 head rows in the persistent kernel (several row
    tiles in the unembedding), every acceptance length forced once."""
    cfg = _c1_small(n_layers=2, n_draft=8)
    K = cfg["n_draft"]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, perturb=True)

    def forced(step, b, st, blk):
        full = X.H.true_continuation(orc, st, blk[0], K, GREEDY)
        j = step % (K + 1)
        if j < K:
            full[j + 1] = (full[j + 1] + 1) % cfg["vocab"]
        return full

    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, K + 1, si.first_block(cfg, 1), forced=forced)
    _report(tal, "c1-shape B1 K8 single launch")
    assert set(tal.accept_hist) == set(range(1, K + 2))
    eng.xsm_check_device()


@pytest.mark.parametrize("single_launch", [1, 0])
def test_single_launch_with_sampling_rules(X, single_launch):
    """Top-K_a acceptance with categorical draws, the probability threshold, and probability-tree
    draws at a batch small enough for the persistent kernel, which runs the accept checks and the
    draws as per-row tasks on its own workgroups (single_launch=0: the verify / emit kernels)."""
    cfg = _c1_small(n_layers=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, prefix_lens=[70, 21], perturb=True)
    eng.xsm_set_option(X.xsm.XSM_OPT_SINGLE_LAUNCH, single_launch)
    for name, vp in (("top-8 categorical", VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=7)),
                     ("threshold", VerifyParams(mode=2, delta=0.0004, temperature=1.0, sample=1, seed=8)),
                     ("tree K_s=3", VerifyParams(mode=1, top_ka=8, temperature=0.04, sample=2, seed=9, top_ks=3))):
        tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 4, si.first_block(cfg, 2))
        _report(tal, f"c1-shape {name} single_launch={single_launch}")
    eng.xsm_check_device()


def test_single_launch_long_context_split_keys(X):
    cfg = _c1_small(n_layers=2, max_ctx=4608, prefix=0)
    n_pos = 4352
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, max_ctx=cfg["max_ctx"], kv_dtype=np.float32)
    fill = si.make_kv_fill(cfg, 1, n_pos)
    fill[:, 0] = si.bf16_round(fill[:, 0] * 6.0)
    for l in range(cfg["n_layers"]):
        states[0].k[l][:n_pos] = np.transpose(fill[l, 0, 0], (1, 0, 2))
        states[0].v[l][:n_pos] = np.transpose(fill[l, 1, 0], (1, 0, 2))
        eng.xsm_debug_kv_import(l, 0, 0, 0, fill[l, 0, 0])
        eng.xsm_debug_kv_import(l, 1, 0, 0, fill[l, 1, 0])
    states[0].n = n_pos - 30          # ragged tail inside a 64-key chunk, 16 key slices
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 4, si.first_block(cfg, 1))
    _report(tal, "single-launch ctx 4.3k")
    eng.xsm_check_device()


@pytest.mark.parametrize("rule", ["greedy", "sampled"])
def test_single_launch_timeout_is_reported_in_band_and_falls_back(X, rule):
    """The failure path of the single-launch step, forced from the host (the device-side error word
    is set as a timed-out wait would set it; no wait is made to spin and every kernel exits
    normally): the step's own outputs must say that nothing was produced, xsm_check_device must
    report it once, and the following steps must run on the per-stage kernels and match the
    oracle.  Both with the greedy last stage and with the per-row check and draw tasks."""
    cfg = _c1_small(n_layers=2)
    torch = X.torch
    vp = GREEDY if rule == "greedy" else VerifyParams(mode=1, top_ka=8, temperature=0.8, sample=1, seed=17)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, prefix_lens=[70, 21], perturb=True)
    first = si.first_block(cfg, 2)
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 2, first)
    _report(tal, f"before the injected timeout ({rule})")
    eng.xsm_check_device()
    vpg = X.H.to_vp_gpu(X.xsm, vp)
    buf = eng.buffers(2, spec=True)
    lens = [st.n for st in states]
    buf.kv_len.copy_(torch.tensor(lens, dtype=torch.int32)); buf.block.copy_(torch.tensor(first))
    buf.n_accepted.fill_(3); buf.out_tokens.fill_(-7)
    eng.xsm_debug_inject_device_error(77)
    for _ in range(2):                               # the failing step and one enqueued behind it
        eng.xsm_spec_step(buf, vpg, max(lens))
    torch.cuda.synchronize()
    assert buf.n_accepted.tolist() == [0, 0]
    assert all(int(f) & X.xsm.XSM_FLAG_DEVICE_TIMEOUT for f in buf.flags.tolist())
    assert buf.kv_len.tolist() == lens and buf.block.tolist() == first.tolist()
    assert (buf.out_tokens == -7).all()
    with pytest.raises(X.xsm.XsmError, match="timed out"):
        eng.xsm_check_device()
    eng.xsm_check_device()                           # reported once
    X.xsm.xsm_debug_trace_enable(True); X.xsm.xsm_debug_trace_report()
    tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, vp, 3, first)
    ran = X.xsm.xsm_debug_trace_report(); X.xsm.xsm_debug_trace_enable(False)
    _report(tal, f"after the injected timeout: per-stage kernels ({rule})")
    assert "step_small" not in ran and "fattn" in ran, sorted(ran)
    eng.xsm_check_device()


def test_single_launch_free_running_equals_per_stage(X):
    """Same engine, same start: the persistent kernel and the per-stage kernels must emit the
    same tokens step for step (both are fixed-order reductions over identical bf16 operands).
    The two may part only at a step that one of them flagged as a near-tie; the comparison stops
    there, and at least ten steps must have been compared before it."""
    cfg = _c1_small()
    torch = X.torch
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 1, perturb=False)
    vpg = X.H.to_vp_gpu(X.xsm, GREEDY)
    outs = []
    for mode in (1, 0):
        eng.xsm_set_option(X.xsm.XSM_OPT_SINGLE_LAUNCH, mode)
        buf = eng.buffers(1, spec=True)
        buf.kv_len.fill_(cfg["prefix"]); buf.block.copy_(torch.tensor(si.first_block(cfg, 1)))
        steps = []
        for i in range(40):
            eng.xsm_spec_step(buf, vpg, cfg["prefix"] + 5 * i)
            torch.cuda.synchronize()
            n = int(buf.n_accepted[0]); assert 1 <= n <= cfg["n_draft"] + 1
            steps.append((buf.out_tokens[0, :n].tolist(), buf.block[0].tolist(), int(buf.flags[0]) & 1))
        outs.append(steps)
    eng.xsm_check_device()
    same = 0
    for (ta, ba, fa), (tb, bb, fb) in zip(*outs):
        if (ta, ba) != (tb, bb):
            assert fa or fb, f"step {same}: single launch {ta} {ba}, per-stage {tb} {bb}, no near-tie flagged"
            break
        same += 1
    print(f"[single vs per-stage] {same} of 40 steps identical before the first flagged divergence", flush=True)
    X.H.SUMMARY.append(f"[single vs per-stage free-running] {same} of 40 steps identical")
    assert same >= 10


@pytest.mark.parametrize("rule", ["greedy", "tree"])
def test_single_launch_same_step_for_300_epochs(X, rule):
    """The exchange words' 8-bit tag wraps every 255 steps, and the step that starts a new cycle
    scrubs the exchange region first: the same step (same lengths, same block, same seed) repeated
    300 times must give the same tokens and bit-identical logits every time, before, at and after
    the wrap, and the per-stage kernels' tokens."""
    cfg = _c1_small(n_layers=2)
    torch = X.torch
    vp = GREEDY if rule == "greedy" else VerifyParams(mode=1, top_ka=8, temperature=0.5, sample=2, seed=31, top_ks=2)
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, prefix_lens=[70, 21], perturb=True)
    vpg = X.H.to_vp_gpu(X.xsm, vp)
    first = torch.tensor(si.first_block(cfg, 2))
    lens = torch.tensor([70, 21], dtype=torch.int32)
    buf = eng.buffers(2, spec=True, debug=True)

    def step():
        buf.kv_len.copy_(lens); buf.block.copy_(first)
        eng.xsm_spec_step(buf, vpg, 70)
        torch.cuda.synchronize()
        return (buf.n_accepted.tolist(), buf.out_tokens.tolist(), buf.block.tolist(), buf.flags.tolist())

    X.xsm.xsm_debug_trace_enable(True); X.xsm.xsm_debug_trace_report()
    ref = step()
    z_ref = buf.logits.clone()
    for i in range(1, 300):
        got = step()
        assert got == ref, f"step {i}: {got} vs {ref}"
        if i in (254, 255, 256, 299):
            assert torch.equal(buf.logits, z_ref), f"step {i}: logits differ from the first step's"
    ran = X.xsm.xsm_debug_trace_report(); X.xsm.xsm_debug_trace_enable(False)
    assert ran["step_small"][0] == 300, sorted(ran)
    eng.xsm_check_device()
    eng.xsm_set_option(X.xsm.XSM_OPT_SINGLE_LAUNCH, 0)
    per_stage = step()
    assert per_stage[:3] == ref[:3] or (per_stage[3][0] | per_stage[3][1] | ref[3][0] | ref[3][1]) & 1
    eng.xsm_check_device()


@pytest.mark.parametrize("path", ["single_launch", "per_stage_sampling"])
def test_step_replayed_from_a_captured_graph(X, path):
    """A step enqueues kernels only (no allocation, copy, memset or synchronisation) and keeps its
    epoch and lengths on the device, so a caller may capture it in a HIP graph: six replays, with
    eager work and synchronisation between them, must reproduce six eager steps from the same start."""
    torch = X.torch
    if path == "single_launch":
        cfg, vp, n_seq, lens = _c1_small(n_layers=2), GREEDY, 2, [70, 21]
    else:
        cfg, vp, n_seq, lens = _mid_cfg(seed=61, n_layers=2), VerifyParams(mode=1, top_ka=4, temperature=0.9, sample=1, seed=5), 3, [37, 20, 9]
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, n_seq, prefix_lens=lens)
    vpg = X.H.to_vp_gpu(X.xsm, vp)
    buf = eng.buffers(n_seq, spec=True)
    first = torch.tensor(si.first_block(cfg, n_seq))
    start_len = torch.tensor(lens, dtype=torch.int32)
    bound = max(lens) + 6 * (cfg["n_draft"] + 1)

    def reset():
        buf.kv_len.copy_(start_len); buf.block.copy_(first)

    def snapshot():
        torch.cuda.synchronize()
        return [t.cpu().clone() for t in (buf.n_accepted, buf.out_tokens, buf.block, buf.kv_len, buf.flags)]

    reset()
    eager = []
    for _ in range(6):
        eng.xsm_spec_step(buf, vpg, bound)
        eager.append(snapshot())
    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            eng.xsm_spec_step(buf, vpg, bound)
    torch.cuda.current_stream().wait_stream(side)
    reset()                                   # (capture enqueues nothing, the state is still the start state)
    scratch = torch.zeros(1 << 16, device=eng.device)
    for i in range(6):
        graph.replay()
        got = snapshot()
        for a, b, name in zip(got, eager[i], ("n_accepted", "out_tokens", "block", "kv_len", "flags")):
            if name == "out_tokens":          # only the first n_accepted entries are defined
                for r in range(n_seq):
                    k = int(got[0][r])
                    assert torch.equal(a[r, :k], b[r, :k]), (i, name, r)
            else:
                assert torch.equal(a, b), (i, name)
        scratch.add_(1.0)                     # the program's own eager work between replays
        torch.cuda.synchronize()
    eng.xsm_check_device()


def test_model_without_draft_heads(X):
    """Degenerate case K = 0: no decoding heads, only next-token decoding exists (both dtypes'
    kernels); a speculative step is refused."""
    for cfg in (si.tiny_config(n_layers=2, d_model=64, n_heads=2, head_dim=32, d_ffn=128, vocab=64, n_draft=0,
                               dtype="fp32", max_ctx=96, seed=13),
                _mid_cfg(seed=53, n_layers=2, n_draft=0)):
        w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2, prefix_lens=[9, 4])
        tal = X.H.lockstep(cfg, orc, states, eng, X.xsm, GREEDY, 5, [[1], [2]], plain=True)
        _report(tal, f"K=0 plain {cfg['dtype']}")
        with pytest.raises(X.xsm.XsmError, match="n_draft"):
            eng.xsm_spec_step(eng.buffers(2, spec=False), X.H.to_vp_gpu(X.xsm, GREEDY), 32)


def test_argument_and_device_side_errors(X):
    cfg = _mid_cfg(seed=28, n_layers=1)
    torch = X.torch
    w, orc, states, eng = X.H.setup_pair(cfg, X.pkg.Engine, 2)
    vpg = X.H.to_vp_gpu(X.xsm, GREEDY)
    buf = eng.buffers(2, spec=True)
    buf.kv_len.fill_(cfg["prefix"]); buf.block.fill_(3)
    with pytest.raises(X.xsm.XsmError, match="max_ctx"):
        eng.xsm_spec_step(buf, vpg, cfg["max_ctx"] - 2)
    big = eng.buffers(3, spec=True)
    with pytest.raises(X.xsm.XsmError, match="max_batch"):
        eng.xsm_spec_step(big, vpg, 10)
    bad = X.xsm.xsm_verify_params(1, 0, 0.5, 1.0, 0, 0)
    with pytest.raises(X.xsm.XsmError, match="top_ka"):
        eng.xsm_spec_step(buf, bad, 100)
    empty = eng.buffers(2, spec=True)
    empty.n_seq = 0                                   # an empty batch is an argument error, nothing is enqueued
    with pytest.raises(X.xsm.XsmError):
        eng.xsm_spec_step(empty, vpg, 100)
    # device-side: sequence 0 has a token outside the vocabulary, sequence 1 is fine
    buf.block[0, 2] = cfg["vocab"] + 5
    eng.xsm_spec_step(buf, vpg, cfg["prefix"])
    torch.cuda.synchronize()
    assert int(buf.n_accepted[0]) == 0 and int(buf.flags[0]) & 4
    assert 1 <= int(buf.n_accepted[1]) <= cfg["n_draft"] + 1 and (int(buf.flags[1]) & ~1) == 0
    assert int(buf.kv_len[0]) == cfg["prefix"]
    # a length beyond the caller's bound is skipped, not run
    buf.block.fill_(3); buf.kv_len[0] = cfg["prefix"] + 50
    eng.xsm_spec_step(buf, vpg, cfg["prefix"] + 10)
    torch.cuda.synchronize()
    assert int(buf.n_accepted[0]) == 0 and int(buf.flags[0]) & 2
