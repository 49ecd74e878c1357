"""Invariants the paper fixes for the speculative step, checked on the oracle.

Greedy verification (top-K_a with K_a = 1, Sec. 5.4) must reproduce plain
greedy next-token decoding token for token; every step accepts between 1 and
K+1 tokens (Alg. 1 inner loop bounds); the cache after a step is exactly the
cache of the accepted tokens; logits at a block row do not depend on later
candidates (Sec. 3.1, Eq. 1)."""
import copy

import numpy as np
import pytest
from scipy import stats

import synth_inputs as si
from oracle import Oracle, VerifyParams, accept, rank_of, sample, softmax

GREEDY = VerifyParams(mode=0, sample=0)


def _setup(cfg, perturb=True, cap=None):
    w = si.make_weights(cfg, perturb=perturb)
    orc = Oracle(cfg, w)
    st = orc.new_state(cap=cap or cfg["max_ctx"])
    cond = si.make_cond(cfg, 1)
    orc.prefill(st, si.make_prefix(cfg, 1)[0], None if cond is None else cond[0])
    return orc, st


@pytest.mark.parametrize("K", [1, 2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("seed", [7, 8])
def test_greedy_spec_equals_plain_greedy_tiny(K, seed):
    cfg = si.tiny_config(n_draft=K, seed=seed)
    orc, st = _setup(cfg)
    st2 = copy.deepcopy(st)
    blk = si.first_block(cfg, 1)[0]
    spec, steps, hist = orc.generate_spec(st, blk, 40, GREEDY)
    plain = orc.generate_plain(st2, blk[0], 40, GREEDY)
    assert spec == plain
    assert all(1 <= a <= K + 1 for a in hist)
    assert 1.0 <= sum(hist) / steps <= K + 1


def test_greedy_spec_equals_plain_greedy_config0():
    cfg = si.get_config("c0")
    orc, st = _setup(cfg, perturb=False)
    st2 = copy.deepcopy(st)
    blk = si.first_block(cfg, 1)[0]
    spec, steps, hist = orc.generate_spec(st, blk, 512, GREEDY)
    plain = orc.generate_plain(st2, blk[0], 512, GREEDY)
    assert spec == plain
    assert all(1 <= a <= cfg["n_draft"] + 1 for a in hist)
    # the identity-plus-noise heads repeat the backbone's token, so some drafts do get accepted
    assert len(set(hist)) > 1


def test_rollback_restores_exact_cache_and_ignores_stale_slots():
    cfg = si.tiny_config(n_draft=4)
    orc, st = _setup(cfg)
    st_plain = copy.deepcopy(st)
    st_poison = copy.deepcopy(st)
    blk = list(si.first_block(cfg, 1)[0])
    blk_p = list(blk)
    toks = [blk[0]]
    for _ in range(12):
        r = orc.spec_step(st, blk, GREEDY)
        # same step on a state whose slots >= n were overwritten with NaN beforehand
        for l in range(orc.L):
            st_poison.k[l][st_poison.n:] = np.nan
            st_poison.v[l][st_poison.n:] = np.nan
        rp = orc.spec_step(st_poison, blk_p, GREEDY)
        assert rp["out_tokens"] == r["out_tokens"] and rp["next_block"] == r["next_block"]
        np.testing.assert_array_equal(rp["Z0"], r["Z0"])
        toks += r["out_tokens"]
        blk, blk_p = r["next_block"], rp["next_block"]
    # cache built by next-token stepping over the same accepted tokens
    for t in toks[:-1]:
        orc.forward_block(st_plain, orc.w["E"][[t]])
        st_plain.n += 1
    assert st_plain.n == st.n
    for l in range(orc.L):
        np.testing.assert_allclose(st.k[l][:st.n], st_plain.k[l][:st.n], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(st.v[l][:st.n], st_plain.v[l][:st.n], rtol=1e-12, atol=1e-14)


def test_block_causality():
    cfg = si.tiny_config(n_draft=5)
    orc, st = _setup(cfg)
    blk = np.array([3, 1, 4, 1, 5, 9])
    _, Z = orc.forward_block(copy.deepcopy(st), orc.w["E"][blk])
    for j in range(5):
        alt = blk.copy()
        alt[j + 1:] = (alt[j + 1:] + 7) % cfg["vocab"]
        _, Z2 = orc.forward_block(copy.deepcopy(st), orc.w["E"][alt])
        np.testing.assert_allclose(Z2[:j + 1], Z[:j + 1], rtol=1e-12, atol=1e-14)
        assert np.abs(Z2[j + 1:] - Z[j + 1:]).max() > 1e-9


def test_forced_drafts_hit_every_accept_length():
    cfg = si.tiny_config(n_draft=4)
    K = 4
    orc, st = _setup(cfg)
    first = int(si.first_block(cfg, 1)[0][0])
    truth = orc.generate_plain(copy.deepcopy(st), first, K + 1, GREEDY)
    full = [first] + truth[:K]
    r = orc.spec_step(copy.deepcopy(st), full, GREEDY)
    assert r["n_accepted"] == K + 1 and r["out_tokens"] == truth[:K + 1]
    for j in range(1, K + 1):                       # corrupt candidate j only
        blk = list(full)
        blk[j] = (blk[j] + 1) % cfg["vocab"]
        r = orc.spec_step(copy.deepcopy(st), blk, GREEDY)
        assert r["a"] == j - 1
        assert r["out_tokens"] == truth[:j]         # accepted prefix + resampled true token


def test_top_ka_full_vocab_accepts_everything_and_heads_on_all_rows_agree():
    cfg = si.tiny_config(n_draft=4)
    orc, st = _setup(cfg)
    vp = VerifyParams(mode=1, top_ka=cfg["vocab"], sample=0)
    blk = list(si.first_block(cfg, 1)[0])
    for _ in range(5):
        ra = orc.spec_step(copy.deepcopy(st), blk, vp, heads_on_all_rows=True)
        r = orc.spec_step(st, blk, vp)
        assert r["n_accepted"] == cfg["n_draft"] + 1
        assert r["next_block"] == ra["next_block"]
        np.testing.assert_allclose(r["Zh"], ra["Zh"], rtol=1e-12)
        blk = r["next_block"]


def test_threshold_mode():
    cfg = si.tiny_config(n_draft=3)
    orc, st = _setup(cfg)
    blk = si.first_block(cfg, 1)[0]
    plain = orc.generate_plain(copy.deepcopy(st), blk[0], 30, GREEDY)
    # p > 0.5 makes the token the unique argmax, so argmax resampling equals plain greedy
    for delta in (0.5, 0.8):
        spec, _, _ = orc.generate_spec(copy.deepcopy(st), blk, 30, VerifyParams(mode=2, delta=delta, sample=0))
        assert spec == plain
    # delta > 1 never accepts; positions key the RNG, so sampled output equals plain sampling
    vp = VerifyParams(mode=2, delta=1.5, temperature=0.8, sample=1, seed=99)
    spec, steps, hist = orc.generate_spec(copy.deepcopy(st), blk, 30, vp)
    assert hist == [1] * steps
    assert spec == orc.generate_plain(copy.deepcopy(st), blk[0], 30, vp)
    # strictness: probability exactly delta is rejected
    z = np.log(np.array([0.5, 0.25, 0.25]))
    assert not accept(z, 0, VerifyParams(mode=2, delta=0.5))
    assert accept(z, 0, VerifyParams(mode=2, delta=0.49))


def test_rank_and_accept_on_hand_made_rows():
    z = np.array([0.1, 2.0, 2.0, -1.0, 0.5])
    assert [rank_of(z, i) for i in range(5)] == [3, 0, 1, 4, 2]       # equal logits: lower index first
    assert accept(z, 1, VerifyParams(mode=0)) and not accept(z, 2, VerifyParams(mode=0))
    assert accept(z, 2, VerifyParams(mode=1, top_ka=2)) and not accept(z, 4, VerifyParams(mode=1, top_ka=2))
    assert accept(z, 4, VerifyParams(mode=1, top_ka=3))
    tok, dg = sample(z, VerifyParams(sample=0), 0, 0, 0)
    assert tok == 1 and dg["margin"] == 0.0
    # temperature does not change ranks
    assert rank_of(z / 0.8, 4) == rank_of(z, 4)


def test_categorical_sampler_distribution():
    rng = np.random.default_rng(11)
    z = rng.standard_normal(12) * 2
    vp = VerifyParams(sample=1, temperature=0.8, seed=2024)
    draws = np.array([sample(z, vp, pos, 1, 0)[0] for pos in range(6000)])
    p = softmax(z / 0.8)
    counts = np.bincount(draws, minlength=12)
    keep = p * 6000 >= 5
    chi = stats.chisquare(np.append(counts[keep], counts[~keep].sum()),
                          np.append(p[keep], p[~keep].sum()) * 6000)
    assert chi.pvalue > 1e-3
    # inverse CDF over ascending index: u just below / above a boundary
    z2 = np.log(np.array([0.25, 0.25, 0.5]))
    from oracle import philox
    for pos in range(50):
        u = philox.uniform24(7, pos, 0, 0)
        tok, _ = sample(z2, VerifyParams(sample=1, seed=7), pos, 0, 0)
        assert tok == (0 if u < 0.25 else 1 if u < 0.5 else 2)


@pytest.mark.parametrize("K", [2, 4])
def test_greedy_spec_equals_plain_greedy_with_cross_attention_heads(K):
    """The invariant does not depend on what the heads are (Sec. 4.2): with cross-attention
    heads reading the condition, greedy speculative output is still plain greedy decoding, and
    the heads on all rows vs on the accepted row agree."""
    cfg = si.tiny_config(n_draft=K, n_cond=6, head_kind="ca", seed=21)
    orc, st = _setup(cfg)
    st2, st3 = copy.deepcopy(st), copy.deepcopy(st)
    blk = si.first_block(cfg, 1)[0]
    spec, steps, hist = orc.generate_spec(st, blk, 40, GREEDY)
    plain = orc.generate_plain(st2, blk[0], 40, GREEDY)
    assert spec == plain
    assert all(1 <= a <= K + 1 for a in hist)
    a = orc.spec_step(copy.deepcopy(st3), blk, GREEDY)
    b = orc.spec_step(st3, blk, GREEDY, heads_on_all_rows=True)
    assert a["next_block"] == b["next_block"]
    np.testing.assert_allclose(a["Zh"], b["Zh"], rtol=1e-12, atol=1e-14)


# ---- top-K_s probability-tree sampling (appendix "Sampling strategies") ------------------------
def test_pts_without_pruning_is_the_flattened_outer_product():
    """With no pruning the leaves in depth-first order are the C-order flattening of the outer
    product of the per-level top-K_s probabilities, so the draw must be the searchsorted index of
    u*S in that table (built here with numpy's outer / ravel, not by recursion)."""
    from oracle import pts_sample, PTS_HEAD, uniform24
    rng = np.random.default_rng(3)
    K, V, Ks, T = 3, 11, 3, 0.7
    for trial in range(40):
        Zh = rng.standard_normal((K, V)) * 2.0
        vp = VerifyParams(sample=2, temperature=T, seed=900 + trial, top_ks=Ks, pts_prune=0.0)
        toks, dg = pts_sample(Zh, vp, pos=17 + trial, seq_id=trial % 3)
        P = [softmax(Zh[d] / T) for d in range(K)]
        order = [sorted(range(V), key=lambda v: (-P[d][v], v))[:Ks] for d in range(K)]
        table = np.array([1.0])
        for d in range(K):
            table = np.outer(table, P[d][order[d]]).ravel()
        cdf = np.cumsum(table)
        u = uniform24(vp.seed, 17 + trial, PTS_HEAD, trial % 3)
        idx = int(np.searchsorted(cdf, u * cdf[-1], side="right"))
        digits = np.unravel_index(idx, (Ks,) * K)
        assert toks == [order[d][digits[d]] for d in range(K)]
        assert dg["n_paths"] == Ks ** K


def test_pts_special_cases_and_pruning():
    from oracle import pts_sample
    rng = np.random.default_rng(5)
    Zh = rng.standard_normal((4, 9))
    # K_s = 1: the path of the most probable tokens, whatever the uniform
    for seed in range(5):
        toks, _ = pts_sample(Zh, VerifyParams(sample=2, seed=seed, top_ks=1, pts_prune=0.0), 3, 0)
        assert toks == [int(np.argmax(z)) for z in Zh]
    # nothing survives: same fallback
    toks, dg = pts_sample(Zh, VerifyParams(sample=2, seed=1, top_ks=3, pts_prune=2.0), 3, 0)
    assert toks == [int(np.argmax(z)) for z in Zh] and dg["n_paths"] == 0
    # hand-made tree: level probabilities (0.9, 0.1) and (0.8, 0.2); threshold 0.05 cuts only the
    # path 0.1*0.2 = 0.02, leaving weights 0.72, 0.18, 0.08
    z1 = np.log(np.array([0.9, 0.1])); z2 = np.log(np.array([0.2, 0.8]))
    Z = np.stack([z1, z2])
    seen = {}
    for seed in range(400):
        vp = VerifyParams(sample=2, seed=seed, top_ks=2, pts_prune=0.05)
        toks, dg = pts_sample(Z, vp, 0, 0)
        assert dg["n_paths"] == 3 and tuple(toks) != (1, 0)
        seen[tuple(toks)] = seen.get(tuple(toks), 0) + 1
    exp = np.array([0.72, 0.18, 0.08]); exp = exp / exp.sum() * 400
    obs = np.array([seen.get((0, 1), 0), seen.get((0, 0), 0), seen.get((1, 1), 0)])
    assert stats.chisquare(obs, exp).pvalue > 1e-3


def test_pts_first_level_marginal_distribution():
    """Without pruning the first token's marginal is head 1's distribution truncated to its top K_s."""
    from oracle import pts_sample
    rng = np.random.default_rng(8)
    Zh = rng.standard_normal((3, 12)) * 1.5
    Ks, T, N = 4, 0.8, 3000
    p = softmax(Zh[0] / T)
    top = sorted(range(12), key=lambda v: (-p[v], v))[:Ks]
    counts = {v: 0 for v in top}
    for i in range(N):
        toks, _ = pts_sample(Zh, VerifyParams(sample=2, temperature=T, seed=31, top_ks=Ks, pts_prune=0.0), pos=i, seq_id=0)
        counts[toks[0]] += 1
    exp = np.array([p[v] for v in top]); exp = exp / exp.sum() * N
    assert stats.chisquare(np.array([counts[v] for v in top]), exp).pvalue > 1e-3


def test_spec_step_with_pts_keeps_the_backbone_token_an_independent_draw():
    cfg = si.tiny_config(n_draft=3, seed=13)
    orc, st = _setup(cfg)
    blk = si.first_block(cfg, 1)[0]
    vp_is = VerifyParams(mode=1, top_ka=4, temperature=0.9, sample=1, seed=5)
    vp_pts = VerifyParams(mode=1, top_ka=4, temperature=0.9, sample=2, seed=5, top_ks=2)
    a = orc.spec_step(copy.deepcopy(st), blk, vp_is)
    b = orc.spec_step(copy.deepcopy(st), blk, vp_pts)
    assert a["n_accepted"] == b["n_accepted"] and a["next_block"][0] == b["next_block"][0]
    from oracle import pts_sample
    toks, _ = pts_sample(b["Zh"], vp_pts, st.n + b["a"] + 1, st.seq_id)
    assert b["next_block"][1:] == toks
