"""Lock-step comparison of the HIP library against the CPU oracle.

The oracle drives: every step the GPU receives the oracle's draft block and
cache lengths (both live in caller-visible device arrays), so a single flagged
near-tie cannot desynchronise the two sides.  Cache rows written by a step
depend only on the input block, so the GPU cache stays valid under this
teacher forcing.  A decision is *flagged, not counted* when the oracle's own
margin for it is within 1e-2 (logit gap).  Categorical and probability-tree draws:
an fp32 model's draw is compared with the oracle's OWN draw (logits agree to 1e-6, so the
inverse CDFs do too), flagged when the oracle's uniform lies within 1e-4 of a CDF edge
(edges are 1/V apart on average, so a wider band would flag every draw from V = 500 on);
a bf16 model's draw is compared with the oracle's sampler re-run on the GPU's logits row
(a bf16 forward moves every CDF edge by more than the edge spacing at V >= 1000), flagged
within 2e-5.  A case in which more than a quarter of the decisions are flagged fails:
`report` bounds the count and puts the tally on pytest's terminal summary."""
from __future__ import annotations

import copy
import dataclasses
from dataclasses import dataclass, field

import numpy as np

import synth_inputs as si
from oracle import Oracle, VerifyParams, pts_sample, sample

TIE = 1e-2
# bf16 models: categorical draws are decided on the same inputs on both sides, the oracle's
# float64 inverse CDF evaluated on the GPU's own fp32 logits (a 1e-3 logit difference between a
# bf16 forward and the float64 forward moves every CDF edge by far more than the spacing of
# the edges at V >= 1000).  What remains is fp32-vs-fp64 rounding of the running sum.
CDF_TIE = 2e-5
# fp32 models: the GPU's draw against the oracle's own draw from its own logits.  Logits agree to
# 1e-6 there, so every CDF edge does to a few 1e-6 of the total; the band is 100 times that and
# still flags only 2e-4 * V of the draws (a 1e-3 band would flag all of them from V = 500 on).
CDF_TIE_OWN = 1e-4
# share of a case's decisions that may be near-ties before the case counts as not compared
MAX_FLAGGED_FRAC = 0.25
SUMMARY: list = []          # one line per reported case, printed by conftest's terminal summary


def own_draws(cfg) -> bool:
    """fp32 models compare draws with the oracle's own; bf16 models on the GPU's logits."""
    return cfg["dtype"] != "bf16"


def report(tal, name, max_flagged_frac: float = MAX_FLAGGED_FRAC):
    """Print and record the tally of one case; fail on a mismatch or when so many decisions
    were near-ties that the case compared too little."""
    line = (f"[{name}] rows {tal.rows} max_rel {tal.max_rel:.3e} decisions {tal.decisions} "
            f"flagged {tal.flagged} mismatches {len(tal.mismatches)} accept_hist {tal.accept_hist}")
    print(line, flush=True)
    SUMMARY.append(line)
    assert not tal.mismatches, tal.mismatches[:5]
    assert tal.decisions > 0, f"{name}: no decision was compared"
    assert tal.flagged <= max(2, max_flagged_frac * tal.decisions), \
        f"{name}: {tal.flagged} of {tal.decisions} decisions were near-ties, too few were compared"


def logit_tol(cfg):
    return 2e-2 if cfg["dtype"] == "bf16" else 1e-5


def rel_err(z_gpu: np.ndarray, z_ref: np.ndarray) -> float:
    """max_v |z_gpu - z_ref| / max_v |z_ref| for one row."""
    return float(np.max(np.abs(z_gpu.astype(np.float64) - z_ref)) / np.max(np.abs(z_ref)))


def accept_margin(z: np.ndarray, x: int, vp: VerifyParams) -> float:
    """Oracle-side distance of the accept decision from flipping."""
    if vp.mode == 2:
        # p = softmax(z/T)[x] crosses delta when z[x] moves by about T |ln(p / delta)|: the same
        # logit scale as the rank rule's margin
        e = np.exp((z - z.max()) / vp.temperature)
        p = e[x] / e.sum()
        return float(vp.temperature * abs(np.log(p) - np.log(vp.delta))) if p > 0 and vp.delta > 0 else np.inf
    ka = 1 if vp.mode == 0 else vp.top_ka
    srt = np.sort(z)[::-1]
    others = np.delete(z, x)
    rank = int(np.sum(z > z[x]) + np.sum(z[:x] == z[x]))
    so = np.sort(others)[::-1]
    if rank < ka:                      # accepted: flips if the ka-th best other token overtakes it
        return float(z[x] - so[ka - 1]) if ka - 1 < so.size else np.inf
    return float(so[ka - 1] - z[x])    # rejected: flips if it passes the ka-th best other token


def check_draw(tal, where, what, dg: dict, tok_gpu: int, tok_oracle: int, z_gpu, vp, pos, head, seq_id,
               own: bool = False):
    """One token draw.  argmax: oracle token unless its top-1/top-2 margin is a near-tie.
    categorical: the oracle's own draw (own=True, fp32 models), else the oracle's sampler re-run
    on the GPU's logits row."""
    tal.decisions += 1
    if dg["kind"] == "argmax":
        if dg["margin"] <= TIE:
            tal.flagged += 1
        elif tok_gpu != tok_oracle:
            tal.mismatches.append(f"{where}: {what} gpu {tok_gpu} oracle {tok_oracle}")
        return
    if own:
        if dg["gap"] <= CDF_TIE_OWN:
            tal.flagged += 1
        elif tok_gpu != tok_oracle:
            tal.mismatches.append(f"{where}: {what} gpu {tok_gpu} oracle's own draw {tok_oracle} (u={dg['u']:.6f})")
        return
    ref, dg2 = sample(z_gpu.astype(np.float64), vp, pos, head, seq_id)
    if dg2["gap"] <= CDF_TIE:
        tal.flagged += 1
    elif tok_gpu != ref:
        tal.mismatches.append(f"{where}: {what} gpu {tok_gpu} oracle-on-gpu-logits {ref} (u={dg2['u']:.6f})")


def check_pts(tal, where, toks_gpu, zh_gpu, vp, pos, seq_id, own_ref=None):
    """One probability-tree draw of the K head tokens: the oracle's sampler re-run on the GPU's
    head logits; flagged when the uniform falls within CDF_TIE of a path boundary or a path's
    weight within 1e-4 (relative) of the cut-off.  own_ref = (tokens, diagnostics, oracle's head
    logits): compare with the oracle's own draw instead (fp32 models), flagged within CDF_TIE_OWN."""
    tal.decisions += 1
    if own_ref is not None:
        ref, dg, zh_gpu = own_ref[0], own_ref[1], own_ref[2]
    else:
        ref, dg = pts_sample(np.asarray(zh_gpu, np.float64), vp, pos, seq_id)
    lo = dataclasses.replace(vp, pts_prune=vp.pts_prune * (1 - 1e-4))
    hi = dataclasses.replace(vp, pts_prune=vp.pts_prune * (1 + 1e-4))
    stable = pts_sample(np.asarray(zh_gpu, np.float64), lo, pos, seq_id)[1]["n_paths"] == \
        pts_sample(np.asarray(zh_gpu, np.float64), hi, pos, seq_id)[1]["n_paths"]
    tal.pts_paths.append(dg["n_paths"])
    if dg["gap"] <= (CDF_TIE_OWN if own_ref is not None else CDF_TIE) or not stable:
        tal.flagged += 1
    elif [int(t) for t in toks_gpu] != [int(t) for t in ref]:
        tal.mismatches.append(f"{where}: tree draw gpu {[int(t) for t in toks_gpu]} "
                              f"{'oracle own draw' if own_ref is not None else 'oracle-on-gpu-logits'} {ref} "
                              f"(u={dg['u']:.6f}, paths {dg['n_paths']})")


@dataclass
class Tally:
    rows: int = 0
    decisions: int = 0
    flagged: int = 0
    mismatches: list = field(default_factory=list)
    max_rel: float = 0.0
    accept_hist: dict = field(default_factory=dict)
    pts_paths: list = field(default_factory=list)      # surviving paths of every probability-tree draw


def to_vp_gpu(xsm, vp: VerifyParams):
    return xsm.xsm_verify_params(vp.mode, vp.top_ka, vp.delta, vp.temperature, vp.sample, vp.seed,
                                 vp.top_ks, vp.pts_prune)


def setup_pair(cfg, engine_cls, n_seq, prefix_lens=None, perturb=True, max_ctx=None, kv_dtype=np.float64,
               options=()):
    """Weights, oracle states and a GPU engine prefilled with the same condition prefixes.
    prefix_lens: per-sequence prefix lengths (ragged batches); default cfg['prefix'].
    options: (option, value) pairs set on the engine before the prefill."""
    w = si.make_weights(cfg, perturb=perturb)
    orc = Oracle(cfg, w, kv_dtype=kv_dtype)
    eng = engine_cls(cfg, max_batch=n_seq, max_ctx=max_ctx or cfg["max_ctx"])
    eng.xsm_load_weights(si.pack_canonical(cfg, w))
    for opt, val in options:
        eng.xsm_set_option(opt, val)
    prefix_lens = prefix_lens or [cfg["prefix"]] * n_seq
    pmax = max(prefix_lens)
    prefix = si.make_prefix(cfg, n_seq, P=pmax) if pmax > 0 else None
    cond = si.make_cond(cfg, n_seq)
    states = []
    for b in range(n_seq):
        st = orc.new_state(cap=max_ctx or cfg["max_ctx"], seq_id=b)
        orc.prefill(st, None if prefix is None else prefix[b, :prefix_lens[b]], None if cond is None else cond[b])
        states.append(st)
    # GPU: one prefill call per distinct length (a call takes one P for all its sequences)
    d_cond = None if cond is None else eng.to_device(cond)
    for P in sorted(set(prefix_lens)):
        slots = [b for b in range(n_seq) if prefix_lens[b] == P]
        dp = None if P == 0 else eng.to_device(prefix[slots, :P])
        dc = None if d_cond is None else d_cond[slots].contiguous()
        eng.xsm_prefill(slots, dp, dc)
    eng.torch.cuda.synchronize()
    return w, orc, states, eng


def lockstep(cfg, orc, states, eng, xsm, vp: VerifyParams, n_steps: int, first_blocks, plain=False,
             forced=None, tally: Tally | None = None, slots=None) -> Tally:
    """Run n_steps with the oracle driving.  forced(step, b, state, block) may replace the block
    (e.g. with the true continuation) before both sides run it.  slots[i] is the cache slot of
    batch row i (default: row i uses slot i)."""
    torch = eng.torch
    tal = tally or Tally()
    n_seq = len(states)
    K = 0 if plain else cfg["n_draft"]
    R = K + 1
    buf = eng.buffers(n_seq, spec=not plain, debug=True)
    if slots is not None:
        buf.slot.copy_(torch.tensor(list(slots), dtype=torch.int32))
    blocks = [list(map(int, bl[:R])) for bl in first_blocks]
    vpg = to_vp_gpu(xsm, vp)
    tol = logit_tol(cfg)
    own = own_draws(cfg)
    for step in range(n_steps):
        if forced is not None:
            blocks = [forced(step, b, states[b], blocks[b]) for b in range(n_seq)]
        lens = [st.n for st in states]
        buf.kv_len.copy_(torch.tensor(lens, dtype=torch.int32))
        buf.block.copy_(torch.tensor(blocks, dtype=torch.int32))
        if plain:
            eng.xsm_plain_step(buf, vpg, max(lens))
        else:
            eng.xsm_spec_step(buf, vpg, max(lens))
        torch.cuda.synchronize()
        g_logits = buf.logits.cpu().numpy()
        g_heads = None if plain else buf.head_logits.cpu().numpy()
        g_acc = buf.n_accepted.cpu().numpy()
        g_out = buf.out_tokens.cpu().numpy()
        g_blk = buf.block.cpu().numpy()
        g_len = buf.kv_len.cpu().numpy()
        g_flags = buf.flags.cpu().numpy()
        for b in range(n_seq):
            st = states[b]
            blk = blocks[b]
            r = orc.plain_step(st, blk[0], vp) if plain else orc.spec_step(st, blk, vp)
            where = f"step {step} seq {b}"
            assert (g_flags[b] & ~1) == 0, f"{where}: device flagged input error {g_flags[b]}"
            for j in range(R):
                e = rel_err(g_logits[b, j], r["Z0"][j])
                tal.max_rel = max(tal.max_rel, e)
                tal.rows += 1
                assert e <= tol, f"{where}: backbone logits row {j} rel err {e:.3e} > {tol}"
            # accept scan: every decision up to and including the first rejection
            a = r["n_accepted"] - 1
            safe = True
            for j in range(1, min(a + 1, K) + 1):
                tal.decisions += 1
                if accept_margin(r["Z0"][j - 1], blk[j], vp) <= TIE:
                    safe = False
            tal.accept_hist[a + 1] = tal.accept_hist.get(a + 1, 0) + 1
            if not safe:
                tal.flagged += 1
                blocks[b] = r["next_block"]
                continue
            if int(g_acc[b]) != a + 1:
                tal.mismatches.append(f"{where}: n_accepted gpu {g_acc[b]} oracle {a + 1}")
                blocks[b] = r["next_block"]
                continue
            assert int(g_len[b]) == st.n, f"{where}: kv_len {g_len[b]} vs {st.n}"
            assert list(g_out[b, :a]) == r["out_tokens"][:a], f"{where}: accepted prefix differs"
            # draws: backbone row, then heads
            n0 = lens[b]
            assert int(g_out[b, a]) == int(g_blk[b, 0]), f"{where}: emitted token != next block head"
            check_draw(tal, where, "y0", r["diag"][0], int(g_out[b, a]), r["out_tokens"][a],
                       g_logits[b, a], vp, n0 + a + 1, 0, st.seq_id, own=own)
            for k in range(1, K + 1):
                e = rel_err(g_heads[b, k - 1], r["Zh"][k - 1])
                tal.max_rel = max(tal.max_rel, e)
                tal.rows += 1
                assert e <= tol, f"{where}: head {k} logits rel err {e:.3e} > {tol}"
                if vp.sample != 2:
                    check_draw(tal, where, f"head {k}", r["diag"][k], int(g_blk[b, k]), r["next_block"][k],
                               g_heads[b, k - 1], vp, n0 + a + 1 + k, k, st.seq_id, own=own)
            if vp.sample == 2 and K > 0:
                check_pts(tal, where, g_blk[b, 1:], g_heads[b], vp, n0 + a + 1, st.seq_id,
                          own_ref=(r["next_block"][1:], r["diag"][1], r["Zh"]) if own else None)
            blocks[b] = r["next_block"]
    return tal


def true_continuation(orc, st, first_token: int, K: int, vp: VerifyParams):
    """Block whose candidates are what plain decoding would produce (all accepted under greedy)."""
    toks = orc.generate_plain(copy.deepcopy(st), first_token, K, vp)
    return [int(first_token)] + toks
