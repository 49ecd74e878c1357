"""Pins for the oracle's building blocks against library routines and closed
forms (none of them re-types the oracle's own formula), and for the cached
incremental forward against a full-sequence causal forward assembled from
torch's own layers."""
import numpy as np
import scipy.special
import scipy.stats
import torch
import torch.nn.functional as TF

import synth_inputs as si
from oracle import Oracle, VerifyParams, gelu_erf, rmsnorm, rope_rotate, silu, softmax

torch.set_default_dtype(torch.float64)


def test_rmsnorm_vs_torch():
    rng = np.random.default_rng(0)
    x, g = rng.standard_normal((7, 96)), rng.standard_normal(96)
    ref = TF.rms_norm(torch.tensor(x), (96,), torch.tensor(g), eps=1e-6).numpy()
    np.testing.assert_allclose(rmsnorm(x, g, 1e-6), ref, rtol=1e-13, atol=1e-14)
    # eps sits inside the root: an all-zero row maps to zero, not NaN
    assert np.all(rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-6) == 0.0)


def test_activations_vs_libraries():
    x = np.linspace(-9, 9, 721)
    np.testing.assert_allclose(gelu_erf(x), TF.gelu(torch.tensor(x)).numpy(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(gelu_erf(x), x * scipy.stats.norm.cdf(x), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(silu(x), TF.silu(torch.tensor(x)).numpy(), rtol=1e-13, atol=1e-15)
    z = np.random.default_rng(1).standard_normal((5, 33)) * 8
    np.testing.assert_allclose(softmax(z), scipy.special.softmax(z, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(softmax(z).sum(-1), 1.0, rtol=1e-14)
    assert np.isfinite(softmax(np.array([[1e4, 0.0, -1e4]]))).all()          # max-subtraction


def test_rope_properties():
    rng = np.random.default_rng(2)
    hd, theta = 16, 10000.0
    q, k = rng.standard_normal((1, 1, hd)), rng.standard_normal((1, 1, hd))
    # position 0 is the identity; norms are preserved
    np.testing.assert_array_equal(rope_rotate(q, np.array([0]), theta), q)
    np.testing.assert_allclose(np.linalg.norm(rope_rotate(q, np.array([37]), theta)), np.linalg.norm(q))
    # the q.k product depends on the position difference only
    def dot(pq, pk):
        return float(np.sum(rope_rotate(q, np.array([pq]), theta) * rope_rotate(k, np.array([pk]), theta)))
    assert abs(dot(40, 33) - dot(107, 100)) < 1e-12
    assert abs(dot(40, 33) - dot(41, 33)) > 1e-6
    # closed form via complex multiplication: pair (i, i+hd/2) is one complex number
    pos = np.array([3, 250, 9001])
    x = rng.standard_normal((3, 2, hd))
    freq = torch.tensor(theta) ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = torch.tensor(pos, dtype=torch.float64)[:, None] * freq[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    xc = torch.complex(torch.tensor(x[..., :hd // 2]), torch.tensor(x[..., hd // 2:])) * rot
    ref = torch.cat([xc.real, xc.imag], dim=-1).numpy()
    np.testing.assert_allclose(rope_rotate(x, pos, theta), ref, rtol=1e-12, atol=1e-13)
    # highest-frequency pair (i = 0) turns by exactly pos radians
    e0 = np.zeros((1, 1, hd)); e0[0, 0, 0] = 1.0
    r = rope_rotate(e0, np.array([2]), theta)[0, 0]
    np.testing.assert_allclose([r[0], r[hd // 2]], [np.cos(2.0), np.sin(2.0)], rtol=1e-14)


def _torch_full_forward(cfg, w, rows, cond=None):
    """Whole-sequence causal forward from torch's own layers (linear, rms_norm,
    scaled_dot_product_attention with is_causal, gelu); rotary phase applied as a
    complex multiplication.  rows: [T, d] input embeddings at positions 0..T-1."""
    d, H, hd, L = cfg["d_model"], cfg["n_heads"], cfg["head_dim"], cfg["n_layers"]
    tw = {k: torch.tensor(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    X = torch.tensor(np.asarray(rows, dtype=np.float64))
    T = X.shape[0]
    freq = torch.tensor(cfg["rope_theta"]) ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * freq[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[None]            # [1, T, hd/2]

    def rope(t):                                                    # [H, T, hd]
        c = torch.complex(t[..., :hd // 2], t[..., hd // 2:]) * rot
        return torch.cat([c.real, c.imag], dim=-1)

    for l in range(L):
        A = TF.rms_norm(X, (d,), tw[f"l{l}.g1"], eps=cfg["rms_eps"])
        q, k, v = TF.linear(A, tw[f"l{l}.Wqkv"]).split(d, dim=-1)
        q, k, v = (t.reshape(T, H, hd).transpose(0, 1) for t in (q, k, v))
        o = TF.scaled_dot_product_attention(rope(q), rope(k), v, is_causal=True)
        X = X + TF.linear(o.transpose(0, 1).reshape(T, d), tw[f"l{l}.Wo"])
        if cfg["n_cond"] > 0:
            c = torch.tensor(np.asarray(cond, dtype=np.float64))
            A = TF.rms_norm(X, (d,), tw[f"l{l}.gc"], eps=cfg["rms_eps"])
            qc = TF.linear(A, tw[f"l{l}.Wcq"]).reshape(T, H, hd).transpose(0, 1)
            kc, vc = TF.linear(c, tw[f"l{l}.Wckv"]).split(d, dim=-1)
            kc, vc = (t.reshape(-1, H, hd).transpose(0, 1) for t in (kc, vc))
            oc = TF.scaled_dot_product_attention(qc, kc, vc)
            X = X + TF.linear(oc.transpose(0, 1).reshape(T, d), tw[f"l{l}.Wco"])
        A = TF.rms_norm(X, (d,), tw[f"l{l}.g2"], eps=cfg["rms_eps"])
        X = X + TF.linear(TF.gelu(TF.linear(A, tw[f"l{l}.W1"])), tw[f"l{l}.W2"])
    Hf = TF.rms_norm(X, (d,), tw["gf"], eps=cfg["rms_eps"])
    return Hf.numpy(), TF.linear(Hf, tw["WU"]).numpy()


def _check_incremental_vs_full(cfg):
    w = si.make_weights(cfg, perturb=True)
    orc = Oracle(cfg, w)
    P = cfg["prefix"]
    prefix = si.make_prefix(cfg, 1)[0]
    cond = si.make_cond(cfg, 1)
    cond = None if cond is None else cond[0]
    st = orc.new_state(cap=64)
    orc.prefill(st, prefix, cond)
    assert st.n == P
    rng = np.random.default_rng(3)
    toks, logits = [], []
    K = cfg["n_draft"]
    for _ in range(3):          # three full blocks, all rows kept (teacher forcing)
        blk = rng.integers(0, cfg["vocab"], K + 1)
        Hf, Z0 = orc.forward_block(st, orc.w["E"][blk])
        st.n += K + 1
        toks += list(blk)
        logits.append(Z0)
    rows = np.concatenate([prefix, np.asarray(w["E"], np.float64)[toks]], axis=0)
    _, Zfull = _torch_full_forward(cfg, w, rows, cond)
    np.testing.assert_allclose(np.concatenate(logits), Zfull[P:], rtol=1e-9, atol=1e-11)


def test_cached_block_forward_equals_full_causal_forward():
    _check_incremental_vs_full(si.tiny_config(n_layers=3, prefix=7, n_draft=4))


def test_cached_forward_with_cross_attention():
    _check_incremental_vs_full(si.tiny_config(n_cond=11, prefix=4, n_draft=3))
    _check_incremental_vs_full(si.tiny_config(n_cond=6, prefix=0, n_draft=2))


def test_head_reduces_to_closed_form_with_identity_weights():
    cfg = si.tiny_config()
    w = si.make_weights(cfg)
    for k in range(1, cfg["n_draft"] + 1):
        w[f"h{k}.W"] = np.eye(cfg["d_model"], dtype=np.float32)
        w[f"h{k}.b"] = np.zeros(cfg["d_model"], np.float32)
    orc = Oracle(cfg, w)
    g = np.random.default_rng(4).standard_normal(cfg["d_model"])
    ref = (torch.tensor(g) + TF.silu(torch.tensor(g))).numpy() @ np.asarray(w["WU"], np.float64).T
    Zh = orc.head_logits(g)
    for k in range(cfg["n_draft"]):
        np.testing.assert_allclose(Zh[k], ref, rtol=1e-12, atol=1e-14)
    # distinct heads give distinct rows once their matrices differ
    w2 = si.make_weights(cfg, perturb=True)
    Zh2 = Oracle(cfg, w2).head_logits(g)
    assert np.abs(Zh2[0] - Zh2[1]).max() > 1e-6
    tw = torch.tensor(np.asarray(w2["h2.W"], np.float64))
    r = torch.tensor(g) + TF.silu(TF.linear(torch.tensor(g), tw, torch.tensor(np.asarray(w2["h2.b"], np.float64))))
    np.testing.assert_allclose(Zh2[1], TF.linear(r, torch.tensor(np.asarray(w2["WU"], np.float64))).numpy(),
                               rtol=1e-12, atol=1e-14)


# ---- cross-attention decoding heads (Eq. 4; Table 3 rows D/E) ---------------------------------
def _ca_setup(n_cond=9, seed=5, **kw):
    cfg = si.tiny_config(n_cond=n_cond, head_kind="ca", prefix=3, **kw)
    w = si.make_weights(cfg, perturb=True)
    orc = Oracle(cfg, w)
    st = orc.new_state()
    cond = si.make_cond(cfg, 1)[0]
    orc.prefill(st, si.make_prefix(cfg, 1)[0], cond)
    g = np.random.default_rng(seed).standard_normal(cfg["d_model"])
    return cfg, w, orc, st, cond, g


def test_ca_head_closed_forms():
    f64 = lambda x: np.asarray(x, np.float64)
    # zero output projection: the attention branch vanishes, logits = W^(d) h
    cfg, w, orc, st, cond, g = _ca_setup()
    for k in range(1, cfg["n_draft"] + 1):
        w[f"h{k}.Wo"] = np.zeros_like(w[f"h{k}.Wo"])
    orc0 = Oracle(cfg, w)
    Zh = orc0.head_logits(g, st)
    for k in range(cfg["n_draft"]):
        np.testing.assert_allclose(Zh[k], f64(w[f"h{k + 1}.WU"]) @ g, rtol=1e-12, atol=1e-14)
    # one condition token: the softmax is 1, r = h + Wo Wv c
    cfg, w, orc, st, cond, g = _ca_setup(n_cond=1)
    Zh = orc.head_logits(g, st)
    d = cfg["d_model"]
    for k in range(1, cfg["n_draft"] + 1):
        v = f64(w[f"h{k}.Wkv"])[d:] @ f64(cond[0])
        r = g + f64(w[f"h{k}.Wo"]) @ v
        np.testing.assert_allclose(Zh[k - 1], f64(w[f"h{k}.WU"]) @ r, rtol=1e-12, atol=1e-14)
    # zero query projection: uniform attention, r = h + Wo mean_t(Wv c_t)
    cfg, w, orc, st, cond, g = _ca_setup(n_cond=7)
    for k in range(1, cfg["n_draft"] + 1):
        w[f"h{k}.Wq"] = np.zeros_like(w[f"h{k}.Wq"])
    Zh = Oracle(cfg, w).head_logits(g, st)
    for k in range(1, cfg["n_draft"] + 1):
        vbar = (f64(cond) @ f64(w[f"h{k}.Wkv"])[d:].T).mean(0)
        r = g + f64(w[f"h{k}.Wo"]) @ vbar
        np.testing.assert_allclose(Zh[k - 1], f64(w[f"h{k}.WU"]) @ r, rtol=1e-12, atol=1e-13)


def test_ca_head_against_torch_attention():
    cfg, w, orc, st, cond, g = _ca_setup(n_cond=13, seed=11)
    H, hd, d = cfg["n_heads"], cfg["head_dim"], cfg["d_model"]
    t = lambda x: torch.tensor(np.asarray(x, np.float64))
    Zh = orc.head_logits(g, st)
    for k in range(1, cfg["n_draft"] + 1):
        q = TF.linear(t(g), t(w[f"h{k}.Wq"])).reshape(1, H, 1, hd)
        kv = TF.linear(t(cond), t(w[f"h{k}.Wkv"]))
        kk = kv[:, :d].reshape(-1, H, hd).permute(1, 0, 2)[None]
        vv = kv[:, d:].reshape(-1, H, hd).permute(1, 0, 2)[None]
        o = TF.scaled_dot_product_attention(q, kk, vv).reshape(d)
        r = t(g) + TF.linear(o, t(w[f"h{k}.Wo"]))
        np.testing.assert_allclose(Zh[k - 1], TF.linear(r, t(w[f"h{k}.WU"])).numpy(), rtol=1e-10, atol=1e-12)
    # heads differ from each other and depend on the condition
    assert np.abs(Zh[0] - Zh[1]).max() > 1e-6
    st2 = orc.new_state()
    orc.prefill(st2, si.make_prefix(cfg, 1)[0], cond[::-1].copy() * 0.5)
    assert np.abs(orc.head_logits(g, st2)[0] - Zh[0]).max() > 1e-6
