"""Plain float64 numpy implementation of one multi-head speculative decoding
step, the plain next-token step and the condition prefill.  TEST INFRASTRUCTURE
ONLY: imported by tests, the smoke check and the benchmark's CPU-baseline leg.

What is computed, with the passage it follows:

* backbone: N decoder blocks over the draft block x_{s:s+D} against a key-value
  cache holding x_0..x_{s-1}, causal within the block (Sec. 4.1 first
  paragraph; Sec. 4.2; Alg. 1 "forward with causal mask"); each block is
  self-attention, optional cross-attention to the condition c, feed-forward;
* backbone distribution p^(0)_{s+1} = softmax(W^(0) h_s) (Eq. 3);
* D decoding heads reading the same final hidden state h_s, head d predicting
  position s+d+1 (Eq. 4), here in the MLP variant of the ablation (Table 3 rows
  B/C): r = h + SiLU(W_d h + b_d), logits through the shared unembedding; or
  (head_kind "ca", Table 3 rows D/E) Eq. 4 as printed: a cross-attention layer
  of the hidden state over the condition tokens, then the head's own
  unembedding W^(d).  The paper does not spell the layer out; the reading here
  is one multi-head attention with a residual connection and no extra norm:
  q = Wq_d h, keys/values = Wk_d c, Wv_d c (cached at prefill),
  r = h + Wo_d softmax(q k^T / sqrt(hd)) v, logits = W^(d) r;
* verification: accept candidates while the criterion holds, stop at the first
  failure, then resample D+1 tokens from p^(0) and the heads at the first
  rejected position (Sec. 4.2; Alg. 1 inner while and the resample line);
* criteria: probability threshold p^(0)_i(x_i) > delta, or top-K_a membership
  (Sec. 5.4 "Verification criterion"); K_a = 1 is greedy verification;
* sampling of the heads' tokens: independent draws, or top-K_s probability-tree
  sampling with pruning at 1e-5 (appendix "Sampling strategies", Table 5);
* the cache "rollback" is implied by s <- s*: the next pass overwrites slots
  from the new s on, so only the length changes.

Details the paper leaves open (norm type, activation, positional encoding,
where the final norm sits) follow the synthetic workload definition: pre-RMSNorm
with eps inside the root, rotary embedding on q/k with half-split pairing
(i, i + hd/2) and frequency theta^(-2i/hd), exact erf GELU, no projection
biases, untied embedding / unembedding, final RMSNorm before both W^(0) and the
heads.

Notation: K = number of heads (paper's D), R = K+1 block rows, n = cached
positions.  Block row j holds the token at absolute position n + j; logits row j
is the distribution of position n + j + 1.

Pins (tests/test_oracle_*.py): greedy speculative output equals plain greedy
decoding; accept counts in [1, K+1]; rollback exactness with NaN-poisoned stale
slots; block causality; forced drafts hit every accept length; K_a = V accepts
all; delta > 1 equals plain sampled decoding; incremental cached forward equals
a full-sequence causal forward built from torch's library attention; building
blocks against scipy/torch routines; Philox against an independent big-int
implementation and published known-answer values; the cross-attention head
against its closed forms (zero output projection, one condition token, zero query
projection) and torch's library attention; probability-tree sampling against the
flattened outer product of the per-level weights (no pruning), a hand-made pruned tree,
K_s = 1, and a chi-square test of its first-level marginal.
The stochastic path's exact sampled sequences have no external pin beyond the
chi-square test of the sampler's distribution: parity unpinned for those.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
from scipy.special import erf

from .philox import uniform24

F64 = np.float64


# ----------------------------------------------------------------------------
# building blocks
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x * g / sqrt(mean(x^2) + eps), row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x * g / np.sqrt(ms + eps)


def rope_rotate(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding.  x: [R, H, hd], pos: [R] absolute positions.
    Pair (i, i+hd/2) is rotated by the angle pos * theta^(-2i/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=F64)
    freq = theta ** (-2.0 * i / hd)
    ang = pos.astype(F64)[:, None] * freq[None, :]            # [R, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def gelu_erf(x: np.ndarray) -> np.ndarray:
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax(z: np.ndarray) -> np.ndarray:
    e = np.exp(z - np.max(z, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


# ----------------------------------------------------------------------------
# verification and sampling
# ----------------------------------------------------------------------------
@dataclass
class VerifyParams:
    mode: int = 0            # 0 greedy (K_a = 1), 1 top-K_a, 2 probability threshold
    top_ka: int = 1
    delta: float = 0.5
    temperature: float = 1.0
    sample: int = 0          # 0 argmax, 1 categorical (independent sampling), 2 probability-tree sampling
    seed: int = 0
    top_ks: int = 2          # K_s of the probability tree
    pts_prune: float = 1e-5  # branches whose cumulative weight falls below this are cut


def rank_of(z: np.ndarray, x: int) -> int:
    """Number of tokens ranked strictly ahead of x: larger logit, or equal logit
    and lower index."""
    zx = z[x]
    return int(np.sum(z > zx) + np.sum(z[:x] == zx))


def accept(z: np.ndarray, x: int, vp: VerifyParams) -> bool:
    """Acceptance criterion for candidate x against backbone logits z."""
    if vp.mode == 2:
        return bool(softmax(z / vp.temperature)[x] > vp.delta)
    ka = 1 if vp.mode == 0 else vp.top_ka
    return rank_of(z, x) < ka


def sample(z: np.ndarray, vp: VerifyParams, pos: int, head: int, seq_id: int):
    """Draw a token from logits z (argmax, or categorical; under probability-tree sampling the
    backbone's token is a categorical draw).  Returns (token, diagnostics)."""
    if vp.sample == 0:
        tok = int(np.argmax(z))                   # first index among equal maxima
        top2 = np.partition(z, -2)[-2:] if z.size > 1 else np.array([-np.inf, z[0]])
        return tok, {"kind": "argmax", "margin": float(top2[1] - top2[0])}
    w = np.exp((z - np.max(z)) / vp.temperature)
    cdf = np.cumsum(w)
    S = cdf[-1]
    u = uniform24(vp.seed, pos, head, seq_id)
    hit = np.nonzero(cdf > u * S)[0]
    tok = int(hit[0]) if hit.size else int(np.nonzero(w > 0)[0][-1])
    edges = np.concatenate([[0.0], cdf])
    gap = float(np.min(np.abs(edges - u * S)) / S)
    return tok, {"kind": "cdf", "u": u, "gap": gap}


PTS_HEAD = 254      # Philox "head" coordinate of the one uniform a probability-tree draw consumes


def pts_sample(Zh: np.ndarray, vp: VerifyParams, pos: int, seq_id: int):
    """Top-K_s probability-tree sampling of the K head tokens (appendix "Sampling strategies").

    Level d of the tree holds the K_s most probable tokens of head d's distribution
    softmax(z_d / T) (equal probabilities ordered by lower index) with their probabilities
    m as edge weights; a path's weight is the product of its edges; a branch is cut as soon as
    its cumulative weight falls below vp.pts_prune; one complete path is drawn with probability
    proportional to its weight, by inverse CDF over the surviving paths in depth-first order
    (most probable child first) with one uniform.  If no complete path survives, the path of
    the most probable token of every head is taken.  Returns (tokens, diagnostics)."""
    K = Zh.shape[0]
    tops = []
    for d in range(K):
        p = softmax(np.asarray(Zh[d], F64) / vp.temperature)
        order = np.lexsort((np.arange(p.size), -p))[:vp.top_ks]
        tops.append([(int(v), float(p[v])) for v in order])
    leaves = []

    def grow(d, toks, w):
        if d == K:
            leaves.append((toks, w))
            return
        for v, m in tops[d]:
            if w * m >= vp.pts_prune:
                grow(d + 1, toks + [v], w * m)

    grow(0, [], 1.0)
    u = uniform24(vp.seed, pos, PTS_HEAD, seq_id)
    if not leaves:
        return [t[0][0] for t in tops], {"kind": "pts", "u": u, "gap": 1.0, "n_paths": 0}
    cdf = np.cumsum([w for _, w in leaves])
    S = cdf[-1]
    hit = np.nonzero(cdf > u * S)[0]
    i = int(hit[0]) if hit.size else len(leaves) - 1
    edges = np.concatenate([[0.0], cdf])
    gap = float(np.min(np.abs(edges - u * S)) / S)
    # how close any cut decision or any top-K_s membership was (for near-tie flags of a comparison)
    return list(leaves[i][0]), {"kind": "pts", "u": u, "gap": gap, "n_paths": len(leaves)}


# ----------------------------------------------------------------------------
# model
# ----------------------------------------------------------------------------
@dataclass
class SeqState:
    """One sequence: n cached positions and per-layer K/V [cap, H, hd]."""
    n: int
    k: list
    v: list
    ck: list = field(default_factory=list)     # cross-attention condition keys per layer
    cv: list = field(default_factory=list)
    hk: list = field(default_factory=list)     # condition keys / values of the cross-attention heads
    hv: list = field(default_factory=list)
    seq_id: int = 0


class Oracle:
    def __init__(self, cfg: dict, weights: dict, kv_dtype=np.float64):
        self.cfg = cfg
        self.L, self.d, self.H = cfg["n_layers"], cfg["d_model"], cfg["n_heads"]
        self.hd, self.F, self.V, self.K = cfg["head_dim"], cfg["d_ffn"], cfg["vocab"], cfg["n_draft"]
        self.n_cond = cfg["n_cond"]
        self.theta, self.eps = float(cfg["rope_theta"]), float(cfg["rms_eps"])
        self.kv_dtype = kv_dtype
        self.head_kind = cfg.get("head_kind", "mlp")
        assert self.head_kind in ("mlp", "ca") and (self.head_kind == "mlp" or self.n_cond > 0)
        self.w = {k: np.asarray(v, dtype=F64) for k, v in weights.items()}

    # -- state -----------------------------------------------------------------
    def new_state(self, cap: int | None = None, seq_id: int = 0) -> SeqState:
        cap = self.cfg["max_ctx"] if cap is None else cap
        mk = lambda: np.full((cap, self.H, self.hd), np.nan, dtype=self.kv_dtype)
        return SeqState(0, [mk() for _ in range(self.L)], [mk() for _ in range(self.L)],
                        seq_id=seq_id)

    # -- backbone ----------------------------------------------------------------
    def _attend(self, q, kc, vc, limits):
        """q: [R, H, hd]; kc, vc: [T, H, hd]; row j sees cache positions < limits[j]."""
        out = np.empty_like(q)
        scale = 1.0 / np.sqrt(self.hd)
        for j in range(q.shape[0]):
            T = int(limits[j])
            s = np.einsum("hd,thd->ht", q[j], kc[:T].astype(F64)) * scale
            p = softmax(s)
            out[j] = np.einsum("ht,thd->hd", p, vc[:T].astype(F64))
        return out

    def forward_block(self, st: SeqState, X: np.ndarray):
        """Run all blocks over rows X [R, d] placed at positions n..n+R-1; writes
        their keys/values into the cache (length unchanged).  Returns (Hf, Z0):
        final-normed hidden states and backbone logits (Eq. 3)."""
        w, d, H, hd = self.w, self.d, self.H, self.hd
        X = np.array(X, dtype=F64)
        R, n = X.shape[0], st.n
        pos = np.arange(n, n + R)
        for l in range(self.L):
            A = rmsnorm(X, w[f"l{l}.g1"], self.eps)
            QKV = A @ w[f"l{l}.Wqkv"].T
            q = rope_rotate(QKV[:, :d].reshape(R, H, hd), pos, self.theta)
            k = rope_rotate(QKV[:, d:2 * d].reshape(R, H, hd), pos, self.theta)
            v = QKV[:, 2 * d:].reshape(R, H, hd)
            st.k[l][n:n + R] = k
            st.v[l][n:n + R] = v
            o = self._attend(q, st.k[l], st.v[l], pos + 1)          # causal: keys 0..n+j
            X = X + o.reshape(R, d) @ w[f"l{l}.Wo"].T
            if self.n_cond > 0:
                A = rmsnorm(X, w[f"l{l}.gc"], self.eps)
                qc = (A @ w[f"l{l}.Wcq"].T).reshape(R, H, hd)
                oc = self._attend(qc, st.ck[l], st.cv[l], np.full(R, self.n_cond))
                X = X + oc.reshape(R, d) @ w[f"l{l}.Wco"].T
            A = rmsnorm(X, w[f"l{l}.g2"], self.eps)
            X = X + gelu_erf(A @ w[f"l{l}.W1"].T) @ w[f"l{l}.W2"].T
        Hf = rmsnorm(X, w["gf"], self.eps)
        return Hf, Hf @ w["WU"].T

    def head_logits(self, g: np.ndarray, st: SeqState | None = None) -> np.ndarray:
        """Logits of the K decoding heads from one hidden state g [d] -> [K, V] (Eq. 4)."""
        w = self.w
        out = np.empty((self.K, self.V), dtype=F64)
        for k in range(1, self.K + 1):
            if self.head_kind == "ca":
                q = (w[f"h{k}.Wq"] @ g).reshape(1, self.H, self.hd)
                o = self._attend(q, st.hk[k - 1], st.hv[k - 1], np.array([self.n_cond]))
                r = g + w[f"h{k}.Wo"] @ o.reshape(self.d)
                out[k - 1] = w[f"h{k}.WU"] @ r
            else:
                r = g + silu(w[f"h{k}.W"] @ g + w[f"h{k}.b"])
                out[k - 1] = w["WU"] @ r
        return out

    # -- entry points --------------------------------------------------------------
    def prefill(self, st: SeqState, prefix_emb: np.ndarray, cond: np.ndarray | None = None):
        """Condition prefix through the backbone with a full causal mask, filling
        cache positions 0..P-1; condition tokens are projected once per layer."""
        if self.n_cond > 0:
            c = np.asarray(cond, dtype=F64)
            st.ck, st.cv = [], []
            for l in range(self.L):
                kv = c @ self.w[f"l{l}.Wckv"].T
                st.ck.append(kv[:, :self.d].reshape(-1, self.H, self.hd).astype(self.kv_dtype))
                st.cv.append(kv[:, self.d:].reshape(-1, self.H, self.hd).astype(self.kv_dtype))
            if self.head_kind == "ca":
                st.hk, st.hv = [], []
                for k in range(1, self.K + 1):
                    kv = c @ self.w[f"h{k}.Wkv"].T
                    st.hk.append(kv[:, :self.d].reshape(-1, self.H, self.hd).astype(self.kv_dtype))
                    st.hv.append(kv[:, self.d:].reshape(-1, self.H, self.hd).astype(self.kv_dtype))
        st.n = 0
        P = 0 if prefix_emb is None else prefix_emb.shape[0]
        if P > 0:
            self.forward_block(st, prefix_emb)
            st.n = P

    def spec_step(self, st: SeqState, block, vp: VerifyParams, heads_on_all_rows: bool = False):
        """One iteration of Alg. 1's outer loop.  block = [last accepted token,
        K candidates].  Returns a dict; st.n advances by n_accepted."""
        K, n = self.K, st.n
        t = [int(x) for x in block]
        assert len(t) == K + 1
        Hf, Z0 = self.forward_block(st, self.w["E"][t])
        a = 0
        for j in range(1, K + 1):
            if not accept(Z0[j - 1], t[j], vp):
                break
            a += 1
        y0, diag0 = sample(Z0[a], vp, n + a + 1, 0, st.seq_id)
        if heads_on_all_rows:      # Alg. 1's literal for-loop over heads on h_{s:s+D}
            Zh = np.stack([self.head_logits(Hf[j], st) for j in range(K + 1)])[a]
        else:                      # only h_{s*-1} is consumed by the resample line
            Zh = self.head_logits(Hf[a], st)
        ys, diags = [], [diag0]
        if vp.sample == 2 and K > 0:     # the backbone token is an independent draw; the heads' tokens one tree draw
            ys, dg = pts_sample(Zh, vp, n + a + 1, st.seq_id)
            diags += [dg] * K
        else:
            for k in range(1, K + 1):
                y, dg = sample(Zh[k - 1], vp, n + a + 1 + k, k, st.seq_id)
                ys.append(y)
                diags.append(dg)
        st.n = n + a + 1
        return {"out_tokens": t[1:a + 1] + [y0], "n_accepted": a + 1, "next_block": [y0] + ys,
                "Z0": Z0, "Zh": Zh, "Hf": Hf, "a": a, "diag": diags}

    def plain_step(self, st: SeqState, token: int, vp: VerifyParams):
        """Next-token decoding: one row, sample from p^(0) only."""
        n = st.n
        Hf, Z0 = self.forward_block(st, self.w["E"][[int(token)]])
        y0, diag0 = sample(Z0[0], vp, n + 1, 0, st.seq_id)
        st.n = n + 1
        return {"out_tokens": [y0], "n_accepted": 1, "next_block": [y0], "Z0": Z0, "Hf": Hf,
                "diag": [diag0]}

    # -- generation loops (Alg. 1 outer loop; EOS disabled for synthetic runs) ------
    def generate_spec(self, st: SeqState, first_block, n_tokens: int, vp: VerifyParams):
        toks, steps, block = [], 0, list(first_block)
        hist = []
        while len(toks) < n_tokens:
            r = self.spec_step(st, block, vp)
            toks += r["out_tokens"]
            hist.append(r["n_accepted"])
            block = r["next_block"]
            steps += 1
        return toks[:n_tokens], steps, hist

    def generate_plain(self, st: SeqState, first_token: int, n_tokens: int, vp: VerifyParams):
        toks, tok = [], int(first_token)
        while len(toks) < n_tokens:
            r = self.plain_step(st, tok, vp)
            tok = r["out_tokens"][0]
            toks.append(tok)
        return toks
