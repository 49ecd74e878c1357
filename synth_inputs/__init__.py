"""Seeded synthetic inputs for the multi-head speculative decoding step.

This module only *draws numbers*: model shapes, random-init weights, condition
prefixes, condition tokens, first draft blocks.  It holds none of the method's
arithmetic (no normalisation, attention, heads, verification or sampling), so
both the CPU oracle's tests and the HIP path's tests/bench can feed the two
sides identical inputs without sharing any computation.

Recipe (stands in for the paper's trained mesh-generation backbone, whose
weights and test meshes are not available): every tensor is drawn from
``numpy.random.Generator(PCG64(seed))`` in a fixed order, weights N(0, 0.02),
draft-head matrices identity + N(0, 0.01), gains 1, biases 0, condition
prefixes / condition tokens N(0, 1).  For bf16 configurations each value is
rounded once to bf16 (round-to-nearest-even) so that every consumer reads the
same bits; arrays are returned as float32 holding exactly those values.
"""
from __future__ import annotations

import numpy as np

# --- model/workload shapes -------------------------------------------------
# Shapes of the synthetic workloads.  K (n_draft) is the paper's D, the number
# of decoding heads (Sec. 4.1); vocabularies are mesh-sized (Table 1).  Optional
# key head_kind: "mlp" (default) or "ca" (cross-attention heads, needs n_cond > 0).
CONFIGS = {
    # tiny fp32 correctness model
    "c0": dict(n_layers=2, d_model=128, n_heads=4, head_dim=32, d_ffn=512, vocab=512,
               n_draft=4, n_cond=0, dtype="f32", prefix=64, batch=1, seed=0,
               max_ctx=1024, gen_tokens=512),
    # single-sequence latency model
    "c1": dict(n_layers=24, d_model=1024, n_heads=16, head_dim=64, d_ffn=4096, vocab=4096,
               n_draft=4, n_cond=0, dtype="bf16", prefix=257, batch=1, seed=1,
               max_ctx=4608, gen_tokens=4096),
    # batched, top-8 acceptance at temperature 0.8
    "c2": dict(n_layers=24, d_model=1024, n_heads=16, head_dim=64, d_ffn=4096, vocab=4096,
               n_draft=6, n_cond=0, dtype="bf16", prefix=257, batch=16, seed=1,
               max_ctx=8192, gen_tokens=0),
    # cross-attention-conditioned backbone
    "c3": dict(n_layers=24, d_model=1536, n_heads=24, head_dim=64, d_ffn=6144, vocab=8192,
               n_draft=4, n_cond=2048, dtype="bf16", prefix=0, batch=8, seed=3,
               max_ctx=16384, gen_tokens=0),
    # throughput sweep backbone (batch and K vary)
    "c4": dict(n_layers=12, d_model=1024, n_heads=16, head_dim=64, d_ffn=4096, vocab=4096,
               n_draft=4, n_cond=0, dtype="bf16", prefix=257, batch=1, seed=4,
               max_ctx=10240, gen_tokens=0),
}

ROPE_THETA = 10000.0
RMS_EPS = 1e-6
SOS = 0


def get_config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    cfg["name"] = name
    cfg.setdefault("rope_theta", ROPE_THETA)
    cfg.setdefault("rms_eps", RMS_EPS)
    return cfg


def tiny_config(**overrides) -> dict:
    """A few-thousand-parameter model for brute-force checks."""
    cfg = dict(n_layers=2, d_model=32, n_heads=2, head_dim=16, d_ffn=64, vocab=16,
               n_draft=3, n_cond=0, dtype="f32", prefix=5, batch=1, seed=7,
               max_ctx=256, gen_tokens=40, name="tiny",
               rope_theta=ROPE_THETA, rms_eps=RMS_EPS)
    cfg.update(overrides)
    return cfg


# --- bf16 rounding (storage format only) -------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> uint16 bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bf16, returned as float32."""
    return bf16_to_f32(bf16_bits(x))


def _store(cfg: dict, x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    return bf16_round(x) if cfg["dtype"] == "bf16" else x


# --- weights -----------------------------------------------------------------
def tensor_order(cfg: dict) -> list[tuple[str, tuple[int, ...]]]:
    """Names and shapes of all weight tensors, in canonical file order.

    All matrices are [out_features][in_features], row-major.
    """
    d, F, V, L, K = cfg["d_model"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"], cfg["n_draft"]
    out = [("E", (V, d))]
    for l in range(L):
        out += [(f"l{l}.g1", (d,)), (f"l{l}.Wqkv", (3 * d, d)), (f"l{l}.Wo", (d, d))]
        if cfg["n_cond"] > 0:
            out += [(f"l{l}.gc", (d,)), (f"l{l}.Wcq", (d, d)), (f"l{l}.Wckv", (2 * d, d)),
                    (f"l{l}.Wco", (d, d))]
        out += [(f"l{l}.g2", (d,)), (f"l{l}.W1", (F, d)), (f"l{l}.W2", (d, F))]
    out += [("gf", (d,)), ("WU", (V, d))]
    for k in range(1, K + 1):
        if cfg.get("head_kind", "mlp") == "ca":     # cross-attention decoding head with its own unembedding (Eq. 4)
            out += [(f"h{k}.Wq", (d, d)), (f"h{k}.Wkv", (2 * d, d)), (f"h{k}.Wo", (d, d)), (f"h{k}.WU", (V, d))]
        else:
            out += [(f"h{k}.W", (d, d)), (f"h{k}.b", (d,))]
    return out


def make_weights(cfg: dict, seed: int | None = None, perturb: bool = False) -> dict:
    """Random-init weights.  ``perturb`` additionally randomises gains (N(1,0.1))
    and head biases (N(0,0.02)) so tests exercise them; the benchmark recipe
    keeps gains 1 and biases 0."""
    rng = np.random.Generator(np.random.PCG64(cfg["seed"] if seed is None else seed))
    d = cfg["d_model"]
    w = {}
    for name, shape in tensor_order(cfg):
        leaf = name.split(".")[-1]
        if leaf in ("g1", "g2", "gc", "gf"):
            x = np.ones(shape, np.float32)
            if perturb:
                x = x + 0.1 * rng.standard_normal(shape, dtype=np.float32)
        elif leaf == "b":
            x = np.zeros(shape, np.float32)
            if perturb:
                x = 0.02 * rng.standard_normal(shape, dtype=np.float32)
        elif name.startswith("h") and leaf == "W":
            x = np.eye(d, dtype=np.float32) + 0.01 * rng.standard_normal(shape, dtype=np.float32)
        else:
            x = 0.02 * rng.standard_normal(shape, dtype=np.float32)
        w[name] = _store(cfg, x)
    return w


def pack_canonical(cfg: dict, w: dict) -> np.ndarray:
    """Concatenate all tensors in canonical order into one flat array of the
    storage type (uint16 bf16 bit patterns, or float32)."""
    parts = []
    for name, shape in tensor_order(cfg):
        x = w[name]
        assert x.shape == shape, (name, x.shape, shape)
        parts.append(bf16_bits(x).ravel() if cfg["dtype"] == "bf16" else
                     np.ascontiguousarray(x, np.float32).ravel())
    return np.concatenate(parts)


# --- activations / tokens ------------------------------------------------------
def make_prefix(cfg: dict, n_seq: int, P: int | None = None, seed: int | None = None) -> np.ndarray:
    """Condition prefix embeddings [n_seq][P][d] ~ N(0,1); sequence b is seeded
    independently with (seed, b)."""
    P = cfg["prefix"] if P is None else P
    seed = cfg["seed"] if seed is None else seed
    out = np.empty((n_seq, P, cfg["d_model"]), np.float32)
    for b in range(n_seq):
        rng = np.random.Generator(np.random.PCG64([seed, 1000 + b]))
        out[b] = rng.standard_normal((P, cfg["d_model"]), dtype=np.float32)
    return _store(cfg, out)


def make_cond(cfg: dict, n_seq: int, seed: int | None = None) -> np.ndarray | None:
    """Cross-attention condition tokens [n_seq][n_cond][d] ~ N(0,1)."""
    if cfg["n_cond"] == 0:
        return None
    seed = cfg["seed"] if seed is None else seed
    out = np.empty((n_seq, cfg["n_cond"], cfg["d_model"]), np.float32)
    for b in range(n_seq):
        rng = np.random.Generator(np.random.PCG64([seed, 2000 + b]))
        out[b] = rng.standard_normal((cfg["n_cond"], cfg["d_model"]), dtype=np.float32)
    return _store(cfg, out)


def first_block(cfg: dict, n_seq: int, seed: int | None = None) -> np.ndarray:
    """First draft block per sequence: [SOS, K candidates uniform on {0..V-1}]
    (Alg. 1, initialisation line)."""
    seed = cfg["seed"] if seed is None else seed
    rng = np.random.Generator(np.random.PCG64([seed, 3000]))
    blk = rng.integers(0, cfg["vocab"], size=(n_seq, cfg["n_draft"] + 1), dtype=np.int64)
    blk[:, 0] = SOS
    return blk.astype(np.int32)


def make_kv_fill(cfg: dict, n_seq: int, n_pos: int, seed: int | None = None) -> np.ndarray:
    """Synthetic cache contents for long-context cases: array
    [n_layers][2][n_seq][n_heads][n_pos][head_dim], N(0, 0.64) like projected
    unit-RMS activations under N(0,0.02) weights at d=1024."""
    seed = cfg["seed"] if seed is None else seed
    rng = np.random.Generator(np.random.PCG64([seed, 4000]))
    shape = (cfg["n_layers"], 2, n_seq, cfg["n_heads"], n_pos, cfg["head_dim"])
    x = 0.64 * rng.standard_normal(shape, dtype=np.float32)
    return _store(cfg, x)
