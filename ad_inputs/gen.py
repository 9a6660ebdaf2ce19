"""Seeded generators for every synthetic input of the five workloads.

Everything here is a draw from numpy's ``default_rng(seed)`` or an integer edit of a
token list that the caller supplies.  No Transformer arithmetic, no rounding, no
position table: each consumer (the CPU oracle, the HIP library) does its own.

Weight tensors are named; a matrix is always stored ``[out_features, in_features]``
so that ``y = x @ W.T + b``.  One model = shared embedding + encoder + decoder; the
verifier and the drafter are two such models with different seeds.
"""
from __future__ import annotations

import numpy as np

# Reserved token ids.  Content tokens are drawn from [FIRST_CONTENT, vocab).
SPECIAL = {"bos": 0, "pad": 1, "eos": 2, "unk": 3, "mask": 4}
FIRST_CONTENT = 5

DIMS = {
    # name: enc layers, dec layers, d_model, heads, ffn, vocab
    "tiny": dict(enc_layers=2, dec_layers=2, d_model=128, n_heads=4, d_ffn=512, vocab=2000),
    "base": dict(enc_layers=6, dec_layers=6, d_model=512, n_heads=8, d_ffn=2048, vocab=32000),
    "big": dict(enc_layers=6, dec_layers=6, d_model=1024, n_heads=16, d_ffn=4096, vocab=32000),
    # deep encoder, shallow decoder at the big width (the paper's second input-guided model) and a
    # small model of the same asymmetry for parity tests
    "deep_shallow": dict(enc_layers=12, dec_layers=2, d_model=1024, n_heads=16, d_ffn=4096, vocab=32000),
    "tiny_deep": dict(enc_layers=3, dec_layers=1, d_model=128, n_heads=4, d_ffn=512, vocab=2000),
    # heads of width 128 (the widest the attention kernels take)
    "wide_head": dict(enc_layers=2, dec_layers=2, d_model=256, n_heads=2, d_ffn=512, vocab=2000),
    # small shapes for brute-force tests of the invariant
    "nano": dict(enc_layers=1, dec_layers=1, d_model=16, n_heads=2, d_ffn=32, vocab=8),
    "micro": dict(enc_layers=1, dec_layers=2, d_model=32, n_heads=2, d_ffn=64, vocab=64),
}

# The five workloads.  `dtype` is the arithmetic contract of the HIP path.
CONFIGS = {
    0: dict(model="tiny", dtype="fp32", mode="positional", batch=1, n_sent=1, src_len=("fixed", 24),
            max_out=("fixed", 32), k=8, rate=0.1, seed=1000),
    1: dict(model="base", dtype="bf16", mode="guide", batch=1, n_sent=256, src_len=("normal", 25, 8, 5, 64),
            max_out=("src",), rate=0.1, seed=1001),
    2: dict(model="base", dtype="bf16", mode="guide", batch=32, n_sent=256, src_len=("uniform", 10, 60),
            max_out=("src",), rate=0.1, seed=1002),
    3: dict(model="base", dtype="bf16", mode="positional", drafter=True, batch=1, n_sent=256,
            src_len=("uniform", 20, 80), max_out=("src",), k=25, rate=0.3, seed=1003),
    4: dict(model="big", dtype="bf16", mode="positional", drafter=True, batch=8, n_sent=32,
            src_len=("fixed", 512), max_out=("fixed", 128), k=25, rate=0.3, seed=1004),
    # input-guided decoding with the deep-encoder / shallow-decoder model, lengths as workload 1
    5: dict(model="deep_shallow", dtype="bf16", mode="guide", batch=1, n_sent=64, src_len=("normal", 25, 8, 5, 64),
            max_out=("src",), rate=0.1, seed=1005),
}


def model_dims(name: str) -> dict:
    return dict(DIMS[name])


def _attn_spec(prefix: str, d: int):
    out = []
    for p in ("q", "k", "v", "o"):
        out.append((f"{prefix}.w{p}", (d, d), "matrix"))
        out.append((f"{prefix}.b{p}", (d,), "bias"))
    return out


def _ln_spec(prefix: str, d: int):
    return [(f"{prefix}.g", (d,), "ln_gain"), (f"{prefix}.b", (d,), "ln_bias")]


def _ffn_spec(prefix: str, d: int, f: int):
    return [(f"{prefix}.w1", (f, d), "matrix"), (f"{prefix}.b1", (f,), "bias"),
            (f"{prefix}.w2", (d, f), "matrix"), (f"{prefix}.b2", (d,), "bias")]


def param_spec(dims: dict, tie_output: bool = False):
    """Ordered list of (name, shape, kind) for one encoder-decoder model.

    `emb` is the one embedding table of the joint source-target vocabulary (encoder
    and decoder inputs).  `out.w` is the output projection; with tie_output it is
    absent and `emb` serves as the output projection too."""
    d, f, v = dims["d_model"], dims["d_ffn"], dims["vocab"]
    spec = [("emb", (v, d), "matrix")]
    if not tie_output:
        spec.append(("out.w", (v, d), "matrix"))
    for l in range(dims["enc_layers"]):
        spec += _attn_spec(f"enc.{l}.self", d) + _ln_spec(f"enc.{l}.ln1", d)
        spec += _ffn_spec(f"enc.{l}.ffn", d, f) + _ln_spec(f"enc.{l}.ln2", d)
    for l in range(dims["dec_layers"]):
        spec += _attn_spec(f"dec.{l}.self", d) + _ln_spec(f"dec.{l}.ln1", d)
        spec += _attn_spec(f"dec.{l}.cross", d) + _ln_spec(f"dec.{l}.ln2", d)
        spec += _ffn_spec(f"dec.{l}.ffn", d, f) + _ln_spec(f"dec.{l}.ln3", d)
    return spec


def init_weights(dims: dict, seed: int, std: float = 0.02, tie_output: bool = False) -> dict:
    """fp32 tensors: matrices, embeddings and biases N(0, std); LN gain 1+N(0,std), LN bias N(0,std)."""
    rng = np.random.default_rng(seed)
    out = {}
    for name, shape, kind in param_spec(dims, tie_output):
        w = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        if kind == "ln_gain":
            w = w + np.float32(1.0)
        out[name] = np.ascontiguousarray(w, dtype=np.float32)
    return out


def _draw_len(rule, rng, n):
    kind = rule[0]
    if kind == "fixed":
        return np.full(n, rule[1], dtype=np.int32)
    if kind == "uniform":
        return rng.integers(rule[1], rule[2] + 1, size=n).astype(np.int32)
    if kind == "normal":
        x = np.rint(rng.normal(rule[1], rule[2], size=n))
        return np.clip(x, rule[3], rule[4]).astype(np.int32)
    raise ValueError(kind)


def draw_sources(cfg: dict, vocab: int, n_sent: int | None = None):
    """Source sentences of one workload: list of int32 arrays of content ids, and max_out per sentence."""
    rng = np.random.default_rng(cfg["seed"])
    n = cfg["n_sent"] if n_sent is None else n_sent
    lens = _draw_len(cfg["src_len"], rng, n)
    srcs = [rng.integers(FIRST_CONTENT, vocab, size=int(L)).astype(np.int32) for L in lens]
    if cfg["max_out"][0] == "src":
        max_out = lens.copy()
    else:
        max_out = np.full(n, cfg["max_out"][1], dtype=np.int32)
    return srcs, max_out


def _other_content(rng, vocab: int, avoid: int) -> int:
    """Uniform content id different from `avoid`."""
    t = int(rng.integers(FIRST_CONTENT, vocab - 1))
    if t >= avoid and avoid >= FIRST_CONTENT:
        t += 1
    return t


def edit_guide(g, rate: float, seed: int, vocab: int) -> np.ndarray:
    """Guide sequence for input-guided decoding: `g` with i.i.d. per-token edits.

    Each token of g is edited with probability `rate`; an edit is, with equal
    probability, a substitution, a deletion, or an insertion of a random token
    before it.  Returns content ids only (no sentinels)."""
    rng = np.random.default_rng(seed)
    out = []
    for t in np.asarray(g, dtype=np.int64).tolist():
        if rng.random() < rate:
            kind = int(rng.integers(0, 3))
            if kind == 0:
                out.append(_other_content(rng, vocab, t))
            elif kind == 1:
                pass
            else:
                out.append(_other_content(rng, vocab, t))
                out.append(t)
        else:
            out.append(t)
    return np.asarray(out, dtype=np.int32)


def positional_draft(g, rate: float, seed: int, vocab: int):
    """Positional draft D with D[p] = g[p] except at pre-drawn positions (i.i.d., `rate`)
    where a different content id is substituted.  Returns (D, wrong_mask)."""
    rng = np.random.default_rng(seed)
    g = np.asarray(g, dtype=np.int32)
    wrong = rng.random(g.shape[0]) < rate
    d = g.copy()
    for p in np.nonzero(wrong)[0].tolist():
        d[p] = _other_content(rng, vocab, int(g[p]))
    return d, wrong
