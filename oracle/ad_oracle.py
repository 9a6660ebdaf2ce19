"""CPU oracle for Aggressive Decoding — TEST INFRASTRUCTURE, not a product path.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It shares no code with the HIP library and never calls it.

What it computes, each part written out from the paper's definitions:

* the encoder-decoder Transformer that scores P(y_{i+1} | y_{<=i}, x) (Section 2,
  training equation: all positions scored in parallel under teacher forcing);
* greedy autoregressive decoding (Section 2, inference equation; Section 3.1.2);
* the parallel verification step (Section 3.2, verify paragraph: the verifier
  equation, the bifurcation position c, the accepted block);
* Input-guided Aggressive Decoding (Section 3.1, Algorithm 1);
* Generalized Aggressive Decoding (Section 3.2, draft and verify substeps) with a
  non-autoregressive block drafter (Section 3.2.1);
* the relaxed verification of GAD++ (Section 3.2.3: a drafted token stands if it is among the
  verifier's top-beta candidates and its log-likelihood is within tau of the top-1's).

Arithmetic is plain numpy in the dtype chosen at construction (float32 by default,
float64 for a reference of higher precision).  A matmul is the only library
primitive.  Nothing is blocked, fused or reordered.

Readings where the paper is silent (the Transformer is the conventional one):
post-LN residual blocks, ReLU, embedding scaled by sqrt(d) plus sinusoidal
positions, one embedding table for the joint vocabulary (encoder and decoder inputs),
an output projection `out.w` of its own unless the parameter set omits it (then the
embedding table is the output projection too), biases on all projections but the
output one, LayerNorm eps 1e-5, scores scaled by
1/sqrt(d_head), argmax ties go to the lowest token id.

`contract=True` additionally rounds to bfloat16 exactly where the bf16 HIP path
does (weight matrices; every GEMM's left operand; Q, K, V; softmax numerators
before they multiply V), so that a disagreement between the two can be classified
as a legitimate near-tie.  With `contract=False` nothing is rounded.

Pins: see tests/test_oracle_*.py (stock-library Transformer special case, closed
forms for positions/LayerNorm/softmax, teacher-forcing equivalence, brute force of
the greedy-identity invariant, closed-form iteration counts).
Parity unpinned: absolute logits of the paper's trained models and its task
metrics (no weights or data exist here).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

NEVER = -1  # draft id that equals no prediction (Algorithm 1's trailing [PAD])


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even); result keeps the input dtype."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(a.dtype)


def sinusoid_positions(n_pos: int, d: int, dtype=np.float64) -> np.ndarray:
    """PE(p, 2i) = sin(p / 10000^(2i/d)), PE(p, 2i+1) = cos(p / 10000^(2i/d)); p is 0-based."""
    pe = np.zeros((n_pos, d), dtype=np.float64)
    for i in range(d // 2):
        freq = 1.0 / (10000.0 ** (2.0 * i / d))
        for p in range(n_pos):
            pe[p, 2 * i] = math.sin(p * freq)
            pe[p, 2 * i + 1] = math.cos(p * freq)
    return pe.astype(dtype)


def argmax_lowest(v: np.ndarray) -> int:
    """Index of the maximum; the lowest index among equal maxima."""
    return int(np.flatnonzero(v == v.max())[0])


class Model:
    """One encoder-decoder Transformer (verifier or drafter)."""

    def __init__(self, dims: dict, params: dict, dtype=np.float32, contract: bool = False,
                 max_pos: int = 1024):
        self.d = dims["d_model"]
        self.H = dims["n_heads"]
        self.dh = self.d // self.H
        self.F = dims["d_ffn"]
        self.V = dims["vocab"]
        self.n_enc = dims["enc_layers"]
        self.n_dec = dims["dec_layers"]
        if contract and dtype != np.float64:
            # In float32 a BLAS matmul's rounding depends on how many rows share the
            # call; a bf16 rounding point turns that 1e-7 into 4e-3 and the greedy
            # identity is lost at near-ties.  float64 keeps the oracle row-count blind.
            raise ValueError("contract mode computes in float64")
        self.dtype = dtype
        self.contract = contract
        self.p = {}
        for name, w in params.items():
            w = np.asarray(w, dtype=np.float32)
            if contract and w.ndim == 2:
                w = bf16_round(w)
            self.p[name] = w.astype(dtype)
        self.pe = sinusoid_positions(max_pos, self.d, dtype)
        self.scale = dtype(1.0 / math.sqrt(self.dh))
        self.sqrt_d = dtype(math.sqrt(self.d))

    # ---- elementary pieces -------------------------------------------------
    def _r(self, a):
        """bf16 rounding point of the contract (identity otherwise)."""
        return bf16_round(a) if self.contract else a

    def linear(self, x, w, b=None):
        y = self._r(x) @ self.p[w].T
        if b is not None:
            y = y + self.p[b]
        return y.astype(self.dtype)

    def layer_norm(self, x, prefix):
        mu = x.mean(axis=-1, keepdims=True)
        var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
        y = (x - mu) / np.sqrt(var + self.dtype(1e-5))
        return (y * self.p[prefix + ".g"] + self.p[prefix + ".b"]).astype(self.dtype)

    def embed(self, tokens, positions):
        e = self.p["emb"][np.asarray(tokens, dtype=np.int64)]
        return (e * self.sqrt_d + self.pe[np.asarray(positions, dtype=np.int64)]).astype(self.dtype)

    def attention(self, q, k, v, n_visible):
        """Multi-head scaled dot-product attention.  Row i sees keys [0, n_visible[i])."""
        q, k, v = self._r(q), self._r(k), self._r(v)
        T = q.shape[0]
        out = np.zeros((T, self.d), dtype=self.dtype)
        for h in range(self.H):
            sl = slice(h * self.dh, (h + 1) * self.dh)
            s = (q[:, sl] @ k[:, sl].T) * self.scale
            for i in range(T):
                s[i, n_visible[i]:] = -np.inf
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            out[:, sl] = (self._r(e) @ v[:, sl]) / e.sum(axis=1, keepdims=True)
        return out

    def ffn(self, x, prefix):
        hdn = np.maximum(self.linear(x, prefix + ".w1", prefix + ".b1"), 0)
        return self.linear(hdn, prefix + ".w2", prefix + ".b2")

    def logits(self, x):
        return self.linear(x, "out.w" if "out.w" in self.p else "emb")

    # ---- encoder -----------------------------------------------------------
    def encode(self, src):
        """memory = Encoder(x_1..x_n): bidirectional self-attention, no sentinels."""
        n = len(src)
        x = self.embed(src, np.arange(n))
        see_all = [n] * n
        for l in range(self.n_enc):
            a = f"enc.{l}.self"
            q = self.linear(x, a + ".wq", a + ".bq")
            k = self.linear(x, a + ".wk", a + ".bk")
            v = self.linear(x, a + ".wv", a + ".bv")
            att = self.attention(q, k, v, see_all)
            x = self.layer_norm(x + self.linear(att, a + ".wo", a + ".bo"), f"enc.{l}.ln1")
            x = self.layer_norm(x + self.ffn(x, f"enc.{l}.ffn"), f"enc.{l}.ln2")
        return x

    def cross_kv(self, memory):
        """Keys and values of the encoder memory for every decoder layer."""
        out = []
        for l in range(self.n_dec):
            c = f"dec.{l}.cross"
            out.append((self.linear(memory, c + ".wk", c + ".bk"),
                        self.linear(memory, c + ".wv", c + ".bv")))
        return out

    # ---- decoder, full recomputation -----------------------------------------
    def decode_full(self, memory, tokens, causal: bool = True):
        """Logits at every row of `tokens` (positions 0..T-1), recomputing everything.

        causal=True: row i sees rows 0..i (autoregressive scoring).
        causal=False: every row sees every row (the block drafter)."""
        T = len(tokens)
        S = memory.shape[0]
        x = self.embed(tokens, np.arange(T))
        vis = [i + 1 for i in range(T)] if causal else [T] * T
        mem_kv = self.cross_kv(memory)
        for l in range(self.n_dec):
            a, c = f"dec.{l}.self", f"dec.{l}.cross"
            q = self.linear(x, a + ".wq", a + ".bq")
            k = self.linear(x, a + ".wk", a + ".bk")
            v = self.linear(x, a + ".wv", a + ".bv")
            att = self.attention(q, k, v, vis)
            x = self.layer_norm(x + self.linear(att, a + ".wo", a + ".bo"), f"dec.{l}.ln1")
            q = self.linear(x, c + ".wq", c + ".bq")
            att = self.attention(q, mem_kv[l][0], mem_kv[l][1], [S] * T)
            x = self.layer_norm(x + self.linear(att, c + ".wo", c + ".bo"), f"dec.{l}.ln2")
            x = self.layer_norm(x + self.ffn(x, f"dec.{l}.ffn"), f"dec.{l}.ln3")
        return self.logits(x)


class DecoderState:
    """Incremental autoregressive decoder of one sequence: keeps the self-attention
    keys and values of the rows accepted so far; rows past `length` are dead."""

    def __init__(self, model: Model, memory):
        self.m = model
        self.S = memory.shape[0]
        self.mem_kv = model.cross_kv(memory)
        self.K = [np.zeros((0, model.d), dtype=model.dtype) for _ in range(model.n_dec)]
        self.V = [np.zeros((0, model.d), dtype=model.dtype) for _ in range(model.n_dec)]
        self.length = 0

    def forward(self, tokens):
        """Feed `tokens` at positions length..length+k-1 under the causal mask; append
        their keys/values; return logits [k, V].  `length` itself is not advanced."""
        m, L, k = self.m, self.length, len(tokens)
        x = m.embed(tokens, L + np.arange(k))
        vis = [L + i + 1 for i in range(k)]
        for l in range(m.n_dec):
            a, c = f"dec.{l}.self", f"dec.{l}.cross"
            q = m.linear(x, a + ".wq", a + ".bq")
            self.K[l] = np.concatenate([self.K[l][:L], m.linear(x, a + ".wk", a + ".bk")], axis=0)
            self.V[l] = np.concatenate([self.V[l][:L], m.linear(x, a + ".wv", a + ".bv")], axis=0)
            att = m.attention(q, self.K[l], self.V[l], vis)
            x = m.layer_norm(x + m.linear(att, a + ".wo", a + ".bo"), f"dec.{l}.ln1")
            q = m.linear(x, c + ".wq", c + ".bq")
            att = m.attention(q, self.mem_kv[l][0], self.mem_kv[l][1], [self.S] * k)
            x = m.layer_norm(x + m.linear(att, c + ".wo", c + ".bo"), f"dec.{l}.ln2")
            x = m.layer_norm(x + m.ffn(x, f"dec.{l}.ffn"), f"dec.{l}.ln3")
        return m.logits(x)

    def keep(self, new_length: int):
        """Rollback: rows at and beyond `new_length` are discarded."""
        self.length = new_length


@dataclass
class Stats:
    iterations: int = 0        # verify forwards (an AR step is a verify of one row)
    rows_verified: int = 0     # decoder rows fed over all verify forwards
    draft_rows: int = 0        # decoder rows fed to the drafter
    accepted: list = field(default_factory=list)  # tokens appended per iteration


def _truncate(tokens, out_len, max_len, eos):
    """Tokens actually appended: cut after the first EOS and at max_len."""
    keep = []
    for t in tokens:
        if out_len + len(keep) >= max_len:
            break
        keep.append(int(t))
        if t == eos:
            break
    return keep


def greedy(model: Model, src, max_len: int, eos: int, bos: int, incremental: bool = True,
           return_logits: bool = False):
    """o_0=[BOS]; o_{t+1} = argmax P(. | o_{<=t}, x) until [EOS] or max_len tokens."""
    memory = model.encode(src)
    out, rows = [], []
    st = DecoderState(model, memory) if incremental else None
    prev = bos
    while len(out) < max_len:
        if incremental:
            lg = st.forward([prev])[0]
            st.keep(st.length + 1)
        else:
            lg = model.decode_full(memory, [bos] + out, causal=True)[-1]
        prev = argmax_lowest(lg)
        out.append(prev)
        rows.append(lg)
        if prev == eos:
            break
    return (out, np.stack(rows)) if return_logits else out


def gadpp_requirement(row_logits: np.ndarray, token: int, beta: int, tau: float) -> bool:
    """GAD++ requirement for one position (Section 3.2.3, its two inequalities), written out
    from the definition: log P(token) >= log P(the beta-th ranked token) and
    log P(top-1) - log P(token) <= tau.

    log P = logit - logsumexp(logits), so both inequalities are statements about logits: the
    normaliser is the same on both sides and cancels.  They are decided on the float32 values of
    the logits (the precision the HIP path decides them in); the gap is one float32 subtraction.
    The never-matching id meets no requirement."""
    if token < 0:
        return False
    lg = np.asarray(row_logits, dtype=np.float32)
    ranked = np.sort(lg)[::-1]                   # descending: ranked[b - 1] is the b-th ranked score
    beta = min(int(beta), lg.shape[0])
    in_top_beta = lg[token] >= ranked[beta - 1]
    within_tau = np.float32(ranked[0] - lg[token]) <= np.float32(tau)
    return bool(in_top_beta and within_tau)


def verify(st: DecoderState, pending: int, draft, return_logits: bool = False, beta: int = 1, tau: float = 0.0):
    """Parallel verification of a k-token draft after the accepted prefix.

    Rows fed: (o_j, d_1, .., d_{k-1}); row i predicts position j+i.  The last draft
    token is compared but never fed.  o_hat_i = arg max of row i (verifier equation); with
    beta > 1 (GAD++, Section 3.2.3) o_hat_i = d_i wherever d_i meets the GAD++ requirement.
    c = first i with d_i != o_hat_i, else k.
    Accepted block = (d_1..d_{c-1}, o_hat_c) = o_hat_{1..c}.  The caller appends and
    calls st.keep()."""
    k = len(draft)
    fed = [int(pending)] + [int(t) for t in draft[:k - 1]]
    assert min(fed) >= 0, "the never-matching id may only be the last draft token"
    lg = st.forward(fed)
    o_hat = [argmax_lowest(lg[i]) for i in range(k)]
    if beta > 1:
        for i in range(k):
            if gadpp_requirement(lg[i], int(draft[i]), beta, tau):
                o_hat[i] = int(draft[i])
    c = k
    for i in range(k):
        if int(draft[i]) != o_hat[i]:
            c = i + 1
            break
    return (o_hat, c, lg) if return_logits else (o_hat, c)


def suffix_match(o, x):
    """Algorithm 1's test: the shortest suffix o_{j-q..j} (q >= 0) that occurs exactly
    once in x gives its end index i; none if some suffix never occurs or q runs out.
    `o` = (o_0..o_j), `x` = guide with sentinels."""
    j = len(o) - 1
    for q in range(j + 1):
        suf = list(o[j - q:])
        ends = [i for i in range(q, len(x)) if list(x[i - q:i + 1]) == suf]
        if len(ends) == 1:
            return ends[0]
        if len(ends) == 0:
            return None
    return None


def iad(model: Model, src, guide, max_len: int, eos: int, bos: int, k_max: int | None = None):
    """Algorithm 1.  x = ([BOS], guide_1..guide_n, [PAD]); [PAD] is the id that never
    matches, so a bifurcation always exists.  Without a suffix match the step is an
    ordinary autoregressive one (a verify of the single never-matching draft)."""
    x = [bos] + [int(t) for t in guide] + [NEVER]
    st = DecoderState(model, model.encode(src))
    o, stats = [bos], Stats()
    while o[-1] != eos and len(o) - 1 < max_len:
        i = suffix_match(o, x)
        draft = x[i + 1:] if i is not None else []
        if not draft:
            draft = [NEVER]
        room = max_len - (len(o) - 1)
        cap = room if k_max is None else min(room, k_max)
        draft = draft[:cap]
        o_hat, c = verify(st, o[-1], draft)
        add = _truncate(o_hat[:c], len(o) - 1, max_len, eos)
        st.keep(st.length + len(add))
        o += add
        stats.iterations += 1
        stats.rows_verified += len(draft)
        stats.accepted.append(len(add))
    return o[1:], stats


def draft_nat(drafter: Model, memory, prefix, k: int, mask_id: int):
    """Block drafter: decoder input (o_0..o_j, [MASK] x k), bidirectional attention;
    the k drafted tokens are the argmax at the k mask rows."""
    lg = drafter.decode_full(memory, list(prefix) + [mask_id] * k, causal=False)
    return [argmax_lowest(lg[len(prefix) + i]) for i in range(k)]


def gad(verifier: Model, src, k: int, max_len: int, eos: int, bos: int, drafter: Model | None = None,
        mask_id: int | None = None, draft_override=None, beta: int = 1, tau: float = 0.0):
    """Draft-then-verify iterations until [EOS] or max_len.

    The draft comes from the block drafter, or, if `draft_override` (a positional
    sequence D with D[p] proposed for output position p) is given, from D; when both
    are given the drafter still runs and its output is discarded.  beta > 1 verifies with the
    GAD++ requirement (the output then need not be the greedy one)."""
    st = DecoderState(verifier, verifier.encode(src))
    mem_d = drafter.encode(src) if drafter is not None else None
    o, stats = [bos], Stats()
    while o[-1] != eos and len(o) - 1 < max_len:
        j = len(o) - 1
        kk = min(k, max_len - j)
        if drafter is not None:
            draft = draft_nat(drafter, mem_d, o, kk, mask_id)
            stats.draft_rows += len(o) + kk
        if draft_override is not None:
            # D has no entry past its end: the block stops there (at least one row)
            draft = [int(t) for t in draft_override[j:j + kk]] or [NEVER]
        o_hat, c = verify(st, o[-1], draft, beta=beta, tau=tau)
        add = _truncate(o_hat[:c], j, max_len, eos)
        st.keep(st.length + len(add))
        o += add
        stats.iterations += 1
        stats.rows_verified += len(draft)
        stats.accepted.append(len(add))
    return o[1:], stats
