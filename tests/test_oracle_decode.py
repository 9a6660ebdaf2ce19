"""Pins of the oracle's decoding logic: teacher-forcing equivalence, the greedy-identity
invariant by brute force, closed-form iteration structure, suffix matching.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from ad_inputs import SPECIAL, edit_guide, init_weights, model_dims, positional_draft
from oracle import ad_oracle as O

BOS, EOS, MASK = SPECIAL["bos"], SPECIAL["eos"], SPECIAL["mask"]


def make(name, seed, dtype=np.float64, contract=False, tie=False):
    dims = model_dims(name)
    return dims, O.Model(dims, init_weights(dims, seed, tie_output=tie), dtype, contract=contract, max_pos=96)


def src_for(dims, seed, n):
    return np.random.default_rng(seed).integers(5, dims["vocab"], size=n).astype(np.int32)


# ------------------------------------------------------------ teacher forcing equivalence (Section 2)
@pytest.mark.parametrize("contract", [False, True])
def test_incremental_equals_full_recompute(contract):
    dims, m = make("micro", 21, contract=contract)
    src = src_for(dims, 1, 9)
    memory = m.encode(src)
    toks = [BOS] + list(src_for(dims, 2, 10))
    full = m.decode_full(memory, toks, causal=True)
    st = O.DecoderState(m, memory)
    got = []
    for chunk in ([0, 1], [2], [3, 4, 5, 6], [7, 8, 9, 10]):   # ragged blocks, appended one after another
        got.append(st.forward([toks[i] for i in chunk]))
        st.keep(st.length + len(chunk))
    assert np.allclose(np.concatenate(got), full, atol=1e-10)


def test_rollback_discards_rejected_rows():
    dims, m = make("micro", 22)
    src = src_for(dims, 3, 7)
    memory = m.encode(src)
    toks = [BOS] + list(src_for(dims, 4, 6))
    st = O.DecoderState(m, memory)
    st.forward(toks[:2]); st.keep(2)
    st.forward([9, 10, 11, 12])          # a rejected block: nothing kept
    st.keep(2)
    again = st.forward(toks[2:5])
    full = m.decode_full(memory, toks[:5])
    assert np.allclose(again, full[2:5], atol=1e-10)


def test_verify_rows_are_greedy_steps_and_k1_is_an_ar_step():
    dims, m = make("micro", 23)
    src = src_for(dims, 5, 8)
    g, glog = O.greedy(m, src, 12, EOS, BOS, return_logits=True)
    g2 = O.greedy(m, src, 12, EOS, BOS, incremental=False)
    assert g == g2
    st = O.DecoderState(m, m.encode(src))
    # a fully right draft: row i reproduces greedy step i
    o_hat, c, lg = O.verify(st, BOS, g[:6], return_logits=True)
    assert o_hat == g[:6] and c == 6
    assert np.allclose(lg, glog[:6], atol=1e-10)
    st.keep(3)
    # k = 1 with the never-matching id: an ordinary autoregressive step
    o_hat, c, lg = O.verify(st, g[2], [O.NEVER], return_logits=True)
    assert c == 1 and o_hat == [g[3]] and np.allclose(lg[0], glog[3], atol=1e-10)


# ------------------------------------------------------------ the invariant, by brute force
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_every_draft_yields_greedy_brute_force(seed):
    """For every prefix of the greedy output and EVERY draft in V^k (k<=3), the accepted
    block is the greedy continuation: matched draft prefix plus the first corrected token."""
    dims, m = make("nano", seed)
    V = dims["vocab"]
    src = src_for(dims, seed, 5)
    g = O.greedy(m, src, 6, EOS, BOS)
    memory = m.encode(src)
    o = [BOS] + g
    for j in range(len(g)):
        for k in (1, 2, 3):
            for draft in itertools.product(range(V), repeat=k):
                st = O.DecoderState(m, memory)
                if j:
                    st.forward(o[:j]); st.keep(j)
                o_hat, c = O.verify(st, o[j], list(draft))
                assert 1 <= c <= k
                cont = (g + [None] * k)[j:j + c]          # greedy continuation, where it exists
                for t in range(c):
                    if cont[t] is None or (t and g[j + t - 1] == EOS):
                        break                               # beyond the end of the greedy output
                    assert o_hat[t] == cont[t]
                # c is the first mismatch of draft vs o_hat, else k
                mism = [i for i in range(k) if draft[i] != o_hat[i]]
                assert c == (mism[0] + 1 if mism else k)


@pytest.mark.parametrize("seed", [2, 3, 4, 5])
def test_every_guide_yields_greedy_brute_force(seed):
    """Algorithm 1 with every guide of length <= 3 over the whole vocabulary."""
    dims, m = make("nano", seed)
    V = dims["vocab"]
    src = src_for(dims, seed + 10, 4)
    g = O.greedy(m, src, 6, EOS, BOS)
    n_multi = 0
    for n in range(0, 4):
        for guide in itertools.product(range(V), repeat=n):
            out, st = O.iad(m, src, list(guide), 6, EOS, BOS)
            assert out == g, (guide, out, g)
            assert sum(st.accepted) == len(g)
            n_multi += any(a > 1 for a in st.accepted)
    assert n_multi > 0 or len(g) < 2  # some guides really were accepted in blocks


@pytest.mark.parametrize("contract,tie", [(False, False), (True, False), (False, True)])
def test_all_right_all_wrong_random_drafts_tiny(contract, tie):
    dims, m = make("tiny", 1000, contract=contract, tie=tie)
    V = dims["vocab"]
    src = src_for(dims, 1000, 24)
    T, k = 32, 8
    g = O.greedy(m, src, T, EOS, BOS)
    assert len(g) == T or g[-1] == EOS
    T = len(g)
    # all right: ceil(T/k) verify forwards
    out, st = O.gad(m, src, k, 32, EOS, BOS, draft_override=g)
    assert out == g and st.iterations == math.ceil(T / k)
    # all wrong: T forwards, one token each
    wrong = [(t + 1 - 5) % (V - 5) + 5 for t in g]
    out, st = O.gad(m, src, k, 32, EOS, BOS, draft_override=wrong)
    assert out == g and st.iterations == T and set(st.accepted) == {1}
    # random substitutions: block boundaries are a function of the mask alone
    for s in range(3):
        D, bad = positional_draft(g, 0.1 + 0.2 * s, 50 + s, V)
        out, st = O.gad(m, src, k, 32, EOS, BOS, draft_override=D)
        assert out == g
        expect, j = [], 0
        while j < T:
            kk = min(k, T - j)
            w = [p for p in range(j, j + kk) if bad[p]]
            c = (w[0] - j + 1) if w else kk
            expect.append(c); j += c
        assert st.accepted == expect
    # guide = greedy output itself: a single verify forward (no edit, nothing to re-decode)
    out, st = O.iad(m, src, g, 32, EOS, BOS)
    assert out == g
    if len(set(g)) == len(g):
        assert st.iterations == 1
    # edited guides
    for s in range(3):
        out, st = O.iad(m, src, edit_guide(g, 0.1, s, V), 32, EOS, BOS)
        assert out == g
    # block size cap
    out, st = O.iad(m, src, g, 32, EOS, BOS, k_max=5)
    assert out == g and max(st.accepted) <= 5


def test_gad_with_block_drafter_is_greedy():
    dims, ver = make("micro", 31)
    _, dr = make("micro", 32)
    src = src_for(dims, 6, 10)
    g = O.greedy(ver, src, 14, EOS, BOS)
    for k in (1, 3, 5):
        out, st = O.gad(ver, src, k, 14, EOS, BOS, drafter=dr, mask_id=MASK)
        assert out == g
        assert st.draft_rows > 0 and st.rows_verified >= len(g)
    # the drafter's draft is a function of the prefix only: k masks, bidirectional
    mem = dr.encode(src)
    d3 = O.draft_nat(dr, mem, [BOS] + g[:4], 3, MASK)
    lg = dr.decode_full(mem, [BOS] + g[:4] + [MASK] * 3, causal=False)
    assert d3 == [int(np.argmax(lg[5 + i])) for i in range(3)]


def test_a_verifier_that_drafts_for_itself_accepts_everything():
    """If the drafter's proposal equals the verifier's own greedy continuation, every
    iteration accepts its whole block: iterations = ceil(T/k)."""
    dims, ver = make("micro", 33)
    src = src_for(dims, 7, 9)
    g = O.greedy(ver, src, 13, EOS, BOS)
    for k in (2, 4, 13):
        out, st = O.gad(ver, src, k, 13, EOS, BOS, draft_override=g)
        assert out == g and st.iterations == math.ceil(len(g) / k)


def test_eos_and_max_len_truncate_the_accepted_block():
    # find a nano model whose greedy output ends with EOS before max_len
    for seed in range(1, 60):
        dims, m = make("nano", seed)
        src = src_for(dims, seed, 4)
        g = O.greedy(m, src, 8, EOS, BOS)
        if g[-1] == EOS and 2 <= len(g) < 8:
            break
    else:
        pytest.skip("no EOS-terminated sample")
    # a draft that is right up to EOS and proposes more afterwards: nothing after EOS is kept
    D = g + [5, 6, 7, 5, 6, 7, 5, 6]
    out, st = O.gad(m, src, 8, 8, EOS, BOS, draft_override=D)
    assert out == g and st.iterations == 1
    out, st = O.iad(m, src, g[:-1] + [5, 6], 8, EOS, BOS)
    assert out == g
    # max_len in the middle of an accepted block
    out, st = O.gad(m, src, 8, len(g) - 1, EOS, BOS, draft_override=D)
    assert out == g[:-1]


# ------------------------------------------------------------ suffix match (Algorithm 1, the if-test)
def _occurrence_ends(sub, x):
    """Independent formulation through strings: end indices of (overlapping) occurrences."""
    s = "".join(chr(65 + t) for t in sub)
    xs = "".join(chr(65 + t) for t in x)
    ends, start = [], xs.find(s)
    while start != -1:
        ends.append(start + len(s) - 1)
        start = xs.find(s, start + 1)
    return ends


def test_suffix_match_brute_force():
    for n in range(1, 6):
        for x in itertools.product(range(3), repeat=n):
            for j in range(0, 4):
                for o in itertools.product(range(3), repeat=j + 1):
                    got = O.suffix_match(list(o), list(x))
                    expect = None
                    for q in range(j + 1):
                        ends = _occurrence_ends(o[j - q:], x)
                        if len(ends) == 1:
                            expect = ends[0]
                        if len(ends) <= 1:
                            break
                    assert got == expect


def test_suffix_match_worked_cases():
    # o_0 = x_0 = BOS is unique: the initial aggressive decoding is a suffix match at i = 0
    assert O.suffix_match([0], [0, 7, 8, 9, -1]) == 0
    # a repeated token needs a longer suffix to become unique
    assert O.suffix_match([0, 7, 8], [0, 7, 8, 7, 9, -1]) == 2
    assert O.suffix_match([0, 5, 7], [0, 7, 8, 7, 9, -1]) is None     # "7" twice, "5 7" never
    assert O.suffix_match([0, 8, 7], [0, 7, 8, 7, 9, -1]) == 3        # "8 7" once
    assert O.suffix_match([0, 6], [0, 7, 8, -1]) is None


# ------------------------------------------------------------ GAD++ requirement (Section 3.2.3)
def test_gadpp_requirement_worked_cases():
    """Hand-worked rows.  Scores 2.0 > 1.5 > 0.25 > -1.0: token 1 is ranked 2nd with gap 0.5,
    token 2 is ranked 3rd with gap 1.75."""
    row = np.array([2.0, 1.5, 0.25, -1.0])
    assert O.gadpp_requirement(row, 1, beta=2, tau=1.0)
    assert not O.gadpp_requirement(row, 1, beta=2, tau=0.25)      # in the top 2, gap too large
    assert O.gadpp_requirement(row, 1, beta=2, tau=0.5)           # the gap bound is inclusive
    assert not O.gadpp_requirement(row, 2, beta=2, tau=5.0)       # ranked 3rd
    assert O.gadpp_requirement(row, 2, beta=3, tau=1.75)          # the rank bound is inclusive
    assert not O.gadpp_requirement(row, 2, beta=3, tau=1.5)
    assert O.gadpp_requirement(row, 0, beta=1, tau=0.0)           # the top-1 token always stands
    assert not O.gadpp_requirement(row, O.NEVER, beta=4, tau=100.0)
    # equal scores: a token that ties with the beta-th ranked one is in the top beta
    tie = np.array([1.0, 0.5, 0.5, 0.5, -2.0])
    assert all(O.gadpp_requirement(tie, t, beta=2, tau=1.0) for t in (1, 2, 3))
    assert not O.gadpp_requirement(tie, 4, beta=4, tau=10.0)


def test_gadpp_requirement_equals_the_log_likelihood_definition_and_the_count_form():
    """Against the definition on log-likelihoods in float64 (log-softmax, ranking by a sort of
    its own) on rows whose scores and gaps are exact in float32 (multiples of 1/8), so that the
    precision of the decision plays no part; and against the count form the HIP path uses:
    token within the top beta <=> fewer than beta scores are strictly greater."""
    rng = np.random.default_rng(5)
    for trial in range(300):
        V = int(rng.integers(2, 12))
        row = rng.integers(-24, 25, size=V) / 8.0                  # ties do occur
        beta = int(rng.integers(1, V + 2))
        tau = float(rng.integers(0, 40)) / 8.0
        logp = row - (np.log(np.sum(np.exp(row - row.max()))) + row.max())
        order = sorted(range(V), key=lambda t: -logp[t])
        kth = logp[order[min(beta, V) - 1]]
        for t in range(V):
            want = bool(logp[t] >= kth - 1e-12 and logp[order[0]] - logp[t] <= tau + 1e-12)
            assert O.gadpp_requirement(row, t, beta, tau) == want
            count_form = int(np.sum(row > row[t])) < beta and row.max() - row[t] <= tau
            assert O.gadpp_requirement(row, t, beta, tau) == bool(count_form)


def test_gadpp_requirement_grows_with_beta_and_tau():
    rng = np.random.default_rng(6)
    row = rng.normal(size=40)
    for t in range(40):
        prev = False
        for beta, tau in ((1, 0.0), (2, 0.5), (3, 1.0), (5, 3.0), (40, 100.0)):
            now = O.gadpp_requirement(row, t, beta, tau)
            assert now or not prev
            prev = now
        assert prev                                                 # beta = V, huge tau: everything stands


def test_gadpp_special_cases_of_the_decode_loop():
    """beta = 1 (or tau = 0) is the vanilla verification: greedy output.  beta = V with an
    unbounded gap accepts every drafted token: the output is the draft, ceil(T/k) iterations."""
    dims, ver = make("micro", 41)
    src = src_for(dims, 8, 9)
    g = O.greedy(ver, src, 12, EOS, BOS)
    D = [int(t) for t in positional_draft(g, 0.4, 9, dims["vocab"])[0]]
    ref, st_ref = O.gad(ver, src, 4, 12, EOS, BOS, draft_override=D)
    assert ref == g
    for beta, tau in ((1, 5.0), (7, 0.0)):
        out, st = O.gad(ver, src, 4, 12, EOS, BOS, draft_override=D, beta=beta, tau=tau)
        assert out == g and st.accepted == st_ref.accepted
    Dn = [t if t != EOS else 5 for t in D][:12]                     # no EOS: nothing truncates the blocks
    out, st = O.gad(ver, src, 4, 12, EOS, BOS, draft_override=Dn, beta=dims["vocab"], tau=1e9)
    assert out == Dn and st.iterations == math.ceil(len(Dn) / 4)


def test_gadpp_accepts_a_superset_and_bifurcates_at_the_first_failure():
    """One verify call: o_hat equals the draft exactly where the requirement holds and the arg max
    elsewhere; c is the first position where it fails."""
    dims, ver = make("micro", 42)
    src = src_for(dims, 10, 8)
    g = O.greedy(ver, src, 10, EOS, BOS)
    rng = np.random.default_rng(11)
    st = O.DecoderState(ver, ver.encode(src))
    draft = [int(t) for t in rng.integers(5, dims["vocab"], size=6)]
    draft[0] = g[0]
    o_hat, c, lg = O.verify(st, BOS, draft, return_logits=True, beta=3, tau=1.0)
    met = [O.gadpp_requirement(lg[i], draft[i], 3, 1.0) for i in range(6)]
    assert met[0]
    for i in range(6):
        assert o_hat[i] == (draft[i] if met[i] else O.argmax_lowest(lg[i]))
    assert c == (met.index(False) + 1 if False in met else 6)
    o_hat1, c1 = O.verify(O.DecoderState(ver, ver.encode(src)), BOS, draft)
    assert c >= c1


# ----------------------------------------------------------------------------------------------
# Algorithm 1 against the decoding examples the paper prints (tests/golden/iad_case_study.txt).

def _case_study():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "iad_case_study.txt")
    lines = [ln.split(":", 1)[1].split() for ln in open(path) if not ln.startswith("#") and ln.strip()]
    return [([int(t) for t in lines[i]], [int(t) for t in lines[i + 1]], lines[i + 2]) for i in range(0, len(lines), 3)]


class _KnowsTheOutput:
    """Stand-in for the incremental decoder: fed a prefix that agrees with the known greedy
    output it scores that output's next token highest, after a disagreement a token of its own."""
    g, vocab, fed_rows = None, 0, None

    def __init__(self, model, memory):
        self.tokens, self.length = [], 0

    def forward(self, tokens):
        type(self).fed_rows.append(len(tokens))
        self.tokens = self.tokens[:self.length] + [int(t) for t in tokens]
        lg = np.zeros((len(tokens), self.vocab))
        for i in range(len(tokens)):
            n = self.length + i + 1                       # row i has seen o_0 .. o_{n-1}
            ok = self.tokens[1:n] == self.g[:n - 1] and n - 1 < len(self.g)
            lg[i, self.g[n - 1] if ok else self.vocab - 1] = 1.0
        return lg

    def keep(self, new_length):
        self.length = new_length


class _NoModel:
    def encode(self, src):
        return np.zeros((1, 1))


@pytest.mark.parametrize("case", range(7))
def test_algorithm_1_reproduces_the_papers_decoding_examples(case, monkeypatch):
    """Section 4.1.2's table shows, for seven input / output pairs, which output words one
    iteration accepted from a draft and which came from single autoregressive steps.  With the
    output as the model's greedy continuation, the oracle's Algorithm 1 (suffix match included) and
    the library's own loop must cut the output into exactly those iterations."""
    x, o, blocks = _case_study()[case]
    g = o + [EOS]
    _KnowsTheOutput.g, _KnowsTheOutput.vocab, _KnowsTheOutput.fed_rows = g, max(x + o) + 2, []
    monkeypatch.setattr(O, "DecoderState", _KnowsTheOutput)
    out, st = O.iad(_NoModel(), [], x, len(g) + 4, EOS, BOS)
    assert out == g
    acc, rows = list(st.accepted), list(_KnowsTheOutput.fed_rows)
    # the table does not show the end-of-sequence token: it rides on the last block or is a step of its own
    if acc[-1] == 1:
        acc, rows = acc[:-1], rows[:-1]
    else:
        acc[-1] -= 1
    want = [int(b[1:]) for b in blocks]
    assert acc == want
    # an iteration with a draft from the input feeds several rows, an autoregressive step one
    assert ["A" if r > 1 else "R" for r in rows] == [b[0] for b in blocks]
    # the library's loop over the same stand-in
    import paper_2205_10350_amd as ad
    out_l, acc_l, _ = ad.host_simulate(0, np.array(g, dtype=np.int32), np.array(x, dtype=np.int32), k_max=64,
                                       max_out=len(g) + 4, eos=EOS, bos=BOS)
    assert out_l == g and acc_l == list(st.accepted)
