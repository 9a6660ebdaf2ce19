"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer results (tokens, accepted lengths, iteration structure) are compared
exactly; logits within 1e-4 (fp32 mode) / 2e-2 (bf16 mode).

How an arg-max disagreement in bf16 mode is judged.  bf16 rounding of activations amplifies
the fp32 summation-order difference between the two implementations up to the bf16 noise
level of the logits (a few 1e-3 for the base model), so a top-2 margin below that can
legitimately resolve differently.  The tests therefore check, exactly, that the fused
epilogue returns the arg max of the library's OWN logits (lowest id on ties), check the
logits against the oracle within tolerance, and bound the positions where the two arg maxes
differ: the oracle's top-2 margin there must be below twice the logit deviation of that row
(anything larger would contradict the logit check) and below half the logit tolerance (1e-2 at
the stated weight scale), such rows must stay under 1 % of the rows checked (one row in
checks of under a hundred), every one is reported as a warning (pytest prints them in its
summary also for passing runs), and a margin of 1e-3 or more, the threshold the workload's
statement names, is marked in its warning."""
import math
import warnings

import numpy as np
import pytest

import paper_2205_10350_amd as ad
from ad_inputs import CONFIGS, SPECIAL, draw_sources, edit_guide, init_weights, model_dims, positional_draft
from oracle import ad_oracle as O

pytestmark = pytest.mark.gpu
BOS, EOS, MASK = SPECIAL["bos"], SPECIAL["eos"], SPECIAL["mask"]
TOL = {"fp32": 1e-4, "bf16": 2e-2}


def _bf16_weights(w):
    return {k: (O.bf16_round(v) if v.ndim == 2 else v) for k, v in w.items()}


class Rig:
    """A context plus the oracle models that correspond to its arithmetic."""

    def __init__(self, name, dtype, seed, *, B=1, max_src=64, max_len=32, k_max=40, drafter=False, tie=False,
                 std=0.02, special=SPECIAL):
        self.dims = model_dims(name)
        self.dtype = dtype
        self.w = init_weights(self.dims, seed, std=std, tie_output=tie)
        self.wd = init_weights(self.dims, seed + 7, std=std, tie_output=tie) if drafter else None
        self.cfg = ad.make_config(self.dims, max_batch=B, max_src=max_src, max_len=max_len, k_max=k_max, dtype=dtype,
                                  special=special, tie_output=tie, debug_logits=True)
        self.ctx = ad.Context(self.cfg, self.w, self.wd)
        self.eos = special["eos"]
        # the stated tolerances belong to N(0, 0.02) weights; logits (and their bf16 rounding
        # noise) grow at least linearly with the weight scale of the stress cases
        self.tol = TOL[dtype] * (std / 0.02 if dtype == "bf16" else 1.0)
        pos = max(max_src, max_len + k_max) + 1
        if dtype == "bf16":
            # exact arithmetic over the bf16-rounded weights (the logit reference) and the
            # contract emulation (same rounding points as the kernels; the token reference)
            self.exact = O.Model(self.dims, _bf16_weights(self.w), np.float64, max_pos=pos)
            self.tok = O.Model(self.dims, self.w, np.float64, contract=True, max_pos=pos)
            self.dr = O.Model(self.dims, self.wd, np.float64, contract=True, max_pos=pos) if drafter else None
        else:
            self.exact = self.tok = O.Model(self.dims, self.w, np.float64, max_pos=pos)
            self.dr = O.Model(self.dims, self.wd, np.float64, max_pos=pos) if drafter else None

    def close(self):
        self.ctx.close()


def _sources(dims, seed, lens):
    rng = np.random.default_rng(seed)
    return [rng.integers(5, dims["vocab"], size=n).astype(np.int32) for n in lens]


def _check_rows(rig, logits, o_hat, ref_logits, ref_tok_logits, label, log):
    """logits/o_hat from the GPU; ref_logits from the exact oracle; ref_tok_logits from the token oracle."""
    tol = rig.tol
    dev = np.abs(logits - ref_logits).max(axis=1)
    assert dev.max() < tol, (label, dev.max())
    for r in range(logits.shape[0]):
        own = int(np.flatnonzero(logits[r] == logits[r].max())[0])
        assert o_hat[r] == own, (label, r, "fused arg max differs from the arg max of the library's own logits")
        ref = O.argmax_lowest(ref_tok_logits[r])
        if own != ref:
            srt = np.sort(ref_tok_logits[r])
            margin = float(srt[-1] - srt[-2])
            dev_tok = float(np.abs(logits[r] - ref_tok_logits[r]).max())
            log.append((label, r, own, ref, margin, dev_tok))
            assert margin <= 2 * dev_tok + 1e-12 and margin < 0.5 * tol, (label, r, margin, dev_tok)
    return dev.max()


# rows checked / rows whose arg max differs from the oracle's / largest oracle margin among them, per label
NEAR_TIES = {}


def _report(log, rows_checked=None, label=None):
    """Every near-tie as a warning; with rows_checked, the bound on how many there may be."""
    for lab, r, own, ref, margin, dev in log:
        warnings.warn(f"[near-tie] {lab} row {r}: gpu {own} oracle {ref} oracle margin {margin:.3e} logit dev {dev:.3e}"
                      f"{'  (margin >= 1e-3)' if margin >= 1e-3 else ''}")
    if rows_checked is not None:
        worst = max([m for _, _, _, _, m, _ in log], default=0.0)
        NEAR_TIES[label] = (rows_checked, len(log), worst)
        allowed = max(1, rows_checked // 100)
        assert len(log) <= allowed, (label, f"{len(log)} near-tie rows among {rows_checked}, at most {allowed} allowed")
        warnings.warn(f"[parity] {label}: {rows_checked} rows against the oracle, {len(log)} arg-max disagreements, "
                      f"largest oracle margin among them {worst:.3e}")


# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,dtype,seed,std", [
    ("tiny", "fp32", 1000, 0.02), ("tiny", "bf16", 1000, 0.02),
    ("tiny", "fp32", 31, 0.15), ("micro", "fp32", 32, 0.3), ("tiny", "bf16", 33, 0.15),
    ("tiny_deep", "fp32", 34, 0.02), ("tiny_deep", "bf16", 35, 0.02),   # 3 encoder layers, 1 decoder layer
])
def test_verify_logits_teacher_forced(name, dtype, seed, std):
    """One verify forward over the oracle's own greedy prefix: logits, arg max, accepted length.
    The large-std cases make attention sharply peaked so that a mask or head-slicing slip would
    move logits far beyond the tolerance."""
    rig = Rig(name, dtype, seed, std=std)
    try:
        src = _sources(rig.dims, seed, [24])[0]
        g, lg_tok = O.greedy(rig.tok, src, 32, rig.eos, BOS, return_logits=True)
        lg_exact = rig.exact.decode_full(rig.exact.encode(src), [BOS] + g[:-1])
        log = []
        # whole output in ragged blocks: 1, 7, 13, rest — cache append and causal mask across calls
        rig.ctx.encode(ad.AD_VERIFIER, [src])
        j = 0
        for k in (1, 7, 13, 40):
            k = min(k, len(g) - j)
            if k <= 0 or (j and g[j - 1] == rig.eos):
                break
            n, nx, ver = rig.ctx.verify([g[j:j + k]], want_verified=True)
            logits = rig.ctx.debug_logits()
            assert logits.shape[0] == k
            _check_rows(rig, logits, ver[0, :k], lg_exact[j:j + k], lg_tok[j:j + k], f"{name}/{dtype} j={j}", log)
            if log:
                break          # the accepted prefix no longer is the oracle's (the next call would feed the library's token)
            assert n[0] == k and nx[0] == g[j + k - 1]
            j += k
        if log:
            # the rest of the sentence in ONE call on a fresh encode: the draft rows feed the oracle's
            # own prefix whatever the library would accept, so every row is still teacher-forced
            rig.ctx.encode(ad.AD_VERIFIER, [src])
            n, nx, ver = rig.ctx.verify([g], want_verified=True)
            log = []
            _check_rows(rig, rig.ctx.debug_logits(), ver[0, :len(g)], lg_exact, lg_tok, f"{name}/{dtype} whole", log)
        _report(log, len(g), f"{name}/{dtype}/{seed}")
        if dtype == "fp32":
            assert not log
    finally:
        rig.close()


@pytest.mark.parametrize("name,dtype,seed,B", [("tiny", "fp32", 1000, 1), ("tiny", "fp32", 5, 3), ("tiny", "bf16", 6, 3),
                                              ("tiny_deep", "fp32", 8, 2), ("tiny_deep", "bf16", 9, 2)])
def test_decodes_are_greedy_identical_and_match_oracle(name, dtype, seed, B):
    """Workload 0 (tiny, fp32, k = 8, substitution rate 0.1) and batched variants: greedy,
    input-guided and draft-verify outputs are identical to each other and to the oracle; the
    iteration structure equals the oracle's."""
    rig = Rig(name, dtype, seed, B=B, drafter=True)
    try:
        srcs = _sources(rig.dims, seed, [24 - 5 * b for b in range(B)])
        gs = [O.greedy(rig.tok, s, 32, rig.eos, BOS) for s in srcs]
        out_g, st_g = rig.ctx.decode_greedy(srcs)
        assert out_g == gs
        assert st_g["iterations"] == max(len(g) for g in gs) and st_g["tokens_out"] == sum(len(g) for g in gs)
        guides = [edit_guide(g, 0.1, seed + b, rig.dims["vocab"]) for b, g in enumerate(gs)]
        out_i, st_i = rig.ctx.decode_iad(srcs, guides)
        assert out_i == gs
        ref = [O.iad(rig.tok, s, gd, 32, rig.eos, BOS, k_max=rig.cfg.k_max) for s, gd in zip(srcs, guides)]
        assert st_i["rows_verified"] == sum(r[1].rows_verified for r in ref)
        assert st_i["iterations"] == max(r[1].iterations for r in ref)
        Ds = [positional_draft(g, 0.1, seed + b, rig.dims["vocab"])[0] for b, g in enumerate(gs)]
        out_d, st_d = rig.ctx.decode_gad(srcs, 8, use_drafter=False, draft_override=Ds)
        assert out_d == gs
        ref = [O.gad(rig.tok, s, 8, 32, rig.eos, BOS, draft_override=D) for s, D in zip(srcs, Ds)]
        assert st_d["rows_verified"] == sum(r[1].rows_verified for r in ref)
        assert st_d["iterations"] == max(r[1].iterations for r in ref)
        # the real block drafter in the loop (random drafter: nearly nothing accepted, still greedy)
        out_n, st_n = rig.ctx.decode_gad(srcs, 5, use_drafter=True)
        assert out_n == gs and st_n["draft_rows"] > 0
        # source as its own guide (the plain input-guided setting)
        out_s, _ = rig.ctx.decode_iad(srcs, None)
        assert out_s == gs
    finally:
        rig.close()


def test_all_right_all_wrong_drafts_iteration_counts():
    rig = Rig("tiny", "fp32", 1000)
    try:
        src = _sources(rig.dims, 1000, [24])[0]
        g = O.greedy(rig.tok, src, 32, rig.eos, BOS)
        T, V = len(g), rig.dims["vocab"]
        out, st = rig.ctx.decode_gad([src], 8, draft_override=[g])
        assert out == [g] and st["iterations"] == math.ceil(T / 8)
        wrong = [(t - 5 + 1) % (V - 5) + 5 for t in g]
        out, st = rig.ctx.decode_gad([src], 8, draft_override=[wrong])
        assert out == [g] and st["iterations"] == T
        out, st = rig.ctx.decode_iad([src], [g])
        assert out == [g]
        if len(set(g)) == len(g):
            assert st["iterations"] == 1
    finally:
        rig.close()


def test_rows_do_not_depend_on_block_or_batch_shape():
    """Bit-exact: a row's logits are the same whether it is verified alone, in a block of k, or
    next to other sequences (what makes draft-and-verify greedy-identical on this hardware)."""
    rig = Rig("tiny", "bf16", 77, B=3, k_max=40)
    try:
        srcs = _sources(rig.dims, 77, [24, 11, 17])
        out_g, _ = rig.ctx.decode_greedy(srcs)
        # (a) sequence 0 alone, one row at a time
        rig.ctx.encode(ad.AD_VERIFIER, srcs[:1])
        single = []
        for t in range(20):
            rig.ctx.verify([[out_g[0][t]]])
            single.append(rig.ctx.debug_logits()[0])
        single = np.stack(single)
        # (b) sequence 0 alone, one block of 20 (17..32 rows exercise the second row tile)
        rig.ctx.encode(ad.AD_VERIFIER, srcs[:1])
        rig.ctx.verify([out_g[0][:20]])
        block = rig.ctx.debug_logits()
        assert np.array_equal(single.view(np.uint32), block.view(np.uint32))
        # (c) inside a ragged batch: blocks of 9 + 11 with other sequences around it
        rig.ctx.encode(ad.AD_VERIFIER, [srcs[1], srcs[0], srcs[2]])
        rig.ctx.verify([out_g[1][:3], out_g[0][:9], out_g[2][:17]])
        a = rig.ctx.debug_logits()[3:12]
        rig.ctx.verify([[], out_g[0][9:20], out_g[2][17:18]])
        b = rig.ctx.debug_logits()[:11]
        assert np.array_equal(np.concatenate([a, b]).view(np.uint32), block.view(np.uint32))
        # (d) 84 packed rows: sequence 0 straddles the boundary between two 64-row tiles
        rig.ctx.encode(ad.AD_VERIFIER, [srcs[1], srcs[0], srcs[2]])
        rig.ctx.verify([out_g[1][:32], out_g[0][:20], out_g[2][:32]])
        c = rig.ctx.debug_logits()[32:52]
        assert np.array_equal(c.view(np.uint32), block.view(np.uint32))
    finally:
        rig.close()


@pytest.mark.gpu
def test_rows_do_not_depend_on_the_row_regime_of_the_gemm_kernels():
    """Base model, bit-exact: the logits of one sequence's 36-row block verified alone (16 rows per
    workgroup), among 9 / 16 / 20 / 26 sequences (324 / 576 / 720 / 936 packed rows: 16-row chunks with more
    strips per workgroup; from 520 rows 32 rows per workgroup in workgroups of 8 and 16 waves) and among 30
    (1080 rows: the many-row variants)."""
    B = 30
    rig = Rig("base", "bf16", 83, B=B, max_src=40, max_len=48, k_max=40)
    try:
        V = rig.dims["vocab"]
        rng = np.random.default_rng(83)
        srcs = _sources(rig.dims, 83, [12 + (7 * b) % 25 for b in range(B)])
        blocks = [[int(t) for t in rng.integers(5, V, size=36)] for _ in range(B)]
        rig.ctx.encode(ad.AD_VERIFIER, srcs[:1])
        rig.ctx.verify(blocks[:1])
        alone = rig.ctx.debug_logits().view(np.uint32).copy()
        assert alone.shape[0] == 36
        for n in (9, 16, 20, 26, 30):
            # sequence 0 sits in the middle of the batch
            order = list(range(1, n // 2 + 1)) + [0] + list(range(n // 2 + 1, n))
            rig.ctx.encode(ad.AD_VERIFIER, [srcs[i] for i in order])
            rig.ctx.verify([blocks[i] for i in order])
            lg = rig.ctx.debug_logits().view(np.uint32)
            at = 36 * (n // 2)
            assert np.array_equal(lg[at:at + 36], alone), n
    finally:
        rig.close()


def test_rows_do_not_depend_on_the_attention_kernel_the_key_bound_selects():
    """Base model, bit-exact.  A verify call whose longest prefix + block stays within 64 keys runs the compact
    self-attention kernel, any other the generic one, and the bound is part of the call shape a graph is kept for.
    One sequence is verified 8 rows at a time along its own greedy output (every block is accepted whole, so the
    prefix grows by 8 per call and passes 64 keys at the ninth call; the call shape stays the same throughout: the early
    calls are replayed from a graph built with the compact kernel, the late ones must not be).  Every call's logits must
    equal those of the same rows (a) with graphs off and (b) verified beside a second sequence whose 70-row block forces
    the generic kernel in every call."""
    rig = Rig("base", "bf16", 91, B=2, max_src=40, max_len=96, k_max=72)
    try:
        V = rig.dims["vocab"]
        rng = np.random.default_rng(91)
        srcs = _sources(rig.dims, 91, [23, 31])
        g = rig.ctx.decode_greedy(srcs[:1], max_out=[88])[0][0]
        assert len(g) == 88
        other = [int(t) for t in rng.integers(5, V, size=70)]

        def run(graphs, beside):
            rig.ctx.set_option(ad.AD_OPT_GRAPHS, graphs)
            rig.ctx.encode(ad.AD_VERIFIER, srcs if beside else srcs[:1])
            out = []
            for i in range(0, 88, 8):
                n, _ = rig.ctx.verify([g[i:i + 8]] + ([other] if beside else []))
                assert n[0] == 8, (i, n)
                out.append(rig.ctx.debug_logits().view(np.uint32)[:8].copy())
            return out

        a = run(1, False)
        b = run(0, False)
        c = run(1, True)
        for i in range(len(a)):
            assert np.array_equal(a[i], b[i]), ("graphs on / off", i)
            assert np.array_equal(a[i], c[i]), ("compact / generic kernel", i)
    finally:
        rig.ctx.set_option(ad.AD_OPT_GRAPHS, 1)
        rig.close()


def test_rows_do_not_depend_on_the_cross_attention_kernel_the_source_bound_selects():
    """Base model with a source capacity of 80, bit-exact: a batch whose longest source has at most 64 tokens runs the
    compact cross-attention kernels, any other the generic ones; the logits of sequence 0 (a 30-token source, blocks of
    1, 20 and 40 rows) must be the same alone and beside a 75-token source."""
    rig = Rig("base", "bf16", 93, B=2, max_src=80, max_len=48, k_max=40)
    try:
        V = rig.dims["vocab"]
        rng = np.random.default_rng(93)
        srcs = _sources(rig.dims, 93, [30, 75])
        block = [int(t) for t in rng.integers(5, V, size=40)]
        for rows in (1, 20, 40):
            rig.ctx.encode(ad.AD_VERIFIER, srcs[:1])
            rig.ctx.verify([block[:rows]])
            alone = rig.ctx.debug_logits().view(np.uint32)[:rows].copy()
            rig.ctx.encode(ad.AD_VERIFIER, srcs)
            rig.ctx.verify([block[:rows], block[:3]])
            assert np.array_equal(rig.ctx.debug_logits().view(np.uint32)[:rows], alone), rows
    finally:
        rig.close()


def test_ragged_batch_rollback_and_inactive_sequences():
    rig = Rig("tiny", "fp32", 9, B=4, k_max=12)
    try:
        srcs = _sources(rig.dims, 9, [24, 7, 15, 1])
        gs = [O.greedy(rig.tok, s, 32, rig.eos, BOS) for s in srcs]
        rig.ctx.encode(ad.AD_VERIFIER, srcs)
        V = rig.dims["vocab"]
        # per-sequence drafts: right for 5 / wrong at once / inactive / right for 12
        other = lambda t: (t - 5 + 1) % (V - 5) + 5
        d0 = gs[0][:5] + [other(gs[0][5])] + gs[0][6:9]
        n, nx, ver = rig.ctx.verify([d0, [other(gs[1][0]), 9, 9], [], gs[3][:12]], want_verified=True)
        assert n.tolist() == [6, 1, 0, 12]
        assert nx.tolist()[:2] == [gs[0][5], gs[1][0]] and nx[3] == gs[3][11]
        assert ver[0, :6].tolist() == gs[0][:6] and (ver[2] == ad.AD_NEVER).all()
        assert rig.ctx.output() == [gs[0][:6], gs[1][:1], [], gs[3][:12]]
        # rejected rows were rolled back: continuing gives the greedy continuation
        n, nx = rig.ctx.verify([gs[0][6:12], gs[1][1:4], gs[2][:7], [ad.AD_NEVER]])
        assert n.tolist() == [6, 3, 7, 1]
        assert rig.ctx.output() == [gs[0][:12], gs[1][:4], gs[2][:7], gs[3][:13]]
    finally:
        rig.close()


def test_eos_and_output_limit_truncate_on_device():
    """[EOS] is whatever id the configuration names: pick one the greedy output contains."""
    probe = Rig("tiny", "fp32", 12)
    src = _sources(probe.dims, 12, [20])[0]
    g_free = O.greedy(probe.tok, src, 32, -5, BOS)
    probe.close()
    first = next(i for i in range(5, 32) if g_free[i] not in g_free[:i])   # first occurrence at index >= 5
    special = dict(SPECIAL, eos=int(g_free[first]))
    rig = Rig("tiny", "fp32", 12, special=special, B=2)
    try:
        g = O.greedy(rig.tok, src, 32, rig.eos, BOS)
        assert g[-1] == rig.eos and len(g) == first + 1
        out, st = rig.ctx.decode_greedy([src, src], max_out=[32, 4])
        assert out == [g, g[:4]]
        # a draft that is right beyond [EOS]: the block is cut after [EOS]
        out, st = rig.ctx.decode_gad([src, src], 16, draft_override=[g_free, g_free], max_out=[32, 4])
        assert out == [g, g[:4]] and st["iterations"] == 1
        rig.ctx.encode(ad.AD_VERIFIER, [src, src], max_out=[32, 4])
        n, nx = rig.ctx.verify([g_free[:16], g_free[:16]])
        assert n.tolist() == [len(g), 4] and nx[0] == rig.eos
        with pytest.raises(ad.AdError) as e:      # finished sequences take no more rows
            rig.ctx.verify([[5], []])
        assert e.value.code == ad.AD_ESTATE
    finally:
        rig.close()


def test_block_drafter_matches_oracle():
    for dtype in ("fp32", "bf16"):
        rig = Rig("tiny", dtype, 21, B=2, drafter=True)
        try:
            srcs = _sources(rig.dims, 21, [18, 9])
            gs = [O.greedy(rig.tok, s, 32, rig.eos, BOS) for s in srcs]
            rig.ctx.encode(ad.AD_VERIFIER, srcs)
            rig.ctx.encode(ad.AD_DRAFTER, srcs)
            log = []
            for step, (a, b) in enumerate([(0, 0), (4, 2), (3, 0)]):
                if step:
                    n, _ = rig.ctx.verify([gs[0][pa:pa + a], gs[1][pb:pb + b]])
                    assert n.tolist() == [a, b]
                    pa += a; pb += b
                else:
                    pa = pb = 0
                k = 6
                dr = rig.ctx.draft_nat(k)
                logits = rig.ctx.debug_logits()
                for i, (s, p) in enumerate(zip(srcs, (pa, pb))):
                    mem = rig.dr.encode(s)
                    toks = [BOS] + gs[i][:p] + [MASK] * k
                    ref = rig.dr.decode_full(mem, toks, causal=False)[p + 1:]
                    got = logits[i * k:(i + 1) * k]
                    assert np.abs(got - ref).max() < TOL[dtype]
                    for r in range(k):
                        own = int(np.flatnonzero(got[r] == got[r].max())[0])
                        assert dr[i, r] == own
                        if own != O.argmax_lowest(ref[r]):
                            srt = np.sort(ref[r]); log.append((f"draft {dtype}", r, own, 0, float(srt[-1] - srt[-2]), 0.0))
            _report(log)
            assert dtype != "fp32" or not log
        finally:
            rig.close()


def test_block_drafter_skips_finished_sequences():
    """Three sequences, the middle one finished (its output limit reached): the drafter's rows are
    those of the other two (mask rows first, prefix rows behind), its drafts land in their slots and
    the finished sequence gets the never-matching id."""
    rig = Rig("tiny", "fp32", 23, B=3, drafter=True)
    try:
        srcs = _sources(rig.dims, 23, [12, 7, 15])
        gs = [O.greedy(rig.tok, s, 32, rig.eos, BOS) for s in srcs]
        rig.ctx.encode(ad.AD_VERIFIER, srcs, max_out=[32, 2, 32])
        rig.ctx.encode(ad.AD_DRAFTER, srcs)
        n, _ = rig.ctx.verify([gs[0][:3], gs[1][:2], gs[2][:5]])
        assert n.tolist() == [3, 2, 5]
        k = 4
        dr = rig.ctx.draft_nat(k)
        logits = rig.ctx.debug_logits()
        assert logits.shape[0] == 2 * k
        assert dr[1].tolist() == [ad.AD_NEVER] * k
        for live, (i, p) in enumerate(((0, 3), (2, 5))):
            toks = [BOS] + gs[i][:p] + [MASK] * k
            ref = rig.dr.decode_full(rig.dr.encode(srcs[i]), toks, causal=False)[p + 1:]
            got = logits[live * k:(live + 1) * k]
            assert np.abs(got - ref).max() < TOL["fp32"]
            assert dr[i].tolist() == [O.argmax_lowest(r) for r in ref]
    finally:
        rig.close()


def test_argument_errors_on_device_context():
    rig = Rig("tiny", "fp32", 3, B=2, k_max=4, max_src=16, max_len=8)
    try:
        src = _sources(rig.dims, 3, [10])[0]
        with pytest.raises(ad.AdError) as e:
            rig.ctx.verify([[5]])
        assert e.value.code == ad.AD_ESTATE            # before encode
        with pytest.raises(ad.AdError) as e:
            rig.ctx.draft_nat(2)
        assert e.value.code == ad.AD_ESTATE            # no drafter weights
        rig.ctx.encode(ad.AD_VERIFIER, [src])
        for bad in ([[5, 6, 7, 8, 9]], [[5, 40000]], [[ad.AD_NEVER, 5]]):
            d = np.full((1, 8), 0, dtype=np.int32)
            d[0, :len(bad[0])] = bad[0]
            import ctypes as C
            k = np.array([len(bad[0])], dtype=np.int32); n = np.zeros(1, np.int32); nx = np.zeros(1, np.int32)
            P = C.POINTER(C.c_int32)
            rc = rig.ctx.L.ad_verify(rig.ctx.h, d.ctypes.data_as(P), k.ctypes.data_as(P), n.ctypes.data_as(P),
                                     nx.ctypes.data_as(P), None)
            assert rc == ad.AD_EINVAL, bad
        # state untouched by the failed calls
        g = O.greedy(rig.tok, src, 8, rig.eos, BOS)
        n, nx = rig.ctx.verify([g[:4]])
        assert n[0] == 4
        with pytest.raises(ad.AdError):
            rig.ctx.encode(ad.AD_VERIFIER, [np.arange(5, 5 + 17)])   # longer than max_src
    finally:
        rig.close()


# ----------------------------------------------------------------------------------------------
# Full-size workloads (base / big models): sampled rows against the oracle, plus properties
# that hold at any size.

def _teacher_forced_base(rig, srcs, n_check, label):
    """Every row of the first n_check sentences against the oracle, teacher-forced on the oracle's
    own greedy output: ONE verify call per sentence with that output as the draft (the rows a call
    feeds are the pending token and the draft, whatever it goes on to accept), so a near-tie in one
    row never cuts the comparison of the rows after it.  Needs k_max >= the sentence's length."""
    log = []
    worst = 0.0
    rows = 0
    for s in srcs[:n_check]:
        T = len(s)
        assert T <= rig.cfg.k_max
        g, lg_tok = O.greedy(rig.tok, s, T, rig.eos, BOS, return_logits=True)
        lg_exact = rig.exact.decode_full(rig.exact.encode(s), [BOS] + g[:-1])
        rig.ctx.encode(ad.AD_VERIFIER, [s], max_out=[T])
        n, nx, ver = rig.ctx.verify([g], want_verified=True)
        logits = rig.ctx.debug_logits()
        assert logits.shape[0] == len(g)
        worst = max(worst, _check_rows(rig, logits, ver[0, :len(g)], lg_exact, lg_tok, label, log))
        rows += len(g)
    _report(log, rows, label)
    warnings.warn(f"[parity] {label}: max |logit - oracle| = {worst:.3e} over {rows} rows")
    return log


def test_workload1_base_iad_batch1():
    cfg = CONFIGS[1]
    rig = Rig("base", "bf16", cfg["seed"], max_src=64, max_len=64, k_max=72)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=12)
        _teacher_forced_base(rig, srcs, 2, "workload1 (2 sentences)")
        for s, mo in zip(srcs, max_out):
            out_g, _ = rig.ctx.decode_greedy([s], max_out=[mo])
            guide = edit_guide(out_g[0], cfg["rate"], cfg["seed"], rig.dims["vocab"])
            out_i, st = rig.ctx.decode_iad([s], [guide], max_out=[mo])
            assert out_i == out_g and len(out_g[0]) == mo
            _, acc, st_sim = ad.host_simulate(0, out_g[0], guide, k_max=72, max_out=int(mo))
            assert st["iterations"] == st_sim["iterations"] and st["rows_verified"] == st_sim["rows_verified"]
    finally:
        rig.close()


def test_workload5_deep_encoder_shallow_decoder_iad_batch1():
    """Input-guided decoding with the 12 + 2 layer model at the big width (Section 4.1's second
    model shape): teacher-forced logits of one sentence, greedy identity and iteration structure."""
    cfg = CONFIGS[5]
    rig = Rig("deep_shallow", "bf16", cfg["seed"], max_src=64, max_len=64, k_max=72)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=6)
        _teacher_forced_base(rig, srcs, 1, "workload5")
        for s, mo in zip(srcs, max_out):
            out_g, _ = rig.ctx.decode_greedy([s], max_out=[mo])
            guide = edit_guide(out_g[0], cfg["rate"], cfg["seed"], rig.dims["vocab"])
            out_i, st = rig.ctx.decode_iad([s], [guide], max_out=[mo])
            assert out_i == out_g and len(out_g[0]) == mo
            _, acc, st_sim = ad.host_simulate(0, out_g[0], guide, k_max=72, max_out=int(mo))
            assert st["iterations"] == st_sim["iterations"] and st["rows_verified"] == st_sim["rows_verified"]
    finally:
        rig.close()


def test_workload2_base_iad_batch32():
    cfg = CONFIGS[2]
    rig = Rig("base", "bf16", CONFIGS[1]["seed"], B=32, max_src=64, max_len=64, k_max=72)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=32)
        out_g, st_g = rig.ctx.decode_greedy(srcs, max_out=max_out)
        assert [len(o) for o in out_g] == max_out.tolist()
        guides = [edit_guide(g, cfg["rate"], cfg["seed"] + b, rig.dims["vocab"]) for b, g in enumerate(out_g)]
        out_i, st_i = rig.ctx.decode_iad(srcs, guides, max_out=max_out)
        assert out_i == out_g                      # ragged accepted lengths + rollback, bit-exact
        assert st_i["iterations"] < st_g["iterations"]
        rows = sum(ad.host_simulate(0, g, gd, k_max=72, max_out=int(mo))[2]["rows_verified"]
                   for g, gd, mo in zip(out_g, guides, max_out))
        assert st_i["rows_verified"] == rows
        # sampled sequences against single-sequence decoding (batch invariance at full size)
        for b in (0, 13, 31):
            single, _ = rig.ctx.decode_greedy([srcs[b]], max_out=[max_out[b]])
            assert single[0] == out_g[b]
    finally:
        rig.close()


def test_workload3_base_gad_batch1():
    cfg = CONFIGS[3]
    rig = Rig("base", "bf16", cfg["seed"], max_src=80, max_len=80, k_max=25, drafter=True)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=4)
        for s, mo in zip(srcs, max_out):
            out_g, _ = rig.ctx.decode_greedy([s], max_out=[mo])
            D, _ = positional_draft(out_g[0], cfg["rate"], cfg["seed"], rig.dims["vocab"])
            out_d, st = rig.ctx.decode_gad([s], cfg["k"], use_drafter=True, draft_override=[D], max_out=[mo])
            assert out_d == out_g
            _, acc, st_sim = ad.host_simulate(1, out_g[0], D, k=cfg["k"], k_max=25, max_out=int(mo))
            assert st["iterations"] == st_sim["iterations"] and st["draft_rows"] > 0
        # the drafter alone, first block, against the oracle
        s = srcs[0]
        rig.ctx.encode(ad.AD_VERIFIER, [s]); rig.ctx.encode(ad.AD_DRAFTER, [s])
        dr = rig.ctx.draft_nat(25)
        got = rig.ctx.debug_logits()
        ref = rig.dr.decode_full(rig.dr.encode(s), [BOS] + [MASK] * 25, causal=False)[1:]
        assert np.abs(got - ref).max() < TOL["bf16"]
        assert dr[0].tolist() == [int(np.flatnonzero(r == r.max())[0]) for r in got]
    finally:
        rig.close()


def test_workload4_big_gad_batch8():
    cfg = CONFIGS[4]
    rig = Rig("big", "bf16", cfg["seed"], B=8, max_src=512, max_len=128, k_max=25, drafter=True)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=8)
        out_g, _ = rig.ctx.decode_greedy(srcs, max_out=max_out)
        Ds = [positional_draft(g, cfg["rate"], cfg["seed"] + b, rig.dims["vocab"])[0] for b, g in enumerate(out_g)]
        out_d, st = rig.ctx.decode_gad(srcs, cfg["k"], use_drafter=True, draft_override=Ds, max_out=max_out)
        assert out_d == out_g and [len(o) for o in out_g] == [128] * 8
        its = max(ad.host_simulate(1, g, D, k=25, k_max=25, max_out=128)[2]["iterations"] for g, D in zip(out_g, Ds))
        assert st["iterations"] == its
        # one sampled sequence, first 12 rows, against the oracle (S = 512 cross-attention keys)
        s = srcs[3]
        g12, lg_tok = O.greedy(rig.tok, s, 12, rig.eos, BOS, return_logits=True)
        lg_exact = rig.exact.decode_full(rig.exact.encode(s), [BOS] + g12[:-1])
        rig.ctx.encode(ad.AD_VERIFIER, [s])
        n, nx, ver = rig.ctx.verify([g12], want_verified=True)
        log = []
        _check_rows(rig, rig.ctx.debug_logits(), ver[0, :12], lg_exact, lg_tok, "workload4", log)
        _report(log, 12, "workload4 (12 rows of one sequence)")
    finally:
        rig.close()


# ----------------------------------------------------------------------------------------------
# Graph replay of a verify call's launches against the same launches made one by one.

@pytest.mark.gpu
@pytest.mark.parametrize("name,B", [("tiny", 2), ("base", 1), ("base", 3)])
def test_graph_replays_equal_eager_launches(name, B):
    """Every replay of a captured call shape, with the library's own eager work (encode, other
    shapes, synchronisations) between the replays, gives the bits the eager launches give."""
    rig = Rig(name, "bf16", 77, B=B, max_src=40, max_len=40, k_max=24, drafter=(name == "tiny" or B == 3))
    try:
        assert rig.ctx.get_option(ad.AD_OPT_GRAPHS) == 1
        V = rig.dims["vocab"]
        srcs = _sources(rig.dims, 77, [28 - 5 * b for b in range(B)])
        rig.ctx.set_option(ad.AD_OPT_GRAPHS, 0)
        out_ref, _ = rig.ctx.decode_greedy(srcs)
        # the same three-call script, six times: eager first, then with graphs (call shapes are
        # captured on their third appearance and replayed on the later ones)
        d1 = [out_ref[b][:4] for b in range(B)]
        d2 = [[(out_ref[b][4] - 5 + 1) % (V - 5) + 5] + out_ref[b][5:9] for b in range(B)]   # wrong first token
        d3 = [out_ref[b][5:9] for b in range(B)]

        def script():
            rig.ctx.encode(ad.AD_VERIFIER, srcs)
            r = []
            for d in (d1, d2, d3):
                r.append(rig.ctx.verify(d, want_verified=True))
                r.append(rig.ctx.debug_logits().view(np.uint32).copy())
            r.append(rig.ctx.output())
            return r

        ref = script()
        rig.ctx.set_option(ad.AD_OPT_GRAPHS, 1)
        for rep in range(5):
            got = script()
            for x, y in zip(ref, got):
                if isinstance(x, tuple):
                    for u, v in zip(x, y):
                        assert np.array_equal(u, v), rep
                elif isinstance(x, np.ndarray):
                    assert np.array_equal(x, y), rep
                else:
                    assert x == y, rep
        assert rig.ctx.get_option(ad.AD_OPT_GRAPHS) == 1, "graph capture failed and was switched off"
        assert rig.ctx.get_option(ad.AD_OPT_GRAPHS_CAPTURED) >= 2
        # the block drafter's forward between replayed verify and encode calls (its own launches are
        # made one by one)
        if rig.wd is not None:
            def draft_script():
                rig.ctx.encode(ad.AD_VERIFIER, srcs); rig.ctx.encode(ad.AD_DRAFTER, srcs)
                a = rig.ctx.draft_nat(6).copy()
                rig.ctx.verify([out_ref[b][:3] for b in range(B)])
                return a, rig.ctx.draft_nat(6).copy(), rig.ctx.draft_nat(4).copy()
            rig.ctx.set_option(ad.AD_OPT_GRAPHS, 0)
            dref = draft_script()
            rig.ctx.set_option(ad.AD_OPT_GRAPHS, 1)
            for rep in range(4):
                for x, y in zip(dref, draft_script()):
                    assert np.array_equal(x, y), rep
        # whole decodes through replays
        guides = [edit_guide(g, 0.1, 5 + b, V) for b, g in enumerate(out_ref)]
        for rep in range(2):
            og, _ = rig.ctx.decode_greedy(srcs)
            oi, _ = rig.ctx.decode_iad(srcs, guides)
            assert og == out_ref and oi == out_ref
    finally:
        rig.close()


@pytest.mark.gpu
@pytest.mark.parametrize("name,B", [("base", 1), ("base", 3), ("big", 2), ("base", 8)])
def test_fused_cross_attention_launch_equals_projection_plus_attention(name, B):
    """AD_OPT_FUSE_CROSSQ: the decoder layers' cross-attention as one launch (query projection inside)
    against the two launches it replaces: logits, arg max, accepted lengths, outputs and the block
    drafter's tokens bit for bit, on ragged blocks of more than 16 and more than 32 rows."""
    rig = Rig(name, "bf16", 91, B=B, max_src=48, max_len=80, k_max=72, drafter=True)
    try:
        assert rig.ctx.get_option(ad.AD_OPT_FUSE_CROSSQ) == 1
        V = rig.dims["vocab"]
        srcs = _sources(rig.dims, 91, [41 - 4 * b for b in range(B)])
        out_ref, _ = rig.ctx.decode_greedy(srcs)
        # all accepted; 18 / 27 / 36 rows, and with eight sequences blocks of 1 .. 71 rows (chunks of 32 query
        # rows per workgroup instead of 16: the launch would exceed a workgroup per compute unit)
        lens = [17 + 9 * b for b in range(B)] if B < 8 else [70, 3, 64, 17, 33, 1, 48, 65]
        d1 = [out_ref[b][:min(lens[b], len(out_ref[b]) - 7)] for b in range(B)]
        d2 = [[(out_ref[b][len(d1[b])] - 5 + 1) % (V - 5) + 5] + out_ref[b][len(d1[b]) + 1:len(d1[b]) + 6]
              for b in range(B)]                                               # wrong first token
        res = {}
        for mode in (0, 1):
            rig.ctx.set_option(ad.AD_OPT_FUSE_CROSSQ, mode)
            assert rig.ctx.get_option(ad.AD_OPT_FUSE_CROSSQ) == mode
            rig.ctx.encode(ad.AD_VERIFIER, srcs); rig.ctx.encode(ad.AD_DRAFTER, srcs)
            a = rig.ctx.verify(d1, want_verified=True)
            la = rig.ctx.debug_logits().view(np.uint32).copy()
            dr = rig.ctx.draft_nat(7).copy()
            b_ = rig.ctx.verify(d2, want_verified=True)
            lb = rig.ctx.debug_logits().view(np.uint32).copy()
            res[mode] = (a, la, b_, lb, dr, rig.ctx.output())
        (a0, la0, b0, lb0, dr0, o0), (a1, la1, b1, lb1, dr1, o1) = res[0], res[1]
        for x, y in zip(a0 + b0, a1 + b1):
            assert np.array_equal(x, y)
        assert np.array_equal(la0, la1) and np.array_equal(lb0, lb1) and np.array_equal(dr0, dr1)
        assert o0 == o1
        assert a1[0].tolist() == [len(d) for d in d1] and b1[0].tolist() == [1] * B
        # whole decodes (graph replays included) with either setting
        guides = [edit_guide(g, 0.1, 3 + b, V) for b, g in enumerate(out_ref)]
        for mode in (0, 1, 0, 1):
            rig.ctx.set_option(ad.AD_OPT_FUSE_CROSSQ, mode)
            oi, _ = rig.ctx.decode_iad(srcs, guides)
            assert oi == out_ref
    finally:
        rig.close()


def test_waiting_on_the_mapped_result_equals_waiting_on_the_stream():
    """AD_OPT_SPIN_WAIT only changes how the host learns that a verify call has finished: tokens,
    accepted lengths and iteration structure are the same either way, also right after other
    calls have left unrelated words in the staging buffer (an encode, an output read-back)."""
    rig = Rig("tiny", "bf16", 77, B=3, k_max=8)
    try:
        srcs = _sources(rig.dims, 77, [9, 14, 11])
        ref, _ = rig.ctx.decode_greedy(srcs, max_out=[20, 20, 20])
        guides = [edit_guide(g, 0.2, 5 + i, rig.dims["vocab"]) for i, g in enumerate(ref)]
        results = {}
        for mode in (1, 0, 1):
            rig.ctx.set_option(ad.AD_OPT_SPIN_WAIT, mode)
            assert rig.ctx.get_option(ad.AD_OPT_SPIN_WAIT) == mode
            out, st = rig.ctx.decode_iad(srcs, guides, max_out=[20, 20, 20])
            assert out == ref
            rig.ctx.encode(ad.AD_VERIFIER, srcs, max_out=[20, 20, 20])
            trace = []
            for step in range(4):
                n, nx = rig.ctx.verify([list(g[sum(t[0][b] for t in trace):][:5]) or [ad.AD_NEVER] for b, g in enumerate(ref)])
                trace.append((n.tolist(), nx.tolist()))
                assert rig.ctx.output()[0] == ref[0][:sum(t[0][0] for t in trace)]
            results.setdefault("trace", trace)
            assert trace == results["trace"]
            results.setdefault("iters", st["iterations"])
            assert st["iterations"] == results["iters"]
    finally:
        rig.close()
