"""Full-size parity cases: the shapes and launch configurations bench.py times, against the oracle
element by element, plus the shipped arg-max path (no logits in memory) against the logits path.

Teacher forcing is done with ONE verify call per sentence: the rows a call feeds are the pending
token and the draft, so with the oracle's own greedy output as the draft every row sees the
oracle's prefix, and an arg-max disagreement in one row (a near-tie, see test_gpu_parity's header)
does not stop the rows after it from being compared."""
import warnings

import numpy as np
import pytest

import paper_2205_10350_amd as ad
from ad_inputs import CONFIGS, SPECIAL, draw_sources, edit_guide, init_weights, model_dims
from oracle import ad_oracle as O
from test_gpu_parity import NEAR_TIES, Rig, _check_rows, _report, _sources, _teacher_forced_base

pytestmark = pytest.mark.gpu
BOS, EOS = SPECIAL["bos"], SPECIAL["eos"]


def test_workload1_every_row_of_16_sentences_teacher_forced():
    cfg = CONFIGS[1]
    rig = Rig("base", "bf16", cfg["seed"], max_src=64, max_len=64, k_max=72)
    try:
        srcs, _ = draw_sources(cfg, rig.dims["vocab"], n_sent=16)
        _teacher_forced_base(rig, srcs, 16, "workload1")
        assert NEAR_TIES["workload1"][0] >= 300          # rows checked
    finally:
        rig.close()


def test_workload3_every_row_of_16_sentences_teacher_forced():
    """Source lengths of the block-drafting workload (20..80): the verifier's rows against a long
    prefix; k_max is raised to the longest sentence so that one call covers it."""
    cfg = CONFIGS[3]
    rig = Rig("base", "bf16", cfg["seed"], max_src=80, max_len=80, k_max=80)
    try:
        srcs, _ = draw_sources(cfg, rig.dims["vocab"], n_sent=16)
        _teacher_forced_base(rig, srcs, 16, "workload3")
        assert NEAR_TIES["workload3"][0] >= 600
    finally:
        rig.close()


def test_workload2_first_iteration_batch_of_32_against_the_oracle():
    """The batch-32 call shape bench.py times (32 ragged sequences, whole guide + sentinel each,
    about 1150 packed rows, the many-row launch shapes): the logits of four sampled sequences,
    every row, against the oracle.  The sampled sequences draft the oracle's greedy output (so
    their rows are teacher-forced), the others the library's own."""
    cfg = CONFIGS[2]
    rig = Rig("base", "bf16", CONFIGS[1]["seed"], B=32, max_src=64, max_len=64, k_max=72)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=32)
        out_g, _ = rig.ctx.decode_greedy(srcs, max_out=max_out)
        sampled = (0, 9, 18, 31)
        ref = {}
        for b in sampled:
            g, lg_tok = O.greedy(rig.tok, srcs[b], int(max_out[b]), rig.eos, BOS, return_logits=True)
            lg_exact = rig.exact.decode_full(rig.exact.encode(srcs[b]), [BOS] + g[:-1])
            ref[b] = (g, lg_tok, lg_exact)
        drafts = [list(ref[b][0]) if b in ref else list(out_g[b]) for b in range(32)]
        rows = sum(len(d) for d in drafts)
        assert rows >= 1080, rows
        rig.ctx.encode(ad.AD_VERIFIER, srcs, max_out=max_out)
        n, nx, ver = rig.ctx.verify(drafts, want_verified=True)
        logits = rig.ctx.debug_logits()
        assert logits.shape[0] == rows
        log, checked, r0 = [], 0, 0
        for b in range(32):
            k = len(drafts[b])
            if b in ref:
                g, lg_tok, lg_exact = ref[b]
                _check_rows(rig, logits[r0:r0 + k], ver[b, :k], lg_exact, lg_tok, f"workload2 seq {b}", log)
                checked += k
            else:
                assert n[b] == k        # its own greedy output as the draft: accepted whole
            r0 += k
        _report(log, checked, "workload2 (4 of 32 sequences, first-iteration batch)")
    finally:
        rig.close()


def test_workload4_full_block_of_8x25_rows_against_the_oracle():
    """Transformer-big, batch 8, 512-token sources, one 25-row block per sequence (200 packed rows,
    512 cross-attention keys): every row of two sequences against the oracle."""
    cfg = CONFIGS[4]
    rig = Rig("big", "bf16", cfg["seed"], B=8, max_src=512, max_len=128, k_max=25)
    try:
        srcs, max_out = draw_sources(cfg, rig.dims["vocab"], n_sent=8)
        rng = np.random.default_rng(404)
        sampled = (2, 7)
        ref = {}
        for b in sampled:
            g, lg_tok = O.greedy(rig.tok, srcs[b], 25, rig.eos, BOS, return_logits=True)
            lg_exact = rig.exact.decode_full(rig.exact.encode(srcs[b]), [BOS] + g[:-1])
            ref[b] = (g, lg_tok, lg_exact)
        drafts = [list(ref[b][0]) if b in ref else [int(t) for t in rng.integers(5, rig.dims["vocab"], size=25)]
                  for b in range(8)]
        rig.ctx.encode(ad.AD_VERIFIER, srcs, max_out=max_out)
        n, nx, ver = rig.ctx.verify(drafts, want_verified=True)
        logits = rig.ctx.debug_logits()
        assert logits.shape[0] == 200
        log = []
        for b in sampled:
            g, lg_tok, lg_exact = ref[b]
            _check_rows(rig, logits[25 * b:25 * b + 25], ver[b, :25], lg_exact, lg_tok, f"workload4 seq {b}", log)
        _report(log, 50, "workload4 (2 of 8 sequences, 8 x 25 block, 512 source tokens)")
    finally:
        rig.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_heads_of_width_128(dtype):
    """Head width 128 (d 256, 2 heads): the widest the attention kernels take, on the matrix cores
    in bf16 mode: teacher-forced logits against the oracle, greedy identity of the decodes."""
    rig = Rig("wide_head", dtype, 128, B=2, max_src=40, max_len=32, k_max=32, drafter=True)
    try:
        srcs = _sources(rig.dims, 128, [30, 17])
        _teacher_forced_base(rig, [s[:len(s)] for s in srcs], 2, f"wide_head/{dtype}")
        out_g, _ = rig.ctx.decode_greedy(srcs)
        guides = [edit_guide(g, 0.1, 128 + b, rig.dims["vocab"]) for b, g in enumerate(out_g)]
        out_i, st = rig.ctx.decode_iad(srcs, guides)
        assert out_i == out_g
        # the drafter's bidirectional attention at this head width
        rig.ctx.encode(ad.AD_VERIFIER, srcs); rig.ctx.encode(ad.AD_DRAFTER, srcs)
        dr = rig.ctx.draft_nat(6)
        got = rig.ctx.debug_logits()
        for i, s in enumerate(srcs):
            want = rig.dr.decode_full(rig.dr.encode(s), [BOS] + [SPECIAL["mask"]] * 6, causal=False)[1:]
            assert np.abs(got[6 * i:6 * i + 6] - want).max() < rig.tol
    finally:
        rig.close()


def test_rows_of_the_wide_model_do_not_depend_on_the_gemm_kernel_the_row_count_selects():
    """Big model (d 1024, FFN 4096), bit-exact: the logits of one sequence's 25-row block verified
    alone (the attention output projections and FFN2 run in the kernel that puts a strip's
    512-slices side by side in the waves) and in the middle of 8 sequences (200 packed rows: the
    kernel that walks the slices one after the other, several strips per workgroup)."""
    dims = model_dims("big")
    w = init_weights(dims, 411)
    ctx = ad.Context(ad.make_config(dims, max_batch=8, max_src=40, max_len=40, k_max=32, dtype="bf16", special=SPECIAL,
                                    debug_logits=True), w)
    try:
        V = dims["vocab"]
        rng = np.random.default_rng(411)
        srcs = [rng.integers(5, V, size=int(n)).astype(np.int32) for n in rng.integers(10, 40, size=8)]
        blocks = [[int(t) for t in rng.integers(5, V, size=25)] for _ in range(8)]
        ctx.encode(ad.AD_VERIFIER, srcs[:1])
        ctx.verify(blocks[:1])
        alone = ctx.debug_logits().view(np.uint32).copy()
        assert alone.shape[0] == 25
        for n in (3, 8):   # 75 rows: still the first kernel, several row chunks; 200 rows: the other
            order = list(range(1, n // 2 + 1)) + [0] + list(range(n // 2 + 1, n))
            ctx.encode(ad.AD_VERIFIER, [srcs[i] for i in order])
            ctx.verify([blocks[i] for i in order])
            lg = ctx.debug_logits().view(np.uint32)
            at = 25 * (n // 2)
            assert np.array_equal(lg[at:at + 25], alone), n
    finally:
        ctx.close()


@pytest.mark.parametrize("name,src_lens", [("base", [300, 130, 512, 257, 40, 384, 129, 200]),
                                           ("big", [512, 500, 129, 512, 300, 512, 40, 260])])
def test_long_source_rows_do_not_depend_on_how_the_cross_attention_splits_the_keys(name, src_lens):
    """Sources of more than 128 tokens, bit-exact.  One row tile per workgroup (a sequence alone, or few rows of
    each): the four waves of the cross-attention kernel split the keys in super-blocks of 128; several row tiles
    per workgroup (40 rows of each of 8 sequences): every wave walks all keys with four accumulators; the
    projection and attention as two launches: the generic attention kernel.  All three sum a row's keys in the
    order the key index fixes, so the logits of sequence 0 agree whatever the launch is; sources of 40, 129, 130
    tokens leave waves without keys, 512 fills all four."""
    dims = model_dims(name)
    w = init_weights(dims, 977)
    B = len(src_lens)
    ctx = ad.Context(ad.make_config(dims, max_batch=B, max_src=512, max_len=16, k_max=40, dtype="bf16", special=SPECIAL,
                                    debug_logits=True), w)
    try:
        V = dims["vocab"]
        rng = np.random.default_rng(977)
        srcs = [rng.integers(5, V, size=n).astype(np.int32) for n in src_lens]
        blocks = [[int(t) for t in rng.integers(5, V, size=40)] for _ in range(B)]
        got = {}
        for fuse in (1, 0):
            ctx.set_option(ad.AD_OPT_FUSE_CROSSQ, fuse)
            for tag, ns, rows in (("8x40", B, 40), ("8x7", B, 7), ("1x40", 1, 40), ("1x1", 1, 1)):
                ctx.encode(ad.AD_VERIFIER, srcs[:ns])
                ctx.verify([b[:rows] for b in blocks[:ns]])
                got[(tag, fuse)] = ctx.debug_logits().view(np.uint32)[:rows * ns].copy()
        ref = got[("1x40", 1)]
        assert ref.shape[0] == 40
        for fuse in (1, 0):
            assert np.array_equal(got[("1x40", fuse)], ref), fuse
            assert np.array_equal(got[("8x40", fuse)][:40], ref), fuse
            assert np.array_equal(got[("8x7", fuse)][:7], ref[:7]), fuse
            assert np.array_equal(got[("1x1", fuse)], ref[:1]), fuse
        # every sequence of the batch, not only the first: one launch style against the other
        assert np.array_equal(got[("8x40", 1)], got[("8x40", 0)])
        assert np.array_equal(got[("8x7", 1)], got[("8x7", 0)])
    finally:
        ctx.set_option(ad.AD_OPT_FUSE_CROSSQ, 1)
        ctx.close()


def _ctx_pair(name, seed, **cap):
    """Two contexts over the same weights: one keeps the logits (its output projection stores
    them), the other runs the shipped epilogue that never writes them."""
    dims = model_dims(name)
    w = init_weights(dims, seed)
    a = ad.Context(ad.make_config(dims, dtype="bf16", special=SPECIAL, debug_logits=True, **cap), w)
    b = ad.Context(ad.make_config(dims, dtype="bf16", special=SPECIAL, debug_logits=False, **cap), w)
    return dims, w, a, b


@pytest.mark.parametrize("name,B,rows_each", [("base", 1, 1), ("base", 1, 25), ("base", 1, 65), ("base", 8, 25),
                                              ("base", 32, 37), ("big", 1, 25), ("big", 8, 25)])
def test_arg_max_without_logits_equals_arg_max_of_the_logits(name, B, rows_each):
    """The production epilogue (running arg max inside the output projection, logits never in
    memory) at 1, 25, 65, 200 and about 1180 rows, base and big widths: every row's arg max, the
    accepted lengths and next tokens equal those of a context that stores the logits, and the
    arg max of those logits."""
    dims, w, dbg, prod = _ctx_pair(name, 909, max_batch=B, max_src=40, max_len=80, k_max=72)
    try:
        V = dims["vocab"]
        rng = np.random.default_rng(rows_each * 100 + B)
        srcs = [rng.integers(5, V, size=int(n)).astype(np.int32) for n in rng.integers(10, 40, size=B)]
        # two calls: the first leaves a cache the second attends to; ragged in batches
        d1 = [[int(t) for t in rng.integers(5, V, size=3 + (b % 3))] for b in range(B)]
        d2 = [[int(t) for t in rng.integers(5, V, size=max(1, rows_each - (b % 4 if B > 1 else 0)))] for b in range(B)]
        res = []
        for ctx in (dbg, prod):
            ctx.encode(ad.AD_VERIFIER, srcs)
            res.append((ctx.verify(d1, want_verified=True), ctx.verify(d2, want_verified=True), d2))
            if ctx is dbg:
                logits = ctx.debug_logits()
        (a1, a2, d2), (b1, b2, _) = res
        for x, y in zip(a1 + a2, b1 + b2):
            assert np.array_equal(x, y)
        r0 = 0
        for b in range(B):
            k = len(d2[b])
            own = [int(np.flatnonzero(r == r.max())[0]) for r in logits[r0:r0 + k]]
            assert b2[2][b, :k].tolist() == own
            r0 += k
    finally:
        dbg.close()
        prod.close()


def test_decodes_without_logits_equal_oracle_tokens():
    """Greedy, input-guided and batched decodes through the production epilogue: token for token
    those of the logits-keeping context, and the oracle's as far as its own top-2 margins leave no
    doubt (up to the oracle's first step with a margin under 2e-2, the logit tolerance; after a
    step that could resolve either way the two free-running sequences need not agree)."""
    cfg = CONFIGS[1]
    dims, w, dbg, prod = _ctx_pair("base", cfg["seed"], max_batch=4, max_src=64, max_len=64, k_max=72)
    try:
        srcs, max_out = draw_sources(cfg, dims["vocab"], n_sent=8)
        tok = O.Model(dims, w, np.float64, contract=True, max_pos=200)
        compared = 0
        for s, mo in zip(srcs, max_out):
            ga, _ = dbg.decode_greedy([s], max_out=[mo])
            gb, _ = prod.decode_greedy([s], max_out=[mo])
            assert ga == gb
            guide = edit_guide(ga[0], cfg["rate"], cfg["seed"], dims["vocab"])
            ia, sa = dbg.decode_iad([s], [guide], max_out=[mo])
            ib, sb = prod.decode_iad([s], [guide], max_out=[mo])
            assert ia == ib == ga and sa["iterations"] == sb["iterations"] and sa["rows_verified"] == sb["rows_verified"]
            g, lg = O.greedy(tok, s, int(mo), EOS, BOS, return_logits=True)
            srt = np.sort(lg, axis=1)
            small = np.flatnonzero(srt[:, -1] - srt[:, -2] < 2e-2)
            n_clear = int(small[0]) if small.size else len(g)
            assert gb[0][:n_clear] == g[:n_clear]
            compared += n_clear
        assert compared >= 15, compared
        # a batch of four through both contexts
        ga, _ = dbg.decode_greedy(srcs[:4], max_out=max_out[:4])
        guides = [edit_guide(g, cfg["rate"], cfg["seed"] + b, dims["vocab"]) for b, g in enumerate(ga)]
        ib, _ = prod.decode_iad(srcs[:4], guides, max_out=max_out[:4])
        assert ib == ga
    finally:
        dbg.close()
        prod.close()


@pytest.mark.parametrize("name,B", [("tiny", 2), ("base", 1), ("base", 3)])
def test_drafter_encoder_beside_the_verifier_encoder_equals_one_after_the_other(name, B):
    """The two encoders of a draft-then-verify decode on two streams (the drafter's in a second
    block of activation buffers) against the same two forwards back to back on one stream: the
    drafter's logits and tokens bit for bit, whole decodes token for token, over several sentences in
    a row (the next sentence's drafter encoder must wait for the previous sentence's drafts)."""
    rig = Rig(name, "bf16", 77, B=B, max_src=48, max_len=40, k_max=8, drafter=True)
    try:
        assert rig.ctx.get_option(ad.AD_OPT_OVERLAP_ENCODERS) == 1
        V = rig.dims["vocab"]
        sents = [_sources(rig.dims, 770 + i, [40 - 5 * b - i for b in range(B)]) for i in range(4)]
        res = {}
        for overlap in (0, 1):
            rig.ctx.set_option(ad.AD_OPT_OVERLAP_ENCODERS, overlap)
            got = []
            for rep in range(2):            # twice: the second pass replays the encoders' graphs
                for srcs in sents:
                    rig.ctx.encode(ad.AD_VERIFIER, srcs)
                    rig.ctx.encode(ad.AD_DRAFTER, srcs)
                    d1 = rig.ctx.draft_nat(8)
                    l1 = rig.ctx.debug_logits()
                    n, nx = rig.ctx.verify([list(map(int, d1[b])) for b in range(B)])
                    d2 = rig.ctx.draft_nat(5)
                    l2 = rig.ctx.debug_logits()
                    out, st = rig.ctx.decode_gad(srcs, 8, use_drafter=True)
                    got.append((d1.copy(), l1, n.copy(), nx.copy(), d2.copy(), l2, out, st["iterations"]))
            res[overlap] = got
        for a, b in zip(res[0], res[1]):
            assert np.array_equal(a[0], b[0]) and np.array_equal(a[4], b[4])
            assert np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
            assert np.array_equal(a[5].view(np.uint32), b[5].view(np.uint32))
            assert np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])
            assert a[6] == b[6] and a[7] == b[7]
        # and the drafter's first block against the oracle (the memory the second stream produced)
        rig.ctx.set_option(ad.AD_OPT_OVERLAP_ENCODERS, 1)
        srcs = sents[0]
        rig.ctx.encode(ad.AD_VERIFIER, srcs); rig.ctx.encode(ad.AD_DRAFTER, srcs)
        rig.ctx.draft_nat(8)
        got = rig.ctx.debug_logits()
        for i, s in enumerate(srcs):
            want = rig.dr.decode_full(rig.dr.encode(s), [BOS] + [SPECIAL["mask"]] * 8, causal=False)[1:]
            assert np.abs(got[8 * i:8 * i + 8] - want).max() < rig.tol
    finally:
        rig.close()
