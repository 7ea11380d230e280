"""Pins of the CPU oracle against what the paper and the mathematics fix (CPU only).

Each test names the passage it checks.  A plausible mistake in the oracle (a dropped term, a wrong
sign or index, a transposed operand, an off-by-one in N_left) fails at least one of them.
"""
import math
from fractions import Fraction
import os

import numpy as np
import pytest

import np_reference as ref
from oracle import psa_oracle as po

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- decoders, via one-token attention
@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
def test_single_token_attention_returns_value_bits_exactly(dtype):
    """Sec. 2.1: with one key, softmax is 1 and O = v.  Run over EVERY finite 16-bit pattern as a
    value, this pins the oracle's own fp16 / bf16 decoders against numpy's converters."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = po.decode(bits, dtype)
    bits = bits[np.isfinite(vals)]
    d = 128
    n = len(bits) // d
    bits = bits[: n * d].reshape(n, 1, 1, d)         # n pages, 1 head, 1 token, d channels
    rng = np.random.default_rng(0)
    k = rng.integers(0, 0x3C00, size=bits.shape, dtype=np.uint16)   # small finite keys
    q = rng.integers(0, 0x3C00, size=(n, 1, d), dtype=np.uint16)
    pb = po.Problem(q, k, bits, np.arange(n, dtype=np.int32).reshape(n, 1), np.ones(n, np.int32), dtype)
    out, _ = po.dense_attention(pb)
    assert np.array_equal(out[:, 0, :], po.decode(bits[:, 0, 0, :], dtype))


# ---------------------------------------------------------------- dense attention, Sec. 2.1
@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_dense_matches_library_softmax(dtype, seed):
    rng = np.random.default_rng(seed)
    pb = ref.random_problem(rng, B=3, Hq=6, Hkv=2, d=32, T=4, ctx=(1, 14, 32), dtype=dtype)
    out, lse = po.dense_attention(pb)
    rout, rlse = ref.dense(pb)
    np.testing.assert_allclose(out, rout, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, rlse, rtol=1e-12, atol=1e-13)


def test_dense_identical_keys_gives_mean_of_values():
    rng = np.random.default_rng(5)
    pb = ref.random_problem(rng, B=1, Hq=2, Hkv=1, d=8, T=4, ctx=(11,), shuffle=True)
    pb.k_pool[...] = pb.k_pool[0, 0, 0][None, None, None, :]
    out, lse = po.dense_attention(pb)
    _, v = ref.stream_kv(pb, 0, 0)
    np.testing.assert_allclose(out[0, 0], v.mean(0), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(out[0, 1], v.mean(0), rtol=1e-13, atol=1e-14)


def test_dense_empty_request_gives_zero():
    rng = np.random.default_rng(6)
    pb = ref.random_problem(rng, B=2, Hq=2, Hkv=1, d=8, T=4, ctx=(0, 5))
    out, lse = po.dense_attention(pb)
    assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0]))


def test_dense_transposed_q_k_would_fail():
    """q and k enter only through q.k; V only through P.V: swapping K and V pools must change the
    result (guards against a transposed operand going unnoticed by symmetric inputs)."""
    rng = np.random.default_rng(7)
    pb = ref.random_problem(rng, B=1, Hq=2, Hkv=1, d=8, T=4, ctx=(12,))
    out, _ = po.dense_attention(pb)
    swapped = po.Problem(pb.q, pb.v_pool, pb.k_pool, pb.block_table, pb.ctx_lens, pb.dtype)
    out2, _ = po.dense_attention(swapped)
    assert np.abs(out - out2).max() > 1e-3


# ---------------------------------------------------------------- block metadata, Sec. 2.2
@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
def test_metadata_is_bitwise_min_max_over_valid_tokens(dtype):
    rng = np.random.default_rng(11)
    pb = ref.random_problem(rng, B=2, Hq=4, Hkv=2, d=16, T=8, ctx=(19, 40), dtype=dtype)
    fill = pb.page_fill()
    meta = po.block_metadata(pb, fill)
    kd = po.decode(pb.k_pool, dtype)
    for p in range(pb.k_pool.shape[0]):
        f = fill[p]
        for h in range(2):
            if f == 0:
                assert not meta[p, h].any()
                continue
            lo, hi = kd[p, h, :f].min(0), kd[p, h, :f].max(0)
            assert np.array_equal(po.decode(meta[p, h, 0], dtype), lo)
            assert np.array_equal(po.decode(meta[p, h, 1], dtype), hi)
            # the result is one of the block's own bit patterns
            for c in range(16):
                assert meta[p, h, 0, c] in pb.k_pool[p, h, :f, c]
                assert meta[p, h, 1, c] in pb.k_pool[p, h, :f, c]


def test_metadata_signed_zero_order_and_full_pages_default():
    T, d = 4, 2
    k = np.zeros((1, 1, T, d), dtype=np.uint16)
    k[0, 0, :, 0] = [0x0000, 0x8000, 0x0000, 0x8000]   # +0 -0 +0 -0
    k[0, 0, :, 1] = [0x8000, 0x8000, 0x3C00, 0xBC00]   # -0 -0 +1 -1
    pb = po.Problem(np.zeros((1, 1, d), np.uint16), k, k.copy(), np.zeros((1, 1), np.int32),
                    np.array([T], np.int32), po.F16)
    meta = po.block_metadata(pb, None)              # NULL fill = all tokens valid
    assert meta[0, 0, 0, 0] == 0x8000 and meta[0, 0, 1, 0] == 0x0000
    assert meta[0, 0, 0, 1] == 0xBC00 and meta[0, 0, 1, 1] == 0x3C00
    meta2 = po.block_metadata(pb, np.array([2], np.int32))   # only the first two tokens
    assert meta2[0, 0, 0, 1] == 0x8000 and meta2[0, 0, 1, 1] == 0x8000


# ---------------------------------------------------------------- criticality score, Alg. 1 line 5
@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
def test_score_bounds_every_token_logit_and_is_tight_for_one_token(dtype):
    rng = np.random.default_rng(21)
    pb = ref.random_problem(rng, B=2, Hq=6, Hkv=2, d=16, T=4, ctx=(13, 29), dtype=dtype)
    meta = po.block_metadata(pb, pb.page_fill())
    ub, cs = po.block_scores(pb, meta)
    G, T = 3, 4
    for r in range(2):
        n = int(pb.num_blocks()[r])
        for hq in range(6):
            s = ref.logits(pb, r, hq)
            for b in range(n):
                blk = s[b * T:(b + 1) * T]
                assert ub[r, hq, b] >= blk.max() - 1e-12
                if len(blk) == 1:        # one valid token: the cuboid is a point, the bound is tight
                    assert abs(ub[r, hq, b] - blk[0]) < 1e-12
        for h in range(2):
            np.testing.assert_array_equal(cs[r, h, :n], ub[r, h * G:(h + 1) * G, :n].max(0))
    assert (13 % T == 1)   # the case above really contains a one-token block


def test_score_matches_closed_form_choice_of_corner():
    """The maximum of q.k over a box is reached at the corner that takes kmax where q > 0 and kmin
    where q < 0 (textbook LP over a box); library-routine form of the same number."""
    rng = np.random.default_rng(22)
    pb = ref.random_problem(rng, B=1, Hq=2, Hkv=1, d=32, T=8, ctx=(64,))
    meta = po.block_metadata(pb, pb.page_fill())
    ub, _ = po.block_scores(pb, meta)
    for hq in range(2):
        q = po.decode(pb.q[0, hq], pb.dtype)
        for b in range(8):
            page = pb.block_table[0, b]
            lo, hi = po.decode(meta[page, 0, 0], pb.dtype), po.decode(meta[page, 0, 1], pb.dtype)
            corner = np.where(q > 0, hi, lo)
            assert abs(ub[0, hq, b] - q @ corner / math.sqrt(32)) < 1e-12


# ---------------------------------------------------------------- ranking, Alg. 1 line 6
def test_order_is_descending_permutation_with_ties_to_smaller_index():
    rng = np.random.default_rng(31)
    pb = ref.random_problem(rng, B=2, Hq=2, Hkv=2, d=8, T=2, ctx=(40, 23))
    keys = np.full((2, 2, 20), -np.inf)
    keys[0, :, :20] = rng.integers(0, 5, size=(2, 20))       # many ties
    keys[1, :, :12] = rng.integers(0, 3, size=(2, 12))
    order = po.block_order(pb, keys)
    for r, n in ((0, 20), (1, 12)):
        for h in range(2):
            o = order[r, h, :n]
            assert sorted(o.tolist()) == list(range(n))
            k = keys[r, h, o]
            assert np.all(np.diff(k) <= 0)
            same = np.diff(k) == 0
            assert np.all(np.diff(o)[same] > 0)
            assert np.all(order[r, h, n:] == -1)
            # library routine: stable argsort of the negated keys
            assert np.array_equal(o, np.argsort(-keys[r, h, :n], kind="stable"))


@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
def test_center_score_is_the_mean_of_the_extreme_logits_of_the_cuboid(dtype):
    """Cuboid-centre scorer: q.(kmin+kmax)/2/sqrt(d).  Brute force over the cuboid's corners gives the
    largest and the smallest logit it allows (LP over a box); the centre's logit is their mean, it lies
    between the block's smallest and largest possible logit, and it is the exact logit when the block
    holds one token.  The group reduce stays a max."""
    rng = np.random.default_rng(23)
    pb = ref.random_problem(rng, B=2, Hq=6, Hkv=2, d=16, T=4, ctx=(13, 29), dtype=dtype)
    meta = po.block_metadata(pb, pb.page_fill())
    ce, cs = po.block_scores(pb, meta, po.CUBOID_CENTER)
    ub, _ = po.block_scores(pb, meta, po.UPPER_BOUND)
    G, T = 3, 4
    for r in range(2):
        n = int(pb.num_blocks()[r])
        for hq in range(6):
            q = po.decode(pb.q[r, hq], pb.dtype)
            s = ref.logits(pb, r, hq)
            for b in range(n):
                page = pb.block_table[r, b]
                lo, hi = po.decode(meta[page, hq // G, 0], pb.dtype), po.decode(meta[page, hq // G, 1], pb.dtype)
                top = q @ np.where(q > 0, hi, lo) / math.sqrt(16)
                bottom = q @ np.where(q > 0, lo, hi) / math.sqrt(16)
                assert abs(top - ub[r, hq, b]) < 1e-12
                assert abs(ce[r, hq, b] - 0.5 * (top + bottom)) < 1e-12
                assert abs(ce[r, hq, b] - q @ (0.5 * (lo + hi)) / math.sqrt(16)) < 1e-12
                blk = s[b * T:(b + 1) * T]
                assert bottom - 1e-12 <= blk.min() and blk.max() <= top + 1e-12
                if len(blk) == 1:
                    assert abs(ce[r, hq, b] - blk[0]) < 1e-12
        for h in range(2):
            np.testing.assert_array_equal(cs[r, h, :n], ce[r, h * G:(h + 1) * G, :n].max(0))


def _nearest_16bit(x: Fraction, dtype: int) -> int:
    """The storage type's bit pattern nearest to the exact rational x (ties to the even pattern), found by
    exact comparison: every finite non-negative pattern is tried as a neighbour of x's truncation."""
    neg = x < 0
    a = -x if neg else x
    top = 0x7bff if dtype == po.F16 else 0x7f7f                      # largest finite pattern
    vals = lambda b: Fraction(float(po.decode(np.array([b], dtype=np.uint16), dtype)[0]))
    lo, hi = 0, top                                                   # patterns are monotone in value
    while lo < hi:
        mid = (lo + hi + 1) // 2
        if vals(mid) <= a:
            lo = mid
        else:
            hi = mid - 1
    below, above = lo, min(lo + 1, top)
    d0, d1 = a - vals(below), vals(above) - a
    pick = below if (d0 < d1 or (d0 == d1 and below % 2 == 0) or above == below) else above
    return pick | (0x8000 if neg else 0)


@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
def test_mean_key_metadata_is_the_exactly_rounded_mean_of_the_valid_keys(dtype):
    """Mean-key metadata against exact rational arithmetic: the mean of the block's valid keys per channel,
    rounded once to the nearest pattern of the storage type (ties to even).  Partly filled pages count their
    valid tokens only, an empty page gives +0, a one-token page gives the token itself."""
    rng = np.random.default_rng(29)
    pb = ref.random_problem(rng, B=2, Hq=4, Hkv=2, d=8, T=4, ctx=(13, 6), dtype=dtype)
    fill = pb.page_fill()
    # values that stress the rounding: tiny and large magnitudes, exact ties (x and x + 1 ulp average to a tie)
    k = pb.k_pool.copy()
    k[0, 0, 0, 0], k[0, 0, 1, 0], k[0, 0, 2, 0], k[0, 0, 3, 0] = 0x3c00, 0x3c01, 0x3c00, 0x3c01
    k[0, 0, :, 1] = [0x0001, 0x0001, 0x0002, 0x0000]                       # subnormals
    k[0, 1, :, 2] = [0x8000, 0x8000, 0x8000, 0x8000]                       # all -0
    pb = po.Problem(pb.q, k, pb.v_pool, pb.block_table, pb.ctx_lens, pb.dtype)
    means = po.block_means(pb, fill)
    P, H, T, D = pb.k_pool.shape
    assert means[0, 1, 2] == 0                                            # a zero mean is +0, whatever the zeros' signs
    for p in range(P):
        for h in range(H):
            for c in range(D):
                n = int(fill[p])
                if n == 0:
                    assert means[p, h, c] == 0
                    continue
                vals = [Fraction(float(po.decode(pb.k_pool[p, h, t, c:c + 1], dtype)[0])) for t in range(n)]
                exact = sum(vals) / n
                if exact == 0:
                    assert means[p, h, c] == 0
                    continue
                assert means[p, h, c] == _nearest_16bit(exact, dtype), (p, h, c)
                if n == 1:
                    assert means[p, h, c] == pb.k_pool[p, h, 0, c]


@pytest.mark.parametrize("dtype", [po.F16, po.BF16])
def test_mean_key_score_is_the_mean_of_the_blocks_token_logits(dtype):
    """Scorer 2: q . mean / sqrt(d) = the mean of the scaled logits of the block's tokens, up to the rounding of
    the stored mean (half a unit in the last place per channel); the group reduce is a max; with one token per
    block the score is that token's logit exactly."""
    rng = np.random.default_rng(31)
    pb = ref.random_problem(rng, B=2, Hq=6, Hkv=2, d=16, T=4, ctx=(13, 29), dtype=dtype)
    means = po.block_means(pb, pb.page_fill())
    per_head, cs = po.block_scores(pb, means, po.MEAN_KEY)
    G, T = 3, 4
    ulp = 2.0 ** (-10 if dtype == po.F16 else -7)
    for r in range(2):
        n = int(pb.num_blocks()[r])
        for hq in range(6):
            q = po.decode(pb.q[r, hq], pb.dtype)
            s = ref.logits(pb, r, hq)
            for b in range(n):
                blk = s[b * T:(b + 1) * T]
                mean_vec = po.decode(means[pb.block_table[r, b], hq // G], pb.dtype)
                bound = float(np.abs(q) @ (np.abs(mean_vec) * ulp * 0.5 + 2.0 ** -24)) / math.sqrt(16) + 1e-12
                assert abs(per_head[r, hq, b] - blk.mean()) <= bound
                assert abs(per_head[r, hq, b] - q @ mean_vec / math.sqrt(16)) < 1e-12
                if len(blk) == 1:
                    assert abs(per_head[r, hq, b] - blk[0]) < 1e-12
        for h in range(2):
            np.testing.assert_array_equal(cs[r, h, :n], per_head[r, h * G:(h + 1) * G, :n].max(0))


def test_scorer_changes_the_ranking_not_the_rule():
    """With either scorer the progressive loop is the same function of the ranking it is given."""
    pb = _problem(51)
    for scorer in (po.UPPER_BOUND, po.CUBOID_CENTER, po.MEAN_KEY):
        res = po.psa_decode(pb, 0.9, 2, scorer=scorer)
        meta = po.block_means(pb, pb.page_fill()) if scorer == po.MEAN_KEY else po.block_metadata(pb, pb.page_fill())
        _, cs = po.block_scores(pb, meta, scorer)
        again = po.psa_decode_ordered(pb, po.block_order(pb, cs), 0.9, 2)
        assert np.array_equal(res.n_selected, again.n_selected) and np.array_equal(res.out, again.out)
        np.testing.assert_allclose(po.attend_prefix(pb, res.order, res.n_selected), res.out, rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- progressive loop, Alg. 1 lines 7-19
def _problem(seed, dtype=po.F16, **kw):
    rng = np.random.default_rng(seed)
    args = dict(B=3, Hq=4, Hkv=2, d=16, T=4, ctx=(37, 64, 5), dtype=dtype, scale=1.5)
    args.update(kw)
    return ref.random_problem(rng, **args)


@pytest.mark.parametrize("m", [1, 3, 4, 100])
def test_threshold_one_equals_dense(m):
    """Strict '>' (line 17) never fires at eps = 1, so lines 11-12 must rebuild exact attention."""
    pb = _problem(41)
    res = po.psa_decode(pb, 1.0, m)
    rout, _ = ref.dense(pb)
    np.testing.assert_allclose(res.out, rout, rtol=1e-11, atol=1e-12)
    G = 2
    assert np.array_equal(res.n_selected, np.repeat(pb.num_blocks(), 4).reshape(3, 4))
    assert np.all(res.mass_est == 1.0)
    assert np.array_equal(res.blocks_read, res.n_selected.reshape(3, 2, G).max(-1))


@pytest.mark.parametrize("eps,m", [(0.5, 1), (0.8, 1), (0.9, 2), (0.95, 4), (0.99, 3)])
def test_selected_set_is_ranked_prefix_and_output_is_attention_over_it(eps, m):
    """Lines 11-12 are the online-softmax merge: at the stop, O_acc equals plain softmax attention
    over exactly the consumed blocks, which are the first n of the ranking."""
    pb = _problem(42)
    res = po.psa_decode(pb, eps, m, curves=True)
    for r in range(3):
        for hq in range(4):
            n = res.n_selected[r, hq]
            blocks = res.order[r, hq // 2, :n]
            np.testing.assert_allclose(res.out[r, hq], ref.attend_blocks(pb, r, hq, blocks),
                                       rtol=1e-11, atol=1e-12)
    # the oracle's own by-definition prefix attention agrees too
    np.testing.assert_allclose(po.attend_prefix(pb, res.order, res.n_selected), res.out,
                               rtol=1e-11, atol=1e-12)


@pytest.mark.parametrize("eps,m", [(0.3, 1), (0.7, 1), (0.9, 1), (0.9, 4), (0.97, 5)])
def test_stop_rule_first_admissible_index_against_brute_force(eps, m):
    """Lines 12-18 with AS_b from scipy.logsumexp over the block's logits: curve, stop index,
    estimate, and the paper's claim that the estimate exceeds eps unless all blocks are used."""
    pb = _problem(43)
    res = po.psa_decode(pb, eps, m, curves=True)
    nb = pb.num_blocks()
    for r in range(3):
        for hq in range(4):
            N = int(nb[r])
            o = res.order[r, hq // 2, :N]
            lse = ref.block_lse(pb, r, hq)[o]
            p = ref.p_acc_curve(lse)
            np.testing.assert_allclose(res.p_acc[r, hq, :N], p, rtol=1e-10)
            np.testing.assert_allclose(res.block_lse[r, hq, :N], lse, rtol=1e-10, atol=1e-10)
            assert np.all(np.diff(p) >= -1e-12)                       # non-decreasing
            n = ref.first_stop(p, eps, m)
            assert res.n_selected[r, hq] == n
            assert abs(res.mass_est[r, hq] - p[n - 1]) < 1e-10
            assert res.mass_est[r, hq] > eps or n == N
            assert n % m == 0 or n == N
            # true mass curve = cumulative share of the exponentiated logits
            a = np.exp(lse - lse.max())
            np.testing.assert_allclose(res.true_mass[r, hq, :N], np.cumsum(a) / a.sum(), rtol=1e-10)


@pytest.mark.parametrize("eps", [0.6, 0.9, 0.97])
def test_microbatch_identity(eps):
    """P_acc(n) is non-decreasing, hence n(m) = min(N, m * ceil(n(1) / m))  (Sec. 3.2, microbatch)."""
    pb = _problem(44)
    n1 = po.psa_decode(pb, eps, 1).n_selected
    N = np.repeat(pb.num_blocks(), 4).reshape(3, 4)
    for m in (2, 3, 4, 7, 16):
        nm = po.psa_decode(pb, eps, m).n_selected
        assert np.array_equal(nm, np.minimum(N, m * ((n1 + m - 1) // m)))


def test_threshold_zero_stops_after_first_microbatch_and_single_block_is_exact():
    pb = _problem(45)
    N = np.repeat(pb.num_blocks(), 4).reshape(3, 4)
    for m in (1, 3, 50):
        res = po.psa_decode(pb, 0.0, m)
        assert np.array_equal(res.n_selected, np.minimum(m, N))
    one = _problem(46, B=1, ctx=(3,))                   # N = 1
    res = po.psa_decode(one, 0.5, 1)
    assert np.all(res.n_selected == 1) and np.all(res.mass_est == 1.0)
    rout, _ = ref.dense(one)
    np.testing.assert_allclose(res.out, rout, rtol=1e-12, atol=1e-13)


def test_empty_request():
    pb = _problem(47, ctx=(0, 9, 0))
    res = po.psa_decode(pb, 0.9, 1)
    for r in (0, 2):
        assert np.all(res.out[r] == 0) and np.all(res.n_selected[r] == 0)
        assert np.all(res.mass_est[r] == 0) and np.all(res.blocks_read[r] == 0)


def test_true_mass_dominates_estimate_under_ideal_order():
    """Sec. 3.2 calls AS_min an upper bound of the unread blocks' AS.  That holds when blocks come
    in descending true AS; then P_acc(n) <= true accumulated weight for every n (brute force)."""
    for seed in range(8):
        pb = _problem(100 + seed, B=2, Hq=2, Hkv=2, ctx=(61, 40))      # G = 1: one head per ranking
        keys = np.full((2, 2, 16), -np.inf)
        for r in range(2):
            for h in range(2):
                l = ref.block_lse(pb, r, h)
                keys[r, h, :len(l)] = l
        order = po.block_order(pb, keys)
        res = po.psa_decode_ordered(pb, order, 0.9, 1, curves=True)
        for r in range(2):
            N = int(pb.num_blocks()[r])
            assert np.all(res.true_mass[r, :, :N] >= res.p_acc[r, :, :N] - 1e-12)
            n = res.n_selected[r]
            for h in range(2):
                assert res.true_mass[r, h, n[h] - 1] > 0.9 or n[h] == N


def test_heads_of_a_group_stop_independently_and_blocks_read_is_their_max():
    """Sec. 3.2, batched form: a query that passed the threshold is removed, the rest go on."""
    pb = _problem(48, B=1, Hq=4, Hkv=1, ctx=(64,))
    res = po.psa_decode(pb, 0.8, 1)
    assert len(set(res.n_selected[0].tolist())) > 1          # the case really has different stops
    assert res.blocks_read[0, 0] == res.n_selected[0].max()
    # each head alone (G = 1 problem with the same shared ranking) gives the same stop and output
    for g in range(4):
        solo = po.Problem(pb.q[:, g:g + 1], pb.k_pool, pb.v_pool, pb.block_table, pb.ctx_lens, pb.dtype)
        r1 = po.psa_decode_ordered(solo, res.order, 0.8, 1)
        assert r1.n_selected[0, 0] == res.n_selected[0, g]
        np.testing.assert_array_equal(r1.out[0, 0], res.out[0, g])


# ---------------------------------------------------------------- closed-form hand case
def test_three_block_hand_case():
    """d = 4 (sqrt d = 2), q = (2,0,0,0), keys (x,0,0,0): the scaled logit of a token is x.
    Blocks of two tokens with x = 2, 1, 0 give AS = 2e^2, 2e, 2 (up to the common reference), so by
    lines 12-16:  P_acc(1) = 2e^2 / (2e^2 + 2*2e^2) = 1/3,
                  P_acc(2) = (2e^2 + 2e) / (2e^2 + 2e + 1*2e) = (e + 1) / (e + 2),   P_acc(3) = 1.
    With eps = 0.5 the loop stops at n = 2 and O = (e*v_0 + v_1) / (e + 1) channel-wise, where v_b
    is the mean of block b's two values."""
    one, two = 0x3C00, 0x4000
    k = np.zeros((3, 1, 2, 4), np.uint16)
    k[1, 0, :, 0] = two          # physical page 1 = logical block 0
    k[2, 0, :, 0] = one          # page 2 = block 1
    v = np.zeros((3, 1, 2, 4), np.uint16)     # page 0 = block 2: x = 0
    v[1, 0, 0, :] = [one, 0, two, 0]
    v[1, 0, 1, :] = [one, two, 0, 0]          # block 0 mean: (1, 1, 1, 0)
    v[2, 0, :, :] = [[0, 0, 0, two], [0, 0, 0, two]]   # block 1 mean: (0, 0, 0, 2)
    q = np.array([[[two, 0, 0, 0]]], np.uint16)
    pb = po.Problem(q, k, v, np.array([[1, 2, 0]], np.int32), np.array([6], np.int32), po.F16)
    res = po.psa_decode(pb, 0.5, 1, curves=True)
    e = math.e
    assert res.order[0, 0].tolist() == [0, 1, 2]
    np.testing.assert_allclose(res.cs[0, 0], [2.0, 1.0, 0.0], atol=1e-15)
    np.testing.assert_allclose(res.p_acc[0, 0], [1 / 3, (e + 1) / (e + 2), 1.0], rtol=1e-14)
    assert res.n_selected[0, 0] == 2 and res.blocks_read[0, 0] == 2
    assert abs(res.mass_est[0, 0] - (e + 1) / (e + 2)) < 1e-14
    np.testing.assert_allclose(res.out[0, 0], np.array([e, e, e, 2.0]) / (e + 1), rtol=1e-14)
    # eps just below and above P_acc(1)
    assert po.psa_decode(pb, 0.33, 1).n_selected[0, 0] == 1
    assert po.psa_decode(pb, 0.34, 1).n_selected[0, 0] == 2
    assert po.psa_decode(pb, 0.8, 1).n_selected[0, 0] == 3      # (e+1)/(e+2) = 0.788 < 0.8


# ---------------------------------------------------------------- the paper's worked example
def test_worked_example_microbatches_behaviour():
    """Sec. 3.2, figure 'an example of executing PSA': 12 ranked blocks, microbatch m = 4,
    eps = 0.98; the accumulated weight is examined after each microbatch (0.61, 0.91, 0.98) and the
    computation ends with the third.  The figure's labels are criticality scores, not AS values
    (no N_left satisfies lines 15-16 for them), so only the behaviour is pinned: tests happen at
    n = 4, 8, 12 and nowhere else, and the run lasts three microbatches.  Arithmetic unpinned."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "worked_example_sec3_2.txt"))
            if l.strip() and not l.startswith("#")]
    labels = np.array([float(x) for x in rows[0]])
    m, eps = int(rows[1][0]), float(rows[1][1])
    printed = [float(x) for x in rows[2]]
    assert len(labels) == 12 and m == 4 and eps == 0.98 and len(printed) == 3
    # one token per block whose logit is log(label): AS_b is proportional to the label, and the
    # ranking by the (tight, one-token) bound is the printed order.  d = 4, q = (2,0,0,0).
    T = 1
    k = np.zeros((12, 1, T, 4), np.float16)
    k[:, 0, 0, 0] = np.log(labels)
    pb = po.Problem(np.array([[[0x4000, 0, 0, 0]]], np.uint16), k.view(np.uint16),
                    np.zeros((12, 1, T, 4), np.uint16), np.arange(12, dtype=np.int32)[None],
                    np.array([12], np.int32), po.F16)
    res = po.psa_decode(pb, eps, m, curves=True)
    assert res.order[0, 0].tolist() == list(range(12))
    assert res.n_selected[0, 0] == 12                      # three microbatches of four
    for mm in (1, 2, 3, 4, 6):
        n = po.psa_decode(pb, eps, mm).n_selected[0, 0]
        assert n % mm == 0 or n == 12
    # with m = 4 a stop can only land on 4, 8 or 12 whatever the threshold
    for e_ in np.linspace(0.05, 0.999, 40):
        assert po.psa_decode(pb, float(e_), 4).n_selected[0, 0] in (4, 8, 12)


# ---------------------------------------------------------------- fixed-budget control (Sec. 1, 2.2)
@pytest.mark.parametrize("k", [1, 2, 5, 9, 100])
def test_topk_is_attention_over_the_k_best_scored_blocks(k):
    """Brute force: pick the k largest criticality scores per KV head (ties to the smaller block),
    attend those blocks by the definition of softmax attention."""
    pb = _problem(47)
    res = po.topk_attention(pb, k)
    _, cs = po.block_scores(pb, po.block_metadata(pb, pb.page_fill()))
    nb = pb.num_blocks()
    for r in range(3):
        N = int(nb[r])
        for hq in range(4):
            sel = np.argsort(-cs[r, hq // 2, :N], kind="stable")[:k]
            assert res.n_selected[r, hq] == min(k, N)
            np.testing.assert_allclose(res.out[r, hq], ref.attend_blocks(pb, r, hq, sel), rtol=1e-11, atol=1e-12)
            # the reported estimate is the P_acc curve read at min(k, N)
            p = ref.p_acc_curve(ref.block_lse(pb, r, hq)[res.order[r, hq // 2, :N]])
            assert abs(res.mass_est[r, hq] - p[min(k, N) - 1]) < 1e-10
    assert np.array_equal(res.blocks_read, np.repeat(np.minimum(k, nb)[:, None], 2, 1))


def test_topk_with_budget_covering_everything_is_dense_and_empty_request_is_zero():
    pb = _problem(48, ctx=(37, 0, 5))
    res = po.topk_attention(pb, 1000)
    rout, _ = ref.dense(pb)
    np.testing.assert_allclose(res.out, rout, rtol=1e-11, atol=1e-12)
    assert np.all(res.mass_est[[0, 2]] == 1.0)
    assert not res.out[1].any() and np.all(res.n_selected[1] == 0) and np.all(res.mass_est[1] == 0)


@pytest.mark.parametrize("k", [1, 3, 8])
def test_topk_equals_progressive_loop_with_threshold_zero_and_microbatch_k(k):
    """Algorithm 1 tests the stop only every m blocks; with eps = 0 the first test passes, so the
    loop with m = k is the fixed top-k baseline."""
    pb = _problem(49)
    a, b = po.topk_attention(pb, k), po.psa_decode(pb, 0.0, k)
    assert np.array_equal(a.n_selected, b.n_selected)
    np.testing.assert_allclose(a.out, b.out, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(a.mass_est, b.mass_est, rtol=1e-12)


def test_prefix_lse_is_logsumexp_of_the_attended_logits_and_true_mass_follows():
    """The log-denominator of attention over a ranked prefix, against scipy's logsumexp over the same
    tokens' logits; over all blocks it is the dense one; exp(prefix - dense) is the true-mass curve."""
    from scipy.special import logsumexp
    pb = _problem(50)
    res = po.psa_decode(pb, 0.8, 1, curves=True)
    _, lse = po.attend_prefix(pb, res.order, res.n_selected, want_lse=True)
    _, dense_lse = ref.dense(pb)
    nb = pb.num_blocks()
    for r in range(3):
        for hq in range(4):
            n = res.n_selected[r, hq]
            blocks = res.order[r, hq // 2, :n]
            want = logsumexp(ref.block_lse(pb, r, hq)[blocks])
            assert abs(lse[r, hq] - want) < 1e-10
            assert abs(np.exp(lse[r, hq] - dense_lse[r, hq]) - res.true_mass[r, hq, n - 1]) < 1e-10
    full = np.repeat(nb[:, None], 4, 1).astype(np.int32)
    _, lse_all = po.attend_prefix(pb, res.order, full, want_lse=True)
    np.testing.assert_allclose(lse_all, dense_lse, rtol=0, atol=1e-10)


# ---------------------------------------------------------------- incremental decode (Sec. 3.1)
def test_append_puts_the_token_at_the_end_of_the_request_and_metadata_follows():
    """After an append, the request's key/value sequence is the old one plus the new token; the
    metadata of the new cache (built the plain way) is numpy's min/max over each block's valid tokens;
    attention over the new cache therefore sees exactly one more token."""
    rng = np.random.default_rng(60)
    full = ref.random_problem(rng, B=3, Hq=4, Hkv=2, d=16, T=4, ctx=(12, 12, 4))     # pages for three blocks each
    pb = po.Problem(full.q, full.k_pool, full.v_pool, full.block_table, np.array([7, 8, 0], dtype=np.int32), full.dtype)
    k_new = rng.integers(0, 0x3c00, size=(3, 2, 16), dtype=np.uint16)       # positive finite halves
    v_new = rng.integers(0, 0x3c00, size=(3, 2, 16), dtype=np.uint16)
    new, status = po.append_kv(pb, k_new, v_new)
    assert np.array_equal(status, [0, 0, 0]) and np.array_equal(new.ctx_lens, [8, 9, 1])
    for r in range(3):
        for h in range(2):
            k1, v1 = ref.stream_kv(new, r, h)
            assert len(k1) == pb.ctx_lens[r] + 1
            if pb.ctx_lens[r] > 0:
                k0, v0 = ref.stream_kv(pb, r, h)
                assert np.array_equal(k1[:-1], k0) and np.array_equal(v1[:-1], v0)
            assert np.array_equal(k1[-1], po.decode(k_new[r, h], pb.dtype))
            assert np.array_equal(v1[-1], po.decode(v_new[r, h], pb.dtype))
    meta = po.block_metadata(new, new.page_fill())
    T = 4
    for r in range(3):
        for b in range(int(new.num_blocks()[r])):
            page = new.block_table[r, b]
            valid = min(T, int(new.ctx_lens[r]) - b * T)
            kk = po.decode(new.k_pool[page, :, :valid, :], new.dtype)
            assert np.array_equal(po.decode(meta[page, :, 0], new.dtype), kk.min(1))
            assert np.array_equal(po.decode(meta[page, :, 1], new.dtype), kk.max(1))
    # untouched: the old problem object
    assert np.array_equal(pb.ctx_lens, [7, 8, 0])


def test_append_refuses_a_full_row_and_a_page_outside_the_pool():
    rng = np.random.default_rng(61)
    pb = ref.random_problem(rng, B=2, Hq=2, Hkv=1, d=16, T=4, ctx=(8, 3))           # rows of two blocks
    pb.block_table[1, 0] = 999
    tok = np.zeros((2, 1, 16), dtype=np.uint16)
    new, status = po.append_kv(pb, tok, tok)
    assert np.array_equal(status, [2, 1]) and np.array_equal(new.ctx_lens, [8, 3])
    assert np.array_equal(new.k_pool, pb.k_pool)
