"""CPU tests of the parity checker itself (tests/gpu_common.py): it is fed stand-ins for the GPU's outputs that
are computed by the oracle, with a deviation planted on purpose, and must put each head into the right class --
or refuse.  This pins the RULE the GPU tests apply (selected sets equal except blocks within 1e-3 of the stopping
boundary; a different stop only through a ranking that swaps blocks whose scores agree within the score error, or
with P_acc on the threshold), independently of what any kernel happens to produce."""
from types import SimpleNamespace

import numpy as np
import pytest
import torch

import gpu_common as gc
from oracle import psa_oracle as po
from workloads import generate_layer, get_config

EPS, M = 0.9, 1


def _problem():
    cfg = get_config(1).scaled(batch=1, ctx=2048, num_q_heads=8, num_kv_heads=4)
    li = generate_layer(cfg, device="cpu")
    return gc.to_problem(li)


def _stand_in(pb, order, scores):
    """What a GPU that ranks like `order` (with its own `scores`) and otherwise follows Algorithm 1 exactly would
    return: the oracle run over that ranking."""
    res = po.psa_decode_ordered(pb, order, EPS, M)
    _, lse = po.attend_prefix(pb, order, res.n_selected, want_lse=True)
    t = torch.from_numpy
    return SimpleNamespace(out=t(res.out.astype(np.float32)), n_selected=t(res.n_selected), mass_est=t(res.mass_est.astype(np.float32)),
                           blocks_read=t(res.blocks_read), order=t(order.copy()), scores=t(scores.astype(np.float32)),
                           lse=t(lse.astype(np.float32)))


def _twin_last_selected(pb, ora, hq, G, lower=None):
    """Rewrites the keys of the block ranked right after head hq's stop so that its per-channel minimum and
    maximum -- hence its score -- equal those of the last selected block, while its tokens (hence its AS)
    differ: token 0 = the minima, token 1 = the maxima, the rest copies of token 0.  With lower = (channel, k)
    the twin's maximum in that channel is moved k representable steps towards zero, which separates the two
    scores by a small, known amount."""
    h = hq // G
    n = int(ora.n_selected[0, hq])
    a, b = int(ora.order[0, h, n - 1]), int(ora.order[0, h, n])
    pa, pbk = int(pb.block_table[0, a]), int(pb.block_table[0, b])
    ka = po.decode(pb.k_pool[pa, h], pb.dtype)               # [16][128]
    lo_t, hi_t = ka.argmin(0), ka.argmax(0)
    kmin = pb.k_pool[pa, h][lo_t, np.arange(ka.shape[1])]
    kmax = pb.k_pool[pa, h][hi_t, np.arange(ka.shape[1])]
    k_pool = pb.k_pool.copy()
    k_pool[pbk, h, :, :] = kmin
    k_pool[pbk, h, 1, :] = kmax
    if lower is not None:
        c, k = lower
        k_pool[pbk, h, 1, c] = kmax[c] - np.uint16(k)        # same sign, smaller magnitude (k is small)
    return po.Problem(pb.q, k_pool, pb.v_pool, pb.block_table, pb.ctx_lens, pb.dtype), a, b


def test_identical_outputs_are_set_equal():
    pb = _problem()
    ora = po.psa_decode(pb, EPS, M)
    rep = gc.check_decode_against_oracle(pb, _stand_in(pb, ora.order, ora.cs), EPS, M)
    assert rep.set_equal == rep.heads == 8 and rep.worst_out_elem <= 1e-6
    rep.assert_accounted(max_rank_swaps=0, max_stop_flips=0)


def _first_head_whose_stop_moves(pb):
    """Searches the heads for one where ranking the twin before the last selected block changes the stop."""
    ora0 = po.psa_decode(pb, EPS, M)
    B, Hq, H = pb.q.shape[0], pb.q.shape[1], pb.k_pool.shape[1]
    G = Hq // H
    hits = []
    for hq in range(Hq):
        if int(ora0.n_selected[0, hq]) >= int(pb.num_blocks()[0]):
            continue
        pb2, a, b = _twin_last_selected(pb, ora0, hq, G)
        ora = po.psa_decode(pb2, EPS, M)
        h = hq // G
        n = int(ora.n_selected[0, hq])
        ranks = {int(x): i for i, x in enumerate(ora.order[0, h])}
        if ora.cs[0, h, a] != ora.cs[0, h, b] or abs(ranks[a] - ranks[b]) != 1:
            continue
        order = ora.order.copy()
        ra, rb = ranks[a], ranks[b]
        order[0, h, ra], order[0, h, rb] = order[0, h, rb], order[0, h, ra]
        alt = po.psa_decode_ordered(pb2, order, EPS, M)
        hits.append((hq, pb2, ora, order, a, b, bool((alt.n_selected != ora.n_selected).any())))
    return hits


def test_a_swap_of_equal_scored_blocks_is_a_rank_swap_or_a_boundary_tie_never_a_failure():
    pb = _problem()
    hits = _first_head_whose_stop_moves(pb)
    assert hits, "the construction found no head to twin"
    seen_swap = seen_tie = False
    for hq, pb2, ora, order, a, b, moved in hits:
        h = hq // (pb.q.shape[1] // pb.k_pool.shape[1])
        scores = ora.cs.copy()
        lo, hi = sorted((a, b))
        # the stand-in's own scores must order the pair the other way round: a hair apart, as binary32 would
        later = order[0, h].tolist().index(a) > order[0, h].tolist().index(b)
        scores[0, h, a if later else b] -= 2e-6
        rep = gc.check_decode_against_oracle(pb2, _stand_in(pb2, order, scores), EPS, M)
        rep.assert_accounted(max_rank_swaps=8, max_stop_flips=0)
        assert rep.set_equal + rep.set_tolerated + rep.rank_swap_stops == rep.heads
        assert rep.worst_swap_gap <= 1e-12
        seen_swap |= rep.rank_swap_stops > 0
        seen_tie |= rep.set_tolerated > 0
        assert (rep.rank_swap_stops > 0) == moved
    assert seen_swap, "no head's stop moved: the rank-swap class was not exercised"


@pytest.mark.parametrize("lo,hi,caught_by", [(2.8e-4, 4.8e-4, "apart in score"), (2e-3, 2e-2, None)])
def test_a_swap_of_blocks_further_apart_than_the_score_error_is_refused(lo, hi, caught_by):
    """The stand-in ranks a block before one that scores a little higher, right at a head's stop, so that the stops
    differ.  A gap just above the score error (2.5e-4) can come with scores that are each within the score error
    of the oracle's, and passes the rank-by-rank ranking check (1e-3): the bound on swapped scores must catch it.
    A larger gap is caught earlier."""
    pb = _problem()
    ora0 = po.psa_decode(pb, EPS, M)
    G = pb.q.shape[1] // pb.k_pool.shape[1]
    N = int(pb.num_blocks()[0])
    refused = 0
    for hq in range(pb.q.shape[1]):
        h = hq // G
        if int(ora0.n_selected[0, hq]) >= N:
            continue
        found = None
        for c in range(0, 128, 3):
            for k in (1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144):
                pb2, a, b = _twin_last_selected(pb, ora0, hq, G, lower=(c, k))
                _, cs = po.block_scores(pb2, po.block_metadata(pb2, pb2.page_fill()))
                if lo <= cs[0, h, a] - cs[0, h, b] <= hi:
                    found = (pb2, a, b)
                    break
            if found:
                break
        if not found:
            continue
        pb2, a, b = found
        ora = po.psa_decode(pb2, EPS, M)
        rk = ora.order[0, h].tolist()
        ra, rb = rk.index(a), rk.index(b)
        if rb != ra + 1:
            continue
        order = ora.order.copy()
        order[0, h, ra], order[0, h, rb] = b, a
        alt = po.psa_decode_ordered(pb2, order, EPS, M)
        if not (alt.n_selected != ora.n_selected).any():
            continue
        scores = ora.cs.copy()                  # consistent with the stand-in's ranking: the pair meets in the middle
        mid = 0.5 * (ora.cs[0, h, a] + ora.cs[0, h, b])
        scores[0, h, a], scores[0, h, b] = mid - 1e-6, mid + 1e-6
        with pytest.raises(AssertionError, match=caught_by):
            gc.check_decode_against_oracle(pb2, _stand_in(pb2, order, scores), EPS, M)
        refused += 1
    assert refused >= 1, "the construction found no head whose stop moves"


def test_an_element_wise_error_is_caught_where_the_norm_is_not():
    """One output element off by 0.3 % of the row's largest entry: relative L2 stays below 2e-3 on a 128-long row,
    the element-wise bound must fire."""
    pb = _problem()
    ora = po.psa_decode(pb, EPS, M)
    good = _stand_in(pb, ora.order, ora.cs)
    row = good.out[0, 0]
    big = float(row.abs().max())
    l2 = float(row.norm())
    bump = 3e-3 * big
    assert bump / l2 < gc.OUT_RTOL * 0.99, "the case must pass the norm check to mean anything"
    bad = SimpleNamespace(**vars(good))
    bad.out = good.out.clone()
    bad.out[0, 0, int(row.abs().argmin())] += bump
    with pytest.raises(AssertionError, match="element-wise"):
        gc.check_decode_against_oracle(pb, bad, EPS, M)


def test_a_wrong_stop_with_matching_rankings_is_refused():
    pb = _problem()
    ora = po.psa_decode(pb, EPS, M)
    res = _stand_in(pb, ora.order, ora.cs)
    n = res.n_selected.clone()
    n[0, 1] += 1                                # one block too many on one head, everything else consistent with it
    out = po.attend_prefix(pb, ora.order, n.numpy())
    _, lse = po.attend_prefix(pb, ora.order, n.numpy(), want_lse=True)
    bad = SimpleNamespace(**vars(res))
    bad.n_selected, bad.out, bad.lse = n, torch.from_numpy(out.astype(np.float32)), torch.from_numpy(lse.astype(np.float32))
    G = pb.q.shape[1] // pb.k_pool.shape[1]
    bad.blocks_read = n.reshape(1, -1, G).max(-1).values.to(torch.int32)
    with pytest.raises(AssertionError):
        gc.check_decode_against_oracle(pb, bad, EPS, M)
