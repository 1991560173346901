"""Pins of the oracle's ANN selection (AnnSA / AnnCA): brute force, closed forms, invariants.

Sec. 5.1 fixes the goal (the keys with the largest dot products), Sec. 5.3 the existential rule for
prompt tokens (kept when at least one query of the frame is its neighbour), Sec. 5.4 the per-query
restriction computed block-sparse.  Granularity, budget and tie-breaks are this build's reading.
"""
import numpy as np
import pytest

import oracle


def brute_top(score, n_out):
    """Indices of the n_out largest scores, ties to the smaller index, ascending (stable sort on -score)."""
    order = np.argsort(-score.astype(np.int64), kind="stable")
    return np.sort(order[:n_out])


def rand_codes(rng, *shape):
    return rng.integers(-60, 61, size=shape).astype(np.int8)


def test_cross_is_token_level_topk_of_max_over_block_queries():
    rng = np.random.default_rng(0)
    H, n_q, n_p, r, BQ, n_sel = 2, 150, 97, 32, 64, 10
    qc, pc = rand_codes(rng, H, n_q, r), rand_codes(rng, H, n_p, r)
    sel, nsel = oracle.ann_select_cross(qc, pc, BQ, n_sel)
    n_qb = 3
    assert sel.shape == (H, n_qb, n_sel) and np.all(nsel == n_sel)
    for h in range(H):
        S = qc[h].astype(np.int64) @ pc[h].astype(np.int64).T           # [n_q, n_p]
        for b in range(n_qb):
            blk = S[b * BQ:min((b + 1) * BQ, n_q)].max(axis=0)
            assert np.array_equal(sel[h, b], brute_top(blk, n_sel))


def test_self_with_unit_blocks_and_per_query_reps_is_cross():
    rng = np.random.default_rng(1)
    H, n_q, n_p, r, BQ, n_sel = 2, 100, 80, 32, 32, 7
    qc, pc = rand_codes(rng, H, n_q, r), rand_codes(rng, H, n_p, r)
    a = oracle.ann_select_cross(qc, pc, BQ, n_sel)
    b = oracle.ann_select_self(qc, pc, np.full(H, n_p, np.int32), BQ, BQ, 1, n_sel)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_self_against_brute_force_with_block_max_and_mean_reps():
    rng = np.random.default_rng(2)
    H, n_q, C, r, BQ, n_rep, BK, n_sel = 2, 200, 400, 32, 64, 4, 16, 6
    g = BQ // n_rep
    qc, kc = rand_codes(rng, H, n_q, r), rand_codes(rng, H, C, r)
    length = np.array([400, 333], np.int32)
    sel, nsel = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel)
    n_qb = (n_q + BQ - 1) // BQ
    for h in range(H):
        L = int(length[h]); n_kb = (L + BK - 1) // BK
        for b in range(n_qb):
            reps = []
            for u in range(n_rep):
                q0 = b * BQ + u * g
                if q0 >= n_q:
                    continue
                s = qc[h, q0:min(q0 + g, n_q)].astype(np.int64).sum(axis=0)
                reps.append(np.floor_divide(s + g // 2, g))
            S = np.stack(reps) @ kc[h, :L].astype(np.int64).T             # [n_reps, L]
            per_key = S.max(axis=0)
            blk = np.array([per_key[k * BK:min((k + 1) * BK, L)].max() for k in range(n_kb)])
            assert np.array_equal(sel[h, b, :n_sel], brute_top(blk, n_sel))
            assert nsel[h, b] == n_sel


@pytest.mark.parametrize("codes,expect", [((1, 2), 0), ((-1, -2), 1), ((0, -1), 0), ((-1, -1), 1), ((1, 0), 0)])
def test_mean_rep_rounding_closed_form(codes, expect):
    # r = 1, one summary of g = 2 queries: rep = floor((c0 + c1 + 1) / 2); key block 0 holds code +1,
    # block 1 code -1, so the top-1 block is 0 when rep >= 0 (tie -> lower index) and 1 when rep < 0.
    # (1,2)->2, (-1,-2)->-1, (0,-1)->0, (-1,-1)->-1, (1,0)->1
    qc = np.array(codes, np.int8).reshape(1, 2, 1)
    kc = np.array([1, -1], np.int8).reshape(1, 2, 1)
    sel, nsel = oracle.ann_select_self(qc, kc, np.array([2], np.int32), 2, 1, 1, 1)
    assert sel[0, 0, 0] == expect and nsel[0, 0] == 1


def test_budget_at_least_all_blocks_lists_everything_ascending_with_padding():
    rng = np.random.default_rng(3)
    H, n_q, C, r = 2, 64, 256, 32
    qc, kc = rand_codes(rng, H, n_q, r), rand_codes(rng, H, C, r)
    length = np.array([256, 70], np.int32)
    sel, nsel = oracle.ann_select_self(qc, kc, length, 32, 4, 16, 20)
    assert nsel[0].tolist() == [16, 16] and nsel[1].tolist() == [5, 5]
    assert np.array_equal(sel[0, 0, :16], np.arange(16)) and np.all(sel[0, :, 16:] == -1)
    assert np.array_equal(sel[1, 1, :5], np.arange(5)) and np.all(sel[1, :, 5:] == -1)


def test_output_strictly_ascending_and_ties_go_to_lowest_index():
    H, n_q, C, r = 1, 32, 128, 32
    qc = np.ones((H, n_q, r), np.int8)
    kc = np.ones((H, C, r), np.int8)                        # every block scores the same
    sel, nsel = oracle.ann_select_self(qc, kc, np.array([C], np.int32), 32, 4, 16, 3)
    assert sel[0, 0].tolist() == [0, 1, 2]
    kc[0, 5 * 16 + 3] = 2                                    # one key lifts block 5
    sel, _ = oracle.ann_select_self(qc, kc, np.array([C], np.int32), 32, 4, 16, 3)
    assert sel[0, 0].tolist() == [0, 1, 5]


def test_permuting_key_blocks_permutes_the_selection():
    rng = np.random.default_rng(4)
    H, n_q, C, r, BK, n_sel = 1, 64, 320, 32, 16, 5
    qc, kc = rand_codes(rng, H, n_q, r), rand_codes(rng, H, C, r)
    length = np.array([C], np.int32)
    sel, _ = oracle.ann_select_self(qc, kc, length, 32, 4, BK, n_sel)
    perm = rng.permutation(C // BK)
    kc2 = kc.reshape(H, C // BK, BK, r)[:, perm].reshape(H, C, r)       # new block i = old block perm[i]
    sel2, _ = oracle.ann_select_self(qc, kc2, length, 32, 4, BK, n_sel)
    for b in range(sel.shape[1]):
        assert sorted(perm[sel2[0, b]].tolist()) == sel[0, b].tolist()    # scores here are distinct


def test_dead_keys_and_empty_cache():
    rng = np.random.default_rng(5)
    H, n_q, C, r = 2, 40, 64, 32
    qc, kc = rand_codes(rng, H, n_q, r), rand_codes(rng, H, C, r)
    kc[:, 20:] = 127                                         # would win every comparison if visible
    qc[:] = np.abs(qc)
    sel, nsel = oracle.ann_select_self(qc, kc, np.array([20, 0], np.int32), 16, 4, 8, 2)
    assert np.all(sel[0] < 3) and np.all(nsel[0] == 2)
    assert np.all(sel[1] == -1) and np.all(nsel[1] == 0)


def test_selection_finds_the_blocks_that_hold_the_exact_nearest_keys():
    # ANN goal (Sec. 5.1): the keys with the largest dot products.  On clustered data the block that
    # holds a query block's own cluster must be selected.
    from workloads import FrameStream, make_codec, CONFIGS
    c = CONFIGS["cfg1"]
    fs = FrameStream.from_config("cfg1")
    codec = make_codec(0, 1, c["d"], c["r"])
    K, _ = fs.next_frame()
    Q = fs.queries(1)
    qc = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    kc = oracle.encode(K, codec.R, codec.qscale, codec.shift)
    BQ, BK = 32, 32                                          # 2 clusters per block on both sides, aligned
    sel, _ = oracle.ann_select_self(qc, kc, np.full(c["H"], c["T"], np.int32), BQ, 4, BK, 1)
    hit = (sel[:, :, 0] == np.arange(c["T"] // BQ)[None, :]).mean()
    assert hit == 1.0


def test_forced_sink_and_local_blocks_are_always_selected_and_the_rest_is_the_plain_ranking():
    # first n_sink and last n_local live key blocks always present (Sec. 2: the sink frames of rolling-window generators,
    # and a local window); the rest of the budget = the plain top ranking restricted to the other blocks (brute force)
    rng = np.random.default_rng(12)
    H, n_q, C, r, BQ, n_rep, BK, n_sel = 2, 200, 64 * 30, 32, 64, 4, 64, 9
    qc = rng.integers(-40, 41, size=(H, n_q, r)).astype(np.int8)
    kc = rng.integers(-40, 41, size=(H, C, r)).astype(np.int8)
    length = np.array([C, 64 * 17 + 5], np.int32)
    plain, nplain = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel)
    same, nsame = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel, 0, 0)
    assert np.array_equal(plain, same) and np.array_equal(nplain, nsame)
    for n_sink, n_local in ((2, 0), (0, 3), (2, 3), (4, 5)):
        sel, nsel = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel, n_sink, n_local)
        for h in range(H):
            n_kb = (int(length[h]) + BK - 1) // BK
            forced = set(range(n_sink)) | set(range(n_kb - n_local, n_kb))
            big, _ = oracle.ann_select_self(qc[h:h + 1], kc[h:h + 1], length[h:h + 1], BQ, n_rep, BK, n_kb)   # budget = all
            for b in range(sel.shape[1]):
                row = sel[h, b, :nsel[h, b]].tolist()
                assert nsel[h, b] == n_sel and row == sorted(row) and forced <= set(row)
                # ranking of the other blocks: recompute their scores by brute force
                g = BQ // n_rep
                reps = []
                for u in range(n_rep):
                    q0, q1 = b * BQ + u * g, min(b * BQ + (u + 1) * g, n_q)
                    if q0 < n_q:
                        reps.append(np.floor_divide(qc[h, q0:q1].astype(np.int64).sum(axis=0) + g // 2, g))
                reps = np.array(reps)
                L = int(length[h])
                sc = np.array([(kc[h, kb * BK:min((kb + 1) * BK, L)].astype(np.int64) @ reps.T).max() for kb in range(n_kb)])
                others = [kb for kb in range(n_kb) if kb not in forced]
                order = sorted(others, key=lambda kb: (-sc[kb], kb))[: n_sel - len(forced)]
                assert sorted(order + sorted(forced)) == row
    # forced blocks fill the whole budget, or the cache has fewer blocks than the budget
    sel, nsel = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, 5, 2, 3)
    assert sel[1, 0].tolist() == [0, 1, 15, 16, 17]
    short = np.array([64 * 3, 64 * 2], np.int32)
    sel, nsel = oracle.ann_select_self(qc, kc, short, BQ, n_rep, BK, 8, 2, 3)
    assert sel[0, 0].tolist() == [0, 1, 2, -1, -1, -1, -1, -1] and nsel[1, 0] == 2
