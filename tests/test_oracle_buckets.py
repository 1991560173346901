"""Pins of the prompt-induced bucket selection (Sec. 5.4, first paragraph: self-attention restricted to the semantic
buckets that cross-attention pruning found; a query belongs to one or more buckets and attends only to keys of the same
bucket(s)).  The oracle is checked against a hand example, brute force written with Python sets, the literal
"same bucket" rule at token granularity, and invariances that a wrong index, a dropped bucket or a wrong tie rule break."""
import numpy as np
import pytest

import oracle


def rand_codes(rng, lo, hi, *shape):
    return rng.integers(lo, hi + 1, size=shape).astype(np.int8)


# ------------------------------------------------------------------------------------------ bucket assignment

def test_bucket_of_a_code_is_its_nearest_prompt_token_hand_example():
    # prompt codes along three axes; every code falls to the axis it points along, then to the second strongest
    pcode = np.zeros((1, 3, 4), np.int8)
    pcode[0, 0, 0] = 10
    pcode[0, 1, 1] = 10
    pcode[0, 2, 2] = 10
    code = np.array([[[9, 1, 0, 5], [1, 2, 8, 0], [0, 7, 6, 0], [-3, -2, -1, 9], [4, 4, 0, 0]]], np.int8)
    b = oracle.prompt_buckets(code, pcode, m=2)
    assert b[0].tolist() == [[0, 1], [2, 1], [1, 2], [2, 1], [0, 1]]   # row 3: products -30, -20, -10; row 4: tie 40 = 40 -> smaller id first
    assert oracle.prompt_buckets(code, pcode, m=1)[0, :, 0].tolist() == [0, 2, 1, 2, 0]
    # more buckets asked for than prompt tokens: the tail is -1
    assert oracle.prompt_buckets(code, pcode, m=4)[0, 0].tolist() == [0, 1, 2, -1]


@pytest.mark.parametrize("seed,span", [(0, 40), (1, 2)])
def test_bucket_assignment_equals_a_stable_sort_of_the_products(seed, span):
    rng = np.random.default_rng(seed)
    H, n, n_p, r, m = 2, 50, 37, 32, 3
    code, pcode = rand_codes(rng, -span, span, H, n, r), rand_codes(rng, -span, span, H, n_p, r)   # span 2: many ties
    b = oracle.prompt_buckets(code, pcode, m=m)
    prod = np.einsum("hnr,hpr->hnp", code.astype(np.int64), pcode.astype(np.int64))
    ref = np.argsort(-prod, axis=2, kind="stable")[:, :, :m]
    assert np.array_equal(b, ref)


# ------------------------------------------------------------------------------------------ selection on buckets

def brute_select(qb, kb_, length, n_p, BQ, BK, n_sel, n_sink=0, n_local=0):
    H, n_q, m = qb.shape
    n_qb = -(-n_q // BQ)
    sel = -np.ones((H, n_qb, n_sel), np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        L = int(length[h])
        n_kb = -(-L // BK)
        for b in range(n_qb):
            own = {int(t) for t in qb[h, b * BQ:(b + 1) * BQ].ravel() if 0 <= t < n_p}
            cand = []
            for k in range(n_kb):
                has = {int(t) for t in kb_[h, k * BK:min((k + 1) * BK, L)].ravel() if 0 <= t < n_p}
                forced = k < n_sink or k >= n_kb - n_local
                shared = len(own & has)
                if forced or shared > 0:
                    cand.append((0 if forced else 1, -shared, k))
            chosen = sorted(k for _, _, k in sorted(cand)[:n_sel])
            sel[h, b, :len(chosen)] = chosen
            nsel[h, b] = len(chosen)
    return sel, nsel


@pytest.mark.parametrize("seed,m,n_p,BQ,BK,n_sel,sink,local", [
    (0, 1, 12, 8, 4, 3, 0, 0), (1, 2, 40, 16, 8, 5, 0, 0), (2, 3, 9, 4, 4, 50, 0, 0), (3, 1, 64, 8, 8, 4, 1, 2),
    (4, 2, 500, 32, 16, 6, 2, 0)])
def test_selection_equals_brute_force_on_sets(seed, m, n_p, BQ, BK, n_sel, sink, local):
    rng = np.random.default_rng(seed)
    H, n_q, C = 3, 70, 200
    qb = rng.integers(-1, n_p, size=(H, n_q, m)).astype(np.int32)        # -1 entries are ignored
    kb_ = rng.integers(-1, n_p, size=(H, C, m)).astype(np.int32)
    length = np.array([200, 131, 0], np.int32)
    ref = brute_select(qb, kb_, length, n_p, BQ, BK, n_sel, sink, local)
    got = oracle.ann_select_buckets(qb, kb_, length, n_p, BQ, BK, n_sel, sink, local)
    assert np.array_equal(got[1], ref[1])
    assert np.array_equal(got[0], ref[0])


def test_token_granularity_is_the_literal_same_bucket_rule():
    # one query per block, one key per block, one bucket each, budget beyond the cache: query i keeps key j iff equal bucket
    rng = np.random.default_rng(5)
    n_q, C, n_p = 20, 60, 7
    qb = rng.integers(0, n_p, size=(1, n_q, 1)).astype(np.int32)
    kb_ = rng.integers(0, n_p, size=(1, C, 1)).astype(np.int32)
    sel, nsel = oracle.ann_select_buckets(qb, kb_, np.array([C], np.int32), n_p, 1, 1, C)
    for i in range(n_q):
        same = np.flatnonzero(kb_[0, :, 0] == qb[0, i, 0])
        assert nsel[0, i] == len(same)
        assert np.array_equal(sel[0, i, :len(same)], same)
        assert (sel[0, i, len(same):] == -1).all()


def test_blocks_without_a_shared_bucket_are_never_selected_and_ranking_counts_shared_buckets():
    # query block owns {0, 1, 2}; key blocks own {0,1,2}, {5}, {1,2}, {2,9}, {7,8}
    qb = np.array([[[0], [1], [2], [2]]], np.int32)
    kb_ = np.array([[[0], [1], [2], [5], [5], [5], [1], [2], [2], [2], [9], [9], [7], [8], [8]]], np.int32)
    length = np.array([15], np.int32)
    sel, nsel = oracle.ann_select_buckets(qb, kb_, length, 10, 4, 3, 4)
    assert nsel[0, 0] == 3 and sel[0, 0].tolist() == [0, 2, 3, -1]        # blocks 1 and 4 share nothing
    sel, nsel = oracle.ann_select_buckets(qb, kb_, length, 10, 4, 3, 2)
    assert sel[0, 0].tolist() == [0, 2]                                      # 3 and 2 shared buckets beat 1
    sel, nsel = oracle.ann_select_buckets(qb, kb_, length, 10, 4, 3, 1)
    assert sel[0, 0].tolist() == [0]
    # forced blocks are kept although they share nothing, and take their part of the budget
    sel, nsel = oracle.ann_select_buckets(qb, kb_, length, 10, 4, 3, 3, 0, 1)
    assert sel[0, 0].tolist() == [0, 2, 4]
    # dead keys own nothing: with 7 live slots block 2 has only key 6 (bucket 1)
    sel, nsel = oracle.ann_select_buckets(qb, kb_, np.array([7], np.int32), 10, 4, 3, 4)
    assert sel[0, 0].tolist() == [0, 2, -1, -1]


def test_relabelling_the_buckets_changes_nothing_and_more_buckets_per_token_only_add_candidates():
    rng = np.random.default_rng(6)
    H, n_q, C, n_p = 2, 64, 256, 30
    qb = rng.integers(0, n_p, size=(H, n_q, 2)).astype(np.int32)
    kb_ = rng.integers(0, n_p, size=(H, C, 2)).astype(np.int32)
    length = np.array([256, 100], np.int32)
    base = oracle.ann_select_buckets(qb, kb_, length, n_p, 16, 8, 6)
    perm = rng.permutation(n_p).astype(np.int32)
    again = oracle.ann_select_buckets(perm[qb], perm[kb_], length, n_p, 16, 8, 6)
    assert np.array_equal(base[0], again[0]) and np.array_equal(base[1], again[1])
    # candidates with the first bucket only are a subset of those with both (budget beyond the block count)
    one = oracle.ann_select_buckets(qb[:, :, :1], kb_[:, :, :1], length, n_p, 16, 8, 40)
    two = oracle.ann_select_buckets(qb, kb_, length, n_p, 16, 8, 40)
    for h in range(H):
        for b in range(4):
            assert set(one[0][h, b, :one[1][h, b]]) <= set(two[0][h, b, :two[1][h, b]])


def test_end_to_end_on_clustered_codes_queries_find_the_keys_of_their_own_prompt_cluster():
    # codes of three well separated groups, one prompt token per group: a query block made of group g keeps exactly
    # the key blocks that contain a key of group g
    rng = np.random.default_rng(7)
    r = 32
    centres = rng.integers(-60, 61, size=(3, r))
    pcode = centres[None].astype(np.int8)
    grp_k = rng.integers(0, 3, size=96)
    kcode = np.clip(centres[grp_k] + rng.integers(-3, 4, size=(96, r)), -127, 127).astype(np.int8)[None]
    grp_q = np.repeat(np.arange(3), 8)
    qcode = np.clip(centres[grp_q] + rng.integers(-3, 4, size=(24, r)), -127, 127).astype(np.int8)[None]
    qb, kb_ = oracle.prompt_buckets(qcode, pcode), oracle.prompt_buckets(kcode, pcode)
    assert np.array_equal(qb[0, :, 0], grp_q) and np.array_equal(kb_[0, :, 0], grp_k)
    sel, nsel = oracle.ann_select_buckets(qb, kb_, np.array([96], np.int32), 3, 8, 4, 24)
    for g in range(3):
        want = [k for k in range(24) if (grp_k[4 * k:4 * k + 4] == g).any()]
        assert sel[0, g, :nsel[0, g]].tolist() == want
