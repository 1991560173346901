"""Pins of the oracle's sign-code (LSH) functions, Sec. 5.1 LSH paragraph and its use in Sec. 5.3 / 5.4.

Each pin fixes the oracle to something other than its own formula: a worked example done by hand, invariances of
a hyperplane hash, the 1 - angle/pi collision law of random hyperplanes, brute force in Python integers.
"""
import numpy as np
import pytest

import oracle


def bits_of(words, n_bits):
    """Unpack [.., W] uint32 words into a [.., n_bits] 0/1 array with Python-level shifts."""
    words = np.asarray(words)
    out = np.zeros(words.shape[:-1] + (n_bits,), np.int64)
    for j in range(n_bits):
        out[..., j] = (words[..., j // 32].astype(np.int64) >> (j % 32)) & 1
    return out


def test_sign_code_worked_example():
    # d = 4, qscale = 1: x = (1, -2, 0.5, 0) quantises to (1, -2, 0, 0)  (0.5 rounds half to even = 0)
    x = np.array([[1.0, -2.0, 0.5, 0.0]], np.float32)
    R = np.ones((4, 32), np.int8)
    R[1, 1] = -1                 # column 1: 1 + 2 + 0 + 0 = 3   -> bit 1
    R[:, 2] = -1                 # column 2: -(1 - 2) = 1        -> bit 1
    R[0, 3] = -1                 # column 3: -1 - 2 = -3         -> bit 0
    R[1, 4] = -1; R[0, 4] = -1   # column 4: -1 + 2 = 1          -> bit 1
    R[:, 5] = [1, 1, -1, -1]     # column 5: 1 - 2 = -1          -> bit 0
    # every other column is all ones: 1 - 2 + 0 + 0 = -1 -> bit 0
    w = oracle.encode_sign(x, R, 1.0)
    assert w.shape == (1, 1) and w.dtype == np.uint32
    assert int(w[0, 0]) == (1 << 1) | (1 << 2) | (1 << 4)


def test_zero_projection_counts_as_positive_and_bits_are_packed_low_first():
    x = np.zeros((1, 8), np.float32)
    R = np.where(np.arange(8 * 64).reshape(8, 64) % 3 == 0, 1, -1).astype(np.int8)
    w = oracle.encode_sign(x, R, 10.0)
    assert w.tolist() == [[0xFFFFFFFF, 0xFFFFFFFF]]            # every projection is 0: ties are ones
    # a vector that only column 37 sees on the negative side: x = e_0, R[0] = +1 except column 37
    x = np.zeros((1, 8), np.float32); x[0, 0] = 1.0
    R = np.ones((8, 64), np.int8); R[0, 37] = -1
    w = oracle.encode_sign(x, R, 1.0)
    assert w.tolist() == [[0xFFFFFFFF, 0xFFFFFFFF ^ (1 << (37 - 32))]]


def test_sign_code_invariances():
    rng = np.random.default_rng(5)
    d, n_bits = 64, 128
    R = rng.choice(np.array([-1, 1], np.int8), size=(d, n_bits))
    x = rng.standard_normal((50, d)).astype(np.float32)
    q = 127 / 8.0
    base = oracle.encode_sign(x, R, q)
    # a positive power-of-two factor that keeps every coordinate inside the 8-bit range scales the quantised
    # vector exactly by an integer... only when no rounding happens: use an already-integer grid
    xi = np.round(x * 8).astype(np.float32)                                  # integers in about [-30, 30]
    a = oracle.encode_sign(xi, R, 1.0)
    b = oracle.encode_sign(xi * 2, R, 1.0)                                   # still within +-127
    assert np.array_equal(a, b)
    # negation flips every bit whose projection is not zero
    neg = oracle.encode_sign(-xi, R, 1.0)
    proj = np.round(xi).astype(np.int64) @ R.astype(np.int64)
    flipped = bits_of(a, n_bits) != bits_of(neg, n_bits)
    assert np.array_equal(flipped, proj != 0)
    # bf16 storage of values that are exact in bf16 gives the same code as fp32 storage
    from workloads import to_storage
    xe = (rng.integers(-16, 17, size=(20, d)) / 4.0).astype(np.float32)
    assert np.array_equal(oracle.encode_sign(to_storage(xe, "bf16"), R, q), oracle.encode_sign(xe, R, q))
    assert base.shape == (50, n_bits // 32)


def test_collision_rate_follows_the_angle():
    """Random hyperplanes: P[bits equal] = 1 - angle/pi.  With +-1 projection entries and d = 128 the projections
    are close to Gaussian, so the law holds to within sampling noise of 4096 bits plus a small bias."""
    rng = np.random.default_rng(11)
    d, n_bits = 128, 4096
    R = rng.choice(np.array([-1, 1], np.int8), size=(d, n_bits))
    u = rng.standard_normal(d); u /= np.linalg.norm(u)
    v = rng.standard_normal(d); v -= v.dot(u) * u; v /= np.linalg.norm(v)
    for theta in (0.0, 0.3, 0.8, np.pi / 2, 2.2, np.pi):
        a = (40 * u).astype(np.float32)
        b = (40 * (np.cos(theta) * u + np.sin(theta) * v)).astype(np.float32)
        bits = bits_of(oracle.encode_sign(np.stack([a, b]), R, 127 / 16.0), n_bits)
        frac = float((bits[0] == bits[1]).mean())
        assert abs(frac - (1 - theta / np.pi)) < 0.035, (theta, frac)


def brute_select(qbits, kbits, length, n_bits, BQ, n_rep, BK, n_sel):
    """Independent Python-integer implementation: majority summaries, popcount of XNOR, repeated arg-max."""
    H, n_q, W = qbits.shape
    C = kbits.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    g = BQ // n_rep
    mask = (1 << n_bits) - 1
    as_int = lambda row: sum(int(row[w]) << (32 * w) for w in range(W))
    sel = np.full((H, n_qb, n_sel), -1, np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        L = min(int(length[h]), C)
        n_kb = (L + BK - 1) // BK
        keys = [as_int(kbits[h, k]) for k in range(L)]
        for b in range(n_qb):
            reps = []
            for u in range(n_rep):
                qs = [as_int(qbits[h, q]) for q in range(b * BQ + u * g, min(b * BQ + (u + 1) * g, n_q))]
                if not qs:
                    continue
                r = 0
                for j in range(n_bits):
                    ones = sum((q >> j) & 1 for q in qs)
                    if 2 * ones >= len(qs):
                        r |= 1 << j
                reps.append(r)
            score = []
            for kb in range(n_kb):
                score.append(max(bin(~(r ^ keys[k]) & mask).count("1")
                                 for k in range(kb * BK, min((kb + 1) * BK, L)) for r in reps))
            order = sorted(range(n_kb), key=lambda kb: (-score[kb], kb))[:min(n_sel, n_kb)]
            order.sort()
            sel[h, b, :len(order)] = order
            nsel[h, b] = len(order)
    return sel, nsel


@pytest.mark.parametrize("n_q,C,lens,n_bits,BQ,n_rep,BK,n_sel", [
    (20, 37, [37, 20], 64, 8, 2, 4, 3),
    (9, 16, [16, 0], 32, 4, 4, 1, 5),          # cross-attention form: every query its own summary, single keys
    (16, 24, [24, 23], 96, 16, 1, 8, 7),        # budget above the number of key blocks
])
def test_selection_matches_brute_force(n_q, C, lens, n_bits, BQ, n_rep, BK, n_sel):
    rng = np.random.default_rng(n_q + C)
    H, W = 2, n_bits // 32
    qbits = rng.integers(0, 2 ** 32, size=(H, n_q, W), dtype=np.uint64).astype(np.uint32)
    kbits = rng.integers(0, 2 ** 32, size=(H, C, W), dtype=np.uint64).astype(np.uint32)
    kbits[:, ::3] = kbits[:, 1:2]                                    # plenty of ties
    length = np.array(lens, np.int32)
    sel, nsel = oracle.ann_select_lsh(qbits, kbits, length, BQ, n_rep, BK, n_sel)
    sel_b, nsel_b = brute_select(qbits, kbits, length, n_bits, BQ, n_rep, BK, n_sel)
    assert np.array_equal(nsel, nsel_b) and np.array_equal(sel, sel_b)


def test_majority_summary_by_hand_and_the_block_that_holds_it_wins():
    # three queries in one run: bits (low four) 0b0011, 0b0101, 0b1001 -> majority 0b0001; n_bits = 32, the
    # other 28 bits all zero in queries and keys
    q = np.array([[[0b0011], [0b0101], [0b1001]]], np.uint32)
    keys = np.zeros((1, 8, 1), np.uint32)
    keys[0, :, 0] = [0b1110, 0b0110, 0b1000, 0b0011, 0b0101, 0b0001, 0b1111, 0b0111]
    #  equal bits with 0b0001 (of 32):  28+0, 28+1, 28+2, 28+3, 28+3, 32, 28+1, 28+2
    sel, nsel = oracle.ann_select_lsh(q, keys, np.array([8], np.int32), 3, 1, 1, 3)
    assert nsel.tolist() == [[3]] and sel.tolist() == [[[3, 4, 5]]]     # 32, then the two 31s (lowest indices)
    # with a tie at the budget's edge the lower index wins: budget 2 -> key 5 (32) and key 3 (31, before key 4)
    sel, nsel = oracle.ann_select_lsh(q, keys, np.array([8], np.int32), 3, 1, 1, 2)
    assert sel.tolist() == [[[3, 5]]]
    # dead slots are invisible: with len = 5 key 5 is gone
    sel, nsel = oracle.ann_select_lsh(q, keys, np.array([5], np.int32), 3, 1, 1, 2)
    assert sel.tolist() == [[[3, 4]]]


def test_neighbours_in_angle_are_what_the_hash_selects():
    """End to end on real vectors: keys close in angle to the queries of a block share most hash bits and their
    key block is selected first."""
    rng = np.random.default_rng(3)
    d, n_bits, BK = 64, 256, 8
    R = rng.choice(np.array([-1, 1], np.int8), size=(d, n_bits))
    centre = rng.standard_normal(d).astype(np.float32)
    Q = (centre + 0.1 * rng.standard_normal((1, 16, d))).astype(np.float32)
    K = rng.standard_normal((1, 64, d)).astype(np.float32)
    K[0, 40:48] = centre + 0.1 * rng.standard_normal((8, d))           # key block 5 holds the neighbours
    qs = oracle.encode_sign(Q, R, 127 / 4.5)
    ks = oracle.encode_sign(K, R, 127 / 4.5)
    sel, nsel = oracle.ann_select_lsh(qs, ks, np.array([64], np.int32), 16, 4, BK, 1)
    assert sel.tolist() == [[[5]]]


# ------------------------------------------------------------------ hash tables: same bucket(s), multi-probe
# (Sec. 5.1, LSH paragraph: a query only compares against keys that land in the same bucket(s); Sec. 2: multi-table
# bucket probing)

def brute_select_buckets(qbits, kbits, length, n_bits, band, radius, BQ, n_rep, BK, n_sel, n_sink=0, n_local=0):
    """Python integers and sets: bucket ids per table, probe sets by explicit bit flips."""
    from itertools import combinations
    H, n_q, W = qbits.shape
    C = kbits.shape[1]
    n_qb = (n_q + BQ - 1) // BQ
    g = BQ // n_rep
    T = n_bits // band
    as_int = lambda words: sum(int(w) << (32 * i) for i, w in enumerate(words))
    bucket = lambda code, t: (code >> (t * band)) & ((1 << band) - 1)

    def probes(bk):   # the bucket itself and every bucket at most `radius` bit flips away
        out = {bk}
        for k in range(1, radius + 1):
            for pos in combinations(range(band), k):
                x = bk
                for p in pos:
                    x ^= 1 << p
                out.add(x)
        return out

    sel = -np.ones((H, n_qb, n_sel), np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        L = min(int(length[h]), C)
        n_kb = (L + BK - 1) // BK
        keys = [as_int(kbits[h, k]) for k in range(L)]
        for b in range(n_qb):
            reps = []
            for u in range(n_rep):
                qs = [as_int(qbits[h, q]) for q in range(b * BQ + u * g, min(b * BQ + (u + 1) * g, n_q))]
                if qs:
                    reps.append(sum(1 << j for j in range(n_bits) if 2 * sum((q >> j) & 1 for q in qs) >= len(qs)))
            probe_sets = [[probes(bucket(r, t)) for t in range(T)] for r in reps]
            cand = []
            for kb in range(n_kb):
                best = max(sum(bucket(keys[k], t) in ps[t] for t in range(T))
                           for k in range(kb * BK, min((kb + 1) * BK, L)) for ps in probe_sets)
                forced = kb < n_sink or kb >= n_kb - n_local
                if forced or best >= 1:
                    cand.append((0 if forced else 1, -best, kb))
            chosen = sorted(kb for _, _, kb in sorted(cand)[:n_sel])
            sel[h, b, :len(chosen)] = chosen
            nsel[h, b] = len(chosen)
    return sel, nsel


@pytest.mark.parametrize("n_q,C,lens,n_bits,band,radius,BQ,n_rep,BK,n_sel,sink,local", [
    (20, 37, [37, 20], 64, 8, 0, 8, 2, 4, 3, 0, 0),
    (20, 37, [37, 20], 64, 8, 1, 8, 2, 4, 3, 0, 0),
    (9, 16, [16, 0], 32, 4, 0, 4, 4, 1, 20, 0, 0),      # single keys and queries, budget beyond the candidates
    (16, 48, [48, 41], 128, 16, 2, 16, 1, 8, 4, 1, 1),  # wide bands, two flips, forced blocks
    (12, 40, [40, 40], 64, 32, 3, 4, 2, 2, 6, 0, 0),
    (10, 30, [30, 7], 64, 2, 0, 5, 5, 3, 4, 0, 0)])
def test_bucket_selection_matches_brute_force_on_probe_sets(n_q, C, lens, n_bits, band, radius, BQ, n_rep, BK, n_sel, sink, local):
    rng = np.random.default_rng(n_q + C + band + radius)
    H, W = 2, n_bits // 32
    qbits = rng.integers(0, 2 ** 32, size=(H, n_q, W), dtype=np.uint64).astype(np.uint32)
    kbits = rng.integers(0, 2 ** 32, size=(H, C, W), dtype=np.uint64).astype(np.uint32)
    kbits[:, ::3] = kbits[:, 1:2]
    kbits[:, 5::7] = qbits[:, :1] ^ np.uint32(1 << 3)                  # near copies of a query: collide in most tables
    length = np.array(lens, np.int32)
    got = oracle.ann_select_lsh_buckets(qbits, kbits, length, band, radius, BQ, n_rep, BK, n_sel, sink, local)
    ref = brute_select_buckets(qbits, kbits, length, n_bits, band, radius, BQ, n_rep, BK, n_sel, sink, local)
    assert np.array_equal(got[1], ref[1]) and np.array_equal(got[0], ref[0])


def test_one_table_of_all_bits_is_bucket_equality_and_one_bit_tables_count_equal_bits():
    rng = np.random.default_rng(11)
    qbits = rng.integers(0, 4, size=(1, 6, 1), dtype=np.uint64).astype(np.uint32)       # 2 significant bits: many equal codes
    kbits = rng.integers(0, 4, size=(1, 40, 1), dtype=np.uint64).astype(np.uint32)
    length = np.array([40], np.int32)
    # one table over the whole code, single queries and keys, budget beyond the cache: exactly the keys with the query's code
    sel, nsel = oracle.ann_select_lsh_buckets(qbits, kbits, length, 32, 0, 1, 1, 1, 40)
    for i in range(6):
        same = np.flatnonzero(kbits[0, :, 0] == qbits[0, i, 0])
        assert nsel[0, i] == len(same) and np.array_equal(sel[0, i, :len(same)], same)
    # one-bit tables: a pair's collisions are its equal bits, so the ranking is that of ann_select_lsh whenever every
    # block has a collision (always, with 32 one-bit tables of codes that agree in their 30 high bits)
    a = oracle.ann_select_lsh_buckets(qbits, kbits, length, 1, 0, 2, 1, 4, 3)
    b = oracle.ann_select_lsh(qbits, kbits, length, 2, 1, 4, 3)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_probing_more_buckets_only_adds_candidates_and_full_radius_admits_everything():
    rng = np.random.default_rng(12)
    qbits = rng.integers(0, 2 ** 32, size=(1, 8, 2), dtype=np.uint64).astype(np.uint32)
    kbits = rng.integers(0, 2 ** 32, size=(1, 64, 2), dtype=np.uint64).astype(np.uint32)
    length = np.array([64], np.int32)
    prev = None
    for radius in range(0, 9):
        sel, nsel = oracle.ann_select_lsh_buckets(qbits, kbits, length, 8, radius, 8, 2, 4, 16)
        cur = set(sel[0, 0, :nsel[0, 0]].tolist())
        if prev is not None:
            assert prev <= cur
        prev = cur
    assert cur == set(range(16))          # radius = band width: every bucket is probed
