"""Pins of the oracle's TempCache merge (Sec. 5.2, Lemma 1, representative-key ablation).

What the paper fixes: the match is the top-1 neighbour of a current-frame token among previous keys;
keys merge when their similarity passes a threshold; the most recent key represents the group; the
group's value is the mean and its multiplicity enters attention as + log m; no redundancy => nothing
changes.  The eviction policy of a full cache is not in the paper: invariants only (parity unpinned).
"""
import numpy as np
import pytest

import oracle
from workloads import CONFIGS, FrameStream, make_codec, to_f32, f32_to_bf16_bits

from test_oracle_attention import dense_attention

TAU2 = lambda tau: int(round(tau * tau * 65536))
NEVER = 2 * 65536          # tau^2 = 2: no pair can pass
ALWAYS = 0                 # any positive dot product passes


def stream_cfg1(**over):
    c = dict(CONFIGS["cfg1"]); c.update(over)
    return c, FrameStream.from_config("cfg1", **over), make_codec(0, 1, c["d"], c["r"])


def compress(cache, codec, K, V, **kw):
    return oracle.tempcache_compress(cache, codec.R, codec.qscale, codec.shift, K, V, **kw)


def test_identity_merge_when_nothing_passes_the_threshold():
    c, fs, codec = stream_cfg1()
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 4 * T, d, c["r"], "fp32")
    frames = [fs.next_frame() for _ in range(3)]
    for f, (K, V) in enumerate(frames):
        mm, mg, st = compress(cache, codec, K, V, tau2_q16=NEVER, frame_id=f)
        assert not mg.any()
        assert np.array_equal(mm, np.broadcast_to(f * T + np.arange(T, dtype=np.int32), (H, T)))
        assert st[:, :5].tolist() == [[(f + 1) * T, 0, T, 0, 0]] * H
    Kcat = np.concatenate([k for k, _ in frames], axis=1)
    Vcat = np.concatenate([v for _, v in frames], axis=1)
    assert np.array_equal(cache.K[:, :3 * T], Kcat) and np.array_equal(cache.V[:, :3 * T], Vcat)
    assert np.all(cache.cnt[:, :3 * T] == 1) and np.all(cache.len == 3 * T)
    assert np.array_equal(cache.code[:, :3 * T], oracle.encode(Kcat, codec.R, codec.qscale, codec.shift))
    assert np.array_equal(cache.stamp[:, :3 * T], np.broadcast_to(np.repeat(np.arange(3), T), (H, 3 * T)))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_exact_duplicates_merge_into_their_predecessor_and_attention_is_exact(dtype):
    # drift 0 on every token: each new key equals its predecessor bit for bit (Lemma 1 end to end)
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.0, dtype=dtype)
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 2 * T, d, c["r"], dtype)
    K0, V0 = fs.next_frame()
    rng = np.random.default_rng(0)
    frames = [(K0, V0)]
    for f in range(1, 4):                                   # same keys, fresh values
        Vf = to_f32(V0) + rng.standard_normal(V0.shape).astype(np.float32)
        frames.append((K0, Vf.astype(np.float32) if dtype == "fp32" else f32_to_bf16_bits(Vf)))
    prev = None
    for f, (K, V) in enumerate(frames):
        mm, mg, st = compress(cache, codec, K, V, cand=prev, tau2_q16=TAU2(0.9), frame_id=f)
        prev = mm
        if f:
            assert mg.all() and np.array_equal(mm, np.broadcast_to(np.arange(T, dtype=np.int32), (H, T)))
    assert np.all(cache.len == T) and np.all(cache.cnt[:, :T] == 4) and np.all(cache.stamp[:, :T] == 3)
    assert np.array_equal(cache.K[:, :T], K0)
    Q = fs.queries(1)
    sel, nsel = oracle.full_selection(H, T, 128, cache.len, 64)
    O, _ = oracle.sparse_attn_fwd(Q, cache.K, cache.V, cache.cnt, cache.len, sel, nsel, 128, 64, d ** -0.5)
    Kcat = np.concatenate([to_f32(k) for k, _ in frames], axis=1)
    Vcat = np.concatenate([to_f32(v) for _, v in frames], axis=1)
    tol = 1e-5 if dtype == "fp32" else 2e-2                 # bf16: the stored running mean is rounded 3 times
    for h in range(H):
        Od, _ = dense_attention(to_f32(Q)[h], Kcat[h], Vcat[h], d ** -0.5)
        assert np.abs(O[h] - Od).max() < tol


def test_match_is_the_brute_force_top1_in_code_space():
    # tau2 = 0 merges every token whose best candidate has a positive dot product: merge_map shows j*
    c, fs, codec = stream_cfg1()
    H, T, d = c["H"], c["T"], c["d"]
    for metric in (0, 1):
        cache = oracle.Cache.empty(H, 3 * T, d, c["r"], "fp32")
        K0, V0 = fs.next_frame()
        compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=0)
        K1, V1 = fs.next_frame()
        old_code = cache.code.copy()
        mm, mg, _ = compress(cache, codec, K1, V1, tau2_q16=ALWAYS, metric=metric, frame_id=1)
        cp = oracle.encode(K1, codec.R, codec.qscale, codec.shift).astype(np.int64)
        for h in range(H):
            cj = old_code[h, :T].astype(np.int64)
            S = cp[h] @ cj.T
            if metric == 0:
                S = 2 * S - (cj * cj).sum(axis=1)[None, :]
            jstar = S.argmax(axis=1)                        # first maximum = smallest slot
            assert mg[h].mean() > 0.95
            assert np.array_equal(mm[h][mg[h] == 1], jstar[mg[h] == 1])


def test_code_space_top1_recovers_the_exact_nearest_neighbour_of_drifted_tokens():
    c, fs, codec = stream_cfg1()
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 2 * T, d, c["r"], "fp32")
    K0, V0 = fs.next_frame()
    compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=0)
    K1, V1 = fs.next_frame()
    mm, mg, _ = compress(cache, codec, K1, V1, tau2_q16=TAU2(0.98), frame_id=1)
    hits, total = 0, 0
    for h in range(H):
        D = ((K1[h][:, None, :].astype(np.float64) - K0[h][None, :, :]) ** 2).sum(axis=2)
        nn = D.argmin(axis=1)
        drifted = D.min(axis=1) < 64 * 0.02 ** 2 * 4        # a drifted copy sits within ~2 sigma_d sqrt(d)
        assert 0.6 < drifted.mean() < 0.8                   # the generator drifts p = 0.7 of the tokens
        hits += (mm[h][drifted] == nn[drifted]).sum(); total += drifted.sum()
        assert mg[h][drifted].all() and not mg[h][~drifted].any()
    assert hits == total


def test_threshold_is_the_cosine_of_the_quantised_keys_and_merging_is_monotone():
    c, fs, codec = stream_cfg1(sigma_d=0.25)                # spread similarities around the thresholds
    H, T, d = c["H"], c["T"], c["d"]
    K0, V0 = fs.next_frame()
    K1, V1 = fs.next_frame()
    q = lambda x: np.clip(np.rint(x * codec.qscale), -127, 127).astype(np.float64)
    n_prev = None
    for tau in (0.5, 0.8, 0.9, 0.95, 0.99):
        cache = oracle.Cache.empty(H, 2 * T, d, c["r"], "fp32")
        compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=0)
        mm_all, _, _ = compress(cache.copy(), codec, K1, V1, tau2_q16=ALWAYS, frame_id=1)   # shows j*
        mm, mg, st = compress(cache, codec, K1, V1, tau2_q16=TAU2(tau), frame_id=1)
        n = int(mg.sum())
        assert n_prev is None or n <= n_prev                 # lower threshold => at least as much merging
        n_prev = n
        a = q(K1)
        for h in range(H):
            b = q(K0[h][np.maximum(mm_all[h], 0) % T])
            cos = (a[h] * b).sum(1) / np.sqrt((a[h] ** 2).sum(1) * (b ** 2).sum(1))
            clear = np.abs(cos - tau) > 1e-3
            has_match = mm_all[h] < T                        # tokens whose match had dot > 0
            assert np.array_equal(mg[h][clear & has_match] == 1, (cos > tau)[clear & has_match])
    assert n_prev < T * H                                    # the strictest threshold rejects something


def test_several_tokens_joining_one_slot_mean_value_count_and_last_key_representative():
    d, r = 8, 4
    R = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]] * 2, np.int8)
    qscale, shift = 16.0, 1
    cache = oracle.Cache.empty(1, 8, d, r, "fp32")
    base = np.array([1.0, 2.0, -1.0, 0.5, 3.0, -2.0, 1.5, 0.25], np.float32)
    far = -base[::-1].copy()
    K0 = np.stack([base, far])[None]
    V0 = np.stack([np.full(d, 1.0), np.full(d, 10.0)])[None].astype(np.float32)
    oracle.tempcache_compress(cache, R, qscale, shift, K0, V0, tau2_q16=NEVER, frame_id=0)
    # three new tokens: two near 'base' (the second one exactly equal => best score), one unrelated
    near = base + np.array([0.125, 0, 0, 0, 0, 0, 0, 0], np.float32)
    other = np.array([-3.0, 0.1, 2.5, -1.0, 0.2, 0.3, -2.2, 1.7], np.float32)
    K1 = np.stack([near, base, other])[None]
    V1 = np.stack([np.full(d, 2.0), np.full(d, 6.0), np.full(d, -4.0)])[None].astype(np.float32)
    mm, mg, st = oracle.tempcache_compress(cache, R, qscale, shift, K1, V1, tau2_q16=TAU2(0.9), frame_id=1)
    assert mg[0].tolist() == [1, 1, 0] and mm[0].tolist() == [0, 0, 2]
    assert st[0, :5].tolist() == [3, 2, 1, 0, 0]
    assert cache.cnt[0, :3].tolist() == [3, 1, 1] and cache.stamp[0, :3].tolist() == [1, 0, 1]
    assert np.array_equal(cache.K[0, 0], base)               # exact copy scores highest: it is the representative
    assert np.allclose(cache.V[0, 0], (1.0 + 2.0 + 6.0) / 3)
    assert np.array_equal(cache.K[0, 2], other) and np.array_equal(cache.V[0, 2], V1[0, 2])
    assert np.array_equal(cache.code[0, 0], oracle.encode(base[None], R, qscale, shift)[0])
    # ties between joiners go to the smaller token index: two exact copies with different values
    cache2 = oracle.Cache.empty(1, 8, d, r, "fp32")
    oracle.tempcache_compress(cache2, R, qscale, shift, K0, V0, tau2_q16=NEVER, frame_id=0)
    K2 = np.stack([far, base, base])[None]
    mm, mg, _ = oracle.tempcache_compress(cache2, R, qscale, shift, K2, V1, tau2_q16=TAU2(0.9), frame_id=1)
    assert mm[0].tolist() == [1, 0, 0] and cache2.cnt[0, :2].tolist() == [3, 2]


def test_mean_key_representative_worked_example_and_multiplicity_weights():
    # appendix, representative-selection ablation: mean-key averages the keys of the group.  Hand-computed values
    # (all exactly representable, so float32 arithmetic is exact): slot 0 holds `base` with multiplicity 1.
    d, r = 8, 4
    R = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]] * 2, np.int8)
    qscale, shift = 16.0, 1
    base = np.array([1.0, 2.0, -1.0, 0.5, 3.0, -2.0, 1.5, 0.25], np.float32)
    far = -base[::-1].copy()
    K0 = np.stack([base, far])[None]
    V0 = np.stack([np.full(d, 1.0), np.full(d, 10.0)])[None].astype(np.float32)
    near = base + np.array([0.75, 0, 0, 0, 0, 0, -0.375, 0], np.float32)
    other = np.array([-3.0, 0.1, 2.5, -1.0, 0.2, 0.3, -2.2, 1.7], np.float32)
    K1 = np.stack([near, base, other])[None]
    V1 = np.stack([np.full(d, 2.0), np.full(d, 6.0), np.full(d, -4.0)])[None].astype(np.float32)
    last, mean = (oracle.Cache.empty(1, 8, d, r, "fp32") for _ in range(2))
    outs = []
    for cache, mode in ((last, 0), (mean, 1)):
        oracle.tempcache_compress(cache, R, qscale, shift, K0, V0, tau2_q16=NEVER, frame_id=0, rep_mode=mode)
        outs.append(oracle.tempcache_compress(cache, R, qscale, shift, K1, V1, tau2_q16=TAU2(0.9), frame_id=1,
                                              rep_mode=mode))
    # the mode changes what is stored, not what is decided in this call
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)
    assert outs[1][1][0].tolist() == [1, 1, 0]
    expect = base + np.array([0.25, 0, 0, 0, 0, 0, -0.125, 0], np.float32)       # (base + near + base) / 3
    assert np.array_equal(mean.K[0, 0], expect) and np.array_equal(last.K[0, 0], base)
    assert np.array_equal(mean.code[0, 0], oracle.encode(expect[None], R, qscale, shift)[0])
    for field in ("V", "cnt", "stamp", "len"):
        assert np.array_equal(getattr(mean, field), getattr(last, field))
    assert np.array_equal(mean.K[0, 1:3], last.K[0, 1:3]) and np.array_equal(mean.code[0, 1:3], last.code[0, 1:3])
    # second frame: the stored mean counts three times: (3 * expect + k) / 4
    k = expect + np.array([0, 1.0, 0, 0, 0, 0, 0, 0], np.float32)
    oracle.tempcache_compress(mean, R, qscale, shift, k[None, None], V1[:, :1], tau2_q16=TAU2(0.9), frame_id=2,
                              rep_mode=1)
    assert mean.cnt[0, 0] == 4
    assert np.array_equal(mean.K[0, 0], expect + np.array([0, 0.25, 0, 0, 0, 0, 0, 0], np.float32))


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_mean_key_of_exact_duplicates_is_the_key_itself(dtype):
    # drift 0: every group consists of bit-identical keys, so both representatives coincide for the whole rollout
    # (m * k + k + ... over m + g is exact in float32 for these multiplicities) and so does everything derived
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.0, dtype=dtype)
    H, T, d = c["H"], c["T"], c["d"]
    caches = [oracle.Cache.empty(H, 2 * T, d, c["r"], dtype) for _ in range(2)]
    K0, V0 = fs.next_frame()
    prev = [None, None]
    for f in range(4):
        for m, cache in enumerate(caches):
            mm, mg, st = compress(cache, codec, K0, V0, cand=prev[m], tau2_q16=TAU2(0.98), frame_id=f, rep_mode=m)
            prev[m] = mm
        assert (f == 0) or mg.all()
    for field in ("K", "V", "code", "cnt", "stamp", "len"):
        assert np.array_equal(getattr(caches[0], field), getattr(caches[1], field)), field
    assert caches[1].cnt[:, :T].min() == 4


def test_mean_key_stays_inside_the_hull_of_its_group_and_its_code_is_the_code_of_the_stored_key():
    # drifting tokens: per coordinate the stored mean lies between the smallest and the largest member seen so far
    # (up to one rounding), and the slot's code is always the code of what is stored
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.02)
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 2 * T, d, c["r"], "fp32")
    lo = hi = None
    prev = None
    for f in range(5):
        K, V = fs.next_frame()
        mm, mg, st = compress(cache, codec, K, V, cand=prev, tau2_q16=TAU2(0.98), frame_id=f, rep_mode=1)
        prev = mm
        if f == 0:
            lo, hi = K.copy(), K.copy()
            continue
        assert mg.mean() > 0.9 and (mm[mg == 1] == np.broadcast_to(np.arange(T), (H, T))[mg == 1]).all()
        for h in range(H):
            idx = np.nonzero(mg[h])[0]
            lo[h, idx] = np.minimum(lo[h, idx], K[h, idx])
            hi[h, idx] = np.maximum(hi[h, idx], K[h, idx])
        live = cache.K[:, :T]
        assert (live >= lo - 1e-6).all() and (live <= hi + 1e-6).all()
        assert np.array_equal(cache.code[:, :T], oracle.encode(live, codec.R, codec.qscale, codec.shift))
    assert cache.cnt[:, :T].max() == 5


def test_medoid_representative_hand_example_and_weight_of_the_stored_key():
    # appendix, representative-selection ablation, medoid key.  Slot 0 holds `base`; three joiners lie on a line through
    # it (base + 1, 2, 3 steps): with multiplicity 1 the medoid of {base, +1, +2, +3} is +1 (costs 14, 6, 6, 14 in units
    # of step^2: the tie between +1 and +2 goes to the smaller token); with multiplicity 10 the stored key outweighs the
    # joiners and stays.
    d, r = 8, 4
    R = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]] * 2, np.int8)
    qscale, shift = 16.0, 1
    base = np.array([1.0, 2.0, -1.0, 0.5, 3.0, -2.0, 1.5, 0.25], np.float32)
    step = np.array([0.125, 0, 0, 0, 0, 0, 0, 0], np.float32)          # two code units along every column of R
    far = -base[::-1].copy()
    K0 = np.stack([base, far])[None]
    V0 = np.zeros_like(K0)
    K1 = np.stack([base + 3 * step, base + step, base + 2 * step])[None]   # tokens 0, 1, 2 = +3, +1, +2
    for cnt0, expect in ((1, base + step), (10, base)):
        c = oracle.Cache.empty(1, 8, d, r, "fp32")
        oracle.tempcache_compress(c, R, qscale, shift, K0, V0, tau2_q16=NEVER, frame_id=0, rep_mode=2)
        c.cnt[0, 0] = cnt0
        codes = oracle.encode(np.concatenate([base[None], K1[0]]), R, qscale, shift).astype(np.int64)
        assert len({tuple(x) for x in codes}) == 4                       # the four members have four different codes
        mm, mg, _ = oracle.tempcache_compress(c, R, qscale, shift, K1, np.zeros_like(K1), tau2_q16=TAU2(0.9), frame_id=1,
                                              rep_mode=2)
        assert mg[0].tolist() == [1, 1, 1] and mm[0].tolist() == [0, 0, 0]
        assert np.array_equal(c.K[0, 0], expect), cnt0
        assert np.array_equal(c.code[0, 0], oracle.encode(expect[None], R, qscale, shift)[0])
        assert c.cnt[0, 0] == cnt0 + 3 and c.stamp[0, 0] == 1


def test_medoid_representative_is_the_brute_force_weighted_medoid_in_code_space():
    # loose threshold: big groups.  Same decisions as the last-key mode within a call; the stored key is the member with
    # the smallest weighted total squared code distance (stored key first, then tokens ascending, among equals).
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.3)
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 2 * T, d, c["r"], "fp32")
    twin = oracle.Cache.empty(H, 2 * T, d, c["r"], "fp32")
    prev = None
    groups_seen = moved = stayed = 0
    shift_dir = np.sign(np.random.default_rng(2).standard_normal(d)).astype(np.float32)
    for f in range(4):
        K, V = fs.next_frame()
        K = (K + 0.3 * f * shift_dir).astype(np.float32)      # the whole frame moves: joiners sit together, off the stored key
        before = cache.copy()
        mm, mg, st = compress(cache, codec, K, V, cand=prev, tau2_q16=TAU2(0.6), frame_id=f, rep_mode=2)
        if f == 0:
            compress(twin, codec, K, V, tau2_q16=TAU2(0.6), frame_id=f)
            prev = mm
            continue
        ck = oracle.encode(K, codec.R, codec.qscale, codec.shift).astype(np.int64)
        for h in range(H):
            for j in np.unique(mm[h][mg[h] == 1]):
                members = np.nonzero((mg[h] == 1) & (mm[h] == j))[0]
                cold = before.code[h, j].astype(np.int64)
                cand_codes = np.concatenate([cold[None], ck[h, members]])
                w = np.concatenate([[before.cnt[h, j]], np.ones(members.size, np.int64)])
                dist = ((cand_codes[:, None, :] - cand_codes[None, :, :]) ** 2).sum(axis=2)
                cost = (dist * w[None, :]).sum(axis=1)
                best = int(np.argmin(cost))                               # first minimum: stored key, then tokens ascending
                want = before.K[h, j] if best == 0 else K[h, members[best - 1]]
                assert np.array_equal(cache.K[h, j], want), (f, h, j)
                assert np.array_equal(cache.code[h, j], cand_codes[best].astype(np.int8))
                groups_seen += members.size > 1
                moved += best != 0
                stayed += best == 0
        prev = mm
    assert groups_seen > 20 and moved > 20 and stayed > 20               # the cases are all there


def test_equally_scored_candidates_the_smallest_slot_wins():
    # slots 1, 3 and 4 hold the same key (same code, same score for any probe): the match goes to the smallest of them
    # that the candidate list names, whatever the order of the list and however often it repeats an id
    d, r = 8, 4
    R = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]] * 2, np.int8)
    qscale, shift = 16.0, 1
    base = np.array([1.0, 2.0, -1.0, 0.5, 3.0, -2.0, 1.5, 0.25], np.float32)
    other = np.array([-3.0, 0.1, 2.5, -1.0, 0.2, 0.3, -2.2, 1.7], np.float32)
    K0 = np.stack([other, base, -other, base, base])[None]
    V0 = np.zeros_like(K0)
    for cand, expect in ((None, 1), ([[4, 1, 3]], 1), ([[4, 3]], 3), ([[0, 3, 3, 1, 4]], 1), ([[2, 7, -1, 4, 3]], 3),
                         ([[9, 4, 4]], 4), ([[4, 4, 0, 3, 3, 2]], 3)):
        cache = oracle.Cache.empty(1, 8, d, r, "fp32")
        oracle.tempcache_compress(cache, R, qscale, shift, K0, V0, tau2_q16=NEVER, frame_id=0)
        mm, mg, _ = oracle.tempcache_compress(cache, R, qscale, shift, base[None, None], V0[:, :1],
                                              cand=None if cand is None else np.array(cand, np.int32),
                                              tau2_q16=TAU2(0.9), frame_id=1)
        assert mg[0, 0] == 1 and mm[0, 0] == expect, (cand, mm)


def test_match_over_shuffled_and_repeated_candidate_lists_is_the_brute_force_over_the_set():
    # a cache in which many keys occur twice (ties at the top are the rule), candidate lists in random order with
    # repeated, negative and dead ids: the match is the arg-max over the SET of valid ids, smallest slot among equals
    c, fs, codec = stream_cfg1()
    H, T, d = c["H"], c["T"], c["d"]
    rng = np.random.default_rng(7)
    K0, V0 = fs.next_frame()
    K0[:, T // 2:] = K0[:, :T // 2][:, rng.permutation(T // 2)]          # second half repeats the first, permuted
    K1, V1 = fs.next_frame()
    K1[:, ::3] = K0[:, :T:3]                                             # a third of the new tokens are exact copies
    for metric in (0, 1):
        for trial in range(4):
            cache = oracle.Cache.empty(H, 3 * T, d, c["r"], "fp32")
            compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=0)
            n_cand = [T // 4, T, 2 * T, 5][trial]
            cand = rng.integers(-2, T + 3, size=(H, n_cand)).astype(np.int32)
            cand[:, n_cand // 2:] = cand[:, :n_cand - n_cand // 2]            # every id at least twice, far apart
            cand = np.stack([row[rng.permutation(n_cand)] for row in cand])
            old_code = cache.code.copy().astype(np.int64)
            mm, mg, _ = compress(cache, codec, K1, V1, cand=cand, tau2_q16=ALWAYS, metric=metric, frame_id=1)
            cp = oracle.encode(K1, codec.R, codec.qscale, codec.shift).astype(np.int64)
            n_ties = 0
            for h in range(H):
                ids = np.unique(cand[h][(cand[h] >= 0) & (cand[h] < T)])     # ascending set of valid ids
                for i in range(T):
                    S = old_code[h, ids] @ cp[h, i]
                    if metric == 0:
                        S = 2 * S - (old_code[h, ids] ** 2).sum(axis=1)
                    n_ties += int((S == S.max()).sum() > 1)
                    if mg[h, i]:
                        assert mm[h, i] == ids[int(np.argmax(S))], (metric, trial, h, i)   # first maximum = smallest id
            assert trial == 3 or n_ties >= 16               # the case does exercise ties
            assert mg.mean() > 0.5


def test_mean_key_arithmetic_is_float32_in_token_order():
    # the stored mean key decides later integers, so its arithmetic is part of the definition: float32,
    # multiplicity * old key, joiners added in ascending token order, one division.  Values that float32 cannot
    # represent exactly: on some coordinates a float64 accumulation (rounded once at the end) and the reverse order of
    # the additions give other bits, and the oracle must show exactly the defined ones.
    d, r = 8, 4
    R = np.array([[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]] * 2, np.int8)
    qscale, shift = 16.0, 1
    rng = np.random.default_rng(11)
    far = np.array([-3.0, 0.1, 2.5, -1.0, 0.2, 0.3, -2.2, 1.7], np.float32)
    differs64 = differs_rev = 0
    for trial in range(40):
        base = (rng.standard_normal(d) * 1.7 + 0.3).astype(np.float32)
        joiners = (base[None] + 0.01 * rng.standard_normal((3, d))).astype(np.float32)
        cache = oracle.Cache.empty(1, 8, d, r, "fp32")
        K0 = np.stack([base, -base])[None]
        V0 = np.zeros_like(K0)
        oracle.tempcache_compress(cache, R, qscale, shift, K0, V0, tau2_q16=NEVER, frame_id=0, rep_mode=1)
        cache.cnt[0, 0] = 3                                              # as if three keys had merged before
        mm, mg, _ = oracle.tempcache_compress(cache, R, qscale, shift, joiners[None], np.zeros((1, 3, d), np.float32),
                                              tau2_q16=TAU2(0.9), frame_id=1, rep_mode=1)
        assert mg[0].tolist() == [1, 1, 1] and mm[0].tolist() == [0, 0, 0]
        acc = np.float32(3.0) * base                                      # float32 throughout
        for k in joiners:
            acc = (acc + k).astype(np.float32)
        want = (acc / np.float32(6.0)).astype(np.float32)
        assert np.array_equal(cache.K[0, 0], want), trial
        f64 = ((3.0 * base.astype(np.float64) + joiners.astype(np.float64).sum(axis=0)) / 6.0).astype(np.float32)
        rev = np.float32(3.0) * base
        for k in joiners[::-1]:
            rev = (rev + k).astype(np.float32)
        rev = (rev / np.float32(6.0)).astype(np.float32)
        differs64 += int(not np.array_equal(want, f64))
        differs_rev += int(not np.array_equal(want, rev))
    assert differs64 >= 5 and differs_rev >= 5        # the pin can tell the definitions apart


def test_decisions_use_the_cache_as_it_was_at_entry():
    # two identical new tokens and an empty cache: nothing to match, both are appended (no merge inside a call)
    c, fs, codec = stream_cfg1()
    K, V = fs.next_frame()
    K[:, 1] = K[:, 0]
    cache = oracle.Cache.empty(c["H"], 2 * c["T"], c["d"], c["r"], "fp32")
    mm, mg, st = compress(cache, codec, K, V, tau2_q16=ALWAYS, frame_id=0)
    assert not mg.any() and np.all(st[:, 0] == c["T"])


def test_candidate_list_restricts_the_match_and_ignores_invalid_ids():
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.0)
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 3 * T, d, c["r"], "fp32")
    K0, V0 = fs.next_frame()
    compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=0)
    compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=1)        # slots T..2T-1 duplicate 0..T-1
    cand = np.concatenate([np.arange(T, 2 * T), [-1, 5 * T, T, T]]).astype(np.int32)
    cand = np.broadcast_to(cand, (H, cand.size)).copy()
    mm, mg, _ = compress(cache.copy(), codec, K0, V0, cand=cand, tau2_q16=TAU2(0.9), frame_id=2)
    assert mg.all() and np.array_equal(mm, np.broadcast_to(T + np.arange(T, dtype=np.int32), (H, T)))
    mm, mg, _ = compress(cache.copy(), codec, K0, V0, cand=None, tau2_q16=TAU2(0.9), frame_id=2)
    assert mg.all() and np.array_equal(mm, np.broadcast_to(np.arange(T, dtype=np.int32), (H, T)))   # tie -> lowest slot
    empty = np.full((H, 4), -1, np.int32)
    mm, mg, st = compress(cache.copy(), codec, K0, V0, cand=empty, tau2_q16=ALWAYS, frame_id=2)
    assert not mg.any() and np.all(st[:, 2] == T)


def test_zero_key_never_merges():
    c, fs, codec = stream_cfg1()
    K, V = fs.next_frame()
    cache = oracle.Cache.empty(c["H"], 2 * c["T"], c["d"], c["r"], "fp32")
    compress(cache, codec, K, V, tau2_q16=NEVER, frame_id=0)
    mm, mg, _ = compress(cache, codec, np.zeros_like(K), V, tau2_q16=ALWAYS, frame_id=1)
    assert not mg.any()


def test_probe_argument_changes_the_match_but_not_the_verified_key():
    # probe = some other vector (the paper's wording matches by the query): the match follows the probe,
    # the merge test and the stored representative still use the new key
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.0)
    H, T, d = c["H"], c["T"], c["d"]
    K0, V0 = fs.next_frame()
    cache = oracle.Cache.empty(H, 2 * T, d, c["r"], "fp32")
    compress(cache, codec, K0, V0, tau2_q16=NEVER, frame_id=0)
    P = np.roll(K0, 1, axis=1)                                # probe of token i = key of token i-1
    mm, mg, _ = compress(cache, codec, K0, V0, P_new=P, metric=0, tau2_q16=TAU2(0.9), frame_id=1)
    # the probe finds slot i-1, whose key differs from K0[i] unless they are near-duplicates: few merges,
    # and every merged token went to slot i-1
    idx = np.arange(T)
    for h in range(H):
        m = mg[h] == 1
        assert np.array_equal(mm[h][m], ((idx - 1) % T)[m])
        assert np.array_equal(cache.K[h][mm[h][m]], K0[h][m])


def test_eviction_invariants_when_the_cache_is_full():
    c, fs, codec = stream_cfg1()
    H, T, d = c["H"], c["T"], c["d"]
    C = 2 * T + 40
    cache = oracle.Cache.empty(H, C, d, c["r"], "fp32")
    prev, inserted, lost = None, 0, np.zeros(H, np.int64)
    for f in range(8):
        K, V = fs.next_frame()
        before = cache.copy()
        mm, mg, st = compress(cache, codec, K, V, cand=prev, tau2_q16=TAU2(0.98), frame_id=f)
        prev = mm
        inserted += T
        for h in range(H):
            L0, L1 = int(before.len[h]), int(cache.len[h])
            n_merged, n_app, n_evict, n_drop = st[h, 1:5]
            assert L1 == st[h, 0] <= C and n_merged + n_app + n_drop == T
            assert L1 == L0 + n_app - n_evict
            touched = np.unique(mm[h][mg[h] == 1])
            dst = mm[h][(mg[h] == 0) & (mm[h] >= 0)]
            assert len(set(dst.tolist())) == dst.size                     # one slot per appended token
            victims = dst[dst < L0]
            assert victims.size == n_evict and not np.intersect1d(victims, touched).size
            if n_evict:
                untouched = np.setdiff1d(np.arange(L0), touched)
                keys = np.stack([before.stamp[h][untouched], untouched], axis=1)
                order = untouched[np.lexsort((keys[:, 1], keys[:, 0]))]
                assert np.array_equal(np.sort(order[:n_evict]), np.sort(victims))   # the oldest, lowest slots
                assert np.all(np.diff(victims) > 0)                       # filled in ascending slot order
                lost[h] += before.cnt[h][victims].sum()
            lost[h] += n_drop
            assert np.all(cache.stamp[h][touched] == f) and np.all(cache.stamp[h][dst] == f)
            assert cache.cnt[h, :L1].sum() == inserted - lost[h]         # multiplicity is conserved
            assert np.all(cache.cnt[h, :L1] >= 1)
    assert lost.min() > 0                                                 # the test did reach eviction


def test_tokens_are_dropped_when_no_victim_is_left():
    # capacity smaller than one frame of unmatched tokens: the tail of the frame cannot be stored
    c, fs, codec = stream_cfg1()
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 100, d, c["r"], "fp32")
    K, V = fs.next_frame()
    mm, mg, st = compress(cache, codec, K, V, tau2_q16=NEVER, frame_id=0)
    assert st[:, :5].tolist() == [[100, 0, 100, 0, T - 100]] * H
    assert np.array_equal(mm[0, :100], np.arange(100)) and np.all(mm[:, 100:] == -1)


def test_bounded_cache_keeps_a_long_rollout_flat():
    # the point of the method: with temporal merging the live cache stops growing with the rollout
    c, fs, codec = stream_cfg1(p=1.0, sigma_d=0.01)
    H, T, d = c["H"], c["T"], c["d"]
    cache = oracle.Cache.empty(H, 4 * T, d, c["r"], "fp32")
    prev = None
    for f in range(12):
        K, V = fs.next_frame()
        prev, _, _ = compress(cache, codec, K, V, cand=prev, tau2_q16=TAU2(0.98), frame_id=f)
    assert np.all(cache.len == T) and np.all(cache.cnt[:, :T] == 12)
