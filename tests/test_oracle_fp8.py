"""Pins of the oracle's 8-bit floating-point K/V path (E4M3 storage of keys and values for the attention itself).

The format is fixed by its definition (OCP 8-bit floating point, E4M3 "FN": bias 7, subnormals, no infinities, largest
finite value 448), so the codec is pinned by closed forms, by brute force over all codes and by an independent library
routine (torch's float8_e4m3fn conversion on the CPU).  The attention over the 8-bit cache is pinned by dense softmax
attention written in numpy on the decoded values, by Lemma 1, and by its coincidence with the ordinary oracle on
values that E4M3 represents exactly.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import to_f32, to_storage

from test_oracle_attention import dense_attention


def all_codes():
    return np.arange(256, dtype=np.uint8)


def test_decode_follows_the_format_definition():
    v = oracle.fp8_decode(all_codes())
    assert v[0x38] == 1.0 and v[0x7E] == 448.0 and v[0x01] == 2.0 ** -9 and v[0x08] == 2.0 ** -6
    assert v[0xC0] == -2.0 and v[0x00] == 0.0 and v[0x80] == 0.0 and np.signbit(v[0x80])
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.isfinite(np.delete(v, [0x7F, 0xFF])).all()
    for c in range(256):
        if c & 0x7F == 0x7F:
            continue
        e, m = (c >> 3) & 15, c & 7
        want = (m / 8.0) * 2.0 ** -6 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7)
        assert v[c] == (-want if c & 0x80 else want)
    pos = v[:0x7F]
    assert (np.diff(pos) > 0).all()                                   # codes order like their values


def test_decode_matches_the_library_conversion():
    codes = np.delete(all_codes(), [0x7F, 0xFF])
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(oracle.fp8_decode(codes), lib)


def test_encode_inverts_decode_and_is_the_nearest_code_with_ties_to_even():
    codes = np.delete(all_codes(), [0x7F, 0xFF])
    vals = oracle.fp8_decode(codes).astype(np.float32)
    back = oracle.fp8_encode(vals)
    assert np.array_equal(back[codes != 0x80], codes[codes != 0x80])   # -0 may come back as either zero
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.standard_normal(4000) * 3, rng.standard_normal(2000) * 0.01, rng.uniform(-460, 460, 2000),
                        [0.0, 448.0, 449.0, 1e9, -1e9, 2.0 ** -10, 3 * 2.0 ** -10]]).astype(np.float32)
    c = oracle.fp8_encode(x)
    table = oracle.fp8_decode(np.arange(0x7F, dtype=np.uint8))       # non-negative finite values, ascending
    for xi, ci in zip(x, c):
        a = min(abs(float(xi)), 448.0)
        err = np.abs(table - a)
        assert abs(table[ci & 0x7F] - a) == err.min()                  # nearest
        assert bool(ci & 0x80) == bool(np.signbit(xi))
    # exact midpoints go to the even mantissa: between 1.0 (0x38) and 1.125 (0x39) -> 0x38; 1.125 / 1.25 -> 0x3A
    mids = np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10, 416.0 + 16.0], np.float32)
    assert oracle.fp8_encode(mids).tolist() == [0x38, 0x3A, 0x00, 0x02, 0x7E]
    assert oracle.fp8_encode(np.array([1e9, -1e9, 448.0, 460.0], np.float32)).tolist() == [0x7E, 0xFE, 0x7E, 0x7E]


def test_encode_matches_the_library_conversion_in_range():
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(20000) * 2, rng.standard_normal(5000) * 0.02,
                        rng.uniform(-440, 440, 5000)]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.fp8_encode(x), lib)
    xb = to_f32(to_storage(x, "bf16"))                                  # values as a bf16 cache stores them
    lib = torch.from_numpy(xb).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(oracle.fp8_encode(xb), lib)


def make_cache(rng, H, C, d, lens, dtype="bf16", grid=False):
    c = oracle.Cache.empty(H, C, d, 32, dtype)
    draw = (lambda s: rng.integers(-16, 17, size=s) / 8.0) if grid else (lambda s: rng.standard_normal(s) * 1.2)
    c.K[:] = to_storage(draw((H, C, d)).astype(np.float32), dtype)
    c.V[:] = to_storage(draw((H, C, d)).astype(np.float32), dtype)
    c.cnt[:] = rng.integers(1, 5, size=(H, C))
    c.stamp[:] = rng.integers(0, 6, size=(H, C))
    c.len[:] = lens
    return c


def test_kv_to_fp8_layout_dead_slots_and_incremental_blocks():
    rng = np.random.default_rng(5)
    H, C, d = 2, 200, 16                                              # 4 blocks of 64, the last one ragged
    c = make_cache(rng, H, C, d, [200, 130])
    K8, V8T = oracle.kv8_empty(H, C, d)
    assert K8.shape == (H, 256, d) and V8T.shape == (H, 4, d, 64)
    K8[:], V8T[:] = 0x55, 0x55                                        # whatever was there before
    oracle.kv_to_fp8(c, K8, V8T)
    kf, vf = to_f32(c.K), to_f32(c.V)
    for h in range(H):
        L = int(c.len[h])
        assert np.array_equal(K8[h, :L], oracle.fp8_encode(kf[h, :L]))
        for slot in (0, 63, 64, L - 1):
            assert np.array_equal(V8T[h, slot // 64, :, slot % 64], oracle.fp8_encode(vf[h, slot]))
        last = (L - 1) // 64
        assert (K8[h, L:(last + 1) * 64] == 0).all() and (V8T[h, last, :, L - last * 64:] == 0).all()   # dead slots of a live block
        assert (K8[h, (last + 1) * 64:] == 0x55).all()                 # blocks without a live slot are not touched
    # incremental: only blocks that hold a live slot stamped >= stamp_lo are rewritten, and those wholly
    before = (K8.copy(), V8T.copy())
    c.stamp[:] = 0
    c.stamp[0, 70] = 9
    c.stamp[1, 150] = 9                                               # dead slot (len 130): does not count
    c.K[:] = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
    oracle.kv_to_fp8(c, K8, V8T, stamp_lo=9)
    assert np.array_equal(K8[0, 64:128], oracle.fp8_encode(to_f32(c.K)[0, 64:128]))
    K8[0, 64:128] = before[0][0, 64:128]
    assert np.array_equal(K8, before[0])


def full_sel(H, n_q, BQ, lens, BK=64):
    return oracle.full_selection(H, n_q, BQ, np.asarray(lens, np.int32), BK)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_dense_limit_equals_dense_attention_on_the_decoded_values(dtype):
    rng = np.random.default_rng(6)
    H, C, d, n_q = 2, 256, 32, 40
    c = make_cache(rng, H, C, d, [256, 190], dtype)
    Q = to_storage((rng.standard_normal((H, n_q, d)) * 1.1).astype(np.float32), dtype)
    K8, V8T = oracle.kv8_empty(H, C, d)
    oracle.kv_to_fp8(c, K8, V8T)
    sel, nsel = full_sel(H, n_q, 32, c.len)
    O, lse = oracle.sparse_attn_fwd_fp8(Q, K8, V8T, None, c.len, C, sel, nsel, 32, 64, d ** -0.5)
    q8 = oracle.fp8_decode(oracle.fp8_encode(to_f32(Q)))
    for h in range(H):
        L = int(c.len[h])
        k = oracle.fp8_decode(K8[h, :L])
        v = oracle.fp8_decode(np.ascontiguousarray(V8T[h].transpose(0, 2, 1)).reshape(-1, d)[:L])
        Od, lsed = dense_attention(q8[h], k, v, d ** -0.5)
        assert np.abs(O[h] - Od).max() < 1e-12 and np.abs(lse[h] - lsed).max() < 1e-12
        # and it is an 8-bit approximation of the attention on the stored values, not something else
        Of, _ = dense_attention(to_f32(Q)[h].astype(np.float64), to_f32(c.K)[h, :L].astype(np.float64),
                                to_f32(c.V)[h, :L].astype(np.float64), d ** -0.5)
        assert 1e-4 < np.abs(O[h] - Of).max() < 0.25


def test_values_that_e4m3_holds_exactly_give_the_ordinary_oracle_bit_for_bit():
    rng = np.random.default_rng(7)
    H, C, d, n_q = 2, 192, 16, 70
    c = make_cache(rng, H, C, d, [192, 100], "bf16", grid=True)        # multiples of 1/8 up to 2: exact in E4M3
    Q = to_storage((rng.integers(-16, 17, size=(H, n_q, d)) / 8.0).astype(np.float32), "bf16")
    K8, V8T = oracle.kv8_empty(H, C, d)
    oracle.kv_to_fp8(c, K8, V8T)
    sel = np.array([[[0, 2, -1], [1, -1, -1], [0, 1, 2]]] * H, np.int32)
    nsel = np.array([[2, 1, 3]] * H, np.int32)
    a = oracle.sparse_attn_fwd_fp8(Q, K8, V8T, c.cnt, c.len, C, sel, nsel, 32, 64, 0.25)
    b = oracle.sparse_attn_fwd(Q, c.K, c.V, c.cnt, c.len, sel, nsel, 32, 64, 0.25)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_lemma1_holds_on_the_quantised_cache():
    # exact duplicates of quantised keys: representatives with multiplicity and mean value reproduce the dense attention
    # over the duplicates.  The mean of the group's values must itself be a stored (E4M3) value for the identity to be
    # exact, so every member of a group carries the same value.
    rng = np.random.default_rng(8)
    d, n_q, n_rep = 16, 24, 64
    reps_k = (rng.integers(-12, 13, size=(n_rep, d)) / 4.0).astype(np.float32)
    reps_v = (rng.integers(-12, 13, size=(n_rep, d)) / 4.0).astype(np.float32)
    mult = rng.integers(1, 5, size=n_rep)
    Kd = np.repeat(reps_k, mult, axis=0)
    Vd = np.repeat(reps_v, mult, axis=0)
    Q = (rng.integers(-12, 13, size=(1, n_q, d)) / 4.0).astype(np.float32)
    c = oracle.Cache.empty(1, 64, d, 32, "fp32")
    c.K[0], c.V[0], c.cnt[0], c.len[0] = reps_k, reps_v, mult, n_rep
    K8, V8T = oracle.kv8_empty(1, 64, d)
    oracle.kv_to_fp8(c, K8, V8T)
    sel, nsel = full_sel(1, n_q, 32, c.len)
    O, _ = oracle.sparse_attn_fwd_fp8(Q, K8, V8T, c.cnt, c.len, 64, sel, nsel, 32, 64, d ** -0.5)
    Od, _ = dense_attention(Q[0].astype(np.float64), Kd.astype(np.float64), Vd.astype(np.float64), d ** -0.5)
    assert np.abs(O[0] - Od).max() < 1e-12
    Ono, _ = oracle.sparse_attn_fwd_fp8(Q, K8, V8T, None, c.len, 64, sel, nsel, 32, 64, d ** -0.5)
    assert np.abs(Ono[0] - Od).max() > 1e-3                              # without the multiplicities it is another result
