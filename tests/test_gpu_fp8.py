"""GPU parity of the 8-bit floating-point K/V path: fastar_kv_to_fp8 bit for bit, sparse_attn_fwd_fp8 within a
tolerance, both against the CPU oracle on the same seeded inputs, through the C ABI.

Tolerance of the attention (derived, then written here): keys, values and queries are the same E4M3 values on both
sides and the scores are accumulated in fp32 from exact products, so what differs is the rounding of the softmax weights
to E4M3 (3 mantissa bits: relative error up to 2^-4 per weight, also in the row sum the kernel divides by) and of the
output to bf16.  An output is a convex combination of values; perturbing the weights by a relative eps moves it by at
most 2 eps times the spread of the contributing values around it.  With eps = 2^-4 and spreads of about 1 (values
N(0, 1.2)) the bound is about 0.13, the typical error (independent roundings over tens of keys) a few hundredths:
max-abs <= 0.1, and mean-abs <= 0.01 so that a systematic error cannot hide under the bound.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_01801_amd as fa
from workloads import CONFIGS, FrameStream, make_codec, to_f32, to_storage

from gpu_util import dev_cache, dev_codec, storage_to_f64, to_dev, to_host

pytestmark = pytest.mark.gpu

ATOL_MAX, ATOL_MEAN = 0.1, 0.01


def rand_cache(rng, H, C, d, lens, dtype):
    c = oracle.Cache.empty(H, C, d, 32, dtype)
    c.K[:] = to_storage((rng.standard_normal((H, C, d)) * 1.2).astype(np.float32), dtype)
    c.V[:] = to_storage((rng.standard_normal((H, C, d)) * 1.2).astype(np.float32), dtype)
    c.cnt[:] = rng.integers(1, 6, size=(H, C))
    c.stamp[:] = rng.integers(0, 5, size=(H, C))
    c.len[:] = lens
    return c


@pytest.mark.parametrize("dtype,C,lens", [("bf16", 640, [640, 333, 1]), ("fp32", 200, [200, 130, 0]),
                                          ("bf16", 64 * 50 + 17, [3217, 3000, 64])])
def test_kv_to_fp8_bit_exact_and_incremental(dtype, C, lens):
    rng = np.random.default_rng(C)
    H, d = 3, 128
    c = rand_cache(rng, H, C, d, lens, dtype)
    # awkward values: beyond the format's range, subnormal, exact ties between neighbouring codes, signed zeros
    special = np.array([500.0, -1e6, 448.0, 2.0 ** -10, 3 * 2.0 ** -10, 1.0625, 1.1875, -0.0, 0.0, 2.0 ** -12, 0.0146], np.float32)
    if lens[0] > 4:
        c.K[0, 0, :special.size] = to_storage(special, dtype)
        c.V[0, 1, :special.size] = to_storage(-special, dtype)
    for h in range(H):                                    # dead slots are never read: poison them
        c.K[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), dtype)
        c.V[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), dtype)
    K8r, V8r = oracle.kv8_empty(H, C, d)
    K8r[:], V8r[:] = 0x11, 0x11
    K8, V8 = to_dev(K8r), to_dev(V8r)
    gpu = dev_cache(c)
    oracle.kv_to_fp8(c, K8r, V8r)
    fa.kv_to_fp8(gpu, K8, V8)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(K8), K8r) and np.array_equal(to_host(V8), V8r)
    # a later frame rewrites a few slots: only their blocks change
    c.stamp[:, : min(lens)] = np.where(rng.random((H, min(lens))) < 0.02, 7, c.stamp[:, : min(lens)])
    c.K[:, : min(lens)] = to_storage((rng.standard_normal((H, min(lens), d))).astype(np.float32), dtype)
    gpu = dev_cache(c)
    oracle.kv_to_fp8(c, K8r, V8r, stamp_lo=7)
    fa.kv_to_fp8(gpu, K8, V8, stamp_lo=7)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(K8), K8r) and np.array_equal(to_host(V8), V8r)


def check_fp8_attention(Q, c, sel, nsel, scale, use_cnt=True):
    H, C, d = c.K.shape
    K8r, V8r = oracle.kv8_empty(H, C, d)
    oracle.kv_to_fp8(c, K8r, V8r)
    K8, V8 = fa.kv8_empty(H, C, d)
    fa.kv_to_fp8(dev_cache(c), K8, V8)
    cnt = c.cnt if use_cnt else None
    O, lse = fa.sparse_attn_fwd_fp8(to_dev(Q), K8, V8, None if cnt is None else to_dev(cnt), to_dev(c.len), C,
                                    to_dev(sel), to_dev(nsel), 128, 64, scale)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(K8), K8r) and np.array_equal(to_host(V8), V8r)
    O_r, lse_r = oracle.sparse_attn_fwd_fp8(Q, K8r, V8r, cnt, c.len, C, sel, nsel, 128, 64, scale)
    got = storage_to_f64(to_host(O))
    assert np.isfinite(got).all()
    err = np.abs(got - O_r)
    assert err.max() <= ATOL_MAX, f"max |O - O_ref| = {err.max()}"
    assert err.mean() <= ATOL_MEAN, f"mean |O - O_ref| = {err.mean()}"
    lg = to_host(lse).astype(np.float64)
    empty = np.isneginf(lse_r)
    assert np.array_equal(np.isneginf(lg), empty)
    assert np.abs(lg[~empty] - lse_r[~empty]).max() <= 0.05
    return err.max(), err.mean()


@pytest.mark.parametrize("H,n_q,C,lens,n_sel,seed", [
    (2, 256, 1280, [1280, 546], 5, 0),            # ragged last block, cfg1-like sizes at d = 128
    (3, 300, 64 * 40, [2560, 2000, 0], 9, 1),     # ragged queries, an empty head
    (2, 4680, 64 * 100 + 5, [6405, 6300], 30, 2), # many tiles, capacity that is no multiple of the block
    (1, 130, 640, [640], 10, 3),                  # every block selected
])
def test_fp8_attention_matches_the_oracle(H, n_q, C, lens, n_sel, seed):
    rng = np.random.default_rng(seed)
    d = 128
    c = rand_cache(rng, H, C, d, lens, "bf16")
    for h in range(H):
        c.K[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), "bf16")   # dead slots: poison
        c.V[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), "bf16")
    Q = to_storage((rng.standard_normal((H, n_q, d)) * 1.1).astype(np.float32), "bf16")
    n_qb = (n_q + 127) // 128
    n_kb = (C + 63) // 64
    sel = np.full((H, n_qb, n_sel), -1, np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        for b in range(n_qb):
            m = int(rng.integers(max(1, n_sel // 2), n_sel + 1))
            row = np.sort(rng.choice(n_kb, size=min(m, n_kb), replace=False)).astype(np.int32)
            if rng.random() < 0.4 and row.size > 2:
                row[rng.integers(0, row.size)] = -1                     # padding inside the list
            sel[h, b, :row.size] = row
            nsel[h, b] = row.size
    check_fp8_attention(Q, c, sel, nsel, d ** -0.5)
    check_fp8_attention(Q, c, sel, nsel, d ** -0.5, use_cnt=False)


@pytest.mark.parametrize("H,n_q,C,n_sel", [
    (20, 3600, 64 * 300, 150),     # 580 query blocks: 73 per XCD range, 9 of them left over by the whole round
    (33, 2048, 64 * 256, 128),     # 528 blocks: 2 per range left over
])
def test_fp8_attention_with_a_workspace_splits_the_launch_and_matches_the_plain_one_and_the_oracle(H, n_q, C, n_sel):
    # sparse_attn_fwd_fp8_ws: the query blocks that whole rounds of workgroups leave over are cut into equal shares of
    # their tiles and combined from fragments.  Against the plain launch everywhere, against the oracle on sampled
    # (head, query block) pairs: whole ones, cut ones, a short and an empty list, a head that is not full.
    rng = np.random.default_rng(H + n_sel)
    d = 128
    g = torch.Generator(device="cuda").manual_seed(H * 7 + n_sel)
    Q = (torch.randn(H, n_q, d, device="cuda", generator=g) * 1.1).bfloat16()
    K = torch.randn(H, C, d, device="cuda", generator=g).bfloat16()
    V = torch.randn(H, C, d, device="cuda", generator=g).bfloat16()
    cnt = torch.randint(1, 6, (H, C), device="cuda", generator=g, dtype=torch.int32)
    lens = np.full(H, C, np.int32)
    lens[3] = C // 2 + 17
    gpu = fa.Cache.empty(H, C, d, 32, torch.bfloat16)
    gpu.K.copy_(K); gpu.V.copy_(V); gpu.cnt.copy_(cnt); gpu.stamp.zero_(); gpu.len.copy_(to_dev(lens))
    K8, V8 = fa.kv8_empty(H, C, d)
    fa.kv_to_fp8(gpu, K8, V8)
    n_qb, n_kb = -(-n_q // 128), C // 64
    sel = np.stack([np.stack([np.sort(rng.choice(n_kb, n_sel, replace=False)) for _ in range(n_qb)]) for _ in range(H)]).astype(np.int32)
    nsel = np.full((H, n_qb), n_sel, np.int32)
    total = n_qb * H
    per = -(-total // 8)
    tail_per = per % 64
    assert per > 64 and 0 < tail_per <= 24, "the shape is meant to take the split launch"
    to_item = lambda vi: (vi // tail_per) * per + (per - tail_per) + vi % tail_per
    W = 8 * tail_per * n_sel
    cut = sorted({to_item((i * W // 512) // n_sel) for i in range(1, 512) if (i * W // 512) % n_sel} - set(range(total, 8 * per)))
    short_item, empty_item = cut[1], to_item(1) if to_item(1) not in cut[:3] else to_item(2)
    nsel.reshape(-1)[short_item] = n_sel // 3
    sel.reshape(total, n_sel)[short_item, n_sel // 3:] = -1
    nsel.reshape(-1)[empty_item] = 0
    sel.reshape(total, n_sel)[empty_item, :] = -1
    ws = torch.empty(fa.workspace_bytes(fa.OP_ATTN, H, n_q, C), dtype=torch.uint8, device="cuda")
    args = (Q, K8, V8, cnt, to_dev(lens), C, to_dev(sel), to_dev(nsel), 128, 64, d ** -0.5)
    O_ws, lse_ws = fa.sparse_attn_fwd_fp8(*args, ws=ws)
    O_pl, lse_pl = fa.sparse_attn_fwd_fp8(*args)
    torch.cuda.synchronize()
    a, b = storage_to_f64(to_host(O_ws)), storage_to_f64(to_host(O_pl))
    # a fragment rounds its weights to E4M3 against its own reference maximum: the two launches differ like either does from the oracle
    assert np.isfinite(a).all() and np.abs(a - b).max() <= ATOL_MAX and np.abs(a - b).mean() <= ATOL_MEAN
    lw, lp = to_host(lse_ws).astype(np.float64), to_host(lse_pl).astype(np.float64)
    fin = np.isfinite(lp)
    assert np.array_equal(fin, np.isfinite(lw)) and np.abs(lw[fin] - lp[fin]).max() <= 0.05
    Kc, Vc = to_host(K8), to_host(V8)
    sample = sorted(set([0, n_qb - 1, total - 1, short_item, empty_item, 3 * n_qb] + cut[:2] + cut[-1:]))
    for item in sample:
        h, bq = divmod(item, n_qb)
        q0, q1 = bq * 128, min((bq + 1) * 128, n_q)
        O_r, lse_r = oracle.sparse_attn_fwd_fp8(to_host(Q[h:h + 1, q0:q1]), Kc[h:h + 1], Vc[h:h + 1], to_host(cnt[h:h + 1]),
                                                lens[h:h + 1], C, sel[h:h + 1, bq:bq + 1], nsel[h:h + 1, bq:bq + 1], 128, 64,
                                                d ** -0.5)
        err = np.abs(a[h, q0:q1] - O_r[0])
        assert err.max() <= ATOL_MAX and err.mean() <= ATOL_MEAN, f"item {item}: {err.max()} {err.mean()}"
        ok = np.isfinite(lse_r[0])
        assert np.array_equal(ok, np.isfinite(lw[h, q0:q1])) and np.abs(lw[h, q0:q1][ok] - lse_r[0][ok]).max(initial=0.0) <= 0.05


def test_fp8_attention_with_steadily_climbing_logits_and_a_dominant_key():
    # the reference maximum is updated lazily: scores that climb along the key list, and one key that dominates a row
    rng = np.random.default_rng(9)
    H, n_q, C, d = 1, 128, 64 * 24, 128
    c = rand_cache(rng, H, C, d, [C], "bf16")
    k = to_f32(c.K)
    ramp = np.linspace(0.2, 3.0, C)[None, :, None].astype(np.float32)
    qdir = rng.standard_normal(d).astype(np.float32)
    qdir /= np.linalg.norm(qdir)
    k = k * 0.3 + ramp * qdir[None, None, :] * 3.0
    c.K[:] = to_storage(k, "bf16")
    Q = to_storage((qdir[None, None, :] * 6.0 + 0.1 * rng.standard_normal((H, n_q, d))).astype(np.float32), "bf16")
    sel = np.arange(24, dtype=np.int32)[None, None, :].repeat(H, 0)
    nsel = np.full((H, 1), 24, np.int32)
    check_fp8_attention(Q, c, sel, nsel, d ** -0.5)


def test_fp8_attention_on_a_tempcache_rollout_cfg2_heads():
    # the Wan-shaped layer on two heads: cache built by the oracle's TempCache, selection by the oracle's AnnSA
    c = dict(CONFIGS["cfg2"])
    H, T, d, r = 2, c["T"], c["d"], c["r"]
    fs = FrameStream(c["seed"], c["cfg_id"], H, d, T, c["n_c"], c["p"], c["sigma_d"], "bf16")
    codec = make_codec(c["seed"], c["cfg_id"], d, r)
    cache = oracle.Cache.empty(H, 6 * T, d, r, "bf16")
    prev = None
    for f in range(6):
        K, V = fs.next_frame()
        prev, _, _ = oracle.tempcache_compress(cache, codec.R, codec.qscale, codec.shift, K, V, cand=prev,
                                               tau2_q16=int(round(0.98 ** 2 * 65536)), frame_id=f)
    Q = fs.queries(1)
    qc = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    sel, nsel = oracle.ann_select_self(qc, cache.code, cache.len, 128, 4, 64, 12)
    emax, emean = check_fp8_attention(Q, cache, sel, nsel, d ** -0.5)
    # and the 8-bit result stays close to the attention on the bf16 cache itself
    O16, _ = oracle.sparse_attn_fwd(Q, cache.K, cache.V, cache.cnt, cache.len, sel, nsel, 128, 64, d ** -0.5)
    K8r, V8r = oracle.kv8_empty(H, 6 * T, d)
    oracle.kv_to_fp8(cache, K8r, V8r)
    O8, _ = oracle.sparse_attn_fwd_fp8(Q, K8r, V8r, cache.cnt, cache.len, 6 * T, sel, nsel, 128, 64, d ** -0.5)
    assert np.abs(O8 - O16).mean() < 0.05


def test_fp8_entry_points_reject_unsupported_shapes():
    L = fa.lib()
    Q = torch.zeros((1, 128, 128), dtype=torch.bfloat16, device="cuda")
    K8, V8 = fa.kv8_empty(1, 128)
    ln = torch.tensor([128], dtype=torch.int32, device="cuda")
    sel = torch.zeros((1, 1, 2), dtype=torch.int32, device="cuda")
    ns = torch.ones((1, 1), dtype=torch.int32, device="cuda")
    O = torch.empty_like(Q)
    args = lambda d, BQ, BK: (Q.data_ptr(), 128, K8.data_ptr(), V8.data_ptr(), None, ln.data_ptr(), 1, 128, d,
                              sel.data_ptr(), ns.data_ptr(), BQ, BK, 2, 0.1, O.data_ptr(), None, None)
    assert L.sparse_attn_fwd_fp8(*args(64, 128, 64)) == -2
    assert L.sparse_attn_fwd_fp8(*args(128, 64, 64)) == -2
    assert L.sparse_attn_fwd_fp8(*args(128, 128, 32)) == -2
    assert L.sparse_attn_fwd_fp8(*args(128, 128, 64)) == 0
    torch.cuda.synchronize()
