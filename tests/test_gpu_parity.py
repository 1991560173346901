"""GPU parity: every entry point of libfastar.so against the CPU oracle on the same seeded inputs.

Index outputs (codes, merge maps, selections, cache bookkeeping) must match bit for bit; attention
outputs within 2e-2 max-abs (bf16) / 1e-4 (fp32); running-mean values within a few units of the
storage format's last place.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_01801_amd as fa
from workloads import CONFIGS, FrameStream, PromptSet, make_codec, to_f32, to_storage

from gpu_util import assert_cache_equal, dev_cache, dev_codec, host_cache, storage_to_f64, to_dev, to_host

pytestmark = pytest.mark.gpu

TAU2 = lambda tau: int(round(tau * tau * 65536))
ATOL = {"fp32": 1e-4, "bf16": 2e-2}
VTOL = {"fp32": 1e-5, "bf16": 5e-2}


def sync():
    torch.cuda.synchronize()


def test_init_is_idempotent_and_optional():
    # the one-time kernel set-up may be called any number of times, before or after other entry points
    fa.init()
    fa.init()


# ----------------------------------------------------------------------------------------- encode

@pytest.mark.parametrize("dtype,d,r,n", [("fp32", 64, 32, 515), ("bf16", 128, 32, 4681), ("bf16", 64, 64, 33),
                                         ("fp32", 128, 64, 1000), ("bf16", 128, 32, 1), ("fp32", 64, 32, 16)])
@pytest.mark.parametrize("shift", [4, 6, 8, 9, 1])
def test_encode_bit_exact(dtype, d, r, n, shift):
    # shift: the precision ladder of the quantisation ablation (4: the default, about 8 significant bits; 6; 8; 9:
    # codes in {-1, 0, 1}; 1: nearly everything saturates)
    rng = np.random.default_rng(d * 1000 + r + n)
    codec = make_codec(0, 7, d, r)
    codec.shift = shift
    x = (rng.standard_normal((n, d)) * 1.3).astype(np.float32)
    x[0, :4] = [100.0, -100.0, 0.0, 4.5]                       # saturation and exact grid points
    xs = to_storage(x, dtype)
    ref = oracle.encode(xs, codec.R, codec.qscale, codec.shift)
    got = to_host(fa.encode(to_dev(xs), dev_codec(codec)))
    assert np.array_equal(got, ref)


def test_encode_rounding_half_cases_match():
    # coordinates that land exactly on .5 after scaling (qscale = 2): ties must go to even on both sides
    d, r = 64, 32
    codec = make_codec(0, 8, d, r)
    codec.qscale = np.float32(2.0)
    rng = np.random.default_rng(5)
    x = (rng.integers(-40, 41, size=(256, d)) * 0.25).astype(np.float32)
    for dtype in ("fp32", "bf16"):
        xs = to_storage(x, dtype)
        ref = oracle.encode(xs, codec.R, codec.qscale, codec.shift)
        assert np.array_equal(to_host(fa.encode(to_dev(xs), dev_codec(codec))), ref)


# ----------------------------------------------------------------------------------------- selection

def rand_codes(rng, lo, hi, *shape):
    return rng.integers(lo, hi + 1, size=shape).astype(np.int8)


@pytest.mark.parametrize("H,n_q,C,r,BQ,n_rep,BK,n_sel,lens,span", [
    (2, 256, 1280, 32, 128, 4, 64, 5, [1280, 546], 60),          # cfg1-shaped
    (3, 300, 64 * 40, 32, 128, 4, 64, 7, [2560, 2000, 0], 3),    # heavy ties, ragged tail, empty head
    (2, 4680, 64 * 700, 32, 128, 4, 64, 70, [44800, 31111], 50), # rows longer than one scan chunk
    (2, 200, 640, 64, 64, 8, 32, 4, [640, 333], 40),             # r = 64, BK = 32, n_rep = 8
    (1, 130, 512, 32, 128, 1, 64, 20, [500], 30),                # one summary per block, budget > blocks
    (1, 64, 256, 32, 32, 32, 64, 2, [256], 20),                  # per-query summaries
    (4, 300, 32 * 16400, 32, 128, 4, 32, 90, [524800, 524799, 131000, 40], 40),  # long caches: the streaming kernel
    (2, 200, 96 * 33000, 64, 64, 2, 96, 33, [3168000, 300001], 40),              # the same, r = 64, three groups per block
    (4, 300, 32 * 8200, 32, 128, 4, 32, 90, [262400, 262399, 131000, 40], 40),   # long caches below its threshold
])
def test_ann_select_self_bit_exact(H, n_q, C, r, BQ, n_rep, BK, n_sel, lens, span):
    rng = np.random.default_rng(n_q + C)
    qc, kc = rand_codes(rng, -span, span, H, n_q, r), rand_codes(rng, -span, span, H, C, r)
    length = np.array(lens, np.int32)
    ref_sel, ref_nsel = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel)
    sel, nsel = fa.ann_select_self(to_dev(qc), to_dev(kc), to_dev(length), BQ, n_rep, BK, n_sel)
    assert np.array_equal(to_host(nsel), ref_nsel)
    assert np.array_equal(to_host(sel), ref_sel)


@pytest.mark.parametrize("H,n_q,C,lens,n_sel,n_sink,n_local", [
    (2, 300, 64 * 40, [2560, 1000], 9, 2, 3),            # rows of 40 / 16 blocks (three radix passes)
    (3, 3600, 64 * 3600, [230400, 200001, 64], 360, 4, 56),   # world-model rows (selection from registers), one tiny head
    (2, 200, 64 * 30, [1920, 130], 5, 2, 3),             # forced blocks fill the budget; a head with fewer blocks than that
    (1, 128, 64 * 200, [12800], 20, 0, 7), (1, 128, 64 * 200, [12800], 20, 6, 0)])
def test_ann_select_self_with_forced_sink_and_local_blocks(H, n_q, C, lens, n_sel, n_sink, n_local):
    rng = np.random.default_rng(n_q + C + n_sink)
    qc, kc = rand_codes(rng, -40, 40, H, n_q, 32), rand_codes(rng, -40, 40, H, C, 32)
    length = np.array(lens, np.int32)
    ref_sel, ref_nsel = oracle.ann_select_self(qc, kc, length, 128, 4, 64, n_sel, n_sink, n_local)
    sel, nsel = fa.ann_select_self(to_dev(qc), to_dev(kc), to_dev(length), 128, 4, 64, n_sel, n_sink=n_sink, n_local=n_local)
    assert np.array_equal(to_host(nsel), ref_nsel)
    assert np.array_equal(to_host(sel), ref_sel)
    with pytest.raises(fa.FastarError):
        fa.ann_select_self(to_dev(qc), to_dev(kc), to_dev(length), 128, 4, 64, 4, n_sink=3, n_local=2)


@pytest.mark.parametrize("H,n_q,n_p,r,BQ,n_sel,span", [
    (2, 256, 64, 32, 128, 16, 60), (2, 4680, 512, 32, 128, 64, 50), (1, 300, 2048, 32, 128, 64, 4),
    (2, 100, 97, 64, 64, 10, 30), (1, 50, 20, 32, 128, 64, 30),
    (2, 4680, 512, 32, 1560, 64, 50), (1, 3600, 2048, 64, 3600, 64, 20),   # one selection per frame (query block = frame)
])
def test_ann_select_cross_bit_exact(H, n_q, n_p, r, BQ, n_sel, span):
    rng = np.random.default_rng(n_q + n_p)
    qc, pc = rand_codes(rng, -span, span, H, n_q, r), rand_codes(rng, -span, span, H, n_p, r)
    ref_sel, ref_nsel = oracle.ann_select_cross(qc, pc, BQ, n_sel)
    sel, nsel = fa.ann_select_cross(to_dev(qc), to_dev(pc), BQ, n_sel)
    assert np.array_equal(to_host(nsel), ref_nsel)
    assert np.array_equal(to_host(sel), ref_sel)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_selection_on_seeded_random_shapes(seed):
    """AnnSA and AnnCA on a dozen random shapes per seed: both code widths, every summary count, key blocks of 32..128
    rows, ragged query blocks and caches (an empty head now and then), budgets from one block to more than there are,
    narrow code ranges (many ties) and wide ones.  Selections are bit-exact."""
    rng = np.random.default_rng(100 + seed)
    for case in range(12):
        H, r = int(rng.integers(1, 5)), int(rng.choice([32, 64]))
        n_rep = int(rng.choice([1, 2, 4, 8, 16, 32]))
        BQ = n_rep * int(rng.integers(1, 128 // n_rep + 1))
        BK = 32 * int(rng.integers(1, 5))
        n_q, C = int(rng.integers(1, 900)), int(rng.integers(1, 6000))
        n_blocks = (C + BK - 1) // BK
        n_sel = int(rng.integers(1, n_blocks + 8))
        lens = [int(rng.integers(0, C + 1)) for _ in range(H)]
        if rng.random() < 0.3:
            lens[0] = C
        if rng.random() < 0.2:
            lens[-1] = 0
        span = int(rng.choice([1, 3, 40, 127]))
        qc, kc = rand_codes(rng, -span, span, H, n_q, r), rand_codes(rng, -span, span, H, C, r)
        length = np.array(lens, np.int32)
        what = f"seed {seed} case {case}: H={H} r={r} n_rep={n_rep} BQ={BQ} BK={BK} n_q={n_q} C={C} n_sel={n_sel} lens={lens}"
        ref_sel, ref_nsel = oracle.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel)
        sel, nsel = fa.ann_select_self(to_dev(qc), to_dev(kc), to_dev(length), BQ, n_rep, BK, n_sel)
        assert np.array_equal(to_host(nsel), ref_nsel), what
        assert np.array_equal(to_host(sel), ref_sel), what

        n_p, BQc, n_selc = int(rng.integers(1, 1500)), int(rng.integers(1, 400)), int(rng.integers(1, 100))
        pc = rand_codes(rng, -span, span, H, n_p, r)
        what = f"seed {seed} case {case}: H={H} r={r} BQ={BQc} n_q={n_q} n_p={n_p} n_sel={n_selc}"
        ref_sel, ref_nsel = oracle.ann_select_cross(qc, pc, BQc, n_selc)
        sel, nsel = fa.ann_select_cross(to_dev(qc), to_dev(pc), BQc, n_selc)
        assert np.array_equal(to_host(nsel), ref_nsel), what
        assert np.array_equal(to_host(sel), ref_sel), what


def test_selection_is_deterministic_across_repeats():
    rng = np.random.default_rng(11)
    qc, kc = rand_codes(rng, -2, 2, 4, 1000, 32), rand_codes(rng, -2, 2, 4, 64 * 300, 32)
    length = to_dev(np.array([19200, 19000, 64, 1], np.int32))
    q, k = to_dev(qc), to_dev(kc)
    first = fa.ann_select_self(q, k, length, 128, 4, 64, 30)
    first = (first[0].clone(), first[1].clone())
    for _ in range(10):
        again = fa.ann_select_self(q, k, length, 128, 4, 64, 30)
        assert torch.equal(again[0], first[0]) and torch.equal(again[1], first[1])


# ----------------------------------------------------------------------------------------- sign codes (LSH)

def as_u32(t):
    return to_host(t).view(np.uint32)


@pytest.mark.parametrize("dtype,d,n_bits,n", [("fp32", 64, 64, 515), ("bf16", 128, 128, 4681), ("bf16", 64, 256, 33),
                                              ("fp32", 128, 256, 1000), ("bf16", 128, 64, 1), ("fp32", 64, 128, 16)])
def test_encode_sign_bit_exact(dtype, d, n_bits, n):
    rng = np.random.default_rng(d + n_bits + n)
    R = rng.choice(np.array([-1, 1], np.int8), size=(d, n_bits))
    x = rng.standard_normal((n, d)).astype(np.float32) * 1.5
    x[::7] = np.round(x[::7])                                       # projections that land on zero happen
    x[::11] = 0.0
    xs = to_storage(x, dtype)
    ref = oracle.encode_sign(xs, R, 127 / 4.5)
    got = fa.encode_sign(to_dev(xs), to_dev(R), 127 / 4.5)
    sync()
    assert np.array_equal(as_u32(got), ref)


@pytest.mark.parametrize("H,n_q,C,n_bits,BQ,n_rep,BK,n_sel,lens,flip", [
    (2, 256, 1280, 128, 128, 4, 64, 5, [1280, 546], 0.3),            # cfg1-shaped
    (3, 300, 64 * 40, 128, 128, 4, 64, 7, [2560, 2000, 0], 0.02),     # heavy ties, ragged tail, empty head
    (2, 1000, 64 * 300, 64, 128, 4, 64, 40, [19200, 13111], 0.3),
    (2, 200, 640, 256, 64, 8, 16, 9, [640, 333], 0.2),                # several key blocks per wavefront round
    (1, 130, 1024, 128, 128, 1, 128, 3, [1000], 0.3),                 # key blocks of two rounds
    (2, 300, 97, 128, 128, 128, 1, 20, [97, 50], 0.1),                # cross-attention form: BK = 1, n_rep = BQ
])
def test_ann_select_lsh_bit_exact(H, n_q, C, n_bits, BQ, n_rep, BK, n_sel, lens, flip):
    rng = np.random.default_rng(n_q + C + n_bits)
    W = n_bits // 32
    # codes that cluster: a few prototypes with a fraction of their bits flipped, so that scores repeat and spread
    proto = rng.integers(0, 2, size=(8, n_bits))
    def draw(n):
        b = proto[rng.integers(0, 8, size=n)] ^ (rng.random((n, n_bits)) < flip)
        words = np.zeros((n, W), np.uint32)
        for j in range(n_bits):
            words[:, j // 32] |= (b[:, j].astype(np.uint32) << np.uint32(j % 32))
        return words
    qb = np.stack([draw(n_q) for _ in range(H)])
    kb = np.stack([draw(C) for _ in range(H)])
    length = np.array(lens, np.int32)
    ref_sel, ref_nsel = oracle.ann_select_lsh(qb, kb, length, BQ, n_rep, BK, n_sel)
    sel, nsel = fa.ann_select_lsh(to_dev(qb.view(np.int32)), to_dev(kb.view(np.int32)), to_dev(length), BQ, n_rep, BK,
                                  n_sel)
    sync()
    assert np.array_equal(to_host(nsel), ref_nsel)
    assert np.array_equal(to_host(sel), ref_sel)


@pytest.mark.parametrize("band,radius", [(4, 0), (8, 0), (8, 1), (16, 2), (32, 5), (8, 9), (16, 0)])
@pytest.mark.parametrize("H,n_q,C,n_bits,BQ,n_rep,BK,n_sel,lens,flip,sink,local", [
    (2, 256, 1280, 128, 128, 4, 64, 5, [1280, 546], 0.3, 0, 0),
    (3, 300, 64 * 40, 64, 128, 4, 64, 7, [2560, 2000, 0], 0.02, 1, 2),   # heavy ties, empty head, forced blocks
    (2, 200, 640, 256, 64, 8, 16, 30, [640, 333], 0.45, 0, 0),            # nearly random codes: few collisions, budget > candidates
    (2, 300, 97, 128, 128, 128, 1, 20, [97, 50], 0.1, 0, 0),              # cross-attention form
])
def test_ann_select_lsh_buckets_bit_exact(band, radius, H, n_q, C, n_bits, BQ, n_rep, BK, n_sel, lens, flip, sink, local):
    rng = np.random.default_rng(n_q + C + n_bits + band + radius)
    W = n_bits // 32
    proto = rng.integers(0, 2, size=(8, n_bits))
    def draw(n):
        b = proto[rng.integers(0, 8, size=n)] ^ (rng.random((n, n_bits)) < flip)
        words = np.zeros((n, W), np.uint32)
        for j in range(n_bits):
            words[:, j // 32] |= (b[:, j].astype(np.uint32) << np.uint32(j % 32))
        return words
    qb = np.stack([draw(n_q) for _ in range(H)])
    kb = np.stack([draw(C) for _ in range(H)])
    length = np.array(lens, np.int32)
    ref_sel, ref_nsel = oracle.ann_select_lsh_buckets(qb, kb, length, band, radius, BQ, n_rep, BK, n_sel, sink, local)
    sel, nsel = fa.ann_select_lsh_buckets(to_dev(qb.view(np.int32)), to_dev(kb.view(np.int32)), to_dev(length), band,
                                          radius, BQ, n_rep, BK, n_sel, sink, local)
    sync()
    assert np.array_equal(to_host(nsel), ref_nsel)
    assert np.array_equal(to_host(sel), ref_sel)


def test_sign_codes_select_then_attend_end_to_end():
    """Hash the cache keys and the queries, select on shared bits, attend: the whole variant against the oracle."""
    c = dict(CONFIGS["cfg1"])
    fs = FrameStream(c["seed"], c["cfg_id"], c["H"], c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
    frames = [fs.next_frame() for _ in range(4)]
    K = np.concatenate([f[0] for f in frames], axis=1)
    V = np.concatenate([f[1] for f in frames], axis=1)
    Q = fs.queries(1)
    rng = np.random.default_rng(2)
    R = rng.choice(np.array([-1, 1], np.int8), size=(c["d"], 128))
    q = 127 / 4.5
    H, C = K.shape[0], K.shape[1]
    length = np.full((H,), C, np.int32)
    qb_r, kb_r = oracle.encode_sign(Q, R, q), oracle.encode_sign(K, R, q)
    sel_r, nsel_r = oracle.ann_select_lsh(qb_r, kb_r, length, 128, 4, 64, 5)
    O_r, _ = oracle.sparse_attn_fwd(Q, K, V, None, length, sel_r, nsel_r, 128, 64, c["d"] ** -0.5)
    dQ, dK, dV, dR, dlen = to_dev(Q), to_dev(K), to_dev(V), to_dev(R), to_dev(length)
    qb, kb = fa.encode_sign(dQ, dR, q), fa.encode_sign(dK, dR, q)
    sel, nsel = fa.ann_select_lsh(qb, kb, dlen, 128, 4, 64, 5)
    O, _ = fa.sparse_attn_fwd(dQ, dK, dV, None, dlen, sel, nsel, 128, 64, c["d"] ** -0.5)
    sync()
    assert np.array_equal(as_u32(qb), qb_r) and np.array_equal(as_u32(kb), kb_r)
    assert np.array_equal(to_host(sel), sel_r) and np.array_equal(to_host(nsel), nsel_r)
    assert np.abs(storage_to_f64(to_host(O)) - O_r).max() <= ATOL[c["dtype"]]


def test_per_frame_prompt_selection_then_cross_attention_per_frame():
    """AnnCA with the frame as the query block (Sec. 5.3 selects prompt tokens per frame): one selection per frame, its
    list shared by the query blocks of that frame's attention call."""
    c = dict(CONFIGS["cfg2"]); c["H"] = 2
    fs = FrameStream(c["seed"], c["cfg_id"], c["H"], c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
    ps = PromptSet(c["seed"], c["cfg_id"], fs.centreK, 512, 32, 3, c["dtype"])
    codec = make_codec(c["seed"], c["cfg_id"], c["d"], c["r"])
    T, H, n_sel = c["T"], c["H"], 64
    fs.next_frame()
    Q = fs.queries(2)                                             # two frames of queries
    qc_r = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    pc_r = oracle.encode(ps.K, codec.R, codec.qscale, codec.shift)
    sel_r, nsel_r = oracle.ann_select_cross(qc_r, pc_r, T, n_sel)            # [H, 2 frames, n_sel]
    dcodec = dev_codec(codec)
    qc, pc = fa.encode(to_dev(Q), dcodec), fa.encode(to_dev(ps.K), dcodec)
    sel, nsel = fa.ann_select_cross(qc, pc, T, n_sel)
    sync()
    assert np.array_equal(to_host(sel), sel_r) and np.array_equal(to_host(nsel), nsel_r)
    plen = np.full((H,), 512, np.int32)
    n_qb = (T + 127) // 128
    for f in range(2):
        Qf = np.ascontiguousarray(Q[:, f * T:(f + 1) * T])
        sel_f = np.ascontiguousarray(np.repeat(sel_r[:, f:f + 1], n_qb, axis=1))
        nsel_f = np.ascontiguousarray(np.repeat(nsel_r[:, f:f + 1], n_qb, axis=1))
        check_attention(Qf, ps.K, ps.V, None, plen, sel_f, nsel_f, 128, 1, c["d"] ** -0.5, c["dtype"])


@pytest.mark.parametrize("H,n_q,n_p,r,n_sel", [(2, 4680, 512, 32, 64), (1, 300, 2048, 64, 64), (2, 200, 40, 32, 64),
                                               (3, 129, 97, 32, 17), (1, 128, 512, 32, 1)])
def test_fused_prompt_selection_and_attention_matches_the_two_calls(H, n_q, n_p, r, n_sel):
    """ann_cross_attn_fwd against the oracle's selection followed by its attention over that selection, and against the
    library's own two-call path (ragged query tail, fewer prompt tokens than the budget, budgets below a full tile)."""
    rng = np.random.default_rng(n_q + n_p + n_sel)
    d = 128
    codec = make_codec(0, 4, d, r)
    Q = to_storage(rng.standard_normal((H, n_q, d)).astype(np.float32), "bf16")
    Kp = to_storage(rng.standard_normal((H, n_p, d)).astype(np.float32), "bf16")
    Vp = to_storage(rng.standard_normal((H, n_p, d)).astype(np.float32), "bf16")
    qc_r = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    pc_r = oracle.encode(Kp, codec.R, codec.qscale, codec.shift)
    sel_r, nsel_r = oracle.ann_select_cross(qc_r, pc_r, 128, n_sel)
    plen = np.full((H,), n_p, np.int32)
    scale = d ** -0.5
    O_r, _ = oracle.sparse_attn_fwd(Q, Kp, Vp, None, plen, sel_r, nsel_r, 128, 1, scale)
    dQ, dK, dV = to_dev(Q), to_dev(Kp), to_dev(Vp)
    dcodec = dev_codec(codec)
    qc, pc = fa.encode(dQ, dcodec), fa.encode(dK, dcodec)
    sel, nsel, O = fa.ann_cross_attn_fwd(dQ, qc, dK, dV, pc, 128, n_sel, scale)
    sel2, nsel2 = fa.ann_select_cross(qc, pc, 128, n_sel)
    O2, _ = fa.sparse_attn_fwd(dQ, dK, dV, None, to_dev(plen), sel2, nsel2, 128, 1, scale)
    sync()
    assert np.array_equal(to_host(sel), sel_r) and np.array_equal(to_host(nsel), nsel_r)
    assert np.array_equal(to_host(sel2), sel_r)
    Of = storage_to_f64(to_host(O))
    assert np.isfinite(Of).all()
    assert np.abs(Of - O_r).max() <= ATOL["bf16"]
    assert np.abs(Of - storage_to_f64(to_host(O2))).max() <= ATOL["bf16"]


def test_fused_prompt_attention_rejects_what_it_is_not_built_for():
    Q = torch.zeros((1, 128, 64), dtype=torch.bfloat16, device="cuda")
    code = torch.zeros((1, 128, 32), dtype=torch.int8, device="cuda")
    with pytest.raises(fa.FastarError):
        fa.ann_cross_attn_fwd(Q, code, Q, Q, code, 128, 16, 0.125)            # d = 64
    Q = torch.zeros((1, 128, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fa.FastarError):
        fa.ann_cross_attn_fwd(Q, code, Q, Q, code, 128, 65, 0.125)            # more than one tile of tokens
    with pytest.raises(fa.FastarError):
        fa.ann_cross_attn_fwd(Q, code, Q, Q, code, 64, 16, 0.125)             # query blocks of 64


# ----------------------------------------------------------------------------------------- attention

def random_selection(rng, H, n_qb, n_sel, lens, BK, empty_some=True):
    sel = np.full((H, n_qb, n_sel), -1, np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        n_kb = (lens[h] + BK - 1) // BK
        for b in range(n_qb):
            if n_kb == 0 or (empty_some and b == 1):
                continue
            m = int(rng.integers(1, min(n_sel, n_kb) + 1))
            sel[h, b, :m] = np.sort(rng.choice(n_kb, size=m, replace=False))
            nsel[h, b] = m
    return sel, nsel


def check_attention(Q, K, V, cnt, length, sel, nsel, BQ, BK, scale, dtype):
    O_ref, lse_ref = oracle.sparse_attn_fwd(Q, K, V, cnt, length, sel, nsel, BQ, BK, scale)
    O, lse = fa.sparse_attn_fwd(to_dev(Q), to_dev(K), to_dev(V), None if cnt is None else to_dev(cnt), to_dev(length),
                                to_dev(sel), to_dev(nsel), BQ, BK, scale)
    sync()
    O = storage_to_f64(to_host(O))
    lse = to_host(lse).astype(np.float64)
    assert np.isfinite(O).all()
    err = np.abs(O - O_ref).max()
    assert err <= ATOL[dtype], f"max |O - O_ref| = {err}"
    fin = np.isfinite(lse_ref)
    assert np.array_equal(np.isneginf(lse), ~fin)
    assert np.abs(lse[fin] - lse_ref[fin]).max(initial=0.0) <= (1e-4 if dtype == "fp32" else 2e-2)
    return err


@pytest.mark.parametrize("dtype,H,n_q,C,d,BQ,BK,n_sel,lens,use_cnt", [
    ("fp32", 2, 256, 1280, 64, 128, 64, 6, [1280, 546], True),       # cfg1-shaped
    ("fp32", 1, 100, 300, 128, 64, 16, 9, [291], False),
    ("bf16", 3, 700, 64 * 50, 128, 128, 64, 12, [3200, 2011, 0], True),   # ragged query tail, ragged / empty caches
    ("bf16", 2, 300, 2048, 128, 128, 1, 64, [2048, 1500], False),    # token-granular gather (cross-attention)
    ("bf16", 2, 260, 1024, 64, 64, 64, 5, [1024, 1000], True),       # d = 64, BQ = 64
    ("bf16", 1, 128, 512, 128, 64, 8, 40, [509], True),              # small key blocks
    ("bf16", 2, 200, 640, 64, 128, 64, 10, [640, 600], False),
    ("bf16", 1, 300, 64 * 20, 128, 128, 64, 20, [1280], True),       # odd number of query blocks: a lone block in the last workgroup
    ("bf16", 1, 100, 640, 128, 128, 32, 7, [640], True),             # a single query block
    ("bf16", 5, 128, 64 * 9, 128, 128, 64, 9, [576, 64, 0, 576, 1], False),   # neighbours with 9 / 1 / 0 tiles
    ("bf16", 2, 384, 64 * 150, 128, 128, 64, 140, [9600, 9017], True),   # lists longer than 64 and 128 entries
    ("bf16", 2, 300, 1000, 128, 128, 64, 16, [1000, 777], True),     # capacity that is no multiple of the key block
    ("bf16", 2, 384, 270000, 128, 128, 64, 20, [270000, 123457], True),   # K and V beyond the memory-side cache: other variant
])
def test_sparse_attention_matches_oracle(dtype, H, n_q, C, d, BQ, BK, n_sel, lens, use_cnt):
    rng = np.random.default_rng(n_q * 7 + C)
    Q = to_storage(rng.standard_normal((H, n_q, d)).astype(np.float32), dtype)
    K = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), dtype)
    V = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), dtype)
    length = np.array(lens, np.int32)
    for h in range(H):                                               # poison dead slots: they must stay invisible
        K[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), dtype)
        V[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.inf, np.float32), dtype)
    cnt = rng.integers(1, 9, size=(H, C)).astype(np.int32) if use_cnt else None
    n_qb = (n_q + BQ - 1) // BQ
    sel, nsel = random_selection(rng, H, n_qb, n_sel, lens, BK)
    check_attention(Q, K, V, cnt, length, sel, nsel, BQ, BK, d ** -0.5, dtype)


def test_attention_skips_negative_and_dead_entries_inside_a_list():
    """Entries that are negative or name a key block beyond len count as listed but contribute nothing."""
    rng = np.random.default_rng(77)
    H, n_q, C, d, BQ, BK, n_sel = 2, 256, 64 * 40, 128, 128, 64, 70
    lens = [64 * 30 + 5, 64 * 12]
    Q = to_storage(rng.standard_normal((H, n_q, d)).astype(np.float32), "bf16")
    K = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
    V = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
    length = np.array(lens, np.int32)
    for h in range(H):
        K[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), "bf16")
        V[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.inf, np.float32), "bf16")
    cnt = rng.integers(1, 9, size=(H, C)).astype(np.int32)
    n_qb = n_q // BQ
    sel = np.full((H, n_qb, n_sel), -1, np.int32)
    nsel = np.zeros((H, n_qb), np.int32)
    for h in range(H):
        n_kb = (lens[h] + BK - 1) // BK
        for b in range(n_qb):
            m = n_sel - 3 * b
            row = rng.integers(0, C // BK, size=m).astype(np.int32)    # some of them name dead blocks
            row[rng.random(m) < 0.2] = -1
            row[0] = -1 if b == 0 else n_kb - 1                        # a list that starts with nothing / with the partial block
            row[-1] = C // BK - 1
            sel[h, b, :m] = row
            nsel[h, b] = m
    sel[1, 1, :nsel[1, 1]] = -1                                        # a list of nothing at all
    check_attention(Q, K, V, cnt, length, sel, nsel, BQ, BK, d ** -0.5, "bf16")


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_attention_on_seeded_random_shapes(seed):
    """bf16, d 128, key blocks of 64 rows: a dozen random shapes per seed (ragged queries and caches, capacities that are
    no multiple of the block, lists of 0..150 entries with repeats, negative and dead entries, with and without
    multiplicities, query scales 0.3..3) against the oracle."""
    rng = np.random.default_rng(seed)
    d, BQ, BK = 128, 128, 64
    for case in range(12):
        H, n_q, C = int(rng.integers(1, 5)), int(rng.integers(1, 700)), int(rng.integers(64, 64 * 60))
        n_sel = int(rng.integers(1, 150))
        lens = [int(rng.integers(0, C + 1)) for _ in range(H)]
        if rng.random() < 0.3:
            lens[0] = C
        Q = to_storage(rng.standard_normal((H, n_q, d)).astype(np.float32) * rng.choice([0.3, 1.0, 3.0]), "bf16")
        K = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
        V = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
        for h in range(H):                                           # poison dead slots
            K[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), "bf16")
            V[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.inf, np.float32), "bf16")
        cnt = rng.integers(1, 9, size=(H, C)).astype(np.int32) if rng.random() < 0.7 else None
        n_qb = (n_q + BQ - 1) // BQ
        sel = np.full((H, n_qb, n_sel), -1, np.int32)
        nsel = np.zeros((H, n_qb), np.int32)
        for h in range(H):
            for b in range(n_qb):
                m = int(rng.integers(0, n_sel + 1))
                row = rng.integers(0, (C + BK - 1) // BK, size=m).astype(np.int32)
                if m and rng.random() < 0.5:
                    row[rng.random(m) < 0.15] = -1
                sel[h, b, :m] = row
                nsel[h, b] = m
        check_attention(Q, K, V, cnt, np.array(lens, np.int32), sel, nsel, BQ, BK, d ** -0.5, "bf16")


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_attention_on_seeded_random_shapes_of_every_kernel(seed):
    """The same over everything sparse_attn_fwd supports: fp32 (any query block up to 128, any key block up to 64) and
    bf16 (query blocks of 64 / 128, key blocks 1 .. 64), both head widths, so that every kernel behind the entry point
    sees ragged shapes, repeated / negative / dead entries and poisoned dead slots."""
    rng = np.random.default_rng(300 + seed)
    for case in range(16):
        dtype, d = str(rng.choice(["fp32", "bf16"])), int(rng.choice([64, 128]))
        if dtype == "bf16":
            BQ, BK = int(rng.choice([64, 128])), int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        else:
            BQ, BK = int(rng.integers(1, 129)), int(rng.integers(1, 65))
        H, n_q, C = int(rng.integers(1, 4)), int(rng.integers(1, 500)), int(rng.integers(BK, 3000))
        n_sel = int(rng.integers(1, 100))
        lens = [int(rng.integers(0, C + 1)) for _ in range(H)]
        if rng.random() < 0.3:
            lens[0] = C
        Q = to_storage(rng.standard_normal((H, n_q, d)).astype(np.float32) * rng.choice([0.3, 1.0, 3.0]), dtype)
        K = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), dtype)
        V = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), dtype)
        for h in range(H):                                           # poison dead slots
            K[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.nan, np.float32), dtype)
            V[h, lens[h]:] = to_storage(np.full((C - lens[h], d), np.inf, np.float32), dtype)
        cnt = rng.integers(1, 9, size=(H, C)).astype(np.int32) if rng.random() < 0.7 else None
        n_qb = (n_q + BQ - 1) // BQ
        sel = np.full((H, n_qb, n_sel), -1, np.int32)
        nsel = np.zeros((H, n_qb), np.int32)
        for h in range(H):
            for b in range(n_qb):
                m = int(rng.integers(0, n_sel + 1))
                row = rng.integers(0, (C + BK - 1) // BK, size=m).astype(np.int32)
                if m and rng.random() < 0.5:
                    row[rng.random(m) < 0.15] = -1
                sel[h, b, :m] = row
                nsel[h, b] = m
        try:
            check_attention(Q, K, V, cnt, np.array(lens, np.int32), sel, nsel, BQ, BK, d ** -0.5, dtype)
        except AssertionError as e:
            raise AssertionError(f"seed {seed} case {case}: {dtype} d={d} BQ={BQ} BK={BK} H={H} n_q={n_q} C={C} "
                                 f"n_sel={n_sel} lens={lens} cnt={'yes' if cnt is not None else 'no'}: {e}") from e


def test_dense_limit_on_clustered_data_fp32_and_bf16():
    for name, dtype in (("cfg1", "fp32"), ("cfg1", "bf16")):
        c = CONFIGS[name]
        fs = FrameStream.from_config(name, dtype=dtype)
        frames = [fs.next_frame() for _ in range(3)]
        K = np.concatenate([k for k, _ in frames], axis=1)
        V = np.concatenate([v for _, v in frames], axis=1)
        Q = fs.queries(1)
        length = np.full(c["H"], K.shape[1], np.int32)
        sel, nsel = oracle.full_selection(c["H"], Q.shape[1], 128, length, 64)
        check_attention(Q, K, V, None, length, sel, nsel, 128, 64, c["d"] ** -0.5, dtype)


# ----------------------------------------------------------------------------------------- TempCache

def run_rollout(name, n_frames, C, tau, dtype=None, H=None, windowed=True, metric=0, probe_queries=False, rep_mode=0,
                persistent=False, r=None, shift=None, frame_shift=0.0):
    over = {}
    if dtype:
        over["dtype"] = dtype
    if r:
        over["r"] = r
    c = dict(CONFIGS[name]); c.update(over)
    if H:
        c["H"] = H
    fs = FrameStream(c["seed"], c["cfg_id"], c["H"], c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
    codec = make_codec(c["seed"], c["cfg_id"], c["d"], c["r"])
    if shift:
        codec.shift = shift
    ref = oracle.Cache.empty(c["H"], C, c["d"], c["r"], c["dtype"])
    gpu = dev_cache(ref)
    dcodec = dev_codec(codec)
    prev_ref, prev_gpu = None, None
    ws = None
    if persistent:   # one workspace for the whole rollout, zero-filled once
        ws = torch.zeros(fa.workspace_bytes(fa.OP_COMPRESS, c["H"], c["T"], C, c["r"]), dtype=torch.uint8, device="cuda")
    shift_dir = np.sign(np.random.default_rng(2).standard_normal(c["d"])).astype(np.float32)
    for f in range(n_frames):
        K, V = fs.next_frame()
        if frame_shift:    # the whole frame moves: the joiners of a slot sit together, off the stored key
            K = to_storage((to_f32(K) + frame_shift * f * shift_dir).astype(np.float32), c["dtype"])
        P = fs.queries(1) if probe_queries else None
        mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K, V, P_new=P,
                                                     cand=prev_ref if windowed else None, metric=metric,
                                                     tau2_q16=TAU2(tau), frame_id=f, rep_mode=rep_mode)
        mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dcodec, to_dev(K), to_dev(V),
                                                 P_new=None if P is None else to_dev(P),
                                                 cand=prev_gpu if windowed else None, metric=metric,
                                                 tau2_q16=TAU2(tau), frame_id=f, rep_mode=rep_mode, ws=ws,
                                                 ws_persistent=persistent)
        sync()
        assert np.array_equal(to_host(mg_g), mg_r), f"merged flags, frame {f}"
        assert np.array_equal(to_host(mm_g), mm_r), f"merge map, frame {f}"
        assert np.array_equal(to_host(st_g), st_r), f"stats, frame {f}"
        assert_cache_equal(host_cache(gpu), ref, VTOL[c["dtype"]])
        prev_ref, prev_gpu = mm_r, mm_g
    return c, fs, codec, ref, gpu


def test_tempcache_rollout_cfg1_bit_exact():
    c, fs, codec, ref, gpu = run_rollout("cfg1", 6, 6 * 256, 0.98)
    assert ref.len.max() < 6 * 256 and ref.cnt.max() > 1          # merging did happen


def test_tempcache_eviction_and_drops_bit_exact():
    c, fs, codec, ref, gpu = run_rollout("cfg1", 8, 2 * 256 + 40, 0.98)
    run_rollout("cfg1", 2, 100, 2.0 ** 0.5)                            # capacity below one frame: drops


@pytest.mark.parametrize("C,n_stamps", [(37440, 30), (37440, 1), (37440, 70000), (60000, 300), (1000, 5),
                                        (100000, 300), (100000, 2), (270000, 40)])   # 25 / 66 slots per planning thread
def test_tempcache_eviction_on_a_full_synthetic_cache(C, n_stamps):
    # a full cache with random stamps (many ties, or several significant bytes): one call must evict exactly the
    # oldest untouched slots, lowest slot first on ties, and refill them in ascending slot order
    rng = np.random.default_rng(C + n_stamps)
    H, d, r, T = 2, 64, 32, 300
    codec = make_codec(0, 9, d, r)
    ref = oracle.Cache.empty(H, C, d, r, "fp32")
    ref.K[:] = rng.standard_normal((H, C, d)).astype(np.float32)
    ref.V[:] = rng.standard_normal((H, C, d)).astype(np.float32)
    ref.code[:] = oracle.encode(ref.K, codec.R, codec.qscale, codec.shift)
    ref.cnt[:] = rng.integers(1, 4, size=(H, C))
    ref.stamp[:] = rng.integers(0, n_stamps, size=(H, C)) - (n_stamps // 3)     # negative stamps too
    ref.len[:] = [C, C - 17]
    gpu = dev_cache(ref)
    K_new = rng.standard_normal((H, T, d)).astype(np.float32)
    K_new[:, :100] = ref.K[:, 5:105]                       # a third of the frame duplicates live slots: they merge
    V_new = rng.standard_normal((H, T, d)).astype(np.float32)
    cand = np.broadcast_to(np.arange(0, 400, dtype=np.int32), (H, 400)).copy()
    mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new, V_new, cand=cand,
                                                 tau2_q16=TAU2(0.9), frame_id=10 ** 6)
    mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand),
                                             tau2_q16=TAU2(0.9), frame_id=10 ** 6)
    sync()
    assert st_r[0, 3] > 100 and mg_r[:, :100].all()          # the case does evict and does merge
    assert np.array_equal(to_host(st_g), st_r)
    assert np.array_equal(to_host(mg_g), mg_r)
    assert np.array_equal(to_host(mm_g), mm_r)
    assert_cache_equal(host_cache(gpu), ref, VTOL["fp32"])


@pytest.mark.parametrize("dtype,d,r,n_cand,probe,metric", [
    ("bf16", 128, 32, 700, False, 0), ("bf16", 128, 64, 700, False, 0), ("bf16", 64, 32, 37, False, 1),
    ("bf16", 64, 64, 1000, False, 0), ("fp32", 128, 32, 1000, False, 0), ("fp32", 128, 64, 333, False, 1),
    ("fp32", 64, 32, 2100, False, 0), ("fp32", 64, 64, 64, False, 0),          # window in LDS, probes encoded in-kernel
    ("bf16", 128, 32, 700, True, 1), ("fp32", 64, 64, 1000, True, 0),          # window in LDS, separate probes
    ("bf16", 128, 32, 4000, False, 0), ("fp32", 64, 64, 2500, True, 0),        # window too large for LDS: chunked match
    ("bf16", 128, 64, 0, False, 0), ("fp32", 64, 32, 0, True, 1)])             # no list: every live slot
def test_tempcache_every_match_path_bit_exact(dtype, d, r, n_cand, probe, metric):
    # one call on a random cache: ragged token count, candidate lists with repeats, ids past the live length and -1
    rng = np.random.default_rng(d + r + n_cand)
    H, T, C = 2, 203, 2600
    codec = make_codec(0, 9, d, r)
    as_dt = lambda a: to_storage(a.astype(np.float32), dtype)
    ref = oracle.Cache.empty(H, C, d, r, dtype)
    ref.K[:] = as_dt(rng.standard_normal((H, C, d)))
    ref.K[:, 1000:1400] = ref.K[:, 0:400]                        # repeated keys: equally scored candidates
    ref.K[:, 1500:1600] = ref.K[:, 100:200]
    ref.V[:] = as_dt(rng.standard_normal((H, C, d)))
    ref.code[:] = oracle.encode(ref.K, codec.R, codec.qscale, codec.shift)
    ref.cnt[:] = rng.integers(1, 4, size=(H, C))
    ref.stamp[:] = rng.integers(0, 9, size=(H, C))
    ref.len[:] = [2300, 1999]
    gpu = dev_cache(ref)
    K_new = as_dt(rng.standard_normal((H, T, d)))
    src = rng.integers(0, 1900, size=(H, T))
    for h in range(H):
        K_new[h, :150] = ref.K[h, src[h, :150]]                  # most of the frame repeats live slots
    V_new = as_dt(rng.standard_normal((H, T, d)))
    P_new = as_dt(np.where(rng.random((H, T, 1)) < 0.8, to_f32(K_new), rng.standard_normal((H, T, d)))) if probe else None
    cand = None
    if n_cand:
        cand = rng.integers(0, 2350, size=(H, n_cand)).astype(np.int32)   # some ids are past the live length
        cand[:, : min(150, n_cand)] = src[:, : min(150, n_cand)]
        if n_cand >= 700:                                         # both copies of repeated keys, in shuffled order
            twins = np.concatenate([np.arange(0, 200), np.arange(1000, 1200), np.arange(1500, 1600)])
            for h in range(H):
                cand[h, 200:700] = rng.permutation(twins)
        cand[:, ::17] = -1
        cand[:, 5::29] = cand[:, 4::29][:, : cand[:, 5::29].shape[1]]     # repeated ids
    args = dict(cand=cand, metric=metric, tau2_q16=TAU2(0.9), frame_id=9)
    mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new, V_new, P_new=P_new, **args)
    args["cand"] = None if cand is None else to_dev(cand)
    mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new),
                                             P_new=None if P_new is None else to_dev(P_new), **args)
    sync()
    assert mg_r.sum() > 50                                        # the case does merge
    assert np.array_equal(to_host(mg_g), mg_r)
    assert np.array_equal(to_host(mm_g), mm_r)
    assert np.array_equal(to_host(st_g), st_r)
    assert_cache_equal(host_cache(gpu), ref, VTOL[dtype])


@pytest.mark.parametrize("order,C,n_cand,r", [
    ("ascending", 2600, 900, 32),       # already ascending, every id twice in a row: staged as it stands
    ("descending", 2600, 900, 32),      # sorted the wrong way round
    ("shuffled", 2600, 1800, 64),       # every id twice, far apart
    ("sparse", 300000, 40, 32),         # few ids spread over a long cache: the in-kernel sort needs many passes
    ("sparse", 300000, 700, 64),
    ("long", 9000, 6000, 32),           # list beyond the LDS window: chunked match with full (score, slot) keys
])
def test_tempcache_candidate_list_is_a_set_and_ties_go_to_the_smallest_slot(order, C, n_cand, r):
    # the cache holds every key of its first quarter three more times, so nearly every token has four equally scored
    # candidates; whatever the order and repetition of the list, the match is the smallest listed slot among them
    rng = np.random.default_rng(C + n_cand + r)
    H, T, d = 2, 150, 64
    codec = make_codec(0, 9, d, r)
    ref = oracle.Cache.empty(H, C, d, r, "fp32")
    L = C - 7
    q = L // 4
    base = rng.standard_normal((H, q, d)).astype(np.float32)
    ref.K[:, :L] = rng.standard_normal((H, L, d)).astype(np.float32)
    for k in range(4):
        ref.K[:, k * q:(k + 1) * q] = base
    ref.V[:] = rng.standard_normal((H, C, d)).astype(np.float32)
    ref.code[:] = oracle.encode(ref.K, codec.R, codec.qscale, codec.shift)
    ref.cnt[:] = 1
    ref.stamp[:] = 3
    ref.len[:] = [L, L - 11]
    gpu = dev_cache(ref)
    src = rng.integers(0, q, size=(H, T))
    K_new = np.stack([base[h, src[h]] for h in range(H)])
    V_new = rng.standard_normal((H, T, d)).astype(np.float32)
    uniq = n_cand // 2 if order != "sparse" else n_cand
    cand = np.empty((H, n_cand), np.int32)
    for h in range(H):
        # copies of the tokens' sources from random quarters, filled up with random slots
        n_src = min(T, uniq // 2)
        ids = np.concatenate([src[h][:n_src] + q * rng.integers(0, 4, size=n_src),
                              rng.integers(0, L + 5, size=uniq - n_src)])
        if order == "ascending":
            cand[h] = np.repeat(np.sort(ids), 2)
        elif order == "descending":
            cand[h] = np.repeat(np.sort(ids)[::-1], 2)
        elif order == "sparse":
            cand[h] = rng.permutation(ids)
        else:
            cand[h] = rng.permutation(np.concatenate([ids, ids]))
    cand[:, 7::31] = -1
    args = dict(tau2_q16=TAU2(0.9), frame_id=9)
    mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new, V_new, cand=cand, **args)
    mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand), **args)
    sync()
    assert mg_r.sum() > 10                                        # the case does merge
    assert np.array_equal(to_host(mg_g), mg_r)
    assert np.array_equal(to_host(mm_g), mm_r)
    assert np.array_equal(to_host(st_g), st_r)
    assert_cache_equal(host_cache(gpu), ref, VTOL["fp32"])


@pytest.mark.parametrize("dtype,d,r,H,T,n_cand,persistent", [
    ("bf16", 128, 32, 24, 1501, 3000, True), ("bf16", 128, 32, 24, 1501, 3000, False),
    ("fp32", 64, 64, 22, 1530, 1800, True), ("bf16", 64, 32, 26, 1300, 3500, True)])
def test_tempcache_many_workgroups_take_the_wide_window_kernel(dtype, d, r, H, T, n_cand, persistent):
    # more than two rounds of 64-token workgroups over the chip with a window that fills a compute unit's LDS: the
    # launcher takes the instantiation with 256 tokens per workgroup (ragged last workgroup, shuffled lists with
    # repeats and dead ids, repeated keys, two calls on one workspace)
    rng = np.random.default_rng(d + r + H + n_cand)
    C = 5000
    codec = make_codec(0, 9, d, r)
    as_dt = lambda a: to_storage(a.astype(np.float32), dtype)
    ref = oracle.Cache.empty(H, C, d, r, dtype)
    ref.K[:] = as_dt(rng.standard_normal((H, C, d)))
    ref.K[:, 2000:2600] = ref.K[:, 0:600]                        # repeated keys: equally scored candidates
    ref.V[:] = as_dt(rng.standard_normal((H, C, d)))
    ref.code[:] = oracle.encode(ref.K, codec.R, codec.qscale, codec.shift)
    ref.cnt[:] = rng.integers(1, 4, size=(H, C))
    ref.stamp[:] = rng.integers(0, 9, size=(H, C))
    ref.len[:] = rng.integers(3800, 4400, size=H)
    gpu = dev_cache(ref)
    ws = torch.zeros(fa.workspace_bytes(fa.OP_COMPRESS, H, T, C, r), dtype=torch.uint8, device="cuda")
    cand = None
    for f in (9, 10):
        K_new = as_dt(rng.standard_normal((H, T, d)))
        src = rng.integers(0, 3700, size=(H, T))
        for h in range(H):
            K_new[h, :1000] = ref.K[h, src[h, :1000]]             # most of the frame repeats live slots
        V_new = as_dt(rng.standard_normal((H, T, d)))
        if cand is None:
            cand = rng.integers(0, 4500, size=(H, n_cand)).astype(np.int32)
            cand[:, :1000] = src[:, :1000]
            cand[:, 1000:1400] = rng.integers(2000, 2600, size=(H, 400))
            cand[:, ::19] = -1
            cand = np.stack([row[rng.permutation(n_cand)] for row in cand])
        args = dict(tau2_q16=TAU2(0.9), frame_id=f)
        mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new, V_new, cand=cand, **args)
        mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand),
                                                 ws=ws, ws_persistent=persistent, **args)
        sync()
        assert mg_r.sum() > 100 * H
        assert np.array_equal(to_host(st_g), st_r), f"stats, frame {f}"
        assert np.array_equal(to_host(mg_g), mg_r), f"merged flags, frame {f}"
        assert np.array_equal(to_host(mm_g), mm_r), f"merge map, frame {f}"
        assert_cache_equal(host_cache(gpu), ref, VTOL[dtype])
        cand = np.ascontiguousarray(np.concatenate([mm_r, mm_r[:, : n_cand - T]], axis=1)[:, :n_cand])


@pytest.mark.parametrize("path,H,T,C,persistent", [
    ("own_histogram", 2, 700, 16 * 256 * 17, True),    # long cache: the plan's workgroups meet for the age histogram
    ("general", 3, 300, 4 * 2048, False),              # a stamp in the future: the general path, three meetings
])
def test_tempcache_plan_that_gives_up_leaves_the_cache_untouched_and_says_so(path, H, T, C, persistent):
    # The eviction plan's workgroups wait for each other through global memory, bounded.  The test hook makes those
    # waits run out (they expect one arrival more than will ever come, for 50 polls): the call must finish, report
    # status 1 for every head, apply nothing (cache bit for bit as before, every token reported dropped), and the same
    # call on a fresh workspace with the normal waits must equal the oracle.
    rng = np.random.default_rng(C + T)
    d, r, dtype = 128, 32, "bf16"
    codec = make_codec(0, 9, d, r)
    as_dt = lambda a: to_storage(a.astype(np.float32), dtype)
    ref = oracle.Cache.empty(H, C, d, r, dtype)
    ref.K[:] = as_dt(rng.standard_normal((H, C, d)))
    ref.V[:] = as_dt(rng.standard_normal((H, C, d)))
    ref.code[:] = oracle.encode(ref.K, codec.R, codec.qscale, codec.shift)
    ref.cnt[:] = rng.integers(1, 4, size=(H, C))
    ref.stamp[:] = rng.integers(0, 9, size=(H, C))
    if path == "general":
        ref.stamp[:, 17] = 40                                      # above the call's frame id
    ref.len[:] = C                                                 # full: every unmerged token needs a victim
    gpu = dev_cache(ref)
    before = host_cache(gpu)
    K_new = as_dt(rng.standard_normal((H, T, d)))
    src = rng.integers(0, C, size=(H, T))
    for h in range(H):
        K_new[h, : T // 2] = ref.K[h, src[h, : T // 2]]            # half of the frame repeats live slots
    V_new = as_dt(rng.standard_normal((H, T, d)))
    cand = np.ascontiguousarray(src[:, rng.permutation(T)]).astype(np.int32)
    args = dict(tau2_q16=TAU2(0.9), frame_id=9)
    n_ws = fa.workspace_bytes(fa.OP_COMPRESS, H, T, C, r)
    ws = torch.zeros(n_ws, dtype=torch.uint8, device="cuda")
    fa.debug_plan_wait(50, 1)
    try:
        mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand),
                                                 ws=ws, ws_persistent=persistent, **args)
        sync()
    finally:
        fa.debug_plan_wait(-1, 0)
    st = to_host(st_g)
    assert (st[:, 7] == 1).all() and (st[:, 0] == C).all() and (st[:, 4] == T).all() and (st[:, 1:4] == 0).all()
    assert (to_host(mm_g) == -1).all() and (to_host(mg_g) == 0).all()
    after = host_cache(gpu)
    for name in ("K", "V", "code", "cnt", "stamp", "len"):
        assert np.array_equal(getattr(after, name), getattr(before, name)), name
    # the same call with the normal waits, on a fresh workspace
    ws2 = torch.zeros(n_ws, dtype=torch.uint8, device="cuda")
    mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new, V_new, cand=cand, **args)
    mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand),
                                             ws=ws2, ws_persistent=persistent, **args)
    sync()
    assert (st_r[:, 3] > 0).all() and (st_r[:, 7] == 0).all() and mg_r.sum() > H * T // 4      # evictions and merges
    assert np.array_equal(to_host(st_g), st_r) and np.array_equal(to_host(mg_g), mg_r) and np.array_equal(to_host(mm_g), mm_r)
    assert_cache_equal(host_cache(gpu), ref, VTOL[dtype])
    if persistent:   # the workspace of the call that gave up is not clean: a further call on it says so and applies nothing
        _, _, st3 = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand),
                                          ws=ws, ws_persistent=True, tau2_q16=TAU2(0.9), frame_id=10)
        sync()
        assert (to_host(st3)[:, 7] != 0).all()
        assert_cache_equal(host_cache(gpu), ref, VTOL[dtype])


@pytest.mark.parametrize("name,dtype,H,frames,C", [("cfg1", None, None, 6, 6 * 256), ("cfg1", "bf16", None, 6, 3 * 256),
                                                   ("cfg2", None, 2, 4, 3 * 1560)])
def test_tempcache_mean_key_representative_bit_exact(name, dtype, H, frames, C):
    # the stored mean key decides later codes, matches and cosine tests: every frame of the rollout must agree bit for
    # bit (assert_cache_equal compares keys and codes exactly), through merges of several tokens per slot and evictions
    c, fs, codec, ref, gpu = run_rollout(name, frames, C, 0.98, dtype=dtype, H=H, rep_mode=fa.REP_MEAN)
    assert ref.cnt.max() >= 4


@pytest.mark.parametrize("name,dtype,H,frames,C,tau,fshift,r", [
    ("cfg1", None, None, 5, 2 * 256, 0.6, 0.3, None),      # big groups that move: the medoid is often a joiner
    ("cfg1", "bf16", None, 5, 2 * 256, 0.6, 0.3, 64),      # the same with 64-byte codes in bf16
    ("cfg1", None, None, 6, 6 * 256, 0.98, 0.0, None),     # single joiners: the stored key always stays
    ("cfg2", None, 2, 4, 3 * 1560, 0.9, 0.1, None)])
def test_tempcache_medoid_key_representative_bit_exact(name, dtype, H, frames, C, tau, fshift, r):
    # appendix ablation, medoid key: weighted medoid in code space, exact integers, so everything is bit-exact
    c, fs, codec, ref, gpu = run_rollout(name, frames, C, tau, dtype=dtype, H=H, rep_mode=2, frame_shift=fshift, r=r,
                                         persistent=True)
    assert int(ref.cnt.max()) >= 3


def test_tempcache_mean_key_with_many_joiners_per_slot():
    # low threshold on the clustered stream: whole clusters fold into single slots, so slots take many joiners per call
    c, fs, codec, ref, gpu = run_rollout("cfg1", 4, 5 * 256, 0.5, rep_mode=fa.REP_MEAN)
    assert ref.cnt.max() > 8


@pytest.mark.parametrize("T,C,lens,n_cand,tau", [
    (1, 300, [200, 0], 50, 0.9),           # a single token per head; one head still empty
    (5000, 6000, [800, 799], 900, 0.9),    # more tokens than the plan keeps in registers, most of them appended
    (300, 77, [77, 60], 64, 0.9),          # capacity far below one frame: evictions and drops
    (64, 512, [300, 300], 128, 0.9),       # exactly one workgroup of tokens
    (200, 512, [100, 250], -1, 0.9),       # every candidate id invalid: nothing can match
    (200, 512, [0, 0], 100, 0.9),          # empty cache with a (stale) candidate list
    (130, 4096, [4096, 4000], 3776, 0.5),  # the largest window that is staged in LDS, loose threshold: big groups
])
def test_tempcache_edge_shapes_bit_exact(T, C, lens, n_cand, tau):
    rng = np.random.default_rng(T + C + n_cand)
    H, d, r = 2, 64, 32
    codec = make_codec(0, 9, d, r)
    ref = oracle.Cache.empty(H, C, d, r, "fp32")
    ref.K[:] = rng.standard_normal((H, C, d)).astype(np.float32)
    ref.V[:] = rng.standard_normal((H, C, d)).astype(np.float32)
    ref.code[:] = oracle.encode(ref.K, codec.R, codec.qscale, codec.shift)
    ref.cnt[:] = rng.integers(1, 4, size=(H, C))
    ref.stamp[:] = rng.integers(0, 5, size=(H, C))
    ref.len[:] = lens
    gpu = dev_cache(ref)
    K_new = rng.standard_normal((H, T, d)).astype(np.float32)
    lo = max(min(lens), 1)
    src = rng.integers(0, lo, size=(H, T))
    for h in range(H):
        if lens[h] > 0:
            K_new[h, : (2 * T) // 3] = ref.K[h, src[h, : (2 * T) // 3]] + 0.01 * rng.standard_normal(((2 * T) // 3, d)).astype(np.float32)
    V_new = rng.standard_normal((H, T, d)).astype(np.float32)
    if n_cand < 0:
        cand = np.full((H, 40), -1, np.int32)
        cand[:, ::2] = C + 5
    else:
        cand = rng.integers(0, max(max(lens), 1), size=(H, n_cand)).astype(np.int32)
        k = min(n_cand, T)
        cand[:, :k] = src[:, :k]
    mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new, V_new, cand=cand,
                                                 tau2_q16=TAU2(tau), frame_id=7)
    mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K_new), to_dev(V_new), cand=to_dev(cand),
                                             tau2_q16=TAU2(tau), frame_id=7)
    sync()
    assert np.array_equal(to_host(st_g), st_r)
    assert np.array_equal(to_host(mg_g), mg_r)
    assert np.array_equal(to_host(mm_g), mm_r)
    assert_cache_equal(host_cache(gpu), ref, VTOL["fp32"])


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_tempcache_on_seeded_random_shapes(seed):
    """Eight random configurations per seed (storage type, head and code width, frame size, capacity from below one
    frame to many, threshold, metric, representative, candidate list or whole cache), three frames each on one cache:
    frames repeat earlier tokens with a little noise, so calls merge, append, evict and drop in mixtures.  Bookkeeping
    bit-exact after every frame."""
    rng = np.random.default_rng(200 + seed)
    for case in range(8):
        dtype, d, r = str(rng.choice(["fp32", "bf16"])), int(rng.choice([64, 128])), int(rng.choice([32, 64]))
        H, T = int(rng.integers(1, 4)), int(rng.integers(1, 700))
        C = int(rng.integers(max(T // 2, 1), 5 * T + 64))
        tau, metric = float(rng.choice([0.5, 0.9, 0.98])), int(rng.integers(0, 2))
        rep_mode = int(rng.integers(0, 2))
        windowed = rng.random() < 0.7
        what = f"seed {seed} case {case}: {dtype} d={d} r={r} H={H} T={T} C={C} tau={tau} metric={metric} rep={rep_mode} windowed={windowed}"
        codec = make_codec(seed, case, d, r)
        ref = oracle.Cache.empty(H, C, d, r, dtype)
        gpu = dev_cache(ref)
        dcodec = dev_codec(codec)
        pool = rng.standard_normal((H, T, d)).astype(np.float32)            # the tokens every frame drifts from
        prev_ref = prev_gpu = None
        for f in range(3):
            fresh = rng.random((H, T, 1)) < 0.3
            K = np.where(fresh, rng.standard_normal((H, T, d)), pool + 0.02 * rng.standard_normal((H, T, d)))
            K, V = to_storage(K.astype(np.float32), dtype), to_storage(rng.standard_normal((H, T, d)).astype(np.float32), dtype)
            use = windowed and prev_ref is not None
            mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K, V,
                                                         cand=prev_ref if use else None, metric=metric,
                                                         tau2_q16=TAU2(tau), frame_id=f, rep_mode=rep_mode)
            mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dcodec, to_dev(K), to_dev(V), cand=prev_gpu if use else None,
                                                     metric=metric, tau2_q16=TAU2(tau), frame_id=f, rep_mode=rep_mode)
            sync()
            assert np.array_equal(to_host(st_g), st_r), f"{what}: stats, frame {f}"
            assert np.array_equal(to_host(mg_g), mg_r), f"{what}: merged flags, frame {f}"
            assert np.array_equal(to_host(mm_g), mm_r), f"{what}: merge map, frame {f}"
            assert_cache_equal(host_cache(gpu), ref, VTOL[dtype])
            prev_ref, prev_gpu = mm_r, mm_g


@pytest.mark.parametrize("name,dtype,H,frames,C,tau,rep", [
    ("cfg1", None, None, 6, 6 * 256, 0.98, 0), ("cfg1", "bf16", None, 8, 2 * 256 + 40, 0.98, 0),
    ("cfg2", None, 2, 5, 3 * 1560, 0.98, 0), ("cfg1", None, None, 4, 5 * 256, 0.5, 1), ("cfg1", None, None, 2, 100, 2.0 ** 0.5, 0)])
def test_tempcache_rollout_on_a_persistent_workspace(name, dtype, H, frames, C, tau, rep):
    # the workspace is zero-filled once and every call leaves it clean: the match launch goes straight on to the
    # threshold test (no clearing launch); merges, big groups, evictions and drops must come out bit for bit the same
    c, fs, codec, ref, gpu = run_rollout(name, frames, C, tau, dtype=dtype, H=H, rep_mode=rep, persistent=True)


@pytest.mark.parametrize("shift", [4, 6, 8, 9])
def test_code_precision_ladder_rollout_and_selection_bit_exact(shift):
    # appendix ablation "Quantization precision for ANN matching": every code precision that the benchmark reports
    # (bench.py --code-shift) runs the whole index path here: TempCache rollout (match, threshold, evictions: the
    # coarser the codes, the more equally scored candidates), query codes, AnnSA and AnnCA selections
    c, fs, codec, ref, gpu = run_rollout("cfg1", 6, 4 * 256, 0.98, dtype="bf16", persistent=True, shift=shift)
    Q = fs.queries(1)
    qc_r = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    qc = fa.encode(to_dev(Q), dev_codec(codec))
    assert np.array_equal(to_host(qc), qc_r)
    sel_r, nsel_r = oracle.ann_select_self(qc_r, ref.code, ref.len, c["BQ"], c["n_rep"], c["BK"], 5)
    sel, nsel = fa.ann_select_self(qc, gpu.code, gpu.len, c["BQ"], c["n_rep"], c["BK"], 5)
    assert np.array_equal(to_host(sel), sel_r) and np.array_equal(to_host(nsel), nsel_r)
    pk = to_storage(np.random.default_rng(shift).standard_normal((c["H"], 96, c["d"])).astype(np.float32), "bf16")
    pc_r = oracle.encode(pk, codec.R, codec.qscale, codec.shift)
    pc = fa.encode(to_dev(pk), dev_codec(codec))
    assert np.array_equal(to_host(pc), pc_r)
    csel_r, cnsel_r = oracle.ann_select_cross(qc_r, pc_r, c["BQ"], 16)
    csel, cnsel = fa.ann_select_cross(qc, pc, c["BQ"], 16)
    assert np.array_equal(to_host(csel), csel_r) and np.array_equal(to_host(cnsel), cnsel_r)


@pytest.mark.parametrize("dtype,persistent", [("fp32", True), ("bf16", True), ("bf16", False)])
def test_tempcache_rollout_with_64_byte_codes(dtype, persistent):
    # r = 64: the window kernel's largest instantiations (most static LDS), with and without the fused threshold test
    run_rollout("cfg1", 5, 4 * 256, 0.98, dtype=dtype, persistent=persistent, r=64)


def test_tempcache_persistent_workspace_mixes_with_the_other_paths_and_reports_a_dirty_one():
    # first frame without a candidate list (chunked match), then windowed frames, all on one persistent workspace
    c = dict(CONFIGS["cfg1"])
    fs = FrameStream(c["seed"], c["cfg_id"], c["H"], c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
    codec = make_codec(c["seed"], c["cfg_id"], c["d"], c["r"])
    C = 5 * c["T"]
    ref = oracle.Cache.empty(c["H"], C, c["d"], c["r"], c["dtype"])
    gpu = dev_cache(ref)
    ws = torch.zeros(fa.workspace_bytes(fa.OP_COMPRESS, c["H"], c["T"], C, c["r"]), dtype=torch.uint8, device="cuda")
    prev_r = prev_g = None
    for f in range(4):
        K, V = fs.next_frame()
        P = fs.queries(1) if f == 2 else None                    # one frame with separate probes in between
        mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K, V, P_new=P, cand=prev_r,
                                                     tau2_q16=TAU2(0.98), frame_id=f)
        mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K), to_dev(V),
                                                 P_new=None if P is None else to_dev(P), cand=prev_g,
                                                 tau2_q16=TAU2(0.98), frame_id=f, ws=ws, ws_persistent=True)
        sync()
        assert np.array_equal(to_host(mm_g), mm_r) and np.array_equal(to_host(st_g), st_r), f"frame {f}"
        assert_cache_equal(host_cache(gpu), ref, VTOL[c["dtype"]])
        prev_r, prev_g = mm_r, mm_g
    # a workspace that is neither zero-filled nor left by a finished call is reported (cache far from full: no eviction)
    K, V = fs.next_frame()
    dirty = torch.full_like(ws, 0x5B)
    _, _, st = fa.tempcache_compress(gpu, dev_codec(codec), to_dev(K), to_dev(V), cand=prev_g, tau2_q16=TAU2(0.98),
                                     frame_id=9, ws=dirty, ws_persistent=True)
    sync()
    assert (to_host(st)[:, 7] == 3).all()


def test_tempcache_whole_cache_match_and_inner_product_probe():
    run_rollout("cfg1", 4, 5 * 256, 0.9, windowed=False)
    run_rollout("cfg1", 4, 5 * 256, 0.9, windowed=True, metric=1, probe_queries=True)


def test_tempcache_bf16_wan_shaped_heads():
    # two heads of the Wan-shaped layer: 1560 tokens per frame (not a multiple of any tile), d = 128
    c, fs, codec, ref, gpu = run_rollout("cfg2", 4, 4 * 1560, 0.98, H=2)
    assert 0.7 < 1 - (ref.len[0] - 1560) / (3 * 1560) < 0.9            # about p = 0.8 of each frame merges


def test_tempcache_then_select_then_attend_end_to_end_cfg1():
    c, fs, codec, ref, gpu = run_rollout("cfg1", 5, 5 * 256, 0.98)
    Q = fs.queries(1)
    dcodec = dev_codec(codec)
    qc_ref = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    qc = fa.encode(to_dev(Q), dcodec)
    assert np.array_equal(to_host(qc), qc_ref)
    n_sel = 5
    sel_r, nsel_r = oracle.ann_select_self(qc_ref, ref.code, ref.len, 128, 4, 64, n_sel)
    sel, nsel = fa.ann_select_self(qc, gpu.code, gpu.len, 128, 4, 64, n_sel)
    assert np.array_equal(to_host(sel), sel_r) and np.array_equal(to_host(nsel), nsel_r)
    O_ref, _ = oracle.sparse_attn_fwd(Q, ref.K, ref.V, ref.cnt, ref.len, sel_r, nsel_r, 128, 64, c["d"] ** -0.5)
    O, _ = fa.sparse_attn_fwd(to_dev(Q), gpu.K, gpu.V, gpu.cnt, gpu.len, sel, nsel, 128, 64, c["d"] ** -0.5)
    assert np.abs(to_host(O).astype(np.float64) - O_ref).max() <= 1e-4
    # cross-attention leg
    ps = PromptSet(c["seed"], c["cfg_id"], fs.centreK, c["n_p"], c["n_pc"], c["n_near"], c["dtype"])
    pc_ref = oracle.encode(ps.K, codec.R, codec.qscale, codec.shift)
    pc = fa.encode(to_dev(ps.K), dcodec)
    csel_r, cnsel_r = oracle.ann_select_cross(qc_ref, pc_ref, 128, c["n_sel_cross"])
    csel, cnsel = fa.ann_select_cross(qc, pc, 128, c["n_sel_cross"])
    assert np.array_equal(to_host(csel), csel_r) and np.array_equal(to_host(cnsel), cnsel_r)
    n_p = c["n_p"]
    plen = np.full(c["H"], n_p, np.int32)
    O_ref, _ = oracle.sparse_attn_fwd(Q, ps.K, ps.V, None, plen, csel_r, cnsel_r, 128, 1, c["d"] ** -0.5)
    O, _ = fa.sparse_attn_fwd(to_dev(Q), to_dev(ps.K), to_dev(ps.V), None, to_dev(plen), csel, cnsel, 128, 1,
                              c["d"] ** -0.5)
    assert np.abs(to_host(O).astype(np.float64) - O_ref).max() <= 1e-4


@pytest.mark.parametrize("BQ", [128, 64])
def test_attention_with_logits_that_keep_growing_along_the_key_list(BQ):
    """The bf16 d = 128 kernels follow the running maximum lazily (the reference of the exponentials moves only
    when a score exceeds it by a margin); keys whose scores climb steadily, by less and by more than that margin
    per tile, must give the same softmax as the oracle's plain definition."""
    rng = np.random.default_rng(77)
    H, n_q, C, d, BK = 2, 256, 64 * 24, 128, 64
    base = rng.standard_normal((H, 1, d)).astype(np.float32)
    Q = to_storage(base + 0.3 * rng.standard_normal((H, n_q, d)).astype(np.float32), "bf16")
    ramp = np.linspace(0.0, 1.0, C, dtype=np.float32)[None, :, None]
    ramp = np.where(np.arange(C)[None, :, None] < C // 2, 0.25 * ramp, ramp * ramp * 3.0)    # slow, then fast
    K = to_storage(base * ramp + 0.3 * rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
    V = to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16")
    length = np.full((H,), C, np.int32)
    cnt = rng.integers(1, 5, size=(H, C)).astype(np.int32)
    n_qb, n_sel = n_q // BQ, C // BK
    sel = np.tile(np.arange(n_sel, dtype=np.int32), (H, n_qb, 1))
    sel[1] = sel[1, :, ::-1]                                         # head 1 meets the largest scores first
    nsel = np.full((H, n_qb), n_sel, np.int32)
    for scale in (d ** -0.5, 4.0 * d ** -0.5):
        check_attention(Q, K, V, cnt, length, sel, nsel, BQ, BK, scale, "bf16")


# ----------------------------------------------------------------------------------------- argument checks

# ----------------------------------------------------------------------------------------- HIP graph

def test_selection_and_attention_replay_from_a_hip_graph():
    """No entry point allocates, synchronises or clears memory with a memset, so a chunk's calls can be captured once
    and replayed.  Every replay (different queries each time, eager work and synchronisations in between) must
    reproduce the eager result bit for bit."""
    H, n_q, C, d, r, BQ, BK, n_rep, n_sel, n_p, n_sel_x = 3, 640, 64 * 40, 128, 32, 128, 64, 4, 9, 256, 64
    rng = np.random.default_rng(5)
    codec = make_codec(11, 2, d, r)
    dcodec = dev_codec(codec)
    K = to_dev(to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16"))
    V = to_dev(to_storage(rng.standard_normal((H, C, d)).astype(np.float32), "bf16"))
    Kp = to_dev(to_storage(rng.standard_normal((H, n_p, d)).astype(np.float32), "bf16"))
    Vp = to_dev(to_storage(rng.standard_normal((H, n_p, d)).astype(np.float32), "bf16"))
    cnt = to_dev(rng.integers(1, 6, size=(H, C)).astype(np.int32))
    length = to_dev(np.array([C, C - 100, 64 * 7 + 3], np.int32))
    kcode = fa.encode(K, dcodec)
    pcode = fa.encode(Kp, dcodec)
    Qs = [to_dev(to_storage(rng.standard_normal((H, n_q, d)).astype(np.float32), "bf16")) for _ in range(3)]
    n_qb = n_q // BQ
    dev = "cuda"

    def buffers():
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        return dict(qcode=e((H, n_q, r), torch.int8), sel=(e((H, n_qb, n_sel), torch.int32), e((H, n_qb), torch.int32)),
                    O=(e((H, n_q, d), torch.bfloat16), e((H, n_q), torch.float32)),
                    X=(e((H, n_qb, n_sel_x), torch.int32), e((H, n_qb), torch.int32), e((H, n_q, d), torch.bfloat16)),
                    ws=e((fa.workspace_bytes(fa.OP_SELECT_SELF, H, n_q, C, r, BQ, BK, n_rep),), torch.uint8))

    def calls(Q, b):
        fa.encode(Q, dcodec, out=b["qcode"])
        fa.ann_select_self(b["qcode"], kcode, length, BQ, n_rep, BK, n_sel, ws=b["ws"], out=b["sel"])
        fa.sparse_attn_fwd(Q, K, V, cnt, length, b["sel"][0], b["sel"][1], BQ, BK, d ** -0.5, out=b["O"])
        fa.ann_cross_attn_fwd(Q, b["qcode"], Kp, Vp, pcode, BQ, n_sel_x, d ** -0.5, out=b["X"])

    eager = []
    for Q in Qs:
        b = buffers()
        calls(Q, b)
        sync()
        eager.append(b)
    Qg = torch.empty_like(Qs[0])
    g_buf = buffers()
    Qg.copy_(Qs[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # one run outside the capture, on a side stream
        calls(Qg, g_buf)
    torch.cuda.current_stream().wait_stream(side)
    sync()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls(Qg, g_buf)
    for rep in range(2):
        for i, Q in enumerate(Qs):
            Qg.copy_(Q)                      # eager work between the replays
            for t in g_buf["O"] + g_buf["X"] + g_buf["sel"]:
                t.zero_()
            sync()
            graph.replay()
            sync()
            ref = eager[i]
            for name in ("sel", "O", "X"):
                for a, b_ in zip(g_buf[name], ref[name]):
                    assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                                       b_.view(torch.int16) if b_.dtype == torch.bfloat16 else b_), (rep, i, name)


def test_tempcache_frames_replayed_from_hip_graphs():
    """Each frame's compress call captured in a graph of its own and run by replaying it (persistent workspace,
    preallocated outputs): state and outputs as the oracle's, frame after frame, through merging and eviction."""
    c = dict(CONFIGS["cfg1"])
    C, tau, n_frames = 2 * c["T"] + 40, 0.98, 8
    fs = FrameStream(c["seed"], c["cfg_id"], c["H"], c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
    codec = make_codec(c["seed"], c["cfg_id"], c["d"], c["r"])
    ref = oracle.Cache.empty(c["H"], C, c["d"], c["r"], c["dtype"])
    gpu = dev_cache(ref)
    dcodec = dev_codec(codec)
    ws = torch.zeros(fa.workspace_bytes(fa.OP_COMPRESS, c["H"], c["T"], C, c["r"]), dtype=torch.uint8, device="cuda")
    outs = [(torch.empty((c["H"], c["T"]), dtype=torch.int32, device="cuda"),
             torch.empty((c["H"], c["T"]), dtype=torch.uint8, device="cuda"),
             torch.empty((c["H"], 8), dtype=torch.int32, device="cuda")) for _ in range(2)]
    prev_ref, prev_gpu = None, None
    evicted = 0
    for f in range(n_frames):
        K, V = fs.next_frame()
        mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K, V, cand=prev_ref,
                                                     tau2_q16=TAU2(tau), frame_id=f)
        Kd, Vd = to_dev(K), to_dev(V)
        out = outs[f & 1]
        sync()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fa.tempcache_compress(gpu, dcodec, Kd, Vd, cand=prev_gpu, tau2_q16=TAU2(tau), frame_id=f, ws=ws, out=out,
                                  ws_persistent=True)
        graph.replay()
        sync()
        assert np.array_equal(to_host(out[1]), mg_r), f"merged flags, frame {f}"
        assert np.array_equal(to_host(out[0]), mm_r), f"merge map, frame {f}"
        assert np.array_equal(to_host(out[2]), st_r), f"stats, frame {f}"
        assert_cache_equal(host_cache(gpu), ref, VTOL[c["dtype"]])
        evicted += int(st_r[:, 3].sum())
        prev_ref, prev_gpu = mm_r, out[0]
    assert evicted > 0, "the rollout was meant to reach eviction"


def test_bad_arguments_are_rejected_on_the_host():
    q = torch.zeros((1, 128, 32), dtype=torch.int8, device="cuda")
    k = torch.zeros((1, 256, 32), dtype=torch.int8, device="cuda")
    length = torch.full((1,), 256, dtype=torch.int32, device="cuda")
    with pytest.raises(fa.FastarError, match="invalid"):
        fa.ann_select_self(q, k, length, 128, 3, 64, 2)              # BQ not a multiple of n_rep
    with pytest.raises(fa.FastarError, match="unsupported"):
        fa.ann_select_self(q, k, length, 128, 4, 48, 2)              # BK not a multiple of 32
    with pytest.raises(fa.FastarError, match="workspace"):
        fa.ann_select_self(q, k, length, 128, 4, 64, 2, ws=torch.empty(256, dtype=torch.uint8, device="cuda"))
    Q = torch.zeros((1, 128, 96), dtype=torch.bfloat16, device="cuda")
    sel = torch.zeros((1, 1, 2), dtype=torch.int32, device="cuda")
    nsel = torch.zeros((1, 1), dtype=torch.int32, device="cuda")
    with pytest.raises(fa.FastarError, match="unsupported"):
        fa.sparse_attn_fwd(Q, Q, Q, None, length, sel, nsel, 128, 64, 0.1)   # d = 96
    Q = torch.zeros((1, 128, 128), dtype=torch.bfloat16, device="cuda")
    for bad_scale in (0.0, -0.1, float("inf"), float("nan")):
        with pytest.raises(fa.FastarError, match="invalid"):
            fa.sparse_attn_fwd(Q, Q, Q, None, length, sel, nsel, 128, 64, bad_scale)
    with pytest.raises(fa.FastarError, match="unsupported"):
        fa.sparse_attn_fwd(Q, Q, Q, None, length, sel, nsel, 128, 48, 0.1)    # bf16: BK no power of two
    with pytest.raises(fa.FastarError, match="unsupported"):
        fa.sparse_attn_fwd(Q, Q, Q, None, length, sel, nsel, 96, 64, 0.1)     # bf16: BQ neither 64 nor 128
    Qf = torch.zeros((1, 128, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(fa.FastarError, match="unsupported"):
        fa.sparse_attn_fwd(Qf, Qf, Qf, None, length, sel, nsel, 128, 96, 0.1)  # fp32: BK beyond 64
    with pytest.raises(fa.FastarError, match="unsupported"):
        fa.sparse_attn_fwd(Qf, Qf, Qf, None, length, sel, nsel, 256, 64, 0.1)  # fp32: BQ beyond 128


# ----------------------------------------------------------------------------------------- persistent attention

@pytest.mark.parametrize("H,n_q,C,n_sel,lens_cut,with_cnt", [
    (20, 3600, 64 * 400, 200, 0, True),      # 580 query blocks, ragged last block of every head, shares of 226.6 tiles
    (9, 7700, 64 * 300, 150, 1, True),       # 549 blocks; one head short, one empty: lists shorter than the share arithmetic assumes
    (33, 2048, 64 * 256, 128, 0, False),     # 528 blocks, no multiplicities
])
def test_persistent_attention_matches_the_oracle_and_the_plain_launch(H, n_q, C, n_sel, lens_cut, with_cnt):
    # sparse_attn_fwd_ws splits the launch here (more query blocks than the chip holds at once, a short last round): the
    # query blocks left over by the whole rounds go to the persistent kernel in equal shares of their tiles, blocks cut by
    # share boundaries are combined from fragments.  Oracle on sampled (head, query block) pairs incl. cut and whole ones.
    rng = np.random.default_rng(H + n_q)
    g = torch.Generator(device="cuda").manual_seed(H * 1000 + n_sel)
    Q = torch.randn(H, n_q, 128, device="cuda", generator=g).bfloat16()
    K = torch.randn(H, C, 128, device="cuda", generator=g).bfloat16()
    V = torch.randn(H, C, 128, device="cuda", generator=g).bfloat16()
    Q[:, ::7] *= 3.0                                           # some peaked rows
    cnt = torch.randint(1, 6, (H, C), device="cuda", generator=g, dtype=torch.int32) if with_cnt else None
    lens = np.full(H, C, np.int32)
    if lens_cut:
        lens[3], lens[5] = C // 3 + 17, 0
    n_qb, n_kb = -(-n_q // 128), C // 64
    sel = np.stack([np.stack([np.sort(rng.choice(n_kb, n_sel, replace=False)) for _ in range(n_qb)]) for _ in range(H)]).astype(np.int32)
    nsel = np.full((H, n_qb), n_sel, np.int32)
    nsel[0, 1], nsel[1, 0] = n_sel // 3, 0                     # short and empty lists
    sel[0, 1, n_sel // 3:] = -1
    sel[1, 0, :] = -1
    ws = torch.empty(fa.workspace_bytes(fa.OP_ATTN, H, n_q, C), dtype=torch.uint8, device="cuda")
    args = (Q, K, V, cnt, to_dev(lens), to_dev(sel), to_dev(nsel), 128, 64, 128 ** -0.5)
    O_ws, lse_ws = fa.sparse_attn_fwd(*args, ws=ws)
    O_pl, lse_pl = fa.sparse_attn_fwd(*args)
    sync()
    O_ws_h, O_pl_h = to_host(O_ws), to_host(O_pl)
    assert np.abs(to_f32(O_ws_h).astype(np.float64) - to_f32(O_pl_h)).max() <= 2e-2
    lw, lp = to_host(lse_ws), to_host(lse_pl)
    fin = np.isfinite(lp)
    assert np.array_equal(fin, np.isfinite(lw)) and np.abs(lw[fin] - lp[fin]).max() <= 1e-2   # sums of rounded P against different references
    # the oracle on a sample of blocks: the first ones, the special ones, and blocks around share boundaries
    NT = n_sel
    total = n_qb * H
    per = -(-total // 8)
    tail_per = per % 64
    assert per > 64 and 0 < tail_per <= 24, "the shape is meant to take the split launch"
    W = 8 * tail_per * NT
    to_item = lambda vi: (vi // tail_per) * per + (per - tail_per) + vi % tail_per   # position in the left-over sequence -> pair
    cut_items = sorted({to_item((i * W // 512) // NT) for i in range(1, 512) if (i * W // 512) % NT} - set(range(total, 8 * per)))
    whole_tail = sorted({to_item(vi) for vi in range(8 * tail_per)} - set(cut_items) - set(range(total, 8 * per)))
    sample = sorted(set([0, 1, n_qb, n_qb - 1, total - 1] + cut_items[:3] + cut_items[-2:] + [cut_items[len(cut_items) // 2]] + whole_tail[:1]))
    Kh, Vh, Qh = to_host(K), to_host(V), to_host(Q)
    cnt_h = to_host(cnt) if with_cnt else None
    for item in sample:
        h, b = divmod(item, n_qb)
        q0, q1 = b * 128, min((b + 1) * 128, n_q)
        O_r, lse_r = oracle.sparse_attn_fwd(Qh[h:h + 1, q0:q1], Kh[h:h + 1], Vh[h:h + 1], None if cnt_h is None else cnt_h[h:h + 1],
                                            lens[h:h + 1], sel[h:h + 1, b:b + 1], nsel[h:h + 1, b:b + 1], 128, 64, 128 ** -0.5)
        err = np.abs(to_f32(O_ws_h[h, q0:q1]).astype(np.float64) - O_r[0]).max()
        assert err <= ATOL["bf16"], f"item {item}: {err}"
        lr = lse_r[0]
        ok = np.isfinite(lr)
        assert np.array_equal(ok, np.isfinite(lw[h, q0:q1])) and np.abs(lw[h, q0:q1][ok] - lr[ok]).max(initial=0.0) <= 2e-2


def test_attention_with_a_workspace_runs_small_shapes_as_before_and_rejects_a_short_workspace():
    rng = np.random.default_rng(5)
    H, n_q, C, n_sel = 2, 300, 640, 4
    Q, K, V = (to_dev(to_storage(rng.standard_normal((H, n, 128)).astype(np.float32), "bf16")) for n in (n_q, C, C))
    lens = to_dev(np.array([640, 300], np.int32))
    sel = to_dev(np.stack([np.stack([np.sort(rng.choice(10, n_sel, replace=False)) for _ in range(3)]) for _ in range(H)]).astype(np.int32))
    nsel = to_dev(np.full((H, 3), n_sel, np.int32))
    ws = torch.empty(fa.workspace_bytes(fa.OP_ATTN, H, n_q, C), dtype=torch.uint8, device="cuda")
    a = fa.sparse_attn_fwd(Q, K, V, None, lens, sel, nsel, 128, 64, 0.1, ws=ws)
    b = fa.sparse_attn_fwd(Q, K, V, None, lens, sel, nsel, 128, 64, 0.1)
    sync()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    with pytest.raises(fa.FastarError):
        fa.sparse_attn_fwd(Q, K, V, None, lens, sel, nsel, 128, 64, 0.1, ws=ws[:1024])
