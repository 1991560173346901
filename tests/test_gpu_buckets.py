"""GPU parity of the prompt-induced bucket selection (ann_prompt_buckets, ann_select_buckets) against the oracle:
bucket ids and selected sets bit for bit, on seeded codes with heavy ties, ragged prompt lengths, index lists with
repeats and skips, ragged / empty caches, forced blocks, and the Wan-shaped and world-model-shaped layers."""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_01801_amd as fa
from workloads import CONFIGS, FrameStream, PromptSet, make_codec

from gpu_util import to_dev, to_host

pytestmark = pytest.mark.gpu


def rand_codes(rng, lo, hi, *shape):
    return rng.integers(lo, hi + 1, size=shape).astype(np.int8)


@pytest.mark.parametrize("H,n,n_p,r,m,span", [
    (2, 300, 64, 32, 1, 60), (2, 1000, 512, 32, 2, 40), (1, 130, 77, 64, 3, 50),     # ragged last prompt block, r = 64
    (3, 257, 5, 32, 8, 30),                                                           # more buckets than prompt tokens
    (2, 400, 2048, 32, 2, 3), (1, 4680, 512, 32, 1, 127),                             # heavy ties; extreme codes
    (1, 64, 1, 64, 1, 127)])
def test_prompt_buckets_bit_exact(H, n, n_p, r, m, span):
    rng = np.random.default_rng(n + n_p + m)
    code, pcode = rand_codes(rng, -span, span, H, n, r), rand_codes(rng, -span, span, H, n_p, r)
    ref = oracle.prompt_buckets(code, pcode, m)
    got = to_host(fa.prompt_buckets(to_dev(code), to_dev(pcode), m))
    assert np.array_equal(got, ref)


def test_prompt_buckets_of_listed_rows_only():
    rng = np.random.default_rng(3)
    H, C, n_p, r, m = 2, 900, 200, 32, 2
    code, pcode = rand_codes(rng, -50, 50, H, C, r), rand_codes(rng, -50, 50, H, n_p, r)
    ref = oracle.prompt_buckets(code, pcode, m)
    idx = rng.integers(-2, C + 3, size=(H, 333)).astype(np.int32)      # repeats, negative and too large entries
    out = torch.full((H, C, m), -7, dtype=torch.int32, device="cuda")
    got = to_host(fa.prompt_buckets(to_dev(code), to_dev(pcode), m, idx=to_dev(idx), out=out))
    for h in range(H):
        named = np.zeros(C, bool)
        named[idx[h][(idx[h] >= 0) & (idx[h] < C)]] = True
        assert np.array_equal(got[h][named], ref[h][named])
        assert (got[h][~named] == -7).all()


@pytest.mark.parametrize("H,n_q,C,lens,m,n_p,BQ,BK,n_sel,sink,local", [
    (2, 300, 64 * 40, [2560, 1000], 1, 64, 128, 64, 9, 0, 0),
    (3, 700, 64 * 100, [6400, 6399, 0], 2, 512, 128, 64, 12, 0, 0),            # ragged tail, empty head
    (2, 300, 64 * 40, [2560, 70], 1, 2048, 128, 64, 6, 2, 3),                  # forced blocks, widest masks, a tiny head
    (1, 4680, 64 * 585, [37440], 2, 512, 128, 64, 52, 0, 0),                   # Wan-shaped
    (2, 3600, 64 * 3600, [230400, 200001], 1, 512, 128, 64, 360, 4, 56),       # world-model rows
    (1, 200, 32 * 50, [1600], 3, 40, 64, 32, 100, 0, 0),                       # budget beyond the candidates
    (1, 3120, 64 * 80, [5120], 1, 300, 1560, 64, 8, 0, 0)])                    # one query block per frame
def test_ann_select_buckets_bit_exact(H, n_q, C, lens, m, n_p, BQ, BK, n_sel, sink, local):
    rng = np.random.default_rng(n_q + C + n_p)
    # every key block draws its keys' buckets from a palette of three prompt tokens, every query from a quarter of the
    # prompt tokens: many key blocks share nothing with a query block, many tie; a few entries are -1 or out of range
    n_kb = -(-C // BK)
    palette = rng.integers(0, n_p, size=(H, n_kb, 3))
    pick = rng.integers(0, 3, size=(H, n_kb * BK, m))
    kb = np.take_along_axis(np.repeat(palette, BK, axis=1), pick, axis=2)[:, :C]
    kb = np.where(rng.random(kb.shape) < 0.05, rng.integers(-1, n_p + 2, size=kb.shape), kb).astype(np.int32)
    qb = rng.integers(-1, max(2, n_p // 4), size=(H, n_q, m)).astype(np.int32)
    if BQ > 1000:
        qb = np.where(qb >= 0, qb % 5, qb)        # a whole frame per query block: keep its bucket set small
    length = np.array(lens, np.int32)
    ref_sel, ref_nsel = oracle.ann_select_buckets(qb, kb, length, n_p, BQ, BK, n_sel, sink, local)
    sel, nsel = fa.ann_select_buckets(to_dev(qb), to_dev(kb), to_dev(length), n_p, BQ, BK, n_sel, sink, local)
    assert np.array_equal(to_host(nsel), ref_nsel)
    assert np.array_equal(to_host(sel), ref_sel)
    if n_sel == 100:   # this case has fewer candidates than budget
        assert (ref_nsel < min(n_sel, -(-C // BK))).all()


def test_buckets_end_to_end_on_the_synthetic_layer():
    # codes of the tiny workload: queries, cached keys and prompt keys through the GPU encode, buckets, selection, and
    # the attention over that selection against the oracle's
    c = CONFIGS["cfg1"]
    H, T, d, r = c["H"], c["T"], c["d"], c["r"]
    fs = FrameStream.from_config("cfg1")
    codec = make_codec(c["seed"], c["cfg_id"], d, r)
    frames = [fs.next_frame() for _ in range(4)]
    K = np.concatenate([f[0] for f in frames], axis=1)
    V = np.concatenate([f[1] for f in frames], axis=1)
    Q = fs.queries(1)
    ps = PromptSet(c["seed"], c["cfg_id"], fs.centreK, 64, 8, 3, c["dtype"])
    kc = oracle.encode(K, codec.R, codec.qscale, codec.shift)
    qc = oracle.encode(Q, codec.R, codec.qscale, codec.shift)
    pc = oracle.encode(ps.K, codec.R, codec.qscale, codec.shift)
    length = np.full(H, K.shape[1], np.int32)
    n_p = pc.shape[1]
    qb_r, kb_r = oracle.prompt_buckets(qc, pc, 2), oracle.prompt_buckets(kc, pc, 2)
    sel_r, nsel_r = oracle.ann_select_buckets(qb_r, kb_r, length, n_p, c["BQ"], c["BK"], 6)
    qb_g, kb_g = fa.prompt_buckets(to_dev(qc), to_dev(pc), 2), fa.prompt_buckets(to_dev(kc), to_dev(pc), 2)
    assert np.array_equal(to_host(qb_g), qb_r) and np.array_equal(to_host(kb_g), kb_r)
    sel_g, nsel_g = fa.ann_select_buckets(qb_g, kb_g, to_dev(length), n_p, c["BQ"], c["BK"], 6)
    assert np.array_equal(to_host(sel_g), sel_r) and np.array_equal(to_host(nsel_g), nsel_r)
    O, _ = fa.sparse_attn_fwd(to_dev(Q), to_dev(K), to_dev(V), None, to_dev(length), sel_g, nsel_g, c["BQ"], c["BK"], d ** -0.5)
    O_r, _ = oracle.sparse_attn_fwd(Q, K, V, None, length, sel_r, nsel_r, c["BQ"], c["BK"], d ** -0.5)
    assert np.abs(to_host(O).astype(np.float64) - O_r).max() <= 1e-4


def test_unsupported_and_invalid_arguments_are_rejected():
    code = torch.zeros((1, 64, 32), dtype=torch.int8, device="cuda")
    with pytest.raises(fa.FastarError):
        fa.prompt_buckets(code, torch.zeros((1, 2049, 32), dtype=torch.int8, device="cuda"))
    with pytest.raises(fa.FastarError):
        fa.prompt_buckets(code, code, m=9)
    b = torch.zeros((1, 64, 1), dtype=torch.int32, device="cuda")
    ln = torch.full((1,), 64, dtype=torch.int32, device="cuda")
    with pytest.raises(fa.FastarError):
        fa.ann_select_buckets(b, b, ln, 16, 32, 32, 2, n_sink=2, n_local=1)
    with pytest.raises(fa.FastarError):
        fa.ann_select_buckets(b, b, ln, 4096, 32, 32, 2)
