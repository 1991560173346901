"""GPU parity at the benchmark's full shapes, in the launch configuration bench.py times.

The GPU runs every head; the CPU oracle replays a subset of heads from the same inputs (heads are
independent in every step of the method, so a head slice of the inputs gives exactly the head slice
of the outputs).  Index outputs must match bit for bit, attention within 2e-2 max-abs (bf16).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2602_01801_amd as fa
from workloads import CONFIGS, FrameStream, PromptSet, make_codec, to_f32

from gpu_util import dev_codec, storage_to_f64, to_dev, to_host

pytestmark = pytest.mark.gpu

TAU2 = lambda tau: int(round(tau * tau * 65536))


def rollout(name, n_frames, cap_frames, heads, tau=0.98):
    """Compress n_frames frames on the GPU (all heads) and in the oracle (`heads` only), checking every call."""
    c = CONFIGS[name]
    H, T, d, r = c["H"], c["T"], c["d"], c["r"]
    fs = FrameStream.from_config(name)
    codec = make_codec(c["seed"], c["cfg_id"], d, r)
    dcodec = dev_codec(codec)
    C = cap_frames * T
    gpu = fa.Cache.empty(H, C, d, r, torch.bfloat16)
    ref = oracle.Cache.empty(len(heads), C, d, r, "bf16")
    prev_g = prev_r = None
    ws = torch.empty(fa.workspace_bytes(fa.OP_COMPRESS, H, T, C, r), dtype=torch.uint8, device="cuda")
    for f in range(n_frames):
        K, V = fs.next_frame()
        mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dcodec, to_dev(K), to_dev(V), cand=prev_g, tau2_q16=TAU2(tau),
                                                 frame_id=f, ws=ws)
        mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift,
                                                     np.ascontiguousarray(K[heads]), np.ascontiguousarray(V[heads]),
                                                     cand=prev_r, tau2_q16=TAU2(tau), frame_id=f)
        assert np.array_equal(to_host(mm_g)[heads], mm_r), f"merge map, frame {f}"
        assert np.array_equal(to_host(mg_g)[heads], mg_r), f"merged flags, frame {f}"
        assert np.array_equal(to_host(st_g)[heads], st_r), f"stats, frame {f}"
        prev_g, prev_r = mm_g.clone(), mm_r
    # cache bookkeeping of the sampled heads
    assert np.array_equal(to_host(gpu.len)[heads], ref.len)
    for i, h in enumerate(heads):
        L = int(ref.len[i])
        assert np.array_equal(to_host(gpu.K[h, :L]), ref.K[i, :L])
        assert np.array_equal(to_host(gpu.code[h, :L]), ref.code[i, :L])
        assert np.array_equal(to_host(gpu.cnt[h, :L]), ref.cnt[i, :L])
        assert np.array_equal(to_host(gpu.stamp[h, :L]), ref.stamp[i, :L])
        dv = np.abs(storage_to_f64(to_host(gpu.V[h, :L])) - storage_to_f64(ref.V[i, :L])).max()
        assert dv <= 5e-2, f"running-mean values, head {h}: {dv}"
    return c, fs, codec, dcodec, gpu, ref


def select_and_attend(c, fs, codec, dcodec, gpu, ref, heads, n_sel):
    H, d = c["H"], c["d"]
    BQ, BK, n_rep = c["BQ"], c["BK"], c["n_rep"]
    Q = fs.queries(c["chunk_frames"])
    qc = fa.encode(to_dev(Q), dcodec)
    qc_r = oracle.encode(np.ascontiguousarray(Q[heads]), codec.R, codec.qscale, codec.shift)
    assert np.array_equal(to_host(qc)[heads], qc_r)
    sel, nsel = fa.ann_select_self(qc, gpu.code, gpu.len, BQ, n_rep, BK, n_sel)
    sel_r, nsel_r = oracle.ann_select_self(qc_r, ref.code, ref.len, BQ, n_rep, BK, n_sel)
    assert np.array_equal(to_host(nsel)[heads], nsel_r)
    assert np.array_equal(to_host(sel)[heads], sel_r)
    O, lse = fa.sparse_attn_fwd(to_dev(Q), gpu.K, gpu.V, gpu.cnt, gpu.len, sel, nsel, BQ, BK, d ** -0.5)
    # the oracle attends over ITS cache state (values differ from the GPU's by bf16 rounding of the running mean)
    O_r, lse_r = oracle.sparse_attn_fwd(np.ascontiguousarray(Q[heads]), ref.K, ref.V, ref.cnt, ref.len, sel_r, nsel_r,
                                        BQ, BK, d ** -0.5)
    err = np.abs(storage_to_f64(to_host(O))[heads] - O_r).max()
    assert err <= 2e-2, f"max |O - O_ref| = {err}"
    assert np.abs(to_host(lse)[heads].astype(np.float64) - lse_r).max() <= 2e-2
    return Q, qc, qc_r


def test_wan_shaped_layer_full_size():
    # cfg2: 12 heads, d 128, 21 frames of 1560 tokens merged into a cache capped at 24 frames of slots,
    # 52 of 512 key blocks per query block, 4680 queries
    heads = [0, 7]
    c, fs, codec, dcodec, gpu, ref = rollout("cfg2", 21, 24, heads)
    n_kb = (c["cache_frames"] * c["T"] + c["BK"] - 1) // c["BK"]
    n_sel = int(np.ceil(c["sel_frac"] * n_kb))
    assert n_sel == 52
    Q, qc, qc_r = select_and_attend(c, fs, codec, dcodec, gpu, ref, heads, n_sel)
    # the sign-code (LSH) selection on the same cache and queries: 128 hash bits, same budget
    rng = np.random.default_rng(99)
    Rb = rng.choice(np.array([-1, 1], np.int8), size=(c["d"], 128))
    qb = fa.encode_sign(to_dev(Q), to_dev(Rb), codec.qscale)
    kb = fa.encode_sign(gpu.K, to_dev(Rb), codec.qscale)
    qb_r = oracle.encode_sign(np.ascontiguousarray(Q[heads]), Rb, codec.qscale)
    kb_r = oracle.encode_sign(ref.K, Rb, codec.qscale)
    assert np.array_equal(to_host(qb).view(np.uint32)[heads], qb_r)
    for i, h in enumerate(heads):
        L = int(ref.len[i])
        assert np.array_equal(to_host(kb[h, :L]).view(np.uint32), kb_r[i, :L])
    lsel, lnsel = fa.ann_select_lsh(qb, kb, gpu.len, c["BQ"], c["n_rep"], c["BK"], n_sel)
    lsel_r, lnsel_r = oracle.ann_select_lsh(qb_r, kb_r, ref.len, c["BQ"], c["n_rep"], c["BK"], n_sel)
    assert np.array_equal(to_host(lnsel)[heads], lnsel_r) and np.array_equal(to_host(lsel)[heads], lsel_r)
    O, _ = fa.sparse_attn_fwd(to_dev(Q), gpu.K, gpu.V, gpu.cnt, gpu.len, lsel, lnsel, c["BQ"], c["BK"], c["d"] ** -0.5)
    O_r, _ = oracle.sparse_attn_fwd(np.ascontiguousarray(Q[heads]), ref.K, ref.V, ref.cnt, ref.len, lsel_r, lnsel_r,
                                    c["BQ"], c["BK"], c["d"] ** -0.5)
    assert np.abs(storage_to_f64(to_host(O))[heads] - O_r).max() <= 2e-2
    # cross-attention legs (cfg4): 64 of 512 and of 2048 prompt tokens
    for n_p in (c["n_p"], CONFIGS["cfg4"]["n_p_long"]):
        ps = PromptSet(c["seed"], c["cfg_id"], fs.centreK, n_p, c["n_pc"], c["n_near"], c["dtype"])
        pc = fa.encode(to_dev(ps.K), dcodec)
        pc_r = oracle.encode(np.ascontiguousarray(ps.K[heads]), codec.R, codec.qscale, codec.shift)
        assert np.array_equal(to_host(pc)[heads], pc_r)
        csel, cnsel = fa.ann_select_cross(qc, pc, c["BQ"], c["n_sel_cross"])
        csel_r, cnsel_r = oracle.ann_select_cross(qc_r, pc_r, c["BQ"], c["n_sel_cross"])
        assert np.array_equal(to_host(csel)[heads], csel_r) and np.array_equal(to_host(cnsel)[heads], cnsel_r)
        plen = np.full(c["H"], n_p, np.int32)
        O, _ = fa.sparse_attn_fwd(to_dev(Q), to_dev(ps.K), to_dev(ps.V), None, to_dev(plen), csel, cnsel, c["BQ"], 1,
                                  c["d"] ** -0.5)
        O_r, _ = oracle.sparse_attn_fwd(np.ascontiguousarray(Q[heads]), np.ascontiguousarray(ps.K[heads]),
                                        np.ascontiguousarray(ps.V[heads]), None, plen[: len(heads)], csel_r, cnsel_r,
                                        c["BQ"], 1, c["d"] ** -0.5)
        err = np.abs(storage_to_f64(to_host(O))[heads] - O_r).max()
        assert err <= 2e-2, f"cross-attention n_p={n_p}: {err}"


def test_bounded_cache_evicts_at_full_size():
    # cfg3's cap reached quickly: capacity of 3 frames of slots, 8 frames pushed through
    rollout("cfg2", 8, 3, [3])


def test_world_model_shaped_layer():
    # cfg5's shape (40 heads, 3600 tokens per frame, 128 clusters) on a short rollout
    heads = [0, 39]
    c, fs, codec, dcodec, gpu, ref = rollout("cfg5", 5, 5, heads)
    select_and_attend(c, fs, codec, dcodec, gpu, ref, heads, 29)


def test_dense_limit_uncompressed_wan_cache():
    # plain concatenation of 4 frames (nothing merges at tau^2 = 2) and every block selected:
    # the kernel must reproduce dense softmax attention over 6240 keys
    heads = [5]
    c, fs, codec, dcodec, gpu, ref = rollout("cfg2", 4, 4, heads, tau=2.0 ** 0.5)
    assert int(ref.len[0]) == 4 * c["T"]
    n_kb = (4 * c["T"] + c["BK"] - 1) // c["BK"]
    select_and_attend(c, fs, codec, dcodec, gpu, ref, heads, n_kb)


@pytest.mark.parametrize("with_ws", [True, False])
def test_world_model_attention_on_a_full_cache(with_ws):
    # cfg5 at the size bench.py's default run holds: 40 heads x 230400 live slots (64 frames of 3600), 3600 queries, 360 of
    # 3600 key blocks per query block; 29 x 40 = 1160 query blocks on K and V far beyond the memory-side cache.  Without
    # a workspace the kernel with one block per workgroup is launched; with one (as bench.py calls it) the launch is
    # split: 128 of the 145 (head, block) pairs of every XCD range by one workgroup each, the other 17 in equal shares
    # of their tiles.  The cache is synthetic (seeded normal keys and values, multiplicities 1..6, two heads not quite
    # full); the oracle recomputes, of three heads, the first, a middle and the ragged last query block, and three blocks
    # of head 4, whose blocks 12..28 are pairs 128..144: the first range's left-over ones.
    c = CONFIGS["cfg5"]
    H, d, BQ, BK = c["H"], c["d"], c["BQ"], c["BK"]
    n_q, C, n_sel = c["T"], 64 * c["T"], 360
    assert (H, d, BQ, BK, n_q) == (40, 128, 128, 64, 3600)
    g = torch.Generator(device="cuda").manual_seed(20260205)
    Q = torch.randn((H, n_q, d), device="cuda", generator=g).to(torch.bfloat16)
    K = torch.randn((H, C, d), device="cuda", generator=g).to(torch.bfloat16)
    V = torch.randn((H, C, d), device="cuda", generator=g).to(torch.bfloat16)
    cnt = torch.randint(1, 7, (H, C), device="cuda", generator=g, dtype=torch.int32)
    lens = np.full(H, C, np.int32)
    lens[17], lens[39] = C - 41, C - 64 * 100 - 1
    n_qb, n_kb = (n_q + BQ - 1) // BQ, C // BK
    rng = np.random.default_rng(5)
    sel = np.empty((H, n_qb, n_sel), np.int32)
    for h in range(H):
        for b in range(n_qb):
            sel[h, b] = np.sort(rng.choice(n_kb, n_sel, replace=False))   # the last blocks of heads 17, 39: partly / wholly dead
    nsel = np.full((H, n_qb), n_sel, np.int32)
    ws = torch.empty(fa.workspace_bytes(fa.OP_ATTN, H, n_q, C), dtype=torch.uint8, device="cuda") if with_ws else None
    O, lse = fa.sparse_attn_fwd(Q, K, V, cnt, to_dev(lens), to_dev(sel), to_dev(nsel), BQ, BK, d ** -0.5, ws=ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O.float()).all())
    for h, blocks in ((0, (0, 13, n_qb - 1)), (17, (0, 13, n_qb - 1)), (39, (0, 13, n_qb - 1)), (4, (12, 20, n_qb - 1))):
        Kh, Vh, ch = to_host(K[h:h + 1]), to_host(V[h:h + 1]), to_host(cnt[h:h + 1])
        for b in blocks:
            q0, q1 = b * BQ, min((b + 1) * BQ, n_q)
            O_r, lse_r = oracle.sparse_attn_fwd(to_host(Q[h:h + 1, q0:q1]), Kh, Vh, ch, lens[h:h + 1],
                                                np.ascontiguousarray(sel[h:h + 1, b:b + 1]), nsel[h:h + 1, b:b + 1],
                                                BQ, BK, d ** -0.5)
            err = np.abs(storage_to_f64(to_host(O[h:h + 1, q0:q1])) - O_r).max()
            assert err <= 2e-2, f"head {h} block {b}: max |O - O_ref| = {err}"
            assert np.abs(to_host(lse[h:h + 1, q0:q1]).astype(np.float64) - lse_r).max() <= 2e-2


def test_world_model_selection_on_a_full_cache():
    # AnnSA at the same size: 40 heads x 230400 live codes in blocks of 64, 3600 queries in blocks of 128 with 4 summaries,
    # 360 of 3600 blocks kept: the streaming scoring kernel and the top-k over rows of 3600 scores, as bench.py times
    # them.  Seeded random codes; the oracle replays three heads (one not quite full, one with 100 dead blocks).
    c = CONFIGS["cfg5"]
    H, r, BQ, BK, n_rep = c["H"], c["r"], c["BQ"], c["BK"], c["n_rep"]
    n_q, C, n_sel = c["T"], 64 * c["T"], 360
    g = torch.Generator(device="cuda").manual_seed(20260206)
    qc = torch.randint(-40, 41, (H, n_q, r), device="cuda", generator=g, dtype=torch.int8)
    kc = torch.randint(-40, 41, (H, C, r), device="cuda", generator=g, dtype=torch.int8)
    lens = np.full(H, C, np.int32)
    lens[17], lens[39] = C - 41, C - 64 * 100 - 1
    sel, nsel = fa.ann_select_self(qc, kc, to_dev(lens), BQ, n_rep, BK, n_sel)
    torch.cuda.synchronize()
    heads = [0, 17, 39]
    sel_r, nsel_r = oracle.ann_select_self(to_host(qc[heads]), to_host(kc[heads]), lens[heads], BQ, n_rep, BK, n_sel)
    assert np.array_equal(to_host(nsel)[heads], nsel_r)
    assert np.array_equal(to_host(sel)[heads], sel_r)


def test_world_model_compress_on_a_full_cache():
    # TempCache at the same size: one frame of 40 x 3600 tokens against a full cache of 230400 slots per head with a
    # candidate window of 3600 slots (staged in LDS, as in bench.py --workload cfg5): a third of the tokens repeat live
    # slots and merge, the rest need a slot each, so a full head evicts 2400 of its oldest untouched slots (63 stamp
    # values over 230400 slots: long runs of ties).  Synthetic seeded cache; the oracle replays three heads, whose codes are
    # its own encoding of their keys (the other heads carry random codes: their tokens match nothing and are all appended).
    c = CONFIGS["cfg5"]
    H, d, r, T = c["H"], c["d"], c["r"], c["T"]
    C = 64 * T
    codec = make_codec(c["seed"], c["cfg_id"], d, r)
    g = torch.Generator(device="cuda").manual_seed(20260207)
    gpu = fa.Cache.empty(H, C, d, r, torch.bfloat16)
    gpu.K.copy_(torch.randn((H, C, d), device="cuda", generator=g))
    gpu.V.copy_(torch.randn((H, C, d), device="cuda", generator=g))
    gpu.code.copy_(torch.randint(-40, 41, (H, C, r), device="cuda", generator=g, dtype=torch.int8))
    gpu.cnt.copy_(torch.randint(1, 4, (H, C), device="cuda", generator=g, dtype=torch.int32))
    gpu.stamp.copy_(torch.randint(0, 63, (H, C), device="cuda", generator=g, dtype=torch.int32))
    lens = np.full(H, C, np.int32)
    lens[17], lens[39] = C - 41, C - 1001                     # 2400 / 2359 / 1399 evictions
    gpu.len.copy_(to_dev(lens))
    heads = [0, 17, 39]
    K_h = to_host(gpu.K[heads])
    code_h = oracle.encode(K_h, codec.R, codec.qscale, codec.shift)
    gpu.code[heads] = to_dev(code_h)
    ref = oracle.Cache(K=K_h, V=to_host(gpu.V[heads]), code=code_h, cnt=to_host(gpu.cnt[heads]),
                       stamp=to_host(gpu.stamp[heads]), len=lens[heads].copy())
    n_dup = T // 3
    idx = torch.randint(0, C - 7000, (H, n_dup), device="cuda", generator=g)       # live in every head
    K_new = torch.randn((H, T, d), device="cuda", generator=g).to(torch.bfloat16)
    K_new[:, :n_dup] = torch.gather(gpu.K, 1, idx.unsqueeze(-1).expand(-1, -1, d))
    V_new = torch.randn((H, T, d), device="cuda", generator=g).to(torch.bfloat16)
    cand = torch.randint(0, C, (H, T), device="cuda", generator=g, dtype=torch.int32)   # some past the live length
    cand[:, :n_dup] = idx.to(torch.int32)
    K_new_h, V_new_h, cand_h = to_host(K_new[heads]), to_host(V_new[heads]), to_host(cand[heads])
    mm_g, mg_g, st_g = fa.tempcache_compress(gpu, dev_codec(codec), K_new, V_new, cand=cand, tau2_q16=TAU2(0.98), frame_id=64)
    torch.cuda.synchronize()
    mm_r, mg_r, st_r = oracle.tempcache_compress(ref, codec.R, codec.qscale, codec.shift, K_new_h, V_new_h, cand=cand_h,
                                                 tau2_q16=TAU2(0.98), frame_id=64)
    assert mg_r[:, :n_dup].all() and (st_r[:, 3] > 1000).all() and (st_r[:, 7] == 0).all()   # merges and evictions
    assert np.array_equal(to_host(st_g)[heads], st_r)
    assert np.array_equal(to_host(mg_g)[heads], mg_r)
    assert np.array_equal(to_host(mm_g)[heads], mm_r)
    assert np.array_equal(to_host(gpu.len)[heads], ref.len)
    for i, h in enumerate(heads):
        L = int(ref.len[i])
        assert np.array_equal(to_host(gpu.K[h, :L]), ref.K[i, :L]), f"K head {h}"
        assert np.array_equal(to_host(gpu.code[h, :L]), ref.code[i, :L]), f"code head {h}"
        assert np.array_equal(to_host(gpu.cnt[h, :L]), ref.cnt[i, :L]), f"cnt head {h}"
        assert np.array_equal(to_host(gpu.stamp[h, :L]), ref.stamp[i, :L]), f"stamp head {h}"
        dv = np.abs(storage_to_f64(to_host(gpu.V[h, :L])) - storage_to_f64(ref.V[i, :L])).max()
        assert dv <= 5e-2, f"running-mean values, head {h}: {dv}"
