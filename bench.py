#!/usr/bin/env python3
"""Benchmark of the FAST-AR attention hot path on one MI355X.

A *step* is one generated chunk: TempCache merges of the chunk's frames into the bounded cache, ANN codes of
the queries, AnnSA selection of 10 % of the key blocks per query block, block-sparse self-attention, AnnCA
selection of 64 of 512 prompt tokens and the cross-attention over them.  All inputs are seeded synthetic data
(clustered, temporally repeating K/V) already resident in HBM when the clock starts.

Workloads (--workload):
  cfg5full  (default, the headline) the world-model-scale layer at its full size: 40 heads, d 128, one frame of
            3600 tokens per chunk, a cache of 64 frames = 230 400 live slots per head (5.1 GB), filled by the seeded
            device-side generator; every step merges about 90 % of its frame and evicts for the rest, AnnSA keeps 360
            of 3600 key blocks.
  cfg2      the Wan-1.3B-shaped layer (12 heads, 3 frames of 1560 tokens per chunk, cache capped at 24 frames).
  cfg5      the world-model layer fed through TempCache from an empty cache (the cache stays small).
The default run carries a short cfg2 leg and the two ends of the long-rollout sweep (cfg3) as extra keys.

Prints ONE JSON line: ms per chunk for the whole hot path, the per-stage split with achieved GB/s of the
bandwidth-bound stages, the roofline fraction of the dominant kernel (block-sparse self-attention, bf16 matrix
cores, attended FLOPs only) and the CPU oracle's time for the same chunk on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix-core peak
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense 8-bit floating-point matrix-core peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--ann", choices=["int8", "lsh"], default="int8",
                    help="AnnSA code family: int8 projection codes (default) or 128-bit sign codes (LSH variant)")
    ap.add_argument("--code-shift", type=int, default=None,
                    help="right shift of the projected sums in the int8 code (default 4, about 8 significant bits; "
                         "6 / 8 / 9 leave about 6 / 4 / 2): the bit-width ladder of the paper's quantisation ablation")
    ap.add_argument("--stage-steps", type=int, default=4,
                    help="extra steps after the timed region, instrumented with an event after every stage")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=6,
                    help="untimed steps first; the first four or five launches after an idle queue run 5-25 %% slower "
                         "than the steady state on this chip (clock and power settling)")
    ap.add_argument("--workload", default="cfg5full", choices=["cfg5full", "cfg2", "cfg5"])
    ap.add_argument("--no-extras", action="store_true",
                    help="headline workload only: skip the short cfg2 leg and the sweep ends of the default run")
    ap.add_argument("--tau", type=float, default=0.98)
    ap.add_argument("--ws", choices=["persistent", "scratch"], default="persistent",
                    help="TempCache workspace: kept by the caller across calls (zero-filled once; one launch less per "
                         "frame) or scratch that may hold anything")
    ap.add_argument("--streams", type=int, choices=[1, 2], default=None,
                    help="2: the query codes and the cross-attention path (they depend on Q and the prompt only) run on a "
                         "second stream of the same priority beside the compress calls and are joined before the step "
                         "ends.  Default at the world-model layer (measured: -0.9 %%; the window-match and plan launches "
                         "fill the register files of their compute units, so the second stream's kernels mostly run "
                         "beside the apply launch); 1 at the Wan-shaped layer, where the extra enqueue cost shows")
    ap.add_argument("--cross", choices=["fused", "separate"], default="fused",
                    help="AnnCA as one launch (selection + attention) or as ann_select_cross followed by sparse_attn_fwd")
    ap.add_argument("--cand", choices=["as-is", "sorted"], default="as-is",
                    help="candidate list handed to tempcache_compress: the previous call's merge map as it is (the "
                         "kernel sorts it) or sorted ascending by the caller first (one torch sort per frame, untimed "
                         "work it is not: it runs inside the step)")
    ap.add_argument("--kv", choices=["bf16", "fp8"], default="bf16",
                    help="self-attention over the bf16 cache (default) or over its 8-bit floating-point (E4M3) copy, "
                         "which fastar_kv_to_fp8 brings up to date after the chunk's TempCache calls")
    ap.add_argument("--rep", choices=["last", "mean", "medoid"], default="last",
                    help="representative key of a merged group: the last key (the method) or the mean / medoid key (its ablation)")
    ap.add_argument("--prefill-frames", type=int, default=None, help="frames merged into the cache before timing")
    ap.add_argument("--cap-frames", type=int, default=None, help="cache capacity in frames of slots")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-equivalent", action="store_true",
                    help="skip the leg that times the attention kernel with every live key block selected")
    ap.add_argument("--cpu-heads", type=int, default=2, help="heads of the last chunk replayed on the CPU oracle")
    ap.add_argument("--sweep", action="store_true", help="long-rollout sweep (cfg3): per-step latency and footprint")
    ap.add_argument("--sweep-frames", type=int, default=120)
    ap.add_argument("--out", default=None, help="also write the JSON (and the sweep table) to this file")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="after the timed loop, run one plain device copy of this many MiB (a known-size "
                         "reference for scaling the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class ChunkPipeline:
    """Device buffers and the call sequence of one chunk step.  Nothing is allocated per step."""

    def __init__(self, cfg, C, tau, torch, fa, dev_codec, prompt, n_sel_blocks, sign_matrix=None, rep_mode=0,
                 fused_cross=True, ws_persistent=True):
        self.t, self.fa, self.cfg = torch, fa, cfg
        self.ws_persistent = ws_persistent
        self.sorted_cand = False
        self.kv8 = None        # (K8, V8T) when the self-attention runs over the 8-bit copy of the cache
        self.rep_mode = rep_mode
        self.fused_cross = fused_cross
        H, d, r, T = cfg["H"], cfg["d"], cfg["r"], cfg["T"]
        self.H, self.d, self.r, self.T, self.C = H, d, r, T, C
        self.BQ, self.BK, self.n_rep = cfg["BQ"], cfg["BK"], cfg["n_rep"]
        self.n_q = T * cfg["chunk_frames"]
        self.n_qb = (self.n_q + self.BQ - 1) // self.BQ
        self.n_sel = n_sel_blocks
        self.n_sel_cross = cfg["n_sel_cross"]
        self.tau2 = int(round(tau * tau * 65536))
        self.scale = d ** -0.5
        self.codec = dev_codec
        dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        self.cache = fa.Cache.empty(H, C, d, r, dt)
        dev = "cuda"
        e = lambda shape, dtype: torch.empty(shape, dtype=dtype, device=dev)
        self.ws_c = torch.zeros((fa.workspace_bytes(fa.OP_COMPRESS, H, T, C, r),), dtype=torch.uint8, device=dev)
        self.ws_s = e((fa.workspace_bytes(fa.OP_SELECT_SELF, H, self.n_q, C, r, self.BQ, self.BK, self.n_rep),), torch.uint8)
        self.mm = [(e((H, T), torch.int32), e((H, T), torch.uint8), e((H, 8), torch.int32)) for _ in range(2)]
        self.qcode = e((H, self.n_q, r), torch.int8)
        self.sel = (e((H, self.n_qb, self.n_sel), torch.int32), e((H, self.n_qb), torch.int32))
        self.O = (e((H, self.n_q, d), dt), e((H, self.n_q), torch.float32))
        # workspace of the self-attention call: with it, a launch that would end in a short last round is split (whole
        # rounds of one-block workgroups, then equal shares of the blocks left over)
        self.ws_a = e((fa.workspace_bytes(fa.OP_ATTN, H, self.n_q, C),), torch.uint8) if dt == torch.bfloat16 and d == 128 else None
        self.prev = None
        self.frame_id = 0
        self.side = None       # second stream for the work that depends on Q and the prompt only (set by the caller)
        self.ev_q = None
        # cross-attention: prompt K/V and their codes are fixed for the rollout
        self.pK, self.pV = prompt
        self.n_p = self.pK.shape[1]
        self.pcode = fa.encode(self.pK, self.codec)
        self.plen = torch.full((H,), self.n_p, dtype=torch.int32, device=dev)
        self.ws_x = e((fa.workspace_bytes(fa.OP_SELECT_CROSS, H, self.n_q, self.n_p, r, self.BQ),), torch.uint8)
        self.csel = (e((H, self.n_qb, self.n_sel_cross), torch.int32), e((H, self.n_qb), torch.int32))
        self.Ox = (e((H, self.n_q, d), dt), None)
        # sign-code (LSH) variant of AnnSA: the cache keeps no hash bits, they are recomputed from K every chunk
        self.Rb = sign_matrix
        if sign_matrix is not None:
            W = sign_matrix.shape[1] // 32
            self.qbits = e((H, self.n_q, W), torch.int32)
            self.kbits = e((H, C, W), torch.int32)
            self.ws_l = e((fa.workspace_bytes(fa.OP_SELECT_LSH, H, self.n_q, C, 32 * W, self.BQ, self.BK, self.n_rep),),
                          torch.uint8)

    def compress(self, K, V):
        fa = self.fa
        out = self.mm[self.frame_id & 1]
        cand = self.prev
        if self.sorted_cand and cand is not None:
            cand = self.t.sort(cand, dim=1).values.contiguous()
        fa.tempcache_compress(self.cache, self.codec, K, V, cand=cand, tau2_q16=self.tau2,
                              frame_id=self.frame_id, rep_mode=self.rep_mode, ws=self.ws_c, out=out,
                              ws_persistent=self.ws_persistent)
        self.prev = out[0]
        self.frame_id += 1

    def step(self, frames, Q, ev=None):
        """frames: list of (K, V) device tensors of the chunk; Q [H,n_q,d].  ev: optional event recorder."""
        fa = self.fa
        mark = ev if ev is not None else (lambda name: None)
        if self.side is not None and self.Rb is None and self.fused_cross:
            return self.step_two_streams(frames, Q, mark)
        mark("start")
        first_frame = self.frame_id
        for K, V in frames:
            self.compress(K, V)
        mark("compress")
        if self.kv8 is not None:
            fa.kv_to_fp8(self.cache, self.kv8[0], self.kv8[1], stamp_lo=first_frame)
        mark("quantize")
        fa.encode(Q, self.codec, out=self.qcode)
        if self.Rb is not None:
            fa.encode_sign(Q, self.Rb, self.codec.qscale, out=self.qbits)
            fa.encode_sign(self.cache.K, self.Rb, self.codec.qscale, out=self.kbits)
        mark("encode")
        if self.Rb is not None:
            fa.ann_select_lsh(self.qbits, self.kbits, self.cache.len, self.BQ, self.n_rep, self.BK, self.n_sel,
                              ws=self.ws_l, out=self.sel)
        else:
            fa.ann_select_self(self.qcode, self.cache.code, self.cache.len, self.BQ, self.n_rep, self.BK, self.n_sel,
                               ws=self.ws_s, out=self.sel)
        mark("select_self")
        if self.kv8 is not None:
            fa.sparse_attn_fwd_fp8(Q, self.kv8[0], self.kv8[1], self.cache.cnt, self.cache.len, self.C, self.sel[0],
                                   self.sel[1], self.BQ, self.BK, self.scale, out=self.O, ws=self.ws_a)
        else:
            fa.sparse_attn_fwd(Q, self.cache.K, self.cache.V, self.cache.cnt, self.cache.len, self.sel[0], self.sel[1],
                               self.BQ, self.BK, self.scale, out=self.O, ws=self.ws_a)
        mark("attn_self")
        if self.fused_cross:   # selection and attention over it in one launch; the stage is booked under select_cross
            fa.ann_cross_attn_fwd(Q, self.qcode, self.pK, self.pV, self.pcode, self.BQ, self.n_sel_cross, self.scale,
                                  out=(self.csel[0], self.csel[1], self.Ox[0]))
            mark("select_cross")
        else:
            fa.ann_select_cross(self.qcode, self.pcode, self.BQ, self.n_sel_cross, ws=self.ws_x, out=self.csel)
            mark("select_cross")
            fa.sparse_attn_fwd(Q, self.pK, self.pV, None, self.plen, self.csel[0], self.csel[1], self.BQ, 1, self.scale,
                               out=self.Ox, want_lse=False)
        mark("attn_cross")

    def step_two_streams(self, frames, Q, mark):
        """The same step with the query codes and the whole cross-attention path (they depend on Q and the prompt only) on a
        second stream of the same priority, beside the compress calls: chains of dependent launches that leave most of
        the chip idle.  The step ends when both streams have: the main stream waits for the second one."""
        fa, t = self.fa, self.t
        main, side = t.cuda.current_stream(), self.side
        mark("start")
        first_frame = self.frame_id
        side.wait_stream(main)   # after the previous step's readers of the query codes and of the cross outputs
        with t.cuda.stream(side):
            fa.encode(Q, self.codec, out=self.qcode)
            self.ev_q.record(side)
            fa.ann_cross_attn_fwd(Q, self.qcode, self.pK, self.pV, self.pcode, self.BQ, self.n_sel_cross, self.scale,
                                  out=(self.csel[0], self.csel[1], self.Ox[0]))
        for K, V in frames:
            self.compress(K, V)
        mark("compress")
        if self.kv8 is not None:
            fa.kv_to_fp8(self.cache, self.kv8[0], self.kv8[1], stamp_lo=first_frame)
        mark("quantize")
        main.wait_event(self.ev_q)
        mark("encode")
        fa.ann_select_self(self.qcode, self.cache.code, self.cache.len, self.BQ, self.n_rep, self.BK, self.n_sel,
                           ws=self.ws_s, out=self.sel)
        mark("select_self")
        if self.kv8 is not None:
            fa.sparse_attn_fwd_fp8(Q, self.kv8[0], self.kv8[1], self.cache.cnt, self.cache.len, self.C, self.sel[0],
                                   self.sel[1], self.BQ, self.BK, self.scale, out=self.O, ws=self.ws_a)
        else:
            fa.sparse_attn_fwd(Q, self.cache.K, self.cache.V, self.cache.cnt, self.cache.len, self.sel[0], self.sel[1],
                               self.BQ, self.BK, self.scale, out=self.O, ws=self.ws_a)
        mark("attn_self")
        main.wait_stream(side)
        mark("select_cross")
        mark("attn_cross")

    def dense_equivalent_ms(self, Q, reps=3):
        """The same attention kernel with every live key block selected (the dense limit of the sparse call)."""
        t = self.t
        n_live = (int(self.cache.len.max().item()) + self.BK - 1) // self.BK
        sel = t.arange(n_live, dtype=t.int32, device=Q.device).repeat(self.H, self.n_qb, 1).contiguous()
        nsel = t.full((self.H, self.n_qb), n_live, dtype=t.int32, device=Q.device)
        O = t.empty_like(Q)
        lse = t.empty(Q.shape[:2], dtype=t.float32, device=Q.device)

        def attend():
            if self.kv8 is not None:
                self.fa.sparse_attn_fwd_fp8(Q, self.kv8[0], self.kv8[1], self.cache.cnt, self.cache.len, self.C, sel, nsel,
                                            self.BQ, self.BK, self.scale, out=(O, lse))
            else:
                self.fa.sparse_attn_fwd(Q, self.cache.K, self.cache.V, self.cache.cnt, self.cache.len, sel, nsel, self.BQ,
                                        self.BK, self.scale, out=(O, lse))
        attend()
        e0, e1 = t.cuda.Event(enable_timing=True), t.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            attend()
        e1.record()
        t.cuda.synchronize()
        return e0.elapsed_time(e1) / reps, n_live

    def gathered_bytes(self):
        """Algorithmic bytes of one self-attention launch: Q read and O written, and the K and V rows of every live key
        of every selected key block, once per query block that selected it."""
        t = self.t
        sel, nsel = self.sel
        L = self.cache.len.to(t.int64)[:, None, None]
        kb = sel.to(t.int64)
        valid = (kb >= 0) & (t.arange(self.n_sel, device=sel.device)[None, None, :] < nsel[:, :, None])
        keys = t.clamp(t.minimum((kb + 1) * self.BK, L) - kb * self.BK, min=0) * valid
        es = self.cache.K.element_size()
        return float(keys.sum().item()) * self.d * es * 2 + 2.0 * self.H * self.n_q * self.d * es

    def attended_flops(self):
        """4 * d * sum over (head, query) of the live keys in the selected blocks, for the current selection."""
        t = self.t
        sel, nsel = self.sel
        L = self.cache.len.to(t.int64)[:, None, None]
        kb = sel.to(t.int64)
        valid = (kb >= 0) & (t.arange(self.n_sel, device=sel.device)[None, None, :] < nsel[:, :, None])
        keys = t.clamp(t.minimum((kb + 1) * self.BK, L) - kb * self.BK, min=0) * valid
        q_per_block = t.full((self.n_qb,), self.BQ, device=sel.device, dtype=t.int64)
        q_per_block[-1] = self.n_q - (self.n_qb - 1) * self.BQ
        pairs = (keys.sum(dim=2) * q_per_block[None, :]).sum()
        return 4.0 * self.d * float(pairs.item())


def selection_variants(pipe, Q, cfg, torch, fa, np, to_dev, reps=3):
    """The other selection forms on the cache as the run left it, each timed on its own (events around `reps` calls, a
    warm-up call first): codes of 4 and 2 bits per entry, hash tables over sign codes, prompt-induced buckets.  What a
    variant needs beside the per-chunk call (packed codes / hash bits / bucket ids of the whole cache) is built once,
    outside the timing, as a cache that kept such metadata per slot would have it."""
    from workloads import make_sign_matrix
    H, C, d, r = pipe.H, pipe.C, pipe.d, pipe.r
    BQ, BK, n_rep, n_sel = pipe.BQ, pipe.BK, pipe.n_rep, pipe.n_sel

    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return round(e0.elapsed_time(e1) / reps, 4)

    def density(nsel):
        live_blocks = torch.clamp((pipe.cache.len + BK - 1) // BK, min=1).to(torch.float32)
        return round(float((nsel.to(torch.float32) / live_blocks[:, None]).mean().item()), 4)

    out = {"note": "per-chunk cost of the query side + the selection; ms; density = selected / live key blocks"}
    out["int8_r32"] = {"ms": timed(lambda: (fa.encode(Q, pipe.codec, out=pipe.qcode),
                                             fa.ann_select_self(pipe.qcode, pipe.cache.code, pipe.cache.len, BQ, n_rep, BK,
                                                                n_sel, ws=pipe.ws_s, out=pipe.sel))),
                       "bytes_per_key": r}
    for bits, shift in ((4, 8), (2, 9)):
        codec = fa.Codec(pipe.codec.R, pipe.codec.qscale, shift)
        kp = fa.encode_packed(pipe.cache.K, codec, bits)
        qp = fa.encode_packed(Q, codec, bits)
        sel = (torch.empty_like(pipe.sel[0]), torch.empty_like(pipe.sel[1]))
        out[f"packed_{bits}bit"] = {"ms": timed(lambda: (fa.encode_packed(Q, codec, bits, out=qp),
                                                        fa.ann_select_self_packed(qp, kp, pipe.cache.len, bits, BQ, n_rep,
                                                                                  BK, n_sel, ws=pipe.ws_s, out=sel))),
                                     "bytes_per_key": r * bits // 8, "shift": shift}
        del kp, qp
    Rb = to_dev(make_sign_matrix(cfg["seed"], cfg["cfg_id"], d, 128))
    kbits = fa.encode_sign(pipe.cache.K, Rb, pipe.codec.qscale)
    qbits = fa.encode_sign(Q, Rb, pipe.codec.qscale)
    ws_l = torch.empty(fa.workspace_bytes(fa.OP_SELECT_LSH, H, pipe.n_q, C, 128, BQ, BK, n_rep), dtype=torch.uint8, device="cuda")
    sel = (torch.empty_like(pipe.sel[0]), torch.empty_like(pipe.sel[1]))
    out["lsh_equal_bits_128"] = {"ms": timed(lambda: (fa.encode_sign(Q, Rb, pipe.codec.qscale, out=qbits),
                                                      fa.ann_select_lsh(qbits, kbits, pipe.cache.len, BQ, n_rep, BK, n_sel,
                                                                        ws=ws_l, out=sel))), "bytes_per_key": 16}
    for band, radius in ((8, 0), (8, 1)):
        ms = timed(lambda: (fa.encode_sign(Q, Rb, pipe.codec.qscale, out=qbits),
                            fa.ann_select_lsh_buckets(qbits, kbits, pipe.cache.len, band, radius, BQ, n_rep, BK, n_sel,
                                                      ws=ws_l, out=sel)))
        out[f"lsh_tables_16x{band}bit_radius{radius}"] = {"ms": ms, "bytes_per_key": 16, "density": density(sel[1])}
    del kbits, qbits, ws_l
    m = 2
    kb = fa.prompt_buckets(pipe.cache.code, pipe.pcode, m)
    assign_all = timed(lambda: fa.prompt_buckets(pipe.cache.code, pipe.pcode, m, out=kb))
    idx = pipe.prev if pipe.prev is not None else None
    assign_frame = timed(lambda: fa.prompt_buckets(pipe.cache.code, pipe.pcode, m, idx=idx, out=kb)) if idx is not None else None
    qb = fa.prompt_buckets(pipe.qcode, pipe.pcode, m)
    ws_b = torch.empty(fa.workspace_bytes(fa.OP_SELECT_BUCKETS, H, pipe.n_q, C, pipe.n_p, BQ, BK, 0), dtype=torch.uint8, device="cuda")
    ms = timed(lambda: (fa.prompt_buckets(pipe.qcode, pipe.pcode, m, out=qb),
                        fa.ann_select_buckets(qb, kb, pipe.cache.len, pipe.n_p, BQ, BK, n_sel, ws=ws_b, out=sel)))
    out["prompt_buckets_m2"] = {"ms": ms, "density": density(sel[1]), "bucket_ids_of_the_frames_slots_ms": assign_frame,
                                "bucket_ids_of_the_whole_cache_ms": assign_all, "bytes_per_key": 4 * m}
    return out


def gen_chunks(cfg, n_prefill, n_chunks, cpu_heads):
    """Host-side generation of the whole rollout (uploaded once by the caller).  Returns the prefill frames, the
    chunks [(frames, Q)], the prompt set; host arrays in storage form."""
    from workloads import FrameStream, PromptSet
    fs = FrameStream(cfg["seed"], cfg["cfg_id"], cfg["H"], cfg["d"], cfg["T"], cfg["n_c"], cfg["p"], cfg["sigma_d"],
                     cfg["dtype"])
    prefill = [fs.next_frame() for _ in range(n_prefill)]
    chunks = []
    for _ in range(n_chunks):
        frames = [fs.next_frame() for _ in range(cfg["chunk_frames"])]
        Q = fs.queries(cfg["chunk_frames"])
        chunks.append((frames, Q))
    ps = PromptSet(cfg["seed"], cfg["cfg_id"], fs.centreK, cfg["n_p"], cfg["n_pc"], cfg["n_near"], cfg["dtype"])
    return prefill, chunks, ps


def cpu_baseline(cfg, pipe, oracle_cache, oracle_prev, oracle_fid, host_chunks, ps_host, n_heads, to_host,
                 sign_matrix=None, code_shift=None):
    """The CPU oracle's own rollout on the first n_heads heads: from `oracle_cache` (its state before the first
    chunk the GPU ran) it replays every chunk of host_chunks (same inputs as the GPU); only its last chunk step is
    timed.  Returns the cpu_baseline record, time scaled to all heads."""
    import numpy as np
    import oracle
    from workloads import make_codec
    H = cfg["H"]
    codec = make_codec(cfg["seed"], cfg["cfg_id"], cfg["d"], cfg["r"])
    if code_shift is not None:
        codec.shift = code_shift
    cache = oracle_cache
    threads = len(os.sched_getaffinity(0))
    prev, fid = oracle_prev, oracle_fid

    def push(K, V):
        nonlocal prev, fid
        prev, _, st = oracle.tempcache_compress(cache, codec.R, codec.qscale, codec.shift, K, V, cand=prev,
                                                tau2_q16=pipe.tau2, frame_id=fid, rep_mode=pipe.rep_mode)
        fid += 1
        return st
    for frames, _ in host_chunks[:-1]:
        for K, V in frames:
            push(K, V)
    frames, Qh = host_chunks[-1]
    t0 = time.perf_counter()
    for K, V in frames:
        st_last = push(K, V)
    t1 = time.perf_counter()
    qc = oracle.encode(Qh, codec.R, codec.qscale, codec.shift)
    if sign_matrix is not None:
        qb = oracle.encode_sign(Qh, sign_matrix, codec.qscale)
        kb = oracle.encode_sign(cache.K, sign_matrix, codec.qscale)
        sel, nsel = oracle.ann_select_lsh(qb, kb, cache.len, pipe.BQ, pipe.n_rep, pipe.BK, pipe.n_sel)
    else:
        sel, nsel = oracle.ann_select_self(qc, cache.code, cache.len, pipe.BQ, pipe.n_rep, pipe.BK, pipe.n_sel)
    t2 = time.perf_counter()
    if pipe.kv8 is not None:   # the oracle's own 8-bit copy of ITS cache
        K8r, V8r = oracle.kv8_empty(n_heads, pipe.C, cfg["d"])
        oracle.kv_to_fp8(cache, K8r, V8r)
        O, _ = oracle.sparse_attn_fwd_fp8(Qh, K8r, V8r, cache.cnt, cache.len, pipe.C, sel, nsel, pipe.BQ, pipe.BK, pipe.scale)
    else:
        O, _ = oracle.sparse_attn_fwd(Qh, cache.K, cache.V, cache.cnt, cache.len, sel, nsel, pipe.BQ, pipe.BK, pipe.scale)
    t3 = time.perf_counter()
    pK, pV = ps_host
    pc = oracle.encode(pK, codec.R, codec.qscale, codec.shift)
    csel, cnsel = oracle.ann_select_cross(qc, pc, pipe.BQ, pipe.n_sel_cross)
    plen = np.full(n_heads, pK.shape[1], np.int32)
    Ox, _ = oracle.sparse_attn_fwd(Qh, pK, pV, None, plen, csel, cnsel, pipe.BQ, 1, pipe.scale)
    t4 = time.perf_counter()
    # parity of the GPU's last step against this replay (same inputs, same state)
    from workloads import to_f32
    hs = slice(0, n_heads)
    sel_ok = bool(np.array_equal(to_host(pipe.sel[0])[hs], sel) and np.array_equal(to_host(pipe.sel[1])[hs], nsel))
    csel_ok = bool(np.array_equal(to_host(pipe.csel[0])[hs], csel))
    len_ok = bool(np.array_equal(to_host(pipe.cache.len)[hs], cache.len))
    mm_ok = bool(np.array_equal(to_host(pipe.prev)[hs], prev))
    err = float(np.abs(to_f32(to_host(pipe.O[0][hs])).astype(np.float64) - O).max())
    errx = float(np.abs(to_f32(to_host(pipe.Ox[0][hs])).astype(np.float64) - Ox).max())
    scale = H / n_heads
    recall, density = oracle.recall_density(Qh, cache.K, cache.cnt, cache.len, sel, nsel, pipe.BQ, pipe.BK, pipe.scale,
                                            q_stride=97)
    info = {
        "value": round((t4 - t0) * 1e3 * scale, 1), "unit": "ms/chunk", "cores": threads, "kind": "oracle",
        "sample": f"heads 0..{n_heads - 1} of {H}: the oracle's own replay of the same chunks from the same starting "
                  f"cache, its last chunk step timed ({(t4 - t0):.1f} s of CPU work; the compress stage runs one thread "
                  f"per head, the other stages use all {threads}); time scaled by {scale:g} (extrapolated)",
        "stages_ms_scaled": {"compress": round((t1 - t0) * 1e3 * scale, 1), "encode+select": round((t2 - t1) * 1e3 * scale, 1),
                             "attn_self": round((t3 - t2) * 1e3 * scale, 1), "cross": round((t4 - t3) * 1e3 * scale, 1)},
        "parity_on_sample": {"sel_equal": sel_ok, "cross_sel_equal": csel_ok, "len_equal": len_ok,
                             "merge_map_equal": mm_ok,
                             "attn_self_max_abs_err": err, "attn_cross_max_abs_err": errx},
        "last_step_stats_head0": [int(x) for x in st_last[0][:5]],
        "selection_recall": round(recall, 4), "selection_density": round(density, 4),
    }
    return info


def attn_kernel_name(n_items, H, C, d=128, n_tiles=None):
    """Which bf16 d = 128, BQ = 128, BK = 64 kernel sparse_attn_fwd launches for this many (head, query block) pairs
    and this cache capacity (K and V of all heads within 256 MB: bias rows written in the matrix phase).  n_tiles: 64-key
    tiles per query block when the call carries a workspace (then a launch with a short last round is split)."""
    per_xcd = (n_items + 7) // 8
    tail = per_xcd % 64
    if n_tiles is not None and per_xcd > 64 and 0 < tail <= 24 and n_tiles * (1.2 - 0.0375 * tail) > 30.0:
        return "attn_bf16_d128_sk_kernel + attn_combine_kernel"
    if n_items <= 512 or n_items % 512 == 0 or n_items % 512 >= 256:
        resident = H * C * d * 2 * 2 <= (256 << 20)
        return "attn_bf16_d128_pp_kernel<4, true, %s>" % ("true" if resident else "false")
    return "attn_bf16_d128_kernel<4>"


TRAFFIC_FILES = {"cfg2": "cfg2_chunk_step_hbm_traffic.txt", "cfg5full": "cfg5full_chunk_step_hbm_traffic.txt"}


def profiled_traffic(workload):
    """HBM bytes per launch of the self-attention kernel for this workload as measured by the committed counter
    summary in profiles/ (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size): (bytes, file), or
    (None, None) when no summary for this workload is there.  Lines: '<kernel name> ... <fetch MB> <write MB>'."""
    name = TRAFFIC_FILES.get(workload)
    if name is None:
        return None, None
    best = None
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if "attn_bf16_d128" in line and not line.startswith("#"):
                f = line.split()
                total = (float(f[-2]) + float(f[-1])) * 1e6
                best = total if best is None else max(best, total)   # of several groups of launches: the self-attention ones
    except (OSError, ValueError):
        return None, None
    return best, ("profiles/" + name if best is not None else None)


def build_host_rollout(args, workload, torch, fa, np, to_dev, n_chunks, n_cpu_heads):
    """cfg2 / cfg5: frames generated on the host and merged into an empty cache through tempcache_compress."""
    import oracle
    from workloads import CONFIGS, make_codec, make_sign_matrix
    cfg = dict(CONFIGS[workload])
    T, cf = cfg["T"], cfg["chunk_frames"]
    cap_frames = args.cap_frames or (24 if workload == "cfg2" else cfg["cache_frames"])
    n_prefill = args.prefill_frames if args.prefill_frames is not None else cfg["cache_frames"] - cf
    C = cap_frames * T
    n_kb_quoted = (cfg["cache_frames"] * T + cfg["BK"] - 1) // cfg["BK"]
    n_sel = int(np.ceil(cfg["sel_frac"] * n_kb_quoted))
    codec_h = make_codec(cfg["seed"], cfg["cfg_id"], cfg["d"], cfg["r"])
    if args.code_shift is not None:
        codec_h.shift = args.code_shift
    codec = fa.Codec(to_dev(codec_h.R), float(codec_h.qscale), codec_h.shift)
    prefill, chunks, ps = gen_chunks(cfg, n_prefill, n_chunks, n_cpu_heads)
    dev_chunks = [([(to_dev(K), to_dev(V)) for K, V in frames], to_dev(Q)) for frames, Q in chunks]
    sign_h = make_sign_matrix(cfg["seed"], cfg["cfg_id"], cfg["d"], 128) if args.ann == "lsh" else None
    pipe = ChunkPipeline(cfg, C, args.tau, torch, fa, codec, (to_dev(ps.K), to_dev(ps.V)), n_sel,
                         sign_matrix=None if sign_h is None else to_dev(sign_h),
                         rep_mode={"last": fa.REP_LAST, "mean": fa.REP_MEAN, "medoid": fa.REP_MEDOID}[args.rep],
                         fused_cross=args.cross == "fused", ws_persistent=args.ws == "persistent")
    for K, V in prefill:
        pipe.compress(to_dev(K), to_dev(V))
    torch.cuda.synchronize()
    hs = slice(0, n_cpu_heads)
    cut = lambda a: np.ascontiguousarray(a[hs])

    def oracle_start():
        # the oracle's own prefill from an empty cache, on its heads
        cache = oracle.Cache.empty(n_cpu_heads, C, cfg["d"], cfg["r"], cfg["dtype"])
        prev = None
        for f, (K, V) in enumerate(prefill):
            prev, _, _ = oracle.tempcache_compress(cache, codec_h.R, codec_h.qscale, codec_h.shift, cut(K), cut(V), cand=prev,
                                                   tau2_q16=pipe.tau2, frame_id=f, rep_mode=pipe.rep_mode)
        return cache, prev, len(prefill)
    host_chunks = [([(cut(K), cut(V)) for K, V in frames], cut(Q)) for frames, Q in chunks]
    label = (f"{workload}: {'Wan-1.3B-shaped' if workload == 'cfg2' else 'world-model-scale'} layer rollout, H {cfg['H']} d "
             f"{cfg['d']}, chunk {cf}x{T} = {cf * T} queries, TempCache-bounded cache (cap {cap_frames} frames = {C} "
             f"slots/head, tau {args.tau}) filled through tempcache_compress from empty, AnnSA {n_sel} of {n_kb_quoted} "
             f"key blocks per query block (BQ {cfg['BQ']}, BK {cfg['BK']}), AnnCA {cfg['n_sel_cross']} of {cfg['n_p']} "
             f"prompt tokens")
    return dict(cfg=cfg, pipe=pipe, dev_chunks=dev_chunks, host_chunks=host_chunks, oracle_start=oracle_start,
                ps_host=(cut(ps.K), cut(ps.V)), sign_h=sign_h, codec_h=codec_h, label=label, n_prefill=n_prefill,
                cap_frames=cap_frames, n_sel=n_sel, n_kb_quoted=n_kb_quoted)


def build_cfg5_full(args, torch, fa, np, to_dev, to_host, n_chunks, n_cpu_heads):
    """The world-model layer on a full cache: 64 frames of the seeded device-side stream written into the cache as
    plain concatenation (multiplicity 1, stamp = frame), then the stream goes on through tempcache_compress."""
    import oracle
    from workloads import CONFIGS, PromptSet, make_codec, make_sign_matrix
    from workloads.synth_device import DeviceFrameStream
    cfg = dict(CONFIGS["cfg5"])
    H, d, r, T, cf = cfg["H"], cfg["d"], cfg["r"], cfg["T"], cfg["chunk_frames"]
    n_fill = cfg["cache_frames"]
    C = n_fill * T
    n_kb = (C + cfg["BK"] - 1) // cfg["BK"]
    n_sel = int(np.ceil(cfg["sel_frac"] * n_kb))
    codec_h = make_codec(cfg["seed"], cfg["cfg_id"], d, r)
    if args.code_shift is not None:
        codec_h.shift = args.code_shift
    codec = fa.Codec(to_dev(codec_h.R), float(codec_h.qscale), codec_h.shift)
    stream = DeviceFrameStream(cfg["seed"], cfg["cfg_id"], H, d, T, cfg["n_c"], cfg["p"], cfg["sigma_d"], cfg["dtype"])
    ps = PromptSet(cfg["seed"], cfg["cfg_id"], stream.centreK.cpu().numpy(), cfg["n_p"], cfg["n_pc"], cfg["n_near"],
                   cfg["dtype"])
    sign_h = make_sign_matrix(cfg["seed"], cfg["cfg_id"], d, 128) if args.ann == "lsh" else None
    pipe = ChunkPipeline(cfg, C, args.tau, torch, fa, codec, (to_dev(ps.K), to_dev(ps.V)), n_sel,
                         sign_matrix=None if sign_h is None else to_dev(sign_h),
                         rep_mode={"last": fa.REP_LAST, "mean": fa.REP_MEAN, "medoid": fa.REP_MEDOID}[args.rep],
                         fused_cross=args.cross == "fused", ws_persistent=args.ws == "persistent")
    cache = pipe.cache
    for f in range(n_fill):
        K, V = stream.next_frame()
        cache.K[:, f * T:(f + 1) * T] = K
        cache.V[:, f * T:(f + 1) * T] = V
        cache.stamp[:, f * T:(f + 1) * T] = f
    cache.cnt.fill_(1)
    cache.len.fill_(C)
    fa.encode(cache.K, codec, out=cache.code)
    last = torch.arange((n_fill - 1) * T, n_fill * T, dtype=torch.int32, device="cuda").repeat(H, 1).contiguous()
    pipe.prev = last          # the slots the previous frame wrote
    pipe.frame_id = n_fill
    dev_chunks = []
    for _ in range(n_chunks):
        frames = [stream.next_frame() for _ in range(cf)]
        dev_chunks.append((frames, stream.queries(cf)))
    torch.cuda.synchronize()
    hs = slice(0, n_cpu_heads)
    host_chunks = [([(to_host(K[hs]), to_host(V[hs])) for K, V in frames], to_host(Q[hs])) for frames, Q in dev_chunks]
    # the oracle's starting cache: the generator's keys and values of its heads, ITS OWN codes of them
    K0, V0 = to_host(cache.K[hs]), to_host(cache.V[hs])
    stamp0 = to_host(cache.stamp[hs])

    def oracle_start():
        oc = oracle.Cache(K=K0, V=V0, code=oracle.encode(K0, codec_h.R, codec_h.qscale, codec_h.shift),
                          cnt=np.ones((n_cpu_heads, C), np.int32), stamp=stamp0, len=np.full(n_cpu_heads, C, np.int32))
        return oc, to_host(last[hs]), n_fill
    label = (f"cfg5full: world-model-scale layer at its full size, H {H} d {d}, chunk {cf}x{T} = {cf * T} queries, cache "
             f"of {n_fill} frames = {C} live slots/head ({cache.nbytes() / 1e9:.2f} GB; seeded device-side generator, plain "
             f"concatenation), every step TempCache-merges one frame into it (tau {args.tau}) and evicts for the rest, "
             f"AnnSA {n_sel} of {n_kb} key blocks per query block (BQ {cfg['BQ']}, BK {cfg['BK']}), AnnCA "
             f"{cfg['n_sel_cross']} of {cfg['n_p']} prompt tokens")
    return dict(cfg=cfg, pipe=pipe, dev_chunks=dev_chunks, host_chunks=host_chunks, oracle_start=oracle_start,
                ps_host=(np.ascontiguousarray(ps.K[hs]), np.ascontiguousarray(ps.V[hs])), sign_h=sign_h, codec_h=codec_h,
                label=label, n_prefill=n_fill, cap_frames=n_fill, n_sel=n_sel, n_kb_quoted=n_kb)


def run_layer(args, workload, torch, fa, np, to_dev, to_host, steps, warmup, stage_steps, with_cpu, with_dense,
              with_variants=False):
    """Build one workload, time `steps` chunk steps, return its record."""
    stage_lead = 6 if stage_steps > 0 else 0   # plain steps between the host's synchronisation and the instrumented ones
    n_chunks = warmup + steps + stage_lead + stage_steps
    n_cpu_heads = min(args.cpu_heads, 40)
    t_gen = time.perf_counter()
    if workload == "cfg5full":
        B = build_cfg5_full(args, torch, fa, np, to_dev, to_host, n_chunks, n_cpu_heads)
    else:
        B = build_host_rollout(args, workload, torch, fa, np, to_dev, n_chunks, n_cpu_heads)
    t_gen = time.perf_counter() - t_gen
    cfg, pipe, dev_chunks = B["cfg"], B["pipe"], B["dev_chunks"]
    pipe.sorted_cand = args.cand == "sorted"
    n_streams = args.streams if args.streams is not None else (2 if workload.startswith("cfg5") else 1)
    if n_streams == 2:
        pipe.side = torch.cuda.Stream()   # default priority
        pipe.ev_q = torch.cuda.Event()
    fp8 = args.kv == "fp8"
    if fp8:   # the 8-bit copy of the cache as it stands, kept up to date by every step
        pipe.kv8 = fa.kv8_empty(cfg["H"], pipe.C, cfg["d"])
        fa.kv_to_fp8(pipe.cache, pipe.kv8[0], pipe.kv8[1])
    n_cpu_heads = min(n_cpu_heads, cfg["H"])
    T, cf, C = cfg["T"], cfg["chunk_frames"], pipe.C
    len_prefill = to_host(pipe.cache.len).tolist()

    for w in range(warmup):
        pipe.step(*dev_chunks[w])
    torch.cuda.synchronize()

    # Timed region: K steps; the self-attention launch of every fourth step is bracketed by events (every event is a
    # marker the queue has to drain to: about 6 us of idle chip each, so not every step carries them).
    attn_events = []
    t0 = time.perf_counter()
    for s in range(steps):
        evs = {}

        def mark(name, evs=evs):
            if name in ("select_self", "attn_self"):
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                evs[name] = e
        if s % 4 == 0:
            pipe.step(*dev_chunks[warmup + s], ev=mark)
            attn_events.append(evs)
        else:
            pipe.step(*dev_chunks[warmup + s])
    t_enqueued = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    attn_ms = sum(e["select_self"].elapsed_time(e["attn_self"]) for e in attn_events) / len(attn_events)
    flops = pipe.attended_flops()
    stats_timed = to_host(pipe.mm[(pipe.frame_id - 1) & 1][2])
    # Stage breakdown: a separate pass over the next chunks of the same rollout, an event after every stage.
    stage_names = ["compress", "quantize", "encode", "select_self", "attn_self", "select_cross", "attn_cross"]
    events = []
    side_saved, pipe.side = pipe.side, None   # the breakdown is taken with every stage on one stream, one after the other
    for s in range(stage_lead):
        pipe.step(*dev_chunks[warmup + steps + s])
    for s in range(stage_steps):
        evs = []

        def mark(name, evs=evs):
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            evs.append(e)
        pipe.step(*dev_chunks[warmup + steps + stage_lead + s], ev=mark)
        events.append(evs)
    torch.cuda.synchronize()
    pipe.side = side_saved
    if args.calib_copy_mb > 0:
        src = torch.ones(args.calib_copy_mb << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    stage_ms = {n: 0.0 for n in stage_names}
    for evs in events:
        for i, n in enumerate(stage_names):
            stage_ms[n] += evs[i].elapsed_time(evs[i + 1])
    stage_ms = {n: v / max(stage_steps, 1) for n, v in stage_ms.items()}
    tflops = flops / (attn_ms * 1e-3) / 1e12
    peak_tf = PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS
    len_final = to_host(pipe.cache.len).tolist()
    dense = pipe.dense_equivalent_ms(dev_chunks[warmup + steps - 1][1]) if with_dense else None

    # Algorithmic bytes of the bandwidth-bound stages (per chunk step), for their GB/s against the HBM peak:
    #   encode: every query row in, its code out;  select: every live code once + the query codes;
    #   compress, per frame and head: K and V rows of the frame in (2 rows), the matched slot's K row gathered, one V row
    #   read-modified-written or K and V rows written (2 rows), about 40 B of records, plus the candidate window's codes.
    H, d, r = cfg["H"], cfg["d"], cfg["r"]
    es = 2 if cfg["dtype"] == "bf16" else 4
    live = float(sum(len_final))
    bytes_stage = {
        "encode": H * pipe.n_q * (d * es + r),
        "select_self": live * r + H * pipe.n_q * r + 4.0 * H * pipe.n_qb * pipe.n_sel,
        "compress": cf * H * T * (5 * d * es + 40 + r) + cf * H * T * r,
    }
    stage_gbs = {k: round(v / (stage_ms[k] * 1e-3) / 1e9, 1) for k, v in bytes_stage.items() if stage_ms.get(k, 0) > 0}
    traffic, traffic_src = (None, None) if fp8 else profiled_traffic(workload)
    # Which roofline binds the attention launch.  Its arithmetic intensity (128 flops per gathered byte at BQ 128) is
    # below the chip's balance point, so it is the matrix roofline only while the gathered rows are served from cache.
    # The counter summary of this workload decides: when at least half of the gathered bytes come from HBM, the launch is
    # priced against the HBM roofline, with the algorithmic (gathered) bytes; the matrix-core view is kept beside it.
    gathered = pipe.gathered_bytes()
    hbm_bound = traffic is not None and traffic >= 0.5 * gathered
    gbs = gathered / (attn_ms * 1e-3) / 1e9

    result = {
        "metric": "sparse-attn ms per generated chunk", "value": round(ms_per_step, 4), "unit": "ms/chunk",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "fp8 (E4M3 K/V/Q/P, fp32 accumulation)" if fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": B["label"],
                   "ann": f"int8 projection codes (r 32, shift {B['codec_h'].shift})" if args.ann == "int8" else "sign codes, 128 hash bits (LSH variant)",
                   "self_attention_kv": "8-bit floating-point (E4M3) copy of the cache, updated per chunk by fastar_kv_to_fp8" if fp8 else "bf16 cache",
                   "representative": args.rep + " key",
                   "tempcache_workspace": args.ws,
                   "cross_attention": "one launch (ann_cross_attn_fwd)" if args.cross == "fused" else "ann_select_cross + sparse_attn_fwd",
                   "streams": "2: query codes + cross-attention on a second stream beside the compress calls, joined before "
                              "the step ends" if n_streams == 2 else "1",
                   "prefill_frames": B["n_prefill"], "cache_len_per_head_start": [min(len_prefill), max(len_prefill)],
                   "cache_len_per_head_end": [min(len_final), max(len_final)],
                   "last_timed_compress_stats_head0": {k: int(v) for k, v in zip(
                       ("len", "merged", "appended", "evicted", "dropped"), stats_timed[0][:5])},
                   "cache_bytes": pipe.cache.nbytes()},
        "stages_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "stages_note": f"separate pass of {stage_steps} steps after the timed region (and {stage_lead} plain steps, so that the "
                       f"queue is back in its steady state), one event per stage, all stages on one stream",
        "stages_hbm": {"algorithmic_bytes": {k: int(v) for k, v in bytes_stage.items()}, "achieved_GBs": stage_gbs,
                       "frac_of_peak": {k: round(v / PEAK_HBM_GBS, 4) for k, v in stage_gbs.items()},
                       "peak_GBs": PEAK_HBM_GBS},
        "effective_tflops": round(tflops, 2), "pct_mfma_peak": round(100 * tflops / peak_tf, 2),
        "roofline": {"kernel": ("attn_fp8_d128_kernel" if fp8 else attn_kernel_name(cfg["H"] * pipe.n_qb, cfg["H"], C, n_tiles=(pipe.n_sel * pipe.BK + 63) // 64 if pipe.ws_a is not None else None)) + " (block-sparse self-attention)",
                     "bound": "hbm" if hbm_bound else "mfma",
                     "achieved": round(gbs, 1) if hbm_bound else round(tflops, 2),
                     "peak": PEAK_HBM_GBS if hbm_bound else peak_tf, "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": round(gbs / PEAK_HBM_GBS, 4) if hbm_bound else round(tflops / peak_tf, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_bytes_per_launch": gathered, "flops_per_launch": flops, "avg_launch_ms": round(attn_ms, 4),
                     "launches_timed": len(attn_events),
                     "mfma_view": {"achieved": round(tflops, 2), "peak": peak_tf, "unit": "TFLOP/s", "frac": round(tflops / peak_tf, 4)},
                     "hbm_view": {"achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                                  "measured_traffic_GBs": None if traffic is None else round(traffic / (attn_ms * 1e-3) / 1e9, 1)},
                     "note": "avg_launch_ms: HIP events around the self-attention call of every fourth timed step; bound = hbm when the committed counter summary of this workload shows at least half of the gathered K/V bytes coming from HBM (no reuse in cache), else mfma"},
        "dense_equivalent": None if dense is None else {
            "ms": round(dense[0], 4), "key_blocks": dense[1], "speedup_of_sparse": round(dense[0] / attn_ms, 2),
            "note": "same kernel, every live key block of the final cache selected"},
        "host_gen_s": round(t_gen, 1),
        "host_enqueue_ms_per_step": round((t_enqueued - t0) * 1e3 / steps, 4),
    }
    if with_cpu:
        oc, oprev, ofid = B["oracle_start"]()
        result["cpu_baseline"] = cpu_baseline(cfg, pipe, oc, oprev, ofid, B["host_chunks"], B["ps_host"], n_cpu_heads,
                                              to_host, B["sign_h"], args.code_shift)
    if with_variants:
        result["selection_variants"] = selection_variants(pipe, dev_chunks[-1][1], cfg, torch, fa, np, to_dev)
    return result


def sweep_ends(args, torch, fa, np, to_dev, to_host, n_frames=129):
    """The two ends of the long-rollout sweep (cfg3, TempCache-bounded): chunk time right after the start and once
    the cap of 24 frames of slots is reached and every call evicts."""
    rows = sweep(args, torch, fa, np, to_dev, to_host, n_frames=n_frames, bounded_only=True, quiet=True)
    first = rows[1]["tempcache"]
    capped = [r_["tempcache"] for r_ in rows if r_["tempcache"]["evicted"] > 0]
    out = {"first": dict(frames=rows[1]["frames"], **first)}
    if capped:
        last = capped[-3:]
        out["capped"] = {"frames": rows[-1]["frames"], "ms": round(sum(x["ms"] for x in last) / len(last), 4),
                         "compress_ms": round(sum(x["compress_ms"] for x in last) / len(last), 4),
                         "attn_self_ms": round(sum(x["attn_self_ms"] for x in last) / len(last), 4),
                         "len_max": last[-1]["len_max"], "evicted_per_call_head0": last[-1]["evicted"],
                         "note": "mean of the last three evicting steps"}
        out["capped_over_first"] = round(out["capped"]["ms"] / first["ms"], 3)
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the hot path is per head and needs no collective); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2602_01801_amd as fa

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    fa.lib()
    fa.init()

    def to_dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    def to_host(t):
        if t.dtype == torch.bfloat16:
            return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return t.contiguous().cpu().numpy()

    if args.sweep:
        return sweep(args, torch, fa, np, to_dev, to_host, n_frames=args.sweep_frames)

    result = run_layer(args, args.workload, torch, fa, np, to_dev, to_host, args.steps, args.warmup, args.stage_steps,
                       with_cpu=not args.no_cpu_baseline, with_dense=not args.no_dense_equivalent,
                       with_variants=not args.no_extras and args.ann == "int8" and args.code_shift is None)
    result["peaks_measured"] = {"mfma_bf16_tflops": round(fa.probe_mfma_bf16(), 1),
                                "mfma_bf16_tflops_random_operands": round(fa.probe_mfma_bf16(random_operands=True), 1),
                                "stream_copy_gbs": round(fa.probe_copy(), 1)}
    if args.workload == "cfg5full" and not args.no_extras:
        torch.cuda.empty_cache()
        r2 = run_layer(args, "cfg2", torch, fa, np, to_dev, to_host, 20, 3, 4, with_cpu=False, with_dense=False)
        result["cfg2"] = {k: r2[k] for k in ("ms_per_step", "stages_ms", "stages_hbm", "effective_tflops", "roofline")}
        result["cfg2"]["workload"] = r2["config"]["workload"]
        result["cfg2"]["cache_len_per_head_end"] = r2["config"]["cache_len_per_head_end"]
        torch.cuda.empty_cache()
        result["cfg3_sweep_ends"] = sweep_ends(args, torch, fa, np, to_dev, to_host)
    line = json.dumps(result)
    print(line, flush=True)
    if args.out:
        os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
        with open(args.out, "w") as f:
            f.write(line + "\n")


def sweep(args, torch, fa, np, to_dev, to_host, n_frames, bounded_only=False, quiet=False):
    """Long-rollout sweep of the Wan-shaped layer: the cache grows 3 frames per step up to n_frames;
    each step is run TempCache-bounded (cap 24 frames of slots) and uncompressed (plain concatenation)."""
    from workloads import CONFIGS, FrameStream, PromptSet, make_codec
    cfg = dict(CONFIGS["cfg3"])
    T, cf, H, d, r = cfg["T"], cfg["chunk_frames"], cfg["H"], cfg["d"], cfg["r"]
    cap = cfg["cap_frames"] * T
    codec_h = make_codec(cfg["seed"], cfg["cfg_id"], d, r)
    codec = fa.Codec(to_dev(codec_h.R), float(codec_h.qscale), codec_h.shift)
    fs = FrameStream(cfg["seed"], cfg["cfg_id"], H, d, T, cfg["n_c"], cfg["p"], cfg["sigma_d"], cfg["dtype"])
    ps = PromptSet(cfg["seed"], cfg["cfg_id"], fs.centreK, cfg["n_p"], cfg["n_pc"], cfg["n_near"], cfg["dtype"])
    prompt = (to_dev(ps.K), to_dev(ps.V))
    n_kb_quoted = (21 * T + cfg["BK"] - 1) // cfg["BK"]
    n_sel = int(np.ceil(cfg["sel_frac"] * n_kb_quoted))
    bounded = ChunkPipeline(cfg, cap, args.tau, torch, fa, codec, prompt, n_sel)
    plain = None if bounded_only else ChunkPipeline(cfg, n_frames * T, 2.0 ** 0.5, torch, fa, codec, prompt, n_sel)   # tau^2 = 2: never merges
    rows = []
    spacer = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
    for step in range(n_frames // cf):
        frames = [tuple(to_dev(a) for a in fs.next_frame()) for _ in range(cf)]
        Q = to_dev(fs.queries(cf))
        row = {"frames": (step + 1) * cf}
        for name, pipe in (("tempcache", bounded), ("uncompressed", plain)):
            if pipe is None:
                continue
            evs = []

            def mark(nm, evs=evs):
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                evs.append(e)
            torch.cuda.synchronize()
            # a spacer of plain device work in front: the step's launches are all enqueued while it runs, so the events
            # time the GPU's work on a busy, clocked-up chip and not the host's launch rate on an idle one
            for _ in range(12):
                spacer.add_(1)
            pipe.step(frames, Q, ev=mark)
            torch.cuda.synchronize()
            ms = evs[0].elapsed_time(evs[-1])
            L = to_host(pipe.cache.len)
            live_bytes = int(L.sum()) * (2 * d * 2 + r + 8)
            row[name] = {"ms": round(ms, 3), "attn_self_ms": round(evs[4].elapsed_time(evs[5]), 4),
                         "select_self_ms": round(evs[3].elapsed_time(evs[4]), 4),
                         "compress_ms": round(evs[0].elapsed_time(evs[1]), 4),
                         "len_max": int(L.max()), "live_cache_MB": round(live_bytes / 1e6, 1),
                         "evicted": int(to_host(pipe.mm[(pipe.frame_id - 1) & 1][2])[0, 3])}
        rows.append(row)
        if not quiet:
            print(json.dumps(row), flush=True)
    if args.out and not quiet:
        os.makedirs(os.path.dirname(os.path.abspath(args.out)), exist_ok=True)
        with open(args.out, "w") as f:
            for row in rows:
                f.write(json.dumps(row) + "\n")
    return rows


if __name__ == "__main__":
    main()
