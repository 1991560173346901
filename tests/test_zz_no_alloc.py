"""The entry point that allocates nothing: ann_select_self_static against ann_select_self.

Runs last (file name), through the C ABI, two calls in a row on the shared static scratch, the second with a
smaller input; outputs must be bit-identical to the workspace-taking entry point's.
"""
import ctypes

import numpy as np
import pytest
import torch

import paper_2602_01801_amd as fa

pytestmark = pytest.mark.gpu


def codes(rng, *shape):
    return torch.from_numpy(rng.integers(-60, 61, size=shape).astype(np.int8)).cuda()


def run_both(rng, H, n_q, C, lens, r, BQ, n_rep, BK, n_sel):
    L = fa.lib()
    qc, kc = codes(rng, H, n_q, r), codes(rng, H, C, r)
    length = torch.tensor(lens, dtype=torch.int32, device="cuda")
    n_qb = (n_q + BQ - 1) // BQ
    sel_ref, nsel_ref = fa.ann_select_self(qc, kc, length, BQ, n_rep, BK, n_sel)
    sel = torch.full((H, n_qb, n_sel), -7, dtype=torch.int32, device="cuda")
    nsel = torch.full((H, n_qb), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = L.ann_select_self_static(qc.data_ptr(), n_q, kc.data_ptr(), length.data_ptr(), H, C, r, BQ, n_rep, BK, n_sel,
                                  sel.data_ptr(), nsel.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == 0, L.fastar_strerror(rc).decode()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(nsel, nsel_ref)
    assert torch.equal(sel, sel_ref)
    assert int(nsel.min()) >= 0


def test_static_scratch_selection_matches_the_workspace_one_twice_in_a_row():
    rng = np.random.default_rng(42)
    fa.init()
    # a Wan-shaped call (ragged cache lengths, rows that span several scan chunks), then a much smaller one that
    # leaves most of the first call's scratch contents in place
    run_both(rng, 3, 4680, 64 * 600, [38400, 31111, 64 * 599 + 1], 32, 128, 4, 64, 60)
    run_both(rng, 2, 300, 64 * 40, [2560, 777], 32, 128, 4, 64, 7)
    # and through the binding, r = 64
    qc, kc = codes(rng, 2, 200, 64), codes(rng, 2, 640, 64)
    length = torch.tensor([640, 333], dtype=torch.int32, device="cuda")
    ref = fa.ann_select_self(qc, kc, length, 64, 8, 32, 4)
    out = (torch.empty_like(ref[0]), torch.empty_like(ref[1]))
    fa.ann_select_self_static(qc, kc, length, 64, 8, 32, 4, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out[0], ref[0]) and torch.equal(out[1], ref[1])


def test_static_scratch_rejects_problems_beyond_its_size():
    L = fa.lib()
    fake = ctypes.c_void_p(0x10000)
    # 64 heads x 37 query blocks x 8192 key blocks of scores = 77 MB > 32 MB: refused on the host, nothing launched
    rc = L.ann_select_self_static(fake, 4680, fake, fake, 64, 64 * 8192, 32, 128, 4, 64, 52, fake, fake, None)
    assert rc == -5 and b"static scratch" in L.fastar_strerror(rc)
    assert fa.workspace_bytes(fa.OP_SELECT_SELF, 40, 3600, 230400, 32, 128, 64, 4) <= 32 * 1024 * 1024
