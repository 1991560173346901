"""Host-side checks of bench.py that need no GPU: the one-GPU rule, the kernel the roofline is quoted on, and the
traffic figure read from profiles/."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)
    assert '"metric"' not in p.stdout                       # no result line


def test_roofline_kernel_name_follows_the_dispatch_rule():
    sys.path.insert(0, ROOT)
    import bench
    # cfg2: 37 query blocks x 12 heads fit one round of two-block workgroups; 12 x 37440 slots of K and V = 230 MB
    assert bench.attn_kernel_name(37 * 12, 12, 37440) == "attn_bf16_d128_pp_kernel<4, true, true>"
    assert bench.attn_kernel_name(37 * 12, 12, 196608) == "attn_bf16_d128_pp_kernel<4, true, false>"
    # cfg5: 29 x 40 = 1160 = 2 rounds of 512 + 136 (< 256): one block per workgroup
    assert bench.attn_kernel_name(29 * 40, 40, 230400) == "attn_bf16_d128_kernel<4>"
    assert bench.attn_kernel_name(29 * 40, 40, 230400, n_tiles=360).startswith("attn_bf16_d128_sk_kernel")   # with a workspace: split launch
    assert bench.attn_kernel_name(37 * 12, 12, 37440, n_tiles=52) == "attn_bf16_d128_pp_kernel<4, true, true>"
    assert bench.attn_kernel_name(1024, 40, 230400).startswith("attn_bf16_d128_pp_kernel<4, true, false")
    assert bench.attn_kernel_name(1024 + 256, 8, 1000).startswith("attn_bf16_d128_pp_kernel")
    # the same rule as the launcher's source states it
    src = open(os.path.join(ROOT, "paper_2602_01801_amd", "csrc", "attention.hip")).read()
    assert "n_items <= 512 || n_items % 512 == 0 || n_items % 512 >= 256" in src
    src = open(os.path.join(ROOT, "paper_2602_01801_amd", "csrc", "attention_d128_pp.hip")).read()
    assert "(size_t)H * (size_t)C * D * 2 * 2 <= ((size_t)256 << 20)" in src


def test_traffic_figure_is_read_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    t, src = bench.profiled_traffic("cfg2")
    assert t is not None and 50e6 < t < 400e6               # fetch + write of one self-attention launch at cfg2
    assert src == "profiles/cfg2_chunk_step_hbm_traffic.txt"
    t5, src5 = bench.profiled_traffic("cfg5full")
    assert t5 is not None and 5e9 < t5 < 14e9             # the world-model launch gathers 13.7 GB, most of it from HBM
    assert src5 == "profiles/cfg5full_chunk_step_hbm_traffic.txt"
    # a workload without a committed counter summary reports no traffic rather than another workload's
    assert bench.profiled_traffic("cfg5") == (None, None)
