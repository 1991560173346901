"""Helpers of the GPU parity tests: numpy storage form <-> device tensors, oracle/GPU cache mirrors."""
import numpy as np
import torch

import oracle
import paper_2602_01801_amd as fa


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy storage form (float32 / uint16 bf16 bits / ints) -> contiguous device tensor."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> numpy storage form."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def dev_codec(codec) -> fa.Codec:
    return fa.Codec(R=to_dev(codec.R), qscale=float(codec.qscale), shift=int(codec.shift))


def dev_cache(c: oracle.Cache) -> fa.Cache:
    return fa.Cache(K=to_dev(c.K), V=to_dev(c.V), code=to_dev(c.code), cnt=to_dev(c.cnt), stamp=to_dev(c.stamp),
                    len=to_dev(c.len))


def host_cache(c: fa.Cache) -> oracle.Cache:
    return oracle.Cache(K=to_host(c.K), V=to_host(c.V), code=to_host(c.code), cnt=to_host(c.cnt),
                        stamp=to_host(c.stamp), len=to_host(c.len))


def storage_to_f64(a: np.ndarray) -> np.ndarray:
    from workloads import to_f32
    return to_f32(a).astype(np.float64)


def assert_cache_equal(gpu: oracle.Cache, ref: oracle.Cache, v_tol: float):
    """Index-like state bit-exact on the live slots; mean values within v_tol."""
    assert np.array_equal(gpu.len, ref.len)
    for h in range(ref.len.size):
        L = int(ref.len[h])
        assert np.array_equal(gpu.K[h, :L], ref.K[h, :L]), f"K head {h}"
        assert np.array_equal(gpu.code[h, :L], ref.code[h, :L]), f"code head {h}"
        assert np.array_equal(gpu.cnt[h, :L], ref.cnt[h, :L]), f"cnt head {h}"
        assert np.array_equal(gpu.stamp[h, :L], ref.stamp[h, :L]), f"stamp head {h}"
        dv = np.abs(storage_to_f64(gpu.V[h, :L]) - storage_to_f64(ref.V[h, :L]))
        assert dv.max(initial=0.0) <= v_tol, f"V head {h}: {dv.max()}"
