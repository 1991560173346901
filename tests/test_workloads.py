"""The seeded input generators: determinism, shapes, storage formats, and the structure they promise."""
import numpy as np

from workloads import CONFIGS, FrameStream, PromptSet, bf16_bits_to_f32, f32_to_bf16_bits, make_codec, to_f32


def test_bf16_round_trip_and_ties_to_even():
    x = np.array([1.0, 1.0078125, 1.00390625, 1.01171875, -2.5, 0.0], np.float32)
    b = f32_to_bf16_bits(x)
    # bf16 spacing at 1 is 2^-7.  1 + 2^-8 is half way between 1 and 1 + 2^-7: ties to the even mantissa (1.0);
    # 1 + 3*2^-8 is half way between 1 + 2^-7 and 1 + 2^-6: ties up to the even 1 + 2^-6
    assert bf16_bits_to_f32(b).tolist() == [1.0, 1.0078125, 1.0, 1.015625, -2.5, 0.0]
    y = bf16_bits_to_f32(b)
    assert np.array_equal(f32_to_bf16_bits(y), b)


def test_streams_are_deterministic_and_shaped():
    for name in ("cfg1", "cfg2"):
        c = CONFIGS[name]
        if name == "cfg2":
            c = dict(c, H=2)
            a = FrameStream(c["seed"], c["cfg_id"], 2, c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
            b = FrameStream(c["seed"], c["cfg_id"], 2, c["d"], c["T"], c["n_c"], c["p"], c["sigma_d"], c["dtype"])
        else:
            a, b = FrameStream.from_config(name), FrameStream.from_config(name)
        Ka, Va = a.next_frame(); Kb, Vb = b.next_frame()
        assert Ka.shape == (c["H"], c["T"], c["d"]) and np.array_equal(Ka, Kb) and np.array_equal(Va, Vb)
        assert Ka.dtype == (np.float32 if c["dtype"] == "fp32" else np.uint16)
        assert np.array_equal(a.next_frame()[0], b.next_frame()[0])
        assert a.queries(2).shape == (c["H"], 2 * c["T"], c["d"])


def test_frames_repeat_with_small_drift_on_a_fraction_p_of_tokens():
    c = CONFIGS["cfg1"]
    fs = FrameStream.from_config("cfg1")
    K0, _ = fs.next_frame(); K1, _ = fs.next_frame()
    dist = np.sqrt(((K1 - K0) ** 2).sum(axis=2))                         # [H, T]
    near = dist < 4 * c["sigma_d"] * np.sqrt(c["d"])
    assert abs(near.mean() - c["p"]) < 0.08
    assert np.array_equal(near[0], near[1])                               # the drift mask is shared by heads
    assert dist[~near].min() > 1.0                                        # re-drawn tokens are far away


def test_codec_and_prompt_structure():
    c = CONFIGS["cfg2"]
    codec = make_codec(0, 2, c["d"], c["r"])
    assert codec.R.shape == (128, 32) and set(np.unique(codec.R)) == {-1, 1}
    assert codec.qscale == np.float32(127 / 4.5) and codec.shift == 4
    fs = FrameStream(0, 4, 2, 128, 1560, 64, 0.8, 0.02, "bf16")
    ps = PromptSet(0, 4, fs.centreK, 512, 32, 3, "bf16")
    assert ps.K.shape == (2, 512, 128) and ps.K.dtype == np.uint16 and ps.near_clusters.size == 3
    # tokens of the 'near' clusters sit next to some query-cluster centre, the others do not
    K = to_f32(ps.K)[0]
    dmin = np.sqrt(((K[:, None, :] - fs.centreK[0][None, :, :]) ** 2).sum(axis=2)).min(axis=1)
    is_near = np.isin(ps.cluster, ps.near_clusters)
    assert dmin[is_near].max() < dmin[~is_near].min()
