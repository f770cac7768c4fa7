"""The seeded input generators: determinism, uniqueness, shapes, bf16 rounding."""
import numpy as np
import torch

import synth


def test_frames_are_unique_in_grid_and_deterministic():
    for cid, n in ((1, None), (2, None), (3, 20000), (5, 30000)):
        cfg = synth.CONFIGS[cid]
        a, b = synth.make_frame(cid, n=n), synth.make_frame(cid, n=n)
        assert a.dtype == np.int32 and np.array_equal(a, b)
        per = cfg["n"] if n is None else n
        assert a.shape == (per * cfg["batch"], 4)
        assert len(np.unique(a, axis=0)) == len(a)
        assert a.min() >= 0 and np.all(a[:, 1:] < np.array(cfg["grid"])) and a[:, 0].max() == cfg["batch"] - 1


def test_skewed_frame_has_lone_and_crowded_windows():
    cfg = synth.CONFIGS[5]
    c = synth.make_frame(5)
    L, W, H = cfg["win"]
    key = ((c[:, 0] * 64 + c[:, 1] // L) * 64 + c[:, 2] // W) * 64 + c[:, 3] // H
    cnt = np.unique(key, return_counts=True)[1]
    assert cnt.min() == 1 and cnt.max() > 1500


def test_bf16_rounding_matches_torch():
    x = synth.make_features(5, 1000, 16, "f32")
    want = torch.tensor(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(synth.round_bf16(x), want)
    assert np.array_equal(synth.bf16_bits(x), torch.tensor(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    w = synth.make_layer_weights(1, 16, 2, 32, (4, 4, 1), "bf16")
    assert np.array_equal(synth.round_bf16(w["w_qkv"]), w["w_qkv"]) and w["rel_bias"].shape == (2, 49)
