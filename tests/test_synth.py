"""The seeded input generators: shapes, determinism, bf16 representability, outlier structure."""

import json
import os

import numpy as np
import pytest

from paper_2511_04063_amd import synth


def test_tiny_shapes_and_determinism():
    a = synth.make_inputs("tiny")
    b = synth.make_inputs("tiny")
    assert a["X"].shape == (1, 2048, 256) and a["X"].dtype == np.float32
    assert a["Z0"].shape == (1, 256, 256) and a["Z0"].dtype == np.float32
    assert np.array_equal(a["X"], b["X"]) and np.array_equal(a["Z0"], b["Z0"])
    c = synth.make_inputs("tiny", seed=3)
    assert not np.array_equal(a["X"], c["X"])


def test_outlier_channels_are_scaled():
    a = synth.make_inputs("tiny")
    X = a["X"][0]
    ch = a["outlier_channels"][0]
    assert len(ch) == 4 and len(set(ch.tolist())) == 4
    std = X.std(axis=0)
    others = np.delete(std, ch)
    assert np.all(std[ch] > 40.0) and np.all(others < 1.2)


def test_bf16_rounding_is_nearest_even_and_representable():
    x = np.array([1.0, 1.00390625, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -3.14159, 1e-3, 65504.0], dtype=np.float32)
    r = synth.round_to_bf16(x)
    # representable: low 16 bits are zero
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7: even mantissa wins -> 1.0
    assert r[2] == 1.0
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6: even -> 1 + 2^-6
    assert r[3] == np.float32(1.0 + 2.0 ** -6)
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)
    torch = pytest.importorskip("torch")
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, r)
    bits = synth.bf16_bits(r)
    assert bits.dtype == np.uint16
    assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), r)


def test_student_t_like_config_small():
    cfg = synth.scaled_config("7b", n=256, T=512)
    a = synth.make_inputs(cfg)
    X = a["X"][0]
    assert X.shape == (512, 256)
    assert np.array_equal(synth.round_to_bf16(X), X)      # already bf16-representable
    assert a["outlier_channels"].shape == (1, 3)          # ceil(1 % of 256)
    # heavy tails: excess kurtosis far above the Gaussian's
    body = np.delete(X, a["outlier_channels"][0], axis=1).astype(np.float64)
    k = np.mean(body ** 4) / np.mean(body ** 2) ** 2
    assert k > 6.0


def test_heads_like_config_small():
    cfg = synth.scaled_config("heads", b=3, T=256)
    a = synth.make_inputs(cfg)
    assert a["X"].shape == (3, 256, 128) and a["Z0"].shape == (3, 128, 128)
    assert a["outlier_channels"].shape == (3, 2)
    assert not np.array_equal(a["X"][0], a["X"][1])


def test_golden_file_is_consistent_with_its_config():
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_trajectory.json")
    with open(path) as f:
        gold = json.load(f)
    cfg = synth.CONFIGS["tiny"]
    assert gold["n"] == cfg.n and gold["T"] == cfg.T and gold["steps"] == cfg.steps
    assert len(gold["losses"]) == cfg.steps
    # token-mean Whip of n channels lies in (0, n]
    assert all(0.0 < v <= cfg.n for v in gold["losses"])
    assert all(b < a for a, b in zip(gold["losses"], gold["losses"][1:]))
