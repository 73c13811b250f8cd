"""The seeded input recipes: determinism, shapes, and the bf16 bit conversion
(checked against torch's own float32 -> bfloat16 cast).  CPU only."""
import numpy as np
import torch

from paper_2604_24013_amd import inputs


def test_bf16_bits_match_torch_cast():
    rng = np.random.default_rng(0)
    a = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(0.02),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, -1e-30, 65504.0], dtype=np.float32),
    ])
    bits = inputs.f32_to_bf16_bits(a)
    t = torch.from_numpy(a).to(torch.bfloat16)
    want = t.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, want)
    back = inputs.bf16_bits_to_f32(bits)
    assert np.array_equal(back, t.to(torch.float32).numpy())


def test_streams_are_deterministic_and_distinct():
    w = inputs.scaled(inputs.CONFIGS["c2_rs_7b"], m_chunk=8, n=16, k=24)
    a = inputs.make_rs(w)
    b = inputs.make_rs(w)
    assert np.array_equal(a["A"], b["A"]) and np.array_equal(a["W"], b["W"])
    assert all(np.array_equal(x, y) for x, y in zip(a["R"][1:], b["R"][1:]))
    assert a["A"].dtype == np.uint16 and a["A"].shape == (64, 24) and a["W"].shape == (24, 16)
    assert a["R"][0] is None and len(a["R"]) == 8 and a["R"][3].shape == (8, 16) and a["R"][3].dtype == np.float32
    assert not np.array_equal(a["R"][1], a["R"][2])
    c = inputs.make_rs(w, salt=1)
    assert not np.array_equal(a["A"], c["A"])


def test_config_shapes_follow_the_benchmark_list():
    c = inputs.CONFIGS
    assert (c["c1_rs_f32"].p, c["c1_rs_f32"].m_chunk, c["c1_rs_f32"].k, c["c1_rs_f32"].n) == (2, 128, 512, 256)
    assert (c["c2_rs_7b"].p * c["c2_rs_7b"].m_chunk, c["c2_rs_7b"].k, c["c2_rs_7b"].n) == (4096, 11008 // 8, 4096)
    assert (c["c3_ag_7b"].m_chunk, c["c3_ag_7b"].k, c["c3_ag_7b"].n) == (512, 4096, 3 * 4096 // 8)
    assert (c["c4_ag_70b_up"].p * c["c4_ag_70b_up"].m_chunk, c["c4_ag_70b_up"].k, c["c4_ag_70b_up"].n) == (8192, 8192, 28672 // 8)
    assert (c["c4_rs_70b_down"].k, c["c4_rs_70b_down"].n) == (28672 // 8, 8192)
    assert c["c5_dp"].p * c["c5_dp"].m_chunk == 1_000_000_000


def test_value_distributions():
    w = inputs.scaled(inputs.CONFIGS["c3_ag_7b"], m_chunk=64, n=32, k=256)
    d = inputs.make_ag(w)
    x = inputs.as_f64(d["X"], "bf16")
    assert abs(x.std() - 0.02) < 0.002 and abs(x.mean()) < 0.002
    w5 = inputs.scaled(inputs.CONFIGS["c5_dp"], m_chunk=4096)
    g = inputs.make_dp(w5)
    assert g["bucket"].shape == (8 * 4096,) and abs(g["bucket"].std() - 1e-3) < 1e-4
    assert abs(g["R"][7].std() - 1e-3) < 1e-4
