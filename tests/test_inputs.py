"""Seeded input generator: determinism, chunk independence, formats, distributions (CPU)."""
import numpy as np
import torch

from paper_2512_12949_amd import inputs


def test_counter_based_prefix_and_determinism():
    a = inputs.tensor(17, (3, 1000), "normal", 1.0, "f32")
    b = inputs.tensor(17, (3000,), "normal", 1.0, "f32")
    assert np.array_equal(a.ravel(), b)
    c = inputs.tensor(17, (1200,), "normal", 1.0, "f32")
    assert np.array_equal(c, b[:1200])
    assert not np.array_equal(inputs.tensor(18, (3000,), "normal", 1.0, "f32"), b)


def test_chunk_boundary_is_invisible():
    n = inputs._CHUNK + 1000
    whole = inputs.tensor(5, (n,), "uniform", 1.0, "f32")
    tail = inputs._raw(5, inputs._CHUNK - 10, 1010, "uniform").astype(np.float32)
    assert np.array_equal(whole[inputs._CHUNK - 10:], tail)


def test_distributions():
    x = inputs.tensor(1, (1 << 20,), "normal", 1.0, "f32").astype(np.float64)
    assert abs(x.mean()) < 5e-3 and abs(x.std() - 1.0) < 5e-3
    assert abs((x ** 4).mean() - 3.0) < 0.05
    u = inputs.tensor(2, (1 << 20,), "uniform", 1.0, "f32").astype(np.float64)
    assert u.min() >= -1.0 and u.max() <= 1.0 and abs(u.mean()) < 5e-3
    assert abs(u.var() - 1.0 / 3.0) < 5e-3


def test_bf16_rounding_is_rne_like_torch():
    v = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * np.float32(3.0)
    v[:4] = np.float32([1.00390625, 1.01171875, -1.00390625, 0.0])  # exact ties
    got = inputs.round_to_bf16_bits(v)
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    assert np.array_equal(inputs.bf16_bits_to_f32(got),
                          torch.from_numpy(v).to(torch.bfloat16).float().numpy())


def test_workload_tables():
    w = inputs.WORKLOADS
    assert w["gpt"].shape == (4096, 4096, 16384, 4096) and not w["gpt"].gated
    assert w["llama"].shape == (2048, 4096, 11008, 4096) and w["llama"].gated
    assert w["decode16"].shape == (16, 8192, 28672, 8192)
    assert w["large"].shape == (32768, 1024, 8192, 1024) and w["large"].dtype == "f16"
    assert w["G5"].shape == (128, 4096, 16384, 4096)      # GPT-6.7B row of the GEMM-chain table
    assert w["S3"].shape == (128, 4096, 11008, 4096)      # Llama-2-7b row of the gated table
    assert w["gpt"].flops() == 2 * 4096 * 16384 * (4096 + 4096)
    assert w["gpt"].q_min() == 320 * 2 ** 20 and w["gpt"].q_unfused() == 576 * 2 ** 20
    assert w["large"].q_unfused() == 1184 * 2 ** 20


def test_make_scales_and_row_prefix():
    w = inputs.custom("t", 64, 256, 512, 128, dtype="f32", dist="normal")
    t = inputs.make(w)
    assert t["W3"] is None and t["X"].shape == (64, 256)
    assert abs(t["W1"].astype(np.float64).std() - 256 ** -0.5) < 2e-3
    assert abs(t["W2"].astype(np.float64).std() - 512 ** -0.5) < 2e-3
    assert np.array_equal(inputs.make(w, m_rows=5)["X"], t["X"][:5])


def test_sample_rows():
    r = inputs.sample_rows(1000, 256, 4, 1)
    assert r[0] == 0 and r[-1] == 999 and np.all(np.diff(r) > 0)
    for b in range(4):
        lo, hi = b * 256, min(1000, (b + 1) * 256)
        assert lo in r and hi - 1 in r


def _golden_tables():
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "shape_tables.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                parts = line.split()
                rows[parts[0]] = [int(v) for v in parts[1:]]
    return rows


def test_chain_workloads_match_the_papers_printed_tables():
    """G1-G10 / S1-S8 (Evaluation, tables of gemm-chain and gated-FFN configurations): the
    paper prints (m, n, k, l); the workloads use (M, K, N1, N2) = (m, k, n, l)."""
    rows = _golden_tables()
    for name, (m, n, k, l) in ((k_, v) for k_, v in rows.items() if k_[0] in "GS"):
        w = inputs.WORKLOADS[name]
        assert (w.M, w.K, w.N1, w.N2) == (m, k, n, l), name
        assert w.gated == (name[0] == "S")
    assert sum(1 for k_ in rows if k_[0] == "G") == 10 and sum(1 for k_ in rows if k_[0] == "S") == 8


def test_conv_workloads_match_the_papers_printed_table():
    """C1-C8 (Evaluation, table of conv-chain configurations): IC, H, W, OC1, OC2, k1, k2."""
    rows = _golden_tables()
    names = [k_ for k_ in rows if k_[0] == "C"]
    assert len(names) == 8
    for name in names:
        w = inputs.CONV_WORKLOADS[name]
        assert [w.IC, w.H, w.W, w.OC1, w.OC2, w.k1, w.k2] == rows[name], name
        M, K, N1, N2 = w.gemm_shape()
        assert (M, K, N1, N2) == (w.H * w.W, w.k1 ** 2 * w.IC, w.OC1, w.OC2)
    ops = inputs.make_conv(inputs.CONV_WORKLOADS["C8"])
    assert ops["X"].shape == (1, 7, 7, 512) and ops["W1"].shape == (3, 3, 512, 512) and ops["W2"].shape == (1, 1, 512, 2048)
