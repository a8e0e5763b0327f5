"""The seeded input generators: determinism, the counter-based generator against a
big-integer restatement, and the statistical / structural recipe of each workload."""
import numpy as np
import torch

import synth_inputs as si


def test_counter_rng_matches_big_integer_arithmetic():
    key = si.stream_key(si.BASE_SEED, 3, 1, 4)
    bits = si.raw_bits(16, key, offset=5)
    mask = (1 << 64) - 1
    expect = [si.mix64_int((key + (5 + i) * 0x9E3779B97F4A7C15) & mask) for i in range(16)]
    assert [int(v) & mask for v in bits.tolist()] == expect


def test_streams_are_position_addressed_and_distinct():
    a = si.normal((1000,), 7)
    b = si.normal((10, 100), 7)
    assert torch.equal(a, b.reshape(-1))
    c = si.normal((1000,), 8)
    assert not torch.equal(a, c)
    assert si.stream_key(1, 2, 3) != si.stream_key(1, 3, 2)


def test_normal_moments():
    x = si.normal((400, 500), 99, std=1e-3).double()
    assert abs(x.mean().item()) < 1e-5
    assert abs(x.std().item() / 1e-3 - 1) < 1e-2
    k4 = ((x / 1e-3) ** 4).mean().item()
    assert abs(k4 - 3.0) < 0.1


def test_gradient_recipe_lowrank_plus_noise():
    sig = si.make_signal(96, 160, 8, "1/i", 5)
    A = sig.A.double(); B = sig.sB.double()
    assert torch.allclose(A.T @ A, torch.eye(8, dtype=torch.float64), atol=1e-6)
    s = torch.linalg.norm(B, dim=0)
    assert torch.allclose(s, 1.0 / torch.arange(1, 9, dtype=torch.float64), atol=1e-6)
    g0 = si.gradient(sig, 0.0, 1)
    assert torch.linalg.matrix_rank(g0.double(), tol=1e-5).item() == 8
    g1 = si.gradient(sig, 1e-3, 1); g2 = si.gradient(sig, 1e-3, 2)
    assert abs((g1 - g0).std().item() / 1e-3 - 1) < 0.05
    assert not torch.equal(g1, g2)
    gb = si.gradient(sig, 1e-3, 1, dtype=torch.bfloat16)
    assert gb.dtype == torch.bfloat16 and torch.equal(gb, g1.to(torch.bfloat16))


def test_zipf_ids_and_embedding_gradient():
    ids = si.zipf_ids(256 * 1024, si.VOCAB, 1.1, 13)
    assert ids.min() >= 0 and ids.max() < si.VOCAB
    distinct = torch.unique(ids).numel()
    assert 15000 < distinct < 26000          # about 20k of 32000 rows are touched
    counts = torch.bincount(ids, minlength=si.VOCAB)
    assert counts[0] > counts[10] > counts[1000]
    g, rows = si.embedding_gradient(2000, 16, si.zipf_ids(500, 2000, 1.1, 14), 15)
    nz = (g != 0).any(dim=1).nonzero().flatten()
    assert torch.equal(nz, rows)
    assert abs(g[rows].std().item() / 1e-2 - 1) < 0.1


def test_model_shapes():
    assert len(si.model_shapes("130m")) == 84
    assert len(si.model_shapes("1b")) == 168
    assert si.layer_shapes("130m") == [(768, 768)] * 4 + [(768, 2048)] * 2 + [(2048, 768)]
    w = si.workload("llama-1b")
    assert (w.r, w.p, w.q) == (512, 16, 2) and w.g_dtype == torch.bfloat16
