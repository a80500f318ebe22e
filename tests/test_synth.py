"""Workload tables, the seeded generators, and the compression accounting used by the
heterogeneous-encoder sampler (pinned to the figures the paper prints)."""
import os

import numpy as np

from paper_2206_15014_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table4_heterogeneous_configs.txt")
SCHEME = {"Q4": (4, 4, 4), "Q8": (4, 4, 8), "S4": (2, 4, 4), "S8": (2, 4, 8)}


def test_accounting_reproduces_printed_ratios():
    params = [1, 1, 1, 1, 4, 4]                                 # Q, K, V, AO = H^2; FFN1, FFN2 = 4 H^2
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for task, *cols in rows:
        schemes = [SCHEME[c] for c in cols[:6]]
        ratio, flop = synth.encoder_accounting(schemes, params)
        assert abs(100 * ratio - float(cols[6])) < 0.051, task
        if task not in ("SST-2", "QNLI"):
            assert abs(100 * flop - float(cols[7])) < 0.051, task
        else:
            assert abs(100 * flop - 20.8) < 0.051


def test_table_of_chosen_configurations_is_the_printed_one():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert {r[0]: tuple(r[1:7]) for r in rows} == synth.TABLE4
    assert synth.TABLE4_SCHEME == SCHEME
    gs = synth.table4_encoder("RTE")
    assert len(gs) == 72 and len({g.seed for g in gs}) == 72
    assert [(g.name, g.K, g.O, g.N, g.M, g.bits) for g in gs[:6]] == [
        ("query", 768, 768, 4, 4, 4), ("key", 768, 768, 2, 4, 4), ("value", 768, 768, 4, 4, 4),
        ("attn_out", 768, 768, 2, 4, 8), ("ffn_up", 768, 3072, 4, 4, 4), ("ffn_down", 3072, 768, 2, 4, 4)]
    ratio, flop = synth.encoder_accounting([(g.N, g.M, g.bits) for g in gs], [g.K * g.O for g in gs])
    assert abs(100 * ratio - 88.5) < 0.051 and abs(100 * flop - 25.0) < 0.051


def test_size_column_of_glue_table():
    # Sec. 5.1 table: 324M dense encoder stack; 51.7M at 8-bit 2:4 and 31.4M at 4-bit 2:4
    # (the printed sizes carry about 1 MiB of unquantised biases / norms on top).
    dense_mib = 12 * 12 * 768 * 768 * 4 / 2 ** 20
    assert round(dense_mib) == 324
    assert 0 < 51.7 - dense_mib * synth.stored_fraction(2, 4, 8) < 1.5
    assert 0 < 31.4 - dense_mib * synth.stored_fraction(2, 4, 4) < 1.5
    # nominal figure quoted in the running text of Sec. 5.1 leaves index bits out
    assert 1 - (2 / 4) * (4 / 32) == 0.9375


def test_workload_tables():
    c2, c3, c4, c5 = synth.config2(), synth.config3(), synth.config4(), synth.config5()
    assert [(g.K, g.O) for g in c2] == [(768, 2304), (768, 768), (768, 3072), (3072, 768)]
    assert all(g.T == 4096 and (g.N, g.M, g.bits) == (2, 4, 8) for g in c2)
    assert [(g.K, g.O) for g in c3] == [(1024, 3072), (1024, 1024), (1024, 4096), (4096, 1024)]
    assert all(g.T == 12288 for g in c3)
    assert len(c4) == 8 and {(g.N, g.M, g.bits) for g in c4} == {(1, 4, 4), (2, 8, 4)}
    assert len(c5) == 48 and len({g.seed for g in c5}) == 48
    assert {(g.N, g.M, g.bits) for g in c5} <= set(synth.CONFIG5_OPTIONS)
    ratio, _ = synth.encoder_accounting([(g.N, g.M, g.bits) for g in c5], [g.K * g.O for g in c5])
    assert 0.875 <= ratio <= 0.90
    assert [(g.N, g.M, g.bits) for g in c5] == [(g.N, g.M, g.bits) for g in synth.config5()]


def test_generators_are_seeded_and_shaped():
    g = synth.Gemm("t", 64, 768, 32, 2, 4, 8, (9, 0, 0))
    W, (Xq, s), b = synth.weights(g), synth.activations(g), synth.bias(g)
    assert W.shape == (32, 768) and W.dtype == np.float32 and 0.015 < W.std() < 0.025
    assert Xq.shape == (64, 768) and Xq.dtype == np.int8 and np.abs(Xq.astype(int)).max() == 127
    assert b.shape == (32,)
    assert np.array_equal(W, synth.weights(g)) and np.array_equal(Xq, synth.activations(g)[0])
    x = synth.activations_fp32(g)
    loud = (x.std(axis=0) > 5).sum()
    assert loud == 8                                            # 1 % of 768 channels scaled by 10
    g1, W1, X1, s1 = synth.config1_tensors()
    assert W1.shape == (768, 768) and X1.shape == (128, 768) and (g1.N, g1.M, g1.bits) == (2, 4, 8)
    assert np.float32(np.abs(X1.astype(np.float32) * s1).max()) > 3.0


def test_activation_quantiser_closed_forms():
    x = np.array([[12.7, -12.7, 0.05, 0.15, -0.25, 6.35]], np.float32)
    q, s = synth.quantize_activations(x)
    assert s == np.float32(12.7) / np.float32(127)
    assert q[0, 0] == 127 and q[0, 1] == -127
    q0, s0 = synth.quantize_activations(np.zeros((2, 4), np.float32))
    assert s0 == 1.0 and not q0.any()
