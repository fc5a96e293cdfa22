"""Host-side checks of the workload tables (no GPU): kept dimensions, the
algorithmic byte model, and the byte model against the model sizes the paper
prints (tests/golden/model_size_table.txt)."""
import os

import numpy as np
import pytest

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "model_size_table.txt")


def test_kept_dims_match_benchmark_configs():
    assert wl.kept_dim(1024, 15) == 870
    assert wl.kept_head_dim(64, 15) == 54
    assert [wl.kept_head_dim(128, p) for p in (0, 15, 25, 35)] == [128, 108, 96, 82]
    assert [wl.kept_dim(14336, p) for p in (0, 15, 35)] == [14336, 12185, 9318]
    assert wl.kept_dim(18944, 25) == 14208
    assert wl.kept_dim(5120, 15) == 4352
    ip, op = wl.mamba2_2p7b_layer(15)
    assert ip.n_keep == 2 * 4352 + 336 and op.k_keep == 4352


def test_algorithmic_bytes_llama_layer():
    """Per-linear bytes at M = 1: nibbles + 2.5 B per touched group + x + y."""
    mb = {s.name: s.algorithmic_bytes(1) / 1e6 for s in wl.llama3_8b_layer(0)}
    assert mb["q_proj"] == pytest.approx(8.733, abs=2e-3)
    assert mb["k_proj"] == pytest.approx(2.189, abs=2e-3)
    assert mb["gate_proj"] == pytest.approx(30.544, abs=2e-3)
    assert mb["down_proj"] == pytest.approx(30.544, abs=2e-3)
    total = {p: sum(s.algorithmic_bytes(1) for s in wl.llama3_8b_layer(p)) / 1e6 for p in (0, 15, 35)}
    assert total[0] == pytest.approx(113.48, abs=0.02)
    assert total[15] == pytest.approx(96.38, abs=0.05)
    assert total[35] == pytest.approx(73.69, abs=0.05)


def _weight_bytes(specs, per_group_bytes):
    b = 0.0
    for s in specs:
        b += s.n_keep * s.k_keep / 2 + s.n_keep * s.groups_touched() * per_group_bytes
    return b


@pytest.mark.parametrize("model,layers,vocab,hidden,layer_fn", [
    ("llama-3.1-8b", 32, 128256, 4096, wl.llama3_8b_layer),
    ("qwen-2.5-7b", 28, 152064, 3584, wl.qwen25_7b_layer),
])
def test_byte_model_against_paper_model_sizes(model, layers, vocab, hidden, layer_fn):
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    table = {(m, int(b), int(p)): float(gb) for m, b, p, gb in rows}
    emb_params = 2 * vocab * hidden                      # embedding + output layer
    fp16 = (sum(s.N * s.K for s in layer_fn(0)) * layers + emb_params) * 2 / 1e9
    assert fp16 == pytest.approx(table[(model, 16, 0)], abs=0.1)
    for p in (0, 35):
        # symmetric 4-bit: half a byte per weight plus an fp16 scale per 128 weights
        body = _weight_bytes(layer_fn(p), 2.0) * layers
        emb = emb_params * (0.5 + 2.0 / 128)
        assert (body + emb) / 1e9 == pytest.approx(table[(model, 4, p)], abs=0.1)


def test_generators_are_seeded_and_in_range():
    a = wl.gen_linear(wl.rng_for(0), 64, 256)
    b = wl.gen_linear(wl.rng_for(0), 64, 256)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert a["qweight"].dtype == np.uint32 and a["scales"].dtype == np.float16 and a["zeros"].dtype == np.uint8
    assert a["zeros"].max() <= 15 and 0.005 <= float(a["scales"].min()) and float(a["scales"].max()) <= 0.02
    r = wl.gen_rope_inputs(wl.rng_for(0, 1), wl.small_rope())
    assert r["q"].shape == (1, 8, 54) and r["k"] is None and r["kept_idx"].shape == (8, 27)
    for row in r["kept_idx"]:
        assert len(set(row.tolist())) == 27 and row.min() >= 0 and row.max() < 32
