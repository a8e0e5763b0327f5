"""The paper's byte / memory formulas against the numbers and expressions it prints."""
import os

import pytest

from oracle import accounting as acc
import synth_inputs as si


def read_rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_dense_rows_of_main_results_table(golden_dir):
    for name, hidden, inter, layers, vocab, printed in read_rows(os.path.join(golden_dir, "main_results_adamw_bytes.txt")):
        elems = acc.dense_model_elements(int(hidden), int(inter), int(layers), int(vocab))
        gb = acc.step_bytes([elems], 4) / 1e9
        assert round(gb, 2) == pytest.approx(float(printed), abs=0.0051), (name, gb)


def test_dense_elements_from_block_list():
    # the closed form equals the sum over the block list the benchmarks use
    for model, cfg in si.LLAMA.items():
        blocks = si.model_shapes(model)
        total = sum(acc.synchronized_elements("adamw", m, n, 0) for m, n in blocks) + si.VOCAB * cfg["hidden"]
        assert total == acc.dense_model_elements(cfg["hidden"], cfg["inter"], cfg["layers"], si.VOCAB)


def test_object_and_state_sizes(golden_dir):
    points = [dict(m=512, n=1376, r=64, Vc=32000, re=16), dict(m=7, n=3, r=2, Vc=11, re=5)]
    for row in read_rows(os.path.join(golden_dir, "table_sizes.txt")):
        table, method, expr = row
        for pt in points:
            expect = eval(expr, {}, pt)
            if table == "table1":
                got = acc.synchronized_elements(method, pt["m"], pt["n"], pt["r"])
            elif table == "linear":
                got = acc.state_elements(method, "linear", pt["m"], pt["n"], pt["r"])
            else:
                got = acc.state_elements(method, "embedding", pt["Vc"], pt["m"], pt["re"])
            assert got == expect, row


def test_bytes_per_step_peak_cumulative():
    shapes = [(8, 6), (6, 8)]
    per_step = acc.tsr_schedule_bytes(shapes, r=2, p=1, K=3, T=7, b_dtype=4)
    core = 4 * (4 + 4)
    refresh = 4 * 2 * (4 + 8 * 3 + 3 * 6)
    assert per_step == [core, core, refresh, core, core, refresh, core]
    assert acc.peak_bytes(per_step) == refresh
    assert acc.bytes_per_step(per_step) == pytest.approx((5 * core + 2 * refresh) / 7)
    assert acc.cumulative_bytes(per_step, 3) == 2 * core + refresh


def test_config5_payload_ratio():
    # 350M shapes, r = 256: cores 168 * 256^2 * 4 B vs dense gradients at 4 B
    shapes = si.model_shapes("350m")
    assert len(shapes) == 168
    core = acc.step_bytes((acc.synchronized_elements("tsr", m, n, 256) for m, n in shapes), 4)
    dense = acc.step_bytes((acc.synchronized_elements("adamw", m, n, 256) for m, n in shapes), 4)
    assert core == 168 * 256 * 256 * 4
    assert dense / core == pytest.approx(27.5, abs=0.1)


def test_ablation_byte_ratios_on_60m_shapes():
    """The two byte claims of the ablation paragraph (Section 4.3) from the formulas of Table 1 and
    Section 3.5, on the LLaMA-60M block list with the settings of the paper's 60M run (r = 256,
    embedding rank 64, refresh every 100 steps): two-sided against one-sided cumulative bytes
    ("approximately two-thirds" less), randomized against exact SVD on the refresh step."""
    linear = si.model_shapes("60m")
    r, r_emb, p, K, T = 256, 64, 8, 100, 1000
    vocab_blocks = [(si.VOCAB, si.LLAMA["60m"]["hidden"])] * 2          # embedding and LM head
    def total(method, refresh):
        return (sum(acc.schedule_bytes(linear, r, p, K, T, method, refresh)) +
                sum(acc.schedule_bytes(vocab_blocks, r_emb, p, K, T, method, refresh)))
    two, one = total("tsr", "rsvd"), total("one-sided", "rsvd")
    assert 0.28 < two / one < 0.40, two / one                           # about two-thirds less
    # the refresh step itself (the peak): sketches k (m + n) against the dense m n
    peak_rsvd = max(a + b for a, b in zip(acc.schedule_bytes(linear, r, p, K, K), acc.schedule_bytes(vocab_blocks, r_emb, p, K, K)))
    peak_exact = max(a + b for a, b in zip(acc.schedule_bytes(linear, r, p, K, K, refresh="exact"),
                                           acc.schedule_bytes(vocab_blocks, r_emb, p, K, K, refresh="exact")))
    assert 0.40 < peak_rsvd / peak_exact < 0.55, peak_rsvd / peak_exact  # "nearly half"
    # per-step bytes do not depend on the refresh kind, so over a whole run the two differ less
    assert total("tsr", "rsvd") < total("tsr", "exact")
    assert acc.schedule_bytes(linear, r, p, K, 3) == acc.tsr_schedule_bytes(linear, r, p, K, 3)
    assert acc.exact_svd_refresh_elements(8, 6, 2) == 4 + 48
