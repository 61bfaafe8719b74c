"""The benchmark's own parity gate (bench.Parity / bench.conv_error), exercised on the CPU: a correct result
passes, and a mistake planted on the CPU side -- in the expected values, or in the 'measured' array -- makes
the gate report failure (bench.py then exits non-zero)."""
import os
import sys

import numpy as np

import oracle

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402


def _case():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((1, 8, 9, 10))
    w = rng.standard_normal((6, 8, 3, 3)) * 0.1
    masks = oracle.pattern_dict(3)
    wm = oracle.mask(w, masks, oracle.select(w, masks))
    return oracle.conv2d(x, wm)


def test_gate_passes_a_correct_result():
    ref = _case()
    p = bench.Parity(False)
    got32 = ref.astype(np.float32)  # fp32 rounding only: far inside 2e-3 * rms
    p.add_oracle("case", got32, got32.astype(np.float16).astype(np.float64), ref)
    p.add_rne("case", True)
    assert p.ok() and p.report()["ok"] and p.report()["fp32_out_max_err"] < 1e-6
    assert p.report()["stored_out_max_err"] > p.report()["fp32_out_max_err"]  # the stored rounding is reported apart


def test_gate_fails_on_a_wrong_expected_value():
    ref = _case()
    wrong = ref.copy()
    wrong[0, 3, 4, 5] += 0.01 * np.sqrt(np.mean(ref ** 2))  # one expected value off by 5x the tolerance
    p = bench.Parity(False)
    p.add_oracle("case", ref.astype(np.float32), ref, wrong)
    assert not p.ok() and not p.report()["ok"] and p.report()["failures"]


def test_gate_fails_on_wrong_shape_nan_and_rounding():
    ref = _case()
    p = bench.Parity(False)
    p.add_oracle("shape", ref[:, :-1], ref[:, :-1], ref)
    assert not p.ok()
    p = bench.Parity(False)
    bad = ref.copy()
    bad[0, 0, 0, 0] = np.nan
    p.add_oracle("nan", bad, bad, ref)
    assert not p.ok()
    p = bench.Parity(False)
    p.add_rne("layer 0", False)
    assert not p.ok() and p.report()["stored_equals_rne_of_fp32_out"] is False


def test_fp32_tensors_use_the_max_bound():
    ref = _case()
    e, b = bench.conv_error(ref + 2e-5 * np.max(np.abs(ref)), ref, True)
    assert b == 1e-5 and e > b
    e, b = bench.conv_error(ref + 2e-6 * np.max(np.abs(ref)), ref, True)
    assert e <= b


def test_more_than_one_gpu_is_refused_with_a_message(monkeypatch, capsys):
    # one device only: the command line says so and exits non-zero before anything touches a GPU
    monkeypatch.setattr(sys, "argv", ["bench.py", "--gpus", "2"])
    assert bench.main() == 2
    assert "one GPU only" in capsys.readouterr().err


def test_default_command_line():
    # the defaults the measurement protocol relies on: steady clocks before the timed region, sampled phase events
    import unittest.mock as mock
    with mock.patch.object(sys, "argv", ["bench.py"]):
        args = bench.parse()
    assert args.gpus == 1 and args.steps == 100 and args.warmup >= 300 and args.prewarm_ms >= 100 and args.event_every == 10
