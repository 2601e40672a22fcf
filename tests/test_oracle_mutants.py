"""Do the pins bite?  Copies of the oracle with ONE planted mistake each are compiled on the CPU and
the pins of tests/test_oracle_pins.py are run against them: every mistake must fail at least one pin.
The mistakes are the plausible ones for this method: a flipped residual (the direction Algorithm 4
prints), a non-strict sampler, swapped models in the acceptance test, a dropped term or a wrong
divisor in a margin, a maximum for a minimum, a margin taken over positions that do not count."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "svip_oracle.c")

# (name, text in svip_oracle.c, replacement, pins of which at least one must fail)
MUTANTS = [
    ("residual_direction_as_printed", "double d = p[i] - q[i];\n                w[i] = d > 0.0 ? d : 0.0;",
     "double d = q[i] - p[i];\n                w[i] = d > 0.0 ? d : 0.0;",
     ["test_output_law_through_the_entry_points", "test_exact_output_law_enumeration", "test_verify_margins_hand_worked"]),
    ("sampler_not_strict", "if (C > target) {", "if (C >= target) {", ["test_inverse_cdf_edges"]),
    ("accept_test_models_swapped", "int acc = ua[b * k_max + j] * qx < px;", "int acc = ua[b * k_max + j] * px < qx;",
     ["test_first_rejection_all_patterns", "test_accept_probability_is_min_1_ratio_and_frequency_is_beta"]),
    ("stop_not_strict", "int by_entropy = sqrt(H) > h;\n        int by_cap = (step_j + 1 >= k_max);\n        stop[b] = (unsigned char)(by_entropy || by_cap);\n        margin_h[b] = by_cap ? INFINITY : fabs(sqrt(H) - h);\n    }\n    free(q);\n}\n\n/* ---- verification",
     "int by_entropy = sqrt(H) >= h;\n        int by_cap = (step_j + 1 >= k_max);\n        stop[b] = (unsigned char)(by_entropy || by_cap);\n        margin_h[b] = by_cap ? INFINITY : fabs(sqrt(H) - h);\n    }\n    free(q);\n}\n\n/* ---- verification",
     ["test_stop_is_strict_and_cap_forces_stop"]),
    ("sampler_margin_farther_edge", "*margin = (lo < hi ? lo : hi) / W;", "*margin = (lo > hi ? lo : hi) / W;",
     ["test_sampler_margin_hand_worked"]),
    ("sampler_margin_not_divided", "*margin = (lo < hi ? lo : hi) / W;", "*margin = (lo < hi ? lo : hi);",
     ["test_sampler_margin_hand_worked"]),
    ("stop_margin_on_entropy", "margin_h[b] = by_cap ? INFINITY : fabs(sqrt(H) - h);\n    }\n    free(q);\n}\n\n/* ---- verification",
     "margin_h[b] = by_cap ? INFINITY : fabs(H - h);\n    }\n    free(q);\n}\n\n/* ---- verification",
     ["test_stop_margin_hand_worked"]),
    ("accept_margin_largest", "if (d < mar) mar = d;", "if (d > mar || mar == INFINITY) mar = d;",
     ["test_verify_margins_hand_worked"]),
    ("accept_margin_over_every_position", "if (r == g) {        /* no rejection so far: this decision shapes the output */\n                if (d < mar) mar = d;",
     "if (d < mar) mar = d;\n            if (r == g) {", ["test_verify_margins_hand_worked"]),
    ("accept_margin_without_the_rejecting_test", "if (d < mar) mar = d;\n                if (!acc) r = j;",
     "if (!acc) r = j;\n                if (acc && d < mar) mar = d;", ["test_verify_margins_hand_worked"]),
    ("verify_margin_drops_the_draw", "margin[b] = ms < mar ? ms : mar;", "margin[b] = mar;",
     ["test_verify_margins_hand_worked"]),
    ("entropy_sign", "if (prob[i] > 0.0) H -= prob[i] * log(prob[i]);", "if (prob[i] > 0.0) H += prob[i] * log(prob[i]);",
     ["test_uniform_logits_entropy_is_log_V", "test_spike_over_flat_closed_form"]),
    ("temperature_multiplied", "double e = exp(z[i] / T - m);", "double e = exp(z[i] * T - m);",
     ["test_softmax_entropy_match_scipy_and_invariances"]),
]


def _call(fn):
    marks = getattr(fn, "pytestmark", [])
    params = [m for m in marks if m.name == "parametrize"]
    if not params:
        fn()
        return
    names, values = params[0].args
    for v in values:
        if isinstance(names, str) and "," not in names:
            fn(v)
        else:
            fn(*v)


@pytest.mark.parametrize("name,old,new,expect", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(tmp_path, name, old, new, expect):
    src = open(SRC).read()
    assert src.count(old) == 1, f"{name}: the text to change must occur exactly once in the oracle"
    c, so = tmp_path / "mutant.c", tmp_path / "libmutant.so"
    c.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fno-fast-math", "-o", str(so), str(c), "-lm"])
    good = oracle._load()
    oracle._lib = oracle._bind(ctypes.CDLL(str(so)))
    try:
        failed = []
        for t in expect:
            try:
                _call(getattr(pins, t))
            except AssertionError:
                failed.append(t)
        assert failed, f"{name}: none of {expect} noticed the planted mistake"
    finally:
        oracle._lib = good
