"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the C file is compiled with
-fsanitize=address,undefined into a library of its own and a selection of the pin tests runs through
it in a subprocess that has the sanitizer runtime preloaded.  An out-of-bounds access, a use after
free or undefined arithmetic in the oracle aborts that subprocess.  No GPU needed."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PINS = [
    "tests/test_oracle_pins.py::test_worked_example_d2",
    "tests/test_oracle_pins.py::test_eliminated_hinv_is_inverse_of_remaining_block",
    "tests/test_oracle_pins.py::test_compensated_weights_solve_the_constrained_least_squares",
    "tests/test_oracle_pins.py::test_loss_telescopes_to_half_trace_and_to_output_error",
    "tests/test_oracle_pins.py::test_grid_groups_use_original_columns",
    "tests/test_oracle_pins.py::test_dynamic_order_takes_the_column_with_the_largest_loss_term",
    "tests/test_oracle_pins.py::test_obq_row_is_the_shared_loop_on_that_row_with_the_rows_own_order",
    "tests/test_oracle_pins.py::test_spd_inverse_rejects_non_pd",
    "tests/test_oracle_pins.py::test_column_loop_rejects_bad_perm",
]


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not asan or not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = dict(os.environ)
    env["FOBQ_ORACLE_SANITIZE"] = "1"
    # the runtime must come first among the preloaded libraries; what is preloaded already stays
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # python itself is not instrumented: no leak report for the interpreter, no link-order check
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "libfobq_oracle_san" not in res.stderr, tail
    assert os.path.exists(os.path.join(ROOT, "oracle", "libfobq_oracle_san.so"))
