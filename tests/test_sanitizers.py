"""CPU-only sanitizer target: the plain-C oracle, a host-side bounds model of the selection kernel's
ordered emission and one of the cut of a long prompt into the part read once and the rest (which keys each launch
votes on, where the kept logits go), compiled with -fsanitize=address,undefined and run on small inputs.  A memory error or
undefined behaviour in either ends the program with a non-zero status and a report."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1", "-std=c11",
       "-Wall", "-Werror", "-Wno-unknown-pragmas"]


def build_and_run(tmp_path, name, sources):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / name)
    subprocess.run(["gcc", *SAN, "-o", exe, *sources, "-lm"], check=True, capture_output=True, text=True)
    # (the order check is off: the environment may preload a library of its own ahead of the sanitizer's runtime)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)


def test_c_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    r = build_and_run(tmp_path, "oracle_driver", [os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                                                  os.path.join(ROOT, "oracle", "snapkv_oracle.c")])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all cases passed" in r.stdout


def test_emission_offsets_model_under_sanitizers(tmp_path):
    r = build_and_run(tmp_path, "emission_model", [os.path.join(ROOT, "tests", "sanitize", "emission_model.c")])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all cases passed" in r.stdout


def test_long_prompt_plan_model_under_sanitizers(tmp_path):
    r = build_and_run(tmp_path, "long_plan_model", [os.path.join(ROOT, "tests", "sanitize", "long_plan_model.c")])
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all cases passed" in r.stdout
