"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a driver
calls every oracle function on small ragged shapes and edge cases with exactly-sized buffers.  A second
build with a planted bounds mistake shows that the run would notice one."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moe_oracle.c")
DRIVER = os.path.join(ROOT, "oracle", "sanitize_check.c")
FLAGS = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]


def _build_and_run(src, exe):
    subprocess.run([*FLAGS, "-o", exe, src, DRIVER, "-lm"], check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    r = _build_and_run(SRC, str(tmp_path / "oracle_san"))
    assert r.returncode == 0, r.stdout[-3000:]
    assert "sanitizer run clean" in r.stdout


@pytest.mark.parametrize("old,new", [
    # the invalid-id guard of the dispatch dropped: the bucket counter is indexed outside its array
    ("if (e >= E_local) { e = -1; ++invalid; }", ""),
    # the offsets loop runs one expert too far: one element past the end of two arrays
    ("for (int e = 0; e < E_local; ++e) expert_offsets[e + 1] =", "for (int e = 0; e <= E_local; ++e) expert_offsets[e + 1] ="),
])
def test_a_planted_bounds_mistake_is_caught(tmp_path, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1
    bad = tmp_path / "bad.c"
    bad.write_text(text.replace(old, new))
    r = _build_and_run(str(bad), str(tmp_path / "bad_san"))
    assert r.returncode != 0 and ("AddressSanitizer" in r.stdout or "runtime error" in r.stdout), r.stdout[-2000:]
