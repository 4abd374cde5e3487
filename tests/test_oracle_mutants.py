"""Are the pins sharp?  Every case plants ONE plausible mistake in a copy of the oracle's source (a
transposed operand, a dropped term, a wrong sign, index or constant), compiles the copy and runs the
pin suites against it in a child process: at least one pin has to fail.  The mistakes are planted in
the oracle, on the CPU; nothing here touches the GPU path."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "moe_oracle.c")
PINS = [os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_placement.py")]

# (name, text in moe_oracle.c - must occur exactly once -, replacement)
MUTANTS = [
    ("gate: weight read transposed", "(double)wg[(int64_t)e * d + c]", "(double)wg[(int64_t)c * E + e]"),
    ("softmax: maximum not subtracted in the numerator", "p[t * E + e] = exp(l[e] - m) / s;", "p[t * E + e] = exp(l[e]) / s;"),
    ("top-k: ties go to the highest id", "if (best < 0 || l[e] > l[best]) best = e;", "if (best < 0 || l[e] >= l[best]) best = e;"),
    ("top-k: weights never renormalised", "if (renormalize && k > 1) {", "if (0 && renormalize && k > 1) {"),
    ("top-k: weight is the logit's exponential, not the probability", "topk_w[t * k + j] = exp(l[best] - m) / s;",
     "topk_w[t * k + j] = exp(l[best] - m);"),
    ("dispatch: buckets filled from the last assignment down (not stable)",
     "for (int64_t a = 0; a < A; ++a) {\n        int32_t e = local[a];", "for (int64_t a = A - 1; a >= 0; --a) {\n        int32_t e = local[a];"),
    ("dispatch: expert map ignored", "            e = expert_map ? expert_map[g] : g;", "            e = g;"),
    ("dispatch: offsets are inclusive sums", "expert_offsets[e + 1] = expert_offsets[e] + expert_counts[e];",
     "expert_offsets[e + 1] = expert_offsets[e] + expert_counts[e] + (e == 0);"),
    ("gather: assignment taken for the token", "int64_t t = src_of_sorted[s] / k;", "int64_t t = src_of_sorted[s] / (k > 1 ? 1 : k);"),
    ("FFN: first bias dropped", "if (b1) acc += (double)b1[(int64_t)e * f + u];", ""),
    ("FFN: second bias of expert 0 for everyone", "if (b2) acc += (double)b2[(int64_t)e * d + v];", "if (b2) acc += (double)b2[v];"),
    ("FFN: second weight read transposed", "(double)W2[(int64_t)v * f + u]", "(double)W2[(int64_t)u * d + v]"),
    ("FFN: first weight of expert 0 for everyone", "const float* W1 = w1 + (int64_t)e * f * d;", "const float* W1 = w1;"),
    ("GELU: erf argument not scaled", "erf(z * 0.70710678118654752440)", "erf(z)"),
    ("GELU tanh form: cubic coefficient", "0.044715 * z * z * z", "0.44715 * z * z * z"),
    ("combine: gate weight ignored", "out[t * d + c] += w * y_sorted[(int64_t)s * d + c];", "out[t * d + c] += y_sorted[(int64_t)s * d + c];"),
    ("combine: dropped assignment reads sorted row 0", "if (s < 0) continue;\n            double w", "if (s < 0) s = 0;\n            double w"),
    ("affinity: counts transposed", "counts[((int64_t)l * E + i) * E + p] += 1;", "counts[((int64_t)l * E + p) * E + i] += 1;"),
    ("affinity: invalid successor counted as expert 0", "if (p < 0 || p >= E) continue;\n                counts", "if (p < 0 || p >= E) p = 0;\n                counts"),
    ("affinity: loads only of tokens with a successor", "if (loads) loads[(int64_t)l * E + i] += 1;", "if (loads && l + 1 < L) loads[(int64_t)l * E + i] += 1;"),
    ("conditional probability: written transposed", "prob[((int64_t)l * E + i) * E + p] = s > 0", "prob[((int64_t)l * E + p) * E + i] = s > 0"),
    ("locality: both ends looked up in the map of layer l",
     "if (placement[(int64_t)l * E + i] == placement[(int64_t)(l + 1) * E + p]) c += 1;",
     "if (placement[(int64_t)l * E + i] == placement[(int64_t)l * E + p]) c += 1;"),
    ("locality from counts: both ends looked up in the map of layer l",
     "if (placement[(int64_t)l * E + i] == placement[(int64_t)(l + 1) * E + p])\n                    c += counts",
     "if (placement[(int64_t)l * E + i] == placement[(int64_t)l * E + p])\n                    c += counts"),
    ("transfers: tokens at home counted instead of tokens away", "!= home[n]) c += 1;", "== home[n]) c += 1;"),
    ("volume model: vanilla counted one way only", "vol[0] = 2.0 * g * n * l * p;", "vol[0] = g * n * l * p;"),
    ("volume model: AllGather term of one GPU instead of G", "vol[2] = g * n * (l * p_star + g);", "vol[2] = g * n * (l * p_star + 1.0);"),
    ("volume model: top-2 doubles the AllGather as well", "vol[3] = g * n * (2.0 * l * p_star + g);", "vol[3] = 2.0 * g * n * (l * p_star + g);"),
    ("transfer ratios: a coherent context is always compared with home", "if (gpu != at) moves += 1;", "if (gpu != home[n]) moves += 1;"),
    ("transfer ratios: the context does not stay where its expert was", "            at = gpu;\n", ""),
    ("multi-hop: counts transposed", "c[(int64_t)a * E + b] += 1;", "c[(int64_t)b * E + a] += 1;"),
    ("multi-hop: target layer is always the next one", "int32_t b = trace[(int64_t)m * N + n];", "int32_t b = trace[(int64_t)(l + 1) * N + n];"),
]


def _run_pins(lib):
    env = dict(os.environ)
    if lib:
        env["MOE_ORACLE_LIBRARY"] = lib
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS], cwd=ROOT, env=env,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)


def test_the_unchanged_oracle_passes_its_pins_in_a_child_process(tmp_path):
    lib = str(tmp_path / "same.so")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", lib, SRC, "-lm"], check=True)
    r = _run_pins(lib)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"the mutation list is out of date: {old!r} occurs {text.count(old)} times"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = str(tmp_path / "mutant.so")
    subprocess.run(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-w", "-o", lib, str(src), "-lm"], check=True)
    r = _run_pins(lib)
    assert r.returncode != 0, f"no pin noticed: {name}"
    assert "failed" in r.stdout or "error" in r.stdout.lower() or r.returncode < 0, r.stdout[-2000:]
