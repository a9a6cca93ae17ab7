"""The pins of the oracles must notice a plausible mistake: each case plants one in a copy of an oracle's C
source (never in the real file, never on the GPU), runs the pin tests against that copy in a child process
and expects them to fail.  The mistakes sit in the helpers that all three routes of an oracle share (the
memory rule, Eq. 3's quotient, the prefix sums, the rank), where agreement between the routes proves
nothing, and in each route on its own."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

FIXED = ("oracle/ppo_oracle.c", "PPO_ORACLE_SOURCE", ["tests/test_oracle_pins.py"])
CLUSTER = ("oracle/ppo_cluster_oracle.c", "PPO_CLUSTER_ORACLE_SOURCE", ["tests/test_cluster_oracle_pins.py"])

# (which oracle, text in the source, what replaces it, what the mistake is)
MUTANTS = [
    (FIXED, "return (I->P[e] - I->P[i]) <= (double)I->M[node]; }", "return (I->P[e] - I->P[i]) < (double)I->M[node]; }",
     "a segment that fills a node exactly no longer fits"),
    (FIXED, "return (I->P[e] - I->P[i]) <= (double)I->M[node]; }", "return (I->P[e - 1] - I->P[i]) <= (double)I->M[node]; }",
     "the last layer of a segment is not counted"),
    (FIXED, "return (I->P[e] - I->P[i]) <= (double)I->M[node]; }",
     "return (float)(I->P[e] - I->P[i]) <= I->M[node]; }", "segment size rounded to binary32 before the comparison"),
    (FIXED, "P[i + 1] = P[i] + (double)m[i];", "P[i + 1] = (double)(float)(P[i] + (double)m[i]);",
     "prefix sums accumulated in binary32"),
    (FIXED, "volatile float q = I->t[cut - 1] / I->B[a * I->k + b];", "volatile float q = I->t[cut] / I->B[a * I->k + b];",
     "tensor of the layer after the cut instead of the one before"),
    (FIXED, "volatile float q = I->t[cut - 1] / I->B[a * I->k + b];", "volatile float q = I->t[cut - 1] * I->B[a * I->k + b];",
     "product instead of quotient"),
    (FIXED, "volatile float q = I->t[cut - 1] / I->B[a * I->k + b];", "volatile float q = I->t[cut - 1] / I->B[a * I->k + a];",
     "wrong element of the bandwidth matrix"),
    (FIXED, "if (perm[q] < perm[p]) ++smaller;", "if (perm[q] > perm[p]) ++smaller;", "rank counts the larger successors"),
    (FIXED, "if (g > b) b = g;", "if (g < b || b == 0.0f) b = g;", "definition route: least link time instead of the bottleneck"),
    (FIXED, "float c = prev[i] > g ? prev[i] : g;\n                if (c < best) best = c;",
     "float c = prev[i] > g ? prev[i] : g;\n                if (c > best || best == INFINITY) best = c;",
     "chain DP keeps the worst candidate"),
    (FIXED, "if (rank < best.rank) better = 1;", "if (rank > best.rank) better = 1;", "definition route: highest rank wins ties"),
    (FIXED, "if (c <= beta) { chosen = i; break; }", "if (c <= beta) { chosen = i; }", "cut rule takes the largest cut"),
    (CLUSTER, "return (I->P[e] - I->P[i]) <= (double)I->M[node]; }", "return (I->P[e] - I->P[i]) < (double)I->M[node]; }",
     "a segment that fills a node exactly no longer fits"),
    (CLUSTER, "return (I->P[e] - I->P[i]) <= (double)I->M[node]; }",
     "return (float)(I->P[e] - I->P[i]) <= I->M[node]; }", "segment size rounded to binary32 before the comparison"),
    (CLUSTER, "I->P[i + 1] = I->P[i] + (double)m[i];", "I->P[i + 1] = (double)(float)(I->P[i] + (double)m[i]);",
     "prefix sums accumulated in binary32"),
    (CLUSTER, "volatile float q = I->t[cut - 1] / I->B[a * I->n + b];", "volatile float q = I->t[cut] / I->B[a * I->n + b];",
     "tensor of the layer after the cut instead of the one before"),
    (CLUSTER, "volatile float q = I->t[cut - 1] / I->B[a * I->n + b];", "volatile float q = I->t[cut - 1] / I->B[b * I->n + b];",
     "wrong element of the bandwidth matrix"),
]


@pytest.mark.parametrize("case", range(len(MUTANTS)), ids=[m[3] for m in MUTANTS])
def test_pins_notice_a_planted_mistake(case, tmp_path):
    (source, variable, pin_files), old, new, what = MUTANTS[case]
    text = open(os.path.join(ROOT, source)).read()
    assert text.count(old) >= 1, f"the source no longer holds the text this case alters: {old!r}"
    altered = tmp_path / os.path.basename(source)
    altered.write_text(text.replace(old, new))
    env = dict(os.environ, **{variable: str(altered)})
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *pin_files],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert run.returncode == 1, f"the pins passed with this mistake planted: {what}\n{run.stdout[-2000:]}\n{run.stderr[-1000:]}"
    assert " failed" in run.stdout, run.stdout[-2000:]
