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

CT = ("oracle/ppo_ct_oracle.c", "PPO_CT_ORACLE_SOURCE", ["tests/test_ct_oracle_pins.py"])

# (which oracle, text in the source, what replaces it, what the mistake is)
MUTANTS = [
    (CT, "volatile double d = (I->Q[e] - I->Q[i]) / (double)I->v[node];", "volatile double d = (I->Q[e] - I->Q[i]) * (double)I->v[node];",
     "compute stage: work times speed"),
    (CT, "volatile double d = (I->Q[e] - I->Q[i]) / (double)I->v[node];", "volatile double d = (I->Q[e - 1] - I->Q[i]) / (double)I->v[node];",
     "compute stage: the last layer of the segment is not counted"),
    (CT, "volatile double d = (I->Q[e] - I->Q[i]) / (double)I->v[node];",
     "volatile double d = (double)((float)(I->Q[e] - I->Q[i]) / I->v[node]);", "compute stage: divided in binary32"),
    (CT, "I->Q[i + 1] = I->Q[i] + (double)w[i];", "I->Q[i + 1] = I->Q[i] + (double)m[i];", "compute stage: weights taken for work"),
    (CT, "static float fmax2(float a, float b) { return a > b ? a : b; }", "static float fmax2(float a, float b) { return a < b ? a : b; }",
     "the least stage instead of the largest"),
    (CT, "if (ct_fits(I, 0, e, perm[0])) rows[e] = ct_comp(I, 0, e, perm[0]);", "if (ct_fits(I, 0, e, perm[0])) rows[e] = 0.0f;",
     "per-ordering route: the first segment's compute stage is dropped"),
    (CT, "if (ct_fits(&I, i, L, j)) best = ct_comp(&I, i, L, j);", "if (ct_fits(&I, i, L, j)) best = 0.0f;",
     "subset route: the last segment's compute stage is dropped"),
    (CT, "b = fmax2(b, ct_comp(&I, c[s], c[s + 1], perm[s]));", "if (s > 0) b = fmax2(b, ct_comp(&I, c[s], c[s + 1], perm[s]));",
     "definition route: the first segment's compute stage is dropped"),
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
    (CLUSTER, "if (bf_best_cuts(I, W->seq, p, &b, cut) && (!W->found || b < W->bbeta)) {",
     "if (bf_best_cuts(I, W->seq, p, &b, cut) && (!W->found || b <= W->bbeta)) {",
     "definition route: the last optimal sequence instead of the first"),
    (CLUSTER, "if (!isinf(b) && (!W->found || b < W->bbeta)) {", "if (!isinf(b) && (!W->found || b <= W->bbeta)) {",
     "exhaustive route: the last optimal sequence instead of the first"),
    (CLUSTER, "if (p == I->pmax) return;\n    for (int j = 0; j < I->n; ++j) {\n        if (W->used[j]) continue;\n        W->used[j] = 1; W->seq[p] = j;\n        bf_walk(W, p + 1);",
     "if (p > I->pmax) return;\n    for (int j = 0; j < I->n; ++j) {\n        if (W->used[j]) continue;\n        W->used[j] = 1; W->seq[p] = j;\n        bf_walk(W, p + 1);",
     "definition route: one segment more than allowed"),
    (CLUSTER, "volatile float q = I->t[cut - 1] / I->B[a * I->n + b];", "volatile float q = I->t[cut] / I->B[a * I->n + b];",
     "tensor of the layer after the cut instead of the one before"),
    (CLUSTER, "volatile float q = I->t[cut - 1] / I->B[a * I->n + b];", "volatile float q = I->t[cut - 1] / I->B[b * I->n + b];",
     "wrong element of the bandwidth matrix"),
]


# The Python oracles: (file, pin tests, pytest -k expression, [(text, replacement), ...], what the mistake is).
# The altered file shadows the real one in a copy of the package placed first on the import path.
PY_MUTANTS = [
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("float(B[a][b]) >= thr", "float(B[a][b]) > thr")], "a link at the threshold is left out (Eq. 8 says at or above)"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("if result is None:\n            low = median + 1\n        else:\n            high = median",
       "if result is None:\n            high = median\n        else:\n            low = median + 1")],
     "Alg. 2 bisects the wrong way"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("key=lambda r: (-r[1], r[0])", "key=lambda r: (r[1], r[0])")], "Alg. 3 matches the shortest runs first"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("for X in range(n_classes - 1, -1, -1):", "for X in range(n_classes):")], "Alg. 3 starts with the lowest class"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("g = gamma(t[c - 1], B[nodes[s - 1]][nodes[s]])", "g = gamma(t[c], B[nodes[s - 1]][nodes[s]])")],
     "tensor of the layer after the cut"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("int(math.floor((float(x) - lo) / (hi - lo) * n_classes))", "int(math.floor((float(x) - lo) / hi * n_classes))")],
     "class bins not taken over the range of the sizes"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("key=lambda v: (float(B[cur][v]), -v))", "key=lambda v: (-float(B[cur][v]), -v))")],
     "joint system moves on over the worst link"),
    ("oracle/ppo_heuristic_oracle.py", "tests/test_heuristic_oracle.py", "",
     [("        if not at_start and not at_end and not avail[v]:\n            return False\n", "")],
     "the path search takes nodes that are already used"),
    ("oracle/ppo_partition_oracle.py", "tests/test_partition_oracle.py", "",
     [("P[e] - P[s] <= float(kappa)", "P[e] - P[s] < float(kappa)"), ("P[e] - P[i] <= float(kappa)", "P[e] - P[i] < float(kappa)")],
     "both routes: a segment that fills the node exactly no longer fits"),
    ("oracle/ppo_partition_oracle.py", "tests/test_partition_oracle.py", "",
     [("float(t[c - 1]) + total", "float(t[c]) + total"), ("float(t[e - 1]) if e < L", "float(t[e]) if e < L")],
     "both routes: tensor of the layer after the cut"),
    ("oracle/ppo_partition_oracle.py", "tests/test_partition_oracle.py", "",
     [("P.append(P[-1] + float(x))", "P.append(float(x))")], "segment sizes are not cumulative"),
    ("oracle/ppo_partition_oracle.py", "tests/test_partition_oracle.py", "",
     [("cand = (total, p, cuts)", "cand = (total, -p, cuts)"), ("f[e][0], f[e][1] + 1, e)", "f[e][0], -(f[e][1] + 1), e)")],
     "both routes: ties go to the most segments"),
    ("oracle/ppo_partition_oracle.py", "tests/test_partition_oracle.py", "",
     [("if cand < best:\n                best = cand\n        f[i] = best", "if cand[0] < best[0]:\n                best = cand\n        f[i] = best")],
     "recurrence: ties keep the first end found"),
    ("oracle/ppo_dag_oracle.py", "tests/test_dag_frontend.py", "hand_worked and oracle",
     [("1 + max(lp(u) for u in pred[v])", "1 + min(lp(u) for u in pred[v])")], "depth by the shortest path"),
    ("oracle/ppo_dag_oracle.py", "tests/test_dag_frontend.py", "hand_worked and oracle",
     [("if len(here) == 1 and every_path_reaches(points[-1], here[0]):", "if len(here) == 1:")],
     "a vertex of unique depth that some path goes round"),
    ("oracle/ppo_dag_oracle.py", "tests/test_dag_frontend.py", "hand_worked and oracle",
     [("if lower < depth[v] <= depth[p]]", "if lower <= depth[v] <= depth[p]]")],
     "the previous partition point is counted into the next layer as well"),
    ("oracle/ppo_dag_oracle.py", "tests/test_dag_frontend.py", "hand_worked and oracle",
     [("t.append(float(out_size[p]))", "t.append(float(weight[p]))")], "transfer size taken from the weights"),
]


@pytest.mark.parametrize("case", range(len(PY_MUTANTS)), ids=[m[4] for m in PY_MUTANTS])
def test_pins_notice_a_planted_mistake_in_a_python_oracle(case, tmp_path):
    source, pin_file, select, edits, what = PY_MUTANTS[case]
    shadow = tmp_path / "oracle"
    shadow.mkdir()
    (shadow / "__init__.py").write_text("")
    text = open(os.path.join(ROOT, source)).read()
    for old, new in edits:
        assert text.count(old) >= 1, f"the source no longer holds the text this case alters: {old!r}"
        text = text.replace(old, new)
    (shadow / os.path.basename(source)).write_text(text)
    for other in os.listdir(os.path.join(ROOT, "oracle")):   # what the altered module imports from its own package
        if other.endswith(".py") and other not in ("__init__.py", os.path.basename(source)):
            (shadow / other).write_text(open(os.path.join(ROOT, "oracle", other)).read())
    env = dict(os.environ, PYTHONPATH=os.pathsep.join([str(tmp_path), ROOT, os.environ.get("PYTHONPATH", "")]))
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", "--rootdir", ROOT,
           os.path.join(ROOT, pin_file)]
    if select:
        cmd += ["-k", select]
    # run from the directory that holds the shadow package: the interpreter puts it first on the import path
    run = subprocess.run(cmd, cwd=tmp_path, env=env, capture_output=True, text=True, timeout=600)
    assert "Error while" not in run.stdout and "ModuleNotFoundError" not in run.stdout, run.stdout[-2000:]
    assert run.returncode == 1, f"the pins passed with this mistake planted: {what}\n{run.stdout[-2000:]}\n{run.stderr[-1000:]}"
    assert " failed" in run.stdout, run.stdout[-2000:]


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
