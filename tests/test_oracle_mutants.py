"""Do the pins bite?  Each case plants one plausible mistake in a copy of the CPU checker's source
(a dropped term, a wrong comparison, a transposed order), builds it, and runs the pin tests against
that build in a subprocess: they must fail.  Nothing here touches the GPU or the real checker."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "loki_oracle.c")

MUTANTS = [
    ("fill takes the capacity instead of min(remaining, capacity)",
     "int64_t routed = rem < cap ? rem : cap;", "int64_t routed = cap;"),
    ("units of a child task not scaled by the fan-out denominator",
     "scale[i] = scale[p->parent[i]] * per_level;", "scale[i] = scale[p->parent[i]];"),
    ("SLO not halved for queueing", "lat > room / 2", "lat > room"),
    ("latency equal to the budget counted as a violation", "lat > room / 2", "lat >= room / 2"),
    ("least accurate variant filled first",
     "p->acc_ppm[L->voff[i] + order[j]] < p->acc_ppm[L->voff[i] + v]",
     "p->acc_ppm[L->voff[i] + order[j]] > p->acc_ppm[L->voff[i] + v]"),
    ("equal accuracies ordered by higher index first",
     "p->acc_ppm[L->voff[i] + order[j]] < p->acc_ppm[L->voff[i] + v]",
     "p->acc_ppm[L->voff[i] + order[j]] <= p->acc_ppm[L->voff[i] + v]"),
    ("worker budget met with equality counted as a violation", "if (workers > workers_cap)", "if (workers >= workers_cap)"),
    ("an idle first hosted variant does not count as in use", "int used = (routed > 0) || !t->any;", "int used = (routed > 0);"),
    ("every hosted variant counts as in use", "int used = (routed > 0) || !t->any;", "int used = 1;"),
    ("tie broken towards more workers", "if (workers < b->workers)\n            return 1;", "if (workers > b->workers)\n            return 1;"),
    ("tie broken towards the higher index", "return index < b->index;", "return index > b->index;"),
    ("mean over paths not taken", "out->accuracy = sum / (double)n_paths;", "out->accuracy = sum;"),
    ("communication latency charged once instead of per task on the path",
     "int64_t room = slo_us - comm_us * (int64_t)len;", "int64_t room = slo_us - comm_us;"),
    ("path product taken leaf first",
     "double prod = a[path[len - 1]]; /* root first */\n        for (int s = len - 2; s >= 0; s--)\n            prod = prod * a[path[s]];",
     "double prod = a[path[0]];\n        for (int s = 1; s < len; s++)\n            prod = prod * a[path[s]];"),
    ("leaf sum taken in descending leaf order",
     "for (int leaf = 0; leaf < n; leaf++) {\n        if (!is_leaf[leaf])\n            continue;\n        int path[LO_MAX_TASKS], len = 0;",
     "for (int leaf = n - 1; leaf >= 0; leaf--) {\n        if (!is_leaf[leaf])\n            continue;\n        int path[LO_MAX_TASKS], len = 0;"),
    ("fan-out of the edge not applied to the child's demand",
     "Dn[i] = Dn[p->parent[i]] * (int64_t)p->fanout_q4[i];", "Dn[i] = Dn[p->parent[i]] * 4;"),
    ("zero demand scored with accuracy zero", "a[i] = (double)t[i].first_acc / 1000000.0;", "a[i] = 0.0;"),
    ("unserved demand tolerated", "if (t[i].unserved > 0)", "if (t[i].unserved < 0)"),
    ("per-variant factor not applied", "t->outflow += routed * (int64_t)p->variant_factor_q4[L->voff[i] + k];",
     "t->outflow += routed * 4;"),
    ("batch digit of a variant ignored", "beta[k] = g == 0 ? 0 : (int32_t)((g - 1) % (uint64_t)nb);", "beta[k] = 0;"),
    # objective with profiled path accuracies
    ("routing probabilities read transposed", "c->r->prob[i][prev_variant][k]", "c->r->prob[i][k][prev_variant]"),
    ("share of the path so far not carried down", "double m = depth == 0 ? share : mass * share;", "double m = share;"),
    ("a variant without traffic leads nowhere", "share = k == first_hosted ? 1.0 : 0.0;", "share = 0.0;"),
    ("every leaf reads the first leaf's table", "table += size;", "table += 0;"),
    ("mean over the task paths not taken", "return total / (double)n_paths;", "return total;"),
    ("table stride not advanced with the depth", "path_walk(c, depth + 1, k, m, e, stride * (uint64_t)K);",
     "path_walk(c, depth + 1, k, m, e, stride);"),
    ("frontend split ignored at the root", "share = depth == 0 ? c->r->prob[0][0][k] : c->r->prob[i][prev_variant][k];",
     "share = depth == 0 ? (k == first_hosted ? 1.0 : 0.0) : c->r->prob[i][prev_variant][k];"),
    # eq. (7) on the variant paths with traffic
    ("every pairing of in-use variants counts as a path with traffic",
     "taken = (depth == 0 ? c->r->prob[0][0][k] : c->r->prob[i][prev_variant][k]) > 0.0;",
     "taken = c->r->routed[i][k] > 0;"),
    ("routing table of the path's latency read transposed",
     "taken = (depth == 0 ? c->r->prob[0][0][k] : c->r->prob[i][prev_variant][k]) > 0.0;",
     "taken = (depth == 0 ? c->r->prob[0][0][k] : c->r->prob[i][k][prev_variant]) > 0.0;"),
    ("latency so far not carried down the path", "latency_walk(c, depth + 1, k, lat);", "latency_walk(c, depth + 1, k, 0);"),
    ("path latency at the budget counted as a violation", "if (lat > c->limit)", "if (lat >= c->limit)"),
    ("SLO of the per-path rule not halved", "room / 2 /* SLO halved for queueing */", "room /* SLO halved for queueing */"),
    ("per-path rule on, per-task bound still applied",
     "pipeline_eval(p, t, Dn, workers, slo_us, comm_us, !p->latency_per_path, out);",
     "pipeline_eval(p, t, Dn, workers, slo_us, comm_us, 1, out);"),
    ("only the first leaf's paths checked", "violated |= c.violated;", "violated |= c.violated; break;"),
]


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_a_planted_mistake(what, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site not found: {old!r}"
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "loki_oracle.c")
        open(src, "w").write(text.replace(old, new))
        lib = os.path.join(tmp, "libmutant.so")
        subprocess.run(["gcc", "-O1", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                        "-I", os.path.join(ROOT, "oracle"), "-o", lib, src], check=True)
        env = dict(os.environ, LOKI_ORACLE_LIB=lib, LOKI_ORACLE_MUTANT_TEST="1")
        r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                            os.path.join(ROOT, "tests", "test_oracle_path_tables.py"),
                            os.path.join(ROOT, "tests", "test_oracle_latency_per_path.py"), "-x", "-q", "-p", "no:cacheprovider",
                            "-k", "not slices and not zero_demand and not symmetry and not config5_golden"],
                           env=env, cwd=ROOT, capture_output=True, text=True, timeout=600)
        assert r.returncode != 0, f"no pin noticed: {what}\n{r.stdout[-800:]}"
