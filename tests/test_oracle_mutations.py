"""Do the oracle's pins notice a plausible mistake?  Each case plants one single-token error in a
copy of oracle/qv_oracle.cpp (a dropped term, a swapped operand, a wrong index), builds it, and
runs the pin tests (tests/test_oracle_sampling.py, tests/test_oracle_metrics.py) against that build
in a child process: the run must FAIL.  A mutation that no longer applies to the source fails the
case too, so the list cannot silently go stale.  CPU only; nothing here touches the HIP path."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "qv_oracle.cpp")

MUTATIONS = [
    ("rand_below bound off by one (Floyd draws from j, not j + 1, values)",
     "(uint64_t)(j + 1)", "(uint64_t)(j)"),
    ("Floyd keeps the wrong value on a collision",
     "pos.push_back(taken ? j : t)", "pos.push_back(taken ? t : j)"),
    ("Philox counter words node and hop swapped",
     "uint32_t ctr[4] = {node, hop, slot, 0u}", "uint32_t ctr[4] = {hop, node, slot, 0u}"),
    ("64-bit random word assembled from the wrong halves",
     "((uint64_t)x[1] << 32) | x[0]", "((uint64_t)x[0] << 32) | x[1]"),
    ("Philox round mixes the wrong key word",
     "uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;", "uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k1;"),
    ("hop frontier keeps repeats (no per-hop dedup)",
     "if (seen_here.insert(g).second) next.push_back(g);", "seen_here.insert(g); next.push_back(g);"),
    ("layer frontier never advances (hop k expands the seeds again)",
     "if (!cumulative) cur.swap(next);", "if (cumulative) cur.swap(next);"),
    ("edge lists its target's global instead of local id",
     "row_local[n_edges] = v_local;", "row_local[n_edges] = v;"),
    ("PSGS counts the full degree instead of min(degree, fanout)",
     "S[i] = (double)std::min<int64_t>(deg, l) + incl_weight", "S[i] = (double)deg + incl_weight"),
    ("PSGS uses the fanouts in reverse hop order",
     "int32_t l = fanouts[m - 1];", "int32_t l = fanouts[n_hops - m];"),
    ("FAP weights every hop with the first fanout",
     "double c = p[j] * incl_weight(deg, l, weight_mode)", "double c = p[j] * incl_weight(deg, fanouts[0], weight_mode)"),
    ("FAP mass stays at the source instead of moving along the edge",
     "for (int64_t e = rowptr[j]; e < rowptr[j + 1]; ++e) nxt[col[e]] += c;",
     "for (int64_t e = rowptr[j]; e < rowptr[j + 1]; ++e) nxt[j] += c;"),
    ("placement ranks by ascending probability",
     "return prob[a] > prob[b]", "return prob[a] < prob[b]"),
    ("gather copies from the output row index instead of the id",
     "table + (int64_t)ids[r] * row_bytes", "table + (int64_t)r * row_bytes"),
]


def run_pins_against(tmp_path, source_text):
    mutated = tmp_path / "qv_oracle_variant.cpp"
    mutated.write_text(source_text)
    so = tmp_path / "libqv_oracle_variant.so"
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", "-w", "-o", str(so), str(mutated)])
    env = dict(os.environ, QV_ORACLE_LIB=str(so))
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                           os.path.join(ROOT, "tests", "test_oracle_sampling.py"),
                           os.path.join(ROOT, "tests", "test_oracle_metrics.py")],
                          cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def test_control_the_unmodified_source_passes_in_this_harness(tmp_path):
    run = run_pins_against(tmp_path, open(SOURCE).read())
    assert run.returncode == 0, run.stdout[-800:]


@pytest.mark.parametrize("what,needle,replacement", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_kill_the_mutant(tmp_path, what, needle, replacement):
    src = open(SOURCE).read()
    assert src.count(needle) == 1, "the mutation no longer applies to the oracle source: " + what
    run = run_pins_against(tmp_path, src.replace(needle, replacement))
    assert run.returncode != 0, "no pin noticed: " + what
    assert "failed" in run.stdout or "error" in run.stdout.lower(), run.stdout[-500:]
