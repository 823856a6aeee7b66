"""The oracle's pins must notice a mistake: every mutant below is a copy of oracle/ with ONE
plausible error planted in wfst_oracle.c (a comparison flipped, a tie-break reversed, a limit
changed), and the pin tests are run against that copy in a child process.  A mutant that passes
them means that part of the oracle is held by nothing but itself.  The decode loop, its prune
rule, its tie-breaks and the boosting acceptor are checked against the pins of the decode proper;
the word-boost table, the lattice output and the cost offsets against the pins of those options.

Everything here runs on the CPU; the mistakes are planted in the oracle only.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_decode_pins.py", "tests/test_oracle_pins.py", "tests/test_oracle_boost_fst.py"]
# pins of the options: word-boost table, lattice output, cost offsets
OPTION_PIN_FILES = ["tests/test_oracle_boost.py", "tests/test_oracle_lattice.py", "tests/test_oracle_offset.py"]

# (name, text in wfst_oracle.c, replacement); the text must occur exactly once
MUTANTS = [
    ("running count reaches instead of exceeds",
     "run += hist[j]; if (run > max_active) { k_keep = j; break; }",
     "run += hist[j]; if (run >= max_active) { k_keep = j; break; }"),
    # (not a mutant: `n_in >= max_active` inside oracle_cutoff changes nothing, because with exactly
    #  max_active tokens in the beam the running count never exceeds max_active; what does change
    #  with that comparison is the count of frames where max-active bound, which is the next entry)
    ("max-active counted as binding when the beam holds exactly max_active",
     "    if (n_in > o->max_active) {\n      res->counters[5]++;",
     "    if (n_in >= o->max_active) {\n      res->counters[5]++;"),
    ("histogram leaves out the token whose gap equals the beam",
     "if ((costs[i] - best) <= beam) { hist[bin_of(costs[i], &k)]++; ++n_in; }",
     "if ((costs[i] - best) < beam) { hist[bin_of(costs[i], &k)]++; ++n_in; }"),
    ("beam test is strict",
     "return ((c - k->best) <= k->beam) && (bin_of(c, k) < k->k_keep);",
     "return ((c - k->best) < k->beam) && (bin_of(c, k) < k->k_keep);"),
    ("bin 0 may be pruned",
     "if (k_keep < 1) k_keep = 1;",
     "if (k_keep < 0) k_keep = 1;"),
    ("initial closure has a bin limit",
     "k.best = 0.0f; k.k_keep = 256;\n  eps_closure(p, &cur, map, &k,",
     "k.best = 0.0f; k.k_keep = 128;\n  eps_closure(p, &cur, map, &k,"),
    ("emitting tie goes to the higher arc id",
     "(nc == nxt.t[q].cost && (int32_t)a < nxt.t[q].arc)",
     "(nc == nxt.t[q].cost && (int32_t)a > nxt.t[q].arc)"),
    ("emitting tie keeps the first arrival",
     "(nc == nxt.t[q].cost && (int32_t)a < nxt.t[q].arc)",
     "(0)"),
    ("epsilon tie goes to the higher arc id",
     "(nc == v->t[q].cost && gid < v->t[q].arc)",
     "(nc == v->t[q].cost && gid > v->t[q].arc)"),
    ("final tie (with final costs) goes to the higher state",
     "        if (!(f < INFINITY)) continue;\n        if (bi < 0 || f < bf || (f == bf && cur.t[i].state < cur.t[bi].state) ||",
     "        if (!(f < INFINITY)) continue;\n        if (bi < 0 || f < bf || (f == bf && cur.t[i].state > cur.t[bi].state) ||"),
    ("final tie (no final state) goes to the higher state",
     "        float f = cur.t[i].cost;\n        if (bi < 0 || f < bf || (f == bf && cur.t[i].state < cur.t[bi].state) ||",
     "        float f = cur.t[i].cost;\n        if (bi < 0 || f < bf || (f == bf && cur.t[i].state > cur.t[bi].state) ||"),
    ("cutoff not frozen: closure uses no bin limit",
     "    k.best = best; k.k_keep = k_keep;\n",
     "    k.best = best; k.k_keep = 256; (void)k_keep;\n"),
    ("acoustic cost added with the wrong sign",
     "float ac = -L[p->e_il[a] - 1];",
     "float ac = L[p->e_il[a] - 1];"),
    ("label k reads column k",
     "float ac = -L[p->e_il[a] - 1];",
     "float ac = -L[p->e_il[a] % p->V];"),
    ("boosting acceptor: a mismatch does not retry at the root",
     "  if (i < 0 && b != 0) i = bfst_arc(B, 0, o);",
     "  (void)0;"),
    ("boosting acceptor: a mismatch leaves the B state where it was",
     "  if (i < 0) return 0;\n  *add = 1; *score = B->score[i];",
     "  if (i < 0) return b;\n  *add = 1; *score = B->score[i];"),
    ("boosting acceptor: the B state is not part of the recombination key",
     "if (v->t[q].b == b) return q;",
     "return q;"),
    ("boosting acceptor: epsilon arcs with output labels do not move B",
     "        nb = boost_step(B, b, p->x_ol[a], &add, &sc);",
     "        boost_step(B, b, p->x_ol[a], &add, &sc);"),
    ("boosting acceptor: matched arc does not move B",
     "  *add = 1; *score = B->score[i];\n  return B->to[i];",
     "  *add = 1; *score = B->score[i];\n  return b;"),
    ("boosting acceptor: final tie prefers the higher B state",
     "        if (!(f < INFINITY)) continue;\n        if (bi < 0 || f < bf || (f == bf && cur.t[i].state < cur.t[bi].state) ||\n            (f == bf && cur.t[i].state == cur.t[bi].state && cur.t[i].b < cur.t[bi].b))",
     "        if (!(f < INFINITY)) continue;\n        if (bi < 0 || f < bf || (f == bf && cur.t[i].state < cur.t[bi].state) ||\n            (f == bf && cur.t[i].state == cur.t[bi].state && cur.t[i].b > cur.t[bi].b))"),
    ("boosting acceptor: same arc from two B states, first arrival wins (emitting)",
     " ||\n                 (nc == nxt.t[q].cost && (int32_t)a == nxt.t[q].arc && b < cur.t[nxt.t[q].prev].b)) {",
     ") {"),
    ("boosting acceptor: same arc from two B states, first arrival wins (epsilon)",
     " ||\n                 (nc == v->t[q].cost && gid == v->t[q].arc && b < v->t[v->t[q].prev].b)) {",
     ") {"),
    ("boosting acceptor: same arc from two B states, higher source B state wins",
     "(int32_t)a == nxt.t[q].arc && b < cur.t[nxt.t[q].prev].b",
     "(int32_t)a == nxt.t[q].arc && b > cur.t[nxt.t[q].prev].b"),
    ("final cost ignored",
     "float f = cur.t[i].cost + p->final_cost[cur.t[i].state];",
     "float f = cur.t[i].cost;"),
]


# the same for the optional parts: (name, text, replacement), run against OPTION_PIN_FILES
OPTION_MUTANTS = [
    ("lattice: an emitting link exactly lattice_beam above the destination is left out",
     "if ((nc - C1[j]) <= lattice_beam) PUT(t, i, j, a, nc);",
     "if ((nc - C1[j]) < lattice_beam) PUT(t, i, j, a, nc);"),
    ("lattice: an epsilon link exactly lattice_beam above the destination is left out",
     "if ((nc - C1[j]) <= lattice_beam) PUT(t, i, j, p->Ae + a, nc);",
     "if ((nc - C1[j]) < lattice_beam) PUT(t, i, j, p->Ae + a, nc);"),
    ("lattice: links are measured against the source token's cost",
     "if ((nc - C1[j]) <= lattice_beam) PUT(t, i, j, a, nc);",
     "if ((nc - C0[i]) <= lattice_beam) PUT(t, i, j, a, nc);"),
    ("lattice: epsilon arcs are not links",
     "if ((nc - C1[j]) <= lattice_beam) PUT(t, i, j, p->Ae + a, nc);",
     "(void)j;"),
    ("lattice: the boost of an epsilon arc's word is forgotten",
     "        if (boost && p->x_ol[a] != 0) nc = canon(nc + boost[p->x_ol[a]]);\n        const int32_t j = where[p->x_next[a]];",
     "        const int32_t j = where[p->x_next[a]];"),
    ("lattice with cost offsets: a link is rebased by the wrong set's offset",
     "if (frame_best) nc = canon(nc - frame_best[t]);",
     "if (frame_best && t > 1) nc = canon(nc - frame_best[t - 1]);"),
    ("lattice with cost offsets: links across a frame boundary are not rebased",
     "if (frame_best) nc = canon(nc - frame_best[t]);",
     "(void)frame_best;"),
    ("cost offsets: the closure still measures against the old best",
     "      offset_sum += (double)best;\n      k.best = 0.0f;",
     "      offset_sum += (double)best;"),
    ("cost offsets: the offsets are not added back",
     "      offset_sum += (double)best;\n",
     "      offset_sum += 0.0;\n"),
    ("word boost table: emitting arcs with a word are not boosted",
     "          nb = boost_step(B, b, p->e_ol[a], &add, &sc);\n          if (add) nc = canon(nc + sc);",
     "          nb = boost_step(B, b, p->e_ol[a], &add, &sc);\n          (void)add;"),
    ("word boost table: epsilon arcs with a word are not boosted",
     "        nb = boost_step(B, b, p->x_ol[a], &add, &sc);\n        if (add) nc = canon(nc + sc);",
     "        nb = boost_step(B, b, p->x_ol[a], &add, &sc);\n        (void)add;"),
    ("word boost table: the score of the next word id is taken",
     "if (B->table) { *add = 1; *score = B->table[o]; return 0; }",
     "if (B->table) { *add = 1; *score = B->table[o > 1 ? o - 1 : o]; return 0; }"),
    ("word boost: the score is subtracted",
     "        if (boost && p->e_ol[a] != 0) nc = canon(nc + boost[p->e_ol[a]]);\n          if (frame_best)",
     "        if (boost && p->e_ol[a] != 0) nc = canon(nc - boost[p->e_ol[a]]);\n          if (frame_best)"),
]


def _run_pins(tmp_root, pin_files=None):
    env = dict(os.environ, PYTHONPATH=os.pathsep.join([tmp_root, ROOT]))
    # the child's working directory comes first on its module path: the copy there shadows oracle/
    files = [os.path.join(ROOT, f) for f in (pin_files or PIN_FILES)]
    probe = subprocess.run([sys.executable, "-c", "import oracle; print(oracle.__file__)"],
                           cwd=tmp_root, env=env, capture_output=True, text=True)
    assert probe.stdout.strip().startswith(tmp_root), (probe.stdout, probe.stderr)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + files,
                          cwd=tmp_root, env=env, capture_output=True, text=True)


def _copy_oracle(tmp_path, old=None, new=None):
    dst = tmp_path / "oracle"
    dst.mkdir()
    for f in ("__init__.py", "wfst_oracle.py", "wfst_oracle.c"):
        shutil.copy(os.path.join(ROOT, "oracle", f), dst / f)
    if old is not None:
        src = (dst / "wfst_oracle.c").read_text()
        assert src.count(old) == 1, f"mutation site not found exactly once: {old!r}"
        (dst / "wfst_oracle.c").write_text(src.replace(old, new))
    return str(tmp_path)


def test_unmutated_copy_passes(tmp_path):
    """The harness itself: an exact copy of the oracle, loaded from the side, passes the pins."""
    r = _run_pins(_copy_oracle(tmp_path))
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "passed" in r.stdout


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, old, new):
    r = _run_pins(_copy_oracle(tmp_path, old, new))
    assert r.returncode == 1 and "failed" in r.stdout, f"mutant survived ({name}):\n" + r.stdout[-1500:] + r.stderr[-1500:]


def test_unmutated_copy_passes_the_option_pins(tmp_path):
    r = _run_pins(_copy_oracle(tmp_path), OPTION_PIN_FILES)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]


@pytest.mark.parametrize("name,old,new", OPTION_MUTANTS, ids=[m[0] for m in OPTION_MUTANTS])
def test_option_mutant_is_caught(tmp_path, name, old, new):
    r = _run_pins(_copy_oracle(tmp_path, old, new), OPTION_PIN_FILES)
    assert r.returncode == 1 and "failed" in r.stdout, f"mutant survived ({name}):\n" + r.stdout[-1500:] + r.stderr[-1500:]
