"""The pins of test_oracle_pins.py and test_oracle_prefill.py are only worth something if they
reject a wrong oracle.  Each case below plants one plausible mistake in a copy of the oracle's C
source (a dropped term, a flipped sign, a wrong index, a transposed operand, a weakened
comparison), builds it on the CPU and runs the pins against it: they must fail.  Nothing here
touches the GPU or the real oracle."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "fd_oracle.c")

MUTANTS = [
    ("KV head of a query head taken modulo instead of by division", "int hkv = hq / G;", "int hkv = hq % p->Hkv;"),
    ("lower bound of the guard made non-strict", "if (d <= p->lo || d >= p->hi) cf = 1;", "if (d < p->lo || d >= p->hi) cf = 1;"),
    ("upper bound of the guard made non-strict", "if (d <= p->lo || d >= p->hi) cf = 1;", "if (d <= p->lo || d > p->hi) cf = 1;"),
    ("logit scale dropped", "x[j] = p->s * acc;", "x[j] = acc;"),
    ("guard on x + phi", "double d = x[j] - p->phi;", "double d = x[j] + p->phi;"),
    ("unified weights e^{x + phi}", "double e = exp(x[j] - p->phi);", "double e = exp(x[j] + p->phi);"),
    ("Eq. 2 rescaling factors swapped", "double a1 = exp(M - Mn), a2 = exp(m[c] - Mn);", "double a2 = exp(M - Mn), a1 = exp(m[c] - Mn);"),
    ("Eq. 2 denominators added without rescaling", "L = a1 * L + a2 * l[c];", "L = L + l[c];"),
    ("softmax not normalised", "for (int j = 0; j < n; ++j) w[j] /= l;", ""),
    ("minimum instead of maximum subtracted", "if (x[j] > m) m = x[j];", "if (x[j] < m) m = x[j];"),
    ("fp16 subnormal exponent off by one", "ldexp((double)m, -24)", "ldexp((double)m, -25)"),
    ("V indexed transposed", "out[t] += w[j] * v[(size_t)j * D + t];", "out[t] += w[j] * v[(size_t)t * n + j];"),
    ("sequence stride of the K cache dropped",
     "const uint16_t *kr = p->k + ((size_t)b * p->Hkv + hkv) * (size_t)p->Smax * p->D;",
     "const uint16_t *kr = p->k + ((size_t)b * p->Hkv + hkv) * (size_t)p->D;"),
    ("chunk flags written at the wrong index", "p->chunk_flags[row * nc + c] = cf;", "p->chunk_flags[row + c] = cf;"),
    ("margin ignores the upper bound", "if (db < margin) margin = db;", ""),
]


@pytest.mark.parametrize("what,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_reject_a_planted_mistake(tmp_path, what, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, "the oracle no longer contains the line this case mutates: %r" % old
    mutant_c = tmp_path / "fd_oracle_mutant.c"
    mutant_so = tmp_path / "libfd_oracle_mutant.so"
    mutant_c.write_text(text.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                           "-o", str(mutant_so), str(mutant_c), "-lm"])
    env = dict(os.environ, FD_ORACLE_LIB=str(mutant_so))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert r.returncode != 0, "the pins accept an oracle with this mistake: %s" % what


def test_pins_accept_the_unmutated_copy(tmp_path):
    so = tmp_path / "libfd_oracle_copy.so"
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                           "-o", str(so), SRC, "-lm"])
    env = dict(os.environ, FD_ORACLE_LIB=str(so))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert r.returncode == 0, r.stdout.decode()[-2000:]


PREFILL_SRC = os.path.join(ROOT, "oracle", "fd_prefill_oracle.c")
PREFILL_MUTANTS = [
    ("a token does not see itself", "for (int j = 0; j <= i; ++j) {                            /* token i sees tokens 0..i */",
     "for (int j = 0; j < i; ++j) {"),
    ("weights summed over one key too many", "for (int j = 0; j <= i; ++j) {\n        double w = exp(x[j] - m);",
     "for (int j = 0; j <= i + 1 && j < nb; ++j) {\n        double w = exp(x[j] - m);"),
    ("logit scale dropped", "x[j] = p->s * acc;", "x[j] = acc;"),
    ("KV head taken modulo", "hkv = hq / G;", "hkv = hq % p->Hkv;"),
    ("query row stride dropped", "const uint16_t *qr = p->q + (((size_t)b * p->Hq + hq) * p->Smax + i) * D;",
     "const uint16_t *qr = p->q + (((size_t)b * p->Hq + hq) + i) * D;"),
    ("guard made non-strict", "if (!(d > p->lo && d < p->hi)) bad = 1;", "if (!(d >= p->lo && d <= p->hi)) bad = 1;"),
    ("output not normalised", "for (int t = 0; t < D; ++t) o[t] /= l;", ""),
    ("rows beyond the prompt computed", "if (i >= nb) return;", ""),
]


@pytest.mark.parametrize("what,old,new", PREFILL_MUTANTS, ids=[m[0] for m in PREFILL_MUTANTS])
def test_prefill_pins_reject_a_planted_mistake(tmp_path, what, old, new):
    text = open(PREFILL_SRC).read()
    assert text.count(old) >= 1, "the prefill oracle no longer contains the line this case mutates: %r" % old
    mutant_c = tmp_path / "fd_prefill_oracle_mutant.c"
    mutant_so = tmp_path / "libfd_prefill_oracle_mutant.so"
    mutant_c.write_text(text.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
                           "-o", str(mutant_so), str(mutant_c), "-lm"])
    env = dict(os.environ, FD_PREFILL_ORACLE_LIB=str(mutant_so))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_prefill.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
    assert r.returncode != 0, "the pins accept a prefill oracle with this mistake: %s" % what


# ---- the paged-cache oracle (Python): the same exercise, in process ----
PAGED_SRC = os.path.join(ROOT, "oracle", "fd_paged_oracle.py")
PAGED_MUTANTS = [
    ("pages put back in reverse order", "pid = int(table[b, j])", "pid = int(table[b, (n + P - 1) // P - 1 - j])"),
    ("the partly filled last page dropped", "for j in range((n + P - 1) // P):", "for j in range(n // P):"),
    ("the table read transposed", "pid = int(table[b, j])", "pid = int(table.reshape(-1)[j * B + b])"),
    ("KV heads of a page reversed", "= pool[pid]", "= pool[pid][::-1]"),
    ("rows of a page shifted by one", "= pool[pid]", "= np.roll(pool[pid], 1, axis=1)"),
    ("V gathered from the K pool", "v = gather_pages(v_pool, table, page_size, seq_lens)", "v = gather_pages(k_pool, table, page_size, seq_lens)"),
    ("lengths not clamped to the table's capacity", "n = int(min(max(int(seq_lens[b]), 0), T * P))", "n = int(seq_lens[b])"),
]


def _paged_pin_calls(pins):
    calls = [(pins.test_gather_follows_the_table_token_by_token, (P,)) for P in (4, 16, 32)]
    calls += [(pins.test_identity_table_is_the_contiguous_cache, ())]
    calls += [(pins.test_paged_attention_equals_contiguous_attention, (P,)) for P in (8, 32)]
    calls += [(pins.test_placement_in_the_pool_and_unused_pages_do_not_matter, ()), (pins.test_brute_force_one_row, ()),
              (pins.test_flags_count_logical_positions, ()), (pins.test_lengths_beyond_the_capacity_are_clamped, ())]
    return calls


def _load_paged(text):
    import types
    mod = types.ModuleType("oracle.fd_paged_oracle_variant")
    mod.__package__ = "oracle"
    exec(compile(text, PAGED_SRC, "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("what,old,new", PAGED_MUTANTS, ids=[m[0] for m in PAGED_MUTANTS])
def test_paged_pins_reject_a_planted_mistake(monkeypatch, what, old, new):
    import test_oracle_paged as pins
    text = open(PAGED_SRC).read()
    assert text.count(old) >= 1, "the paged oracle no longer contains the line this case mutates: %r" % old
    monkeypatch.setattr(pins, "po", _load_paged(text.replace(old, new)))
    failed = 0
    for fn, a in _paged_pin_calls(pins):
        try:
            fn(*a)
        except Exception:
            failed += 1
    assert failed, "the pins accept a paged oracle with this mistake: %s" % what


def test_paged_pins_accept_the_unmutated_copy(monkeypatch):
    import test_oracle_paged as pins
    monkeypatch.setattr(pins, "po", _load_paged(open(PAGED_SRC).read()))
    for fn, a in _paged_pin_calls(pins):
        fn(*a)
