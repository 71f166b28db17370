"""Do the pins notice a mistake?  Each case plants ONE plausible mistake in a copy of the oracle's
source (a dropped term, a wrong comparison, a swapped rule), builds it, and runs the pins against
that library in a child process: they must fail.  CPU only; nothing here touches the device path."""
import os
import shlex
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "monolith_oracle.cpp")

# (name, text in the source, replacement, pin tests that must notice)
MUTATIONS = [
    ("eps_inside_root", "double denom = std::sqrt(acc) + eps;", "double denom = std::sqrt(acc + eps);",
     "tests/test_oracle_pins.py -k adagrad"),
    ("sum_instead_of_mean_of_squares", "double acc = (double)e->acc + ss / (double)p.dim;",
     "double acc = (double)e->acc + ss;", "tests/test_oracle_pins.py -k adagrad"),
    ("expiry_strictly_greater", "if (now - it->second.last_seen >= p_.expire_steps) {",
     "if (now - it->second.last_seen > p_.expire_steps) {", "tests/test_oracle_semantics.py -k expiry"),
    ("counter_ageing_off_by_one", "if (expire_steps > 0 && step - last >= expire_steps) count = 0;",
     "if (expire_steps > 0 && step - last > expire_steps) count = 0;", "tests/test_oracle_pins.py -k filter_word"),
    ("bf16_truncates", "u += 0x7FFFu + lsb;", "u += 0u;", "tests/test_oracle_pins.py -k bf16"),
    ("touched_survives_expiry", "        touched_.erase(it->first);\n", "", "tests/test_oracle_maintenance.py -k touched"),
    ("grown_counters_by_low_bits", "grown[i] = filter_[i >> k];", "grown[i] = filter_[i & ((p_.n_filter >> k) - 1)];",
     "tests/test_oracle_maintenance.py -k grow"),
    ("salt_off_by_one", "return mix64(seed + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull);",
     "return mix64(seed + (uint64_t)(i + 2) * 0x9E3779B97F4A7C15ull);", "tests/test_oracle_pins.py -k mixer"),
    ("mixer_shift", "z ^= z >> 27;", "z ^= z >> 26;", "tests/test_oracle_pins.py -k mixer"),
    ("min_of_counters_becomes_first", "count = std::min(count, filter_[filter_index(k, j)] & 255u);",
     "if (j == 0) count = filter_[filter_index(k, j)] & 255u;", "tests/test_oracle_filter.py"),
    ("restore_ignores_last_seen", "    e.last_seen = last_seen[i];", "    e.last_seen = 0;",
     "tests/test_oracle_maintenance.py -k restored_table"),
    ("admission_strictly_above_threshold", "if (count >= p_.freq_threshold) admissible.insert(k);",
     "if (count > p_.freq_threshold) admissible.insert(k);", "tests/test_oracle_semantics.py -k threshold"),
    ("hits_are_counted_too", "      if (k == kEmptyKey || was_hit[i]) continue;\n      for (uint32_t j = 0; j < p_.filter_hashes; ++j) {  // one touch per counter of the key",
     "      if (k == kEmptyKey) continue;\n      for (uint32_t j = 0; j < p_.filter_hashes; ++j) {  // one touch per counter of the key",
     "tests/test_oracle_semantics.py tests/test_oracle_pins.py -k 'filter or counter or tiny'"),
    ("misses_refresh_last_seen_of_nothing_hits_do_not", "if (it != table_.end() && was_hit[i]) it->second.last_seen = step;",
     "if (it != table_.end() && !was_hit[i]) it->second.last_seen = step;", "tests/test_oracle_semantics.py -k 'expiry or last_seen'"),
    ("init_from_wrong_bits", "uint32_t u24 = (uint32_t)(h >> 40);", "uint32_t u24 = (uint32_t)(h >> 39) & 0xFFFFFFu;",
     "tests/test_oracle_pins.py -k init"),
    ("stash_forgotten_by_rehash", "    for (auto& st : stash_) all.push_back(st);\n", "", "tests/test_oracle_maintenance.py -k stash"),
    ("restored_keys_leave_counters_alone", "if ((w & 255u) < least) set_filter_word(i, (w & ~255u) | least);", "",
     "tests/test_oracle_maintenance.py -k restored_keys"),
    ("touched_set_is_never_emptied", "    touched_.clear();\n", "", "tests/test_oracle_maintenance.py -k touched"),
    ("rehash_keeps_the_old_placement_salts", "    p_.s_h0 = salt(placement_seed(p_.seed, generation), 0);",
     "    p_.s_h0 = salt(placement_seed(p_.seed, 0), 0);", "tests/test_oracle_maintenance.py -k rehash"),
    ("gradient_of_the_neighbouring_bag", "(double)grad[b * p_.dim + j];", "(double)grad[(b ? b - 1 : 0) * p_.dim + j];",
     "tests/test_oracle_pins.py -k update_equals"),
    ("counter_index_from_the_low_bits", "    return top_bits(mix64(key ^ p_.s_filter[j]), p_.lg_filter);",
     "    return mix64(key ^ p_.s_filter[j]) & (p_.n_filter - 1);",
     "tests/test_oracle_maintenance.py tests/test_oracle_filter.py -k 'grow or count_min'"),
    ("new_keys_are_stamped_with_step_zero", "  e->last_seen = step;", "  e->last_seen = 0;",
     "tests/test_oracle_semantics.py -k expiry"),
    ("accumulator_starts_at_one", "  e->acc = 0.0f;", "  e->acc = 1.0f;", "tests/test_oracle_pins.py -k 'update_equals or torch_adagrad'"),
    ("quotient_and_remainder_swapped", "uint64_t id_r = id % rows, id_q = id / rows;",
     "uint64_t id_q = id % rows, id_r = id / rows;", "tests/test_oracle_quotient_remainder.py"),
    ("quotient_remainder_product_instead_of_sum", "(double)table_r[id_r * dim + j] + (double)table_q[id_q * dim + j];",
     "(double)table_r[id_r * dim + j] * (double)table_q[id_q * dim + j];", "tests/test_oracle_quotient_remainder.py"),
    ("written_counters_may_hide_a_stored_key", "        if (i < first || i - first >= count) continue;\n        uint32_t w = filter_word(i);\n        if ((w & 255u) < least) set_filter_word(i, (w & ~255u) | least);",
     "        if (i < first || i - first >= count) continue;", "tests/test_oracle_maintenance.py -k written_over"),
    ("fill_limit_admits_what_fits", "    if (size_ + admissible.size() > fill_limit()) {", "    if (false) {",
     "tests/test_oracle_semantics.py -k 'fill_limit and cuckoo'"),
    ("fill_limit_is_the_whole_capacity", "uint64_t fill_limit() const { return p_.capacity - p_.capacity / 32; }",
     "uint64_t fill_limit() const { return p_.capacity; }", "tests/test_oracle_semantics.py -k fill_limit"),
    ("evicted_goes_to_same_table", "      side = 1 - side;  // the evicted element goes to its other sub-table",
     "      side = side;", "tests/test_oracle_pins.py -k cuckoo"),
]


def test_the_unmodified_source_contains_every_mutation_site():
    text = open(SRC).read()
    for name, old, _new, _tests in MUTATIONS:
        assert old in text, "mutation %s no longer matches the source" % name


@pytest.mark.parametrize("name,old,new,tests", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_pins_fail_on_a_planted_mistake(tmp_path, name, old, new, tests):
    text = open(SRC).read()
    assert old in text
    src = tmp_path / "mutant.cpp"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-shared", "-fPIC", str(src), "-o", str(lib)])
    env = dict(os.environ, MONOLITH_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + shlex.split(tests),
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=300)
    assert r.returncode == 1, "the pins did not notice %s:\n%s" % (name, r.stdout.decode()[-600:])
