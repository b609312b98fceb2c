"""The pins must notice a broken oracle: each case plants one plausible mistake in a copy of the
oracle's source (a dropped term, a wrong sign, a sum for a mean, an unstable sort, a wrong constant ...),
builds it, and checks that at least one pin of tests/test_oracle_pins.py fails against it.  CPU only.

A planted mistake may read or write out of bounds (a wrong column, a transposed index), so every pin that is run
against a mutant runs in a child process: a failed assertion there (exit status 3) or a crash both count as
"noticed", and whatever the mutant did to its heap ends with the child."""
import os
import subprocess
import sys
import tempfile

import pytest

from oracle import oracle as O
from tests import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(O.__file__), "persia_oracle.cpp")

# (name, text in the oracle, replacement, pins expected to catch it)
MUTANTS = [
    ("hash_multiplier", "z *= 0x9FB21C651E98DF25ull;", "z *= 0x9FB21C651E98DF27ull;",
     [("test_mix64_is_the_documented_bijection", ())]),
    ("hash_salt_dropped", "return mix64(id + o.slot_salt[slot]) % t.rows;", "return mix64(id) % t.rows;",
     [("test_hash_identity_is_mod_and_mix_is_salted_mod", ())]),
    ("bf16_truncates", "if (lower > 0x8000u || (lower == 0x8000u && odd)) upper += 0x10000u;", "",
     [("test_bf16_round_matches_torch_cast", ())]),
    ("bf16_ties_away", "(lower == 0x8000u && odd)", "(lower == 0x8000u)",
     [("test_bf16_round_matches_torch_cast", ())]),
    ("pool_skips_duplicates", "for (uint32_t d = 0; d < D; ++d) sum[d] += (double)w[d];",
     "if (i == offsets[bag] || ids[i] != ids[i - 1]) for (uint32_t d = 0; d < D; ++d) sum[d] += (double)w[d];",
     [("test_lookup_pool_integer_table_duplicates_and_order", ())]),
    ("pool_wrong_column", "float* out = pooled + (size_t)b * o.width + o.slot_col[s];",
     "float* out = pooled + (size_t)b * o.width + (size_t)s * D;",
     [("test_lookup_pool_mixed_tables_column_layout", ())]),
    ("dedup_unstable", "return a.first < b.first;",
     "return a.first < b.first || (a.first == b.first && a.second > b.second);",
     [("test_dedup_against_dict_and_numpy_unique", (1, 8,))]),
    ("dedup_key_without_table", "occ.emplace_back(((uint64_t)o.slot_table[s] << 32) | hash_row(o, ids[i], s), (uint32_t)bag);",
     "occ.emplace_back(hash_row(o, ids[i], s), (uint32_t)bag);",
     [("test_dedup_against_dict_and_numpy_unique", (2, 100,))]),
    ("grad_transposed_index", "const float* g = d_pooled + (size_t)(bag / S) * o.width + o.slot_col[bag % S];",
     "const float* g = d_pooled + (size_t)(bag % S) * o.width + o.slot_col[bag / S % S];",
     [("test_gradient_matches_autograd_and_count_matrix_transpose", ())]),
    ("sgd_wrong_sign", "w[d] = store_round(t, (double)w[d] - (double)o.lr * G[d]);",
     "w[d] = store_round(t, (double)w[d] + (double)o.lr * G[d]);",
     [("test_sgd_matches_torch_sgd_and_leaves_other_rows_alone", ())]),
    ("adagrad_sum_for_mean", "double a = (double)t.acc[idx] + sq / (double)D;", "double a = (double)t.acc[idx] + sq;",
     [("test_rowwise_adagrad_uses_mean_not_sum_and_eps_outside_sqrt", ())]),
    ("adagrad_eps_inside_root", "double denom = std::sqrt(a) + (double)o.eps;",
     "double denom = std::sqrt(a + (double)o.eps);",
     [("test_rowwise_adagrad_uses_mean_not_sum_and_eps_outside_sqrt", ())]),
    ("adagrad_old_accumulator", "double denom = std::sqrt(a) + (double)o.eps;",
     "double denom = std::sqrt((double)t.acc[idx]) + (double)o.eps;",
     [("test_rowwise_adagrad_dim1_is_textbook_adagrad", ())]),
    ("adagrad_state_not_stored", "t.acc[idx] = (float)a;", "",
     [("test_rowwise_adagrad_dim1_is_textbook_adagrad", ())]),
    ("init_fused_multiply_add", "volatile float prod = (float)k * scale;\n  volatile float v = prod + mid;",
     "volatile float v = (float)((double)k * (double)scale + (double)mid);",
     [("test_init_value_is_exactly_the_two_rounding_definition", ())]),
    ("bf16_store_rounds_twice", "float store_round(const Table& t, double v) { return t.dtype == DT_BF16 ? round_bf16_once(v) : (float)v; }",
     "float store_round(const Table& t, double v) { return t.dtype == DT_BF16 ? round_bf16((float)v) : (float)v; }",
     [("test_bf16_table_update_does_not_round_through_fp32", ())]),
    ("bf16_once_ties_away", "const double r = std::nearbyint(scaled);", "const double r = std::round(scaled);",
     [("test_store_rounds_fp64_to_bf16_once", ())]),
    ("init_ignores_table", "uint64_t table_key = mix64(seed + (uint64_t)(t + 1) * 0x9E3779B97F4A7C15ull);",
     "uint64_t table_key = mix64(seed);", [("test_init_range_uniformity_and_determinism", ())]),
]


ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHILD = """
import sys
sys.path.insert(0, sys.argv[1])
from oracle import oracle as O
from tests import test_oracle_pins as pins
O._lib = O.load(sys.argv[2])
try:
    getattr(pins, sys.argv[3])(*eval(sys.argv[4]))
except AssertionError:
    sys.exit(3)
sys.exit(0)
"""


@pytest.mark.parametrize("name,old,new,catchers", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(name, old, new, catchers):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutant {name}: the oracle text it edits has changed"
    with tempfile.TemporaryDirectory() as d:
        path = os.path.join(d, "mutant.cpp")
        open(path, "w").write(src.replace(old, new))
        lib = os.path.join(d, "libmutant.so")
        subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-o", lib, path], check=True)
        caught = False
        for pin, args in catchers:
            r = subprocess.run([sys.executable, "-c", CHILD, ROOT, lib, pin, repr(args)], capture_output=True, text=True)
            # 3: the pin's assertion failed; a signal (negative) or abort: the mutant crashed -- noticed either way
            assert r.returncode in (0, 3) or r.returncode < 0 or r.returncode in (134, 139), \
                f"mutant {name}: the child could not run pin {pin}: {r.stderr[-2000:]}"
            if r.returncode != 0:
                caught = True
        assert caught, f"mutant {name} passed every pin that should have caught it"
    pin, args = catchers[0]
    getattr(pins, pin)(*args)   # and the real oracle still passes
