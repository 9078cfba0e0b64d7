"""Each plausible mistake, planted in a copy of the oracle source, must fail at least one pin.

The copies are compiled on the CPU into a temporary directory; the committed
oracle is never modified.
"""

import os

import pytest

import oracle
import oracle_pins

# (name, text in px_oracle.cpp, replacement)
MUTANTS = [
    ("coalesce_overwrites", "row[(size_t) d] += load_value(val[w], val_dtype, i * dim + d);",
     "row[(size_t) d] = load_value(val[w], val_dtype, i * dim + d);"),
    ("coalesce_wrong_column", "load_value(val[w], val_dtype, i * dim + d);",
     "load_value(val[w], val_dtype, i * dim);"),
    ("coalesce_wrong_row", "load_value(val[w], val_dtype, i * dim + d);",
     "load_value(val[w], val_dtype, d);"),
    ("coalesce_average_per_occurrence", "if (aggregation == AGG_AVERAGE) s /= (double) n_workers;\n            out_rows",
     "if (aggregation == AGG_AVERAGE) s /= (double) seen[kv.first];\n            out_rows"),
    ("coalesce_skips_range_check", "if (idx[w][i] < 0 || idx[w][i] >= vocab) return -1;",
     "if (idx[w][i] < 0) return -1;"),
    ("coalesce_run_len_off", "seen[idx[w][i]] += 1;", "seen[idx[w][i]] = 1;"),
    ("bf16_shift", "[i] << 16;", "[i] << 15;"),
    ("hash_wraps_at_32", "h *= 2654435761ULL;", "h = (uint32_t) (h * 2654435761ULL);"),
    ("hash_other_constant", "h *= 2654435761ULL;", "h *= 2654435769ULL;"),
    ("offsets_not_cumulative", "out_offsets[p + 1] = out_offsets[p] + fill[(size_t) p];",
     "out_offsets[p + 1] = fill[(size_t) p];"),
    ("perm_holds_ids", "out_perm[next[(size_t) p]++] = (int32_t) k;",
     "out_perm[next[(size_t) p]++] = (int32_t) ids[k];"),
    ("sgd_sign", "(double) w[d] - lr * (double) g[d]", "(double) w[d] + lr * (double) g[d]"),
    ("sgd_ignores_lr", "(double) w[d] - lr * (double) g[d]", "(double) w[d] - (double) g[d]"),
    ("sgd_row_by_visit_order", "const float* g = rows + k * dim;\n        for (int64_t d = 0; d < dim; ++d) w[d] = (float) ((double) w[d] -",
     "const float* g = rows + j * dim;\n        for (int64_t d = 0; d < dim; ++d) w[d] = (float) ((double) w[d] -"),
    ("adagrad_no_square", "(double) a[d] + gd * gd;", "(double) a[d] + gd;"),
    ("adagrad_no_sqrt", "(std::sqrt(ad) + eps)", "(ad + eps)"),
    ("adagrad_old_accumulator", "(std::sqrt(ad) + eps)", "(std::sqrt((double) a[d] - gd * gd) + eps)"),
    ("adagrad_accumulator_not_stored", "a[d] = (float) ad;", ""),
    ("adagrad_eps_inside_root", "(std::sqrt(ad) + eps)", "std::sqrt(ad + eps)"),
    ("adagrad_sign", "(double) w[d] - lr * gd /", "(double) w[d] + lr * gd /"),
    ("lookup_wrong_source_row", "out[k * dim + d] = table[ids[k] * dim + d];", "out[k * dim + d] = table[k * dim + d];"),
    ("lookup_by_visit_order", "out[k * dim + d] = table[ids[k] * dim + d];", "out[j * dim + d] = table[ids[k] * dim + d];"),
    ("lookup_ignores_range", "for (int64_t j = first; j < last && j < n; ++j) {\n        int64_t k = perm ? perm[j] : j;\n        for",
     "for (int64_t j = 0; j < n; ++j) {\n        int64_t k = perm ? perm[j] : j;\n        for"),
    ("dense_overwrites", "s += load_value(bufs[w], in_dtype, j);", "s = load_value(bufs[w], in_dtype, j);"),
    ("dense_wrong_divisor", "if (aggregation == AGG_AVERAGE) s /= (double) n_buffers;",
     "if (aggregation == AGG_AVERAGE) s /= (double) (n_buffers - 1);"),
    ("dense_float_accumulator", "double s = 0.0;\n        for (int w = 0; w < n_buffers; ++w) s +=",
     "float s = 0.0f;\n        for (int w = 0; w < n_buffers; ++w) s += (float)"),
]


@pytest.fixture(scope="module")
def source():
    with open(oracle.SOURCE) as f:
        return f.read()


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, old, new, source, tmp_path):
    assert source.count(old) == 1, "mutation site for %s not unique / not found" % name
    src = tmp_path / "mutant.cpp"
    src.write_text(source.replace(old, new))
    lib_path = oracle.build(str(src), os.path.join(str(tmp_path), "libmutant_%s.so" % name))
    lib = oracle.load(lib_path)
    caught = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(lib)
        except (AssertionError, IndexError):
            caught.append(pin.__name__)
            break       # never keep driving a broken oracle: later pins would index with its output
    assert caught, "no pin notices the planted mistake %r" % name
