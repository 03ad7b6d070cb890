"""Show that the pins bite: each plausible mistake, planted into a temporary copy
of the oracle's C source on the CPU, must make at least one pin fail.  Every planted
mistake keeps all memory accesses inside the arrays the pins pass in (a mutant runs in
this process)."""
import os

import pytest

import oracle_pins

# (label, text in oracle/adam_mini_oracle.c, replacement)
MUTANTS = [
    ("no weight decay", "p[i * stride] = p[i * stride] - lr * lambda * p[i * stride];", "p[i * stride] = p[i * stride];"),
    ("decay sign flipped", "p[i * stride] = p[i * stride] - lr * lambda * p[i * stride];", "p[i * stride] = p[i * stride] + lr * lambda * p[i * stride];"),
    ("beta1 weights swapped", "m[i * stride] = (1.0 - beta1) * gi + beta1 * m[i * stride];", "m[i * stride] = beta1 * gi + (1.0 - beta1) * m[i * stride];"),
    ("m uses beta2", "m[i * stride] = (1.0 - beta1) * gi + beta1 * m[i * stride];", "m[i * stride] = (1.0 - beta2) * gi + beta2 * m[i * stride];"),
    ("sum instead of mean", "double mean_sq = sum_sq / (double)n;", "double mean_sq = sum_sq;"),
    ("mean of |g| instead of g*g", "sum_sq += gi * gi;", "sum_sq += fabs(gi);"),
    ("square of the mean", "double mean_sq = sum_sq / (double)n;", "double mean_sq = sum_sq / (double)n; mean_sq = mean_sq * mean_sq;"),
    ("beta2 weights swapped", "*v = (1.0 - beta2) * stat + beta2 * (*v);", "*v = beta2 * stat + (1.0 - beta2) * (*v);"),
    ("v not accumulated", "*v = (1.0 - beta2) * stat + beta2 * (*v);", "*v = (1.0 - beta2) * stat;"),
    ("no bias correction of m", "double m_hat = m[i * stride] / bias1;", "double m_hat = m[i * stride];"),
    ("no bias correction of v", "double v_hat = *v / bias2;", "double v_hat = *v;"),
    ("bias correction of m uses t+1", "double bias1 = 1.0 - pow(beta1, (double)t);", "double bias1 = 1.0 - pow(beta1, (double)t + 1.0);"),
    ("bias correction of v uses t+1", "double bias2 = 1.0 - pow(beta2, (double)t);", "double bias2 = 1.0 - pow(beta2, (double)t + 1.0);"),
    ("bias2 uses beta1", "double bias2 = 1.0 - pow(beta2, (double)t);", "double bias2 = 1.0 - pow(beta1, (double)t);"),
    ("eps inside the root", "(sqrt(v_hat) + eps)", "sqrt(v_hat + eps)"),
    ("eps dropped", "(sqrt(v_hat) + eps)", "(sqrt(v_hat))"),
    ("eps added twice", "(sqrt(v_hat) + eps)", "(sqrt(v_hat) + eps + eps)"),
    ("no square root", "(sqrt(v_hat) + eps)", "(v_hat + eps)"),
    ("update sign", "p[i * stride] = p[i * stride] - lr * m_hat / (sqrt(v_hat) + eps);", "p[i * stride] = p[i * stride] + lr * m_hat / (sqrt(v_hat) + eps);"),
    ("update uses g not m", "double m_hat = m[i * stride] / bias1;", "double m_hat = amo_grad_at(g, dtype, g_first + i * stride);"),
    ("gradient offset ignored", "amo_step_block(p + first, m + first, v + b, g, dtype, first, block_numel,", "amo_step_block(p + first, m + first, v + b, g, dtype, 0, block_numel,"),
    ("one v for the whole tensor", "amo_step_block(p + first, m + first, v + b,", "amo_step_block(p + first, m + first, v + 0 * b,"),
    ("block id ignores earlier tensors", "return blocks_before + elem / block_numel[tensor];", "return elem / block_numel[tensor];"),
    ("block id counts elements", "blocks_before += numel[k] / block_numel[k];", "blocks_before += numel[k];"),
    ("block id rounds up", "return blocks_before + elem / block_numel[tensor];", "return blocks_before + (elem + block_numel[tensor] - 1) / block_numel[tensor];"),
    ("strided blocks: gradient read with stride 1", "double gi = amo_grad_at(g, dtype, g_first + i * stride);\n    sum_sq", "double gi = amo_grad_at(g, dtype, g_first + i);\n    sum_sq"),
    ("strided blocks: first moment reads the gradient with stride 1", "double gi = amo_grad_at(g, dtype, g_first + i * stride);\n    m[i", "double gi = amo_grad_at(g, dtype, g_first + i);\n    m[i"),
    ("strided blocks: columns taken in reverse", "uint64_t first = strided ? (uint64_t)b : (uint64_t)b * block_numel;", "uint64_t first = strided ? (uint64_t)(n_blocks - 1 - b) : (uint64_t)b * block_numel;"),
    ("strided blocks: stride is block_numel", "uint64_t stride = strided ? (uint64_t)n_blocks : 1;", "uint64_t stride = strided ? block_numel : 1;"),
    ("strided blocks: flag ignored", "uint64_t stride = strided ? (uint64_t)n_blocks : 1;", "uint64_t stride = 1;"),
    ("strided block id uses division", "return blocks_before + elem % (numel[tensor] / block_numel[tensor]);", "return blocks_before + elem / block_numel[tensor];"),
    ("strided block id modulo block_numel", "return blocks_before + elem % (numel[tensor] / block_numel[tensor]);", "return blocks_before + elem % block_numel[tensor];"),
    ("bf16 shifted wrongly", "<< 16;", "<< 15;"),
    ("reducer ignored", "if (reducer != AMO_REDUCE_MEAN) {", "if (0) {"),
    ("1-norm divided by n", "stat = norm1;", "stat = norm1 / (double)n;"),
    ("2-norm without the root", "stat = sqrt(sum_s2);", "stat = sum_s2;"),
    ("2-norm of g instead of g.*g", "sum_s2 += si * si;", "sum_s2 += si;"),
    ("max and min swapped", "if (i == 0 || si > largest) largest = si;", "if (i == 0 || si < largest) largest = si;"),
    ("min starts from zero", "if (i == 0 || si < smallest) smallest = si;", "if (si < smallest) smallest = si;"),
    ("statistics of |g| instead of g.*g", "double si = gi * gi;", "double si = fabs(gi);"),
    ("max does not hand a NaN on", "if (any_nan) stat = NAN;", ""),
    ("alternative statistic strided read with stride 1", "double gi = amo_grad_at(g, dtype, g_first + i * stride);\n      double si", "double gi = amo_grad_at(g, dtype, g_first + i);\n      double si"),
]


def _failing_pins(lib):
    failed = []
    for pin in oracle_pins.ALL_PINS:
        try:
            pin(lib)
        except AssertionError:
            failed.append(pin.__name__)
        except Exception:
            failed.append(pin.__name__)
    return failed


@pytest.mark.parametrize("label,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(oracle, tmp_path, label, old, new):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "adam_mini_oracle.c")).read()
    assert src.count(old) >= 1, "mutation site not found: %r" % old
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    lib = oracle.OracleLib(oracle.compile_c(str(mutated), str(tmp_path / "libmutant.so")))
    assert _failing_pins(lib), "no pin notices: %s" % label


def test_unmutated_passes_all(oracle):
    assert _failing_pins(oracle.default_lib()) == []
