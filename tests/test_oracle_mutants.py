"""Each plausible mistake, planted in a copy of the oracle on the CPU, must be
caught by at least one pin.  The real oracle source is never modified."""
import os
import subprocess

import pytest

import oracle
import oracle_pins as P

SRC = os.path.join(os.path.dirname(oracle.__file__), "omniattn_oracle.c")

# (name, text to find, replacement)
MUTANTS = [
    ("sink_off_by_one", "return (j < S) || (j >= L - W);", "return (j <= S) || (j >= L - W);"),
    ("window_off_by_one", "return (j < S) || (j >= L - W);", "return (j < S) || (j > L - W);"),
    ("no_sink", "return (j < S) || (j >= L - W);", "return (j >= L - W);"),
    ("double_count_overlap", "if (oracle_is_retained(j, L, S, W))\n                idx[n++] = j;",
     "if (oracle_is_retained(j, L, S, W))\n                idx[n++] = j;\n        if (S + W > L && n > 0) idx[n - 1] = idx[0];"),
    ("value_slice_shifted", "o[c] += p * kv[t * QK_DIM + c];", "o[c] += p * kv[t * QK_DIM + c + 64];"),
    ("logit_512_dims", "for (int d = 0; d < QK_DIM; ++d)\n                acc += qd[d] * kv[t * QK_DIM + d];",
     "for (int d = 0; d < V_DIM; ++d)\n                acc += qd[d] * kv[t * QK_DIM + d];"),
    ("scale_dropped", "s[t] = scale * acc;", "s[t] = acc;"),
    ("scale_sqrt576", "s[t] = scale * acc;", "s[t] = acc / 24.0;"),
    ("no_max_in_lse", "lse[i] = m + log(Z);", "lse[i] = log(Z);"),
    ("unnormalised", "double p = exp(s[t] - m) / Z;", "double p = exp(s[t] - m);"),
    ("page_slot_swapped", "int64_t slot = j % PAGE;", "int64_t slot = (j + 1) % PAGE;"),
    ("page_table_stride", "page_table[(int64_t)b * max_pages + j / PAGE]", "page_table[(int64_t)b * (max_pages - 1) + j / PAGE]"),
    ("fp8_scale_ignored", "oracle_fp8_e4m3_to_double(c8[row + d]) * sc;", "oracle_fp8_e4m3_to_double(c8[row + d]);"),
    ("fp8_bias_8", "ldexp(1.0 + (double)m / 8.0, e - 7);", "ldexp(1.0 + (double)m / 8.0, e - 8);"),
    ("fp8_subnormal", "ldexp((double)m / 8.0, -6);", "ldexp((double)m / 8.0, -7);"),
    ("fp8_inf_codes", "if (e == 0xF && m == 0x7)", "if (e == 0xF)"),
    ("bf16_shift", "(uint32_t)bits << 16;", "(uint32_t)bits << 15;"),
    ("empty_set_lse_zero", "lse[i] = -INFINITY;", "lse[i] = 0.0;"),
    ("mq_query_index", "int32_t t = h / Hq;", "int32_t t = h % q_len;"),
    ("mq_length_off_by_one", "int64_t L = L_seq - (q_len - 1 - t);", "int64_t L = L_seq - (q_len - t);"),
    ("mq_not_causal", "int64_t L = L_seq - (q_len - 1 - t);", "int64_t L = L_seq;"),
    ("head_index", "q[((int64_t)b * H + h) * QK_DIM + d]", "q[((int64_t)b * H + (H - 1 - h)) * QK_DIM + d]"),
]


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(name, find, repl, tmp_path, oracle_lib):
    text = open(SRC).read()
    assert text.count(find) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / f"{name}.c"
    src.write_text(text.replace(find, repl))
    lib = str(tmp_path / f"lib{name}.so")
    oracle.build(force=True, src=str(src), out=lib)
    caught = []
    for pin in P.ALL_PINS:
        try:
            pin(lib)
        except AssertionError:
            caught.append(pin.__name__)
            break
        except RuntimeError:          # the mutant made the oracle itself report an error
            caught.append(pin.__name__)
            break
    assert caught, f"no pin catches mutant {name}"
