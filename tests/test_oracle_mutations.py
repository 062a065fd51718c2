"""The pins must reject an oracle with a planted mistake.

Each case copies oracle/liec_oracle.c, plants one plausible mistake (a dropped term, a wrong sign,
index, order or operand) and runs the oracle's pin tests against the copy in a child process: at
least one pin has to fail.  The unmodified copy has to pass the same run.  CPU only.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "liec_oracle.c")
PIN_FILES = ["test_oracle_operators.py", "test_oracle_step.py", "test_oracle_sync.py", "test_oracle_blocksign.py",
             "test_oracle_wire.py", "test_oracle_randk.py"]

# (name, text in the oracle, replacement)
MUTANTS = [
    ("sign_of_zero_negative", "p[j] = (v[j] < 0.0f) ? -scale : scale;", "p[j] = (v[j] <= 0.0f) ? -scale : scale;"),
    ("sign_scale_flipped", "p[j] = (v[j] < 0.0f) ? -scale : scale;", "p[j] = (v[j] < 0.0f) ? scale : -scale;"),
    ("l1_summed_in_fp32", "long double sum = 0.0L;", "float sum = 0.0f;"),
    ("l1_without_abs", "sum += fabsl((long double)v[j]);", "sum += (long double)v[j];"),
    ("scale_divides_by_d_minus_1", "float scale = (float)(l1 / (double)d);", "float scale = (float)(l1 / (double)(d > 1 ? d - 1 : d));"),
    ("topk_ties_to_higher_index", None, lambda text: _within(text, "static int compress_topk(", "/* Definition 3",
                                                              "0xffffffffu - ", "0x00000000u + ")),
    ("topk_key_keeps_the_sign_bit", "return u & 0x7fffffffu;", "return u;"),
    ("topk_keeps_k_minus_1", "for (int64_t r = 0; r < k; ++r) {\n            int64_t j = (int64_t)(0xffffffffu - (uint32_t)(order[r] & 0xffffffffu));\n            p[j] = v[j];",
     "for (int64_t r = 0; r + 1 < k; ++r) {\n            int64_t j = (int64_t)(0xffffffffu - (uint32_t)(order[r] & 0xffffffffu));\n            p[j] = v[j];"),
    ("topk_smallest_instead_of_largest", "return (x < y) - (x > y);", "return (x > y) - (x < y);"),
    ("average_forgets_the_global_error", "v[j] = fmaf(acc, inv_n, e[j]);", "v[j] = fmaf(acc, inv_n, 0.0f);"),
    ("average_rounds_twice", "v[j] = fmaf(acc, inv_n, e[j]);", "v[j] = acc * inv_n + e[j];"),
    ("average_in_reverse_worker_order", "for (int32_t i = 0; i < N; ++i)\n            acc = acc + P[(size_t)i * (size_t)d + (size_t)j];",
     "for (int32_t i = N - 1; i >= 0; --i)\n            acc = acc + P[(size_t)i * (size_t)d + (size_t)j];"),
    ("average_divides_by_n_minus_1", "const float inv_n = 1.0f / (float)N;\n    for (int64_t j = 0; j < d; ++j) {\n        float acc = 0.0f;\n        for (int32_t i = 0; i < N; ++i)\n            acc = acc + P",
     "const float inv_n = 1.0f / (float)(N > 1 ? N - 1 : N);\n    for (int64_t j = 0; j < d; ++j) {\n        float acc = 0.0f;\n        for (int32_t i = 0; i < N; ++i)\n            acc = acc + P"),
    ("error_update_sign", "e_next[j] = v[j] - p[j];", "e_next[j] = p[j] - v[j];"),
    ("local_error_sign", "float local_err = g_i[j] - p_i[j];", "float local_err = p_i[j] - g_i[j];"),
    ("local_error_dropped", "float u = p[j] + local_err;", "float u = p[j];"),
    ("update_associates_the_other_way", "float local_err = g_i[j] - p_i[j];\n        float u = p[j] + local_err;",
     "float local_err = p[j] - p_i[j];\n        float u = local_err + g_i[j];"),
    ("update_rounds_twice", "x_i[j] = fmaf(-lr, u, x_i[j]);", "x_i[j] = x_i[j] - lr * u;"),
    ("sync_update_rounds_twice", "x[(size_t)i * (size_t)d + (size_t)j] = fmaf(-lr, u, x_mean);",
     "x[(size_t)i * (size_t)d + (size_t)j] = x_mean - lr * u;"),
    ("sync_average_rounds_twice", "const float v = fmaf(acc_g, inv_n, e[j]);", "const float v = acc_g * inv_n + e[j];"),
    ("scale_divided_in_fp32", "float scale = (float)(l1 / (double)d);", "float scale = (float)l1 / (float)d;"),
    ("ascent_instead_of_descent", "x_i[j] = fmaf(-lr, u, x_i[j]);", "x_i[j] = fmaf(lr, u, x_i[j]);"),
    ("step_updates_models_with_the_old_error", "liec_oracle_error_update(v, p, d, e);\n        /* worker i",
     "/* worker i"),
    ("workers_all_use_worker_0_message", "liec_oracle_worker_update(g + (size_t)i * (size_t)d, P + (size_t)i * (size_t)d, p, d,",
     "liec_oracle_worker_update(g + (size_t)i * (size_t)d, P, p, d,"),
    ("sync_keeps_the_error", "e[j] = v - p;\n        if (v_out)", "e[j] = v;\n        if (v_out)"),
    ("sync_forgets_to_average_the_models", "const float x_mean = acc_x * inv_n;", "const float x_mean = acc_x;"),
    ("sync_uses_own_model", "x[(size_t)i * (size_t)d + (size_t)j] = fmaf(-lr, u, x_mean);",
     "x[(size_t)i * (size_t)d + (size_t)j] = fmaf(-lr, u, x[(size_t)i * (size_t)d + (size_t)j]);"),
    ("blockwise_scale_uses_the_whole_length", "compress_sign(v + off[b], off[b + 1] - off[b], p ? p + off[b] : NULL, &blk);",
     "compress_sign(v + off[b], off[b + 1] - off[b], p ? p + off[b] : NULL, &blk);\n        blk.scale = (float)(blk.l1 / (double)d);\n        if (p) for (int64_t j = off[b]; j < off[b + 1]; ++j) p[j] = (v[j] < 0.0f) ? -blk.scale : blk.scale;"),
    ("wire_bits_big_endian", "bytes[j / 8] |= (uint8_t)(1u << (j % 8));", "bytes[j / 8] |= (uint8_t)(0x80u >> (j % 8));"),
    ("wire_topk_pairs_unsorted", "free(order);\n    qsort(idx, (size_t)k, sizeof *idx, cmp_u32_asc);\n    for (int64_t r = 0; r < k; ++r)\n        val[r] = v[idx[r]];\n    return 0;\n}\n\n/* Wire form of a random-k",
     "free(order);\n    for (int64_t r = 0; r < k; ++r)\n        val[r] = v[idx[r]];\n    return 0;\n}\n\n/* Wire form of a random-k"),
    ("randk_every_row_draws_the_same_set", "z = mix64(z + (uint64_t)row + gamma);", "z = mix64(z + gamma);"),
    ("randk_every_draw_is_the_same", "z = mix64(z + draw + gamma);", "z = mix64(z + gamma);"),
    ("randk_priority_is_the_index", "uint32_t h = j ^ (uint32_t)(stream & 0xffffffffu);\n    h ^= h >> 16;\n    h *= 0x85EBCA6Bu;",
     "uint32_t h = j ^ (uint32_t)(stream & 0xffffffffu);\n    return h >> 1;\n    h *= 0x85EBCA6Bu;"),
    ("randk_server_draws_with_worker_0_row", "seed, draw, (uint32_t)N, p,", "seed, draw, 0u, p,"),
    ("randk_keeps_the_lowest_priorities", "order[j] = ((uint64_t)liec_oracle_randk_priority(stream, (uint32_t)j) << 32) |\n                   (uint64_t)(0xffffffffu - (uint32_t)j);\n    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);\n    if (p) {",
     "order[j] = ((uint64_t)(0x7fffffffu - liec_oracle_randk_priority(stream, (uint32_t)j)) << 32) |\n                   (uint64_t)(0xffffffffu - (uint32_t)j);\n    qsort(order, (size_t)d, sizeof *order, cmp_u64_desc);\n    if (p) {"),
]


def _within(text, start, end, old, new):
    """Replaces every `old` by `new` between the first `start` and the next `end`."""
    a = text.index(start)
    b = text.index(end, a)
    assert old in text[a:b]
    return text[:a] + text[a:b].replace(old, new) + text[b:]


def _run_pins(src_path, lib_path):
    env = dict(os.environ, LIEC_ORACLE_SRC=src_path, LIEC_ORACLE_LIB=lib_path)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + \
          [os.path.join(ROOT, "tests", f) for f in PIN_FILES]
    return subprocess.run(cmd, capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)


def test_the_unmodified_copy_passes(tmp_path):
    src = tmp_path / "liec_oracle.c"
    src.write_text(open(SRC).read())
    run = _run_pins(str(src), str(tmp_path / "lib.so"))
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, old, new):
    text = open(SRC).read()
    if old is None:
        mutated = new(text)
    else:
        assert text.count(old) >= 1, f"the oracle no longer contains the text this case edits: {old!r}"
        mutated = text.replace(old, new, 1)
    src = tmp_path / "liec_oracle.c"
    src.write_text(mutated)
    run = _run_pins(str(src), str(tmp_path / "lib.so"))
    out = run.stdout + run.stderr
    assert "CalledProcessError" not in out, "the mutated copy must still compile:\n" + out[-1500:]
    assert run.returncode != 0, f"no pin noticed the planted mistake '{name}'"
    assert " failed" in run.stdout, out[-1500:]
