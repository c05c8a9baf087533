"""Mutation audit of the oracle's pins (CPU only).

Each case plants one plausible mistake in a copy of oracle/mt_oracle.c (a dropped term, a wrong sign or index, a
transposed operand, a swapped argument), builds it, and runs tests/test_oracle_pins.py against that library in a
child process: the pins must fail.  A mistake that survives means the pins do not fix that part of the oracle.
The product library is not involved."""
import concurrent.futures as cf
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mt_oracle.c")

# (name, text in the source, replacement); the text must occur exactly once
MUTANTS = [
    ("linear_drops_bias", "if (b) acc += (double)b[n];", ""),
    ("linear_reads_weight_transposed", "acc += (double)xr[k] * (double)wr[k];", "acc += (double)xr[k] * (double)W[k * N + n];"),
    ("layernorm_unbiased_variance", "var /= (double)H;", "var /= (double)(H - 1);"),
    ("layernorm_drops_beta", " + (double)beta[i]);", ");"),
    ("layernorm_drops_gamma", "(double)gamma[i] * ((v - mean) * inv)", "((v - mean) * inv)"),
    ("first_layernorm_drops_residual", "orc_layernorm(X, ao, M, H, L.ln1_g", "orc_layernorm(ao, NULL, M, H, L.ln1_g"),
    ("second_layernorm_takes_layer_input_as_residual", "orc_layernorm(x1, fo, M, H, L.ln2_g", "orc_layernorm(X, fo, M, H, L.ln2_g"),
    ("gelu_argument_unscaled", "erf(v * 0.7071067811865476)", "erf(v)"),
    ("gelu_forms_swapped", "if (tanh_form) {", "if (!tanh_form) {"),
    ("mask_sign", "sc += -10000.0f;", "sc += 10000.0f;"),
    ("mask_on_queries", "if (!mask[b * S + j]) sc", "if (!mask[b * S + i]) sc"),
    ("score_scale_one_over_d", "1.0f / sqrtf((float)d)", "1.0f / (float)d"),
    ("score_scale_missing", "float sc = (float)acc * scale;", "float sc = (float)acc;"),
    ("values_of_head_zero", "(double)v[(b * S + j) * H + a * d + c]", "(double)v[(b * S + j) * H + c]"),
    ("softmax_not_normalised", "p[j] = (float)(exp((double)(s[j] - mx)) / sum);", "p[j] = (float)(exp((double)(s[j] - mx)));"),
    ("position_off_by_one", "(double)pos[s * H + i]", "(double)pos[(s + 1) * H + i]"),
    ("type_embedding_missing", "+ (double)type[(int64_t)(type_ids ? type_ids[b * S + s] : 0) * H + i]);", ");"),
    ("default_segment_is_one", "type_ids[b * S + s] : 0)", "type_ids[b * S + s] : 1)"),
    ("keys_and_values_swapped", "orc_attention(q, k, v, mask", "orc_attention(q, v, k, mask"),
    ("queries_and_keys_swapped", "orc_attention(q, k, v, mask", "orc_attention(k, q, v, mask"),
    ("pooler_reads_last_token", "memcpy(first + b * H, Z + b * S * H,", "memcpy(first + b * H, Z + (b * S + S - 1) * H,"),
    ("pooler_without_tanh", "pool[i] = (float)tanh((double)pool[i]);", "pool[i] = pool[i];"),
    ("every_task_forks_at_the_top", "taps + (int64_t)tasks[t].fork_layer * MH;", "taps + (int64_t)D * MH;"),
    ("task_layers_in_reverse_order", "task_params[t] + l * lsz, z, mask", "task_params[t] + (tasks[t].n_layers - 1 - l) * lsz, z, mask"),
    ("student_runs_the_whole_trunk", "for (int l = 0; l < task->fork_layer; ++l)", "for (int l = 0; l < c->n_trunk_layers; ++l)"),
    ("token_head_drops_bias", "orc_linear(Z, M, H, Wc, bc, n_classes, lg);", "orc_linear(Z, M, H, Wc, NULL, n_classes, lg);"),
    ("token_head_shifted_by_a_position", "logits[r * ld_logits + j] = lg[r * n_classes + j];",
     "logits[r * ld_logits + j] = lg[((r + 1) % M) * n_classes + j];"),
    ("overhead_sums_the_forks", "if (tasks[t].fork_layer > shared) shared = tasks[t].fork_layer;", "shared += tasks[t].fork_layer;"),
    ("feed_forward_without_activation", "orc_gelu_array(u, M * F, c->gelu_tanh, u);", ""),
    ("output_projection_bias_missing", "orc_linear(ctx, M, H, L.Wo, L.bo, H, ao);", "orc_linear(ctx, M, H, L.Wo, NULL, H, ao);"),
]


def _run_pins(lib):
    env = dict(os.environ, ORC_LIB=lib, OMP_NUM_THREADS="2", PYTHONPATH=ROOT)
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, timeout=600)
    return r.returncode, r.stdout.decode(errors="replace")


def _build(src_text, path):
    c = path + ".c"
    open(c, "w").write(src_text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", path, c, "-lm"], check=True)
    return path


def test_unaltered_copy_passes_and_every_planted_mistake_is_caught(tmp_path):
    src = open(SRC).read()
    libs = {}
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, f"{name}: the text to alter occurs {src.count(old)} times in mt_oracle.c"
        libs[name] = _build(src.replace(old, new), str(tmp_path / f"liborc_{name}.so"))
    libs["(unaltered)"] = _build(src, str(tmp_path / "liborc_same.so"))
    with cf.ThreadPoolExecutor(max_workers=4) as pool:
        results = dict(zip(libs, pool.map(_run_pins, libs.values())))
    rc, out = results.pop("(unaltered)")
    assert rc == 0, "the pins fail on an unaltered copy built the same way:\n" + out[-2000:]
    survivors = [name for name, (rc, _) in results.items() if rc == 0]
    assert not survivors, f"planted mistakes the pins do not catch: {survivors}"
    for name, (rc, out) in results.items():          # a mutant must fail an assertion, not crash the interpreter
        assert rc == 1, f"{name}: pytest exit status {rc}\n{out[-1500:]}"
