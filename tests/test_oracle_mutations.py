"""The pins must catch plausible mistakes. Each case plants ONE mistake in a copy of the oracle's
source (on the CPU, never in the GPU path), builds it, and runs the pin tests against that build
in a child process: at least one pin has to fail. An unmutated copy has to pass."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "qsdp_ref.c")

# (name, text to replace, replacement, pin files expected to notice)
MUTANTS = [
    ("coin_flip_rounds_up_for_small_uniforms", "code[i] = (uint8_t)((ti + h) >> 16);",
     "code[i] = (uint8_t)((ti + 65535u - h) >> 16);", ["test_oracle_grad.py"]),
    ("coin_flip_ignores_the_uniform", "code[i] = (uint8_t)((ti + h) >> 16);", "code[i] = (uint8_t)((ti + 32768u) >> 16);",
     ["test_oracle_grad.py"]),
    ("fraction_truncated_to_16_bits", "float t16 = fmaf(d, inv16, 0.5f);", "float t16 = d * inv16;", ["test_oracle_grad.py"]),
    ("position_clamp_one_cell_short", "uint32_t top16 = (uint32_t)((1 << bits) - 1) << 16;",
     "uint32_t top16 = (uint32_t)((1 << bits) - 2) << 16;", ["test_oracle_grad.py"]),
    ("levels_off_by_one", "float Lf = (float)((1 << bits) - 1);\n    float lo, hi, scale, inv;\n    bucket_stats(g,",
     "float Lf = (float)(1 << bits);\n    float lo, hi, scale, inv;\n    bucket_stats(g,", ["test_oracle_grad.py"]),
    ("uniform_high_half_first", "(j % 2u) ? (w >> 16) : (w & 0xFFFFu)", "(j % 2u) ? (w & 0xFFFFu) : (w >> 16)",
     ["test_oracle_rng.py"]),
    ("philox_multipliers_swapped", "(uint64_t)0xD2511F53u * (uint64_t)c0", "(uint64_t)0xCD9E8D57u * (uint64_t)c0",
     ["test_oracle_rng.py"]),
    ("philox_nine_rounds", "round < 10", "round < 9", ["test_oracle_rng.py"]),
    ("shift_sign_flipped", "float k = rintf(t - xi);", "float k = rintf(t + xi);", ["test_oracle_weight.py"]),
    ("shift_missing_from_base", "*base_out = fmaf(xi, scale, lo);", "*base_out = lo;", ["test_oracle_weight.py"]),
    ("lattice_shift_missing_from_base", "*base_out = (k0 + xi) * delta;", "*base_out = k0 * delta;",
     ["test_oracle_weight.py"]),
    ("lattice_saturation_not_counted", "*sat += 1u;", "", ["test_oracle_weight.py"]),
    ("weight_shift_from_gradient_stream", "uint32_t ctr[4] = {0u, 0u, 1u, 0u};", "uint32_t ctr[4] = {0u, 0u, 0u, 0u};",
     ["test_oracle_rng.py"]),
    ("pack_bits_reversed", "words[p / 32] |= (uint32_t)1u << (p % 32);", "words[p / 32] |= (uint32_t)1u << (31 - p % 32);",
     ["test_oracle_codec.py"]),
    ("bf16_truncates", "bitsv += 0x7FFFu + ((bitsv >> 16) & 1u);", "", ["test_oracle_codec.py"]),
    ("f16_ties_round_up", "if (rem > half || (rem == half && (q & 1u))) q += 1u;", "if (rem >= half) q += 1u;",
     ["test_oracle_codec.py"]),
    ("f16_subnormals_flushed", "int drop = he >= 1 ? 13 : 13 + (1 - he);", "if (he < 1) return (uint16_t)sign;\n    int drop = 13;",
     ["test_oracle_codec.py"]),
    ("f16_overflow_saturates", "if (h >= 0x7C00u) h = 0x7C00u;", "if (h >= 0x7C00u) h = 0x7BFFu;", ["test_oracle_codec.py"]),
    ("f16_output_written_as_bf16", "return out_dtype == QSDP_REF_F16 ? qsdp_ref_f32_to_f16(v) : qsdp_ref_f32_to_bf16(v);",
     "return qsdp_ref_f32_to_bf16(v);", ["test_oracle_codec.py"]),
    ("decode_not_fused", "out[i] = fmaf((float)code[i], scale, base);", "out[i] = (float)code[i] * scale + base;",
     ["test_oracle_codec.py"]),
    ("peer_sum_keeps_last_only", "sum[i] = (p == 0) ? val[i] : sum[i] + val[i];", "sum[i] = val[i];",
     ["test_oracle_dequantize_add.py"]),
    ("peer_sum_not_scaled", "out[s + (uint64_t)i] = alpha * sum[i];", "out[s + (uint64_t)i] = sum[i];",
     ["test_oracle_dequantize_add.py"]),
    ("symmetric_grid_uses_max_only", "float a = fmaxf(fabsf(lo), fabsf(hi));", "float a = fabsf(hi);",
     ["test_oracle_variants.py"]),
    ("grad_shift_reuses_weight_stream", "uint32_t ctr[4] = {0u, 0u, 2u, 0u};", "uint32_t ctr[4] = {0u, 0u, 1u, 0u};",
     ["test_oracle_variants.py"]),
    ("no_shift_flag_ignored_for_weights", "return (flags & QSDP_REF_FLAG_NO_SHIFT) ? 0.0f : qsdp_ref_weight_shift(seed);",
     "return qsdp_ref_weight_shift(seed);", ["test_oracle_variants.py"]),
    ("closest_level_takes_last_minimum", "if (d < best_d) {", "if (d <= best_d) {", ["test_oracle_levels.py"]),
    ("level_update_moves_away", "levels[k] = (float)(q - (1.0 - keep[count[k]]) * (q - mean));",
     "levels[k] = (float)(q + (1.0 - keep[count[k]]) * (q - mean));", ["test_oracle_levels.py"]),
    ("level_update_single_step", "levels[k] = (float)(q - (1.0 - keep[count[k]]) * (q - mean));",
     "levels[k] = (float)(q - (1.0 - keep[1]) * (q - mean));", ["test_oracle_levels.py"]),
    ("sequential_fit_moves_away", "q[best] = q[best] - (double)lr * (q[best] - zi);",
     "q[best] = q[best] + (double)lr * (q[best] - zi);", ["test_oracle_levels.py"]),
    ("sequential_fit_searches_the_start_table", "double d = fabs(zi - q[k]);", "double d = fabs(zi - (double)levels[k]);",
     ["test_oracle_levels.py"]),
    ("sequential_fit_jumps_onto_the_value", "q[best] = q[best] - (double)lr * (q[best] - zi);", "q[best] = zi;",
     ["test_oracle_levels.py"]),
    ("level_decode_ignores_table", "float val = fmaf(levels[code[i]], meta[2 * j + 1], meta[2 * j]);",
     "float val = fmaf((float)code[i], meta[2 * j + 1], meta[2 * j]);", ["test_oracle_levels.py"]),
    ("adamw_second_moment_not_squared", "float vi = fmaf(beta2, *var, (omb2 * ghat) * ghat);",
     "float vi = fmaf(beta2, *var, omb2 * ghat);", ["test_oracle_adamw.py"]),
    ("adamw_bias_corrections_swapped", "float upd = (mi / bias1) / (sqrtf(vi / bias2) + eps);",
     "float upd = (mi / bias2) / (sqrtf(vi / bias1) + eps);", ["test_oracle_adamw.py"]),
    ("adamw_decay_dropped", "return fmaf(-lr, fmaf(weight_decay, x, upd), x);", "return fmaf(-lr, upd, x);",
     ["test_oracle_adamw.py"]),
    ("recv_adamw_uses_unscaled_sum", "bucket, alpha, y); /* y holds ghat for now */",
     "bucket, 1.0f, y); /* y holds ghat for now */", ["test_oracle_recv_adamw.py"]),
    ("recv_adamw_moments_swapped", "y[i] = adamw_element(x[i], y[i], &mom[i], &var[i], lr,",
     "y[i] = adamw_element(x[i], y[i], &var[i], &mom[i], lr,", ["test_oracle_recv_adamw.py"]),
    ("step_sign_flipped", "y[i] = fmaf(-lr, ghat[i], x[s + (uint64_t)i]);", "y[i] = fmaf(lr, ghat[i], x[s + (uint64_t)i]);",
     ["test_oracle_fused.py"]),
    ("step_skips_weight_quantizer", "dequant_bucket(wcode, m, wbase, wscale, x + s);",
     "for (int i = 0; i < m; ++i) x[s + (uint64_t)i] = y[i];", ["test_oracle_fused.py"]),
    ("keep_master_still_quantizes", "for (int i = 0; i < m; ++i) x[s + (uint64_t)i] = y[i]; /* the partition stays unquantized */\n        } else {\n            dequant_bucket(wcode, m, wbase, wscale, x + s);\n        }\n        if (wcodes) {\n            pack_bucket(wcode, m, wbits, bucket, wcodes + (uint64_t)j * (uint64_t)wpb);\n            wmeta[2 * j] = wbase;\n            wmeta[2 * j + 1] = wscale;\n        }\n        sat += local;\n    }\n    if (n_saturated) *n_saturated += sat;\n    return QSDP_REF_OK;\n}\n\nint qsdp_ref_fused_step_codes(",
     "dequant_bucket(wcode, m, wbase, wscale, x + s);\n        } else {\n            dequant_bucket(wcode, m, wbase, wscale, x + s);\n        }\n        if (wcodes) {\n            pack_bucket(wcode, m, wbits, bucket, wcodes + (uint64_t)j * (uint64_t)wpb);\n            wmeta[2 * j] = wbase;\n            wmeta[2 * j + 1] = wscale;\n        }\n        sat += local;\n    }\n    if (n_saturated) *n_saturated += sat;\n    return QSDP_REF_OK;\n}\n\nint qsdp_ref_fused_step_codes(",
     ["test_oracle_keep_master.py"]),
    ("keep_master_recv_copies_old_weights", "memcpy(x, ghat, (size_t)n * sizeof(float)); /* x <- y: the partition stays unquantized */",
     "(void)0;", ["test_oracle_keep_master.py"]),
    ("level_coin_flip_inverted", "return i + ((1.0f - 0x1p-17f) - u < p ? 1 : 0);", "return i + ((1.0f - 0x1p-17f) - u < p ? 0 : 1);",
     ["test_oracle_levels_stochastic.py"]),
    ("level_coin_flip_rounds_up_for_small_uniforms", "return i + ((1.0f - 0x1p-17f) - u < p ? 1 : 0);",
     "return i + (u + 0x1p-17f < p ? 1 : 0);", ["test_oracle_levels_stochastic.py"]),
    ("level_coin_flip_uses_distance_to_upper", "float p = (z - levels[i]) * r;", "float p = (levels[i + 1] - z) * r;",
     ["test_oracle_levels_stochastic.py"]),
    ("level_upper_neighbour_skipped", "float gap = levels[i + 1] - levels[i]; /* > 0 by the choice of i */",
     "float gap = levels[K - 1] - levels[i];", ["test_oracle_levels_stochastic.py"]),
    ("recv_step_sign_flipped", "ghat[i] = fmaf(-lr, ghat[i], x[i]); /* y, in place */",
     "ghat[i] = fmaf(lr, ghat[i], x[i]); /* y, in place */", ["test_oracle_recv_step.py"]),
    ("recv_step_average_dropped", "npeers, n, gbits,\n                                     bucket, alpha, ghat);",
     "npeers, n, gbits,\n                                     bucket, 1.0f, ghat);", ["test_oracle_recv_step.py"]),
    ("recv_step_skips_weight_quantizer",
     "        else\n            rc = qsdp_ref_dequantize(codes, meta, n, wbits, bucket, QSDP_REF_F32, x);",
     "        else\n            memcpy(x, ghat, (size_t)n * sizeof(float));", ["test_oracle_recv_step.py"]),
]


def _build(tmp_path, name, text):
    src = tmp_path / f"{name}.c"
    src.write_text(text)
    lib = tmp_path / f"lib{name}.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
                    "-shared", "-I", os.path.join(ROOT, "oracle"), str(src), "-o", str(lib), "-lm"], check=True)
    return str(lib)


def _pins_pass(lib, files):
    env = dict(os.environ, QSDP_REF_LIB=lib)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + [
        os.path.join(ROOT, "tests", f) for f in files]
    return subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True).returncode == 0


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    """Every mutant (and the unmutated copy) built and judged once, a few at a time: name -> the pins passed.
    A mutant whose mutation site is missing maps to None."""
    from concurrent.futures import ThreadPoolExecutor
    text = open(SRC).read()
    root = tmp_path_factory.mktemp("mutants")

    def judge(case):
        name, old, new, files = case
        if old is not None and text.count(old) < 1:
            return name, None
        work = root / name
        work.mkdir()
        lib = _build(work, name, text if old is None else text.replace(old, new, 1))
        return name, _pins_pass(lib, files)

    cases = [("plain", None, None, ["test_oracle_rng.py", "test_oracle_codec.py"])] + MUTANTS
    workers = max(1, min(4, (os.cpu_count() or 2) // 2))
    with ThreadPoolExecutor(max_workers=workers) as pool:
        return dict(pool.map(judge, cases))


def test_unmutated_copy_passes(verdicts):
    assert verdicts["plain"] is True


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(verdicts, name):
    assert verdicts[name] is not None, "mutation site not found: the oracle changed, update this test"
    assert verdicts[name] is False, f"no pin noticed the planted mistake '{name}'"
