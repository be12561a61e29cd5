"""The pins must be sharp: plausible mistakes planted in a copy of the oracle's C source
(on the CPU, never in the HIP path) each have to fail at least one pin."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "cmn_oracle.c")

# (name, text to find, replacement) — each changes the arithmetic in a way a slip could
MUTANTS = [
    ("fold_descending_ranks", "int r = (s + j) % K;", "int r = ((s - j) % K + K) % K;"),
    ("fold_ignores_rotation", "int s = ring_rotate ? c % K : 0;", "int s = 0;"),
    ("fold_starts_one_late", "int s = ring_rotate ? c % K : 0;", "int s = ring_rotate ? (c + 1) % K : 0;"),
    ("fold_drops_last_replica", "for (int j = 1; j < K; ++j) {\n                int r", "for (int j = 1; j < K - 1; ++j) {\n                int r"),
    ("ring_sends_wrong_chunk", "int c = (((r + phase - s) % K) + K) % K;\n                memcpy",
     "int c = (((r + phase + s) % K) + K) % K;\n                memcpy"),
    ("ring_gather_adds", "own[i] = (phase == 0) ? recv[i] + own[i] : recv[i];", "own[i] = recv[i] + own[i];"),
    ("scale_divides_by_k_minus_1", "float s = 1.0f / (float)K;", "float s = 1.0f / (float)(K > 1 ? K - 1 : 1);"),
    ("pack_leaves_padding", "memset(dst + o * eb, 0, (size_t)((L - o) * eb));", "(void)L;"),
    ("pack_swaps_order", "memcpy(dst + o * eb, tensors[t], (size_t)(numel[t] * eb));",
     "memcpy(dst + o * eb, tensors[T - 1 - t], (size_t)(numel[t] * eb));"),
    ("chunk_not_aligned", "int64_t ce = ((per + A - 1) / A) * A;", "int64_t ce = per;"),
    ("chunk_floor_division", "int64_t per = (off[T] + C - 1) / C;", "int64_t per = off[T] / C;"),
    ("sgd_plus_sign", "float vn = t1 - t2;", "float vn = t1 + t2;"),
    ("sgd_uses_new_velocity_twice", "p[i] = p[i] + vn;", "p[i] = p[i] + vn + vn;"),
    ("sgd_momentum_on_gradient", "float t1 = mu * v[i];", "float t1 = mu * gi;"),
    ("sgd_decay_after_lr", "float d = wd * p[i];", "float d = wd * lr * p[i];"),
    ("sgd_decay_uses_velocity", "float d = wd * p[i];", "float d = wd * v[i];"),
    ("half_wrong_bias", "((exp5 + 112u) << 23)", "((exp5 + 111u) << 23)"),
    ("half_subnormal_scale", "(float)man10 * 0x1p-24f", "(float)man10 * 0x1p-25f"),
    ("half_drops_sign_of_subnormal", "bits |= sign << 31;", "(void)sign;"),
    ("half_mantissa_shift", "| (man10 << 13); /* rebias", "| (man10 << 12); /* rebias"),
    ("encode_truncates", "if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;", "(void)rem;"),
    ("encode_ties_away", "(rem == 0x1000u && (h & 1u))) ++h;", "(rem == 0x1000u)) ++h;"),
    ("encode_subnormal_truncates", "if (rem > half || (rem == half && (q & 1u))) ++q;", "(void)rem; (void)half;"),
    ("encode_flushes_subnormals", "if (e < -10) return sign;", "if (e <= 0) return sign;"),
    ("encode_saturates_instead_of_inf", "if (e >= 31) return (uint16_t)(sign | 0x7c00u);", "if (e >= 31) return (uint16_t)(sign | 0x7bffu);"),
    ("bf16_decode_shift", "uint32_t bits = (uint32_t)b << 16;", "uint32_t bits = (uint32_t)b << 15;"),
    ("bf16_encode_truncates", "if (rem > 0x8000u || (rem == 0x8000u && (kept & 1u))) ++kept;", "(void)rem;"),
    ("bf16_encode_ties_away", "(rem == 0x8000u && (kept & 1u))) ++kept;", "(rem == 0x8000u)) ++kept;"),
    ("bf16_nan_becomes_inf", "return (uint16_t)((x >> 16) | 0x0040u);", "return (uint16_t)(x >> 16);"),
    ("int8_scale_of_wrong_chunk", "load_grad(packed[r], dtype, i, scales ? scales[r][c] : 1.0f)", "load_grad(packed[r], dtype, i, scales ? scales[r][0] : 1.0f)"),
    ("int8_scale_of_wrong_replica", "load_grad(packed[r], dtype, i, scales ? scales[r][c] : 1.0f)", "load_grad(packed[r], dtype, i, scales ? scales[s][c] : 1.0f)"),
    ("int8_read_as_unsigned", "float q = (float)((const int8_t *)base)[i];", "float q = (float)((const uint8_t *)base)[i];"),
    ("adam_first_moment_no_decay", "float mn = m[i] + t2;", "float mn = m[i] + t1;"),
    ("adam_second_moment_uses_g", "float t3 = gi * gi;", "float t3 = gi;"),
    ("adam_eps_inside_sqrt", "float s = sqrtf(vn);\n        float den = s + eps;", "float s = sqrtf(vn + eps);\n        float den = s;"),
    ("adam_ascends", "p[i] = p[i] - u;", "p[i] = p[i] + u;"),
    ("adam_uses_old_moment", "float q = mn / den;", "float q = m[i] / den;"),
    ("adam_lr_without_second_correction", "return (float)((double)alpha * sqrt(b2) / b1);", "return (float)((double)alpha / b1);"),
    ("adam_lr_corrections_swapped", "return (float)((double)alpha * sqrt(b2) / b1);", "return (float)((double)alpha * sqrt(b1) / b2);"),
    ("adam_decay_dropped", "gi = gi + dec;", "(void)dec;"),
]


def test_every_mutant_text_is_present_once():
    text = open(SRC).read()
    for name, old, _ in MUTANTS:
        assert text.count(old) == 1, name


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_kill_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    src = tmp_path / "mut.c"
    lib = tmp_path / "libmut.so"
    src.write_text(text.replace(old, new))
    subprocess.run(["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
                    "-fPIC", str(src), "-o", str(lib), "-lm"], check=True)
    env = dict(os.environ, CMN_ORACLE_LIB_FOR_MUTATION_TEST=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, env=env,
                       capture_output=True, text=True)
    assert r.returncode != 0, f"mutant {name} survived every pin:\n{r.stdout[-2000:]}"
    assert re.search(r"\d+ failed", r.stdout), r.stdout[-2000:]
