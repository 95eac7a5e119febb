"""The pins must be able to fail: each plausible mistake below is planted in a copy of the C oracle
(on the CPU, in a temporary directory), and the pin suite is run against that broken build.  Every
mutant has to be caught by at least one pin."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "roast_oracle.c")

MUTANTS = {
    "in_tile_stride_uses_Z1": ("*idx = base + (int64_t)Z2 * o1 + o2;", "*idx = base + (int64_t)Z1 * o1 + o2;"),
    "tile_coordinates_swapped": ("layer, (uint64_t)c1, (uint64_t)c2, m_size", "layer, (uint64_t)c2, (uint64_t)c1, m_size"),
    "sign_dropped_from_hash": ("*sgn = 1 - 2 * (int32_t)(v & 1u);", "*sgn = 1;"),
    "sign_dropped_from_gradient": ("dM[idx] += lambda * (double)s * dW[i * O + j];", "dM[idx] += lambda * dW[i * O + j];"),
    "lambda_dropped_from_gradient": ("dM[idx] += lambda * (double)s * dW[i * O + j];", "dM[idx] += (double)s * dW[i * O + j];"),
    "lambda_dropped_from_w": ("W[i * O + j] = lambda * v;", "W[i * O + j] = v;"),
    "range_excludes_last_offset": ("(uint64_t)(m_size - len) / h->align + 1;", "(uint64_t)(m_size - len) / h->align + (m_size > len ? 0 : 1);"),
    "dx_uses_untransposed_w": ("for (int64_t o = 0; o < O; ++o) acc += g[o] * w[o];", "for (int64_t o = 0; o < O; ++o) acc += g[o] * W[(o % H) * O + (k % O)];"),
    "dw_contracts_wrong_index": ("double x = X[i * H + k];\n      const double* g = dY + i * O;", "double x = X[i * H + (H - 1 - k)];\n      const double* g = dY + i * O;"),
    "lookup_uses_chunk_number_as_offset": ("(double)M[base + i % Z];", "(double)M[base + (i / Z) % Z];"),
    "lookup_gradient_missing_sign": ("dM[base + i % Z] += lambda * (double)g * dOut[n * D + i];", "dM[base + i % Z] += lambda * dOut[n * D + i];"),
    "element_sign_keyed_by_the_block": ("*sgn *= oracle_elem_sign(h, layer, (uint64_t)i, (uint64_t)j);", "*sgn *= oracle_elem_sign(h, layer, (uint64_t)c1, (uint64_t)c2);"),
    "bf16_ties_round_up": ("(rest == 0x8000u && (keep & 1u))", "(rest == 0x8000u)"),
    "offset_hash_ignores_second_key": ("uint64_t t1 = (c1 * (k1 % P)) % P;", "uint64_t t1 = 0; (void)c1; (void)k1;"),
    "product_not_reduced_before_sum": ("uint64_t t2 = (c2 * (k2 % P)) % P;", "uint64_t t2 = (c2 * k2);"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name, tmp_path):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for {name} not found exactly once"
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    lib = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib), str(src), "-lm"],
                   check=True)
    env = dict(os.environ, ROAST_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        os.path.join(ROOT, "tests", "test_sign_variant_pins.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 1, f"mutant {name} survived the pins:\n{r.stdout[-2000:]}"
    assert "failed" in r.stdout
