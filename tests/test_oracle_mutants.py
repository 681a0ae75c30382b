"""The pins must notice plausible mistakes: each mutant below plants ONE mistake in a copy of the
oracle's C source (a dropped term, a wrong sign or index, a transposed operand, a wrong tie rule),
builds it, and runs the pin tests against it in a subprocess.  Every mutant has to fail them.
CPU only; nothing here touches the GPU path."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "shadowkv_oracle.c")

MUTANTS = [
    ("rope-sign", "x[i] = x0 * cs - x1 * sn;", "x[i] = x0 * cs + x1 * sn;"),
    ("rope-frequency", "-2.0 * (double)i / (double)p->head_dim", "-1.0 * (double)i / (double)p->head_dim"),
    ("rope-pairing", "double x0 = x[i], x1 = x[i + half];", "double x0 = x[i], x1 = x[(i + 1) % half + half];"),
    ("score-scale-dropped", "P[g * n_c + j] = dot * scale;", "P[g * n_c + j] = dot;"),
    ("logit-rounded-to-fp32", "P[g * n_c + j] = dot * scale;", "P[g * n_c + j] = (double)(float)(dot * scale);"),
    ("group-max-is-min", "if (P[g * n_c + j] > best) best = P[g * n_c + j];",
     "if (best == -INFINITY || P[g * n_c + j] < best) best = P[g * n_c + j];"),
    ("normaliser-dropped", "double lse = mx + log(se);", "double lse = 0.0 * se;"),
    ("head-mapping", "const uint16_t *qg = q + (bi * hq + h * G + g) * d;\n      double mx = -INFINITY;\n      for (int64_t j = 0; j < n_c; ++j) {",
     "const uint16_t *qg = q + (bi * hq + g * hkv + h) * d;\n      double mx = -INFINITY;\n      for (int64_t j = 0; j < n_c; ++j) {"),
    ("mean-not-divided", "C[j * d + x] = acc / (double)c;", "C[j * d + x] = acc;"),
    ("cosine-max-not-min", "if (cs < mn) mn = cs;", "if (mn == INFINITY || cs > mn) mn = cs;"),
    ("b-transposed", "kv_get(p, B, ((u * r) + rho) * d + x)", "kv_get(p, B, ((u * d) + x) * r + rho)"),
    ("position-offset-dropped", "rope_inplace(p, Kt + row * d, pos0 + (double)n);", "rope_inplace(p, Kt + row * d, (double)n);"),
    ("tie-rule-reversed", "return (x->idx > y->idx) - (x->idx < y->idx);", "return (x->idx < y->idx) - (x->idx > y->idx);"),
    ("attention-not-normalised", "double ov = T ? acc / se : 0.0;", "double ov = T ? acc : 0.0 * se;"),
    ("value-of-wrong-token", "Vt[row * d + x] = kv_get(p, value_store, (u * cap + n) * d + x);",
     "Vt[row * d + x] = kv_get(p, value_store, (u * cap + ch * c) * d + x);"),
    ("outlier-order-by-max", "m[j].key = -mn;", "m[j].key = mn;"),
]

# planted mistakes in the chunk-cache model, run against its own pins
CACHE_MUTANTS = [
    ("cache-hit-moves", "if (hit[j]) continue;\n      while (!victim[slot]) ++slot;", "if (hit[j] && j != 0) continue;\n      while (!victim[slot]) ++slot;"),
    ("cache-empty-slot-matches", "if (cache[slot] >= 0 && cache[slot] == sel[j] && !hit[j]) {", "if (cache[slot] == sel[j] - 1 && !hit[j]) {"),
    ("cache-miss-count", "n_miss[u] = m;", "n_miss[u] = k - m;"),
    ("cache-most-recently-used-evicted", "if (best < 0 || a < b) best = slot;", "if (best < 0 || a > b) best = slot;"),
    ("cache-hit-not-stamped", "hit[j] = 1; keep[slot] = 1; ss[j] = slot; stamp[slot] = clock; --n; break;", "hit[j] = 1; keep[slot] = 1; ss[j] = slot; --n; break;"),
    ("cache-empty-not-preferred", "const int32_t a = cache[slot] < 0 ? -1 : stamp[slot];", "const int32_t a = stamp[slot] + (cache[slot] < 0 ? 1000 : 0);"),
    ("cache-wrong-slot-reported", "cache[slot] = sel[j]; stamp[slot] = clock; ss[j] = slot;", "cache[slot] = sel[j]; stamp[slot] = clock; ss[j] = m;"),
]


# planted mistakes in the capacity layout and in the append of generated tokens
APPEND_MUTANTS = [
    ("append-head-order", "k_pre, ((bi * c + t) * hkv + h) * d + x)", "k_pre, ((bi * hkv + h) * c + t) * d + x)"),
    ("append-b-transposed", "kv_get(p, B, (((bi * hkv + h) * r) + rho) * d + x);", "kv_get(p, B, (((bi * hkv + h) * d) + x) * r + rho);"),
    ("append-chunk-id", "landmark_chunk_ids[u * nc_cap + n_c] = (int32_t)n_ch;", "landmark_chunk_ids[u * nc_cap + n_c] = (int32_t)n_c;"),
    ("append-landmark-sum", "(u * nc_cap + n_c) * d + x, acc / (double)c);", "(u * nc_cap + n_c) * d + x, acc);"),
    ("append-row-offset", "kv_put(p, A, (bi * cap + s + t) * r + rho, acc);", "kv_put(p, A, (bi * cap + s) * r + t + rho, acc);"),
    ("append-stride-of-A", "const int64_t Arow = (bi * cap + n) * r;", "const int64_t Arow = (bi * s + n) * r;"),
    ("append-stride-of-landmarks", "const int64_t L0 = u * nc_cap * d;", "const int64_t L0 = u * n_c * d;"),
]


# planted mistakes in the FP8 (E5M2) storage mode
FP8_MUTANTS = [
    ("fp8-exponent-bias", "a = ldexp(1.0 + (double)m / 4.0, e - 15);", "a = ldexp(1.0 + (double)m / 4.0, e - 16);"),
    ("fp8-fraction-width", "a = ldexp(1.0 + (double)m / 4.0, e - 15);", "a = ldexp(1.0 + (double)m / 8.0, e - 15);"),
    ("fp8-subnormal-scale", "a = ldexp((double)m, -16);", "a = ldexp((double)m, -15);"),
    ("fp8-sign-lost", "return sign ? -a : a;", "return a;"),
    ("fp8-ties-away", "const double r = nearbyint(a / ulp) * ulp;", "const double r = floor(a / ulp + 0.5) * ulp;"),
    ("fp8-truncates", "const double r = nearbyint(a / ulp) * ulp;", "const double r = floor(a / ulp) * ulp;"),
    ("fp8-overflow-saturates", "if (r > 57344.0) return sign | 0x7c;", "if (r > 57344.0) return sign | 0x7b;"),
    ("fp8-subnormal-spacing", "if (E < -14) E = -14;", "if (E < -16) E = -16;"),
    ("fp8-landmark-not-rounded-to-fp8", "if (p->kv_dtype == 1) ((uint8_t *)base)[i] = oracle_f64_to_e5m2(x);",
     "if (p->kv_dtype == 1) ((uint8_t *)base)[i] = oracle_f64_to_e5m2((double)(float)x * (1.0 - 1.0 / 16.0));"),
    ("fp8-copy-in-two-byte-units", "static size_t kv_size(const oracle_params *p) { return p->kv_dtype == 1 ? 1 : 2; }",
     "static size_t kv_size(const oracle_params *p) { return p->kv_dtype == 1 ? 2 : 2; }"),
]


def _pins_for(name):
    if name.startswith("fp8-"):
        return "test_oracle_fp8.py"
    if name.startswith("append-"):
        return "test_oracle_append.py"
    return "test_oracle_cache.py" if name.startswith("cache-") else "test_oracle_pins.py"


ALL_MUTANTS = MUTANTS + CACHE_MUTANTS + APPEND_MUTANTS + FP8_MUTANTS


@pytest.mark.parametrize("name,old,new", ALL_MUTANTS, ids=[m[0] for m in ALL_MUTANTS])
def test_pins_catch_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutant {name}: pattern not found in the oracle source"
    mutated = text.replace(old, new, 1)
    c_file = tmp_path / "mutant.c"
    so_file = tmp_path / "libmutant.so"
    c_file.write_text(mutated)
    subprocess.run(["gcc", "-std=c99", "-O1", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so_file), str(c_file),
                    "-lm"], check=True)
    env = dict(os.environ, SHADOWKV_ORACLE_LIB=str(so_file))
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", _pins_for(name)), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True)
    assert res.returncode != 0, f"mutant '{name}' passed every pin:\n{res.stdout[-2000:]}"


def test_unmutated_source_passes_through_the_same_route(tmp_path):
    so_file = tmp_path / "liboracle.so"
    subprocess.run(["gcc", "-std=c99", "-O1", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(so_file), SRC, "-lm"],
                   check=True)
    env = dict(os.environ, SHADOWKV_ORACLE_LIB=str(so_file))
    res = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                          os.path.join(ROOT, "tests", "test_oracle_cache.py"),
                          os.path.join(ROOT, "tests", "test_oracle_append.py"),
                          os.path.join(ROOT, "tests", "test_oracle_fp8.py"), "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
