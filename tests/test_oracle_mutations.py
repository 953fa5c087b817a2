"""The pins must be able to fail: plant one mistake at a time in a copy of the
oracle's C source (on the CPU, in a temporary directory), rebuild it, and check
that at least one pin test rejects the mutant."""
import importlib.util
import inspect
import os
import shutil
import subprocess

import pytest

from tests import test_oracle_pins as pins

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")

MUTATIONS = [
    ("hash: golden-ratio increment dropped", "uint64_t z = x + UINT64_C(0x9E3779B97F4A7C15);", "uint64_t z = x;"),
    ("hash: first shift", "(z >> 30)", "(z >> 31)"),
    ("hash: second multiplier", "0x94D049BB133111EB", "0x94D049BB133111ED"),
    ("hash: last shift", "return z ^ (z >> 31);", "return z ^ (z >> 30);"),
    ("hash: salt added instead of xored", "raw[i] ^ salt", "raw[i] + salt"),
    ("offsets: 32-bit wrap", "offsets[i + 1] = offsets[i] + len;", "offsets[i + 1] = (int32_t)(offsets[i] + len);"),
    ("offsets: inclusive instead of exclusive", "offsets[0] = 0;\n    for", "offsets[0] = lengths[0];\n    for"),
    ("forward: sign", "acc[d] += w;", "acc[d] -= w;"),
    ("forward: mean not divided", "v /= (double)len;", ";"),
    ("forward: element order reversed", "((const float *)table)[row * D + d]", "((const float *)table)[row * D + (D - 1 - d)]"),
    ("forward: wrong bag end", "int64_t s = offsets[bag], e = offsets[bag + 1];\n            for (int32_t d = 0; d < D; ++d) acc",
     "int64_t s = offsets[bag], e = offsets[bag + 1] - (offsets[bag + 1] > offsets[bag]);\n            for (int32_t d = 0; d < D; ++d) acc"),
    ("forward: out-of-range row read", "if (r < 0 || r >= num_rows[t]) {\n                    if (status) *status |= ORACLE_STATUS_BAD_INDEX;\n                    continue;\n                }\n                for (int32_t d = 0; d < D; ++d) {\n                    double w",
     "if (r < 0 || r > num_rows[t]) {\n                    if (status) *status |= ORACLE_STATUS_BAD_INDEX;\n                    continue;\n                }\n                for (int32_t d = 0; d < D; ++d) {\n                    double w"),
    ("bf16 widen shift", "(uint32_t)b << 16", "(uint32_t)b << 15"),
    ("bf16 rounding half-up", "u += 0x7FFFu + ((u >> 16) & 1u);", "u += 0x8000u;"),
    ("bf16 truncation", "u += 0x7FFFu + ((u >> 16) & 1u);", ""),
    ("backward: mean scale dropped", "if (mode == ORACLE_POOL_MEAN) g /= (double)len;", ""),
    ("backward: accumulator uses sum not mean over D", "sq / (double)D", "sq"),
    ("backward: eps inside the root", "sqrt(s_new) + (double)eps", "sqrt(s_new + (double)eps)"),
    ("backward: old accumulator dropped", "(double)accum[t][r] + sq", "sq"),
    ("backward: accumulator used before update", "double denom = sqrt(s_new)", "double denom = sqrt((double)accum[t][r])"),
    ("backward: step sign", "w - (double)lr * G[d] / denom", "w + (double)lr * G[d] / denom"),
    ("backward: table base missing from key", "lk[n].key = rowbase + r;", "lk[n].key = r;"),
    ("backward: gradient column", "(double)dout[bag * D + d]", "(double)dout[bag * D]"),
    ("backward: gradient of wrong bag", "lk[n].bag = bag;", "lk[n].bag = bag > 0 ? bag - 1 : bag;"),
    ("backward: per-occurrence update", "for (; i < n && lk[i].key == key; ++i) {", "for (int once = 1; once && i < n; ++i, once = 0) {"),
    ("backward: accumulator not stored", "accum[t][r] = (float)s_new;", ""),
    ("quant: 16 levels for INT4", "dtype == ORACLE_INT8 ? 255.0f : 15.0f", "dtype == ORACLE_INT8 ? 255.0f : 16.0f"),
    ("quant: truncation instead of rounding", "rintf((x[d] - bias) / scale)", "floorf((x[d] - bias) / scale)"),
    ("quant: rounding half up", "rintf((x[d] - bias) / scale)", "floorf((x[d] - bias) / scale + 0.5f)"),
    ("quant: nibble order on store", "(code << (4 * (d % 2)))", "(code << (4 * (1 - d % 2)))"),
    ("quant: nibble order on load", ">> (4 * (d % 2))) & 15u", ">> (4 * (1 - d % 2))) & 15u"),
    ("quant: bias not subtracted", "(x[d] - bias) / scale", "x[d] / scale"),
    ("quant: bias is the maximum", "float bias = lo;", "float bias = hi;"),
    ("quant: scale and bias swapped on load", "memcpy(&scale, p, 4);\n    memcpy(&bias, p + 4, 4);",
     "memcpy(&bias, p, 4);\n    memcpy(&scale, p + 4, 4);"),
    ("quant: bias dropped on load", "(double)scale * (double)code + (double)bias", "(double)scale * (double)code"),
    ("quant: row stride unpadded", "return (8 + code_bytes + 15) / 16 * 16;", "return 8 + code_bytes;"),
    ("quant: INT8 codes read as nibbles", "dtype == ORACLE_INT8 ? p[8 + d] :", "dtype != ORACLE_INT8 ? p[8 + d] :"),
    ("cached: hits and misses swapped", "hit_miss[hit ? 0 : 1] += 1;", "hit_miss[hit ? 1 : 0] += 1;"),
    ("checksum: weights start at zero", "sum += (uint64_t)w * (i + 1);", "sum += (uint64_t)w * i;"),
    ("checksum: unweighted", "sum += (uint64_t)w * (i + 1);", "sum += (uint64_t)w;"),
    ("checksum: 32-bit product", "sum += (uint64_t)w * (i + 1);", "sum += (uint64_t)(uint32_t)(w * (uint32_t)(i + 1));"),
    ("checksum: big-endian words", "(uint32_t)p[4 * i] | ((uint32_t)p[4 * i + 1] << 8) | ((uint32_t)p[4 * i + 2] << 16) |\n                     ((uint32_t)p[4 * i + 3] << 24)",
     "(uint32_t)p[4 * i + 3] | ((uint32_t)p[4 * i + 2] << 8) | ((uint32_t)p[4 * i + 1] << 16) |\n                     ((uint32_t)p[4 * i] << 24)"),
    ("policy: counter incremented by two", "freq[r] += 1u;", "freq[r] += 2u;"),
    ("policy: out-of-range entries not counted", "++bad;\n            continue;", "continue;"),
    ("policy: smaller counters preferred", "if (fa != fb) return fa > fb ? -1 : 1;", "if (fa != fb) return fa > fb ? 1 : -1;"),
    ("policy: ties go to the larger row", "return (ra > rb) - (ra < rb);", "return (ra < rb) - (ra > rb);"),
    ("policy: ties broken arbitrarily", "return (ra > rb) - (ra < rb);", "return ((ra ^ 5) > (rb ^ 5)) - ((ra ^ 5) < (rb ^ 5));"),
    ("policy: hot set left in preference order", "qsort(hot_rows_out, (size_t)num_hot, sizeof(int64_t), cmp_i64);", ""),
    ("policy: aging dropped", "freq[r] >>= decay_shift;", ""),
    ("policy: counters aged before the selection", "qsort(order, (size_t)num_rows, sizeof(int64_t), cmp_preference);",
     "for (int64_t r = 0; r < num_rows; ++r) freq[r] >>= decay_shift;\n    qsort(order, (size_t)num_rows, sizeof(int64_t), cmp_preference);"),
    ("policy: counters saturate at 2^31", "freq[r] += 1u;", "if (freq[r] < 0x80000000u) freq[r] += 1u;"),
]


def _pin_calls():
    """Every pin test with every combination of its parametrize marks, as (name, fn, kwargs)."""
    import itertools
    calls = []
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        axes = []
        for mark in getattr(fn, "pytestmark", []):
            if mark.name != "parametrize":
                continue
            names = [n.strip() for n in mark.args[0].split(",")]
            values = [v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,) for v in mark.args[1]]
            axes.append([dict(zip(names, v)) for v in values])
        for combo in itertools.product(*axes):
            kw = {}
            for part in combo:
                kw.update(part)
            calls.append((name, fn, kw))
    return calls


def _load_variant(lib_path, tag):
    spec = importlib.util.spec_from_file_location("emb_oracle_mut_" + tag,
                                                  os.path.join(ORACLE_DIR, "emb_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.build = lambda force=False: lib_path
    return mod


def _killed_by(mod):
    for name, fn, kw in _pin_calls():
        try:
            fn(mod, **kw)
        except AssertionError:
            return name
    return None


def test_unmutated_copy_passes_every_pin(tmp_path):
    shutil.copy(os.path.join(ORACLE_DIR, "emb_oracle.h"), tmp_path)
    shutil.copy(os.path.join(ORACLE_DIR, "emb_oracle.c"), tmp_path)
    lib = str(tmp_path / "lib0.so")
    subprocess.check_call(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-o", lib,
                           str(tmp_path / "emb_oracle.c"), "-lm"])
    assert _killed_by(_load_variant(lib, "clean")) is None


@pytest.mark.parametrize("idx", range(len(MUTATIONS)), ids=[m[0] for m in MUTATIONS])
def test_every_planted_mistake_is_caught(tmp_path, idx):
    what, old, new = MUTATIONS[idx]
    src = open(os.path.join(ORACLE_DIR, "emb_oracle.c")).read()
    assert src.count(old) >= 1, "mutation site not found: " + what
    shutil.copy(os.path.join(ORACLE_DIR, "emb_oracle.h"), tmp_path)
    (tmp_path / "emb_oracle.c").write_text(src.replace(old, new, 1))
    lib = str(tmp_path / ("lib%d.so" % idx))
    subprocess.check_call(["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-w", "-o", lib,
                           str(tmp_path / "emb_oracle.c"), "-lm"])
    assert _killed_by(_load_variant(lib, str(idx))) is not None, "no pin catches: " + what
