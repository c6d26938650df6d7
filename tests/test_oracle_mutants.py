"""Checks that the oracle's pins have teeth: plant one plausible mistake at a time in a COPY of the oracle's
C source (on the CPU, in a temp dir), point the pin tests at that build, and require that at least one pin
fails.  The real oracle is never modified."""
import os

import pytest

from oracle import lckv_oracle as orc
import test_oracle_pins as pins
import test_oracle_prefill_pins as prefill_pins
import test_oracle_project_pins as project_pins
import test_oracle_footprint_pins as footprint_pins

SRC = os.path.join(os.path.dirname(orc.__file__), "lckv_oracle.c")

MUTANTS = {
    "scale dropped": ("s[j] = scale * dot;", "s[j] = dot;"),
    "exponent sign flipped": ("exp(s[j] - smax)", "exp(smax - s[j])"),
    "max not subtracted": ("exp(s[j] - smax)", "exp(s[j])"),
    "scores taken against V": ("const float *k = K + j * row_stride;", "const float *k = V + j * row_stride;"),
    "values taken from K": ("const float *v = V + j * row_stride;", "const float *v = K + j * row_stride;"),
    "not normalised": ("double p = s[j] / denom;", "double p = s[j];"),
    "self always visible": ("(self_visible[l] ? 1 : 0)", "1"),
    "self never visible": ("(self_visible[l] ? 1 : 0)", "0"),
    "gqa heads interleaved": ("g = h / G;", "g = h % Hkv;"),
    "append one position early": ("b * seq + (int64_t)lens[b] * row;",
                                  "b * seq + (int64_t)(lens[b] > 0 ? lens[b] - 1 : 0) * row;"),
    "append V from k_new": ("memcpy(Vc + dst, v_new + src", "memcpy(Vc + dst, k_new + src"),
    "rule 1 uses last layer": (": top_condensed;", ": L - 1;"),
    "rule 2 uses top condensed": ("(rule == LCKV_ORACLE_PAIR_LAST_LAYER) ? L - 1", "(rule == 7) ? L - 1"),
    "every layer reads slot 0": ("const int s = kv_slot[l];", "const int s = 0;"),
    "lengths not bumped": ("lens[b] += 1;", "lens[b] += 0;"),
    "warmup reads shared slot": ("kv_slot[l] = slot_of_layer[l];",
                                 "kv_slot[l] = slot_of_layer[shared_producer < 0 ? l : shared_producer];"),
    "kv head stride wrong": ("b * seq + (int64_t)g * D;", "b * seq + (int64_t)g;"),
    "window starts one early": ("i < sink ? i : n - window + (i - sink);", "i < sink ? i : n - window - 1 + (i - sink);"),
    "sinks not kept": ("int64_t j = i < sink ? i :", "int64_t j = i < sink ? sink + i :"),
    "sink window policy ignored": ("if (window > 0 && n > sink + window) {", "if (0 && n > sink + window) {"),
    "kept values taken from K": ("memcpy(Vk + i * D, Vc + base", "memcpy(Vk + i * D, Kc + base"),
    "prefill: diagonal not masked": ("int64_t n = i + (self_visible ? 1 : 0);", "int64_t n = i + 1;"),
    "prefill: warmup layer misses itself": ("int64_t n = i + (self_visible ? 1 : 0);", "int64_t n = i;"),
    "prefill: rows past the prompt computed": ("if (i >= lens[b]) {", "if (0) {"),
    "prefill: gqa heads interleaved": ("(int64_t)(h / G) * D;", "(int64_t)(h % Hkv) * D;"),
    "project: weight read transposed": ("(double)W[n * hidden + c];", "(double)W[(int64_t)c * N + n];"),
    "rope: rotates the other way": ("v[i] = lo * c - hi * s;\n                v[i + D / 2] = hi * c + lo * s;",
                                    "v[i] = lo * c + hi * s;\n                v[i + D / 2] = hi * c - lo * s;"),
    "rope: second half keeps the wrong sign": ("v[i + D / 2] = hi * c + lo * s;", "v[i + D / 2] = hi * c - lo * s;"),
    "rope: frequency exponent halved": ("pow(rope_base, -2.0 * i / D)", "pow(rope_base, -1.0 * i / D)"),
    "rope: position off by one": ("(double)pos[b] * pow(", "(double)(pos[b] + 1) * pow("),
    "rope: adjacent channels paired": ("const double lo = v[i], hi = v[i + D / 2];\n                v[i] = lo * c - hi * s;"
                                       "\n                v[i + D / 2] = hi * c + lo * s;",
                                       "const double lo = v[2 * i], hi = v[2 * i + 1];\n"
                                       "                v[2 * i] = lo * c - hi * s;\n"
                                       "                v[2 * i + 1] = hi * c + lo * s;"),
    "footprint: values not counted": ("                   + T * (int64_t)Hkv * D * elem_bytes;  /* and its values    */",
                                      "                   ;"),
    "footprint: every layer keeps a cache": ("for (int s = 0; s < n_slots; ++s)          /* every cache that is kept    */",
                                             "for (int s = 0; s < L; ++s)"),
    "footprint: query heads counted": ("bytes += T * (int64_t)Hkv * D * elem_bytes   /* its keys          */",
                                       "bytes += T * (int64_t)Hkv * 8 * D * elem_bytes"),
    "planner: one sequence too many": ("B + 1, T, Hkv, D, elem_bytes) <= budget)", "B, T, Hkv, D, elem_bytes) <= budget)"),
    "rope: only the first head rotated": ("double *v = y + (int64_t)h * D;", "double *v = y + (int64_t)(h > 0 ? 0 : h) * D;"),
}

PIN_FUNCS = [getattr(mod, n) for mod in (pins, prefill_pins, project_pins, footprint_pins) for n in dir(mod) if n.startswith("test_")]


def _run_all_pins():
    """Run every pin (expanding its parametrisation by hand); return the names of those that fail."""
    failed = []
    for f in PIN_FUNCS:
        marks = [m for m in getattr(f, "pytestmark", []) if m.name == "parametrize"]
        cases = [{}]
        for m in marks:
            names = [s.strip() for s in m.args[0].split(",")]
            new = []
            for c in cases:
                for vals in m.args[1]:
                    vals = vals if len(names) > 1 else (vals,)
                    new.append({**c, **dict(zip(names, vals))})
            cases = new
        for kw in cases:
            try:
                f(**kw)
            except BaseException as e:  # noqa: BLE001 - any failure of a pin counts as "caught"
                if isinstance(e, KeyboardInterrupt):
                    raise
                failed.append(f.__name__)
                break
    return failed


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation site %r must occur exactly once in the oracle" % old
    mutant_c = tmp_path / "mutant.c"
    mutant_c.write_text(src.replace(old, new))
    lib = orc.compile_c(str(mutant_c), str(tmp_path / "libmutant.so"))
    try:
        orc.use_library(lib)
        failed = _run_all_pins()
    finally:
        orc.use_library(None)
    assert failed, "no pin noticed the planted mistake: " + name


def test_unmutated_oracle_passes_the_same_runner():
    orc.use_library(None)
    assert _run_all_pins() == []
