"""Do the pins pin? Each case plants one plausible mistake in a COPY of the oracle's source
(a dropped term, a wrong sign or index, a swapped operand, a wrong reading of the algorithm),
builds it on the CPU and runs the oracle's pin tests against the broken build: one must fail.
A mutant that survives means a pin is missing.

The planted mistakes live only in the temporary copy; the HIP path is not involved.
"""
import importlib.util
import os
import subprocess

import pytest

import test_oracle_pins
import test_oracle_pins_extensions

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "gaf_oracle.c")
PIN_MODULES = [test_oracle_pins, test_oracle_pins_extensions]

# (name, text in the oracle, what replaces it). Each text occurs exactly once.
MUTANTS = [
    # Eq. 4
    ("similarity_not_distance", "return 1.0 - xy / (sqrt(xx) * sqrt(yy));", "return xy / (sqrt(xx) * sqrt(yy));"),
    ("distance_sign", "return 1.0 - xy / (sqrt(xx) * sqrt(yy));", "return 1.0 + xy / (sqrt(xx) * sqrt(yy));"),
    ("no_square_roots", "return 1.0 - xy / (sqrt(xx) * sqrt(yy));", "return 1.0 - xy / (xx * yy);"),
    ("one_square_root", "return 1.0 - xy / (sqrt(xx) * sqrt(yy));", "return 1.0 - xy / (sqrt(xx) * yy);"),
    ("zero_norm_gives_zero", "        return 1.0;\n    return 1.0 - xy", "        return 0.0;\n    return 1.0 - xy"),
    ("zero_norm_needs_both", "    if (xx == 0.0 || yy == 0.0)", "    if (xx == 0.0 && yy == 0.0)"),
    ("pair_distance_wrong_norm", "        yy += b * b;\n    }\n    return oracle_distance_from_sums(xy, xx, yy);",
     "        yy += a * b;\n    }\n    return oracle_distance_from_sums(xy, xx, yy);"),
    # Algorithm 1
    ("strict_threshold", "    if (D <= tau) {", "    if (D < tau) {"),
    ("nan_distance_accepted", "    if (D <= tau) {", "    if (!(D > tau)) {"),
    ("inverted_threshold", "    if (D <= tau) {", "    if (D >= tau) {"),
    ("accepted_not_added", "            g[p] += widen(g_i, p, dtype);", "            g[p] += 0.0;"),
    ("running_mean_of_two", "            g[p] += widen(g_i, p, dtype);", "            g[p] = 0.5 * (g[p] + widen(g_i, p, dtype));"),
    ("count_not_incremented", "        *c += 1;\n        *accepted = 1;", "        *accepted = 1;"),
    ("rejected_still_counted", "    } else {\n        *accepted = 0;", "    } else {\n        *c += 1;\n        *accepted = 0;"),
    ("step_norm_of_candidate_dropped", "        gigi += b * b;", "        gigi += a * b;"),
    ("step_norm_of_sum_swapped", "        gg += a * a;", "        gg += b * b;"),
    ("distance_against_candidate_only", "        gig += b * a;", "        gig += b * b;"),
    ("seed_distance_not_zero", "        *dist = 0.0;\n        *accepted = 1;\n        return 0;",
     "        *dist = 1.0;\n        *accepted = 1;\n        return 0;"),
    ("visits_in_reverse_order", "oracle_gaf_step(out, &c, grads[i], P,", "oracle_gaf_step(out, &c, grads[i == 0 ? 0 : N - i], P,"),
    ("seed_is_last_gradient", "oracle_gaf_step(out, &c, grads[i], P,", "oracle_gaf_step(out, &c, grads[N - 1 - i], P,"),
    # Eq. 5 / Eq. 2
    ("normalised_by_N", "        out[p] = out[p] / (double)c;", "        out[p] = out[p] / (double)N;"),
    ("not_normalised", "        out[p] = out[p] / (double)c;", "        out[p] = out[p];"),
    ("plain_average_wrong_divisor", "        out[p] = s / (double)N;", "        out[p] = s / (double)(N - 1);"),
    ("plain_average_skips_first", "        for (int i = 0; i < N; ++i)\n            s += widen(grads[i], p, dtype);",
     "        for (int i = 1; i < N; ++i)\n            s += widen(grads[i], p, dtype);"),
    # input widening
    ("bf16_shift", "<< 16;", "<< 15;"),
    # all pairs
    ("pairwise_not_mirrored", "            gram[(size_t)j * N + i] = s;", "            gram[(size_t)j * N + i] = -s;"),
    ("pairwise_diagonal", "= (i == j) ? 0.0", "= (i == j) ? 1.0"),
    ("pairwise_transposed_norm", "gram[(size_t)i * N + j], gram[(size_t)i * N + i],\n                                            gram[(size_t)j * N + j]);",
     "gram[(size_t)i * N + j], gram[(size_t)i * N + i],\n                                            gram[(size_t)i * N + i]);"),
    # order-indifferent seed
    ("best_seed_tie_to_highest", "        if (c > best_c) {", "        if (c >= best_c) {"),
    ("best_seed_last_never_tried", "    for (int s = 0; s < N && !rc; ++s) {", "    for (int s = 0; s < N - 1 && !rc; ++s) {"),
    ("best_seed_reverse_ring", "            ring[k] = grads[(s + k) % N];", "            ring[k] = grads[(s + N - k) % N];"),
    ("best_seed_mask_not_rotated", "                mask[(s + k) % N] = m[k];", "                mask[k] = m[k];"),
    ("best_seed_dist_not_rotated", "                dist[(s + k) % N] = d[k];", "                dist[k] = d[k];"),
    # GAF-SGD
    ("sgd_no_skip", "    if (c <= 1)\n        return 0;", "    if (c < 1)\n        return 0;"),
    ("sgd_no_weight_decay", "        double d = g_gaf[p] + wd * theta[p];", "        double d = g_gaf[p];"),
    ("sgd_decay_sign", "        double d = g_gaf[p] + wd * theta[p];", "        double d = g_gaf[p] - wd * theta[p];"),
    ("sgd_no_momentum", "        v[p] = mu * v[p] + d;", "        v[p] = d;"),
    ("sgd_dampened", "        v[p] = mu * v[p] + d;", "        v[p] = mu * v[p] + (1.0 - mu) * d;"),
    ("sgd_steps_with_gradient", "        theta[p] = theta[p] - lr * v[p];", "        theta[p] = theta[p] - lr * d;"),
    ("sgd_nesterov", "        theta[p] = theta[p] - lr * v[p];", "        theta[p] = theta[p] - lr * (d + mu * v[p]);"),
    ("sgd_ascent", "        theta[p] = theta[p] - lr * v[p];", "        theta[p] = theta[p] + lr * v[p];"),
    # bucketed
    ("bucket_mask_row", "                                  mask + (size_t)b * N, dist + (size_t)b * N, &count[b]);",
     "                                  mask + (size_t)b * N, dist + (size_t)b * N, &count[0]);"),
    ("bucket_slice_start", "            sl[i] = (const char *)grads[i] + off[b] * es;", "            sl[i] = (const char *)grads[i];"),
]


def test_every_mutant_text_occurs_once():
    src = open(SRC).read()
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, name
        assert old != new, name
    assert len({m[0] for m in MUTANTS}) == len(MUTANTS)


def _pin_cases():
    """Every pin test as (name, function, extra keyword arguments), parametrized ones expanded."""
    cases = []
    for mod in PIN_MODULES:
        for name, fn in sorted(vars(mod).items()):
            if not name.startswith("test_") or not callable(fn):
                continue
            grids = [{}]
            for mark in getattr(fn, "pytestmark", []):
                if mark.name != "parametrize":
                    continue
                names = [n.strip() for n in mark.args[0].split(",")]
                grids = [dict(g, **dict(zip(names, v if len(names) > 1 else (v,))))
                         for g in grids for v in mark.args[1]]
            cases += [(name, fn, g) for g in grids]
    return cases


def _failing_pin(so_path, tag):
    """Runs the pins against the build at so_path (through a private copy of the oracle's
    ctypes front end); returns the name of the first pin that fails, or None."""
    spec = importlib.util.spec_from_file_location("gaf_oracle_" + tag, os.path.join(ROOT, "oracle", "gaf_oracle.py"))
    front = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(front)
    front._OVERRIDE = so_path
    for name, fn, kw in _pin_cases():
        try:
            fn(front, **kw)
        except Exception:      # an assertion, or arithmetic that the broken values derail
            return name
    return None


def _compile(text, tmp_path, name):
    c = tmp_path / (name + ".c")
    so = tmp_path / (name + ".so")
    c.write_text(text)
    subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
                    "-o", str(so), str(c), "-lm"], check=True)
    return str(so)


def test_unmodified_copy_passes(tmp_path):
    """The harness itself: the same pins, run the same way on an untouched copy, pass."""
    assert len(_pin_cases()) >= 24
    assert _failing_pin(_compile(open(SRC).read(), tmp_path, "intact"), "intact") is None


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch(tmp_path, name, old, new):
    so = _compile(open(SRC).read().replace(old, new), tmp_path, name)
    assert _failing_pin(so, name) is not None, "no pin notices the planted mistake '%s'" % name
