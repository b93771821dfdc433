"""Do the pins bite?  Each case below plants one plausible mistake in a COPY of the oracle's C source (a dropped
term, a wrong sign, a swapped index, a wrong range), compiles the copy for the CPU and runs the pins against it: at
least one of the pins named for the case must fail.  The oracle itself is never touched, and nothing here runs on
the GPU.
"""
import importlib.util
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")


def _pins(name):
    spec = importlib.util.spec_from_file_location(f"pins_{name}", os.path.join(HERE, f"{name}.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


eps_pins = _pins("test_oracle_eps")
pins = _pins("test_oracle_pins")
sampler_pins = _pins("test_oracle_sampler")
sketch_pins = _pins("test_oracle_sketch")


def _load_mutant(tmp_path, name, old, new):
    src = open(os.path.join(ORACLE_DIR, "pamm_oracle.c")).read()
    assert src.count(old) == 1, f"mutant {name}: the text to replace must occur exactly once ({src.count(old)})"
    csrc = tmp_path / f"oracle_{name}.c"
    lib = tmp_path / f"liboracle_{name}.so"
    csrc.write_text(src.replace(old, new))
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", str(lib), str(csrc), "-lm"], check=True)
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{name}", os.path.join(ORACLE_DIR, "pamm_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    sys.modules[spec.name] = mod                        # dataclasses look their module up by name
    spec.loader.exec_module(mod)
    mod._SRC, mod._LIB, mod._lib = str(csrc), str(lib), None
    mod.build = lambda force=False: str(lib)            # the mutant library is already built
    return mod


def _fails(fn, *args):
    try:
        fn(*args)
    except AssertionError:
        return True
    except Exception:           # a mutant may also break an invariant so badly that numpy or the wrapper raises
        return True
    return False


MUTANTS = [
    # name, text in pamm_oracle.c, replacement, pins of which at least one must fail
    ("signed_cosine", "double s = (cn2[j] > 0.0) ? (d * d) / cn2[j] : 0.0;     /* ||A_i||^2 csim^2 */",
     "double s = (cn2[j] > 0.0) ? (d * fabs(d)) / cn2[j] : 0.0;",
     [lambda o: pins.test_antiparallel_row_picks_largest_absolute_cosine(o)]),
    ("score_not_normalised", "double s = (cn2[j] > 0.0) ? (d * d) / cn2[j] : 0.0;     /* ||A_i||^2 csim^2 */",
     "double s = d * d;",
     [lambda o: pins.test_assignment_is_brute_force_argmin_of_residual(o, 0), lambda o: pins.test_scale_invariance(o)]),
    ("alpha_without_norm", "double a = (cn2[j1] > 0.0) ? d1 / cn2[j1] : 0.0;           /* Eq. 1 */",
     "double a = d1;",
     [lambda o: pins.test_projection_geometry(o), lambda o: pins.test_generators_represent_themselves(o)]),
    ("alpha_divided_by_norm_not_squared", "double a = (cn2[j1] > 0.0) ? d1 / cn2[j1] : 0.0;           /* Eq. 1 */",
     "double a = (cn2[j1] > 0.0) ? d1 / sqrt(cn2[j1]) : 0.0;",
     [lambda o: pins.test_projection_geometry(o), lambda o: pins.test_generators_represent_themselves(o)]),
    ("highest_j_wins_ties", "if (s > s1) {                   /* strict: lowest j keeps a tie */",
     "if (s >= s1) {",
     [lambda o: pins.test_duplicates_ties_and_zero_rows(o)]),
    ("btilde_without_alpha", "dst[c] += a * decode(B, dtype, (size_t)i * (size_t)m + (size_t)c);",
     "dst[c] += decode(B, dtype, (size_t)i * (size_t)m + (size_t)c);",
     [lambda o: pins.test_regrouping_identity(o, 0), lambda o: pins.test_single_generator_closed_form(o)]),
    ("btilde_wrong_row", "double *dst = Btilde + (int64_t)f[i] * m;",
     "double *dst = Btilde + (int64_t)(k - 1 - f[i]) * m;",
     [lambda o: pins.test_regrouping_identity(o, 0), lambda o: pins.test_all_rows_as_generators_gives_exact_product(o)]),
    ("product_with_transposed_c", "double cjl = C[j * n + l];",
     "double cjl = C[(j * n + l) % (k * n) == j * n + l ? ((l % k) * n + (j % n)) : 0];",
     [lambda o: pins.test_all_rows_as_generators_gives_exact_product(o), lambda o: pins.test_regrouping_identity(o, 0)]),
    ("sampler_draws_from_whole_range", "int64_t r = t + (int64_t)bounded(&st, (uint64_t)(b - t));",
     "int64_t r = (int64_t)bounded(&st, (uint64_t)b);",
     [lambda o: sampler_pins.test_matches_the_written_specification(o, 8192, 16, 0), lambda o: sampler_pins.test_every_ordered_draw_equally_likely(o)]),
    ("bounded_draw_without_rejection", "} while (x < reject_below);", "} while (0);",
     [lambda o: sampler_pins.test_bounded_draw_on_the_published_stream(o, 3 << 62),
      lambda o: sampler_pins.test_bounded_draw_is_uniform_where_a_plain_remainder_is_not(o)]),
    ("bounded_draw_rejects_the_wrong_end", "} while (x < reject_below);", "} while (x > 0ULL - reject_below - 1ULL);",
     [lambda o: sampler_pins.test_bounded_draw_on_the_published_stream(o, 3 << 62)]),
    ("bounded_draw_threshold_not_reduced", "uint64_t reject_below = (0ULL - u) % u;", "uint64_t reject_below = (0ULL - u);",
     [lambda o: sampler_pins.test_bounded_draw_on_the_published_stream(o, (1 << 62) + 1)]),
    ("sampler_forgets_the_exchange", "a[r] = tmp;", "a[r] = a[r];",
     [lambda o: sampler_pins.test_full_draw_is_a_permutation(o, 64), lambda o: sampler_pins.test_distinct_in_range_deterministic_prefix(o, 100, 17)]),
    ("bf16_decoded_from_low_half", "uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;",
     "uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]);",
     [lambda o: pins.test_element_types_decode_exactly(o)]),
    ("absolute_tolerance", "if (eps >= 0.0 && e > eps * na) {",
     "if (eps >= 0.0 && e > eps) {",
     [lambda o: eps_pins.test_kept_rows_are_those_of_the_neighbourhood_condition(o, 0.2)]),
    ("residual_of_the_wrong_generator", "const double *c = C + j1 * n;",
     "const double *c = C + ((j1 + 1) % k) * n;",
     [lambda o: eps_pins.test_kept_rows_are_those_of_the_neighbourhood_condition(o, 0.2)]),
    ("beta_inverted", "return (eta < b) ? (double)b / (double)(b - eta) : 0.0;",
     "return (eta < b && eta > 0) ? (double)b / (double)eta : 1.0;",
     [lambda o: eps_pins.test_beta_makes_column_row_sampling_unbiased(o), lambda o: eps_pins.test_zero_tolerance_is_uniform_column_row_sampling(o)]),
    ("beta_not_applied", "for (int64_t c = 0; c < m; ++c) out[c] *= beta;", ";",
     [lambda o: eps_pins.test_beta_makes_column_row_sampling_unbiased(o)]),
    ("sketch_with_transposed_projection", "d += decode(A, dtype, (size_t)i * (size_t)n + (size_t)l) * decode(Pt, pdtype, (size_t)j * (size_t)n + (size_t)l);",
     "d += decode(A, dtype, (size_t)i * (size_t)n + (size_t)l) * decode(Pt, pdtype, (size_t)((j * n + l) % r) * (size_t)n + (size_t)((j * n + l) / r % n));",
     [lambda o: sketch_pins.test_orthogonal_projection_gives_the_exact_product(o), lambda o: sketch_pins.test_coordinate_selection(o)]),
    ("sketch_grad_takes_the_wrong_sketch_column", "double s = decode(S, sdtype, (size_t)i * (size_t)r + (size_t)j);",
     "double s = decode(S, sdtype, (size_t)i * (size_t)r + (size_t)(r - 1 - j));",
     [lambda o: sketch_pins.test_coordinate_selection(o), lambda o: sketch_pins.test_orthogonal_projection_gives_the_exact_product(o)]),
    ("sketch_grad_last_product_transposed", "double p = decode(Pt, pdtype, (size_t)j * (size_t)n + (size_t)l);     /* P[l][j] */",
     "double p = decode(Pt, pdtype, (size_t)((l * r + j) / n % r) * (size_t)n + (size_t)((l * r + j) % n));",
     [lambda o: sketch_pins.test_orthogonal_projection_gives_the_exact_product(o), lambda o: sketch_pins.test_coordinate_selection(o)]),
    ("sketch_grad_drops_the_sketch", "g[c] += s * decode(B, dtype, (size_t)i * (size_t)m + (size_t)c);",
     "g[c] += decode(B, dtype, (size_t)i * (size_t)m + (size_t)c);",
     [lambda o: sketch_pins.test_rank_one_closed_form(o), lambda o: sketch_pins.test_identity_projection_keeps_everything(o)]),
]


@pytest.mark.parametrize("name,old,new,checks", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(tmp_path, name, old, new, checks):
    mutant = _load_mutant(tmp_path, name, old, new)
    assert any(_fails(check, mutant) for check in checks), f"no pin noticed the mistake '{name}'"


def test_the_unmodified_copy_passes_the_same_pins(tmp_path):
    """The harness itself: a copy with no mistake in it passes every pin the cases above rely on."""
    clean = _load_mutant(tmp_path, "clean", "#include <math.h>", "#include <math.h>\n")
    for _, _, _, checks in MUTANTS:
        for check in checks:
            check(clean)
