"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source
(a wrong sign, a swapped comparison, a dropped term, a wrong index), builds it, swaps it in for
the real library and runs the fast pin tests: at least one of them must fail.  CPU only; the
mistakes live in the checker's copy, never in the product."""
import ctypes as C
import itertools
import os
import subprocess

import pytest

import oracle
import test_oracle_dtur as T_dtur
import test_oracle_grad as T_grad
import test_oracle_round as T_round
import test_oracle_select_weights as T_sel

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "dbw_oracle.c")).read()

# pins cheap enough to re-run for every mutant (the full-shape autograd comparisons stay out)
FAST_PINS = {
    "select": [T_sel.test_selection_brute_force, T_sel.test_selection_degenerate, T_sel.test_selection_special_values,
               T_sel.test_round_time_not_longer_than_full, T_sel.test_worked_example, T_sel.test_round_time,
               T_sel.test_round_time_worked_example],
    "weights": [T_sel.test_weight_invariants, T_sel.test_weights_symmetric_mask_doubly_stochastic,
                T_sel.test_weights_closed_forms, T_sel.test_worked_example],
    "round": [T_round.test_b0_is_full_participation, T_round.test_closed_forms_regular_and_complete,
              T_round.test_ring_one_backup_closed_form, T_round.test_mean_recursion_symmetric_mask,
              T_round.test_unrolled_recursion, T_round.test_convexity_and_constants,
              T_round.test_eta_vector_of_equal_entries_is_the_scalar_round,
              T_round.test_eta_single_worker_moves_the_right_rows,
              T_round.test_eta_unrolled_recursion_with_diagonal_rates, T_sel.test_worked_example],
    "dtur": [T_dtur.test_link_set_is_spanning_tree, T_dtur.test_dtur_epochs, T_dtur.test_dtur_dead_worker],
    "grad": [T_grad.test_mlp_finite_differences, T_grad.test_softmax_zero_init_closed_form,
             T_grad.test_mlp_mse_finite_differences, T_grad.test_cnn_finite_differences],
    "branch": [T_grad.test_near_decisions_of_fully_connected_layers, T_grad.test_near_decisions_of_pooling_windows,
               T_grad.test_flipped_relu_decisions_match_autograd, T_grad.test_flipped_pooling_decisions_match_autograd],
}

MUTANTS = [
    # (name, pins, text in the source, replacement)
    ("ties-go-to-the-higher-index", "select", "ta < tb || (ta == tb && a < b)", "ta < tb || (ta == tb && a > b)"),
    ("slowest-instead-of-fastest", "select", "return ta < tb || (ta == tb && a < b);",
     "return ta > tb || (ta == tb && a < b);"),
    ("one-neighbour-too-many", "select", "mask[order[k]] = (uint8_t)(k < pi);", "mask[order[k]] = (uint8_t)(k <= pi);"),
    ("wait-time-ignores-own-time", "select", "float w = canon_time(t[i]);", "float w = 0.0f;"),
    ("metropolis-min-instead-of-max", "weights", "int m = p[i] > p[j] ? p[i] : p[j];", "int m = p[i] < p[j] ? p[i] : p[j];"),
    ("metropolis-without-the-one", "weights", "w_edge[e] = 1.0 / (1.0 + (double)m);", "w_edge[e] = 1.0 / (double)(m > 0 ? m : 1);"),
    ("self-weight-not-the-complement", "weights", "w_self[i] = 1.0 - s;", "w_self[i] = 1.0 / (1.0 + (double)p[i]);"),
    ("gradient-added-not-subtracted", "round", "if (gi) acc -= eta * (double)gi[c];", "if (gi) acc += eta * (double)gi[c];"),
    ("atc-steps-only-the-own-row", "round", "acc += we[e] * ((double)x[o] - (g ? eta * (double)g[o] : 0.0));",
     "acc += we[e] * (double)x[o];"),
    ("eta-of-the-wrong-worker", "round", "acc += we[e] * ((double)x[o] - (double)eta[j] * (double)g[o]);",
     "acc += we[e] * ((double)x[o] - (double)eta[i] * (double)g[o]);"),
    ("threshold-latest-link", "dtur", "if (best < 0 || est < theta) {", "if (best < 0 || est > theta) {"),
    ("link-established-by-the-faster-end", "dtur", "float est = tu > tv ? tu : tv;", "float est = tu < tv ? tu : tv;"),
    ("threshold-strict", "dtur", "if (canon_time(t[colidx[e]]) <= theta) ++cnt;", "if (canon_time(t[colidx[e]]) < theta) ++cnt;"),
    ("relu-derivative-dropped", "grad", "dz[k] = on[l - 1][k] ? da[k] : 0.0;", "dz[k] = da[k];"),
    ("bias-gradient-dropped", "grad", "gb[o] += dz[o];", "gb[o] += 0.0;"),
    ("weight-gradient-transposed-operand", "grad", "da[k] += (double)W[(size_t)o * in + k] * dz[o];",
     "da[k] += (double)W[(size_t)(o * in + k) % ((size_t)out * in)] * dz[(o + 1) % out];"),
    ("conv-data-gradient-dropped", "grad", "if (din) din[ii] += w * go[oh * Wd + ow];", "if (din) din[ii] += 0.0;"),
    ("conv-weight-gradient-shifted", "grad", "gw += go[oh * Wd + ow] * in[ii];", "gw += go[oh * Wd + ow] * in[ii > 0 ? ii - 1 : ii];"),
    ("pooling-passes-gradient-through-inactive-relu", "grad", "if (pass[q]) dz[arg[q]] += dout[q];",
     "dz[arg[q]] += dout[q];"),
    ("conv-bias-gradient-dropped", "grad", "for (int q = 0; q < H * Wd; ++q) gb[co] += go[q];",
     "for (int q = 0; q < H * Wd; ++q) gb[co] += 0.0;"),
    ("mse-gradient-without-the-inner-product", "grad", "dz[c] = 2.0 * p * (e - inner) * scale;", "dz[c] = 2.0 * p * e * scale;"),
    ("softmax-gradient-sign", "grad", "dz[c] = (exp(z[c] - m) / s - (c == y ? 1.0 : 0.0)) * scale;",
     "dz[c] = ((c == y ? 1.0 : 0.0) - exp(z[c] - m) / s) * scale;"),
    ("nan-time-sorts-first", "select", "static float canon_time(float t) { return isnan(t) ? INFINITY : t; }",
     "static float canon_time(float t) { return isnan(t) ? -INFINITY : t; }"),
    ("wait-time-over-all-neighbours", "select",
     "if (k < pi && canon_time(t[colidx[order[k]]]) > w) w = canon_time(t[colidx[order[k]]]);",
     "if (canon_time(t[colidx[order[k]]]) > w) w = canon_time(t[colidx[order[k]]]);"),
    ("round-time-ignores-who-is-waited-for", "select", "if (listed[i] && wait[i] > sel) sel = wait[i];",
     "if (wait[i] > sel) sel = wait[i];"),
    ("round-time-lists-unselected-neighbours", "select", "if (mask[e]) listed[colidx[e]] = 1;",
     "listed[colidx[e]] = 1;"),
    ("weights-use-own-count-only", "weights", "int m = p[i] > p[j] ? p[i] : p[j];", "int m = p[i];"),
    ("average-includes-backup-workers", "round",
     "if (mask[e]) acc += we[e] * (double)x[(size_t)colidx[e] * ld + c];\n                if (gi) acc -= eta * (double)gi[c];",
     "acc += (1.0 / (1.0 + (double)(rowptr[i + 1] - rowptr[i]))) * (double)x[(size_t)colidx[e] * ld + c];\n                if (gi) acc -= eta * (double)gi[c];"),
    ("average-of-own-row-only", "round",
     "if (mask[e]) acc += we[e] * (double)x[(size_t)colidx[e] * ld + c];\n                if (gi) acc -= eta * (double)gi[c];",
     "if (mask[e]) acc += we[e] * (double)xi[c];\n                if (gi) acc -= eta * (double)gi[c];"),
    ("epoch-never-restarts", "dtur", "if (*n_visited >= n_edges) {", "if (*n_visited > n_edges) {"),
    ("threshold-ties-go-to-the-last-link", "dtur", "if (best < 0 || est < theta) {", "if (best < 0 || est <= theta) {"),
    ("slow-workers-wait-for-everybody", "dtur", "            b[j] = deg;\n", "            b[j] = 0;\n"),
    ("visited-links-are-chosen-again", "dtur", "        if (visited[e]) continue;\n", ""),
    # the branch-decision diagnostics (listing of near decisions, evaluation with decisions flipped)
    ("flipped-relu-only-in-the-forward-pass", "branch", "dz[k] = on[l - 1][k] ? da[k] : 0.0;",
     "dz[k] = z[l - 1][k] > 0.0 ? da[k] : 0.0;"),
    ("flipped-relu-sign-reversed", "branch", "if (f) on[l][o] = f->alt != 0;", "if (f) on[l][o] = f->alt == 0;"),
    ("flip-matches-any-sample", "branch",
     "if (br->flips[f].stage == stage && br->flips[f].sample == sample && br->flips[f].unit == unit)",
     "if (br->flips[f].stage == stage && br->flips[f].unit == unit)"),
    ("flipped-window-keeps-its-position", "branch",
     "if (pass[q]) arg[q] = (c * H + 2 * oh + f->alt / 2) * Wd + 2 * ow + f->alt % 2;", ""),
    ("flipped-window-to-none-still-passes", "branch", "pass[q] = f->alt != 4;", "pass[q] = 1;"),
    ("window-position-transposed", "branch",
     "if (pass[q]) arg[q] = (c * H + 2 * oh + f->alt / 2) * Wd + 2 * ow + f->alt % 2;",
     "if (pass[q]) arg[q] = (c * H + 2 * oh + f->alt % 2) * Wd + 2 * ow + f->alt / 2;"),
    ("rounding-unit-without-the-bias", "branch", "double mag = fabs((double)bias[o]);", "double mag = 0.0;"),
    ("rounding-unit-of-signed-products", "branch",
     "o[oh * Wd + ow] += fabs(w * in[((size_t)ci * H + ih) * Wd + iw]);",
     "o[oh * Wd + ow] += w * in[((size_t)ci * H + ih) * Wd + iw];"),
    ("pooling-gap-against-one-unit-only", "branch",
     "note_near(br, stage, sample, q, w, (z[bi] - z[ii]) / (ORC_U * (mag[bi] + mag[ii])));",
     "note_near(br, stage, sample, q, w, (z[bi] - z[ii]) / (ORC_U * mag[bi]));"),
    ("inactive-window-lists-nothing", "branch", "else if (!pass[q])             /* a non-positive value turns positive */",
     "else if (0)"),
    ("near-list-alt-is-the-current-outcome", "branch", "note_near(br, 16 + l, s, o, !on[l][o], fabs(v) / (ORC_U * mag));",
     "note_near(br, 16 + l, s, o, on[l][o], fabs(v) / (ORC_U * mag));"),
]


def _expand(fn):
    """Calls of a pin test function with every combination of its parametrize marks."""
    marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
    names = [m.args[0] for m in marks]
    for combo in itertools.product(*[m.args[1] for m in marks]):
        yield lambda combo=combo: fn(oracle, **dict(zip(names, combo)))


def _run_pins(group):
    failures = 0
    for fn in FAST_PINS[group]:
        for call in _expand(fn):
            try:
                call()
            except Exception:        # an assertion of the pin, or the mutant breaking an invariant on the way
                failures += 1
    return failures


@pytest.fixture
def swapped_library():
    real = oracle.lib()
    yield
    oracle._lib = real


def test_pins_pass_on_the_real_oracle():
    for group in FAST_PINS:
        assert _run_pins(group) == 0, group


@pytest.mark.parametrize("name,group,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_a_planted_mistake(tmp_path, swapped_library, name, group, old, new):
    assert SRC.count(old) == 1, f"mutation site not unique or missing: {old!r}"
    src = tmp_path / "mutant.c"
    src.write_text(SRC.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(src), "-lm"])
    mutant = C.CDLL(str(so))
    mutant.orc_select.restype = C.c_int
    mutant.orc_spanning_tree.restype = C.c_int
    oracle._lib = mutant
    assert _run_pins(group) > 0, f"no pin noticed the mistake '{name}'"
