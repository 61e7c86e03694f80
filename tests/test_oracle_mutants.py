"""The pins must be able to fail: plausible mistakes planted in a copy of the oracle (on the CPU) have to be
caught by at least one of them.  Each mutant is the oracle's own source with one line changed."""
import importlib.util
import os
import sys
import types

import pytest

import test_oracle_pins as pins

ORACLE_SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "spcfg_oracle.py")

MUTANTS = {
    "right projection of leaves uses L": ("b1 = _log_project(R_P, e)", "b1 = _log_project(L_P, e)"),
    "right projection of spans uses L": ("bw = _log_project(R_N, ow)", "bw = _log_project(L_N, ow)"),
    "last split point dropped": ("terms = np.stack([a[(i, k)] + b[(k, j)] for k in range(i + 1, j)])",
                                 "terms = np.stack([a[(i, k)] + b[(k, j)] for k in range(i + 1, max(i + 2, j - 1))])"),
    "shift not added back in the projection": ("return x + np.log(np.exp(o - x) @ W.T)",
                                               "return np.log(np.exp(o - x) @ W.T)"),
    "transposed projection operand": ("a1 = _log_project(L_P, e)", "a1 = _log_project(L_P[:, ::-1], e)"),
    "grad_R accumulates the left adjoint": ("gR[:, :N] += _outer_sum(lbs, ow)", "gR[:, :N] += _outer_sum(las, ow)"),
    "right child gets no adjoint": ("                lb[(k, j)] = np.logaddexp(lb[(k, j)], lo[(i, j)] + a[(i, k)])\n",
                                    "                pass\n"),
    "root posterior not accumulated": ("    g_root += obar[(0, n)]\n", "    pass\n"),
    "emission gradient misses the right-child term": (
        "g_emit[:] = np.exp(np.logaddexp(_log_adjoint_project(L_P, las), _log_adjoint_project(R_P, lbs)) + e)",
        "g_emit[:] = np.exp(_log_adjoint_project(L_P, las) + e)"),
    "span adjoint misses the R term": (
        "low = np.logaddexp(_log_adjoint_project(L_N, las), _log_adjoint_project(R_N, lbs))",
        "low = _log_adjoint_project(L_N, las)"),
    # the log-space chain rule d logZ / d a = eta * d logZ / d eta vanishes where eta = 0: a reverse pass that
    # divides it by eta afterwards (and takes 0 / 0 = 0) loses the derivative at a parent's dead column block
    "adjoint of eta carried as eta times itself (0 where eta = 0)": (
        "                la[(i, k)] = np.logaddexp(la[(i, k)], lo[(i, j)] + b[(k, j)])\n",
        "                la[(i, k)] = np.logaddexp(la[(i, k)], lo[(i, j)] + b[(k, j)] + np.where(np.isfinite(a[(i, k)]), 0.0, _NEG_INF))\n"),
    "outer product shifted by one maximum only": ("return (np.exp(la - x) * np.exp(x + y)).T @ np.exp(lo - y)",
                                                   "return (np.exp(la - x) * np.exp(x)).T @ np.exp(lo - y)"),
    "adjoint projection multiplies with the transpose": ("return x + np.log(np.exp(la - x) @ W)",
                                                         "return x + np.log(np.exp(la - x) @ W.T[:, :W.shape[1]])"),
    "root weights ignored": ("logZ = _logsumexp0((log_root + o[(0, n)])[:, None])[0]",
                             "logZ = _logsumexp0((o[(0, n)])[:, None])[0]"),
}

PIN_CALLS = [
    lambda: pins.test_logZ_matches_tree_enumeration(2, 3, 3),
    lambda: pins.test_logZ_matches_tree_enumeration(3, 2, 4),
    lambda: pins.test_logZ_matches_dense_rule_tensor_inside(5, 7, 7, 0),
    lambda: pins.test_closed_form_two_words(),
    lambda: pins.test_closed_form_uniform_grammar_counts_trees(5),
    lambda: pins.test_right_branching_grammar_is_a_linear_chain(False),
    lambda: pins.test_symmetries_and_homogeneity(),
    lambda: pins.test_gradients_are_expected_counts_from_enumeration(2, 3, 4),
    lambda: pins.test_gradients_match_central_finite_differences(),
    lambda: pins.test_gradient_invariants(),
    lambda: pins.test_derivative_at_dead_rule_blocks("L", "pre"),
    lambda: pins.test_derivative_at_dead_rule_blocks("R", "non"),
]


def load_mutant(old, new):
    src = open(ORACLE_SRC).read()
    assert src.count(old) == 1, f"mutation site not found exactly once: {old!r}"
    mod = types.ModuleType("oracle_mutant")
    exec(compile(src.replace(old, new), "oracle_mutant.py", "exec"), mod.__dict__)
    return mod


def test_unmutated_copy_passes_every_pin(monkeypatch):
    monkeypatch.setattr(pins, "O", load_mutant("_NEG_INF = -np.inf", "_NEG_INF = -np.inf"))
    for call in PIN_CALLS:
        call()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, monkeypatch):
    old, new = MUTANTS[name]
    monkeypatch.setattr(pins, "O", load_mutant(old, new))
    caught = 0
    for call in PIN_CALLS:
        try:
            call()
        except Exception:  # an assertion or a numerical failure: the pin noticed
            caught += 1
    assert caught >= 1, f"no pin noticed the planted mistake: {name}"
