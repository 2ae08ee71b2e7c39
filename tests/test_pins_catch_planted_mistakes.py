"""Do the pins bite?  Each case below plants ONE plausible mistake in a copy of an
oracle function (a dropped term, a wrong sign or index, a transposed operand, a
missing normalisation), installs the broken copy in place of the original, and
re-runs the pins of tests/test_oracle_pins.py that cover that function.  At
least one of them must fail.  Everything here runs on the CPU; the mistakes are
planted in the oracle only, never in the HIP path.

A mutant is a textual edit of the function's own source, so a case whose
`old` text no longer occurs in the oracle fails loudly instead of silently
testing nothing.
"""
import importlib
import inspect
import textwrap

import pytest

import oracle
from tests import test_oracle_pins as pins

# pins grouped by the oracle function they constrain; the 4096 x 4096 dense eigendecomposition is left out of
# the mutant runs (it takes several seconds per run and the Householder route covers the same ground)
LANCZOS_PINS = [
    pins.test_start_vector_is_normalised, pins.test_breakdown_at_exhausted_krylov_space,
    pins.test_planted_spectrum_top_values, pins.test_planted_spectrum_bottom_values,
    pins.test_tridiagonal_matches_householder_reduction, pins.test_ritz_pairs_match_householder_route,
    pins.test_lanczos_invariants, pins.test_full_spectrum_of_small_diagonal_operator,
]
SHARDED_PINS = [pins.test_row_sharded_algorithm_reproduces_single_device]
STEP_PINS = [
    pins.test_step_closed_form_on_coordinate_subspace, pins.test_step_without_subspace_is_library_sgd_momentum,
    pins.test_step_orthogonality_and_zero_momentum, pins.test_step_solves_quadratic_in_subspace_in_one_step,
    pins.test_step_with_zero_dual_equals_plain_step, pins.test_step_with_dual_closed_form_and_g1_readings,
    pins.test_step_abs_mode_with_dual_and_negative_curvature,
]
ADAMW_PINS = [pins.test_adamw_step_without_subspace_is_library_adamw, pins.test_adamw_step_structure,
              pins.test_adamw_step_dense_closed_form]
ADMM_PINS = [pins.test_admm_outer_rules]
HVP_PINS = [pins.test_hvp_planted_matches_dense_matrix, pins.test_hvp_planted_eigenvectors,
            pins.test_ggn_equals_autograd_hessian_product, pins.test_ggn_dense_kronecker_sum,
            pins.test_ggn_null_space_and_zero_weights]

# (module, function, text in the function's source, replacement, pins that must notice)
MUTANTS = [
    # ---- Algorithm 1
    ("oracle.lanczos", "_run", "Q[:, 0] = keep(v1 / np.sqrt(sqnorm(v1)))", "Q[:, 0] = keep(v1)", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "band[0, i] += along_current", "band[0, i] += float(h @ h)", LANCZOS_PINS),
    ("oracle.lanczos", "_remove_components", "coeff[-1]", "coeff[max(len(coeff) - 2, 0)]", LANCZOS_PINS),   # previous column's
    ("oracle.lanczos", "_run", "Q[:, : i + 1], h, inner", "Q[:, i: i + 1], h, inner", LANCZOS_PINS),      # only the current column
    ("oracle.lanczos", "_run", "Q[:, : i + 1], h, inner", "Q[:, : max(i, 1)], h, inner", LANCZOS_PINS),   # current column left out
    ("oracle.lanczos", "_remove_components", "h - filled @ coeff", "h + filled @ coeff", LANCZOS_PINS),
    ("oracle.lanczos", "_remove_components", "coeff = inner(filled, h)", "coeff = inner(filled, filled[:, -1])", LANCZOS_PINS),
    ("oracle.lanczos", "_remove_components", "h - filled @ coeff", "h - filled @ coeff[::-1]", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "band[1, i] = np.sqrt(sqnorm(h))", "band[1, i] = sqnorm(h)", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "Q[:, i + 1] = keep(h / band[1, i])", "Q[:, i + 1] = keep(h)", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "Q[:, i + 1] = keep(h / band[1, i])", "Q[:, i + 1] = keep(h / band[0, i])", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "if not band[1, i] > breakdown_tol * hnorm[i]:", "if not band[1, i] > 0.0:", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "m_eff = i + 1\n", "m_eff = i\n", LANCZOS_PINS),
    ("oracle.lanczos", "_run", "alpha=band[0], beta=band[1]", "alpha=band[1], beta=band[0]", LANCZOS_PINS),
    ("oracle.lanczos", "lanczos", "inner=lambda D, h: D.T @ h", "inner=lambda D, h: np.abs(D).T @ h", LANCZOS_PINS),
    ("oracle.lanczos", "tridiagonal", "off = np.asarray(beta[: m_eff - 1]", "off = np.asarray(beta[1: m_eff]", LANCZOS_PINS),
    ("oracle.lanczos", "tridiagonal", "np.diag(off, 1) + np.diag(off, -1)", "np.diag(off, 1)", LANCZOS_PINS),
    ("oracle.lanczos", "tridiagonal", "B = np.diag(np.asarray(alpha[:m_eff]", "B = np.diag(np.asarray(alpha[:m_eff][::-1]",
     LANCZOS_PINS),
    # ---- Algorithm 2 emulation
    ("oracle.lanczos", "lanczos_row_sharded", "return float(sum(float(h[b] @ h[b]) for b in blocks))",
     "return float(sum(np.sqrt(float(h[b] @ h[b])) for b in blocks)) ** 2", SHARDED_PINS),          # local norms added
    ("oracle.lanczos", "lanczos_row_sharded", "return np.sum(partial, axis=0)", "return partial[0]", SHARDED_PINS),   # no all-reduce
    ("oracle.lanczos", "lanczos_row_sharded", "float(h[b] @ h[b]) for b in blocks))",
     "float(h[b] @ h[b]) for b in blocks[:1])) * len(blocks)", SHARDED_PINS),                       # local norm only
    ("oracle.lanczos", "row_blocks", "int(edges[c + 1]))", "int(edges[c + 1]) - 1)", SHARDED_PINS),    # a row lost per device
    # ---- Eq. 8 and the selection after it
    ("oracle.ritz", "ritz", "top = np.arange(m_eff - 1, m_eff - 1 - k, -1)", "top = np.arange(m_eff - k, m_eff)", LANCZOS_PINS),
    ("oracle.ritz", "ritz", "top = np.arange(m_eff - 1, m_eff - 1 - k, -1)", "top = np.arange(m_eff - 2, m_eff - 2 - k, -1)",
     LANCZOS_PINS),
    ("oracle.ritz", "ritz", "bottom = np.arange(0, l)", "bottom = np.arange(1, l + 1)", LANCZOS_PINS),
    ("oracle.ritz", "ritz", "bottom = np.arange(0, l)", "bottom = np.arange(l - 1, -1, -1)", LANCZOS_PINS),
    ("oracle.ritz", "ritz", "S = Umat[:, sel]", "S = Umat[sel, :].T", LANCZOS_PINS),
    ("oracle.ritz", "ritz", "np.asarray(Q[:, :m_eff], dtype=np.float64) @ S", "np.asarray(Q[:, 1:m_eff + 1], dtype=np.float64) @ S",
     LANCZOS_PINS),
    ("oracle.ritz", "ritz", "np.abs(S[m_eff - 1, :])", "np.abs(S[0, :])", LANCZOS_PINS),
    ("oracle.ritz", "ritz", "abs(float(beta[m_eff - 1]))", "abs(float(beta[m_eff - 2]))", LANCZOS_PINS),
    # ---- Eq. 4 / Eq. 12 / Eq. 14
    ("oracle.step", "fosi_step", "delta1 = -alpha * (V @ (c / denom))", "delta1 = alpha * (V @ (c / denom))", STEP_PINS),
    ("oracle.step", "fosi_step", "delta1 = -alpha * (V @ (c / denom))", "delta1 = -alpha * (V @ (c * denom))", STEP_PINS),
    ("oracle.step", "fosi_step", "delta1 = -alpha * (V @ (c / denom))", "delta1 = -(V @ (c / denom))", STEP_PINS),
    ("oracle.step", "fosi_step", "denom = a_hat + sig if curv_mode", "denom = a_hat if curv_mode", STEP_PINS),
    ("oracle.step", "fosi_step", "else np.abs(a_hat) + sig", "else np.abs(a_hat + sig)", STEP_PINS),
    ("oracle.step", "fosi_step", "g_tilde, sig = g + np.asarray(pi, dtype=np.float64), float(sigma)",
     "g_tilde, sig = g - np.asarray(pi, dtype=np.float64), float(sigma)", STEP_PINS),
    ("oracle.step", "fosi_step", "in_span = V @ (V.T @ g_tilde)", "in_span = V @ (V.T @ g)", STEP_PINS),
    ("oracle.step", "fosi_step", "c = V.T @ in_span", "c = V.T @ (g_tilde - in_span)", STEP_PINS),
    ("oracle.step", "fosi_step", "x = g_tilde - g1", "x = g_tilde", STEP_PINS),
    ("oracle.step", "fosi_step", "x = g_tilde - g1", "x = g - g1", STEP_PINS),
    ("oracle.step", "fosi_step", "b_new = momentum * b + x", "b_new = momentum * (b + x)", STEP_PINS),
    ("oracle.step", "fosi_step", "b_new = momentum * b + x", "b_new = momentum * b + (1.0 - momentum) * x", STEP_PINS),
    ("oracle.step", "fosi_step", "o = -lr * b_new", "o = lr * b_new", STEP_PINS),
    ("oracle.step", "fosi_step", "o = -lr * b_new", "o = -lr * x", STEP_PINS),
    ("oracle.step", "fosi_step", "delta2 = o - V @ (V.T @ o)", "delta2 = o", STEP_PINS),
    ("oracle.step", "fosi_step", "delta2 = o - V @ (V.T @ o)", "delta2 = o - V @ (V.T @ x)", STEP_PINS),
    ("oracle.step", "fosi_step", "return w + delta1 + delta2, b_new", "return w + delta1 - delta2, b_new", STEP_PINS),
    # ---- the same update with AdamW as base optimiser
    ("oracle.step", "fosi_step_adamw", "m_hat = m_new / (1.0 - beta1 ** step_index)", "m_hat = m_new", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "v_hat = v_new / (1.0 - beta2 ** step_index)", "v_hat = v_new / (1.0 - beta1 ** step_index)",
     ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "(1.0 - beta2) * x * x", "(1.0 - beta2) * x", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "(np.sqrt(v_hat) + eps)", "np.sqrt(v_hat + eps)", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "+ weight_decay * w)", "- weight_decay * w)", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "x = g_tilde - in_span", "x = g_tilde", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "c = V.T @ in_span", "c = V.T @ (g_tilde - in_span)", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "delta2 = o - V @ (V.T @ o)", "delta2 = o", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "denom = a_hat + sig if curv_mode", "denom = a_hat if curv_mode", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "delta1 = -alpha * (V @ (c / denom))", "delta1 = alpha * (V @ (c / denom))", ADAMW_PINS),
    ("oracle.step", "fosi_step_adamw", "else np.abs(a_hat) + sig", "else np.abs(a_hat + sig)", ADAMW_PINS),
    # ---- Algorithm 3 / Eq. 11
    ("oracle.admm", "admm_begin", "/ float(sigma)", "* float(sigma)", ADMM_PINS),
    ("oracle.admm", "admm_begin", "return w, w.copy()", "return w, np.asarray(w_a, dtype=np.float64).copy()", ADMM_PINS),
    ("oracle.admm", "admm_end", "np.asarray(w_a, dtype=np.float64) - np.asarray(w_anchor, dtype=np.float64)",
     "np.asarray(w_anchor, dtype=np.float64) - np.asarray(w_a, dtype=np.float64)", ADMM_PINS),
    ("oracle.admm", "admm_end", "+ float(sigma) * (", "+ (", ADMM_PINS),
    # ---- curvature operators
    ("oracle.hvp", "hvp_planted", "coeff = U64.T @ v64", "coeff = np.abs(U64).T @ v64", HVP_PINS),
    ("oracle.hvp", "hvp_planted", "+ float(shift) * v64", "", HVP_PINS),
    ("oracle.hvp", "hvp_planted", "(np.asarray(lam, dtype=np.float64) * coeff)", "coeff", HVP_PINS),
    ("oracle.hvp", "hvp_softmax_ggn", "np.sum(P * Z, axis=1, keepdims=True)", "np.sum(Z, axis=1, keepdims=True)", HVP_PINS),
    ("oracle.hvp", "hvp_softmax_ggn", "Y = P * Z - P * np.sum(P * Z, axis=1, keepdims=True)", "Y = P * Z", HVP_PINS),
    ("oracle.hvp", "hvp_softmax_ggn", "(X64.T @ Y / B)", "(X64.T @ Y)", HVP_PINS),
    ("oracle.hvp", "hvp_softmax_ggn", "dtype=np.float64).reshape(d, C)", "dtype=np.float64).reshape(C, d).T", HVP_PINS),
    ("oracle.hvp", "softmax_rows", "e.sum(axis=1, keepdims=True)", "e.sum(axis=0, keepdims=True)", HVP_PINS),
]

BUILDERS = {"cfg1": pins.make_cfg1, "cfg2_small": pins.make_cfg2_small, "ggn_small": pins.make_ggn_small}


def _install(monkeypatch, module_name, func_name, old, new):
    """Compiles the function with `old` replaced by `new` and puts it wherever the original is bound."""
    mod = importlib.import_module(module_name)
    original = getattr(mod, func_name)
    src = textwrap.dedent(inspect.getsource(original))
    assert src.count(old) >= 1, f"{module_name}.{func_name} no longer contains {old!r}: update this case"
    namespace = dict(mod.__dict__)
    exec(compile(src.replace(old, new, 1), f"<mutant of {module_name}.{func_name}>", "exec"), namespace)
    mutant = namespace[func_name]
    for holder in (mod, oracle, importlib.import_module("oracle.ritz"), importlib.import_module("oracle.lanczos"), pins):
        if getattr(holder, func_name, None) is original:
            monkeypatch.setattr(holder, func_name, mutant)
    return mutant


def _run(pin, cache):
    args = []
    for name in inspect.signature(pin).parameters:
        if name not in cache:
            cache[name] = BUILDERS[name]()
        args.append(cache[name])
    pin(*args)


@pytest.mark.parametrize("module_name,func_name,old,new,pin_set", MUTANTS,
                         ids=[f"{m[1]}:{m[2][:28].strip()}->{m[3][:28].strip()}" for m in MUTANTS])
def test_a_pin_fails_for_every_planted_mistake(monkeypatch, module_name, func_name, old, new, pin_set):
    _install(monkeypatch, module_name, func_name, old, new)
    cache, caught = {}, []
    for pin in pin_set:
        try:
            _run(pin, cache)
        except Exception as e:        # an assertion, or the broken function blowing up: either way it is noticed
            caught.append((pin.__name__, type(e).__name__))
            break
    assert caught, f"no pin noticed: {module_name}.{func_name}: {old!r} -> {new!r}"


def test_the_unbroken_oracle_passes_the_same_pins():
    cache = {}
    for pin in LANCZOS_PINS + SHARDED_PINS + STEP_PINS + ADAMW_PINS + ADMM_PINS + HVP_PINS:
        _run(pin, cache)
