"""Helpers shared by the tests (no method arithmetic beyond the error metric)."""
import numpy as np

from glowq_inputs import CONFIGS, config_units, gen_activations, gen_module_weight


def rel_err(y, y_ref):
    """Elementwise relative error with an RMS floor:
    max |y - y_ref| / max(|y_ref|, rms(y_ref)).  The floor keeps the measure
    defined where an output happens to be near zero."""
    y = np.asarray(y, np.float64)
    y_ref = np.asarray(y_ref, np.float64)
    rms = float(np.sqrt(np.mean(y_ref ** 2))) if y_ref.size else 1.0
    den = np.maximum(np.abs(y_ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(y - y_ref) / den)) if y_ref.size else 0.0


def recipe_unit(oracle, cfg_id, unit_index, T, r=None, method="svd", shape=None, act=None,
                G=None, seed=None, rows_scale=1, qr="cholesky"):
    """Stored operands of one unit made the way the workload recipe says:
    Gaussian weights -> RTN INT4 -> stacked-error factors -> 16-bit storage."""
    cfg = CONFIGS[cfg_id]
    shape = shape or config_units(cfg_id)[unit_index]
    seed = cfg["seed"] if seed is None else seed
    act = act or cfg["act"]
    G = G or cfg["G"]
    r = cfg["r"] if r is None else r
    W = [gen_module_weight(seed, unit_index, i, o // rows_scale, shape.d_in)
         for i, o in enumerate(shape.d_outs)]
    X = gen_activations(seed, unit_index, T, shape.d_in, act, cfg["outliers"])
    Omega = None
    if method == "alg1":
        Omega = np.random.default_rng([seed, unit_index, 505]).standard_normal((shape.d_in, r + 16))
    unit = oracle.build_unit(W, X, r, G, act, method=method, Omega=Omega, qr=qr)
    unit["W"] = W
    return unit
