"""Random valid postfix expressions for the template tests (test helper only)."""
import numpy as np

SAFE_UNARY = ["neg", "abs", "pow2", "sign", "neq0", "sigmoid", "exp"]
SAFE_BINARY = ["add", "sub", "mul", "min", "max", "lt", "le", "gt", "ge", "eq", "ne"]


def _safe_log():
    return [("abs",), ("const", 0.5), ("add",), ("log",)]


def _safe_sqrt():
    return [("abs",), ("sqrt",)]


def _safe_div():
    return [("abs",), ("const", 0.25), ("add",), ("div",)]


def random_scalar_expr(rng, n_sides, depth=4, leaves=("main", "side", "const"), extra_leaf=None):
    """Random per-element scalar expression (Cell / MAgg / Outer bodies)."""
    def leaf():
        choices = list(leaves) + ([extra_leaf] if extra_leaf else [])
        c = choices[rng.integers(len(choices))]
        if c == "side":
            if n_sides == 0:
                return [("main",)]
            return [("side", int(rng.integers(n_sides)))]
        if c == "const":
            return [("const", float(np.round(rng.uniform(-2, 2), 3)))]
        return [(c,)]

    def build(d):
        if d == 0 or rng.random() < 0.15:
            return leaf()
        p = rng.random()
        if p < 0.35:
            t = rng.integers(len(SAFE_UNARY) + 2)
            inner = build(d - 1)
            if t == len(SAFE_UNARY):
                return inner + _safe_log()
            if t == len(SAFE_UNARY) + 1:
                return inner + _safe_sqrt()
            return inner + [(SAFE_UNARY[t],)]
        a, b = build(d - 1), build(d - 1)
        t = rng.integers(len(SAFE_BINARY) + 1)
        if t == len(SAFE_BINARY):
            return a + b + _safe_div()
        return a + b + [(SAFE_BINARY[t],)]

    return build(depth)


def random_row_expr(rng, side_kinds, depth=4, want="V", sparse_safe=False, reductions=True):
    """Random Row expression producing a row vector ("V") or a per-row scalar ("S").

    ``side_kinds``: list of kinds of the side inputs.  With ``sparse_safe`` the
    program stays zero-preserving w.r.t. the main input (usable on CSR rows);
    ``reductions=False`` leaves out rowsum / dot (a Cell body).
    """
    v_sides = [k for k, s in enumerate(side_kinds) if s in ("matrix", "rowvec")]
    s_sides = [k for k, s in enumerate(side_kinds) if s in ("colvec", "scalar")]
    zp_unary = ["neg", "abs", "pow2", "sign", "neq0"]

    def scalar(d):
        if d == 0 or rng.random() < 0.2:
            if s_sides and rng.random() < 0.5:
                return [("side", int(s_sides[rng.integers(len(s_sides))]))]
            return [("const", float(np.round(rng.uniform(-2, 2), 3)))]
        p = rng.random() if reductions else 0.4 + 0.6 * rng.random()
        if p < 0.4:
            a, _ = vector(d - 1, zp=sparse_safe)
            if rng.random() < 0.5:
                return a + [("rowsum",)]
            b, _ = vector(d - 1, zp=False)
            return a + b + [("dot",)]
        if p < 0.6:
            return scalar(d - 1) + [(SAFE_UNARY[rng.integers(len(SAFE_UNARY))],)]
        return scalar(d - 1) + scalar(d - 1) + [(["add", "sub", "mul", "min", "max"][rng.integers(5)],)]

    def vector(d, zp):
        """returns (tokens, zero_preserving)"""
        if d == 0 or rng.random() < 0.2:
            if zp or not v_sides or rng.random() < 0.5:
                return [("main",)], True
            return [("side", int(v_sides[rng.integers(len(v_sides))]))], False
        p = rng.random()
        if p < 0.25:
            a, za = vector(d - 1, zp)
            if zp:
                return a + [(zp_unary[rng.integers(len(zp_unary))],)], True
            u = SAFE_UNARY[rng.integers(len(SAFE_UNARY))]
            return a + [(u,)], za and u in zp_unary
        if p < 0.55:     # vector * scalar
            a, za = vector(d - 1, zp)
            return a + scalar(d - 1) + [("mul",)], za
        if p < 0.8:      # vector * vector (one side may be dense-valued)
            a, za = vector(d - 1, zp)
            b, zb = vector(d - 1, False)
            return a + b + [("mul",)], za or zb
        a, za = vector(d - 1, zp)
        b, zb = vector(d - 1, zp)
        op = ["add", "sub"][rng.integers(2)] if zp else SAFE_BINARY[rng.integers(len(SAFE_BINARY))]
        return a + b + [(op,)], (za and zb and op in ("add", "sub"))

    if want == "S":
        return scalar(depth)
    toks, z = vector(depth, sparse_safe)
    assert z or not sparse_safe
    return toks
