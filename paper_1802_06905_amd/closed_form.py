"""Closed form of the tiling linear program (paper, Section 5.1 and its figure; verification as in Section 5.2).

Offline tool.  The nine-variable program of Section 5 is written as  max c.x  s.t.  G x <= w + F theta  with
theta = log_M of (B, C, K, W, H, R, S, sigma_w, sigma_h), and the parameter space is cut into convex pieces inside
each of which one affine map theta -> x is the optimiser, by the geometric algorithm the section describes: take a
point inside the unexplored piece, solve the program there to a vertex, read off the tight rows, solve them for x as a
function of theta, keep the set of theta where the slack rows stay satisfied as one region, and go on with the rest of
the piece, cut along that region's faces.

What is this build's own:
  * all of the algebra is exact (fractions): the vertex is found by a rational simplex, tight rows are exact zeros, and
    a region's rows and the affine map have small integer coefficients;
  * the objective may carry a tie-break (weights 1 + tiny preferences), which makes the optimiser unique where the
    program has a whole face of optima, so that the partition does not depend on the sampled points; every region's
    map is still checked to be optimal for the plain objective;
  * the interior point of a piece, the test for an empty or flat piece and the removal of redundant faces are small
    floating-point LPs (scipy's HiGHS);
  * parameters are explored in the box 0 <= theta <= 2 with sigma <= filter extent: a loop bound above M acts like M
    (every tile log is at most 1 by the footprint rows), so the box holds every combinatorial case and a caller clamps
    into it without changing the program's feasible set.

Run as a script (it needs neither the GPU nor the built library):
  python paper_1802_06905_amd/closed_form.py --write --report     regenerates csrc/cacnn_closed_form_table.inc, the table
                                                                  behind cacnn_closed_form_tiling (about two minutes)
  python paper_1802_06905_amd/closed_form.py --paper-space --report   the partition of the paper's own parameter space
                                                                  (filter inside the image), seconds
With the tie-break the whole box has 116 regions (2612 pieces visited), the paper's parameter space 52 (224 pieces);
without it the count depends on the sampled points (57 and 69 regions, 258 and 337 pieces for two seeds in the paper's
space; the paper reports 200 for its own run).  The Section 5.2 check comes out at exactly zero in both directions.
"""
import argparse
import os
import random
import sys
from fractions import Fraction
from typing import List, NamedTuple, Optional, Sequence, Tuple

import numpy as np
from scipy.optimize import linprog

VARS = ("b", "c", "k", "w", "h", "r1", "r2", "s1", "s2")          # r = sigma_w r1 + r2, s = sigma_h s1 + s2
PARAMS = ("B", "C", "K", "W", "H", "R", "S", "sw", "sh")
NV, NP = len(VARS), len(PARAMS)
BOX = 2
_V = {v: i for i, v in enumerate(VARS)}
_P = {p: i for i, p in enumerate(PARAMS)}


def program():
    """(G, w, F): rows of G x <= w + F theta, integers.  Row order: the nine sign rows, the nine loop-bound rows, then
    the Out, Filter and four Image footprint rows (Section 5)."""
    G, w, F = [], [], []

    def row(xs, const, ths):
        g = [0] * NV
        for v, cf in xs.items():
            g[_V[v]] = cf
        f = [0] * NP
        for p, cf in ths.items():
            f[_P[p]] = cf
        G.append(g)
        w.append(const)
        F.append(f)

    for v in VARS:
        row({v: -1}, 0, {})
    for v, p in zip(("b", "c", "k", "w", "h"), ("B", "C", "K", "W", "H")):
        row({v: 1}, 0, {p: 1})
    row({"r2": 1}, 0, {"sw": 1})
    row({"s2": 1}, 0, {"sh": 1})
    row({"r1": 1}, 0, {"R": 1, "sw": -1})
    row({"s1": 1}, 0, {"S": 1, "sh": -1})
    ones = lambda names: {n: 1 for n in names}
    row(ones(("b", "k", "w", "h")), 1, {})
    row(ones(("c", "k", "r1", "r2", "s1", "s2")), 1, {})
    row(ones(("b", "c", "w", "h", "r2", "s2")), 1, {})
    row(ones(("b", "c", "w", "s1", "r2", "s2")), 1, {})
    row(ones(("b", "c", "r1", "h", "r2", "s2")), 1, {})
    row(ones(("b", "c", "r1", "s1", "r2", "s2")), 1, {})
    return G, w, F


G_ROWS, W_ROWS, F_ROWS = program()
NROWS = len(G_ROWS)

# the five terms of Theorem 1 as logs base M: (coefficients of theta, constant); the half-integers are doubled
_LB2 = (
    ({"B": 2, "K": 2, "W": 2, "H": 2}, 0),
    ({"sw": 2, "sh": 2, "B": 2, "C": 2, "W": 2, "H": 2}, 0),
    ({"C": 2, "K": 2, "R": 2, "S": 2}, 0),
    ({"B": 2, "C": 2, "K": 2, "W": 2, "H": 2, "R": 2, "S": 2}, -2),
    ({"B": 2, "C": 2, "K": 2, "W": 2, "H": 2, "R": 1, "S": 1, "sw": 1, "sh": 1}, -1),
)


def bound_terms_log() -> List[Tuple[List[Fraction], Fraction]]:
    out = []
    for co, const in _LB2:
        a = [Fraction(0)] * NP
        for p, cf in co.items():
            a[_P[p]] = Fraction(cf, 2)
        out.append((a, Fraction(const, 2)))
    return out


def parameter_space() -> List[Tuple[List[Fraction], Fraction]]:
    """Rows a.theta <= b of the explored parameter space."""
    rows = []
    for i in range(NP):
        lo = [Fraction(0)] * NP
        lo[i] = Fraction(-1)
        rows.append((lo, Fraction(0)))
        hi = [Fraction(0)] * NP
        hi[i] = Fraction(1)
        rows.append((hi, Fraction(BOX)))
    for s, r in (("sw", "R"), ("sh", "S")):
        a = [Fraction(0)] * NP
        a[_P[s]] = Fraction(1)
        a[_P[r]] = Fraction(-1)
        rows.append((a, Fraction(0)))
    return rows


def filter_inside_image() -> List[Tuple[List[Fraction], Fraction]]:
    """The paper's standing assumption R <= sigma_w W, S <= sigma_h H (Section 2) as rows.  The table is built without
    it, so that any shape can be looked up; the count of regions and the Section 5.2 check are reported with it, because
    Theorem 1's Image term stands for the array's size only then."""
    rows = []
    for r, s, w in (("R", "sw", "W"), ("S", "sh", "H")):
        a = [Fraction(0)] * NP
        a[_P[r]] = Fraction(1)
        a[_P[s]] = Fraction(-1)
        a[_P[w]] = Fraction(-1)
        rows.append((a, Fraction(0)))
    return rows


def default_weights() -> List[Fraction]:
    """Tie-break: among optimal tilings prefer, in this order, a larger tile in b (the fastest index of Image and Out),
    k, c, w, h, then the filter indices.  Powers of two keep sums of different subsets apart."""
    order = ("b", "k", "c", "w", "h", "r1", "s1", "r2", "s2")
    wts = [Fraction(1)] * NV
    for rank, v in enumerate(order):
        wts[_V[v]] = 1 + Fraction(2 ** (NV - 1 - rank), 2 ** 24)
    return wts


# ---------------------------------------------------------------------------------------------------------------
# exact pieces


def rhs_at(theta: Sequence[Fraction]) -> List[Fraction]:
    return [Fraction(W_ROWS[i]) + sum(F_ROWS[i][j] * theta[j] for j in range(NP)) for i in range(NROWS)]


def simplex_vertex(theta: Sequence[Fraction], weights: Sequence[Fraction]) -> List[Fraction]:
    """A vertex maximising weights.x at theta, by a rational tableau simplex with Bland's rule.  x >= 0 is kept by the
    method itself; the other rows get slacks, whose basis is feasible because their right-hand sides are >= 0."""
    rows = list(range(NV, NROWS))
    rhs = rhs_at(theta)
    m = len(rows)
    cols = NV + m + 1
    T = [[Fraction(0)] * cols for _ in range(m + 1)]
    basis = []
    for i, r in enumerate(rows):
        if rhs[r] < 0:
            raise ValueError("theta outside the parameter space")
        for j in range(NV):
            T[i][j] = Fraction(G_ROWS[r][j])
        T[i][NV + i] = Fraction(1)
        T[i][-1] = rhs[r]
        basis.append(NV + i)
    for j in range(NV):
        T[m][j] = -Fraction(weights[j])
    while True:
        enter = next((j for j in range(cols - 1) if T[m][j] < 0), None)
        if enter is None:
            break
        leave, best = None, None
        for i in range(m):
            if T[i][enter] > 0:
                ratio = T[i][-1] / T[i][enter]
                if leave is None or ratio < best or (ratio == best and basis[i] < basis[leave]):
                    leave, best = i, ratio
        if leave is None:
            raise ArithmeticError("unbounded")   # cannot happen: every variable has an upper row
        piv = T[leave][enter]
        T[leave] = [v / piv for v in T[leave]]
        for i in range(m + 1):
            if i != leave and T[i][enter] != 0:
                f = T[i][enter]
                T[i] = [a - f * b for a, b in zip(T[i], T[leave])]
        basis[leave] = enter
    x = [Fraction(0)] * NV
    for i, bj in enumerate(basis):
        if bj < NV:
            x[bj] = T[i][-1]
    return x


class Form(NamedTuple):
    X: Tuple[Tuple[Fraction, ...], ...]   # x = X theta + x0
    x0: Tuple[Fraction, ...]
    tight: Tuple[int, ...]

    def at(self, theta):
        return [self.x0[i] + sum(self.X[i][j] * theta[j] for j in range(NP)) for i in range(NV)]


def solve_tight_rows(tight: Sequence[int], fixed=None) -> Optional[Form]:
    """Solve the tight rows, taken as equalities, for x as an affine function of theta.  None if they do not determine
    x, or if they only hold together on a thinner set of theta (the sampled point sat on a border).
    fixed: {parameter index: value} for parameters that do not vary; rows only need to agree on that slice."""
    fixed = fixed or {}
    A = [[Fraction(v) for v in G_ROWS[r]] + [Fraction(W_ROWS[r])] + [Fraction(v) for v in F_ROWS[r]] for r in tight]
    piv_rows = []
    r = 0
    for col in range(NV):
        p = next((i for i in range(r, len(A)) if A[i][col] != 0), None)
        if p is None:
            return None
        A[r], A[p] = A[p], A[r]
        pv = A[r][col]
        A[r] = [v / pv for v in A[r]]
        for i in range(len(A)):
            if i != r and A[i][col] != 0:
                f = A[i][col]
                A[i] = [a - f * b for a, b in zip(A[i], A[r])]
        piv_rows.append(r)
        r += 1
    for i in range(r, len(A)):
        # left over: 0 = const + (coefficients).theta, which has to hold on the whole slice
        if any(A[i][NV + 1 + j] != 0 for j in range(NP) if j not in fixed):
            return None
        if A[i][NV] + sum(A[i][NV + 1 + j] * v for j, v in fixed.items()) != 0:
            return None
    # parameters that do not vary go into the constant, so that one function has one representation
    X = tuple(tuple(Fraction(0) if j in fixed else A[i][NV + 1 + j] for j in range(NP)) for i in range(NV))
    x0 = tuple(A[i][NV] + sum(A[i][NV + 1 + j] * v for j, v in fixed.items()) for i in range(NV))
    return Form(X, x0, tuple(tight))


def region_rows(form: Form) -> List[Tuple[List[Fraction], Fraction]]:
    """Rows a.theta <= b that say: every row of the program that is not tight stays satisfied at form.at(theta)."""
    out = []
    for r in range(NROWS):
        if r in form.tight:
            continue
        a = [sum(G_ROWS[r][i] * form.X[i][j] for i in range(NV)) - F_ROWS[r][j] for j in range(NP)]
        b = W_ROWS[r] - sum(G_ROWS[r][i] * form.x0[i] for i in range(NV))
        if all(v == 0 for v in a):
            if b < 0:
                raise ArithmeticError("a slack row that is violated everywhere")
            continue
        out.append((a, Fraction(b)))
    return out


# ---------------------------------------------------------------------------------------------------------------
# floating-point helpers on pieces of parameter space


def _np_rows(rows):
    A = np.array([[float(v) for v in a] for a, _ in rows], dtype=np.float64).reshape(len(rows), len(rows[0][0]))
    b = np.array([float(c) for _, c in rows], dtype=np.float64)
    return A, b


def chebyshev(rows) -> Tuple[Optional[np.ndarray], float]:
    """Centre and radius of the largest ball inside {a.theta <= b}; radius <= 0 for an empty piece."""
    A, b = _np_rows(rows)
    n = A.shape[1]
    nrm = np.linalg.norm(A, axis=1)
    res = linprog(c=np.r_[np.zeros(n), -1.0], A_ub=np.c_[A, nrm], b_ub=b,
                  bounds=[(None, None)] * n + [(0, BOX)], method="highs")
    if res.status != 0:
        return None, -1.0
    return res.x[:n], float(res.x[n])


def maximise(obj: Sequence[float], rows) -> Optional[float]:
    A, b = _np_rows(rows)
    res = linprog(c=-np.asarray(obj, dtype=np.float64), A_ub=A, b_ub=b, bounds=[(None, None)] * A.shape[1], method="highs")
    if res.status != 0:
        return None
    return float(-res.fun)


def drop_redundant(new_rows, within):
    """Those of new_rows that cut something off {within and the other kept rows}."""
    kept = list(new_rows)
    i = 0
    while i < len(kept):
        a, b = kept[i]
        others = within + kept[:i] + kept[i + 1:]
        top = maximise([float(v) for v in a], others)
        if top is not None and top <= float(b) + 1e-9:
            kept.pop(i)
        else:
            i += 1
    return kept


# ---------------------------------------------------------------------------------------------------------------
# the partition


class Region(NamedTuple):
    rows: List[Tuple[List[Fraction], Fraction]]    # a.theta <= b, parameter-space rows included where they matter
    form: int                                       # index into Partition.forms
    sample: Tuple[Fraction, ...]                    # the interior point it was found from


class Partition(NamedTuple):
    pieces: List[Region]       # what the algorithm visits: convex pieces, several of which may share a closed form
    forms: List[Form]
    free: Tuple[int, ...]      # the parameters the rows of pieces and regions are written in (all nine unless some were fixed)
    regions: List[Region]      # one per closed form: every theta of the space at which that form is feasible.  A form
                               # carries a dual certificate on its tight rows that does not depend on theta, so it is
                               # optimal wherever it is feasible; the pieces of a form lie inside its region
    resampled: int


MIN_RADIUS = 1e-6


def partition(space=None, weights=None, seed: int = 1802, max_regions: int = 20000, fixed=None) -> Partition:
    """The algorithm of Section 5.1's figure, with an explicit stack in place of the recursion.
    fixed: {parameter name: value} holds some parameters at a value (strides 1: sw = sh = 0); the partition is then of
    the remaining ones, and the rows of its pieces and regions have one coefficient per free parameter."""
    space = parameter_space() if space is None else space
    weights = default_weights() if weights is None else weights
    fixed = {_P[k]: Fraction(v) for k, v in (fixed or {}).items()}
    free = tuple(j for j in range(NP) if j not in fixed)
    plain = [Fraction(1)] * NV
    rng = random.Random(seed)

    def project(rows):
        out = []
        for a, b in rows:
            b2 = b - sum(a[j] * v for j, v in fixed.items())
            a2 = [a[j] for j in free]
            if all(v == 0 for v in a2):
                if b2 < 0:
                    raise ValueError("the fixed parameters lie outside the space")
                continue
            out.append((a2, b2))
        return out

    def expand(point):
        theta = [Fraction(0)] * NP
        for j, v in fixed.items():
            theta[j] = v
        for j, v in zip(free, point):
            theta[j] = v
        return tuple(theta)

    space = project(space)
    forms: List[Form] = []
    form_index = {}
    pieces: List[Region] = []
    resampled = 0
    stack = [list(space)]
    while stack:
        piece = stack.pop()
        centre, radius = chebyshev(piece)
        if centre is None or radius < MIN_RADIUS:
            continue                                    # empty, or thinner than the parameter space
        form = None
        for attempt in range(50):
            step = np.array([rng.uniform(-1, 1) for _ in free])
            step *= 0.5 * radius * rng.random() / max(1e-12, float(np.linalg.norm(step)))
            point = tuple(Fraction(float(v)).limit_denominator(1 << 20) for v in (centre + step))
            if any(sum(a[j] * point[j] for j in range(len(free))) >= b for a, b in piece):
                continue
            theta0 = expand(point)
            x = simplex_vertex(theta0, weights)
            rhs = rhs_at(theta0)
            tight = [r for r in range(NROWS) if sum(G_ROWS[r][i] * x[i] for i in range(NV)) == rhs[r]]
            form = solve_tight_rows(tight, fixed)
            if form is not None:
                if sum(x) != sum(simplex_vertex(theta0, plain)):
                    raise ArithmeticError("tie-break weights changed the optimum")
                break
            resampled += 1
        if form is None:
            raise ArithmeticError("no interior sample gave a determined vertex")
        key = (form.X, form.x0)
        if key not in form_index:
            form_index[key] = len(forms)
            forms.append(form)
        faces = drop_redundant(project(region_rows(form)), piece)
        pieces.append(Region(piece + faces, form_index[key], theta0))
        if len(pieces) > max_regions:
            raise ArithmeticError("too many pieces")
        for i, (a, b) in enumerate(faces):
            child = piece + faces[:i] + [([-v for v in a], -b)]
            stack.append(child)
    regions = []
    for n, form in enumerate(forms):
        rows = drop_redundant(list(space) + project(region_rows(form)), [])
        first = next(pc.sample for pc in pieces if pc.form == n)
        regions.append(Region(rows, n, first))
    return Partition(pieces, forms, free, regions, resampled)


# ---------------------------------------------------------------------------------------------------------------
# Section 5.2


def cost_log(form: Form) -> Tuple[List[Fraction], Fraction]:
    """log_M of the words moved with the region's tiling: sum of the seven loop-bound logs + 1 - sum of the tile logs."""
    a = [Fraction(0)] * NP
    for p in ("B", "C", "K", "W", "H", "R", "S"):
        a[_P[p]] += 1
    for j in range(NP):
        a[j] -= sum(form.X[i][j] for i in range(NV))
    return a, Fraction(1) - sum(form.x0)


class Check(NamedTuple):
    worst_excess: float      # max over regions, terms i of max { cost - L_i : theta in region, L_i largest, L_i >= 1 }
    worst_deficit: float     # min over regions, terms i of min { cost - L_i : theta in region }
    cells: int               # (region, term) pairs with a non-empty cell
    regions: int             # regions with a full-dimensional part inside `within`


def verify(part: Partition, within=None) -> Check:
    """Section 5.2's two families of LPs over every region cut down to `within` (default: filter_inside_image())."""
    terms = bound_terms_log()
    within = filter_inside_image() if within is None else within
    worst_excess, worst_deficit, cells = 0.0, float("inf"), 0
    for full in part.regions:
        reg = Region(list(full.rows) + list(within), full.form, full.sample)
        if chebyshev(reg.rows)[1] < MIN_RADIUS:
            continue
        ca, cb = cost_log(part.forms[reg.form])
        for i, (la, lb) in enumerate(terms):
            diff = [float(ca[j] - la[j]) for j in range(NP)]
            const = float(cb - lb)
            low = maximise([-d for d in diff], reg.rows)
            if low is not None:
                worst_deficit = min(worst_deficit, -low + const)
            cell = list(reg.rows)
            for j, (oa, ob) in enumerate(terms):
                if j != i:
                    cell.append(([oa[t] - la[t] for t in range(NP)], lb - ob))     # L_j <= L_i
            cell.append(([-v for v in la], lb - 1))                                 # L_i >= 1
            top = maximise(diff, cell)
            if top is not None:
                cells += 1
                worst_excess = max(worst_excess, top + const)
    inside = sum(1 for r in part.regions if chebyshev(list(r.rows) + list(within))[1] >= MIN_RADIUS)
    return Check(worst_excess, worst_deficit, cells, inside)


# ---------------------------------------------------------------------------------------------------------------
# look-up, and the table for the C side


def clamp(theta: Sequence[float]) -> List[float]:
    """Into the explored box without changing the program: a loop bound above M acts like M."""
    t = [max(0.0, float(v)) for v in theta]
    for p in ("B", "C", "K", "W", "H"):
        t[_P[p]] = min(t[_P[p]], 1.0)
    for s, r in (("sw", "R"), ("sh", "S")):
        sg = min(t[_P[s]], t[_P[r]])
        rest = min(t[_P[r]] - sg, 1.0)
        sg = min(sg, 1.0)
        t[_P[s]], t[_P[r]] = sg, sg + rest
    return t


def locate(part: Partition, theta: Sequence[float], tol: float = 1e-9) -> int:
    """Index of a region that holds theta (borders belong to both sides; the optimum is the same on either)."""
    best, best_v = -1, float("inf")
    point = [theta[j] for j in part.free]
    for n, reg in enumerate(part.regions):
        v = max(sum(float(c) * t for c, t in zip(a, point)) - float(b) for a, b in reg.rows)
        if v <= tol:
            return n
        if v < best_v:
            best, best_v = n, v
    return best


def _int_row(vals: Sequence[Fraction]) -> Tuple[List[int], int]:
    den = 1
    for v in vals:
        den = den * v.denominator // np.gcd(den, v.denominator)
    den = int(den)
    return [int(v * den) for v in vals], den


def table_text(part: Partition) -> str:
    out = ["// Generated by paper_1802_06905_amd/closed_form.py --write; do not edit.",
           "// Closed form of the tiling LP (Section 5.1): regions of theta = log_M(B, C, K, W, H, R, S, sigma_w, sigma_h),",
           "// each with the affine map theta -> tile logs (b, c, k, w, h, r', r'', s', s'') that is optimal inside it.",
           f"static const int kClosedFormRegions = {len(part.regions)};",
           f"static const int kClosedFormForms = {len(part.forms)};",
           f"static const int kClosedFormFaces = {sum(len(r.rows) for r in part.regions)};",
           "// forms: 9 rows of (9 coefficients of theta, constant), integers over the form's common denominator",
           "static const int16_t kClosedFormNum[][9][10] = {"]
    dens = []
    for f in part.forms:
        flat = [v for i in range(NV) for v in (*f.X[i], f.x0[i])]
        ints, den = _int_row(flat)
        dens.append(den)
        rows = ["{" + ", ".join(str(v) for v in ints[i * 10:(i + 1) * 10]) + "}" for i in range(NV)]
        out.append("    {" + ", ".join(rows) + "},")
    out.append("};")
    out.append("static const int16_t kClosedFormDen[] = {" + ", ".join(str(d) for d in dens) + "};")
    out.append("// faces a.theta <= b as (9 integer coefficients, b); a region owns faces [first, first + count)")
    out.append("static const int16_t kClosedFormFace[][10] = {")
    first, spans = 0, []
    for r in part.regions:
        for a, b in r.rows:
            ints, _ = _int_row(list(a) + [b])
            out.append("    {" + ", ".join(str(v) for v in ints) + "},")
        spans.append((first, len(r.rows), r.form))
        first += len(r.rows)
    out.append("};")
    out.append("// regions: first face, number of faces, form")
    out.append("static const int32_t kClosedFormRegion[][3] = {")
    for s in spans:
        out.append("    {%d, %d, %d}," % s)
    out.append("};")
    return "\n".join(out) + "\n"


TABLE_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "cacnn_closed_form_table.inc")


def load_table(path: str = TABLE_PATH) -> Partition:
    """The committed table back as a Partition (regions and forms; no pieces, no samples)."""
    import re
    text = open(path).read()

    def block(name):
        body = text[text.index(name):]
        body = body[body.index("= {") + 3:body.index("};")]
        return [int(v) for v in re.findall(r"-?\d+", body)]

    num, den, face, reg = block("kClosedFormNum["), block("kClosedFormDen["), block("kClosedFormFace["), block("kClosedFormRegion[")
    forms = []
    for n, d in enumerate(den):
        rows = [num[(n * NV + i) * 10:(n * NV + i + 1) * 10] for i in range(NV)]
        X = tuple(tuple(Fraction(v, d) for v in r[:NP]) for r in rows)
        x0 = tuple(Fraction(r[NP], d) for r in rows)
        forms.append(Form(X, x0, ()))
    regions = []
    for n in range(len(reg) // 3):
        first, count, form = reg[3 * n:3 * n + 3]
        rows = [([Fraction(v) for v in face[10 * f:10 * f + NP]], Fraction(face[10 * f + NP])) for f in range(first, first + count)]
        regions.append(Region(rows, form, ()))
    return Partition([], forms, tuple(range(NP)), regions, 0)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--write", action="store_true", help="regenerate " + os.path.relpath(TABLE_PATH))
    ap.add_argument("--report", action="store_true", help="region count and the Section 5.2 check")
    ap.add_argument("--plain", action="store_true", help="no tie-break in the objective (the partition then depends on the seed)")
    ap.add_argument("--paper-space", action="store_true",
                    help="explore only R <= sigma_w W, S <= sigma_h H (the paper's parameter space); not for --write")
    ap.add_argument("--seed", type=int, default=1802)
    a = ap.parse_args(argv)
    if a.paper_space and a.write:
        ap.error("the table covers the whole box: --write goes without --paper-space")
    space = parameter_space() + filter_inside_image() if a.paper_space else None
    part = partition(space=space, weights=[Fraction(1)] * NV if a.plain else None, seed=a.seed)
    print(f"pieces visited {len(part.pieces)}  closed forms = regions {len(part.regions)}  "
          f"faces {sum(len(r.rows) for r in part.regions)}  resampled points {part.resampled}")
    if a.report:
        chk = verify(part)
        print(f"with R <= sigma_w W and S <= sigma_h H: {chk.regions} regions; Section 5.2: max over cells of (cost - largest "
              f"bound term) = {chk.worst_excess:.3e} over {chk.cells} cells; min over regions and terms of (cost - term) = "
              f"{chk.worst_deficit:.3e}")
    if a.write:
        with open(TABLE_PATH, "w") as f:
            f.write(table_text(part))
        print("wrote", TABLE_PATH)
    return 0


if __name__ == "__main__":
    sys.exit(main())
