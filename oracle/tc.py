"""Tensor commitment scheme of Def. 4.1 (Setup / Com / Open / Ver) -- oracle.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Notation follows the paper: shape d = (d_1..d_m), trapdoors tau_1..tau_m, grid
Omega = Omega_1 x ... x Omega_m, f_T the interpolant of the tensor T on the
grid, C_T = g^{f_T(tau)}, quotients q_i with r_{i-1} = q_i (X_i - omega_i) + r_i,
proof (pi_1..pi_m) with pi_i = g^{q_i(tau)}.  Group elements are written
additively here: g^a is [a]G.

Readings taken where the paper is silent or inconsistent:
  * grid nodes: zeta_{j,i} = i + 1 for the 0-based array index i (the paper's
    index set [d] = {1..d} used as field elements);
  * per-variable degree is at most d_j - 1, one SRS element per multi-index of
    prod_j {0..d_j-1};
  * verification uses the SUM form  f_T - y = sum_i q_i (X_i - omega_i), which
    is what the iterated division of Open yields; the printed product form does
    not hold for m > 1 and coincides with the sum form for m = 1 (Def. 2.2);
  * the verifier here knows tau (test harness): it checks the G1 equation
    C - [y]G == sum_i [tau_i - omega_i] pi_i, which the pairing equation implies
    and is implied by.

Tensors are flat row-major lists (last axis fastest), the layout App. A fixes
for coefficient arrays, with the strides generalised to non-uniform shapes.
"""
from . import bls12_381 as ec
from .bls12_381 import R

MAX_ORDER = 4


# --- helpers on shapes --------------------------------------------------------
def prod(xs):
    out = 1
    for x in xs:
        out *= int(x)
    return out


def strides(shape):
    """index(i) = sum_j i_j * stride_j, last axis fastest (App. A layout rule)."""
    st = [1] * len(shape)
    for j in range(len(shape) - 2, -1, -1):
        st[j] = st[j + 1] * int(shape[j + 1])
    return st


def flat_index(idx, shape):
    return sum(int(i) * s for i, s in zip(idx, strides(shape)))


def multi_index(flat, shape):
    out = []
    for s in strides(shape):
        out.append(flat // s)
        flat %= s
    return tuple(out)


def as_flat_ints(T):
    """Accept a flat/nested list or a numpy array; return a flat list of Python ints."""
    if hasattr(T, "reshape"):
        return [int(v) for v in T.reshape(-1).tolist()]
    out = []

    def walk(x):
        if isinstance(x, (list, tuple)):
            for y in x:
                walk(y)
        else:
            out.append(int(x))

    walk(T)
    return out


def embed(q):
    """Integer -> field element: negatives map to r - |q|."""
    return int(q) % R


# --- the grid and its Lagrange basis (Def. 4.1 Com; App. C) ---------------------
def grid_nodes(d):
    return [i + 1 for i in range(d)]


def bary_weights_direct(d):
    """beta_l = 1 / prod_{r != l} (zeta_l - zeta_r), straight from App. C."""
    z = grid_nodes(d)
    out = []
    for l in range(d):
        den = 1
        for k in range(d):
            if k != l:
                den = den * (z[l] - z[k]) % R
        out.append(ec.fr_inv(den))
    return out


def bary_weights(d):
    """Same weights for the integer grid: prod_{r != l}(l - r) = l! (d-1-l)! (-1)^{d-1-l}."""
    fact = [1] * d
    for i in range(1, d):
        fact[i] = fact[i - 1] * i % R
    out = []
    for l in range(d):
        den = fact[l] * fact[d - 1 - l] % R
        if (d - 1 - l) & 1:
            den = (-den) % R
        out.append(ec.fr_inv(den))
    return out


def lagrange_at_direct(d, x):
    """l_i(x) = prod_{k != i} (x - zeta_k)/(zeta_i - zeta_k): the definition, O(d^2)."""
    z = grid_nodes(d)
    out = []
    for i in range(d):
        num, den = 1, 1
        for k in range(d):
            if k != i:
                num = num * (x - z[k]) % R
                den = den * (z[i] - z[k]) % R
        out.append(num * ec.fr_inv(den) % R)
    return out


def lagrange_at(d, x):
    """Barycentric form of App. C: l_i(x) = (beta_i/(x - zeta_i)) / sum_r beta_r/(x - zeta_r).
    x must not be a grid node."""
    z = grid_nodes(d)
    beta = bary_weights(d)
    terms = []
    for i in range(d):
        diff = (x - z[i]) % R
        if diff == 0:
            raise ValueError("evaluation point lies on the grid")
        terms.append(beta[i] * ec.fr_inv(diff) % R)
    total_inv = ec.fr_inv(sum(terms) % R)
    return [t * total_inv % R for t in terms]


# --- Setup (Def. 4.1) ----------------------------------------------------------
class PublicParams:
    """pp = (srs, Omega) plus, for the test harness only, the trapdoors."""

    def __init__(self, shape, tau):
        shape = tuple(int(d) for d in shape)
        if not (1 <= len(shape) <= MAX_ORDER) or any(d < 1 for d in shape):
            raise ValueError("bad shape")
        if len(tau) < len(shape):
            raise ValueError("one trapdoor per axis is required")
        self.shape = shape
        self.m = len(shape)
        self.tau = [int(t) % R for t in tau[: self.m]]
        for d, t in zip(shape, self.tau):
            if t == 0 or 1 <= t <= d:
                raise ValueError("trapdoor on the grid or zero")
        # l_{j,i}(tau_j) for every axis j and node i
        self.ell = [lagrange_at(d, t) for d, t in zip(shape, self.tau)]
        self._srs_lagrange = None
        self._srs_monomial = None

    # -- scalar L_i(tau) = prod_j l_{j,i_j}(tau_j) for suffix axes first_axis..m-1
    def lagrange_scalar(self, idx, first_axis=0):
        s = 1
        for j, i in zip(range(first_axis, self.m), idx):
            s = s * self.ell[j][i] % R
        return s

    def srs_lagrange(self, first_axis=0):
        """S^{(a)}[k_a..k_m] = [prod_{j>=a} l_{j,k_j}(tau_j)] G by naive scalar mult.
        A public linear image of the monomial SRS (tiny sizes only)."""
        if self._srs_lagrange is None:
            self._srs_lagrange = {}
        if first_axis not in self._srs_lagrange:
            sub = self.shape[first_axis:]
            self._srs_lagrange[first_axis] = [
                ec.mul(self.lagrange_scalar(multi_index(f, sub), first_axis), ec.G1)
                for f in range(prod(sub))
            ]
        return self._srs_lagrange[first_axis]

    def srs_monomial(self):
        """g_i = [tau_1^{i_1} ... tau_m^{i_m}] G over I = prod_j {0..d_j-1} (Def. 4.1 Setup)."""
        if self._srs_monomial is None:
            out = []
            for f in range(prod(self.shape)):
                idx = multi_index(f, self.shape)
                s = 1
                for t, i in zip(self.tau, idx):
                    s = s * pow(t, i, R) % R
                out.append(ec.mul(s, ec.G1))
            self._srs_monomial = out
        return self._srs_monomial


def setup(shape, tau):
    return PublicParams(shape, tau)


# --- interpolation: grid values -> monomial coefficients (Def. 4.1 Com) ---------
def lagrange_basis_coeffs(d):
    """Coefficient arrays (low degree first) of l_0(X)..l_{d-1}(X) on the grid."""
    z = grid_nodes(d)
    out = []
    for i in range(d):
        poly = [1]
        den = 1
        for k in range(d):
            if k == i:
                continue
            # poly *= (X - z_k)
            nxt = [0] * (len(poly) + 1)
            for e, c in enumerate(poly):
                nxt[e + 1] = (nxt[e + 1] + c) % R
                nxt[e] = (nxt[e] - c * z[k]) % R
            poly = nxt
            den = den * (z[i] - z[k]) % R
        inv = ec.fr_inv(den)
        out.append([c * inv % R for c in poly])
    return out


def interpolate(T, shape):
    """Monomial coefficients a_k of f_T, f_T(omega) = T[omega] on the grid, one axis at a time."""
    shape = tuple(shape)
    a = [embed(v) for v in as_flat_ints(T)]
    st = strides(shape)
    n = prod(shape)
    for j, d in enumerate(shape):
        basis = lagrange_basis_coeffs(d)
        out = [0] * n
        for base in range(n):
            if (base // st[j]) % d != 0:
                continue                        # visit every line along axis j once
            vals = [a[base + i * st[j]] for i in range(d)]
            for e in range(d):
                out[base + e * st[j]] = sum(vals[i] * basis[i][e] for i in range(d)) % R
        a = out
    return a


# --- the three interpolation forms of App. C, one axis at a time ------------------------------
# Each turns the d grid values of a line into the monomial coefficients (low degree first) of the
# line's interpolant; `interpolate_form` applies one of them along every axis in turn.  They are
# algorithms for the result that `interpolate` writes out from the definition.
def _poly_times_linear(poly, root):
    """poly(X) * (X - root)."""
    out = [0] * (len(poly) + 1)
    for e, c in enumerate(poly):
        out[e + 1] = (out[e + 1] + c) % R
        out[e] = (out[e] - c * root) % R
    return out


def line_newton(vals):
    """Newton form: divided differences a_r = f[zeta_0..zeta_r], then sum_r a_r N_r(X) with
    N_r(X) = prod_{t<r} (X - zeta_t), expanded into monomials."""
    d = len(vals)
    z = grid_nodes(d)
    a = [v % R for v in vals]
    for level in range(1, d):
        for k in range(d - 1, level - 1, -1):
            a[k] = (a[k] - a[k - 1]) * ec.fr_inv((z[k] - z[k - level]) % R) % R
    coeffs = [0] * d
    basis = [1]                                    # N_0
    for r in range(d):
        for e, c in enumerate(basis):
            coeffs[e] = (coeffs[e] + a[r] * c) % R
        basis = _poly_times_linear(basis, z[r])    # N_{r+1}
    return coeffs


def line_gregory(vals):
    """Gregory (Newton-Gregory forward) form on the equispaced grid, h = 1: forward differences
    Delta^r T[0], then sum_r binom(s, r) Delta^r T[0] with s = X - zeta_0, expanded into monomials."""
    d = len(vals)
    z = grid_nodes(d)
    assert all(z[k + 1] - z[k] == 1 for k in range(d - 1))
    diff = [v % R for v in vals]
    delta = [diff[0]]
    for _ in range(1, d):
        diff = [(diff[k + 1] - diff[k]) % R for k in range(len(diff) - 1)]
        delta.append(diff[0])
    coeffs = [0] * d
    binom = [1]                                    # binom(s, 0) as a polynomial in X
    for r in range(d):
        for e, c in enumerate(binom):
            coeffs[e] = (coeffs[e] + delta[r] * c) % R
        # binom(s, r+1) = binom(s, r) * (s - r) / (r + 1),  s - r = X - zeta_0 - r
        binom = [c * ec.fr_inv(r + 1) % R for c in _poly_times_linear(binom, z[0] + r)]
    return coeffs


def line_barycentric(vals):
    """Barycentric form: f(X) = M(X) sum_l beta_l T_l / (X - zeta_l) with M(X) = prod_r (X - zeta_r)
    (the denominator sum_r beta_r / (X - zeta_r) of App. C equals 1 / M(X)); each M(X) / (X - zeta_l)
    by synthetic division."""
    d = len(vals)
    z = grid_nodes(d)
    beta = bary_weights(d)
    master = [1]
    for r in range(d):
        master = _poly_times_linear(master, z[r])
    coeffs = [0] * d
    for l in range(d):
        w = vals[l] % R * beta[l] % R
        quotient = [0] * d                          # M(X) / (X - zeta_l), degree d - 1
        carry = 0
        for e in range(d, 0, -1):
            carry = (master[e] + carry * z[l]) % R
            quotient[e - 1] = carry
        for e in range(d):
            coeffs[e] = (coeffs[e] + w * quotient[e]) % R
    return coeffs


INTERPOLATION_FORMS = {"newton": line_newton, "gregory": line_gregory, "barycentric": line_barycentric}


def interpolate_form(T, shape, form):
    """Monomial coefficients of f_T through one of the forms of App. C, axis by axis."""
    line = INTERPOLATION_FORMS[form]
    shape = tuple(shape)
    a = [embed(v) for v in as_flat_ints(T)]
    st = strides(shape)
    n = prod(shape)
    for j, d in enumerate(shape):
        out = [0] * n
        for base in range(n):
            if (base // st[j]) % d != 0:
                continue
            res = line([a[base + i * st[j]] for i in range(d)])
            for e in range(d):
                out[base + e * st[j]] = res[e]
        a = out
    return a


def eval_poly(coeffs, shape, x):
    """f(x_1..x_m) from the lexicographic coefficient array."""
    total = 0
    for f, c in enumerate(coeffs):
        if c:
            term = c
            for xi, e in zip(x, multi_index(f, shape)):
                term = term * pow(xi, e, R) % R
            total = (total + term) % R
    return total


# --- Com (Def. 4.1), three routes that must agree ------------------------------
def commit_literal(pp, T):
    """Route (a): interpolate, then the multi-exponentiation over the monomial SRS."""
    a = interpolate(T, pp.shape)
    return ec.msm_naive(a, pp.srs_monomial())


def commit_lagrange_naive(pp, T):
    """Route (b): C = sum_i [e(T[i])] S[i] with the Lagrange-basis SRS, term by term."""
    return ec.msm_naive([embed(v) for v in as_flat_ints(T)], pp.srs_lagrange(0))


def contract_suffix(values, shape, ell, first_axis):
    """sum over axes first_axis.. of values[...] * prod_j l_j[k_j], contracting the
    last axis first (nested sums, nothing else)."""
    v = list(values)
    for j in range(len(shape) - 1, first_axis - 1, -1):
        d = shape[j]
        lj = ell[j]
        v = [sum(v[o + k] * lj[k] for k in range(d)) % R for o in range(0, len(v), d)]
    return v


def f_at_tau(pp, T):
    """f_T(tau) = sum_i T[i] L_i(tau)."""
    vals = as_flat_ints(T)
    if len(vals) != prod(pp.shape):
        raise ValueError("tensor does not match the SRS shape")
    (s,) = contract_suffix(vals, pp.shape, pp.ell, 0)
    return s


def commit(pp, T):
    """Route (c): C_T = [f_T(tau)] G, the closed form of Def. 4.1 under a known trapdoor."""
    return ec.mul(f_at_tau(pp, T), ec.G1)


# --- Algorithm 1 (App. A): divide by (x_i - v) on the lexicographic array --------
def divide_by_linear(a, shape, axis, v):
    """Return (q, r) with f = q (x_axis - v) + r and r free of x_axis (the post-condition App. A states).

    Seen along `axis`, the lexicographic array is a bundle of lines: fixing every other index leaves the
    coefficients c_0 .. c_{d-1} of a univariate polynomial in x_axis whose coefficients are monomials in the other
    variables, and dividing f by (x_axis - v) divides every line on its own.  One line, by the division of a
    univariate polynomial by a monic linear factor: the quotient's top coefficient is c_{d-1}, every lower one is
    q_{k-1} = c_k + v q_k, and what is left at degree 0 is the remainder c_0 + v q_0 = (the line's value at v)."""
    d = shape[axis]
    st = strides(shape)[axis]
    n = prod(shape)
    q = [0] * n
    r = [0] * n
    for base in range(n):
        if (base // st) % d != 0:
            continue                                  # `base` addresses degree 0 of a line; its degree k sits at base + k st
        carry = 0                                     # q_k, starting above the top degree
        for k in range(d - 1, 0, -1):
            carry = (a[base + k * st] + v * carry) % R
            q[base + (k - 1) * st] = carry
        r[base] = (a[base] + v * carry) % R
    return q, r


# --- Open (Def. 4.1), routes -----------------------------------------------------
def check_kappa(pp, kappa):
    kappa = tuple(int(k) for k in kappa)
    if len(kappa) != pp.m or any(not (0 <= k < d) for k, d in zip(kappa, pp.shape)):
        raise ValueError("opening index outside the grid")
    return kappa


def open_literal(pp, T, kappa):
    """Route (a): coefficients, Algorithm 1 for i = 1..m, pi_i over the monomial SRS."""
    kappa = check_kappa(pp, kappa)
    omega = [grid_nodes(d)[k] for d, k in zip(pp.shape, kappa)]
    rem = interpolate(T, pp.shape)
    M = pp.srs_monomial()
    proof = []
    for i in range(pp.m):
        q, rem = divide_by_linear(rem, pp.shape, i, omega[i])
        proof.append(ec.msm_naive(q, M))
    y = rem[0]
    assert all(c == 0 for c in rem[1:])
    return y, proof


def quotient_scalars(pp, T, kappa):
    """q_i(tau) for i = 1..m and y, from r_{i-1}(tau) - r_i(tau) = q_i(tau)(tau_i - omega_i).

    omega is a grid node, so r_i is the interpolant of the slice of T with its
    first i indices fixed to kappa_1..kappa_i; R_i := r_i(tau) is that slice
    contracted with the Lagrange values of the remaining axes."""
    kappa = check_kappa(pp, kappa)
    vals = as_flat_ints(T)
    if len(vals) != prod(pp.shape):
        raise ValueError("tensor does not match the SRS shape")
    st = strides(pp.shape)
    Rs = []
    offset = 0
    for i in range(pp.m + 1):
        size = prod(pp.shape[i:])
        (Ri,) = contract_suffix(vals[offset : offset + size], pp.shape, pp.ell, i) if i < pp.m else (vals[offset] % R,)
        Rs.append(Ri)
        if i < pp.m:
            offset += kappa[i] * st[i]
    qs = []
    for i in range(pp.m):
        omega_i = grid_nodes(pp.shape[i])[kappa[i]]
        qs.append((Rs[i] - Rs[i + 1]) * ec.fr_inv(pp.tau[i] - omega_i) % R)
    return Rs[pp.m], qs


def open_(pp, T, kappa):
    """Route (c): y = T[kappa], pi_i = [q_i(tau)] G."""
    y, qs = quotient_scalars(pp, T, kappa)
    return y, [ec.mul(q, ec.G1) for q in qs]


def quotient_values_on_grid(pp, T, kappa, axis):
    """Values of q_{axis+1} on the grid of axes axis..m-1 (evaluation form).

    With g(.) the line of the slice T[kappa_1..kappa_{axis}, ., k_{axis+1}..] along
    `axis`:  q(zeta_k) = (g_k - g_kappa)/(zeta_k - zeta_kappa) for k != kappa, and at
    k = kappa the value of the interpolant of those d-1 values extended to zeta_kappa,
    q(zeta_kappa) = sum_{k != kappa} (beta_k/beta_kappa) (g_k - g_kappa)/(zeta_kappa - zeta_k)
    (derivative of the interpolant in barycentric form, App. C weights)."""
    kappa = check_kappa(pp, kappa)
    vals = as_flat_ints(T)
    st = strides(pp.shape)
    offset = sum(kappa[j] * st[j] for j in range(axis))
    sub = pp.shape[axis:]
    size = prod(sub)
    sl = [v % R for v in vals[offset : offset + size]]
    d = sub[0]
    inner = size // d
    z = grid_nodes(d)
    beta = bary_weights(d)
    kap = kappa[axis]
    out = [0] * size
    for t in range(inner):
        gk = sl[kap * inner + t]
        acc = 0
        for k in range(d):
            if k == kap:
                continue
            qv = (sl[k * inner + t] - gk) * ec.fr_inv(z[k] - z[kap]) % R
            out[k * inner + t] = qv
            # (beta_k/beta_kap) (g_k - g_kap)/(zeta_kap - zeta_k) = -(beta_k/beta_kap) qv
            acc = (acc - beta[k] * ec.fr_inv(beta[kap]) % R * qv) % R
        out[kap * inner + t] = acc
    return out


def open_eval_form(pp, T, kappa):
    """Route (d): quotient values on the grid against the suffix Lagrange SRS (tiny sizes)."""
    kappa = check_kappa(pp, kappa)
    vals = as_flat_ints(T)
    proof = []
    for i in range(pp.m):
        qv = quotient_values_on_grid(pp, vals, kappa, i)
        proof.append(ec.msm_naive(qv, pp.srs_lagrange(i)))
    y = vals[flat_index(kappa, pp.shape)] % R
    return y, proof


# --- Ver (Def. 4.1, sum form, trapdoor-form check in G1) -------------------------
def verify(pp, C, kappa, y, proof):
    kappa = check_kappa(pp, kappa)
    if len(proof) != pp.m:
        return False
    lhs = ec.sub(C, ec.mul(y, ec.G1))
    rhs = ec.INF
    for i in range(pp.m):
        omega_i = grid_nodes(pp.shape[i])[kappa[i]]
        rhs = ec.add(rhs, ec.mul((pp.tau[i] - omega_i) % R, proof[i]))
    return lhs == rhs
