"""Oracle composition of CKKS bootstrapping for sparsely packed ciphertexts (test infrastructure only).

The paper names Bootstrap as the operation that refreshes the level of a ciphertext (Section 2.2) and defers
the construction to the CKKS literature; this file follows the published construction step by step with the
oracle's own primitives:

  ModRaise      the level-1 ciphertext is read as a ciphertext modulo Q_L; it decrypts to t = m + q0 I
  SubSum        trace onto the subring Z[X^(N/2ns)] (log2(n/ns) rotate-and-add steps): t' = (n/ns) t
  CoeffToSlot   slots <- coefficients: w_k = t_k + i t_(k+ns) = (1/ns) conj(U)^T Z, U[j][k] = xi_j^k,
                xi_j = exp(2 pi i 5^j / (4 ns)); one baby-step/giant-step matrix product; then the real
                and imaginary parts with one conjugation
  EvalMod       t mod q0 ~ (q0 / 2 pi) sin(2 pi t / q0): exp(i theta / 2^r) by its Taylor polynomial
                (cosine to theta^8, sine to theta^9), r squarings, imaginary part
  SlotToCoeff   Z'' = U w'' with w'' = eps_lo + i eps_hi

Every constant is folded into the two matrices; "multiply by i" is the monomial X^(N/2), which costs neither
scale nor level.  The ciphertext values are tracked as (residues, level, scale).
"""
import math

import numpy as np


def sparse_secret(o, seed: int, h: int) -> np.ndarray:
    """Ternary secret with exactly h non-zero coefficients: stream kind 11; position = low logN bits of a
    word (redrawn while the position is taken), then one more word whose low bit gives the sign (0: +1)."""
    tag = 11 << 32
    s = np.zeros(o.N, dtype=np.int8)
    i = placed = 0
    while placed < h:
        pos = o.stream_word(seed, tag, i) & (o.N - 1)
        i += 1
        if s[pos] != 0:
            continue
        s[pos] = 1 if (o.stream_word(seed, tag, i) & 1) == 0 else -1
        i += 1
        placed += 1
    return s


def modraise(o, ct: np.ndarray, level_out: int) -> np.ndarray:
    """[2][1][N] modulo q0 -> [2][level_out][N]: the centred coefficients, reduced modulo every q_i."""
    q0 = o.q[0]
    out = np.empty((2, level_out, o.N), dtype=np.uint64)
    for c in range(2):
        x = o.intt(ct[c, 0][None, :], [0])[0]
        xc = [int(v) - q0 if int(v) > (q0 - 1) // 2 else int(v) for v in x.tolist()]
        for i in range(level_out):
            limb = np.array([v % o.q[i] for v in xc], dtype=np.uint64)
            out[c, i] = o.ntt(limb[None, :], [i])[0]
    return out


def special_dft(ns: int) -> np.ndarray:
    """U[j][k] = xi_j^k, xi_j = exp(2 pi i (5^j mod 4 ns) / (4 ns))."""
    e = np.array([pow(5, j, 4 * ns) for j in range(ns)], dtype=np.float64)
    k = np.arange(ns, dtype=np.float64)
    return np.exp(2j * np.pi * np.outer(e, k) / (4 * ns))


class Plan:
    """Shapes, levels and rotation shifts of one bootstrapping for ns slots."""

    def __init__(self, o, ns: int, r: int = 8, level_in: int = None, groups: int = 1):
        """groups = 1: each matrix product is one dense ns x ns matrix.  groups >= 2: the matrices are applied
        as that many sparse factors (products of consecutive butterfly stages), one level each."""
        self.ns, self.r, self.groups = ns, r, groups
        self.L = o.L if level_in is None else level_in
        self.gap = o.n // ns
        lg = int(math.log2(ns))
        self.g1 = 1 << ((lg + 1) // 2)
        self.g2 = ns // self.g1
        self.subsum_shifts = [ns << k for k in range(int(math.log2(self.gap)))]
        self.baby = list(range(1, self.g1))
        self.giant = [self.g1 * b for b in range(1, self.g2)]
        self.out_level = self.L - 5 - r - 2 * groups
        self.factors = butterfly_groups(ns, groups) if groups > 1 else None

    def rotation_shifts(self):
        if self.groups == 1:
            return sorted(set(self.subsum_shifts + self.baby + self.giant))
        sh = set(self.subsum_shifts)
        for G in self.factors:  # a factor and its inverse have the same diagonals
            sh |= set(SparseDiagonals(G).shifts())
        sh.discard(0)
        return sorted(sh)

    def natural_factor(self, o) -> float:
        """Output scale / input scale when the last matrix carries no extra gain: the scale of exp(i theta)
        after the r squarings, over q0 (follows the rescale rule step by step)."""
        q = [float(v) for v in o.q]
        l = self.L - self.groups
        s = q[0] * q[0] / q[l - 5]
        lvl = l - 5
        for _ in range(self.r):
            s = s * s / q[lvl - 1]
            lvl -= 1
        return s / q[0]


def butterfly_stage(ns: int, ln: int) -> np.ndarray:
    """One stage of the special FFT on blocks of `ln` entries: (u, v) -> (u + D v, u - D v) with
    D_j = exp(2 pi i (5^j mod 4 ln) / (4 ln)).  U = B_ns ... B_4 B_2 R, R the bit-reversal permutation."""
    M = np.zeros((ns, ns), dtype=np.complex128)
    lh = ln // 2
    for i in range(0, ns, ln):
        for j in range(lh):
            D = np.exp(2j * np.pi * pow(5, j, 4 * ln) / (4 * ln))
            M[i + j, i + j] = 1.0
            M[i + j, i + j + lh] = D
            M[i + j + lh, i + j] = 1.0
            M[i + j + lh, i + j + lh] = -D
    return M


def butterfly_groups(ns: int, groups: int):
    """[G_1 .. G_groups], G_1 = the first stages (applied first), with U = G_groups ... G_1 R."""
    stages = [butterfly_stage(ns, 2 << s) for s in range(int(math.log2(ns)))]
    per = -(-len(stages) // groups)
    out = []
    for g in range(groups):
        M = np.eye(ns, dtype=np.complex128)
        for B in stages[g * per:(g + 1) * per]:
            M = B @ M
        out.append(M)
    return out


class SparseDiagonals:
    """Baby-step/giant-step layout for a matrix whose non-zero diagonals are d_min + stride e, e = 0 .. E
    (offsets taken in (-ns/2, ns/2]): e = g1 b + a."""

    def __init__(self, M: np.ndarray):
        ns = M.shape[0]
        j = np.arange(ns)
        offs = []
        for d in range(ns):
            if np.abs(M[j, (j + d) % ns]).max() > 1e-12:
                offs.append(d if d <= ns // 2 else d - ns)
        offs.sort()
        self.ns, self.offsets = ns, offs
        self.dmin = offs[0]
        self.stride = math.gcd(*[d - self.dmin for d in offs[1:]]) if len(offs) > 1 else 1
        self.E = (offs[-1] - self.dmin) // self.stride
        self.g1 = int(math.ceil(math.sqrt(self.E + 1)))
        self.g2 = -(-(self.E + 1) // self.g1)

    def giant_shift(self, b: int) -> int:
        return self.dmin + self.stride * self.g1 * b

    def shifts(self):
        return [self.stride * a for a in range(1, self.g1)] + [self.giant_shift(b) for b in range(self.g2)]

    def plaintext_slots(self, M: np.ndarray, n: int):
        """{(b, a): slot vector of diagonal dmin + stride (g1 b + a), rotated right by the giant shift}."""
        ns = self.ns
        j = np.arange(ns)
        out = {}
        for b in range(self.g2):
            G = self.giant_shift(b)
            for a in range(self.g1):
                d = G + self.stride * a
                if d not in self.offsets:
                    continue
                jj = (j - G) % ns
                out[(b, a)] = np.tile(M[jj, (jj + d) % ns], n // ns)
        return out


def encode_sparse(o, M: np.ndarray, level: int):
    """(layout, NTT-domain plaintexts at scale q_(level-1)) of a sparse-diagonal matrix."""
    sd = SparseDiagonals(M)
    scale = float(o.q[level - 1])
    return sd, {k: o.coeffs_to_ntt(o.encode(v, scale), level) for k, v in sd.plaintext_slots(M, o.n).items()}


def sparse_transform(o, ct, sd: SparseDiagonals, pts, rot):
    """sum_b rot_(giant b)( sum_a pt[b, a] * rot_(stride a)(ct) ), then rescale."""
    babies = {0: ct}
    for a in range(1, sd.g1):
        if any((b, a) in pts for b in range(sd.g2)):
            babies[a] = o.hrot(ct, rot[sd.stride * a], sd.stride * a)
    acc = None
    for b in range(sd.g2):
        inner = None
        for a in range(sd.g1):
            if (b, a) not in pts:
                continue
            term = o.pmult(babies[a], pts[(b, a)])
            inner = term if inner is None else o.add(inner, term)
        if inner is None:
            continue
        G = sd.giant_shift(b)
        if G % o.n:
            inner = o.hrot(inner, rot[G], G)
        acc = inner if acc is None else o.add(acc, inner)
    return o.rescale(acc)


def bsgs_plaintext_slots(M: np.ndarray, plan: Plan, n: int):
    """Slot vectors of the pre-rotated diagonals: entry [b][a][j] = M[(j - g1 b) % ns][(j + a) % ns], tiled to n."""
    ns, g1, g2 = plan.ns, plan.g1, plan.g2
    j = np.arange(ns)
    out = []
    for b in range(g2):
        row = []
        for a in range(g1):
            jj = (j - g1 * b) % ns
            d = M[jj, (jj + g1 * b + a) % ns]
            row.append(np.tile(d, n // ns))
        out.append(row)
    return out


def encode_matrix(o, M: np.ndarray, plan: Plan, level: int):
    """NTT-domain plaintexts of the pre-rotated diagonals at scale q_(level-1), `level` limbs each."""
    scale = float(o.q[level - 1])
    return [[o.coeffs_to_ntt(o.encode(v, scale), level) for v in row] for row in bsgs_plaintext_slots(M, plan, o.n)]


def linear_transform(o, ct, pts, rot, plan: Plan):
    """sum_b rot_(g1 b)( sum_a pt[b][a] * rot_a(ct) ), then rescale (level - 1, scale unchanged)."""
    babies = [ct] + [o.hrot(ct, rot[a], a) for a in plan.baby]
    acc = None
    for b in range(plan.g2):
        inner = None
        for a in range(plan.g1):
            term = o.pmult(babies[a], pts[b][a])
            inner = term if inner is None else o.add(inner, term)
        if b:
            inner = o.hrot(inner, rot[plan.g1 * b], plan.g1 * b)
        acc = inner if acc is None else o.add(acc, inner)
    return o.rescale(acc)


def monomial_i(o, level: int, sign: int = 1) -> np.ndarray:
    """NTT-domain plaintext of +-X^(N/2): multiplies every slot by +-i."""
    c = np.zeros(o.N, dtype=np.int64)
    c[o.N // 2] = sign
    return o.coeffs_to_ntt(c, level)


def _const(o, v: float, s: float, level: int):
    iv = int(round(v * s))
    return [iv % o.q[i] for i in range(level)]


def _mul(o, a, b, relin):
    return o.rescale(o.hmult_relin(a, b, relin))


def _lin(o, y, level: int, s_in: float, c0: float, c1: float, target: float):
    """rescale(c1 y) + c0 at scale `target`, one level below y."""
    q = float(o.q[level - 1])
    out = o.rescale(o.cmult(y, _const(o, c1, target * q / s_in, level)))
    return o.add_const(out, _const(o, c0, target, level - 1))


def _quartic(o, y, y2, l: int, s_y: float, s_y2: float, r, target: float, relin):
    """r0 + r1 y + r2 y^2 + r3 y^3 + r4 y^4 at level l-3 and scale `target`; y at level l, y2 = y^2 at l-1."""
    q = [float(v) for v in o.q]
    t_in = target * q[l - 3] / s_y2                    # scale of r2 + r3 y + r4 y2 so that y2 * inner lands on target
    lin23 = o.moddrop(_lin(o, y, l, s_y, r[2], r[3], t_in), l - 2)
    q4 = o.rescale(o.cmult(y2, _const(o, r[4], t_in * q[l - 2] / s_y2, l - 1)))
    inner = o.add(lin23, q4)                           # level l-2
    prod = _mul(o, o.moddrop(y2, l - 2), inner, relin)
    lin01 = o.moddrop(_lin(o, y, l, s_y, r[0], r[1], target), l - 3)
    return o.add(prod, lin01)


def exp_i(o, theta, level: int, scale: float, relin, r: int):
    """exp(i 2^r theta) for a ciphertext with real slots theta: (ct, level - 5 - r, scale)."""
    q = [float(v) for v in o.q]
    l = level
    y = _mul(o, theta, theta, relin)                    # level l-1
    s_y = scale * scale / q[l - 1]
    y2 = _mul(o, y, y, relin)                           # level l-2
    s_y2 = s_y * s_y / q[l - 2]
    cos_c = [(-1) ** k / math.factorial(2 * k) for k in range(5)]
    sin_c = [(-1) ** k / math.factorial(2 * k + 1) for k in range(5)]
    t_p = scale                                         # scale of the sine's even factor, level l-4
    t_s = scale * t_p / q[l - 5]                        # scale of theta * P and of the cosine
    P = _quartic(o, y, y2, l - 1, s_y, s_y2, sin_c, t_p, relin)
    C = _quartic(o, y, y2, l - 1, s_y, s_y2, cos_c, t_s, relin)
    S = _mul(o, o.moddrop(theta, l - 4), P, relin)      # level l-5
    E = o.add(o.moddrop(C, l - 5), o.pmult(S, monomial_i(o, l - 5)))
    lvl, s = l - 5, t_s
    for _ in range(r):
        E = _mul(o, E, E, relin)
        s = s * s / q[lvl - 1]
        lvl -= 1
    return E, lvl, s


def bootstrap(o, ct1, keys, plan: Plan, pts_cts=None, pts_stc=None, gain: float = 1.0):
    """ct1: [2][1][N] at scale delta.  keys: {'relin', 'conj', 'rot': {shift: key}}.
    Returns (ct, level, factor): the refreshed ciphertext at `level`, encrypting the same slots at scale
    delta * factor.  gain multiplies the last matrix (and the factor): with gain = target / (delta *
    natural_factor) the result lands exactly on the scale `target`."""
    L, ns, r = plan.L, plan.ns, plan.r
    relin, conj, rot = keys["relin"], keys["conj"], keys["rot"]
    g = plan.groups
    ct = modraise(o, ct1, L)
    for sh in plan.subsum_shifts:
        ct = o.add(ct, o.hrot(ct, rot[sh], sh))
    scale = float(o.q[0])                               # the raised ciphertext holds t / q0
    if g == 1:
        U = special_dft(ns)
        if pts_cts is None:
            pts_cts = encode_matrix(o, (math.pi / (plan.gap * 2.0**r * ns)) * U.conj().T, plan, L)
        w = linear_transform(o, ct, pts_cts, rot, plan)     # level L-1: (pi / 2^r) w
    else:
        # U^-1 = R^-1 G_1^-1 .. G_g^-1: the slots come out in bit-reversed order, which the slot-wise
        # middle part does not see and the way back (G_g .. G_1, without R) undoes
        if pts_cts is None:
            c = (math.pi / (plan.gap * 2.0**r)) ** (1.0 / g)
            pts_cts = [encode_sparse(o, c * np.linalg.inv(plan.factors[i]), L - (g - 1 - i)) for i in range(g)]
        w = ct
        for i in reversed(range(g)):
            w = sparse_transform(o, w, pts_cts[i][0], pts_cts[i][1], rot)
    lt = L - g
    wc = o.hconj(w, conj)
    th1 = o.add(w, wc)
    th2 = o.pmult(o.sub(w, wc), monomial_i(o, lt, -1))
    E1, lvl, s = exp_i(o, th1, lt, scale, relin, r)
    E2, _, _ = exp_i(o, th2, lt, scale, relin, r)
    iE2 = o.pmult(E2, monomial_i(o, lvl))
    Hp, Hm = o.add(E1, iE2), o.sub(E1, iE2)
    F = o.pmult(o.sub(Hp, o.hconj(Hm, conj)), monomial_i(o, lvl, -1))
    if g == 1:
        if pts_stc is None:
            pts_stc = encode_matrix(o, (gain / (4.0 * math.pi)) * special_dft(ns), plan, lvl)
        out = linear_transform(o, F, pts_stc, rot, plan)
    else:
        if pts_stc is None:
            c = (gain / (4.0 * math.pi)) ** (1.0 / g)
            pts_stc = [encode_sparse(o, c * plan.factors[i], lvl - i) for i in range(g)]
        out = F
        for i in range(g):
            out = sparse_transform(o, out, pts_stc[i][0], pts_stc[i][1], rot)
    return out, lvl - g, gain * s / float(o.q[0])
