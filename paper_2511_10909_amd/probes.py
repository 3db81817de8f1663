"""Closed-loop feature probing, Steps 1 to 3 (paper Sec. 3.1), against any MMA interface.

An *interface* is a callable `f(A, B, C) -> D` on batches of tiles given as numpy arrays of raw bit
patterns (`A[batch][m][k]`, `B[batch][n][k]`, `C/D[batch][m][n]`) with attributes `m, n, k, ta, tb`.
`hardware(instr)` wraps one native MFMA instruction (through `mmaemu_mfma_probe`), `model(...)` a
parameterised model (through `mmaemu_emulate_mma`); tests drive the same probes with the CPU oracle.

  Step 1  independence(iface)                    all d_ij bitwise identical for replicated rows / columns
  Step 2  summation_table(iface)                 d^(i,j) / v for p_i = U, p_j = -U, every other summand v
          infer_tree(table)                      summation tree realisation, telling swamped from
                                                 non-swamped n-term fused sums
  Step 3  fused_precision / rounding_mode        FusedSum(U, -U, eps) with eps halved; U + {0.5, 1.5, 1, 3} eps

Everything here is host logic on a few hundred tiles: input construction, reading results back and the tree
algorithm.  The arithmetic under test runs in the interface.
"""
import numpy as np

E4M3, E5M2, FP16, BF16, FP32 = range(5)          # the library's dtype ids
_FMT = {E4M3: (4, 3, 7), E5M2: (5, 2, 15), FP16: (5, 10, 15), BF16: (8, 7, 127), FP32: (8, 23, 127)}   # ebits, mbits, bias
_NP = {E4M3: np.uint8, E5M2: np.uint8, FP16: np.uint16, BF16: np.uint16, FP32: np.uint32}


def encode(t, sign, sig, exp2):
    """Bit pattern of (-1)^sign * sig * 2^exp2 in format t (sig a positive integer; the value must be exactly
    representable, normal or subnormal, else ValueError).  sig = 0 gives a signed zero."""
    eb, mb, bias = _FMT[t]
    if sig == 0:
        return sign << (eb + mb)
    while sig % 2 == 0:
        sig //= 2
        exp2 += 1
    top = sig.bit_length() - 1 + exp2                 # exponent of the leading bit
    emin = 1 - bias
    emax = (1 << eb) - 2 - bias if t != E4M3 else 8   # OCP E4M3 uses the top exponent for finite values
    if top > emax:
        raise ValueError("too large for the format")
    if top >= emin:
        shift = mb - (sig.bit_length() - 1)
        if shift < 0:
            raise ValueError("too many significant bits")
        man = (sig << shift) & ((1 << mb) - 1)
        code = ((top + bias) << mb) | man
    else:
        shift = exp2 - (emin - mb)
        if shift < 0:
            raise ValueError("below the subnormal grid")
        man = sig << shift
        if man >= (1 << mb):
            raise ValueError("internal: subnormal overflow")
        code = man
    if t == E4M3 and (code & 0x7F) == 0x7F:
        raise ValueError("that E4M3 pattern is NaN")
    return (sign << (eb + mb)) | code


def decode_fp32(bits):
    return float(np.array([bits], dtype=np.uint32).view(np.float32)[0])


def exponent_range(t):
    """(lowest, highest) power of two that format t holds exactly."""
    eb, mb, bias = _FMT[t]
    return 1 - bias - mb, ((1 << eb) - 2 - bias if t != E4M3 else 8)


class Summands:
    """Builds the K + 1 summands p_0 .. p_K of one dot-product-accumulate (p_K is the accumulator) from
    requested values sign * sig * 2^e: a product p_k = a_k b_k puts the significand and sign into a_k and splits
    the exponent between a_k and b_k so that both are representable."""

    def __init__(self, iface):
        self.k, self.ta, self.tb = iface.k, iface.ta, iface.tb

    def product(self, sign, sig, e):
        if sig == 0:
            return encode(self.ta, 0, 0, 0), encode(self.tb, 0, 0, 0)
        lo_b, hi_b = exponent_range(self.tb)
        for eb_ in sorted(range(lo_b, hi_b + 1), key=lambda x: abs(x - e // 2)):
            try:
                return encode(self.ta, sign, sig, e - eb_), encode(self.tb, 0, 1, eb_)
            except ValueError:
                continue
        raise ValueError("summand %d * 2^%d does not fit a product of these formats" % (sig, e))

    def row(self, values):
        """values: K + 1 triples (sign, sig, e).  Returns (a[K], b[K], c)."""
        assert len(values) == self.k + 1
        ab = [self.product(*v) for v in values[:-1]]
        s, sig, e = values[-1]
        return [x for x, _ in ab], [y for _, y in ab], encode(FP32, s, sig, e)

    def max_gap(self):
        """Largest e_u - e_v available to products of the two formats (with e_u even-split friendly)."""
        la, ha = exponent_range(self.ta)
        lb, hb = exponent_range(self.tb)
        return (ha + hb) - (la + lb)

    def default_exponents(self, gap):
        la, ha = exponent_range(self.ta)
        lb, hb = exponent_range(self.tb)
        if gap > (ha + hb) - (la + lb):
            raise ValueError("the formats cannot hold two products 2^%d apart" % gap)
        mid = (ha + hb + la + lb) // 2
        e_u = min(ha + hb, mid + (gap + 1) // 2)
        return e_u, e_u - gap


def run_rows(iface, rows):
    """Evaluates one dot-product-accumulate per row description (a[K], b[K], c): each goes to element (0, 0) of
    a tile of its own, the rest of the tile is zero.  Returns the list of d (FP32 bit patterns)."""
    nb = len(rows)
    A = np.zeros((nb, iface.m, iface.k), dtype=_NP[iface.ta])
    B = np.zeros((nb, iface.n, iface.k), dtype=_NP[iface.tb])
    C = np.zeros((nb, iface.m, iface.n), dtype=np.uint32)
    for t, (a, b, c) in enumerate(rows):
        A[t, 0, :] = a
        B[t, 0, :] = b
        C[t, 0, 0] = c
    D = iface(A, B, C)
    return [int(D[t, 0, 0]) for t in range(nb)]


# ---------------------------------------------------------------------------------------- Step 1
def independence(iface, trials=32, seed=0):
    """Sec. 3.1 Step 1: 2K + 1 random numbers a_0k, b_k0, c_00 replicated over all rows / columns; the MMA is a set
    of independent dot-product-accumulates iff all d_ij of a tile are bitwise identical.  Returns True / False."""
    rng = np.random.default_rng(seed)

    def finite(t, shape):
        eb, mb, _ = _FMT[t]
        x = rng.integers(0, 1 << (eb + mb + 1), size=shape, dtype=np.uint64).astype(_NP[t])
        emask = ((1 << eb) - 1) << mb
        if t == E4M3:
            bad = (x & 0x7F) == 0x7F
        else:
            bad = (x & emask) == emask
        return np.where(bad, x & ~np.array(1 << mb, dtype=_NP[t]), x).astype(_NP[t])     # clear one exponent bit: finite

    a = finite(iface.ta, (trials, 1, iface.k))
    b = finite(iface.tb, (trials, 1, iface.k))
    c = finite(FP32, (trials, 1, 1))
    A = np.repeat(a, iface.m, axis=1)
    B = np.repeat(b, iface.n, axis=1)
    C = np.repeat(np.repeat(c, iface.m, axis=1), iface.n, axis=2)
    D = iface(A, B, C)
    return bool((D == D[:, :1, :1]).all())


# ---------------------------------------------------------------------------------------- Step 2
def summation_table(iface, gap=None):
    """Sec. 3.1 Step 2: for every 0 <= i < j <= K the output d^(i,j) / v with p_i = U = 2^e_u, p_j = -U and every
    other summand v = 2^e_v, where (K - 1) v +- U = +-U in binary32.  Returns a (K+1) x (K+1) list of lists with
    the entries for i < j (None elsewhere)."""
    K = iface.k
    sm = Summands(iface)
    need = 25 + max(K - 1, 1).bit_length()
    if gap is None:
        gap = min(sm.max_gap(), need + 2)
    if gap < need:
        raise ValueError("formats too narrow for K = %d: need U / v >= 2^%d" % (K, need))
    e_u, e_v = sm.default_exponents(gap)
    pairs = [(i, j) for i in range(K + 1) for j in range(i + 1, K + 1)]
    rows = []
    for i, j in pairs:
        vals = [(0, 1, e_v)] * (K + 1)
        vals[i] = (0, 1, e_u)
        vals[j] = (1, 1, e_u)
        rows.append(sm.row(vals))
    out = run_rows(iface, rows)
    table = [[None] * (K + 1) for _ in range(K + 1)]
    v = 2.0 ** e_v
    for (i, j), d in zip(pairs, out):
        q = decode_fp32(d) / v
        if q != int(q) or not (0 <= q <= K):
            raise ValueError("d^(%d,%d) / v = %r is not a count: the U / v construction does not fit this interface" % (i, j, q))
        table[i][j] = int(q)
    return table


def table_from_tree(tree, n):
    """The d^(i,j) / v table a summation tree predicts (inverse of infer_tree; used by tests and to check a result).
    tree: ("leaf", k) or ("sum", swamped, [children])."""
    def leaves(t):
        return [t[1]] if t[0] == "leaf" else [x for ch in t[2] for x in leaves(ch)]
    table = [[None] * n for _ in range(n)]

    def walk(t):
        if t[0] == "leaf":
            return
        groups = [leaves(ch) for ch in t[2]]
        size = sum(len(g) for g in groups)
        for x in range(len(groups)):
            for y in range(x + 1, len(groups)):
                inner = 0 if t[1] else size - len(groups[x]) - len(groups[y])
                for i in groups[x]:
                    for j in groups[y]:
                        table[min(i, j)][max(i, j)] = (n - size) + inner
        for ch in t[2]:
            walk(ch)
    walk(tree)
    return table


def infer_tree(table):
    """Tree realisation (Sec. 3.1 Step 2, extended to tell swamped from non-swamped fused sums).  Top-down: for a
    node with leaf set S (n leaves in all), every pair inside S keeps the n - |S| summands outside S; of those
    inside, a pair whose lowest common parent is this node keeps none if the node swamps its small summands and
    |S| - |X| - |Y| (X, Y the children holding the pair) if it does not, while a pair inside one child X keeps at
    least |S| - |X|.  Returns ("leaf", k) / ("sum", kind, [children]), kind True: swamped fused sum, False:
    non-swamped fused sum, None: binary sum (where the two cannot differ).  The result always reproduces the table;
    where a non-swamped fused sum admits several groupings with the same table, the first one found is returned."""
    n = len(table)

    def s(i, j):
        v = table[min(i, j)][max(i, j)]
        if v is None:
            raise ValueError("table entry (%d, %d) missing" % (min(i, j), max(i, j)))
        return v

    def build(S):
        if len(S) == 1:
            return ("leaf", S[0])
        size = len(S)
        r = {(i, j): s(i, j) - (n - size) for i in S for j in S if i != j}
        if min(r.values()) < 0:
            raise ValueError("no summation tree fits the table (fewer survivors than summands outside %s)" % (S,))
        # children under the swamped / binary hypothesis: pairs that keep something inside S share a child
        comp = {i: i for i in S}

        def find(x):
            while comp[x] != x:
                comp[x] = comp[comp[x]]
                x = comp[x]
            return x
        for (i, j), v in r.items():
            if v > 0:
                comp[find(i)] = find(j)
        groups = {}
        for i in S:
            groups.setdefault(find(i), []).append(i)
        parts = sorted(groups.values(), key=min)
        if len(parts) >= 2:
            kind = None if len(parts) == 2 else True
        else:
            # one component: a non-swamped fused sum of three or more children.  For leaf i in child X the pairs
            # inside X keep at least |S| - |X| and every other pair of i exactly |S| - |X| - |child of the other|,
            # which is less.  The size of X is not known in advance: candidates are tried in increasing order and a
            # choice is kept only if it is consistent with the children found so far.
            def consistent(parts_):
                for a in range(len(parts_)):
                    if any(r[(i, j)] < size - len(parts_[a]) for i in parts_[a] for j in parts_[a] if i != j):
                        return False
                    for b in range(a + 1, len(parts_)):
                        want = size - len(parts_[a]) - len(parts_[b])
                        if any(r[(i, j)] != want for i in parts_[a] for j in parts_[b]):
                            return False
                return True

            def partition(done, rest):
                if not rest:
                    return done if len(done) >= 3 else None
                i = rest[0]
                for x in range(1, len(rest) + 1):
                    same = [j for j in rest[1:] if r[(i, j)] >= size - x]
                    if len(same) != x - 1 or any(r[(i, j)] >= size - x for p_ in done for j in p_):
                        continue
                    cand = done + [[i] + same]
                    if not consistent(cand):
                        continue
                    got = partition(cand, [j for j in rest[1:] if j not in same])
                    if got is not None:
                        return got
                return None
            parts = partition([], sorted(S))
            if parts is None:
                raise ValueError("no summation tree fits the table (children of %s)" % (S,))
            kind = False
        return ("sum", kind, [build(p_) for p_ in parts])

    tree = build(list(range(n)))
    if table_from_tree(tree, n) != [[table[i][j] if j > i else None for j in range(n)] for i in range(n)]:
        raise ValueError("no summation tree fits the table")
    return tree


def tree_to_string(tree, names=None):
    """Compact text form: leaves as p<k> (or names[k]); binary sums '( + )', fused sums 'F[ , , ]' when they swamp
    their small summands and 'Fx[ , , ]' when they do not."""
    if tree[0] == "leaf":
        return names[tree[1]] if names else "p%d" % tree[1]
    kids = [tree_to_string(ch, names) for ch in tree[2]]
    if tree[1] is None:
        return "(" + " + ".join(kids) + ")"
    return ("F[" if tree[1] else "Fx[") + ", ".join(kids) + "]"


# ---------------------------------------------------------------------------------------- Step 3
def fused_precision(iface, i, j, k, e_u=None, max_bits=60):
    """Sec. 3.1 Step 3, FusedSum(U, -U, eps): p_i = U, p_j = -U, p_k = eps with eps halved from U down; returns the
    number of fractional bits e_u - log2(eps_first_lost) - 1 below which eps is lost, or None if eps survives down to
    the smallest value the summand can hold (an exact sum as far as this probe can see)."""
    K = iface.k
    sm = Summands(iface)
    if e_u is None:
        la, ha = exponent_range(iface.ta)
        lb, hb = exponent_range(iface.tb)
        e_u = min(ha + hb, 100)
    rows, es = [], []
    for t in range(0, max_bits + 1):
        vals = [(0, 0, 0)] * (K + 1)
        vals[i] = (0, 1, e_u)
        vals[j] = (1, 1, e_u)
        try:
            vals[k] = (0, 1, e_u - t)
            rows.append(sm.row(vals))
            es.append(e_u - t)
        except ValueError:
            break
    out = run_rows(iface, rows)
    for e, d in zip(es, out):
        if decode_fp32(d) != 2.0 ** e:
            return e_u - e - 1
    return None


def rounding_mode(iface, i, k, frac_bits, e_u=None):
    """Sec. 3.1 Step 3, rounding mode of a sum that keeps `frac_bits` fractional bits below U: with
    eps = U 2^-(frac_bits+1) the four inputs +-U +- {0.5, 1.5} * 2 eps ... are read off as in the paper: the outputs of
    U + 1.5 q, U + 0.5 q, -U - 1.5 q, -U - 0.5 q (q = the last kept place) tell RU / RD / RZ / RA / RN apart, and for
    RN the ties U + {1, 3} q / 2 ... tell the tie rule.  p_i carries +-U, p_k the small part; others are zero.
    Returns one of "RU", "RD", "RZ", "RA", "RNE", "RNO", "RNU", "RND", "RNZ", "RNA", or "composite xxxx" (A: went away
    from zero, Z: toward zero, for +0.75, +0.25, -0.75, -0.25 of a last place) when no single mode fits.  What is seen is the
    composite of every rounding between the summands and the output (an alignment that truncates one place below
    a round-to-nearest conversion reads as "RZ" here), exactly as it is for the paper's probe."""
    K = iface.k
    sm = Summands(iface)
    if e_u is None:
        la, ha = exponent_range(iface.ta)
        lb, hb = exponent_range(iface.tb)
        e_u = min(ha + hb, 100)
    q = e_u - frac_bits                     # exponent of the last kept place

    def case(sign, sig, e):                 # +-(U + sig 2^e)
        vals = [(0, 0, 0)] * (K + 1)
        vals[i] = (sign, 1, e_u)
        vals[k] = (sign, sig, e)
        return sm.row(vals)
    # quarter steps of the last kept place: 1.5 q -> 3 * 2^(q-1), 0.5 q -> 2^(q-1); ties: q/2 ... expressed on the
    # grid of half places: values U + {1, 3} * 2^(q-1) are the two ties between multiples of q
    rows = [case(0, 3, q - 2), case(0, 1, q - 2), case(1, 3, q - 2), case(1, 1, q - 2),      # +-(U + {0.75, 0.25} q)
            case(0, 1, q - 1), case(0, 3, q - 1), case(1, 1, q - 1), case(1, 3, q - 1)]      # +-(U + {0.5, 1.5} q): ties
    out = [decode_fp32(d) for d in run_rows(iface, rows)]
    U, Q = 2.0 ** e_u, 2.0 ** q
    up = [out[0] == U + Q, out[1] == U + Q, out[2] == -U - Q, out[3] == -U - Q]             # rounded away from zero?
    for got, lo in zip(out[:4], (U, U, -U, -U)):
        if got not in (lo, lo + (Q if lo > 0 else -Q)):
            raise ValueError("the sum does not round at 2^%d: got %r next to %r" % (q, got, lo))
    if up == [True, True, False, False]:
        return "RU"
    if up == [False, False, True, True]:
        return "RD"
    if up == [False, False, False, False]:
        return "RZ"
    if up == [True, True, True, True]:
        return "RA"
    if up != [True, False, True, False]:
        # not one rounding but several in a row (e.g. an alignment rounded down one place below a round-to-nearest
        # conversion): report what was seen, in the order +0.75, +0.25, -0.75, -0.25 of a last place
        return "composite " + "".join("A" if x else "Z" for x in up)
    # round to nearest: ties U + 0.5 q (neighbours U [even], U + q [odd]) and U + 1.5 q (neighbours U + q [odd], U + 2q [even])
    t = [out[4] == U + Q, out[5] == U + 2 * Q, out[6] == -U - Q, out[7] == -U - 2 * Q]      # tie went away from zero?
    return {(False, True, False, True): "RNE", (True, False, True, False): "RNO", (True, True, False, False): "RNU",
            (False, False, True, True): "RND", (False, False, False, False): "RNZ", (True, True, True, True): "RNA"}[tuple(t)]


# ---------------------------------------------------------------------------------------- interfaces on the library
class _LibraryInterface:
    def __init__(self, m, n, k, ta, tb):
        self.m, self.n, self.k, self.ta, self.tb = m, n, k, ta, tb

    def _run(self, dA, dB, dC, dD, nb):
        raise NotImplementedError

    def __call__(self, A, B, C):
        import torch
        tdt = {1: torch.uint8, 2: torch.int16, 4: torch.int32}
        nb = A.shape[0]
        dev = "cuda"
        dA = torch.from_numpy(np.ascontiguousarray(A).view({1: np.uint8, 2: np.int16, 4: np.int32}[A.dtype.itemsize])).to(dev)
        dB = torch.from_numpy(np.ascontiguousarray(B).view({1: np.uint8, 2: np.int16, 4: np.int32}[B.dtype.itemsize])).to(dev)
        dC = torch.from_numpy(np.ascontiguousarray(C).view(np.int32)).to(dev)
        dD = torch.empty_like(dC)
        self._run(dA, dB, dC, dD, nb)
        return dD.cpu().numpy().view(np.uint32)


def hardware(instr):
    """The native instruction `instr` (an MFMA_* id of the binding), one issue per tile."""
    from . import binding as mm
    info = mm.mfma_info(instr)

    class H(_LibraryInterface):
        def _run(self, dA, dB, dC, dD, nb):
            mm.mfma_probe(instr, dA, dB, dC, dD, self.k, nb)
    return H(info["m"], info["n"], info["k"], info["a"], info["b"])


def hardware_scaled(instr, scale_a=127, scale_b=127):
    """The block-scaled native instruction `instr` (an MFMA_SCALE_* id) with every E8M0 scale of A set to the code
    `scale_a` and of B to `scale_b` (127 = 2^0): the same probes then read its summation structure."""
    import torch
    from . import binding as mm
    info = mm.mfma_info(instr)

    class H(_LibraryInterface):
        def _run(self, dA, dB, dC, dD, nb):
            sa = torch.full((nb * self.m * (self.k // 32),), scale_a, dtype=torch.uint8, device=dA.device)
            sb = torch.full((nb * self.n * (self.k // 32),), scale_b, dtype=torch.uint8, device=dA.device)
            mm.mfma_probe_scaled(instr, dA, dB, dC, dD, sa, sb, self.k, nb)
    return H(info["m"], info["n"], info["k"], info["a"], info["b"])


def model_scaled(model_kwargs, m, n, k, ta, tb, scale_a=127, scale_b=127, block=32):
    """A parameterised model on m x n x k tiles with every E8M0 block scale of A set to `scale_a`, of B to `scale_b`."""
    import torch
    from . import binding as mm

    class M(_LibraryInterface):
        def _run(self, dA, dB, dC, dD, nb):
            sa = torch.full((nb * self.m * (self.k // block),), scale_a, dtype=torch.uint8, device=dA.device)
            sb = torch.full((nb * self.n * (self.k // block),), scale_b, dtype=torch.uint8, device=dA.device)
            h = mm.model_create(**model_kwargs)
            try:
                mm.emulate_mma_scaled(h, dA, dB, dC, dD, sa, sb, block, self.m, self.n, self.k, nb, (self.ta, self.tb, mm.FP32, mm.FP32))
            finally:
                mm.model_destroy(h)
    return M(m, n, k, ta, tb)


def model(model_kwargs, m, n, k, ta, tb):
    """A parameterised model evaluated by the library on m x n x k tiles."""
    from . import binding as mm

    class M(_LibraryInterface):
        def _run(self, dA, dB, dC, dD, nb):
            h = mm.model_create(**model_kwargs)
            try:
                mm.emulate_mma(h, dA, dB, dC, dD, self.m, self.n, self.k, nb, (self.ta, self.tb, mm.FP32, mm.FP32))
            finally:
                mm.model_destroy(h)
    return M(m, n, k, ta, tb)
