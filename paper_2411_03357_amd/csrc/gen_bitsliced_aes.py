#!/usr/bin/env python3
"""Generates pgcm_bitsliced_gen.h: straight-line code for a bitsliced AES round on gfx950.

Used by the bitsliced counter-mode kernel (pgcm_bitsliced.hip), which exists to MEASURE what an
AES round function without table lookups costs on this chip, beside the table-driven path that
the library's batch calls use.  In the bitsliced form a 32-bit register holds one bit position
of one state byte for 32 independent blocks, so every instruction works on 32 blocks at once
and the S-box becomes a Boolean circuit.

The circuit is derived here from the definition (FIPS-197 5.1.1: inverse in GF(2^8) modulo
x^8 + x^4 + x^3 + x + 1, then the affine map), by the standard route for hardware S-boxes:
  * GF(2^8) is rewritten as a tower GF(((2^2)^2)^2); inversion there needs three multiplications
    and one inversion in GF(2^4), which in turn need three multiplications each in GF(2^2)
    (Karatsuba), 36 AND gates in all; everything else is linear over GF(2);
  * the linear parts (change of basis into the tower, squarings and scalings, change of basis
    back merged with the affine map) are kept as sets of terms to XOR until the very end and
    then shared greedily (the most frequent pair of terms first);
  * the two-input gates are finally packed into the chip's three-input bitwise instruction
    (v_bitop3_b32: any Boolean function of three registers), a gate with its only consumer.
Every candidate tower (the constants of the two extensions, the root that fixes the isomorphism)
is tried and the cheapest circuit kept.  The result is checked against the S-box computed from
the definition for all 256 inputs before anything is written.

MixColumns with AddRoundKey is generated the same way (sets of terms, shared pairs, packing).

  python gen_bitsliced_aes.py            writes pgcm_bitsliced_gen.h beside this file
  python gen_bitsliced_aes.py --check    regenerates in memory and compares with the file
"""
import itertools
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
OUT = os.path.join(HERE, "pgcm_bitsliced_gen.h")


# ---------------------------------------------------------------------------------------------
# the definition: GF(2^8) mod 0x11B, the S-box

def gf256_mul(a, b):
    p = 0
    for _ in range(8):
        if b & 1:
            p ^= a
        b >>= 1
        a <<= 1
        if a & 0x100:
            a ^= 0x11B
    return p


def gf256_inv(a):
    if a == 0:
        return 0
    r = 1
    for _ in range(254):
        r = gf256_mul(r, a)
    return r


def sbox_value(x):
    b = gf256_inv(x)
    r = 0
    for i in range(8):
        bit = ((b >> i) ^ (b >> ((i + 4) % 8)) ^ (b >> ((i + 5) % 8)) ^ (b >> ((i + 6) % 8)) ^
               (b >> ((i + 7) % 8)) ^ (0x63 >> i)) & 1
        r |= bit << i
    return r


# ---------------------------------------------------------------------------------------------
# signals: a signal is (frozenset of atoms, constant); an atom is an input bit or an AND gate

class Builder:
    def __init__(self, ninputs):
        self.ninputs = ninputs
        self.ands = []                     # atom ninputs + k = AND(self.ands[k][0], self.ands[k][1])
        self.and_index = {}

    def inp(self, i):
        return (frozenset([i]), 0)

    @staticmethod
    def zero():
        return (frozenset(), 0)

    @staticmethod
    def xor(a, b):
        return (a[0] ^ b[0], a[1] ^ b[1])

    def and_(self, a, b):
        if not a[0] and not a[1] or not b[0] and not b[1]:
            return self.zero()
        # constants inside AND operands do not occur in this construction
        assert a[1] == 0 and b[1] == 0
        key = frozenset([a[0], b[0]])
        if key not in self.and_index:
            self.and_index[key] = self.ninputs + len(self.ands)
            self.ands.append((a[0], b[0]))
        return (frozenset([self.and_index[key]]), 0)


class Tower:
    """GF(((2^2)^2)^2): GF(4) = {a1 w + a0, w^2 = w + 1}; GF(16) = GF(4)[v]/(v^2 + v + N);
    GF(256) = GF(16)[y]/(y^2 + y + L).  Works on ints (bits as 0/1) or on Builder signals."""

    def __init__(self, n_const, l_const, ops):
        self.N, self.L, self.o = n_const, l_const, ops     # N: 2-bit, L: 4-bit constants

    # --- GF(4): pairs (a0, a1)
    def mul4(self, a, b):
        o = self.o
        m0, m1 = o.and_(a[0], b[0]), o.and_(a[1], b[1])
        m2 = o.and_(o.xor(a[0], a[1]), o.xor(b[0], b[1]))
        return (o.xor(m1, m0), o.xor(m2, m0))

    def sq4(self, a):
        return (self.o.xor(a[0], a[1]), a[1])

    def scale4(self, a, c):
        """a times the constant c (2 bits)"""
        o = self.o
        r = (o.zero(), o.zero())
        if c & 1:
            r = (o.xor(r[0], a[0]), o.xor(r[1], a[1]))
        if c & 2:   # times w: (a1 w + a0) w = (a1 + a0) w + a1
            r = (o.xor(r[0], a[1]), o.xor(r[1], o.xor(a[0], a[1])))
        return r

    def add4(self, a, b):
        return (self.o.xor(a[0], b[0]), self.o.xor(a[1], b[1]))

    # --- GF(16): pairs (A0, A1) of GF(4) elements
    def mul16(self, a, b):
        m0, m1 = self.mul4(a[0], b[0]), self.mul4(a[1], b[1])
        m2 = self.mul4(self.add4(a[0], a[1]), self.add4(b[0], b[1]))
        return (self.add4(self.scale4(m1, self.N), m0), self.add4(m2, m0))

    def sq16(self, a):
        # (A1 v + A0)^2 = A1^2 v^2 + A0^2 = A1^2 v + (A1^2 N + A0^2)
        s0, s1 = self.sq4(a[0]), self.sq4(a[1])
        return (self.add4(self.scale4(s1, self.N), s0), s1)

    def scale16(self, a, c):
        """a times the constant c (4 bits: c0 + c1 v, each 2 bits)"""
        c0, c1 = c & 3, c >> 2
        # (A1 v + A0)(c1 v + c0) = A1 c1 (v + N) + (A1 c0 + A0 c1) v + A0 c0
        a1c1 = self.scale4(a[1], c1)
        lo = self.add4(self.scale4(a1c1, self.N), self.scale4(a[0], c0))
        hi = self.add4(a1c1, self.add4(self.scale4(a[1], c0), self.scale4(a[0], c1)))
        return (lo, hi)

    def add16(self, a, b):
        return (self.add4(a[0], b[0]), self.add4(a[1], b[1]))

    def inv16(self, a):
        d = self.add4(self.add4(self.scale4(self.sq4(a[1]), self.N), self.mul4(a[1], a[0])),
                      self.sq4(a[0]))
        di = self.sq4(d)                              # the inverse in GF(4) is the square
        return (self.mul4(self.add4(a[0], a[1]), di), self.mul4(a[1], di))

    # --- GF(256): pairs (a0, a1) of GF(16) elements
    def mul256(self, a, b):
        m0, m1 = self.mul16(a[0], b[0]), self.mul16(a[1], b[1])
        m2 = self.mul16(self.add16(a[0], a[1]), self.add16(b[0], b[1]))
        return (self.add16(self.scale16(m1, self.L), m0), self.add16(m2, m0))

    def inv256(self, a):
        d = self.add16(self.add16(self.scale16(self.sq16(a[1]), self.L), self.mul16(a[1], a[0])),
                       self.sq16(a[0]))
        di = self.inv16(d)
        return (self.mul16(self.add16(a[0], a[1]), di), self.mul16(a[1], di))


class IntOps:
    @staticmethod
    def zero():
        return 0

    @staticmethod
    def xor(a, b):
        return a ^ b

    @staticmethod
    def and_(a, b):
        return a & b


def to_bits(x):
    b = [(x >> i) & 1 for i in range(8)]
    return (((b[0], b[1]), (b[2], b[3])), ((b[4], b[5]), (b[6], b[7])))


def from_bits(e):
    flat = [e[0][0][0], e[0][0][1], e[0][1][0], e[0][1][1], e[1][0][0], e[1][0][1], e[1][1][0],
            e[1][1][1]]
    return sum(int(b) << i for i, b in enumerate(flat))


def towers():
    """every (N, L, root) for which the tower is a field isomorphic to GF(2^8) mod 0x11B, with
    the 8x8 matrices (as lists of row masks) into and out of the tower representation"""
    for n_const in (1, 2, 3):
        for l_const in range(1, 16):
            t = Tower(n_const, l_const, IntOps)
            mul = lambda x, y: from_bits(t.mul256(to_bits(x), to_bits(y)))
            # a field: every non-zero element has an inverse (checked through the formula)
            one = 1
            ok = all(mul(x, from_bits(t.inv256(to_bits(x)))) == one for x in range(1, 256))
            if not ok:
                continue
            for root in range(2, 256):
                # root must satisfy x^8 + x^4 + x^3 + x + 1 = 0 in the tower field
                p = [1]
                for _ in range(8):
                    p.append(mul(p[-1], root))
                if p[8] ^ p[4] ^ p[3] ^ p[1] ^ p[0] != 0:
                    continue
                # AES element sum x_i X^i  ->  sum x_i root^i
                into = p[:8]                               # column i: image of X^i
                image = {}
                for x in range(256):
                    y = 0
                    for i in range(8):
                        if (x >> i) & 1:
                            y ^= into[i]
                    image[x] = y
                if len(set(image.values())) != 256:
                    continue
                back = {v: k for k, v in image.items()}
                out_cols = [back[1 << i] for i in range(8)]   # tower bit i -> AES byte
                yield n_const, l_const, root, into, out_cols


def sbox_signals(n_const, l_const, into, out_cols):
    """the S-box as eight output signals over eight input bits (bit i of the byte = input i)"""
    b = Builder(8)
    x = [b.inp(i) for i in range(8)]
    # into the tower: tower bit j = XOR of x_i with bit j of into[i] set
    tb = []
    for j in range(8):
        s = b.zero()
        for i in range(8):
            if (into[i] >> j) & 1:
                s = b.xor(s, x[i])
        tb.append(s)
    elem = (((tb[0], tb[1]), (tb[2], tb[3])), ((tb[4], tb[5]), (tb[6], tb[7])))
    inv = Tower(n_const, l_const, b).inv256(elem)
    flat = [inv[0][0][0], inv[0][0][1], inv[0][1][0], inv[0][1][1], inv[1][0][0], inv[1][0][1],
            inv[1][1][0], inv[1][1][1]]
    # back to the AES basis: byte bit k = XOR of tower bits j with bit k of out_cols[j] set
    aes = []
    for k in range(8):
        s = b.zero()
        for j in range(8):
            if (out_cols[j] >> k) & 1:
                s = b.xor(s, flat[j])
        aes.append(s)
    # affine map
    outs = []
    for i in range(8):
        s = aes[i]
        for d in (4, 5, 6, 7):
            s = b.xor(s, aes[(i + d) % 8])
        if (0x63 >> i) & 1:
            s = (s[0], s[1] ^ 1)
        outs.append(s)
    return b, outs


# ---------------------------------------------------------------------------------------------
# from sets of terms to two-input gates (shared pairs), then to three-input instructions

def share_pairs(targets, min_share=2):
    """targets: list of frozensets of atom ids.  Returns (gates, names): gates is a list of
    (new id, a, b) XORs in creation order; names[k] is the id that carries targets[k] (None for
    an empty set).  Greedy: the pair of ids that occurs in most targets becomes a gate."""
    sets = [set(t) for t in targets]
    next_id = [max([max(t) for t in targets if t] + [0]) + 1000]
    gates = []
    chain_heads = set()
    while True:
        count = {}
        for s in sets:
            if len(s) < 2:
                continue
            for p in itertools.combinations(sorted(s), 2):
                count[p] = count.get(p, 0) + 1
        if not count:
            break
        best, times = max(count.items(), key=lambda e: (e[1], -e[0][0], -e[0][1]))
        if times < min_share:
            # nothing left worth sharing: finish every set as a chain ((a ^ b) ^ c) ^ d .., the
            # shape that packs two XORs into every three-input instruction
            for s in sets:
                while len(s) >= 2:
                    a, b = sorted(s)[:2] if not (s & chain_heads) else (
                        sorted(s & chain_heads)[0], sorted(s - (s & chain_heads))[0])
                    nid = next_id[0]
                    next_id[0] += 1
                    gates.append((nid, a, b))
                    s.discard(a)
                    s.discard(b)
                    s.add(nid)
                    chain_heads.add(nid)
            break
        nid = next_id[0]
        next_id[0] += 1
        gates.append((nid, best[0], best[1]))
        for s in sets:
            if best[0] in s and best[1] in s:
                s.discard(best[0])
                s.discard(best[1])
                s.add(nid)
    names = [next(iter(s)) if s else None for s in sets]
    return gates, names


def circuit_from_signals(builder, outs, min_share=2):
    """-> list of two-input gates (id, op, a, b) in an order in which they can be evaluated, and
    the list of (id or None, constant) per output.  ids < ninputs are the inputs."""
    # targets: both operands of every AND gate, and the outputs
    targets = []
    for a, bb in builder.ands:
        targets += [a, bb]
    targets += [o[0] for o in outs]
    xors, names = share_pairs(targets, min_share)
    # order: an XOR gate can be emitted once both its operands exist; an AND once its operand
    # sets are named
    avail = set(range(builder.ninputs))
    gates, pending_x = [], list(xors)
    and_done = [False] * len(builder.ands)
    progress = True
    while progress:
        progress = False
        rest = []
        for nid, a, b in pending_x:
            if a in avail and b in avail:
                gates.append((nid, "xor", a, b))
                avail.add(nid)
                progress = True
            else:
                rest.append((nid, a, b))
        pending_x = rest
        for k in range(len(builder.ands)):
            if and_done[k]:
                continue
            na, nb = names[2 * k], names[2 * k + 1]
            if na in avail and nb in avail:
                gates.append((builder.ninputs + k, "and", na, nb))
                avail.add(builder.ninputs + k)
                and_done[k] = True
                progress = True
    assert not pending_x and all(and_done), "circuit could not be ordered"
    out_names = [(names[2 * len(builder.ands) + i], outs[i][1]) for i in range(len(outs))]
    return gates, out_names


def pack3(gates, out_names, ninputs):
    """packs two-input gates into three-input ones: a gate takes over the function of a gate that
    feeds it when the union of their inputs has at most three members; a gate all of whose
    consumers have done so is no longer needed and is dropped (one that some consumer or an
    output still reads stays, and nothing is lost).  Returns a list of (id, truth table, [inputs])
    with 1..3 inputs; the table's bit (a | b << 1 | c << 2) is the output for inputs a, b, c."""
    fn = {}        # id -> (inputs tuple, function of an environment {input id: bit})
    order = []
    for nid, op, a, b in gates:
        plain = {a: ((a,), (lambda env, s=a: env[s])), b: ((b,), (lambda env, s=b: env[s]))}
        deep = {src: fn[src] if src in fn else plain[src] for src in (a, b)}
        chosen = None
        # both feeders taken over, then either (the one with more inputs first), then neither
        options = [(deep[a], deep[b])]
        one = [(deep[a], plain[b]), (plain[a], deep[b])]
        one.sort(key=lambda pq: -len(set(pq[0][0]) | set(pq[1][0])))
        options += one + [(plain[a], plain[b])]
        for pa, pb in options:
            ins = tuple(sorted(set(pa[0]) | set(pb[0])))
            if len(ins) <= 3:
                chosen = (ins, pa[1], pb[1])
                break
        ins, fa, fb = chosen
        if op == "xor":
            f = (lambda fa, fb: (lambda env: fa(env) ^ fb(env)))(fa, fb)
        else:
            f = (lambda fa, fb: (lambda env: fa(env) & fb(env)))(fa, fb)
        fn[nid] = (ins, f)
        order.append(nid)
    # drop what nothing reads any more
    needed = {name for name, _ in out_names if name is not None}
    for nid in reversed(order):
        if nid in needed:
            needed.update(s for s in fn[nid][0] if s in fn)
    packed = []
    for nid in order:
        if nid not in needed:
            continue
        ins, f = fn[nid]
        tt = 0
        for bits in itertools.product((0, 1), repeat=len(ins)):
            if f(dict(zip(ins, bits))):
                tt |= 1 << sum(bit << i for i, bit in enumerate(bits))
        packed.append((nid, tt, list(ins)))
    return packed


def fold_inversions(packed, out_names):
    """an inverted output whose instruction serves nothing else gets the inversion built into
    the instruction's truth table"""
    used_elsewhere = {}
    for nid, tt, ins in packed:
        for s in ins:
            used_elsewhere[s] = True
    packed = list(packed)
    out_names = list(out_names)
    index = {nid: k for k, (nid, _, _) in enumerate(packed)}
    seen = {}
    for name, _ in out_names:
        seen[name] = seen.get(name, 0) + 1
    for i, (name, const) in enumerate(out_names):
        if const and name in index and not used_elsewhere.get(name) and seen[name] == 1:
            nid, tt, ins = packed[index[name]]
            packed[index[name]] = (nid, tt ^ ((1 << (1 << len(ins))) - 1), ins)
            out_names[i] = (name, 0)
    return packed, out_names


def evaluate_packed(packed, out_names, ninputs, x):
    val = {i: (x >> i) & 1 for i in range(ninputs)}
    for nid, tt, ins in packed:
        idx = sum(val[s] << i for i, s in enumerate(ins))
        val[nid] = (tt >> idx) & 1
    r = 0
    for i, (name, const) in enumerate(out_names):
        bit = (val[name] if name is not None else 0) ^ const
        r |= bit << i
    return r


def best_sbox():
    best = None
    for n_const, l_const, root, into, out_cols in towers():
        b, outs = sbox_signals(n_const, l_const, into, out_cols)
        for min_share in (2, 3, 4):
            gates, out_names = circuit_from_signals(b, outs, min_share)
            packed, out_names = fold_inversions(pack3(gates, out_names, 8), out_names)
            cost = len(packed) + sum(1 for name, c in out_names if c)
            if best is None or cost < best[0]:
                best = (cost, (n_const, l_const, root), gates, packed, out_names, len(b.ands))
    cost, tower, gates, packed, out_names, nands = best
    for x in range(256):
        assert evaluate_packed(packed, out_names, 8, x) == sbox_value(x), "S-box circuit is wrong"
    return best


# ---------------------------------------------------------------------------------------------
# MixColumns followed by AddRoundKey on one column (FIPS-197 5.1.3, 5.1.4): inputs a[r][i]
# (row r, bit i) = atoms 8 r + i, key bits = atoms 32 + 8 r + i; 32 outputs

def mixcolumn_circuit():
    def xtime_terms(row):
        # bit i of 2 * a: a[i - 1], plus a[7] for i in {0, 1, 3, 4}
        out = []
        for i in range(8):
            s = set()
            if i > 0:
                s ^= {8 * row + i - 1}
            if i in (0, 1, 3, 4):
                s ^= {8 * row + 7}
            out.append(s)
        return out

    targets = []
    for r in range(4):
        two = xtime_terms(r)
        three = [xtime_terms((r + 1) % 4)[i] ^ {8 * ((r + 1) % 4) + i} for i in range(8)]
        for i in range(8):
            s = set(two[i]) ^ set(three[i]) ^ {8 * ((r + 2) % 4) + i} ^ {8 * ((r + 3) % 4) + i}
            s ^= {32 + 8 * r + i}
            targets.append(frozenset(s))
    best = None
    for min_share in (2, 3, 4, 5, 99):
        xors, names = share_pairs(targets, min_share)
        gates = [(nid, "xor", a, b) for nid, a, b in xors]
        # order the gates
        avail, ordered, rest = set(range(64)), [], gates
        while rest:
            nxt = []
            for g in rest:
                if g[2] in avail and g[3] in avail:
                    ordered.append(g)
                    avail.add(g[0])
                else:
                    nxt.append(g)
            assert len(nxt) < len(rest)
            rest = nxt
        out_names = [(n, 0) for n in names]
        packed = pack3(ordered, out_names, 64)
        if best is None or len(packed) < len(best[1]):
            best = (ordered, packed, out_names)
    ordered, packed, out_names = best
    # check against the definition on random columns
    import random
    rnd = random.Random(1)
    for _ in range(200):
        a = [rnd.randrange(256) for _ in range(4)]
        k = [rnd.randrange(256) for _ in range(4)]
        x = sum(a[r] << (8 * r) for r in range(4)) | sum(k[r] << (32 + 8 * r) for r in range(4))
        got = evaluate_packed(packed, out_names, 64, x)
        for r in range(4):
            want = (gf256_mul(a[r], 2) ^ gf256_mul(a[(r + 1) % 4], 3) ^ a[(r + 2) % 4] ^
                    a[(r + 3) % 4] ^ k[r])
            assert (got >> (8 * r)) & 0xFF == want, "MixColumns circuit is wrong"
    return len(ordered), packed, out_names


# ---------------------------------------------------------------------------------------------
# C++ text

def emit(packed, out_names, ninputs, in_name, out_name, indent="    "):
    lines = []
    name = {i: "%s[%d]" % (in_name, i) for i in range(ninputs)}
    for nid, tt, ins in packed:
        name[nid] = "t%d" % nid
        args = [name[s] for s in ins]
        if len(ins) == 3:
            expr = "__builtin_amdgcn_bitop3_b32(%s, %s, %s, 0x%02x)" % (
                args[0], args[1], args[2], _bitop3_table(tt))
        elif len(ins) == 2:
            expr = {0x6: "%s ^ %s", 0x8: "%s & %s", 0x9: "~(%s ^ %s)", 0xe: "%s | %s",
                    0x7: "~(%s & %s)"}[tt] % tuple(args)
        else:
            expr = {0x2: "%s", 0x1: "~%s"}[tt] % args[0]
        lines.append("%sconst uint32_t t%d = %s;" % (indent, nid, expr))
    for i, (n, const) in enumerate(out_names):
        src = name[n] if n is not None else "0u"
        lines.append("%s%s[%d] = %s%s;" % (indent, out_name, i, "~" if const else "", src))
    return "\n".join(lines)


def _bitop3_table(tt):
    """our table's bit index is a | b << 1 | c << 2; the instruction's is a << 2 | b << 1 | c"""
    out = 0
    for a in (0, 1):
        for b in (0, 1):
            for c in (0, 1):
                if (tt >> (a | b << 1 | c << 2)) & 1:
                    out |= 1 << (a << 2 | b << 1 | c)
    return out


def generate():
    cost, tower, gates, packed, out_names, nands = best_sbox()
    nxor2 = sum(1 for g in gates if g[1] == "xor")
    mc_gates, mc_packed, mc_out = mixcolumn_circuit()
    inv_out = sum(1 for _, c in out_names if c)
    nxor2 = sum(1 for g in gates if g[1] == "xor")
    text = []
    text.append("// Generated by gen_bitsliced_aes.py; do not edit.  Bitsliced AES round pieces for gfx950:")
    text.append("// a uint32_t holds one bit position of one state byte for 32 blocks.")
    text.append("//   S-box: tower GF(((2^2)^2)^2) with N = %d, L = %d, root 0x%02x: %d AND + %d XOR"
                % (tower[0], tower[1], tower[2], nands, nxor2))
    text.append("//   two-input gates, packed into %d three-input instructions (+ %d output inversions)."
                % (len(packed), inv_out))
    text.append("//   MixColumns + AddRoundKey of one column: %d two-input XORs, packed into %d instructions."
                % (mc_gates, len(mc_packed)))
    text.append("#pragma once")
    text.append("#include <stdint.h>")
    text.append("")
    text.append("namespace pgcm_bitsliced {")
    text.append("")
    text.append("constexpr int kSboxInstructions = %d;" % (len(packed) + inv_out))
    text.append("constexpr int kMixColumnInstructions = %d;" % len(mc_packed))
    text.append("")
    text.append("// x[i] = bit i of the byte, in and out (FIPS-197 5.1.1)")
    text.append("__device__ __forceinline__ void sbox_planes(uint32_t x[8]) {")
    text.append(emit(packed, out_names, 8, "x", "y_"))
    text.append("}")
    # outputs are written to a temporary name first: patch to write x after all reads
    body = "\n".join(text)
    body = body.replace("void sbox_planes(uint32_t x[8]) {\n", "void sbox_planes(uint32_t x[8]) {\n    uint32_t y_[8];\n")
    body = body.replace("}\n" if False else "\n}", "\n    for (int i = 0; i < 8; ++i) x[i] = y_[i];\n}", 1)
    text = [body]
    text.append("")
    text.append("// a[8 r + i] = bit i of the column's byte in row r; a[32 + 8 r + i] = the same bit of the")
    text.append("// round key, as a mask (0 or ~0); o[8 r + i] = MixColumns(a) ^ key (FIPS-197 5.1.3, 5.1.4)")
    text.append("__device__ __forceinline__ void mixcolumn_addkey_planes(const uint32_t a[64], uint32_t o[32]) {")
    text.append(emit(mc_packed, mc_out, 64, "a", "o"))
    text.append("}")
    text.append("")
    text.append("}  // namespace pgcm_bitsliced")
    return "\n".join(text) + "\n"


if __name__ == "__main__":
    text = generate()
    if "--check" in sys.argv:
        sys.exit(0 if open(OUT).read() == text else 1)
    with open(OUT, "w") as f:
        f.write(text)
    print(text.split("#pragma once")[0])
