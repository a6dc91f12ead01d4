"""Integer expressions over symbolic dims: the "operation-inferred constants" of
the RDP lattice (Section 4.1, the domain V').

An expression is a polynomial with integer coefficients over *atoms*.  An atom
is a symbol, floordiv(e, c) / mod(e, c) of a canonical expression e and a
positive integer c that could not be simplified, or bcast(e1, e2): the extent
two aligned dims broadcast to when neither is provably 1 or equal to the other
(Section 4.2, Fig. 4: which of the cases holds is only seen when the symbols are
bound; it evaluates to the common value, or to the other one when one is 1).  Two expressions are equal
exactly when their canonical strings are equal (sound, not complete).

Canonical string: terms sorted by (degree, atom strings); a term is
"coeff", "atom*atom" (coefficient 1) or "coeff*atom*atom"; terms joined by
" + "; the zero polynomial prints as "0".
"""
from __future__ import annotations

from typing import Dict, Tuple

_ATOMS: Dict[str, tuple] = {}   # atom string -> ("sym", name) | ("floordiv", Expr, c) | ("mod", Expr, c) | ("bcast", Expr, Expr)


class BroadcastMismatch(Exception):
    """Two extents that must broadcast are different and neither is 1."""


class Expr:
    __slots__ = ("terms", "_s")

    def __init__(self, terms: Dict[Tuple[str, ...], int]):
        self.terms = {m: c for m, c in terms.items() if c != 0}
        self._s = None

    # -- constructors ------------------------------------------------------
    @staticmethod
    def const(c: int) -> "Expr":
        return Expr({(): int(c)})

    @staticmethod
    def sym(name: str) -> "Expr":
        _ATOMS.setdefault(name, ("sym", name))
        return Expr({(name,): 1})

    @staticmethod
    def parse(text) -> "Expr":
        """An int, a symbol, or a '+'-separated sum of those."""
        if isinstance(text, (int,)) or hasattr(text, "__index__"):
            return Expr.const(int(text))
        e = Expr.const(0)
        for part in str(text).split("+"):
            part = part.strip()
            e = e + (Expr.const(int(part)) if part.lstrip("-").isdigit() else Expr.sym(part))
        return e

    # -- queries -----------------------------------------------------------
    def is_const(self) -> bool:
        return all(m == () for m in self.terms)

    def const_value(self) -> int:
        assert self.is_const()
        return self.terms.get((), 0)

    def is_symbol(self) -> bool:
        if len(self.terms) != 1:
            return False
        (m, c), = self.terms.items()
        return c == 1 and len(m) == 1 and _ATOMS[m[0]][0] == "sym"

    def kind(self) -> str:
        """Lattice class of a defined value (Fig. 2): known / symbolic / op-inferred constant."""
        return "known" if self.is_const() else ("symbolic" if self.is_symbol() else "opinf")

    def __str__(self) -> str:
        if self._s is None:
            parts = []
            for m, c in sorted(self.terms.items(), key=lambda kv: (len(kv[0]), kv[0])):
                if not m:
                    parts.append(str(c))
                elif c == 1:
                    parts.append("*".join(m))
                else:
                    parts.append(str(c) + "*" + "*".join(m))
            self._s = " + ".join(parts) if parts else "0"
        return self._s

    __repr__ = __str__

    def __eq__(self, other) -> bool:
        return isinstance(other, Expr) and str(self) == str(other)

    def __hash__(self):
        return hash(str(self))

    # -- arithmetic --------------------------------------------------------
    def __add__(self, o: "Expr") -> "Expr":
        t = dict(self.terms)
        for m, c in o.terms.items():
            t[m] = t.get(m, 0) + c
        return Expr(t)

    def __neg__(self) -> "Expr":
        return Expr({m: -c for m, c in self.terms.items()})

    def __sub__(self, o: "Expr") -> "Expr":
        return self + (-o)

    def __mul__(self, o: "Expr") -> "Expr":
        t: Dict[Tuple[str, ...], int] = {}
        for m1, c1 in self.terms.items():
            for m2, c2 in o.terms.items():
                m = tuple(sorted(m1 + m2))
                t[m] = t.get(m, 0) + c1 * c2
        return Expr(t)

    def floordiv(self, c: int) -> "Expr":
        """floor(self / c) for an integer c > 0."""
        assert c > 0
        if c == 1:
            return self
        if all(k % c == 0 for k in self.terms.values()):
            return Expr({m: k // c for m, k in self.terms.items()})
        if self.is_const():
            return Expr.const(self.const_value() // c)     # Python's // floors
        if len(self.terms) == 1:
            (m, k), = self.terms.items()
            if k == 1 and len(m) == 1 and _ATOMS[m[0]][0] == "floordiv":
                _, inner, c0 = _ATOMS[m[0]]                # floor(floor(e / a) / b) = floor(e / (a*b))
                return inner.floordiv(c0 * c)
        name = f"floordiv({self}, {c})"
        _ATOMS.setdefault(name, ("floordiv", self, c))
        return Expr({(name,): 1})

    def mod(self, c: int) -> "Expr":
        assert c > 0
        if all(k % c == 0 for k in self.terms.values()):
            return Expr.const(0)
        if self.is_const():
            return Expr.const(self.const_value() % c)
        name = f"mod({self}, {c})"
        _ATOMS.setdefault(name, ("mod", self, c))
        return Expr({(name,): 1})

    def bcast(self, o: "Expr") -> "Expr":
        """Extent of the broadcast of two aligned dims (the larger one when one of them is 1)."""
        if self == o:
            return self
        if self.is_const() and self.const_value() == 1:
            return o
        if o.is_const() and o.const_value() == 1:
            return self
        if self.is_const() and o.is_const():
            raise BroadcastMismatch(f"{self} vs {o}")
        a, b = sorted((self, o), key=str)
        name = f"bcast({a}, {b})"
        _ATOMS.setdefault(name, ("bcast", a, b))
        return Expr({(name,): 1})

    def exact_div(self, o: "Expr"):
        """self / o when o is a single term that divides every term of self, else None."""
        if len(o.terms) != 1:
            return None
        (dm, dc), = o.terms.items()
        out: Dict[Tuple[str, ...], int] = {}
        for m, c in self.terms.items():
            if c % dc != 0:
                return None
            rest = list(m)
            for a in dm:
                if a not in rest:
                    return None
                rest.remove(a)
            out[tuple(rest)] = c // dc
        return Expr(out)

    # -- evaluation ----------------------------------------------------------
    def eval(self, env: Dict[str, int]) -> int:
        total = 0
        for m, c in self.terms.items():
            v = c
            for a in m:
                v *= _eval_atom(a, env)
            total += v
        return total


def _eval_atom(a: str, env: Dict[str, int]) -> int:
    d = _ATOMS[a]
    if d[0] == "sym":
        return int(env[d[1]])
    inner = d[1].eval(env)
    if d[0] == "bcast":
        other = d[2].eval(env)
        if inner == other or other == 1:
            return inner
        if inner == 1:
            return other
        raise BroadcastMismatch(f"{d[1]} = {inner} vs {d[2]} = {other}")
    return inner // d[2] if d[0] == "floordiv" else inner % d[2]
