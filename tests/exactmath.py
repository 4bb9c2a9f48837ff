"""Independent brute-force evaluator used to pin the CPU oracle on tiny inputs.

Pure Python: integers are Python ints, floating values are evaluated in exact rational
arithmetic (``fractions.Fraction``) and rounded explicitly to a binary format, so every
rounding step is visible.  It shares nothing with the oracle or the GPU library.

Conventions follow the readings stated with the design notes: float->int casts truncate
toward zero, saturate, NaN -> 0; int->int casts saturate; conversions to floating types round
to nearest even once; half-precision compute types evaluate in single precision and round
once on store; integer arithmetic wraps; min/max propagate NaN, +0 above -0.
"""
from __future__ import annotations

import math
import struct
from fractions import Fraction

INT_BITS = {"int8": 8, "int16": 16, "int32": 32, "int64": 64,
            "uint8": 8, "uint16": 16, "uint32": 32, "uint64": 64}
SIGNED = ("int8", "int16", "int32", "int64")
UNSIGNED = ("uint8", "uint16", "uint32", "uint64")
REAL = ("half", "float", "double")
COMPLEX = ("chalf", "cfloat", "cdouble")
ALL = ("bool",) + SIGNED + UNSIGNED + REAL + COMPLEX
# format: (precision bits, minimum normal exponent, maximum exponent)
FMT = {"half": (11, -14, 15), "float": (24, -126, 127), "double": (53, -1022, 1023)}
REAL_OF = {"chalf": "half", "cfloat": "float", "cdouble": "double"}
SIZE = {"bool": 1, "int8": 1, "int16": 2, "int32": 4, "int64": 8, "uint8": 1, "uint16": 2,
        "uint32": 4, "uint64": 8, "half": 2, "float": 4, "double": 8, "chalf": 4, "cfloat": 8,
        "cdouble": 16}


def kind(dt: str) -> str:
    if dt == "bool":
        return "b"
    if dt in SIGNED:
        return "i"
    if dt in UNSIGNED:
        return "u"
    if dt in REAL:
        return "f"
    return "c"


def int_range(dt: str):
    n = INT_BITS[dt]
    return (-(1 << (n - 1)), (1 << (n - 1)) - 1) if dt in SIGNED else (0, (1 << n) - 1)


# ---------------------------------------------------------------------------------------
# rounding a rational to a binary floating-point format, nearest-even
# ---------------------------------------------------------------------------------------
def round_fraction(x: Fraction, fmt: str, zero_sign: float = 0.0) -> float:
    """Nearest value of the format (ties to even, gradual underflow, overflow to infinity).
    ``zero_sign`` gives the sign to use when x is exactly zero."""
    p, emin, emax = FMT[fmt]
    if x == 0:
        return -0.0 if math.copysign(1.0, zero_sign) < 0 else 0.0
    neg = x < 0
    a = -x if neg else x
    e = a.numerator.bit_length() - a.denominator.bit_length()
    while Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, emin)
    quantum = Fraction(2) ** (e - p + 1)
    n = a / quantum
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    val = fl * quantum
    if val >= Fraction(2) ** (emax + 1):
        out = math.inf
    else:
        out = float(val)  # exact: every half/float/double value is a double
    return -out if neg else out


def round_real(x: float, fmt: str) -> float:
    """Round a double-held value to a (narrower) format once."""
    if math.isnan(x) or math.isinf(x):
        return x
    if x == 0.0:
        return x
    return round_fraction(Fraction(x), fmt, x)


# ---------------------------------------------------------------------------------------
# element decode / encode
# ---------------------------------------------------------------------------------------
_FMT_CHAR = {"int8": "b", "int16": "h", "int32": "i", "int64": "q", "uint8": "B", "uint16": "H",
             "uint32": "I", "uint64": "Q", "half": "e", "float": "f", "double": "d"}


def decode(dt: str, raw: bytes):
    if dt == "bool":
        return 1 if raw[0] != 0 else 0
    if dt in COMPLEX:
        c = _FMT_CHAR[REAL_OF[dt]]
        return struct.unpack("<" + c + c, raw)
    return struct.unpack("<" + _FMT_CHAR[dt], raw)[0]


def encode(dt: str, v) -> bytes:
    if dt == "bool":
        return bytes([1 if v else 0])
    if dt in COMPLEX:
        c = _FMT_CHAR[REAL_OF[dt]]
        return _pack_real(c, v[0]) + _pack_real(c, v[1])
    if dt in REAL:
        return _pack_real(_FMT_CHAR[dt], v)
    return struct.pack("<" + _FMT_CHAR[dt], v)


def _pack_real(c: str, x: float) -> bytes:
    return struct.pack("<" + c, x)  # x is already a value of the format (or inf / NaN)


# ---------------------------------------------------------------------------------------
# casting rules
# ---------------------------------------------------------------------------------------
def _real_to_int(x: float, lo: int, hi: int) -> int:
    if math.isnan(x):
        return 0
    if math.isinf(x):
        return hi if x > 0 else lo
    t = int(x)  # truncates toward zero, exact
    return min(max(t, lo), hi)


def _int_to_real(i: int, fmt: str) -> float:
    return round_fraction(Fraction(i), fmt)


def convert(v, src: str, dst: str):
    ks, kd = kind(src), kind(dst)
    if kd == "b":
        if ks in "biu":
            return 1 if v != 0 else 0
        if ks == "f":
            return 1 if (v != 0.0) else 0  # NaN != 0 is True
        return 1 if (v[0] != 0.0 or v[1] != 0.0) else 0
    if kd in "iu":
        lo, hi = int_range(dst)
        if ks in "biu":
            return min(max(int(v), lo), hi)
        x = v if ks == "f" else v[0]
        return _real_to_int(x, lo, hi)
    if kd == "f":
        if ks in "biu":
            return _int_to_real(int(v), dst)
        x = v if ks == "f" else v[0]
        return round_real(x, dst)
    # complex destination
    rd = REAL_OF[dst]
    if ks in "biu":
        return (_int_to_real(int(v), rd), 0.0)
    if ks == "f":
        return (round_real(v, rd), 0.0)
    return (round_real(v[0], rd), round_real(v[1], rd))


# ---------------------------------------------------------------------------------------
# promotion: the smallest type whose value set contains both (brute-force containment)
# ---------------------------------------------------------------------------------------
def _value_set(dt: str):
    """(integer lo, integer hi, float precision or 0): the integers a type holds exactly and,
    for floating types, the significand width."""
    if dt == "bool":
        return (0, 1, 0)
    if dt in INT_BITS:
        lo, hi = int_range(dt)
        return (lo, hi, 0)
    p = FMT[dt][0]
    return (-(1 << p), 1 << p, p)


def _contains(big: str, small: str) -> bool:
    bl, bh, bp = _value_set(big)
    sl, sh, sp = _value_set(small)
    if sp and not bp:
        return False  # fractions do not fit an integer type
    if sp and bp:
        return sp <= bp
    return bl <= sl and sh <= bh


def promote(a: str, b: str) -> str:
    if a in COMPLEX or b in COMPLEX:
        ra, rb = REAL_OF.get(a, a), REAL_OF.get(b, b)
        r = promote(ra, rb)
        return {"half": "chalf", "float": "cfloat", "double": "cdouble"}[r]
    order = sorted(("bool",) + SIGNED + UNSIGNED + REAL,
                   key=lambda d: (SIZE[d], {"b": 0, "i": 1, "u": 2, "f": 3}[kind(d)]))
    for c in order:
        if _contains(c, a) and _contains(c, b):
            return c
    return "double"


# ---------------------------------------------------------------------------------------
# arithmetic in a compute type
# ---------------------------------------------------------------------------------------
def _wrap(x: int, dt: str) -> int:
    n = INT_BITS[dt]
    x &= (1 << n) - 1
    if dt in SIGNED and x >> (n - 1):
        x -= 1 << n
    return x


def _arith_fmt(T: str) -> str:
    r = REAL_OF.get(T, T)
    return "double" if r == "double" else "float"  # half types compute in single precision


def _fop(op: str, a: float, b: float, fmt: str) -> float:
    """One correctly rounded IEEE operation on finite or special operands."""
    if math.isnan(a) or math.isnan(b):
        return math.nan
    if op == "add" or op == "sub":
        if op == "sub":
            b = -b
        if math.isinf(a) or math.isinf(b):
            if math.isinf(a) and math.isinf(b) and (a > 0) != (b > 0):
                return math.nan
            return a if math.isinf(a) else b
        s = Fraction(a) + Fraction(b)
        if s == 0:
            # exact zero sum: -0 only when both addends are -0 (round to nearest)
            both_neg = math.copysign(1, a) < 0 and math.copysign(1, b) < 0
            return -0.0 if both_neg else 0.0
        return round_fraction(s, fmt)
    sign = -1.0 if (math.copysign(1, a) < 0) != (math.copysign(1, b) < 0) else 1.0
    if op == "mul":
        if math.isinf(a) or math.isinf(b):
            if a == 0 or b == 0:
                return math.nan
            return sign * math.inf
        pr = Fraction(a) * Fraction(b)
        if pr == 0:
            return sign * 0.0
        return round_fraction(pr, fmt)
    if op == "div":
        if math.isinf(a):
            return math.nan if math.isinf(b) else sign * math.inf
        if math.isinf(b):
            return sign * 0.0
        if b == 0:
            return math.nan if a == 0 else sign * math.inf
        if a == 0:
            return sign * 0.0
        return round_fraction(Fraction(a) / Fraction(b), fmt)
    raise ValueError(op)


def _fsqrt(a: float, fmt: str) -> float:
    if math.isnan(a) or a < 0:
        return math.nan
    if a == 0 or math.isinf(a):
        return a
    p = FMT[fmt][0]
    x = Fraction(a)
    # exact integer square root at enough extra bits, then decide rounding by comparison
    e = x.numerator.bit_length() - x.denominator.bit_length()
    shift = 2 * (p + 8) - e
    if shift % 2:
        shift += 1
    scaled = x * Fraction(2) ** shift
    n = scaled.numerator // scaled.denominator
    r = math.isqrt(n)
    exact = (r * r == n) and scaled.denominator == 1
    approx = Fraction(r) / Fraction(2) ** (shift // 2)
    if not exact:
        # nudge above the floor so that a tie cannot be mistaken (sqrt of a non-square is
        # irrational, hence never exactly at a rounding midpoint)
        approx += Fraction(1, 2) / Fraction(2) ** (shift // 2)
    return round_fraction(approx, fmt)


def _fmax(a: float, b: float) -> float:
    if math.isnan(a) or math.isnan(b):
        return math.nan
    if a > b:
        return a
    if b > a:
        return b
    return b if math.copysign(1, a) < 0 else a


def _fmin(a: float, b: float) -> float:
    if math.isnan(a) or math.isnan(b):
        return math.nan
    if a < b:
        return a
    if b < a:
        return b
    return a if math.copysign(1, a) < 0 else b


ARITH = ("add", "sub", "mul", "div", "min", "max")
BITWISE = ("band", "bor", "bxor")
LOGICAL = ("land", "lor", "lxor")
COMPARE = ("eq", "ne", "lt", "le", "gt", "ge", "absgt")


def compute_type(op: str, da: str, db: str, dout: str) -> str:
    if op in LOGICAL:
        return "bool"
    if op in COMPARE:
        return promote(da, db)
    P = promote(da, db)
    if dout in (da, db) or promote(P, dout) == dout:
        return dout
    return P


def binary_supported(op: str, T: str) -> bool:
    k = kind(T)
    if op in ARITH:
        return k != "b" and not (k == "c" and op in ("min", "max"))
    if op in BITWISE:
        return k in "biu"
    if op in LOGICAL or op in ("eq", "ne", "absgt"):
        return True
    return k != "c"


def apply_binary(op: str, T: str, a, b):
    """a, b are values of type T; returns a value of T (arithmetic, bitwise) or a bool."""
    k = kind(T)
    if op in LOGICAL:
        return {"land": int(bool(a) and bool(b)), "lor": int(bool(a) or bool(b)),
                "lxor": int(bool(a) != bool(b))}[op]
    if op == "absgt":
        if k in "biu":
            return int(abs(int(a)) > abs(int(b)))
        if k == "f":
            return int(abs(a) > abs(b))
        ma = _fop("add", _fop("mul", a[0], a[0], "double"), _fop("mul", a[1], a[1], "double"), "double")
        mb = _fop("add", _fop("mul", b[0], b[0], "double"), _fop("mul", b[1], b[1], "double"), "double")
        return int(ma > mb)
    if op in COMPARE:
        if k == "c":
            eq = a[0] == b[0] and a[1] == b[1]
            return int(eq if op == "eq" else not eq)
        return int({"eq": a == b, "ne": a != b, "lt": a < b, "le": a <= b, "gt": a > b, "ge": a >= b}[op])
    if op in BITWISE:
        r = {"band": int(a) & int(b), "bor": int(a) | int(b), "bxor": int(a) ^ int(b)}[op]
        return r if k == "b" else _wrap(r, T)
    if k in "iu":
        a, b = int(a), int(b)
        if op == "add":
            return _wrap(a + b, T)
        if op == "sub":
            return _wrap(a - b, T)
        if op == "mul":
            return _wrap(a * b, T)
        if op == "div":
            if b == 0:
                return 0
            q = abs(a) // abs(b)
            return _wrap(q if (a < 0) == (b < 0) else -q, T)
        return min(a, b) if op == "min" else max(a, b)
    fmt = _arith_fmt(T)
    if k == "f":
        if op == "min":
            return _fmin(a, b)
        if op == "max":
            return _fmax(a, b)
        return _fop(op, a, b, fmt)
    # complex
    if op in ("add", "sub"):
        return (_fop(op, a[0], b[0], fmt), _fop(op, a[1], b[1], fmt))
    if op == "mul":
        return (_fop("sub", _fop("mul", a[0], b[0], fmt), _fop("mul", a[1], b[1], fmt), fmt),
                _fop("add", _fop("mul", a[0], b[1], fmt), _fop("mul", a[1], b[0], fmt), fmt))
    if op == "div":
        den = _fop("add", _fop("mul", b[0], b[0], fmt), _fop("mul", b[1], b[1], fmt), fmt)
        nre = _fop("add", _fop("mul", a[0], b[0], fmt), _fop("mul", a[1], b[1], fmt), fmt)
        nim = _fop("sub", _fop("mul", a[1], b[0], fmt), _fop("mul", a[0], b[1], fmt), fmt)
        return (_fop("div", nre, den, fmt), _fop("div", nim, den, fmt))
    raise ValueError(op)


UNARY = ("ident", "neg", "abs", "conj", "lnot", "bnot", "sqrt")


def unary_supported(op: str, T: str) -> bool:
    k = kind(T)
    return {"ident": True, "conj": True, "lnot": True, "neg": k != "b",
            "abs": k not in "bc", "bnot": k in "biu", "sqrt": k == "f"}[op]


def apply_unary(op: str, T: str, a):
    k = kind(T)
    if op == "ident":
        return a
    if op == "lnot":
        return int(not a)
    if op == "neg":
        if k in "iu":
            return _wrap(-int(a), T)
        return -a if k == "f" else (-a[0], -a[1])
    if op == "abs":
        if k in "iu":
            return _wrap(abs(int(a)), T)
        return abs(a)
    if op == "conj":
        return (a[0], -a[1]) if k == "c" else a
    if op == "bnot":
        return int(not a) if k == "b" else _wrap(~int(a), T)
    if op == "sqrt":
        return _fsqrt(a, _arith_fmt(T))
    raise ValueError(op)


def same_value(dt: str, x: bytes, y: bytes) -> bool:
    """Bit equality, except that any two NaNs of a floating component count as equal."""
    if x == y:
        return True
    if kind(dt) not in "fc":
        return False
    a, b = decode(dt, x), decode(dt, y)
    if kind(dt) == "f":
        a, b = (a,), (b,)
    rsz = SIZE[dt] // len(a)
    for i, (p, q) in enumerate(zip(a, b)):
        if math.isnan(p) and math.isnan(q):
            continue
        if x[i * rsz:(i + 1) * rsz] != y[i * rsz:(i + 1) * rsz]:
            return False
    return True
