"""Operand encodings.  Test infrastructure: see oracle/__init__.py.

The paper names the operand types of the FDPA models (Algorithm "T-FDPA", its
Require line) but leaves SignedSig(x) and Exp(x) undefined.  The reading used
here is the one its text implies ("exact unnormalized products", Sec. 4.1.3,
paragraph T-FDPA) and that its worked example (Sec. 5, Table "divergent
results") confirms:

    x = (-1)^sign * sig * 2^(-m) * 2^Exp      exactly, with
    sig = M            , Exp = 1 - bias   when the exponent field is 0
    sig = 2^m + M      , Exp = E - bias   otherwise

so subnormals (and zeros) keep the minimum normal exponent and no hidden bit,
and nothing is renormalised.

FP8 flavours are the OCP ones: E4M3 has no infinity and a single NaN mantissa
(S.1111.111), its largest finite value is 448; E5M2 is IEEE-like with
largest finite value 57344.  FP6 (E2M3, E3M2) and FP4 (E2M1) are the OCP
microscaling element formats: every code is a finite number (no infinity, no
NaN); codes are held one per byte in their low 6 / 4 bits, higher bits ignored.
"""
from dataclasses import dataclass
from fractions import Fraction

E4M3, E5M2, FP16, BF16, FP32 = 0, 1, 2, 3, 4
E2M3, E3M2, E2M1 = 6, 7, 8          # (5 is the E8M0 scale code, which is no operand type)
TF32 = 9                            # a binary32 word whose low 13 mantissa bits are ignored (8 exponent, 10 mantissa bits)
FP64 = 10                           # binary64: Algorithms "FMA" / "Phi_FMA" are stated for FP64 as well as FP32


@dataclass(frozen=True)
class Format:
    name: str
    ebits: int
    mbits: int
    bias: int
    ieee_specials: bool  # True: exponent field all-ones = Inf/NaN.  False: E4M3 rule.
    no_specials: bool = False   # every code is finite (FP6, FP4)
    storage_shift: int = 0      # the code sits this many bits above bit 0 of its storage word (TF32: 13)

    @property
    def width(self):
        return 1 + self.ebits + self.mbits

    @property
    def emax_field(self):
        return (1 << self.ebits) - 1


FORMATS = {
    E4M3: Format("e4m3", 4, 3, 7, False),
    E5M2: Format("e5m2", 5, 2, 15, True),
    FP16: Format("fp16", 5, 10, 15, True),
    BF16: Format("bf16", 8, 7, 127, True),
    FP32: Format("fp32", 8, 23, 127, True),
    E2M3: Format("e2m3", 2, 3, 1, False, True),
    E3M2: Format("e3m2", 3, 2, 3, False, True),
    E2M1: Format("e2m1", 2, 1, 1, False, True),
    TF32: Format("tf32", 8, 10, 127, True, False, 13),
    FP64: Format("fp64", 11, 52, 1023, True),
}

ZERO, SUBNORMAL, NORMAL, INF, NAN = "zero", "subnormal", "normal", "inf", "nan"


@dataclass(frozen=True)
class Decoded:
    cls: str
    sign: int   # 0 or 1
    exp: int    # Exp(x): unnormalised exponent (defined for every finite x, zeros included)
    sig: int    # integer significand, < 2^(m+1); value = sig * 2^(exp - m)
    mbits: int

    @property
    def signed_sig(self):
        """SignedSig(x): rational in (-2, 2)."""
        return Fraction((-1) ** self.sign * self.sig, 1 << self.mbits)

    @property
    def value(self):
        """Exact rational value of a finite x."""
        return self.signed_sig * Fraction(2) ** self.exp

    @property
    def finite(self):
        return self.cls in (ZERO, SUBNORMAL, NORMAL)


def decode(bits, fmt_id):
    f = FORMATS[fmt_id]
    bits = (int(bits) >> f.storage_shift) & ((1 << f.width) - 1)
    sign = bits >> (f.ebits + f.mbits)
    E = (bits >> f.mbits) & f.emax_field
    M = bits & ((1 << f.mbits) - 1)
    if f.ieee_specials and E == f.emax_field:
        return Decoded(INF if M == 0 else NAN, sign, 0, 0, f.mbits)
    if not f.ieee_specials and not f.no_specials and E == f.emax_field and M == (1 << f.mbits) - 1:
        return Decoded(NAN, sign, 0, 0, f.mbits)
    if E == 0:
        return Decoded(ZERO if M == 0 else SUBNORMAL, sign, 1 - f.bias, M, f.mbits)
    return Decoded(NORMAL, sign, E - f.bias, (1 << f.mbits) + M, f.mbits)


def flush_subnormal(bits, fmt_id):
    """Input flush (Algorithm "Phi_FTZ-AddMul", FlushSubnormal): subnormal -> +0.0."""
    return 0 if decode(bits, fmt_id).cls == SUBNORMAL else int(bits)          # (a zero word is +0.0 in every format)
