"""CPU oracle for bit-accurate MMA arithmetic models.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) imports, links or executes anything in this package; only the
test-suite, the smoke check and the CPU-baseline leg of the benchmark do.

Contents
--------
formats.py   operand encodings (FP8 E4M3/E5M2, FP16, BF16, FP32) -> sign, Exp, significand
rounding.py  conversion functions rho (RNE-FP32, RZ-FP32) on exact rationals
fdpa.py      the model: chained fused-dot-product-add with truncated alignment
             (paper Sec. 4.1.3, Algorithms "Phi_FDPA", "E-FDPA", "T-FDPA"), special
             values (Sec. 4.2), input/output subnormal flush (Algorithms
             "FTZ-Add/FTZ-Mul" and "Phi_FTZ-AddMul")
fma.py       the model built from the standard fused multiply-add (Sec. 4.1.2, Algorithms "FMA", "Phi_FMA")
exact.py     exact rational dot products and error statistics
stats.py     bitwise comparison statistics (Eq. 2 of the paper: Phi(A,B,C) == interface(A,B,C))
philox.py    Philox-4x32-10 counter-based generator (Salmon et al., SC'11)
gen.py       the synthetic tile generators (CPU twins of the on-device generators)
o2/          the same model in plain C with fixed wide integers, multithreaded,
             for full-size checks and for the timed CPU baseline

Arithmetic is exact: Python int and fractions.Fraction in the *.py files,
unsigned __int128 plus sticky bits in o2/.
"""
