"""CPU oracle for 2D Winograd convolution F(m x m, 3 x 3) with Cook-Toom transforms.

TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product path: only the
test-suite, the smoke check and the benchmark's `cpu_baseline` leg may import
this package.  It shares no code, tables, constants or helpers with the HIP
library; both sides only consume the same caller-supplied arrays and point
sets.

Contents
--------
cook_toom   exact (rational) construction of A, B^T, G from interpolation
            points, the exact bilinear-tensor identity, condition numbers
            (Sec. 2.1, Sec. 2.2, Sec. 2.4 "Symbolic Verification",
            Alg. "Symbolic Cook-Toom Construction").
exact       Winograd and direct convolution in rational arithmetic for tiny
            inputs (App. "Exact Zero with Rational Arithmetic").
conv        fp64 direct convolution (the definition, Sec. 2.1), fp64 Winograd
            convolution (2D nesting, App. "2D Extension via Kronecker
            Products") and the reduced-precision storage emulation
            (Sec. 4.1 / Sec. "Float16 Precision Analysis" setup); the loops
            are plain C in conv_oracle.c.

Parity pins (see tests/test_oracle_*.py): every function here is pinned to
something other than itself -- printed condition numbers, the textbook
F(2,3)/F(4,3) algorithms, exact rational equality with direct convolution, a
library fp64 convolution, exact-rounding special cases of the emulation, and,
for the emulation's general (inexact) case, a replay of its stated arithmetic
contract in exact rational arithmetic with every rounding applied explicitly
(tests/test_oracle_emulation_replay.py), which it must match bit for bit.
"""
