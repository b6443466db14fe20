"""HCCS in pure Python integers -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

A second, independent statement of the method, kept as close to the paper's
notation as Python allows (one row at a time, unbounded integers, no numpy in
the arithmetic).  It exists so that the C oracle in this folder can be
cross-checked on small cases, and it shares nothing with the GPU library.
Only tests may import it.

Passages followed:
  admissible()        Sec. IV-C (integer range constraints) and Eq. (11)
  row_scores()        Eq. (2) clamped distance, Eq. (3) clipped-linear score
  row_u8()            Sec. III-B "int8 output path": Eq. (8) with R = 15
  row_i16()           Alg. 1 / Eq. (6), (7) with T = 32767
  row_clb_u8/_i16()   Sec. III-B leading-bit reciprocal, Eq. (9)
  requant()           this repository's definition of int32 -> int8 logits
  attention()         Q.K^T -> requant -> row_u8 -> P.V
"""

INV_SHIFT = 15
OUT_SHIFT = 0
N_U8 = 255 << INV_SHIFT


def admissible(B, S, D, n, band):
    """True when (B,S,D) may be used for rows of length n.  band 1 is the full
    list of Sec. IV-C; band 0 swaps the int16-path ceiling for n*B <= 255*2^15."""
    if not (1 <= n <= 65536):
        return False
    if not (0 <= D <= 127 and 0 <= S <= 127 and 1 <= B <= 32767):
        return False
    if B - S * D < 0:
        return False
    if n * (B - S * D) < 256:
        return False
    ceiling = 32767 if band == 1 else N_U8
    return n * B <= ceiling


def row_scores(x, B, S, D):
    m = max(x)
    delta = [min(m - xi, D) for xi in x]
    s = [B - S * di for di in delta]
    return m, delta, s


def row_u8(x, B, S, D):
    _, _, s = row_scores(x, B, S, D)
    Z = sum(s)
    rho = N_U8 // Z
    return [(si * rho) >> (INV_SHIFT + OUT_SHIFT) for si in s]


def row_i16(x, B, S, D):
    _, _, s = row_scores(x, B, S, D)
    Z = sum(s)
    rho = 32767 // Z
    return [si * rho for si in s]


def row_clb_u8(x, B, S, D):
    _, _, s = row_scores(x, B, S, D)
    Z = sum(s)
    k = Z.bit_length() - 1
    rho = N_U8 // (1 << k)
    return [min((si * rho) >> (INV_SHIFT + OUT_SHIFT), 255) for si in s]


def row_clb_i16(x, B, S, D):
    _, _, s = row_scores(x, B, S, D)
    Z = sum(s)
    k = Z.bit_length() - 1
    rho = 32767 // (1 << k)
    return [min(si * rho, 32767) for si in s]


def requant(acc, mult, shift):
    """Round-half-up fixed-point rescale of an int32 dot product to an int8
    logit: floor((acc*mult + 2^(shift-1)) / 2^shift), saturated."""
    y = (acc * mult + (1 << (shift - 1))) >> shift  # Python's >> floors
    return max(-128, min(127, y))


def attention(Q, K, V, B, S, D, mult, shift):
    """One (batch, head) block.  Q, K, V are lists of L rows of d ints."""
    L, d = len(Q), len(Q[0])
    O = []
    for i in range(L):
        x = [requant(sum(Q[i][t] * K[j][t] for t in range(d)), mult, shift) for j in range(L)]
        p = row_u8(x, B, S, D)
        O.append([sum(p[j] * V[j][t] for j in range(L)) for t in range(d)])
    return O
