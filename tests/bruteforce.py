"""Exact-rational brute force used to pin the CPU oracle.

Written from the definitions alone (format tables, "smallest power of two", "nearest
grid point, ties to the even code") with fractions.Fraction and Python integers; it
calls nothing under oracle/ and nothing of the GPU package.  Slow on purpose.
"""
from fractions import Fraction

E2M1_GRID = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3),
             Fraction(4), Fraction(6)]
INF = "inf"


def pow2(k):
    return Fraction(2) ** k


def e4m3_fraction(code7):
    """7-bit E4M3 magnitude code -> exact value (OCP e4m3fn: bias 7, subnormal m/8 * 2^-6)."""
    assert 0 <= code7 < 0x7F
    e, m = code7 >> 3, code7 & 7
    if e == 0:
        return Fraction(m, 8) * pow2(-6)
    return (1 + Fraction(m, 8)) * pow2(e - 7)


def f32_bits_to_fraction(bits):
    """Non-negative finite FP32 bit pattern -> exact value."""
    e, m = (bits >> 23) & 0xFF, bits & 0x7FFFFF
    assert e != 255
    if e == 0:
        return Fraction(m, 1 << 23) * pow2(-126)
    return (1 + Fraction(m, 1 << 23)) * pow2(e - 127)


def floor_log2(fr):
    assert fr > 0
    n, d = fr.numerator, fr.denominator
    e = n.bit_length() - d.bit_length()
    if pow2(e) > fr:
        e -= 1
    assert pow2(e) <= fr < pow2(e + 1)
    return e


def round_half_even(fr):
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def fl32(fr):
    """Round a non-negative exact value once to FP32 (nearest-even, gradual underflow).
    Returns a Fraction, or INF on overflow."""
    if fr == 0:
        return Fraction(0)
    e = max(floor_log2(fr), -126)
    quantum = pow2(e - 23)
    r = round_half_even(fr / quantum) * quantum
    if r >= pow2(128):
        return INF
    return r


def smallest_k(gmax):
    """The smallest integer k with gmax <= 6 * 2^k (the ceil(log2(gmax/6)) of the scale rule)."""
    k = floor_log2(gmax) - 4
    while 6 * pow2(k) < gmax:
        k += 1
    assert 6 * pow2(k) >= gmax and 6 * pow2(k - 1) < gmax
    return k


def scale_byte(gmax):
    if gmax == 0:
        return 0
    if gmax == INF:
        return 254
    return min(254, max(0, smallest_k(gmax) + 127))


def nearest_even_code(y, grid):
    """Index of the grid point nearest to y >= 0; ties go to the even index; above the
    grid (or INF) saturates to the last index."""
    if y == INF or y > grid[-1]:
        return len(grid) - 1
    best = min(range(len(grid)), key=lambda c: (abs(y - grid[c]), c & 1))
    return best


def quant_block(values):
    """values: list of 32 (sign, magnitude) with magnitude a Fraction or INF.
    Returns (scale byte, [nibble codes])."""
    mags = [m for _, m in values]
    gmax = INF if INF in mags else max(mags)
    b = scale_byte(gmax)
    codes = []
    for sgn, m in values:
        y = INF if m == INF else m / pow2(b - 127)
        codes.append((sgn << 3) | nearest_even_code(y, E2M1_GRID))
    return b, codes


def quant_block_from_fp8(bytes32, s_bits):
    """32 E4M3 bytes and the FP32 scale's bit pattern -> (scale byte, nibbles), reading
    the element value as the once-rounded FP32 product of E4M3 value and scale."""
    if any((c & 0x7F) == 0x7F for c in bytes32):
        return 0xFF, [0] * 32
    s = f32_bits_to_fraction(s_bits)
    vals = [((c >> 7) & 1, fl32(e4m3_fraction(c & 0x7F) * s)) for c in bytes32]
    return quant_block(vals)


E4M3_GRID = [e4m3_fraction(c) for c in range(0x7F)]


def dequant_tile(nibbles128, sf4):
    """128 nibble codes + 4 scale bytes (none NaN) -> (tile scale as Fraction, 128 E4M3 bytes)."""
    bmax = max(sf4)
    out = []
    for i, n in enumerate(nibbles128):
        b = sf4[i // 32]
        target = E2M1_GRID[n & 7] * pow2(b - 127)            # the element's real value
        in_units = target / pow2(bmax - 6 - 127)             # divided by the tile scale
        out.append(((n >> 3) << 7) | nearest_even_code(in_units, E4M3_GRID))
    return pow2(bmax - 6 - 127), out


def row_to_col_tile(nib, sf_rows):
    """nib[m][k] nibble codes of a 32 x 32 tile, sf_rows[m] the row-scale bytes (none NaN).
    Returns ([32 column scale bytes], codes[k][m])."""
    sc, codes = [], []
    for k in range(32):
        vals = [((nib[m][k] >> 3) & 1, E2M1_GRID[nib[m][k] & 7] * pow2(sf_rows[m] - 127)) for m in range(32)]
        b, c = quant_block(vals)
        sc.append(b)
        codes.append(c)
    return sc, codes


def bf16_fraction(h):
    """BF16 bit pattern (sign stripped by the caller or not) -> (sign, magnitude as Fraction or INF); NaN -> None."""
    sign, e, m = (h >> 15) & 1, (h >> 7) & 0xFF, h & 0x7F
    if e == 0xFF:
        return None if m else (sign, INF)
    if e == 0:
        return sign, Fraction(m, 128) * pow2(-126)
    return sign, (1 + Fraction(m, 128)) * pow2(e - 127)


def quant_block_from_bf16(halves32):
    vals = [bf16_fraction(h) for h in halves32]
    if any(v is None for v in vals):
        return 0xFF, [0] * 32
    return quant_block(vals)


def row_to_fp8_col_column(nibs, sf_bytes):
    """One output column group: nibs[m], sf_bytes[m] for 128 consecutive rows m at one k (no NaN byte).
    The group's scale is the smallest power of two S = 2^(max b - 6 - 127) that keeps the largest
    representable element, 6 * 2^(max b - 127), at 6 * 2^6 = 384 <= 448; each element is its real
    value divided by S, to the nearest E4M3 (ties to the even code).  Returns (S, [128 bytes])."""
    bmax = max(sf_bytes)
    S = pow2(bmax - 6 - 127)
    out = []
    for n, b in zip(nibs, sf_bytes):
        real = E2M1_GRID[n & 7] * pow2(b - 127)
        out.append(((n >> 3) << 7) | nearest_even_code(real / S, E4M3_GRID))
    return S, out


def row_to_fp8_col_requant_column(nibs, sf_bytes):
    """One output column group under the re-quantization reading: the exact values v_m, the smallest power
    of two S with max|v| <= 448 * S (S = 1 for an all-zero group), and v_m / S to the nearest E4M3 (ties to
    the even code).  No NaN byte.  Returns (S, [bytes])."""
    vals = [E2M1_GRID[n & 7] * pow2(b - 127) for n, b in zip(nibs, sf_bytes)]
    amax = max(vals)
    if amax == 0:
        S = Fraction(1)
    else:
        j = floor_log2(amax) - 12
        while 448 * pow2(j) < amax:
            j += 1
        assert 448 * pow2(j) >= amax and 448 * pow2(j - 1) < amax
        S = pow2(j)
    return S, [((n >> 3) << 7) | nearest_even_code(v / S, E4M3_GRID) for n, v in zip(nibs, vals)]
