"""An independently written description of the SPARQ trim, used only to pin the oracle.

Where the oracle works on bits (leading one, shifts), this file works on value
ranges and grids, following the paper's piecewise-linear view (Section 3.1):
each placement option t owns the values below 2**(t+n) not owned by a smaller
option, and inside that region representable values are the multiples of 2**t
up to (2**n - 1) * 2**t.  Trimming picks the largest grid point not above x;
rounding picks the nearest grid point, ties upwards, never leaving the grid.
"""


def options(shift_mask):
    return [t for t in range(9) if (shift_mask >> t) & 1]


def region_step(x, n, shift_mask):
    """Grid step 2**t of the region that owns x."""
    for t in options(shift_mask):
        if x < 2 ** (t + n):
            return 2 ** t
    raise ValueError("value not covered by any placement option")


def grid(n, step):
    return [q * step for q in range(2 ** n)]


def trim_floor(x, n, shift_mask):
    g = grid(n, region_step(x, n, shift_mask))
    return max(v for v in g if v <= x)


def trim_round(x, n, shift_mask):
    g = grid(n, region_step(x, n, shift_mask))
    best = min(abs(x - v) for v in g)
    return max(v for v in g if abs(x - v) == best)      # tie -> the larger one


def trim(x, n, shift_mask, rnd):
    return trim_round(x, n, shift_mask) if rnd else trim_floor(x, n, shift_mask)


def wide_options(n, shift_mask):
    opts = options(shift_mask)
    return sum(1 << t for t in opts if (t + n) in opts and t + 2 * n <= 8)


def pair(a, b, n, shift_mask, rnd, pairing):
    """Eq. 2: a zero partner leaves the other value its full 2n-bit budget."""
    if n == 8:
        return a, b
    if pairing and (a == 0 or b == 0):
        wide = wide_options(n, shift_mask)
        return trim(a, 2 * n, wide, rnd), trim(b, 2 * n, wide, rnd)
    return trim(a, n, shift_mask, rnd), trim(b, n, shift_mask, rnd)
