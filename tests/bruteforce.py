"""Pure-Python (integers, lists, struct) restatement of the codec on tiny inputs.

Used only by the CPU tests to pin oracle/s2r_oracle.py against something that is
not numpy: every loop of Algorithm 1 is written out element by element, hashes
are computed with unbounded Python integers reduced mod 2^64, the bitmap is a
Python list of 0/1 flags, the median is sorted()[...].  Nothing here is imported
by the oracle or by the product.
"""

import struct

MASK64 = (1 << 64) - 1


def f32_bits(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0]


def is_nonzero(x: float) -> bool:
    return (f32_bits(x) & 0x7FFFFFFF) != 0


def splitmix(seed, count):
    s, out = seed & MASK64, []
    for _ in range(count):
        s = (s + 0x9E3779B97F4A7C15) % (1 << 64)
        z = s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) % (1 << 64)
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) % (1 << 64)
        out.append(z ^ (z >> 31))
    return out


def params(seed, d):
    s = splitmix(seed, 4 * d)
    return [(s[4 * j] | 1, s[4 * j + 1], s[4 * j + 2] | 1, s[4 * j + 3]) for j in range(d)]


def h(i, a, b, w):
    L = w.bit_length() - 1
    u = (a * i + b) % (1 << 64)
    return u >> (64 - L) if L else 0


def s(i, c, e):
    v = (c * i + e) % (1 << 64)
    return 1 if (v >> 63) == 0 else -1


def compress(g, d, w, seed):
    """g: list of Python floats that are exactly representable in float32."""
    n = len(g)
    flags = [1 if is_nonzero(x) else 0 for x in g]
    S = [[0.0] * w for _ in range(d)]
    P = params(seed, d)
    for i in range(n):
        if flags[i]:
            for j in range(d):
                a, b, c, e = P[j]
                S[j][h(i, a, b, w)] += s(i, c, e) * g[i]
    return flags, S


def mass_table(g, d, w, seed):
    """M[j][b] = sum of |g(i)| over the non-zero elements i that row j sends to bucket b:
    the insertion loops of Algorithm 1 with |g(i)| in place of s_j(i) g(i)."""
    M = [[0.0] * w for _ in range(d)]
    P = params(seed, d)
    for i, x in enumerate(g):
        if is_nonzero(x):
            for j in range(d):
                a, b, _c, _e = P[j]
                M[j][h(i, a, b, w)] += abs(x)
    return M


def largest_mass_of(i, M, seed):
    """max over the rows j of M[j][h_j(i)]: the largest bucket mass that index i reads."""
    d, w = len(M), len(M[0])
    P = params(seed, d)
    return max(M[j][h(i, P[j][0], P[j][1], w)] for j in range(d))


def words_of(flags):
    n = len(flags)
    out = []
    for wd in range((n + 63) // 64):
        v = 0
        for bit in range(64):
            i = 64 * wd + bit
            if i < n and flags[i]:
                v |= 1 << bit
        out.append(v)
    return out


def aggregate(all_flags, all_S):
    n = len(all_flags[0])
    d, w = len(all_S[0]), len(all_S[0][0])
    C = [1 if any(f[i] for f in all_flags) else 0 for i in range(n)]
    S = [[sum(Sk[j][b] for Sk in all_S) for b in range(w)] for j in range(d)]
    return C, S


def median(xs):
    ys = sorted(xs)
    m = len(ys)
    if m % 2 == 1:
        return ys[m // 2]
    return 0.5 * (ys[m // 2 - 1] + ys[m // 2])


def decompress(C, S, seed):
    d, w = len(S), len(S[0])
    P = params(seed, d)
    out = {}
    for i, f in enumerate(C):
        if f:
            est = []
            for j in range(d):
                a, b, c, e = P[j]
                est.append(s(i, c, e) * S[j][h(i, a, b, w)])
            out[i] = median(est)
    return out


# ---- block-granular variant: the bitmap has one flag per block of B elements
def block_flags(g, B):
    """flags[x] = 1 iff some element of block x (g[xB .. xB+B), cut at len(g)) is non-zero."""
    n = len(g)
    out = []
    x = 0
    while x * B < n:
        out.append(1 if any(is_nonzero(g[i]) for i in range(x * B, min(n, x * B + B))) else 0)
        x += 1
    return out


def decompress_blocks(Cb, S, n, B, seed):
    """{block: [B estimates]} for every set block; positions at or beyond n hold 0.0."""
    d, w = len(S), len(S[0])
    P = params(seed, d)
    out = {}
    for x, f in enumerate(Cb):
        if not f:
            continue
        vals = []
        for o in range(B):
            i = x * B + o
            if i >= n:
                vals.append(0.0)
                continue
            est = []
            for j in range(d):
                a, b, c, e = P[j]
                est.append(s(i, c, e) * S[j][h(i, a, b, w)])
            vals.append(median(est))
        out[x] = vals
    return out
