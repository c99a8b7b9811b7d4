"""Star-shaped loop bodies used to exercise the functor hook in two and three dimensions
(device side, written separately: star_bodies.hip).  Reads are ordered as everywhere in this
repository: v[0] = centre, then for the axes x, y, z in turn the offsets -R..-1, +1..+R.

soft_wave (radius 1, any dimension; made up for these tests): a wave step whose speed grows
with the amplitude,
    f(v, p) = 2 v0 + p (1 + BETA v0^2) L,    L = sum_axes (v- + v+) - 2 ndim v0 .
pair_product (2-D, radius 1): the paper's own example of an uninterpreted loop body
(Section 3.3.1), r[i,j] = f(a, b) with a = u[i-1,j], b = u[i,j-1] -- here i is the x index, j
the y index, and f(a, b) = a b + p a; the other three reads are unused.
lin_wave (radius R): the library's linear wave step without its u_prev term, as a body.
"""

BETA = 0.3


def soft_wave_f(v, p):
    nd = (len(v) - 1) // 2
    lap = sum(v[1:]) - 2.0 * nd * v[0]
    return 2.0 * v[0] + p * (1.0 + BETA * v[0] * v[0]) * lap


def soft_wave_df(v, p):
    nd = (len(v) - 1) // 2
    lap = sum(v[1:]) - 2.0 * nd * v[0]
    g = 1.0 + BETA * v[0] * v[0]
    d = [p * g] * len(v)
    d[0] = 2.0 + p * (2.0 * BETA * v[0] * lap - 2.0 * nd * g)
    return d


def pair_product_f(v, p):
    a, b = v[1], v[3]            # u at (x-1, y) and at (x, y-1)
    return a * b + p * a


def pair_product_df(v, p):
    a, b = v[1], v[3]
    return [0.0, b + p, 0.0, a, 0.0]


def lin_wave(weights):
    """weights[k], k = 0..R: per-axis second-derivative weights.  Returns (f, df)."""
    R = len(weights) - 1
    per_axis = [weights[abs(k)] for k in range(-R, R + 1) if k != 0]

    def table(nread):
        nd = (nread - 1) // (2 * R)
        return [nd * weights[0]] + per_axis * nd

    def f(v, p):
        w = table(len(v))
        return 2.0 * v[0] + p * sum(wk * vk for wk, vk in zip(w, v))

    def df(v, p):
        w = table(len(v))
        d = [p * wk for wk in w]
        d[0] += 2.0
        return d

    return f, df
