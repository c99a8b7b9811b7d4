"""The 3-D wave adjoint with the terms of every u_bar[j] added in the order of the
sequential scatter loop (paper Section 3.2 / 3.5), written with whole-array numpy
operations in the array's own dtype: one rounded product pair and one rounded addition
per term.  Output j receives at most one term per primal iteration, so visiting the
offsets in the order of their source cell (z-R..z-1, y-R..y-1, x-R..x-1, centre, x+1..,
y+1.., z+1..) gives every element exactly the sequence of additions the sequential loop
performs.  test_oracle_wave.py checks this against the oracle bit for bit in fp64; the
GPU tests use it as the fp32 reference of the library's scatter-order mode."""

from jacobians import star_weights


def wave3d_adjoint_scatter_order(c, r_bar, u_bar, radius):
    T = c.dtype.type
    R = radius
    w = [T(x) for x in star_weights(R)]
    nz, ny, nx = c.shape
    out = u_bar.copy()
    I = (slice(R, nz - R), slice(R, ny - R), slice(R, nx - R))
    cI, rI = c[I], r_bar[I]

    def shifted(axis, k):
        s = list(I)
        s[axis] = slice(R + k, c.shape[axis] - R + k)
        return tuple(s)

    def add(axis, k):          # source i in I, target i + k e_axis
        t = (cI * w[abs(k)]) * rI
        tgt = shifted(axis, k)
        out[tgt] = out[tgt] + t

    # target j = source + k e  <=>  source = j - k e: sources below j come first
    for axis in (0, 1, 2):                         # z, y, x: sources (.., j_axis - k), k = R..1
        for k in range(R, 0, -1):
            add(axis, k)
    out[I] = out[I] + (T(2) + cI * T(3) * w[0]) * rI
    for axis in (2, 1, 0):                         # x, y, z: sources (.., j_axis + k), k = 1..R
        for k in range(1, R + 1):
            add(axis, -k)
    return out
