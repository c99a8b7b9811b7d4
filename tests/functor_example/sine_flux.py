"""A made-up nonlinear three-point loop body with a passive coefficient, used to show
that a new stencil needs only a functor (see sine_flux.hip for the device side, written
separately).  The derivative of sin is the statement-level rule of paper Section 3.1.

    f(um, u0, up, p) = u0 + p (sin(up) - sin(um)) u0 + um up / 2
"""
import math


def f(um, u0, up, p):
    return u0 + p * (math.sin(up) - math.sin(um)) * u0 + 0.5 * um * up


def df(um, u0, up, p):
    dm = -p * math.cos(um) * u0 + 0.5 * up
    d0 = 1.0 + p * (math.sin(up) - math.sin(um))
    dp = p * math.cos(up) * u0 + 0.5 * um
    return dm, d0, dp
