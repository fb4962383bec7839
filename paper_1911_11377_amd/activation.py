"""Polynomial activations as sequences of library calls (argument marshalling only).

The paper replaces every non-linear activation by a low-degree polynomial (section 2.2
and the degree-2 polynomial of section 3.1).  Two schedules are provided:
  square : y = RS(Relin(x*x))                                          level l -> l-1
  poly3  : 0.5 + 0.25*y - 0.02*y^3 for y at level l, scale s_y          level l -> l-2
             y2 = RS(Relin(y*y))                       level l-1, scale s_2 = s_y^2/q_{l-1}
             t  = RS(y * round(-0.02*q_{l-1}))         level l-1, scale s_y   (scalar product and rescale in one call)
             y3 = RS(Relin(y2*t))                      level l-2, scale s_3 = s_2*s_y/q_{l-2}
             u  = RS(drop(y -> l-1) * round(0.25*s_2)) level l-2, scale s_y*s_2/q_{l-2} = s_3   (drop, product, rescale in one call)
             out = y3 + u + round(0.5*s_3)
  poly2  : c2*x^2 + c1*x (the degree-2 ReLU substitute of section 3.1) for x at level l, scale s   level l -> l-2
             x2 = RS(Relin(x*x))                       level l-1, scale s_2 = s^2/q_{l-1}
             t2 = RS(x2 * round(c2*q_{l-2}))           level l-2, scale s_2
             t1 = RS(drop(x -> l-1) * round(c1*(s_2/s)*q_{l-2}))   level l-2, scale s_2
             out = t2 + t1
The integer constants depend only on the moduli and the tracked scale.
"""
from dataclasses import dataclass

from . import ckksmi


@dataclass(frozen=True)
class Poly3Constants:
    c_m002: int
    c_025: int
    c_05: int
    out_scale: float


def poly3_constants(q, level, s_y):
    """q: list of ciphertext primes, level: level of y, s_y: its scale"""
    s_2 = s_y * s_y / q[level - 1]
    s_3 = s_2 * s_y / q[level - 2]
    return Poly3Constants(round(-0.02 * q[level - 1]), round(0.25 * s_2), round(0.5 * s_3), s_3)


# coefficients printed in section 3.1 for the polynomial that replaces ReLU
PAPER_POLY2 = (0.000469841857369822, 0.500000000000008)


@dataclass(frozen=True)
class Poly2Constants:
    k2: int
    k1: int
    out_scale: float


def poly2_constants(q, level, s, c2=PAPER_POLY2[0], c1=PAPER_POLY2[1]):
    """q: list of ciphertext primes, level: level of x, s: its scale"""
    s_2 = s * s / q[level - 1]
    return Poly2Constants(round(c2 * q[level - 2]), round(c1 * (s_2 / s) * q[level - 2]), s_2)


def workspace_bytes(ctx, level, batch):
    n = ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch)
    return n + 8 * batch * 2 * ctx.N * (4 * level)


def _carve(ws, words):
    """split a flat int64 torch tensor: first `words` elements, rest"""
    return ws[:words], ws[words:]


def square(ctx, x, evk, y, level, batch, ws, stream=None):
    ctx.hmul_relin_rescale(x, x, evk, y, level, batch, ws, stream=stream)


def poly3(ctx, y, evk, out, level, batch, consts, ws, stream=None):
    ct = batch * 2 * ctx.N
    y2, ws = _carve(ws, ct * (level - 1))
    t, ws = _carve(ws, ct * (level - 1))
    y3 = out
    ctx.hmul_relin_rescale(y, y, evk, y2, level, batch, ws, stream=stream)
    ctx.mul_scalar_rescale(y, consts.c_m002, t, level, batch, ws, stream=stream)
    ctx.hmul_relin_rescale(y2, t, evk, y3, level - 1, batch, ws, stream=stream)
    # u = RS(drop(y) * c) lands on y3 (= out) in the same pass: drop, product, rescale and sum in one call
    ctx.mul_scalar_rescale(y, consts.c_025, out, level - 1, batch, ws, stream=stream, level_in=level, addend=y3)
    ctx.add_const(out, consts.c_05, out, level - 2, batch, stream=stream)


def poly2(ctx, x, evk, out, level, batch, consts, ws, stream=None):
    """out (level-2) = c2*x^2 + c1*x; ws as sized by workspace_bytes(ctx, level, batch)"""
    ct = batch * 2 * ctx.N
    x2, ws = _carve(ws, ct * (level - 1))
    ctx.hmul_relin_rescale(x, x, evk, x2, level, batch, ws, stream=stream)
    ctx.mul_scalar_rescale(x2, consts.k2, out, level - 1, batch, ws, stream=stream)
    # t1 = RS(drop(x) * k1) is added to t2 (in out) by the same pass
    ctx.mul_scalar_rescale(x, consts.k1, out, level - 1, batch, ws, stream=stream, level_in=level, addend=out)

