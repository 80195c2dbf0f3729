"""Neuron-by-neuron bound propagation in pure Python -- TEST INFRASTRUCTURE ONLY (networks of a few neurons).

A brute-force cross-check of the C oracle: no matrices, no layers-as-tensors, just a table of neurons.  Its data
model is its own:

* a neuron is the pair (layer index, position), layer 0 being the input;
* an ``Expr`` is a constant plus a sparse map {neuron: coefficient};
* the certifier's state is ``shapes[layer][position]`` = ``Shape(l, u, L, U)`` -- real bounds and two ``Expr`` bounds,
  the abstract shape of Section 2.1 of the paper.

What is computed follows the paper: Appendix C gives the shape of every kind of neuron for DeepPoly, SkipPoly and
ReuseCert, Section 2.2 the meaning of substituting backwards until a stopping condition holds and of evaluating an
expression term by term, Section 6.2 the depth-limited variants.  ``certify`` walks the layers in order; the two
helpers ``push_down`` (repeated substitution of the deepest layer present) and ``evaluate`` (term-wise bound against
stored real bounds) do the rest.

Far too slow for anything but tiny networks.  Shares no code with the C oracle or the GPU library.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

Neuron = Tuple[int, int]

LOWER, UPPER = 0, 1


class Expr:
    """const + sum over terms of coefficient * neuron."""

    def __init__(self, const=0.0, terms: Optional[Dict[Neuron, float]] = None):
        self.const = float(const)
        self.terms = dict(terms or {})

    def plus(self, other: "Expr", factor: float = 1.0) -> "Expr":
        """self + factor * other."""
        t = dict(self.terms)
        for n, c in other.terms.items():
            t[n] = t.get(n, 0.0) + factor * c
        return Expr(self.const + factor * other.const, t)


class Shape:
    """Abstract shape of one neuron: l <= neuron <= u and L <= neuron <= U."""

    def __init__(self, l, u, L: Optional[Expr] = None, U: Optional[Expr] = None):
        self.l, self.u, self.L, self.U = l, u, L, U


def layer_expressions(layer, below: int, width: int) -> List[Expr]:
    """The expression each neuron of a non-ReLU layer equals, over the layer(s) it reads: weights . predecessors + bias
    (a convolution is that with its kernel laid out over the positions it touches, taps on the zero padding dropped);
    an Add layer (reading taken for residual networks) is the sum of the neuron below and the same position of layer
    ``layer.skip``."""
    if layer.kind == "add":
        return [Expr(0.0, {(below, i): 1.0}).plus(Expr(0.0, {(layer.skip, i): 1.0})) for i in range(width)]
    if layer.kind == "affine":
        rows, cols = layer.W.shape
        return [Expr(float(layer.b[r]), {(below, p): float(layer.W[r, p]) for p in range(cols)}) for r in range(rows)]
    Ci, H, W = layer.in_shape
    Co, _, kh, kw = layer.W.shape
    s, pad = layer.stride, layer.pad
    Ho, Wo = (H + 2 * pad - kh) // s + 1, (W + 2 * pad - kw) // s + 1
    out = []
    for co in range(Co):
        for ho in range(Ho):
            for wo in range(Wo):
                terms = {}
                for ci in range(Ci):
                    for ky in range(kh):
                        for kx in range(kw):
                            y, x = ho * s - pad + ky, wo * s - pad + kx
                            if 0 <= y < H and 0 <= x < W:
                                terms[(below, (ci * H + y) * W + x)] = float(layer.W[co, ci, ky, kx])
                out.append(Expr(float(layer.b[co]), terms))
    return out


def push_down(e: Expr, side: int, shapes, max_steps: int, floor: int) -> Expr:
    """Substitutes backwards: while the expression has terms on a layer above ``floor``, every term on the deepest such
    layer is replaced by coefficient * (L or U of that neuron): for a lower bound L under a coefficient >= 0 and U
    under a negative one, mirrored for an upper bound.  At most ``max_steps`` layers are replaced (< 0: no limit)."""
    steps = 0
    while max_steps < 0 or steps < max_steps:
        open_layers = [n[0] for n in e.terms if n[0] > floor]
        if not open_layers:
            break
        deepest = max(open_layers)
        out = Expr(e.const, {n: c for n, c in e.terms.items() if n[0] != deepest})
        for n, c in e.terms.items():
            if n[0] != deepest:
                continue
            sh = shapes[n[0]][n[1]]
            takes_lower = (c >= 0.0) == (side == LOWER)
            out = out.plus(sh.L if takes_lower else sh.U, c)
        e = out
        steps += 1
    return e


def evaluate(e: Expr, side: int, shapes) -> float:
    """Bound of an expression from the real bounds of the neurons it still mentions, term by term."""
    total = e.const
    for n, c in e.terms.items():
        sh = shapes[n[0]][n[1]]
        takes_lower = (c >= 0.0) == (side == LOWER)
        total += c * (sh.l if takes_lower else sh.u)
    return total


def certify(net, lo, hi, label=None, max_iters: int = -1, certifier: str = "deeppoly", max_iters_last=None):
    """lo, hi: sequences of length n0 (one input).  Returns (shapes, margins, verdict).

    certifier (all Appendix C): "deeppoly"; "skippoly" -- a ReLU neuron's L, U are written over the neurons two layers
    back, by scaling the L, U of the neuron under it; "reusecert" -- substitution never goes below layer 1's
    predecessors (the input), every affine layer between the first and the last keeps the substituted expressions as
    its L, U and leaves l, u at 0, and a ReLU neuron takes the real bounds it needs by evaluating the L, U of the
    neuron under it (each such neuron's Shape then also carries them as cl, cu).
    max_iters: limit on the layers replaced per substitution (Section 6.2); max_iters_last: the limit for the last
    layer and the property rows (default: max_iters); 0 with -1 is CROWN-IBP (Appendix C)."""
    assert certifier in ("deeppoly", "skippoly", "reusecert")
    shapes: List[List[Shape]] = [[Shape(float(a), float(b)) for a, b in zip(lo, hi)]]
    # terms on layers up to `floor` are never substituted: input neurons have no L, U; ReuseCert also stops at layer 1
    floor = 1 if certifier == "reusecert" else 0
    nl = len(net.layers)
    limit = max_iters

    def bound(e: Expr, side: int) -> float:
        return evaluate(push_down(e, side, shapes, limit, floor), side, shapes)

    for k, layer in enumerate(net.layers, start=1):
        under = shapes[k - 1]
        if k == nl and max_iters_last is not None:
            limit = max_iters_last
        row: List[Shape] = []
        if layer.kind == "relu":
            for i, p in enumerate(under):
                if certifier == "reusecert":
                    pl, pu = evaluate(p.L, LOWER, shapes), evaluate(p.U, UPPER, shapes)
                    p.cl, p.cu = pl, pu
                    l = u = 0.0
                    base_L, base_U = p.L, p.U
                else:
                    pl, pu = p.l, p.u
                    l, u = max(pl, 0.0), max(pu, 0.0)
                    itself = Expr(0.0, {(k - 1, i): 1.0})
                    base_L, base_U = (p.L, p.U) if certifier == "skippoly" else (itself, itself)
                # lower: the base expression when l + u >= 0, else 0; upper: the base when the neuron is always active,
                # 0 when never, else the chord through (l, 0) and (u, u).  A bound that is the constant 0 is held as
                # coefficient 0 on the base expression's neurons (the expression of a layer is one coefficient tensor over
                # the layer below, Section 3.2): a depth-limited substitution then still counts that layer as replaced, as
                # the C oracle's dense rows do.  Only networks with Add layers can tell the difference.
                L = base_L if pl + pu >= 0.0 else Expr(0.0).plus(base_L, 0.0)
                if pl >= 0.0:
                    U = base_U
                elif pu <= 0.0:
                    U = Expr(0.0).plus(base_U, 0.0)
                else:
                    slope = pu / (pu - pl)
                    U = Expr(-(pu * pl) / (pu - pl)).plus(base_U, slope)
                row.append(Shape(l, u, L, U))
        else:
            keeps_substituted = certifier == "reusecert" and 1 < k < nl
            assert not (keeps_substituted and layer.kind == "add")
            for e in layer_expressions(layer, k - 1, len(under)):
                if keeps_substituted:
                    row.append(Shape(0.0, 0.0, push_down(e, LOWER, shapes, limit, floor), push_down(e, UPPER, shapes, limit, floor)))
                else:
                    row.append(Shape(bound(e, LOWER), bound(e, UPPER), e, e))
        shapes.append(row)

    margins, verdict = None, None
    if label is not None:
        logits = layer_expressions(net.layers[-1], nl - 1, 0)
        margins = [bound(logits[label].plus(logits[o], -1.0), LOWER) for o in range(len(logits)) if o != label]
        verdict = int(all(m > 0.0 for m in margins))
    return shapes, margins, verdict
