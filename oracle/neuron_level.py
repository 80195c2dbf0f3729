"""Neuron-level DeepPoly in pure Python -- TEST INFRASTRUCTURE ONLY (tiny nets).

A literal transcription of the DeepPoly specification (paper, Appendix C) under
the operational semantics of ``map`` and ``traverse`` (Sections 2.2, 3.2, 4.2):
a polyhedral expression is a constant plus a dictionary {neuron: coefficient},
a neuron is the pair (layer index, position), ``traverse`` is a while loop that
repeatedly takes the not-yet-stopped neurons of highest priority and replaces
each by the user function's result, ``map`` applies the user function to every
(neuron, coefficient) pair, sums the results and adds the constant back.

It exists to cross-check the C oracle by brute force on networks of a few
neurons; it is far too slow for anything else.  Shares no code with either the
C oracle or the GPU library.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

Neuron = Tuple[int, int]          # (layer index, position); layer 0 = input


class PolyExp:
    def __init__(self, const=0.0, terms: Dict[Neuron, float] = None):
        self.const = float(const)
        self.terms = dict(terms or {})

    def add(self, other: "PolyExp") -> "PolyExp":
        t = dict(self.terms)
        for n, c in other.terms.items():
            t[n] = t.get(n, 0.0) + c
        return PolyExp(self.const + other.const, t)

    def scale(self, k: float) -> "PolyExp":
        return PolyExp(self.const * k, {n: c * k for n, c in self.terms.items()})


class Shape:
    """Abstract shape (l, u, L, U) of one neuron."""
    def __init__(self, l, u, L=None, U=None):
        self.l, self.u, self.L, self.U = l, u, L, U


def _affine_rows(layer, n_prev_layer_index, n_prev=None):
    """prev.dot(curr[weight]) + curr[bias] for every neuron of an affine/conv layer; for an Add layer (reading: the
    Affine transformer with unit weights over its two predecessors) prev0 + prev1."""
    rows = []
    if layer.kind == "add":
        for i in range(n_prev):
            e = PolyExp(0.0, {(n_prev_layer_index, i): 1.0})
            rows.append(e.add(PolyExp(0.0, {(layer.skip, i): 1.0})))
        return rows
    if layer.kind == "affine":
        for r in range(layer.W.shape[0]):
            rows.append(PolyExp(float(layer.b[r]),
                                {(n_prev_layer_index, p): float(layer.W[r, p]) for p in range(layer.W.shape[1])}))
        return rows
    Ci, H, W = layer.in_shape
    Co, _, kh, kw = layer.W.shape
    s, pad = layer.stride, layer.pad
    Ho = (H + 2 * pad - kh) // s + 1
    Wo = (W + 2 * pad - kw) // s + 1
    for co in range(Co):
        for ho in range(Ho):
            for wo in range(Wo):
                t = {}
                for ci in range(Ci):
                    for ky in range(kh):
                        for kx in range(kw):
                            hi, wi = ho * s - pad + ky, wo * s - pad + kx
                            if 0 <= hi < H and 0 <= wi < W:
                                t[(n_prev_layer_index, (ci * H + hi) * W + wi)] = float(layer.W[co, ci, ky, kx])
                rows.append(PolyExp(float(layer.b[co]), t))
    return rows


def certify(net, lo, hi, label=None, max_iters: int = -1, certifier: str = "deeppoly", max_iters_last=None):
    """lo, hi: sequences of length n0 (one input).  Returns (shapes, margins, verdict)
    where shapes[layer][pos] is a Shape.

    certifier: "deeppoly"; "skippoly" (Appendix C, SkipPoly: the ReLU transformer writes L, U over the neurons two
    layers back by scaling the predecessor's own L, U); "reusecert" (Appendix C, ReuseCert: stop_traverse(n) =
    n[layer] <= 1, middle affine layers store the traversed expressions as L, U and leave l, u at 0, the ReLU
    transformer concretises the predecessor's stored L, U itself; each Shape of an affine layer additionally
    carries cl, cu = that concretisation).  max_iters_last: iteration limit of the last layer's traversals and the
    property rows (default: max_iters); max_iters = 0 with max_iters_last = -1 is CROWN-IBP (Appendix C)."""
    assert certifier in ("deeppoly", "skippoly", "reusecert")
    shapes: List[List[Shape]] = [[Shape(float(a), float(b)) for a, b in zip(lo, hi)]]

    def map_(e: PolyExp, f) -> PolyExp:
        out = PolyExp(e.const)
        for n, c in e.terms.items():
            out = out.add(f(n, c))
        return out

    limit = [max_iters]

    def traverse(e: PolyExp, priority, stop, f) -> PolyExp:
        iters = 0
        while True:
            active = [n for n in e.terms if not stop(n) and n[0] > 0]   # input neurons have no L/U
            if not active or (limit[0] >= 0 and iters >= limit[0]):
                return e
            best = max(priority(n) for n in active)
            chosen = {n for n in active if priority(n) == best}
            out = PolyExp(e.const, {n: c for n, c in e.terms.items() if n not in chosen})
            for n in chosen:
                out = out.add(f(n, e.terms[n]))
            e = out
            iters += 1

    S = lambda n: shapes[n[0]][n[1]]
    simplify_lower = lambda n, c: PolyExp(c * S(n).l if c >= 0.0 else c * S(n).u)
    simplify_upper = lambda n, c: PolyExp(c * S(n).u if c >= 0.0 else c * S(n).l)
    replace_lower = lambda n, c: (S(n).L if c >= 0.0 else S(n).U).scale(c)
    replace_upper = lambda n, c: (S(n).U if c >= 0.0 else S(n).L).scale(c)
    # backward traversal visits the deepest layer first; with a bounded iteration
    # count the traversal stops early and simplify_* uses the stored l, u reached
    priority2 = lambda n: n[0]
    stop_traverse = (lambda n: n[0] <= 1) if certifier == "reusecert" else (lambda n: False)
    backsubs_lower = lambda e: map_(traverse(e, priority2, stop_traverse, replace_lower), simplify_lower).const
    backsubs_upper = lambda e: map_(traverse(e, priority2, stop_traverse, replace_upper), simplify_upper).const

    nl = len(net.layers)
    for k, layer in enumerate(net.layers, start=1):
        prev = shapes[k - 1]
        cur = []
        if k == nl and max_iters_last is not None:
            limit[0] = max_iters_last
        if layer.kind == "relu":
            for i, p in enumerate(prev):
                n = PolyExp(0.0, {(k - 1, i): 1.0})
                if certifier == "reusecert":
                    # Relu -> (0, 0, relu_n(prev[L].map(simplify_lower), prev[U].map(simplify_upper), prev), compute_upper(...))
                    pl = map_(p.L, simplify_lower).const
                    pu = map_(p.U, simplify_upper).const
                    p.cl, p.cu = pl, pu
                    l, u, below_L, below_U = 0.0, 0.0, p.L, p.U
                else:
                    pl, pu = p.l, p.u
                    l = pl if pl >= 0.0 else 0.0
                    u = pu if pu >= 0.0 else 0.0
                    below_L, below_U = (p.L, p.U) if certifier == "skippoly" else (n, n)
                L = below_L if pl + pu >= 0.0 else PolyExp(0.0)
                if pl >= 0.0:
                    U = below_U
                elif pu <= 0.0:
                    U = PolyExp(0.0)
                else:
                    U = below_U.scale(pu / (pu - pl)).add(PolyExp(-(pu * pl) / (pu - pl)))
                cur.append(Shape(l, u, L, U))
        elif certifier == "reusecert" and not (k == 1 or k == nl):
            assert layer.kind != "add"
            for e in _affine_rows(layer, k - 1):
                cur.append(Shape(0.0, 0.0, traverse(e, priority2, stop_traverse, replace_lower),
                                 traverse(e, priority2, stop_traverse, replace_upper)))
        else:
            for e in _affine_rows(layer, k - 1, len(prev)):
                cur.append(Shape(backsubs_lower(e), backsubs_upper(e), e, e))
        shapes.append(cur)

    margins, verdict = None, None
    if label is not None:
        last = net.layers[-1]
        rows = _affine_rows(last, len(net.layers) - 1)
        margins = []
        for o in range(len(rows)):
            if o == label:
                continue
            margins.append(backsubs_lower(rows[label].add(rows[o].scale(-1.0))))
        verdict = int(all(m > 0.0 for m in margins))
    return shapes, margins, verdict
