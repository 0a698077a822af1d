"""A neutral, data-only description of a fused element-wise + reduce expression.

A GraphSpec is the *input* handed to an evaluator: a list of nodes in static single
assignment order (paper section 2.1.1: variables are produced by at most one apply node).
It evaluates nothing and knows no operation's meaning; the oracle and the GPU binding
each translate it into their own representation.

Conventions (shared by both evaluators because they are the problem statement):
  * every tensor operand has rank ``ndim``; ``bcast[d]`` true means dimension d is
    guaranteed to have extent 1 (the broadcastable pattern of section 2.1.1);
  * value types are "f32" (real) and "i32"; storage types are "f32", "f16", "i32";
  * ``reduce`` axes are numbered in the rank-``ndim`` space; with ``keep=False`` the reduced
    axes are dropped from the shape of an output computed from the result.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

UNARY = ("neg", "abs", "exp", "log", "log1p", "sqrt", "tanh", "sigmoid", "expm1", "sqr", "recip")
BINARY = ("add", "sub", "mul", "div", "max", "min", "pow", "gt", "ge", "lt", "le", "eq", "ne")
TERNARY = ("where",)
REDUCTIONS = ("sum", "max", "min", "prod", "argmax")
STORAGE = ("f32", "f16", "i32")
VALUE_TYPES = ("f32", "i32")


@dataclass
class GraphSpec:
    ndim: int
    nodes: List[tuple] = field(default_factory=list)
    outputs: List[Tuple[int, str]] = field(default_factory=list)
    n_inputs: int = 0
    n_scalars: int = 0

    def _push(self, node: tuple) -> int:
        self.nodes.append(node)
        return len(self.nodes) - 1

    def input(self, storage: str, bcast: Sequence[bool]) -> int:
        assert storage in STORAGE and len(bcast) == self.ndim
        k = self.n_inputs
        self.n_inputs += 1
        return self._push(("input", k, storage, tuple(bool(b) for b in bcast)))

    def scalar(self, vtype: str = "f32") -> int:
        assert vtype in VALUE_TYPES
        k = self.n_scalars
        self.n_scalars += 1
        return self._push(("scalar", k, vtype))

    def const(self, value: float, vtype: str = "f32") -> int:
        assert vtype in VALUE_TYPES
        return self._push(("const", vtype, float(value)))

    def iota(self, axis: int) -> int:
        assert 0 <= axis < self.ndim
        return self._push(("iota", axis))

    def apply(self, op: str, *args: int) -> int:
        arity = 1 if op in UNARY else 2 if op in BINARY else 3 if op in TERNARY else None
        assert arity is not None, op
        assert len(args) == arity, (op, args)
        return self._push(("apply", op, tuple(int(a) for a in args)))

    def cast(self, arg: int, storage: str) -> int:
        assert storage in STORAGE
        return self._push(("cast", int(arg), storage))

    def reduce(self, redop: str, arg: int, axes: Sequence[int], keep: bool = False) -> int:
        assert redop in REDUCTIONS
        return self._push(("reduce", redop, int(arg), tuple(int(a) for a in axes), bool(keep)))

    def grad(self, ys: Sequence[int], ybars: Sequence[int], wrt: Sequence[int]) -> List[int]:
        """Asks the evaluator's own differentiation for d(sum_k <ybar_k, y_k>)/d wrt_j; returns one
        value per wrt.  (Only the GPU library implements it; the oracle is given hand-derived
        gradient expressions or finite differences instead.)"""
        call = self._push(("grad", tuple(int(v) for v in ys), tuple(int(v) for v in ybars), tuple(int(v) for v in wrt)))
        return [self._push(("gradof", call, j)) for j in range(len(wrt))]

    def output(self, value: int, storage: str) -> None:
        assert storage in STORAGE
        self.outputs.append((int(value), storage))

    # sugar used by the workload descriptions
    def add(self, a, b): return self.apply("add", a, b)
    def sub(self, a, b): return self.apply("sub", a, b)
    def mul(self, a, b): return self.apply("mul", a, b)
    def div(self, a, b): return self.apply("div", a, b)
