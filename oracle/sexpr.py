"""TEST INFRASTRUCTURE ONLY -- the paper's program text, read and evaluated by the CPU oracle.

The listings of the paper (Figs. 2a-2c, 5 and 7; the rewrite rules of Figs. 3, 4 and 6) are
s-expressions over the transformers of Table 1 and the operators of Table 2.  `parse` reads such
text into nested Python lists; `evaluate` walks the lists and builds the corresponding
`oracle.access_pattern` nodes, one node per list, in the order they are written.  Nothing here
simplifies, fuses or reorders a program: a reader can follow a listing token by token.

Text conventions (the paper fixes no concrete syntax for literals):
  * a bare symbol that names a tensor is that tensor; any other symbol is looked up among the
    integer definitions (`C`, `Kh`, `Sh` ... of the listings), integers are themselves;
  * `(shape d0 d1 ...)` and `(list i0 i1 ...)` are tuples of integers;
  * `(reshape X (shape c...) (shape d...))` gives the access-pattern shape literal ((c...),(d...))
    of Table 1 as two tuples;
  * `(pad X dim lo hi)` is the zero-padding extension.
"""

from __future__ import annotations

from typing import Dict, List, Mapping, Union

import numpy as np

from . import access_pattern as ap

Tree = Union[str, int, List["Tree"]]

_OPERATORS = {"dotProd": ap.dotProd, "reduceSum": ap.reduceSum, "reduceMax": ap.reduceMax, "relu": ap.relu}


def parse(text: str) -> Tree:
    """One s-expression -> nested lists of symbols (str) and integers (int)."""
    tokens = text.replace("(", " ( ").replace(")", " ) ").split()
    pos = 0

    def read() -> Tree:
        nonlocal pos
        if pos >= len(tokens):
            raise ValueError("unexpected end of program")
        tok = tokens[pos]
        pos += 1
        if tok == "(":
            items: List[Tree] = []
            while pos < len(tokens) and tokens[pos] != ")":
                items.append(read())
            if pos >= len(tokens):
                raise ValueError("missing )")
            pos += 1
            return items
        if tok == ")":
            raise ValueError("unexpected )")
        try:
            return int(tok)
        except ValueError:
            return tok

    tree = read()
    if pos != len(tokens):
        raise ValueError("text after the end of the program")
    return tree


def to_text(tree: Tree) -> str:
    if isinstance(tree, list):
        return "(" + " ".join(to_text(t) for t in tree) + ")"
    return str(tree)


def evaluate(program: Union[str, Tree], tensors: Mapping[str, np.ndarray],
             ints: Mapping[str, int] = ()) -> ap.AP:
    """Build the access pattern a program denotes.  `tensors` maps names to arrays (int64 / float64
    values), `ints` the symbolic integers of the text."""
    tree = parse(program) if isinstance(program, str) else program
    ints = dict(ints)
    leaves: Dict[str, ap.AP] = {}

    def integer(t: Tree) -> int:
        if isinstance(t, int):
            return t
        if isinstance(t, str) and t in ints:
            return int(ints[t])
        raise ValueError(f"not an integer: {to_text(t)}")

    def tup(t: Tree, head: str):
        if not (isinstance(t, list) and t and t[0] == head):
            raise ValueError(f"expected ({head} ...), got {to_text(t)}")
        return tuple(integer(x) for x in t[1:])

    def ev(t: Tree) -> ap.AP:
        if isinstance(t, str):
            if t not in tensors:
                raise ValueError(f"unknown tensor {t}")
            if t not in leaves:
                leaves[t] = ap.tensor(np.asarray(tensors[t]))
            return leaves[t]
        if not isinstance(t, list) or not t or not isinstance(t[0], str):
            raise ValueError(f"not an access pattern: {to_text(t)}")
        head, args = t[0], t[1:]
        if head == "access":
            return ap.access(ev(args[0]), integer(args[1]))
        if head == "transpose":
            return ap.transpose(ev(args[0]), tup(args[1], "list"))
        if head == "cartProd":
            return ap.cart_prod(ev(args[0]), ev(args[1]))
        if head == "windows":
            return ap.windows(ev(args[0]), tup(args[1], "shape"), tup(args[2], "shape"))
        if head == "slice":
            return ap.slice_(ev(args[0]), integer(args[1]), integer(args[2]), integer(args[3]))
        if head == "squeeze":
            return ap.squeeze(ev(args[0]), integer(args[1]))
        if head == "flatten":
            return ap.flatten(ev(args[0]))
        if head == "reshape":
            return ap.reshape(ev(args[0]), tup(args[1], "shape"), tup(args[2], "shape"))
        if head == "pair":
            return ap.pair(ev(args[0]), ev(args[1]))
        if head == "concat":
            return ap.concat(ev(args[0]), ev(args[1]), integer(args[2]))
        if head == "pad":
            return ap.pad(ev(args[0]), integer(args[1]), integer(args[2]), integer(args[3]), 0)
        if head == "compute":
            if args[0] not in _OPERATORS:
                raise ValueError(f"unknown operator {args[0]}")
            return ap.compute(_OPERATORS[args[0]], ev(args[1]))
        if head == "systolicArray":
            return ap.systolic_array(integer(args[0]), integer(args[1]), ev(args[2]), ev(args[3]))
        raise ValueError(f"unknown transformer {head}")

    return ev(tree)
