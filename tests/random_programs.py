"""Seeded random access-pattern programs over the transformers of Table 1 and the operators of
Table 2, for the tests that feed one text to the CPU oracle and to the library.

A program is grown from a leaf `(access t n)` by a random walk over rules whose parameters are drawn
from the current shape, which the oracle's own shape rules supply (the candidate text is evaluated
on the small leaf tensors; a candidate the oracle rejects is dropped).  Nothing here knows how the
library evaluates anything."""

import numpy as np

from oracle import sexpr


def _shape(text, tensors):
    node = sexpr.evaluate(text, tensors)
    return node.shape, node.n_access


def grow(rng, tensors, same_shape, depth):
    """tensors: name -> int64 / float64 array; same_shape: name -> a second leaf of the same shape
    (for pair / concat / cartProd partners).  Returns the program text."""
    names = sorted(tensors)
    leaf = names[int(rng.integers(len(names)))]
    rank = tensors[leaf].ndim
    text = f"(access {leaf} {int(rng.integers(0, rank + 1))})"
    contracted = False

    def twin(t):
        """The same program on the sibling leaves: the same shape, other values."""
        out = []
        for tok in t.replace("(", " ( ").replace(")", " ) ").split():
            out.append(same_shape.get(tok, tok))
        return " ".join(out).replace("( ", "(").replace(" )", ")")

    for _ in range(depth):
        shape, na = _shape(text, tensors)
        nc = len(shape) - na
        rules = ["access", "transpose", "slice", "pad"]
        if len(shape) > 1 and 1 in shape:
            rules.append("squeeze")
        if nc >= 1 and all(d >= 2 for d in shape[na:]):
            rules.append("windows")
        if len(shape) >= 1:
            rules.append("flatten")
        rules += ["pair", "concat"]
        if not contracted and nc >= 1:
            rules += ["dot", "dot"]
        if nc >= 1:
            rules += ["reduceSum", "reduceMax"]
        rule = rules[int(rng.integers(len(rules)))]
        cand = None
        if rule == "access":
            cand = f"(access {text} {int(rng.integers(0, len(shape) + 1))})"
        elif rule == "transpose" and len(shape) >= 2:
            perm = rng.permutation(len(shape))
            cand = f"(transpose {text} (list {' '.join(str(int(p)) for p in perm)}))"
        elif rule == "slice" and len(shape) >= 1:
            d = int(rng.integers(len(shape)))
            if shape[d] >= 2:
                lo = int(rng.integers(0, shape[d] - 1))
                hi = int(rng.integers(lo + 1, shape[d] + 1))
                cand = f"(slice {text} {d} {lo} {hi})"
        elif rule == "pad" and len(shape) >= 1:
            d = int(rng.integers(len(shape)))
            cand = f"(pad {text} {d} {int(rng.integers(0, 3))} {int(rng.integers(0, 3))})"
        elif rule == "squeeze":
            ones = [i for i, v in enumerate(shape) if v == 1]
            cand = f"(squeeze {text} {ones[int(rng.integers(len(ones)))]})"
        elif rule == "windows":
            win = [int(rng.integers(1, min(d, 3) + 1)) for d in shape[na:]]
            st = [int(rng.integers(1, 3)) for _ in shape[na:]]
            cand = (f"(windows {text} (shape {' '.join(map(str, win))}) (shape {' '.join(map(str, st))}))")
        elif rule == "flatten":
            cand = f"(flatten {text})"
        elif rule in ("pair", "concat", "dot"):
            other = twin(text)
            if rule == "pair":
                cand = f"(pair {text} {other})"
            elif rule == "concat" and len(shape) >= 1:
                cand = f"(concat {text} {other} {int(rng.integers(len(shape)))})"
            elif rule == "dot":
                cand = f"(compute dotProd (cartProd {text} {other}))"
        elif rule in ("reduceSum", "reduceMax"):
            cand = f"(compute {rule} {text})"
        if cand is None:
            continue
        try:
            new_shape, _ = _shape(cand, tensors)
        except (ValueError, IndexError, KeyError):
            continue
        if int(np.prod(new_shape, dtype=np.int64)) > 200000 or len(new_shape) > 8:
            continue
        text = cand
        contracted = contracted or rule == "dot"
    return text
