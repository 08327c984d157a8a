"""Reader for the decision-DNNF text format the d4 compiler writes (the compiler behind the paper's
d-DNNF benchmark circuits, Section 6):

    o <id> 0            OR node            a <id> 0            AND node
    t <id> 0            true               f <id> 0            false
    <parent> <child> <lit> ... <lit> 0     arc: under <parent>, the conjunction of <child> and the
                                           listed literals (+-(1-based variable); may be none)

Node ids are positive and declared before use; node 1 is the root.  An arc that carries literals
becomes an AND gate over the child and those literals (just the literals when the child is true); an
OR node's arcs are its alternatives, an AND node's arcs its factors.  A node without arcs is false
(OR) or true (AND).  Input plumbing only: it produces the arrays ``klay_build`` takes (paper
Section 2: an NNF circuit as linked nodes).
"""
from __future__ import annotations

import numpy as np

LIT, AND, OR, TRUE, FALSE = 0, 1, 2, 3, 4


def parse_d4(text: str, num_vars: int | None = None):
    """Returns ``(num_vars, node_type, node_lit, child_ptr, child_idx, roots)`` for ``Circuit(*...)``.

    ``num_vars`` defaults to the largest variable the file mentions."""
    kind = {}
    arcs: dict[int, list[tuple[int, list[int]]]] = {}
    for ln, line in enumerate(text.splitlines(), start=1):
        tok = line.split()
        if not tok or tok[0] == "c":
            continue
        try:
            if tok[0] in ("o", "a", "t", "f"):
                if len(tok) != 3 or tok[2] != "0":
                    raise ValueError
                nid = int(tok[1])
                if nid < 1 or nid in kind:
                    raise ValueError
                kind[nid] = tok[0]
                arcs[nid] = []
            else:
                nums = [int(x) for x in tok]
                if len(nums) < 3 or nums[-1] != 0 or 0 in nums[:-1]:
                    raise ValueError
                parent, child, lits = nums[0], nums[1], nums[2:-1]
                if kind.get(parent) not in ("o", "a") or child not in kind:
                    raise ValueError
                arcs[parent].append((child, lits))
        except ValueError:
            raise ValueError("line %d: malformed d4 line" % ln) from None
    if 1 not in kind:
        raise ValueError("no root: node 1 is not declared")

    node_type: list[int] = []
    node_lit: list[int] = []
    kids: list[list[int]] = []
    lit_node: dict[int, int] = {}

    def new(t, lit=0, ch=()):
        node_type.append(t); node_lit.append(lit); kids.append(list(ch))
        return len(node_type) - 1

    def literal(l):
        if l not in lit_node:
            lit_node[l] = new(LIT, l)
        return lit_node[l]

    out_id: dict[int, int] = {}
    state: dict[int, int] = {}
    stack = [(1, False)]
    while stack:
        nid, expanded = stack.pop()
        if nid in out_id:
            continue
        k = kind[nid]
        if k == "t":
            out_id[nid] = new(TRUE)
        elif k == "f":
            out_id[nid] = new(FALSE)
        elif not expanded:
            if state.get(nid) == 1:
                raise ValueError("d4 nodes form a cycle")
            state[nid] = 1
            stack.append((nid, True))
            for child, _ in arcs[nid]:
                if child not in out_id:
                    if state.get(child) == 1:
                        raise ValueError("d4 nodes form a cycle")
                    stack.append((child, False))
        else:
            terms = []
            for child, lits in arcs[nid]:
                parts = [literal(l) for l in dict.fromkeys(lits)]
                if kind[child] != "t":
                    parts.append(out_id[child])
                terms.append(new(TRUE) if not parts else parts[0] if len(parts) == 1 else new(AND, 0, parts))
            terms = list(dict.fromkeys(terms)) if k == "o" else terms
            if not terms:
                out_id[nid] = new(FALSE if k == "o" else TRUE)
            elif len(terms) == 1:
                out_id[nid] = terms[0]
            else:
                out_id[nid] = new(OR if k == "o" else AND, 0, list(dict.fromkeys(terms)))
            state[nid] = 2
    used = max((abs(l) for l in node_lit), default=0)
    if num_vars is None:
        num_vars = used
    elif used > num_vars:
        raise ValueError("file mentions variable %d, num_vars is %d" % (used, num_vars))
    child_ptr = np.zeros(len(kids) + 1, dtype=np.int64)
    child_ptr[1:] = np.cumsum([len(k) for k in kids])
    child_idx = np.asarray([c for k in kids for c in k], dtype=np.int32)
    return (int(num_vars), np.asarray(node_type, dtype=np.uint8), np.asarray(node_lit, dtype=np.int32), child_ptr,
            child_idx, np.array([out_id[1]], dtype=np.int32))


def load_d4(path: str, num_vars: int | None = None):
    with open(path) as f:
        return parse_d4(f.read(), num_vars)
