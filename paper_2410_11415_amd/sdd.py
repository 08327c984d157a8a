"""Reader for sentential decision diagrams in the text format the SDD package writes
(the paper compiles its benchmark circuits to SDDs, Section 6):

    c <comment>
    sdd <number of nodes>
    F <id>                                     false
    T <id>                                     true
    L <id> <vtree id> <literal>                literal, +-(1-based variable)
    D <id> <vtree id> <k> {<prime id> <sub id>}*k      decision node: OR over AND(prime_i, sub_i)

A node may be listed before or after the nodes it refers to; the root is the one node that no
decision node refers to.  A decision node becomes an OR gate over one AND gate per element;
elements whose sub is false are dropped, a true prime or sub is left out of its AND, and a
decision node with a single remaining element is that element.  Input plumbing only: it produces
the arrays ``klay_build`` takes (paper Section 2: an NNF circuit as linked nodes).
"""
from __future__ import annotations

import numpy as np

LIT, AND, OR, TRUE, FALSE = 0, 1, 2, 3, 4


def parse_sdd(text: str, num_vars: int | None = None):
    """Returns ``(num_vars, node_type, node_lit, child_ptr, child_idx, roots)`` for ``Circuit(*...)``.

    ``num_vars`` defaults to the largest variable the file mentions."""
    lines = [ln.split() for ln in text.splitlines() if ln.strip() and not ln.lstrip().startswith("c")]
    if not lines or lines[0][0] != "sdd" or len(lines[0]) != 2:
        raise ValueError("not an sdd file: missing 'sdd <count>' header")
    count = int(lines[0][1])
    body = lines[1:]
    if len(body) != count:
        raise ValueError("sdd header announces %d nodes, file has %d" % (count, len(body)))
    raw = {}
    for ln, tok in enumerate(body, start=2):
        try:
            kind, sid = tok[0], int(tok[1])
            if kind in ("F", "T") and len(tok) == 2:
                rec = (kind,)
            elif kind == "L" and len(tok) == 4:
                lit = int(tok[3])
                if lit == 0:
                    raise ValueError
                rec = ("L", lit)
            elif kind == "D" and len(tok) >= 4 and len(tok) == 4 + 2 * int(tok[3]) and int(tok[3]) >= 1:
                refs = [int(x) for x in tok[4:]]
                rec = ("D", list(zip(refs[0::2], refs[1::2])))
            else:
                raise ValueError
        except (ValueError, IndexError):
            raise ValueError("line %d: malformed sdd node" % ln) from None
        if sid in raw:
            raise ValueError("line %d: node id %d defined twice" % (ln, sid))
        raw[sid] = rec
    referenced = set()
    for rec in raw.values():
        if rec[0] == "D":
            for pr, sb in rec[1]:
                if pr not in raw or sb not in raw:
                    raise ValueError("decision node refers to an undefined node")
                referenced.update((pr, sb))
    top = [sid for sid in raw if sid not in referenced]
    if len(top) != 1:
        raise ValueError("expected exactly one root, found %d unreferenced nodes" % len(top))

    node_type: list[int] = []
    node_lit: list[int] = []
    kids: list[list[int]] = []

    def new(t, lit=0, ch=()):
        node_type.append(t); node_lit.append(lit); kids.append(list(ch))
        return len(node_type) - 1

    out_id = {}
    # explicit stack: children before parents, whatever the order of the file
    stack = [(top[0], False)]
    state = {}
    while stack:
        sid, expanded = stack.pop()
        if sid in out_id:
            continue
        rec = raw[sid]
        if rec[0] == "F":
            out_id[sid] = new(FALSE)
        elif rec[0] == "T":
            out_id[sid] = new(TRUE)
        elif rec[0] == "L":
            out_id[sid] = new(LIT, rec[1])
        elif not expanded:
            if state.get(sid) == 1:
                raise ValueError("sdd nodes form a cycle")
            state[sid] = 1
            stack.append((sid, True))
            for pr, sb in rec[1]:
                for r in (pr, sb):
                    if r not in out_id:
                        if state.get(r) == 1:
                            raise ValueError("sdd nodes form a cycle")
                        stack.append((r, False))
        else:
            terms = []
            for pr, sb in rec[1]:
                if raw[sb][0] == "F" or raw[pr][0] == "F":
                    continue
                parts = [out_id[r] for r in (pr, sb) if raw[r][0] != "T"]
                if len(parts) == 2 and parts[0] == parts[1]:
                    parts = parts[:1]
                terms.append(new(TRUE) if not parts else parts[0] if len(parts) == 1 else new(AND, 0, parts))
            terms = list(dict.fromkeys(terms))
            out_id[sid] = new(FALSE) if not terms else terms[0] if len(terms) == 1 else new(OR, 0, terms)
            state[sid] = 2
    used = max((abs(l) for l in node_lit), default=0)
    if num_vars is None:
        num_vars = used
    elif used > num_vars:
        raise ValueError("file mentions variable %d, num_vars is %d" % (used, num_vars))
    child_ptr = np.zeros(len(kids) + 1, dtype=np.int64)
    child_ptr[1:] = np.cumsum([len(k) for k in kids])
    child_idx = np.asarray([c for k in kids for c in k], dtype=np.int32)
    return (int(num_vars), np.asarray(node_type, dtype=np.uint8), np.asarray(node_lit, dtype=np.int32), child_ptr,
            child_idx, np.array([out_id[top[0]]], dtype=np.int32))


def load_sdd(path: str, num_vars: int | None = None):
    with open(path) as f:
        return parse_sdd(f.read(), num_vars)
