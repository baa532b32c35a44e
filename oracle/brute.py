"""Brute-force interpreter over operator trees.  TEST INFRASTRUCTURE ONLY.

Walks a whole symbol string through a tree by structural recursion, with no leaf
numbering, no state table and no continuation links: an independent reading of
the operator semantics in the paper's section "Operator Building and State
Tracking" (Wait terminators first, IfElse / DoWhile built on a boolean Wait,
None bodies skipped) used to cross-check the C oracle on tiny inputs.
"""
from wg_synth.templates import EOS, CondWait, DoWhile, IfElse, Sequence, Wait, Write

REJECT, MORE = "reject", "more"       # otherwise: ("done", i) or ("eos", i)


def _allow_set(node):
    if isinstance(node, Wait) and node.denies is not None:
        return set(range(256)) - set(node.denies)
    return set(node.allow or ())


def _cond(node, s, i):
    """Boolean Wait: (True|False, i', took_eos), or REJECT / MORE."""
    allow = _allow_set(node)
    while True:
        if i == len(s):
            return MORE
        x = s[i]
        i += 1
        if x in node.true_waits:
            return (True, i, x == EOS)
        if x in node.false_waits:
            return (False, i, x == EOS)
        if x not in allow:
            return REJECT


def run(node, s, i):
    """Feed s[i:] to `node`.  ("done", j): node finished after consuming s[i:j];
    ("eos", j): an exit was taken on <eos>, which ends the whole output;
    MORE: input ran out inside the node without a rejection; REJECT."""
    if node is None:
        return ("done", i)
    if isinstance(node, Write):
        for b in node.data:
            if i == len(s):
                return MORE
            if s[i] != b:
                return REJECT
            i += 1
        return ("done", i)
    if isinstance(node, Wait):
        allow = _allow_set(node)
        stayed = 0
        while True:
            if i == len(s):
                return MORE
            x = s[i]
            i += 1
            if x in node.wait:
                if x == EOS:
                    return ("eos", i)
                return run(node.body, s, i)
            if x in allow and (node.max is None or stayed < node.max):
                stayed += 1
                continue
            return REJECT
    if isinstance(node, Sequence):
        for kid in node.children:
            r = run(kid, s, i)
            if r in (REJECT, MORE) or r[0] == "eos":
                return r
            i = r[1]
        return ("done", i)
    if isinstance(node, IfElse):
        c = _cond(node.condition, s, i)
        if c in (REJECT, MORE):
            return c
        truth, i, took_eos = c
        if took_eos:
            return ("eos", i)
        return run(node.if_body if truth else node.else_body, s, i)
    if isinstance(node, DoWhile):
        while True:
            r = run(node.body, s, i)
            if r in (REJECT, MORE) or r[0] == "eos":
                return r
            c = _cond(node.condition, s, r[1])
            if c in (REJECT, MORE):
                return c
            truth, i, took_eos = c
            if took_eos:
                return ("eos", i)
            if not truth:
                return ("done", i)
    raise TypeError(node)


def classify(tree, symbols, restart=False):
    """"reject" | "open" (walkable, output unfinished) | "closed" (ended by <eos>)."""
    s = list(symbols)
    i = 0
    while True:
        r = run(tree, s, i)
        if r == REJECT:
            return "reject"
        if r == MORE:
            return "open"
        kind, i = r
        if kind == "done":                      # template finished, <eos> not yet seen
            if i == len(s):
                return "open"
            if s[i] != EOS:
                return "reject"
            i += 1
        if restart:                             # <eos> re-arms the request at its start
            if i == len(s):
                return "closed"
            continue
        return "closed" if all(x == EOS for x in s[i:]) else "reject"


def walkable(tree, symbols, restart=False):
    return classify(tree, symbols, restart) != "reject"
