"""The five benchmark workloads as concrete seeded inputs.

They stand in for the paper's two production workloads (an HTML-like outline
whose tags are known in advance, and a JSON list of reference-lookup objects
with fixed keys and id-valued fields) at the logit width of a Qwen2.5-class
model.  No dataset, tokenizer file or benchmark item is read or reproduced:
every tag name, key and allow set is drawn from the counter-based generator.
"""
from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np

from .rng import STREAM_TEMPLATE, STREAM_TOKENS, Counter, draw
from .templates import (EOS, CondWait, DoWhile, Hole, IfElse, Sequence, Wait, Write, bset,
                        count_leaves, instantiate, to_text)
from .vocab import Vocab, make_vocab

CONFIG_NAMES = {1: "tiny", 2: "html", 3: "json", 4: "mixed", 5: "stress"}

_TAG_ALPHABET = b'abcdefghijklmnopqrstuvwxyz0123456789/ ="'
_KEY_ALPHABET = b"abcdefghijklmnopqrstuvwxyz_"


@dataclass
class Workload:
    index: int
    name: str
    vocab: Vocab
    texts: List[str]                   # one template text per template instance
    args: List[Dict[str, bytes]]       # runtime snippet arguments per instance
    asts: List[object]                 # the same instances as hole-free trees
    request_template: np.ndarray       # [B] instance index of each request
    B: int
    steps: int
    dtype: str                         # "f32" | "bf16"
    sigma: float
    selection: str                     # "argmax" | "stream"
    seed: int = 0
    notes: dict = field(default_factory=dict)

    def token_draws(self, steps=None):
        """uint64 [steps, B]: the seeded token stream (one draw per request-step)."""
        steps = self.steps if steps is None else steps
        k = np.arange(steps, dtype=np.uint64)[:, None]
        b = np.arange(self.B, dtype=np.uint64)[None, :]
        return draw(self.seed, STREAM_TOKENS, b * np.uint64(1 << 32) + k)


def _tag(rng, lo=8, hi=16):
    n = rng.between(lo, hi) - 2
    return b"<" + bytes(rng.choice(_TAG_ALPHABET) for _ in range(n)) + b">"


# ---- config 1 / 2 / 4a: HTML-like outline ------------------------------------------------

def html_template(n_tags, max_bytes):
    """tag0, then (free text up to '<', rest of next tag) repeated.

    A Wait consumes its terminator, so each tag after a Wait is written without
    its leading '<'.
    """
    kids = [Write(Hole("t0"))]
    for i in range(1, n_tags):
        kids.append(Wait(denies=(), wait=bset("<"), max=max_bytes))
        kids.append(Write(Hole("t%d" % i)))
    return Sequence(tuple(kids))


def html_args(rng, n_tags):
    args = {"t0": _tag(rng)}
    for i in range(1, n_tags):
        args["t%d" % i] = _tag(rng)[1:]
    return args


def tiny_template():
    return Sequence((Write(Hole("t0")), Wait(denies=(), wait=bset("<")),
                     Write(Hole("t1")), Write(Hole("t2"))))


# ---- config 3 / 4b: JSON reference lookup ------------------------------------------------

def json_template(max_bytes):
    obj = Sequence((
        Write(Hole("key")),
        IfElse(
            condition=CondWait(allow=bset(" "), true_waits=bset("["), false_waits=bset('"')),
            if_body=Wait(allow=Hole("idx"), wait=bset("]")),
            else_body=Wait(denies=(), wait=bset('"'), max=max_bytes),
        ),
        Write(b"}"),
    ))
    return Sequence((
        Write(b"["),
        DoWhile(body=obj,
                condition=CondWait(allow=bset(" "), true_waits=bset(","), false_waits=bset("]"))),
    ))


def json_args(rng, randomise):
    if randomise:
        n = rng.between(4, 10)
        key = bytes(rng.choice(_KEY_ALPHABET) for _ in range(n))
        extra = bytes(c for c in b" -.:" if rng.below(2))
    else:
        key, extra = b"reference", b""
    return {"key": b'{"' + key + b'":', "idx": b"0123456789," + extra}


# ---- config 5: random operator trees -----------------------------------------------------

_PRINTABLE = bytes(range(0x20, 0x7F))


class TreeGen:
    """Recursive seeded generator of valid operator trees over a byte alphabet.

    Validity kept by construction: true/false sets are disjoint, every Wait has a
    terminator, <eos> is never used inside a tree (the END state handles it), so
    no state is dead as long as the vocabulary holds the single-byte tokens.
    """

    def __init__(self, rng, alphabet=_PRINTABLE, max_depth=4, write_len=(2, 12), big=True):
        self.rng, self.alphabet, self.max_depth = rng, bytes(alphabet), max_depth
        self.write_len, self.big = write_len, big

    def rand_set(self, lo, hi, exclude=()):
        pool = [c for c in self.alphabet if c not in exclude]
        n = min(self.rng.between(lo, hi), len(pool))
        out = set()
        while len(out) < n:
            out.add(self.rng.choice(pool))
        return tuple(sorted(out))

    def cond(self):
        t = self.rand_set(1, 2 if self.big else 1)
        f = self.rand_set(1, 2 if self.big else 1, exclude=t)
        allow = self.rand_set(0, 6 if self.big else 1, exclude=t + f)
        return CondWait(allow=allow, true_waits=t, false_waits=f)

    def wait(self):
        rng = self.rng
        w = self.rand_set(1, 2 if self.big else 1)
        if self.big:
            mx = rng.between(16, 256) if rng.below(2) else None
        else:
            mx = rng.between(0, 3) if rng.below(2) else None
        if rng.below(2):
            return Wait(wait=w, denies=self.rand_set(0, 4 if self.big else 1, exclude=w), max=mx)
        return Wait(wait=w, allow=self.rand_set(4 if self.big else 0, 40, exclude=()), max=mx)

    def block(self, depth, room):
        """A Sequence of 1..4 children using at most `room` leaves (room >= 1)."""
        kids, used = [], 0
        for _ in range(self.rng.between(1, 4)):
            if room - used < 1:
                break
            kid = self.child(depth, room - used)
            kids.append(kid)
            used += count_leaves(kid)
        return Sequence(tuple(kids))

    def child(self, depth, room):
        rng = self.rng
        kind = rng.below(10)
        if depth > self.max_depth or room < 6:
            kind = kind % 5                       # leaves only
        if kind < 4:
            n = min(rng.between(*self.write_len), room)
            return Write(bytes(rng.choice(self.alphabet) for _ in range(n)))
        if kind < 6:
            return self.wait()
        if kind < 8:
            a = self.block(depth + 1, (room - 1) // 2) if rng.below(4) else None
            used = count_leaves(a)
            b = self.block(depth + 1, max(1, (room - 1 - used) // 2)) if rng.below(4) else None
            return IfElse(self.cond(), a, b)
        body = self.block(depth + 1, (room - 1) // 2) if (self.big or rng.below(4)) else None
        return DoWhile(body, self.cond())

    def tree(self, lo, hi):
        target = self.rng.between(lo, hi)
        kids, used = [], 0
        while used < target:
            kid = self.child(1, hi - used)
            kids.append(kid)
            used += count_leaves(kid)
        return Sequence(tuple(kids))


def stress_template(rng):
    return TreeGen(rng).tree(64, 256)


def nesting_depth(node):
    if isinstance(node, Sequence):
        return max([nesting_depth(c) for c in node.children] + [0])
    if isinstance(node, IfElse):
        return 1 + max(nesting_depth(node.if_body), nesting_depth(node.else_body))
    if isinstance(node, DoWhile):
        return 1 + nesting_depth(node.body)
    if isinstance(node, Wait):
        return nesting_depth(node.body)
    return 0


# ---- assembly ----------------------------------------------------------------------------

def make_workload(index, seed=0, B=None, steps=None, V=None):
    """Workload `index` in 1..5; B / steps / V may be overridden to shrink a test case."""
    rng = Counter(seed, STREAM_TEMPLATE, start=index << 24)
    if index == 1:
        vocab = make_vocab(V or 32000, ("uniform", 1, 8), seed)
        tpl = tiny_template()
        a = {"t0": _tag(rng), "t1": _tag(rng)[1:], "t2": _tag(rng)}
        trees, args = [tpl], [a]
        B0, steps0, dtype, sigma, sel = 1, 64, "f32", 1.0, "argmax"
        req = np.zeros(B or B0, dtype=np.int64)
    elif index == 2:
        vocab = make_vocab(V or 128256, ("geometric", 4, 16), seed, utf8_tenths=1)
        trees, args = [html_template(20, 256)], [html_args(rng, 20)]
        B0, steps0, dtype, sigma, sel = 64, 512, "bf16", 2.0, "stream"
        req = np.zeros(B or B0, dtype=np.int64)
    elif index == 3:
        vocab = make_vocab(V or 128256, ("geometric", 4, 16), seed, utf8_tenths=1)
        trees, args = [json_template(256)], [json_args(rng, False)]
        B0, steps0, dtype, sigma, sel = 128, 1024, "f32", 1.0, "stream"
        req = np.zeros(B or B0, dtype=np.int64)
    elif index == 4:
        vocab = make_vocab(V or 151936, ("geometric", 5, 24), seed, utf8_tenths=1)
        B0, steps0, dtype, sigma, sel = 256, 1024, "bf16", 2.0, "stream"
        nb = B or B0
        html, js = html_template(20, 256), json_template(256)
        trees, args = [], []
        for b in range(nb):                       # one template instance per request
            if b % 2 == 0:
                trees.append(html)
                args.append(html_args(rng, 20))
            else:
                trees.append(js)
                args.append(json_args(rng, True))
        req = np.arange(nb, dtype=np.int64)
    elif index == 5:
        vocab = make_vocab(V or 151936, ("geometric", 5, 24), seed, utf8_tenths=1)
        B0, steps0, dtype, sigma, sel = 1024, 4096, "bf16", 2.0, "stream"
        trees = [stress_template(rng) for _ in range(16)]
        args = [{} for _ in trees]
        req = np.arange(B or B0, dtype=np.int64) % 16
    else:
        raise ValueError("config index must be 1..5")
    texts = [to_text(t) for t in trees]
    asts = [instantiate(t, a) for t, a in zip(trees, args)]
    return Workload(index=index, name=CONFIG_NAMES[index], vocab=vocab, texts=texts, args=args,
                    asts=asts, request_template=req, B=B or B0, steps=steps or steps0,
                    dtype=dtype, sigma=sigma, selection=sel, seed=seed)
