"""Operator trees (the paper's Sequence / Write / Wait / IfElse / DoWhile) as data.

These classes only *describe* a template; nothing here steps an FSM.  `to_text`
serialises a tree into the textual syntax that both the oracle and the HIP
library parse on their own (the syntax of the paper's operator listing in the
section on operator building, extended with Write("..."), max=, denies=, $holes).
`instantiate` substitutes runtime snippet arguments for $holes.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple, Union

EOS = 256   # the end-of-sequence symbol; 0..255 are bytes


@dataclass(frozen=True)
class Hole:
    name: str


SetSpec = Union[Hole, Tuple[int, ...]]       # symbols 0..256, or a $hole


@dataclass(frozen=True)
class Write:
    data: Union[bytes, Hole]


@dataclass(frozen=True)
class Wait:
    wait: SetSpec
    allow: Optional[SetSpec] = None          # give allow or denies, not both
    denies: Optional[SetSpec] = None
    max: Optional[int] = None
    body: Optional[object] = None


@dataclass(frozen=True)
class CondWait:
    allow: SetSpec
    true_waits: SetSpec
    false_waits: SetSpec


@dataclass(frozen=True)
class IfElse:
    condition: CondWait
    if_body: Optional[object]
    else_body: Optional[object]


@dataclass(frozen=True)
class DoWhile:
    body: Optional[object]
    condition: CondWait


@dataclass(frozen=True)
class Sequence:
    children: Tuple[object, ...] = field(default_factory=tuple)


def bset(*items):
    """Build a symbol tuple from ints, bytes objects and str (latin-1) pieces."""
    out = []
    for it in items:
        if isinstance(it, int):
            out.append(it)
        elif isinstance(it, (bytes, bytearray)):
            out.extend(it)
        elif isinstance(it, str):
            out.extend(it.encode("latin-1"))
        else:
            out.extend(it)
    return tuple(sorted(set(out)))


def _set_text(s):
    if isinstance(s, Hole):
        return "$" + s.name
    parts = ["<eos>" if x == EOS else "\\x%02X" % x for x in s]
    return "{" + ", ".join(parts) + "}"


def _str_text(b):
    out = []
    for x in b:
        if x == 0x22:
            out.append('\\"')
        elif x == 0x5C:
            out.append("\\\\")
        elif 0x20 <= x < 0x7F and x != 0x24:     # keep '$' escaped to be safe
            out.append(chr(x))
        else:
            out.append("\\x%02X" % x)
    return '"' + "".join(out) + '"'


def to_text(node, indent=0):
    pad = "  " * indent
    if node is None:
        return pad + "None"
    if isinstance(node, Write):
        arg = "$" + node.data.name if isinstance(node.data, Hole) else _str_text(node.data)
        return pad + "Write(" + arg + ")"
    if isinstance(node, Wait):
        kw = []
        if node.allow is not None:
            kw.append("allow=" + _set_text(node.allow))
        if node.denies is not None:
            kw.append("denies=" + _set_text(node.denies))
        kw.append("wait=" + _set_text(node.wait))
        if node.max is not None:
            kw.append("max=%d" % node.max)
        s = pad + "Wait(" + ", ".join(kw)
        if node.body is not None:
            s += ",\n" + pad + "  body=\n" + to_text(node.body, indent + 2)
        return s + ")"
    if isinstance(node, CondWait):
        return (pad + "Wait(allow=" + _set_text(node.allow) + ", true_waits=" +
                _set_text(node.true_waits) + ", false_waits=" + _set_text(node.false_waits) + ")")
    if isinstance(node, IfElse):
        return (pad + "IfElse(\n" + pad + "  condition=\n" + to_text(node.condition, indent + 2) +
                ",\n" + pad + "  if_body=\n" + to_text(node.if_body, indent + 2) +
                ",\n" + pad + "  else_body=\n" + to_text(node.else_body, indent + 2) + ")")
    if isinstance(node, DoWhile):
        return (pad + "DoWhile(\n" + pad + "  body=\n" + to_text(node.body, indent + 2) +
                ",\n" + pad + "  condition=\n" + to_text(node.condition, indent + 2) + ")")
    if isinstance(node, Sequence):
        inner = ",\n".join(to_text(c, indent + 1) for c in node.children)
        return pad + "Sequence(\n" + inner + ")" if node.children else pad + "Sequence()"
    raise TypeError(node)


def _sub_set(s, args):
    if isinstance(s, Hole):
        return tuple(sorted(set(args[s.name])))
    return s


def instantiate(node, args):
    """Replace every $hole by its bytes (Write) or by the set of its bytes (sets)."""
    if node is None:
        return None
    if isinstance(node, Write):
        return Write(bytes(args[node.data.name])) if isinstance(node.data, Hole) else node
    if isinstance(node, Wait):
        return Wait(wait=_sub_set(node.wait, args),
                    allow=None if node.allow is None else _sub_set(node.allow, args),
                    denies=None if node.denies is None else _sub_set(node.denies, args),
                    max=node.max, body=instantiate(node.body, args))
    if isinstance(node, CondWait):
        return CondWait(_sub_set(node.allow, args), _sub_set(node.true_waits, args),
                        _sub_set(node.false_waits, args))
    if isinstance(node, IfElse):
        return IfElse(instantiate(node.condition, args), instantiate(node.if_body, args),
                      instantiate(node.else_body, args))
    if isinstance(node, DoWhile):
        return DoWhile(instantiate(node.body, args), instantiate(node.condition, args))
    if isinstance(node, Sequence):
        return Sequence(tuple(instantiate(c, args) for c in node.children))
    raise TypeError(node)


def count_leaves(node):
    """Number of leaf states a concrete (hole-free) tree occupies, END not included."""
    if node is None:
        return 0
    if isinstance(node, Write):
        return len(node.data)
    if isinstance(node, Wait):
        return 1 + count_leaves(node.body)
    if isinstance(node, CondWait):
        return 1
    if isinstance(node, IfElse):
        return 1 + count_leaves(node.if_body) + count_leaves(node.else_body)
    if isinstance(node, DoWhile):
        return 1 + count_leaves(node.body)
    if isinstance(node, Sequence):
        return sum(count_leaves(c) for c in node.children)
    raise TypeError(node)
