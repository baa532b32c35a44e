"""The template syntax, pinned by hand: for each text below the byte sets and the literal bytes it
means are written out here as plain Python values, derived from the syntax rules alone (the
listing's notation: \\d digits, \\w word characters, \\s white space, \\xHH a byte, \\c the character
c, [a-z] a range, <eos> the end symbol, $name a bound argument), and both readers -- the oracle's
and the library's host compiler, which share no code -- have to agree with these values, not just
with each other."""
import pytest

import paper_2507_16768_amd as wg
from oracle import oracle as O

EOS = 256
DIGITS = set(range(0x30, 0x3A))
LOWER, UPPER = set(range(0x61, 0x7B)), set(range(0x41, 0x5B))

# (text, arguments, stay set, exit-A set, exit-B set or None, max or None) of the checkpoint the text starts with
CHECKPOINTS = [
    (r"Wait(allow={\d}, wait={;})", None, DIGITS, {ord(";")}, None, None),
    (r"Wait(allow={\w}, wait={\.})", None, DIGITS | LOWER | UPPER | {ord("_")}, {ord(".")}, None, None),
    (r"Wait(allow={\s}, wait={x})", None, {9, 10, 11, 12, 13, 32}, {ord("x")}, None, None),
    (r"Wait(allow={[a-cX-Z0-2]}, wait={\]})", None, set(b"abcXYZ012"), {ord("]")}, None, None),
    (r"Wait(allow={\x00, \xff, \x7F}, wait={\x0a})", None, {0, 255, 127}, {10}, None, None),
    (r"Wait(allow={\,, \ , \{, \}, \\}, wait={\"})", None, set(b", {}\\"), {ord('"')}, None, None),
    # denies: every byte but the denied ones stays, except the terminator, which leaves
    (r"Wait(denies={a, b, \n}, wait={<})", None, set(range(256)) - set(b"ab\n<"), {ord("<")}, None, None),
    (r"Wait(denies={}, wait={<, >})", None, set(range(256)) - set(b"<>"), set(b"<>"), None, None),
    # a terminator that is also allowed leaves: exactly one digit
    (r"Wait(allow={\d}, wait={\d})", None, set(), DIGITS, None, None),
    (r"Wait(allow={a}, wait={<eos>})", None, {ord("a")}, {EOS}, None, None),
    (r"Wait(allow=$a, wait={$b, !}, max=3)", {"a": b"xyz", "b": b"\x00\x01"}, set(b"xyz"), {0, 1, ord("!")}, None, 3),
    (r"Wait(allow={q}, wait={;}, max=0)", None, {ord("q")}, {ord(";")}, None, 0),
    (r'IfElse(condition=Wait(allow={\ }, true_waits={\[}, false_waits={\", \x27}), if_body=Write("a"), else_body=None)',
     None, {32}, {ord("[")}, {ord('"'), 0x27}, None),
    (r"DoWhile(body=None, condition=Wait(allow={}, true_waits={+}, false_waits={<eos>}))", None, set(), {ord("+")}, {EOS}, None),
]

# (text, arguments, the literal bytes of its Write states in order)
WRITES = [
    (r'Write("a\"b\\c\n\x41")', None, b'a"b\\c\nA'),
    (r'Write("a,b) c")', None, b"a,b) c"),
    (r'Sequence(Write("<p>"), Write($t), Write(""))', {"t": b"\x00\xfe{"}, b"<p>\x00\xfe{"),
    (r'Write("\t\r\x00")', None, b"\t\r\x00"),
]


@pytest.mark.parametrize("text,args,stay,exit_a,exit_b,mx", CHECKPOINTS)
def test_checkpoint_sets_mean_what_the_syntax_says(text, args, stay, exit_a, exit_b, mx):
    exit_b = exit_b or set()
    # the oracle's reader: one transition per symbol from the start state
    o = O.Oracle([text], [args] if args else None)
    s = o.start_state(0)
    d = o.describe(s)
    assert d["kind"] in ("WAIT", "COND") and d["max"] == (-1 if mx is None else mx)
    targets = {}
    for x in range(257):
        nx = o.step(s, 0, x)
        if x in stay and mx != 0:
            assert nx is not None and nx[0] == s, (text, x)
        elif x in exit_a or x in exit_b:
            assert nx is not None and (nx[0] != s or nx[1] == 0), (text, x)
            targets.setdefault("a" if x in exit_a else "b", set()).add(nx[0])
        else:
            assert nx is None, (text, x)                     # (max=0: an allowed byte has no budget left)
    assert all(len(v) == 1 for v in targets.values())      # one successor per exit
    if exit_b and EOS not in exit_b and EOS not in exit_a:
        assert targets["a"] != targets["b"]
    # the library's host compiler: the class of every symbol in the start state
    t = wg.Table([text], [args] if args else None, wg.EOS_STOP, 8)
    s2 = t.start_state(0)
    info = t.state(s2)
    assert info["kind"] == (3 if d["kind"] == "COND" else 2)
    assert info["max"] == (0xFFFFFFFF if mx is None else mx)
    for x in range(257):
        want = 1 if x in stay else 2 if x in exit_a else 3 if x in exit_b else 0
        if x == EOS:
            want = 2 if (x in exit_a or x in exit_b) else 0   # (which side an accepted <eos> takes is not a class)
        assert t.symbol_class(s2, x) == want, (text, x)


@pytest.mark.parametrize("text,args,data", WRITES)
def test_write_literals_mean_what_the_syntax_says(text, args, data):
    o = O.Oracle([text], [args] if args else None)
    t = wg.Table([text], [args] if args else None, wg.EOS_STOP, 8)
    assert o.num_states == t.num_states == len(data) + 2
    s, s2 = o.start_state(0), t.start_state(0)
    for y in data:
        assert o.describe(s)["kind"] == "LIT" and o.describe(s)["byte"] == y
        info = t.state(s2)
        assert info["kind"] == 1 and info["byte"] == y
        for x in (y, (y + 1) % 256, EOS):
            assert (o.step(s, 0, x) is not None) == (x == y)
            assert t.symbol_class(s2, x) == (2 if x == y else 0)
        s, s2 = o.describe(s)["next"], info["next_a"]
    assert o.describe(s)["kind"] == "END" and t.state(s2)["kind"] == 4
