"""Pins of the CPU oracle to things other than itself (no GPU, no HIP library).

Each test names what it pins: the paper's worked example against the host regex
library, closed forms, brute force over a structurally different interpreter,
numpy routines for packing and masking, and hand-derived conventions.
"""
import itertools
import os
import re

import numpy as np
import pytest

import wg_synth as ws
from oracle import brute
from oracle import oracle as O
from wg_synth.configs import TreeGen
from wg_synth.rng import Counter
from wg_synth.templates import EOS, CondWait, DoWhile, IfElse, Sequence, Wait, Write, bset
from wg_synth.vocab import from_tokens, tiny_vocab


def _ovocab(v):
    return O.OracleVocab(v.bytes, v.offsets, v.eos_id)


def _bits(row, V):
    return np.unpackbits(row.view(np.uint8), bitorder="little")[:V].astype(bool)


def _worked_text(golden_dir):
    with open(os.path.join(golden_dir, "worked_example_template.txt")) as f:
        return "".join(l for l in f if not l.startswith("#"))


_DIG = tuple(range(0x30, 0x3A))
WORKED_AST = Sequence((
    Wait(allow=_DIG, wait=_DIG),
    IfElse(
        condition=CondWait(allow=bset(_DIG, ".", EOS), true_waits=(EOS,), false_waits=bset(".")),
        if_body=None,
        else_body=DoWhile(
            body=Wait(allow=_DIG, wait=_DIG),
            condition=CondWait(allow=bset(_DIG, ".", EOS), true_waits=bset("."), false_waits=(EOS,)),
        ),
    ),
))


# ---- P1: the paper's worked example is the regex \d+(\.\d+)* ----------------------------

def test_worked_example_equals_regex(golden_dir):
    o = O.Oracle([_worked_text(golden_dir)])
    full = re.compile(rb"\d+(\.\d+)*")
    viable = re.compile(rb"(\d+(\.\d+)*\.?)?")        # prefixes of members of the language
    start = (o.start_state(0), 0)
    n_acc = 0
    for n in range(0, 9):
        for tup in itertools.product(b"01.x", repeat=n):
            w = bytes(tup)
            st = o.walk_bytes(start, w)
            assert (st is not None) == bool(viable.fullmatch(w)), w
            accepted = st is not None and o.step(st[0], st[1], EOS) == (O.SID_FINAL, 0)
            assert accepted == bool(full.fullmatch(w)), w
            n_acc += accepted
            # the structurally independent interpreter agrees on both questions
            assert brute.walkable(WORKED_AST, list(w)) == (st is not None), w
            assert (brute.classify(WORKED_AST, list(w) + [EOS]) == "closed") == accepted, w
    assert n_acc > 1000


def test_worked_example_typed_ast_serialises_to_same_machine(golden_dir):
    a = O.Oracle([_worked_text(golden_dir)])
    b = O.Oracle([ws.to_text(WORKED_AST)])
    assert a.num_states == b.num_states == 6            # FINAL + 4 leaves + END
    for s in range(a.num_states):
        assert a.describe(s) == b.describe(s)
        for x in list(b"09.x/:") + [EOS]:
            assert a.step(s, 0, x) == b.step(s, 0, x)


# ---- P2: non-greedy matching -----------------------------------------------------------

def test_non_greedy_wait_then_literal():
    o = O.Oracle(['Sequence(Wait(denies={}, wait={<}), Write("/b>"))'])
    full = re.compile(rb"[^<]*</b>")
    start = (o.start_state(0), 0)
    for n in range(0, 8):
        for tup in itertools.product(b"a</b>", repeat=n):
            w = bytes(tup)
            st = o.walk_bytes(start, w)
            accepted = st is not None and st[0] == o.end_state(0)
            assert accepted == bool(full.fullmatch(w)), w


def test_terminator_wins_over_allow():
    o = O.Oracle(["Sequence(Wait(allow={a, b}, wait={b}), Write(\"c\"))"])
    s0 = (o.start_state(0), 0)
    assert o.walk_bytes(s0, b"aab") == (s0[0] + 1, 0)    # first b leaves the Wait
    assert o.walk_bytes(s0, b"abb") is None             # second b meets the literal c
    assert o.walk_bytes(s0, b"abc") == (o.end_state(0), 0)


# ---- P3: literal states in closed form ---------------------------------------------------

def test_last_literal_admits_exactly_the_prefixes_of_its_remainder():
    w = ws.make_workload(1, V=8000)
    o = O.Oracle(w.texts, w.args, _ovocab(w.vocab))
    lit = w.args[0]["t2"]
    first = o.end_state(0) - len(lit)
    toks = [w.vocab.token(t) for t in range(w.vocab.V)]
    for p in (0, 1, len(lit) // 2, len(lit) - 1):
        rem = lit[p:]
        got = _bits(o.mask_row((first + p, 0)), w.vocab.V)
        want = np.array([len(t) > 0 and rem.startswith(t) for t in toks])
        assert (got == want).all()
        assert got.sum() >= 1


def test_inner_literal_closed_form():
    # literal R followed by a state n: t allowed iff t is a prefix of R, or t = R + u with u
    # allowed from n
    v = ws.make_vocab(6000, ("uniform", 1, 6), seed=3)
    o = O.Oracle(['Sequence(Write("ab"), Wait(allow={[a-z]}, wait={!}), Write("zz"))'], None, _ovocab(v))
    s0 = o.start_state(0)
    nxt = _bits(o.mask_row((s0 + 2, 0)), v.V)
    toks = [v.token(t) for t in range(v.V)]
    index = {}
    for t, b in enumerate(toks):
        index.setdefault(b, t)
    for p, rem in ((0, b"ab"), (1, b"b")):
        got = _bits(o.mask_row((s0 + p, 0)), v.V)
        for t, b in enumerate(toks):
            if len(b) == 0:
                want = False
            elif len(b) <= len(rem):
                want = rem.startswith(b)
            else:
                tail = b[len(rem):]
                # verdict of the tail from the next state: walk it directly
                want = b.startswith(rem) and o.walk_bytes((s0 + 2, 0), tail) is not None
                if tail in index:
                    assert (o.walk_bytes((s0 + 2, 0), tail) is not None) == nxt[index[tail]]
            assert got[t] == want, (p, b)


# ---- P4: Wait states in closed form --------------------------------------------------------

def test_wait_closed_form_and_terminator_crossing():
    v = ws.make_vocab(20000, ("geometric", 4, 16), seed=5, utf8_tenths=1)
    o = O.Oracle(['Sequence(Wait(denies={\\x00}, wait={<}), Write("div>"))'], None, _ovocab(v))
    got = _bits(o.mask_row((o.start_state(0), 0)), v.V)
    lit = b"div>"
    n_cross = 0
    for t in range(v.V):
        b = v.token(t)
        if t == v.eos_id or len(b) == 0:
            want = False
        else:
            j = b.find(b"<")
            head = b if j < 0 else b[:j]
            want = 0 not in head
            if want and j >= 0:                       # crosses the terminator: rest must be
                rest = b[j + 1:]                      # a prefix of the following literal, or
                want = lit.startswith(rest) if len(rest) <= len(lit) else False   # run past END
                n_cross += 1
        assert got[t] == want, b
    assert n_cross > 100


def test_never_exiting_wait_popcount():
    v = ws.make_vocab(20000, ("geometric", 4, 16), seed=6, utf8_tenths=1)
    # the terminator byte 0xFF never occurs inside a random token except as the single byte
    o = O.Oracle(["Wait(allow={[a-z], [0-9]}, wait={\\xFF})"], None, _ovocab(v))
    ok = set(b"abcdefghijklmnopqrstuvwxyz0123456789")
    want = sum(1 for t in range(v.V) if len(v.token(t)) and all(c in ok for c in v.token(t)))
    want += 1                                           # the single-byte token 0xFF itself
    assert int(_bits(o.mask_row((o.start_state(0), 0)), v.V).sum()) == want


def test_bounded_wait_budget():
    v = ws.make_vocab(5000, ("uniform", 1, 8), seed=7)
    o = O.Oracle(['Sequence(Wait(denies={}, wait={<}, max=5), Write("x"))'], None, _ovocab(v))
    s = o.start_state(0)
    for used in range(0, 7):
        got = _bits(o.mask_row((s, used)), v.V)
        left = max(0, 5 - used)
        for t in range(0, v.V, 7):
            b = v.token(t)
            if not b:
                want = False
            else:
                j = b.find(b"<")
                stay = len(b) if j < 0 else j
                want = stay <= left and (j < 0 or b[j + 1:] in (b"", b"x"))
            assert got[t] == want, (used, b)
    assert o.walk_bytes((s, 0), b"abcde") == (s, 5)
    assert o.walk_bytes((s, 0), b"abcdef") is None
    assert o.walk_bytes((s, 5), b"<") == (s + 1, 0)


# ---- P5: brute force on tiny vocabularies and random trees -------------------------------

ALPHA = b"ab<."


def _reach_states(o, tree, rng, n_prefix, restart):
    """Random walkable byte prefixes and the oracle states they lead to."""
    out = [((o.start_state(0), 0), [])]
    for _ in range(n_prefix):
        st, pre = (o.start_state(0), 0), []
        for _ in range(rng.between(1, 12)):
            x = rng.choice(list(ALPHA) + [EOS])
            nx = o.step(st[0], st[1], x)
            if nx is None:
                continue
            st, pre = nx, pre + [x]
        out.append((st, pre))
    return out


@pytest.mark.parametrize("restart", [False, True])
def test_masks_equal_brute_force_on_random_trees(restart):
    v = tiny_vocab(ALPHA, 3)                              # EOS + all 84 strings of length 1..3
    ov = _ovocab(v)
    rng = Counter(11, 2, start=1000 * restart)
    checked = 0
    for case in range(120):
        tree = TreeGen(rng, alphabet=ALPHA, max_depth=2, write_len=(1, 3), big=False).tree(2, 14)
        o = O.Oracle([ws.to_text(tree)], None, ov, restart=restart)
        assert o.num_states == ws.templates.count_leaves(tree) + 2
        for st, pre in _reach_states(o, tree, rng, 6, restart):
            assert brute.walkable(tree, pre, restart)
            got = _bits(o.mask_row(st), v.V)
            for t in range(v.V):
                syms = [EOS] if t == v.eos_id else list(v.token(t))
                want = brute.walkable(tree, pre + syms, restart)
                assert got[t] == want, (ws.to_text(tree), pre, syms)
                checked += 1
    assert checked > 30000


def test_soundness_and_completeness_of_token_paths():
    # Soundness: a sequence of allowed tokens concatenates to a walkable byte string.
    # Completeness: every walkable byte string is reachable through allowed tokens.
    v = tiny_vocab(ALPHA, 2)
    ov = _ovocab(v)
    rng = Counter(12, 2)
    for case in range(25):
        tree = TreeGen(rng, alphabet=ALPHA, max_depth=2, write_len=(1, 3), big=False).tree(2, 10)
        o = O.Oracle([ws.to_text(tree)], None, ov)
        reached = {b""}                                   # byte strings reachable by tokens, len<=4
        frontier = [((o.start_state(0), 0), b"")]
        while frontier:
            st, s = frontier.pop()
            bits = _bits(o.mask_row(st), v.V)
            for t in np.nonzero(bits)[0]:
                if t == v.eos_id:
                    continue
                s2 = s + v.token(int(t))
                if len(s2) > 4:
                    continue
                assert brute.walkable(tree, list(s2)), (ws.to_text(tree), s2)
                if s2 not in reached:
                    reached.add(s2)
                    frontier.append(((o.advance([st], [int(t)])[0][0], o.advance([st], [int(t)])[0][1]), s2))
        for n in range(1, 5):
            for tup in itertools.product(ALPHA, repeat=n):
                if brute.walkable(tree, list(tup)):
                    assert bytes(tup) in reached, (ws.to_text(tree), bytes(tup))


# ---- P6: a mask bit is set exactly when advance does not fail ----------------------------

def test_mask_bit_iff_advance_succeeds():
    w = ws.make_workload(5, V=3000)
    ov = _ovocab(w.vocab)
    o = O.Oracle(w.texts, w.args, ov, restart=True)
    rng = Counter(13, 2)
    for _ in range(12):
        sid = rng.between(0, o.num_states - 1)
        d = o.describe(sid)
        aux = rng.between(0, d["max"]) if d["kind"] == "WAIT" and d["max"] >= 0 else 0
        bits = _bits(o.mask_row((sid, aux)), w.vocab.V)
        toks = np.arange(w.vocab.V, dtype=np.int32)
        nxt = o.advance(np.tile(np.array([sid, aux], dtype=np.uint32), (w.vocab.V, 1)), toks)
        assert ((nxt[:, 0] != O.SID_ERROR) == bits).all()
    err = o.advance([[O.SID_ERROR, 0], [1, 0], [1, 0]], [5, -1, w.vocab.V])
    assert (err[:, 0] == O.SID_ERROR).all() and (err[:, 1] == 0).all()


# ---- P7 / P8: packing and masking against numpy --------------------------------------------

def test_mask_packing_matches_numpy_packbits():
    toks = [b""] + [bytes([65 + (i * 7) % 26]) for i in range(1, 77)]       # V = 77, ragged tail
    toks[10] = b""                                       # a byte-less token that is not EOS
    v = from_tokens(toks)
    o = O.Oracle(["Wait(allow={[A-M]}, wait={Z})"], None, _ovocab(v))
    row = o.mask_row((o.start_state(0), 0))
    verdict = np.array([len(t) == 1 and (65 <= t[0] <= 77 or t[0] == 90) for t in toks])
    want = np.packbits(verdict, bitorder="little")
    want = np.concatenate([want, np.zeros(-len(want) % 4, dtype=np.uint8)]).view("<u4")
    assert row.dtype == np.uint32 and len(row) == 3
    assert (row == want).all()
    assert row[2] >> (77 - 64) == 0                      # bits at and above V are zero
    assert not (row[0] >> 10) & 1 and verdict[9] and verdict[11]
    eos_ok = O.Oracle(["Wait(allow={[A-M]}, wait={<eos>})"], None, _ovocab(v))
    assert eos_ok.mask_row((1, 0))[0] & 1 and not (eos_ok.mask_row((1, 0))[0] >> 10) & 1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_apply_matches_numpy_where(dtype):
    B, V = 5, 1000 + 13
    W = (V + 31) // 32
    x = ws.make_logits(1, B, V, 2.0)
    x[0, 3], x[1, 4], x[2, 5], x[3, 6] = np.nan, -0.0, np.inf, 1e-42      # NaN, -0, inf, subnormal
    r = ws.rng.draw(2, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    r[4, :] = 0xFFFFFFFF
    bits = np.unpackbits(r.view(np.uint8).reshape(B, -1), axis=1, bitorder="little")[:, :V].astype(bool)
    if dtype == "f32":
        raw, ninf = x.view(np.uint32).copy(), np.uint32(0xFF800000)
        buf = x.copy()
        O.apply_mask(buf, r)
        got = buf.view(np.uint32)
        assert np.float32(-np.inf).view(np.uint32) == ninf
    else:
        raw, ninf = ws.to_bf16_bits(x), np.uint16(0xFF80)
        got = O.apply_mask(raw.copy(), r)
    want = np.where(bits, raw, ninf)
    assert (got == want).all()
    assert (got[4] == raw[4]).all()                      # all-ones row is the identity
    again = got.copy()
    if dtype == "f32":
        O.apply_mask(again.view(np.float32), r)
    else:
        O.apply_mask(again, r)
    assert (again == got).all()                          # idempotent


# ---- greedy choice under the mask, against numpy and hand-derived cases ---------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_masked_argmax_matches_numpy_on_ordinary_rows(dtype):
    B, V = 7, 3000 + 5
    W = (V + 31) // 32
    x = ws.make_logits(4, B, V, 2.0)
    m = ws.rng.draw(5, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[:, -1] &= (1 << (V % 32)) - 1
    bits = np.unpackbits(m.view(np.uint8).reshape(B, -1), axis=1, bitorder="little")[:, :V].astype(bool)
    if dtype == "bf16":
        raw = ws.to_bf16_bits(x)
        val = (raw.astype(np.uint32) << 16).view(np.float32)          # many ties after rounding
    else:
        raw, val = x, x
    want = np.argmax(np.where(bits, val.astype(np.float64), -np.inf), axis=1)   # first maximum
    assert (O.masked_argmax(raw, m) == want).all()


def test_masked_argmax_ties_nan_zero_and_empty_rows():
    inf, nan = np.inf, np.nan
    rows = np.array([
        [1.0, 5.0, 5.0, 2.0, 5.0, 0.0, 0.0, 0.0],      # tie between 1, 2, 4 -> 1
        [nan, nan, -inf, nan, 0.0, 0.0, 0.0, 0.0],     # -inf beats NaN -> 2 (4.. are masked off below)
        [nan, nan, nan, nan, 0.0, 0.0, 0.0, 0.0],      # only NaN allowed -> lowest allowed id
        [-0.0, 0.0, -1.0, -0.0, 9.0, 9.0, 9.0, 9.0],   # -0.0 equals +0.0 -> 0
        [3.0, 2.0, 1.0, 0.0, 0.0, 0.0, 0.0, 0.0],      # nothing allowed -> -1
        [1.0, 2.0, 3.0, inf, 4.0, inf, 0.0, nan],      # +inf, first of the two
    ], dtype=np.float32)
    mask = np.array([[0b00011111], [0b00001111], [0b00001010], [0b00001111], [0], [0b11111111]], dtype=np.uint32)
    want = [1, 2, 1, 0, -1, 3]
    assert O.masked_argmax(rows, mask).tolist() == want
    assert O.masked_argmax(ws.to_bf16_bits(np.nan_to_num(rows, nan=0.0)) | np.where(np.isnan(rows), 0x7FC0, 0).astype(np.uint16),
                           mask).tolist() == want


# ---- the k best allowed tokens, against numpy's stable sort and hand-derived cases -----------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("k", [1, 5, 64])
def test_masked_topk_matches_a_stable_sort_on_ordinary_rows(dtype, k):
    B, V = 5, 3000 + 5
    W = (V + 31) // 32
    x = ws.make_logits(6, B, V, 2.0)
    m = ws.rng.draw(7, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[:, -1] &= (1 << (V % 32)) - 1
    bits = np.unpackbits(m.view(np.uint8).reshape(B, -1), axis=1, bitorder="little")[:, :V].astype(bool)
    if dtype == "bf16":
        raw = ws.to_bf16_bits(x)
        val = (raw.astype(np.uint32) << 16).view(np.float32)          # many ties after rounding
    else:
        raw, val = x, x
    ids, vals = O.masked_topk(raw, m, k)
    for b in range(B):
        allowed = np.nonzero(bits[b])[0]
        order = allowed[np.argsort(-val[b, allowed].astype(np.float64), kind="stable")][:k]   # equal values: lower id first
        assert ids[b].tolist() == order.tolist()
        assert (vals[b] == raw[b, order]).all()
    if k == 1:
        assert (ids[:, 0] == O.masked_argmax(raw, m)).all()


def test_masked_topk_ties_nan_zero_and_short_rows():
    inf, nan = np.inf, np.nan
    rows = np.array([
        [1.0, 5.0, 5.0, 2.0, 5.0, 0.0, 0.0, 0.0],      # ties by id, then 3, then 0
        [nan, nan, -inf, nan, 0.0, 0.0, 0.0, 0.0],     # -inf before the NaNs, NaNs by id
        [-0.0, 0.0, -1.0, -0.0, 9.0, 9.0, 9.0, 9.0],   # the three zeros tie: by id
        [3.0, 2.0, 1.0, 0.0, 0.0, 0.0, 0.0, 0.0],      # nothing allowed
        [1.0, 2.0, 3.0, inf, 4.0, inf, 0.0, nan],      # +inf twice, NaN last
    ], dtype=np.float32)
    mask = np.array([[0b00011111], [0b00001111], [0b00001111], [0], [0b11111111]], dtype=np.uint32)
    want = [[1, 2, 4, 3, 0, -1], [2, 0, 1, 3, -1, -1], [0, 1, 3, 2, -1, -1], [-1] * 6, [3, 5, 4, 2, 1, 0]]
    ids, vals = O.masked_topk(rows, mask, 6)
    assert ids.tolist() == want
    ninf = np.array(-inf, dtype=np.float32).view(np.uint32)
    for b in range(len(rows)):
        for r in range(6):
            t = want[b][r]
            # the value is the element itself, bit for bit (a -0.0 stays -0.0, a NaN its payload)
            assert vals[b, r].view(np.uint32) == (rows[b, t].view(np.uint32) if t >= 0 else ninf)
    raw16 = ws.to_bf16_bits(np.nan_to_num(rows, nan=0.0)) | np.where(np.isnan(rows), 0x7FC0, 0).astype(np.uint16)
    ids16, vals16 = O.masked_topk(raw16, mask, 6)
    assert ids16.tolist() == want
    assert vals16[3].tolist() == [0xFF80] * 6 and vals16[4, 0] == 0x7F80
    # eight allowed tokens, k = 8: a permutation of them; k = 3: its first three
    ids8, _ = O.masked_topk(rows[4:5], mask[4:5], 8)
    assert ids8[0].tolist() == [3, 5, 4, 2, 1, 0, 6, 7]
    assert O.masked_topk(rows[4:5], mask[4:5], 3)[0][0].tolist() == [3, 5, 4]


# ---- P10: memoised trajectory masks equal fresh walks ---------------------------------------

def test_trajectory_is_consistent_with_unmemoised_calls():
    w = ws.make_workload(2, V=4000, B=6, steps=80)
    ov = _ovocab(w.vocab)
    o = O.Oracle(w.texts, w.args, ov, restart=True)
    start = np.array([[o.start_state(int(t)), 0] for t in w.request_template], dtype=np.uint32)
    draws = w.token_draws()
    toks, sts, nmemo = o.trajectory(start, draws)
    assert 1 <= nmemo <= 80 * 6
    cur = start.copy()
    for k in range(80):
        for b in range(6):
            row = o.mask_row(tuple(cur[b]))               # fresh walk, exact (sid, aux)
            pop = int(_bits(row, w.vocab.V).sum())
            assert pop >= 1
            assert toks[k, b] == np.nonzero(_bits(row, w.vocab.V))[0][int(draws[k, b] % np.uint64(pop))]
        cur = o.advance(cur, toks[k])
        assert (cur == sts[k]).all()
    assert (cur[:, 0] != O.SID_ERROR).all()


def test_budget_key_reduction_is_sound():
    # the remaining budget of a bounded Wait matters only below the longest token length
    v = ws.make_vocab(3000, ("uniform", 1, 8), seed=8)
    o = O.Oracle(['Sequence(Wait(denies={}, wait={<}, max=40), Write("q"))'], None, _ovocab(v))
    s = o.start_state(0)
    assert v.lmax == 8
    base = o.mask_row((s, 0))
    for aux in range(0, 41):
        rem = o.key_rem((s, aux))
        assert rem == min(40 - aux, 8)
        same = (o.mask_row((s, aux)) == base).all()
        assert same == (rem == 8) or (40 - aux >= 8)
        assert (o.mask_row((s, aux)) == o.mask_row((s, 40 - rem))).all()


# ---- forced continuation of a Write run (jump-forward) ---------------------------------------

def test_forced_bytes_of_a_hand_worked_tree():
    text = """
    Sequence(
      Write("ab"),
      Wait(allow={x}, wait={;}, body=Write("c")),
      IfElse(condition=Wait(allow={}, true_waits={t}, false_waits={f}),
             if_body=Write("T"), else_body=None),
      DoWhile(body=Sequence(Write(""), Write("d")),
              condition=Wait(allow={}, true_waits={+}, false_waits={.})),
      Write("")
    )"""
    o = O.Oracle([text, 'Sequence(Write("zq"), Write("r"))'])
    # ids: 1 a, 2 b, 3 Wait, 4 c, 5 cond, 6 T, 7 d, 8 loop cond, 9 END; template 1: 10 z, 11 q, 12 r, 13 END
    assert o.forced_bytes(1) == (b"ab", 3)                 # up to the Wait
    assert o.forced_bytes(2) == (b"b", 3)
    assert o.forced_bytes(3) == (b"", 3)                   # a Wait forces nothing
    assert o.forced_bytes(4) == (b"c", 5)                  # the Wait's body, then the condition
    assert o.forced_bytes(5) == (b"", 5)
    assert o.forced_bytes(6) == (b"Td", 8)                 # if_body runs on into the loop body
    assert o.forced_bytes(7) == (b"d", 8)
    assert o.forced_bytes(9) == (b"", 9)                   # END: only <eos> follows, no byte
    assert o.forced_bytes(10) == (b"zqr", 13)              # two Writes in a row are one run
    assert o.forced_bytes(10, cap=2) == (b"zq", 12)        # cut at cap: the state after what was written
    assert o.forced_bytes(10, cap=0) == (b"", 10)
    assert o.forced_bytes(0) == (b"", 0)
    assert o.forced_bytes(O.SID_ERROR) == (b"", O.SID_ERROR)
    assert o.forced_bytes(77) == (b"", 77)


@pytest.mark.parametrize("restart", [False, True])
def test_forced_bytes_are_the_only_walkable_continuation(restart):
    """Brute force on random trees: from every reachable state, each forced byte is the one symbol
    of the 257 the machine accepts there, the structural interpreter (no numbering, no state
    table) agrees on the prefix that led to the state, the run ends in the state the walk ends
    in, and that state is not a Write byte: the run is neither too short nor too long."""
    rng = Counter(13, 2, start=5000 * restart)
    seen_runs = 0
    for case in range(80):
        tree = TreeGen(rng, alphabet=ALPHA, max_depth=2, write_len=(0, 4), big=False).tree(2, 16)
        o = O.Oracle([ws.to_text(tree)], None, None, restart=restart)
        for st, pre in _reach_states(o, tree, rng, 10, restart):
            run, end = o.forced_bytes(st[0])
            kind = o.describe(st[0])["kind"] if st[0] < o.num_states else None
            assert (len(run) > 0) == (kind == "LIT")
            cur = st
            for i, y in enumerate(run):
                accepted = [x for x in range(257) if o.step(cur[0], cur[1], x) is not None]
                assert accepted == [y], (ws.to_text(tree), pre, run, i)
                for x in list(ALPHA) + [EOS]:              # the interpreter that knows no state ids
                    assert brute.walkable(tree, pre + list(run[:i]) + [x], restart) == (x == y)
                cur = o.step(cur[0], cur[1], y)
            assert cur[0] == end
            assert end >= o.num_states or o.describe(end)["kind"] != "LIT"
            if len(run) > 1:                                # a cap cuts the run, it does not change it
                assert o.forced_bytes(st[0], cap=len(run) - 1) == (run[:-1], o.walk_bytes(st, run[:-1])[0])
            seen_runs += len(run) > 0
    assert seen_runs > 100


# ---- conventions: numbering, restart, errors (self-consistency only) ------------------------

def test_canonical_numbering_of_a_hand_worked_tree():
    text = """
    Sequence(
      Write("ab"),
      Wait(allow={x}, wait={;}, body=Write("c")),
      IfElse(condition=Wait(allow={}, true_waits={t}, false_waits={f}),
             if_body=Write("T"), else_body=None),
      DoWhile(body=Sequence(Write(""), Write("d")),
              condition=Wait(allow={}, true_waits={+}, false_waits={.})),
      Write("")
    )"""
    o = O.Oracle([text, 'Write("z")'])
    # ids: 1 a, 2 b, 3 Wait, 4 c, 5 cond, 6 T, 7 d, 8 loop cond, 9 END; template 1: 10 z, 11 END
    kinds = [o.describe(s)["kind"] for s in range(o.num_states)]
    assert kinds == ["FINAL", "LIT", "LIT", "WAIT", "LIT", "COND", "LIT", "LIT", "COND", "END",
                     "LIT", "END"]
    assert o.start_state(0) == 1 and o.end_state(0) == 9
    assert o.start_state(1) == 10 and o.end_state(1) == 11
    assert [o.describe(s)["next"] for s in (1, 2, 3, 4, 6, 7, 10)] == [2, 3, 4, 5, 7, 8, 11]
    assert (o.describe(5)["tnext"], o.describe(5)["fnext"]) == (6, 7)     # None body: skip to loop
    assert (o.describe(8)["tnext"], o.describe(8)["fnext"]) == (7, 9)
    assert o.walk_bytes((1, 0), b"abxx;ctTd+d.") == (9, 0)
    assert o.walk_bytes((1, 0), b"ab;cfd.") == (9, 0)
    assert o.step(9, 0, EOS) == (0, 0) and o.step(9, 0, 65) is None
    assert o.step(0, 0, EOS) == (0, 0) and o.step(0, 0, 65) is None
    assert o.step(O.SID_ERROR, 0, EOS) is None


def test_restart_and_stop_after_eos():
    stop = O.Oracle(['Write("a")'])
    rest = O.Oracle(['Write("a")', "Wait(allow={b}, wait={<eos>})"], restart=True)
    assert stop.step(2, 0, EOS) == (0, 0)
    assert rest.step(2, 0, EOS) == (1, 0)
    assert rest.step(3, 0, EOS) == (3, 0)                # exit on <eos> re-arms template 1
    assert rest.step(3, 0, ord("b")) == (3, 0)


@pytest.mark.parametrize("text,frag", [
    ("IfElse(condition=Wait(allow={a}, true_waits={x}, false_waits={x}), if_body=None, else_body=None)", "overlap"),
    ("Sequence(Wait(allow={a}, wait={<eos>}), Write(\"b\"))", "follow"),
    ("Wait(allow={a, <eos>}, wait={b})", "eos"),
    ("Write($missing)", "unbound"),
    ("Wait(allow={a})", "wait="),
    ("Sequence(Write(\"a\")", "expected"),
    ("Frobnicate()", "unknown operator"),
    ("IfElse(condition=Wait(allow={}, wait={a}), if_body=None, else_body=None)", "condition"),
    ("Wait(allow={a}, denies={b}, wait={c})", "not both"),
    ("Write(\"a\") Write(\"b\")", "trailing"),
    ("Sequence(Wait(allow={a}, true_waits={x}, false_waits={y}))", "only valid inside"),
    ("Wait(allow={a}, true_waits={x}, false_waits={y})", "only valid inside"),
    ("Wait(allow={a}, wait={b}, body=Wait(allow={a}, true_waits={x}, false_waits={y}))", "only valid inside"),
])
def test_compile_errors(text, frag):
    with pytest.raises(O.OracleError) as e:
        O.Oracle([text])
    assert frag in str(e.value)


def test_set_syntax():
    o = O.Oracle([r"Wait(allow={\w, \., [x-z\]], \x41, \,, \ , $more}, wait={\n})"],
                 [{"more": b"#%"}])
    s = o.start_state(0)
    allowed = {x for x in range(256) if o.step(s, 0, x) == (s, 0)}
    want = set(b"abcdefghijklmnopqrstuvwxyzABCDEFGHIJKLMNOPQRSTUVWXYZ0123456789_.]A, #%")
    assert allowed == want
    assert o.step(s, 0, 10) == (o.end_state(0), 0)
