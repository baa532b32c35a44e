"""CPU-side checks of the HIP library: it loads, exports the declared ABI, and its host
operator compiler lowers templates to the same machine as the oracle (no kernel runs)."""
import os
import re

import pytest

import paper_2507_16768_amd as wg
import wg_synth as ws
from oracle import oracle as O
from wg_synth.configs import TreeGen
from wg_synth.rng import Counter

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KIND = {0: "FINAL", 1: "LIT", 2: "WAIT", 3: "COND", 4: "END"}


def test_library_exports_every_declared_symbol():
    with open(os.path.join(ROOT, "include", "wg.h")) as f:
        header = f.read()
    declared = set(re.findall(r"\b(wg_[a-z_]+)\s*\(", header))
    assert declared == set(wg.binding.EXPORTS)
    lib = wg.load_library()
    for name in sorted(declared):
        assert hasattr(lib, name), name


def test_topk_limits_are_checked_on_the_host_before_anything_is_launched():
    """Workspace size and argument checks of wg_masked_topk (the pointers are never followed)."""
    import ctypes as C
    L = wg.load_library()
    assert wg.masked_topk_workspace(1, 2000, 8) == 1 * 1 * 8 * 8
    assert wg.masked_topk_workspace(3, 8193, 64) == 3 * 2 * 64 * 8
    assert wg.masked_topk_workspace(256, 151936, 50) == 256 * 19 * 50 * 8
    p, need = C.c_void_p(16), L.wg_masked_topk_workspace(1, 2000, 8)
    bad = [dict(k=0), dict(k=65), dict(ws=need - 1), dict(work=C.c_void_p(20)), dict(work=None), dict(B=0),
           dict(B=65536, ws=1 << 40), dict(dtype=2), dict(stride=1999), dict(V=8192 * 65, stride=8192 * 65, k=64, ws=1 << 40)]
    for case in bad:
        a = dict(B=1, V=2000, stride=2000, k=8, ws=need, work=p, dtype=0)
        a.update(case)
        rc = L.wg_masked_topk(p, a["dtype"], a["B"], a["V"], a["stride"], p, a["k"], p, p, a["work"], a["ws"], None)
        assert rc == -1, case
        assert L.wg_last_error().startswith(b"wg_masked_topk"), case


def test_plain_c_client_builds_against_the_header():
    """tests/abi/c_client.c compiles as C11 against include/wg.h and links the library; without a
    GPU it says so and leaves with status 77 (with one it runs the whole comparison)."""
    import subprocess
    import __graft_entry__ as g
    exe = g.build_c_client()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode in (0, 77), (r.returncode, r.stdout[-300:], r.stderr[-600:])


def test_product_package_does_not_reach_for_the_oracle():
    pkg = os.path.join(ROOT, "paper_2507_16768_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".cpp", ".hip", ".h")):
                with open(os.path.join(dirpath, fn)) as f:
                    text = f.read()
                assert "oracle" not in text.lower(), fn
    for fn in os.listdir(os.path.join(ROOT, "oracle")):
        if fn.endswith((".py", ".c")):
            with open(os.path.join(ROOT, "oracle", fn)) as f:
                text = f.read()
            assert "paper_2507_16768_amd" not in text and "libwgrammar" not in text, fn


def _same_machine(texts, args, restart, lmax=8, table=None):
    o = O.Oracle(texts, args, None, restart=restart)
    t = table or wg.Table(texts, args, flags=wg.EOS_RESTART if restart else wg.EOS_STOP, lmax=lmax)
    assert t.num_states == o.num_states
    for i in range(len(texts)):
        assert t.start_state(i) == o.start_state(i)
    for sid in range(o.num_states):
        d, s = o.describe(sid), t.state(sid)
        assert KIND[s["kind"]] == d["kind"], sid
        assert s["tmpl"] == d["tmpl"]
        if d["kind"] == "LIT":
            assert (s["byte"], s["next_a"]) == (d["byte"], d["next"])
        if d["kind"] == "WAIT":
            assert s["max"] == (d["max"] if d["max"] >= 0 else 0xFFFFFFFF)
            assert s["n_keys"] == (lmax + 1 if d["max"] >= 0 else 1)
        for x in range(257):
            want = o.step(sid, 0, x)
            cls = t.symbol_class(sid, x)
            if d["kind"] == "WAIT" and d["max"] == 0 and cls == 1:
                assert want is None                      # max=0: the class says stay, the bound says no
            elif want is None:
                assert cls == 0, (sid, x)
            elif x == 256:
                assert cls == 2 and s["eos_next"] == want[0], (sid, x)
            elif cls == 1:
                assert want[0] == sid, (sid, x)
            else:
                assert cls in (2, 3) and want[0] == (s["next_a"] if cls == 2 else s["next_b"]), (sid, x)
    return t.num_states


def test_lowering_matches_oracle_on_workloads():
    for idx in (1, 2, 3):
        w = ws.make_workload(idx)
        _same_machine(w.texts, w.args, True, lmax=w.vocab.lmax)
    w = ws.make_workload(4, B=6, V=1000)
    _same_machine(w.texts, w.args, True, lmax=24)
    w = ws.make_workload(5, B=16, V=1000)
    assert _same_machine(w.texts, w.args, True, lmax=24) > 16 * 64


@pytest.mark.parametrize("restart", [False, True])
def test_lowering_matches_oracle_on_random_trees(restart, golden_dir):
    rng = Counter(21, 2, start=7 * restart)
    for _ in range(60):
        trees = [TreeGen(rng, alphabet=b"ab<.", max_depth=3, write_len=(0, 3), big=False).tree(1, 20)
                 for _ in range(rng.between(1, 3))]
        _same_machine([ws.to_text(t) for t in trees], None, restart)
    with open(os.path.join(golden_dir, "worked_example_template.txt")) as f:
        text = "".join(l for l in f if not l.startswith("#"))
    assert _same_machine([text], None, restart) == 6


def test_instances_appended_one_by_one_give_the_same_table():
    """Adding instances to a live table numbers them exactly as compiling them together does,
    and an add that fails to parse leaves nothing behind."""
    for idx, kw in ((3, {}), (5, dict(B=24, V=1000))):
        w = ws.make_workload(idx, **kw)
        lmax = 24
        t = wg.Table(w.texts[:1], w.args[:1] if w.args else None, flags=wg.EOS_RESTART, lmax=lmax)
        i = 1
        while i < len(w.texts):
            n_before = (t.num_states, t.n_templates)
            with pytest.raises(wg.WgError) as e:
                t.add_instances([w.texts[i], "Sequence(Wait(allow={q}, wait={z}), Frobnicate())"],
                                [w.args[i], {}] if w.args else None)
            assert e.value.code == -2 and "template 1" in str(e.value)
            assert (t.num_states, t.n_templates) == n_before
            step = 1 + i % 3
            t.add_instances(w.texts[i:i + step], w.args[i:i + step] if w.args else None)
            i += step
        assert t.n_templates == len(w.texts)
        _same_machine(w.texts, w.args, True, lmax=lmax, table=t)


def _language_equals_regex(rx, alphabet, max_len, extra=()):
    """The template made from `rx`, run by the oracle, accepts exactly what Python's re accepts."""
    import itertools
    import re
    text = wg.regex_to_template(rx)
    o = O.Oracle([text], None, None, restart=False)
    full = re.compile(rx.encode("latin-1") if isinstance(rx, str) else rx)
    start = (o.start_state(0), 0)
    n_acc = 0
    words = itertools.chain(extra, (bytes(t) for n in range(max_len + 1) for t in itertools.product(alphabet, repeat=n)))
    for w in words:
        st = o.walk_bytes(start, w)
        accepted = st is not None and o.step(st[0], st[1], 256) == (O.SID_FINAL, 0)
        assert accepted == bool(full.fullmatch(w)), (rx, text, w)
        n_acc += accepted
    return text, n_acc


@pytest.mark.parametrize("rx,alphabet,max_len,extra", [(c + ((),))[:4] for c in [
    (r"\d+(\.\d+)*", b"01.x", 8),                      # the paper's worked example
    (r'"[^"]*"', b'"a\\', 6),
    (r"ab(cd)?e", b"abcde", 7),
    (r"a(bc|de)f", b"abcdef", 5),
    (r"\[\d+(,\d+)*\]", b"[]1,", 8),
    (r"(ab)+c", b"abc", 8),
    (r"x{2,4}y", b"xy", 7),
    (r"[a-c]{1,3}", b"abcd", 5),
    (r"(ab){1,3}c", b"abc", 8),
    (r"a(b(c)?)?d", b"abcd", 5),
    (r"a(bc|d(e)?)f", b"abcdef", 5),
    (r"x(ab|c\d*)y", b"xabc1y", 6),
    (r"(a|b|c)d", b"abcd", 3),
    (r"a?b", b"ab", 4),
    (r"(ab)*", b"ab", 8),
    (r"", b"a", 2),
    (r"^\w+@\w+\.(com|org)$", b"a@.co", 5,
     (b"a@b.com", b"ab@c.org", b"a_1@b2.org", b"a@b.co", b"a@b.comm", b"@b.com", b"a@b.cog", b"a@@b.com", b"a@b.com.org")),
    (r"-?\d+", b"-12", 5),
    (r"\{\"k\":(true|false)\}", b'{}"k:tf', 4,
     (b'{"k":true}', b'{"k":false}', b'{"k":tru}', b'{"k":truefalse}', b'{"k":true}}', b'{"k":talse}')),
    (r"(?:\x41|\x42)+\n", b"AB\n", 5),
    (r"[^\s,]+(,[^\s,]+)*", b"a, b", 7),
]])
def test_regex_lowering_matches_the_host_regex_engine(rx, alphabet, max_len, extra):
    text, n_acc = _language_equals_regex(rx, alphabet, max_len, extra)
    assert n_acc > 0
    _same_machine([text], None, False)                  # and the library lowers its own output like the oracle


def test_regex_lowering_of_the_worked_example_is_the_listing(golden_dir):
    """The translation gives the paper's operator tree for its own example: same states, same
    byte classes, as the listing kept under tests/golden (the listing's redundant allow members
    aside, which no byte can reach because a wait member wins)."""
    with open(os.path.join(golden_dir, "worked_example_template.txt")) as f:
        listing = "".join(l for l in f if not l.startswith("#"))
    made = wg.Table([wg.regex_to_template(r"\d+(\.\d+)*")])
    paper = wg.Table([listing])
    assert made.num_states == paper.num_states == 6
    for sid in range(6):
        a, b = made.state(sid), paper.state(sid)
        assert {k: a[k] for k in ("kind", "next_a", "next_b", "eos_next")} == \
               {k: b[k] for k in ("kind", "next_a", "next_b", "eos_next")}, sid
        assert [made.symbol_class(sid, x) for x in range(257)] == [paper.symbol_class(sid, x) for x in range(257)]


def test_random_regexes_translate_to_their_own_language_or_are_refused():
    """Seeded random expressions over a small alphabet: whatever the translation accepts must
    mean what the host regex engine says it means; the rest must be refused with a parse error."""
    rng = Counter(77, 5)
    atoms = ["a", "b", "1", ",", "[ab]", "\\d", "[a1]"]

    def gen(depth):
        n = rng.between(1, 3)
        parts = []
        for _ in range(n):
            k = rng.between(0, 9)
            if depth < 2 and k >= 7:
                inner = gen(depth + 1)
                if rng.between(0, 2) == 0:
                    inner += "|" + gen(depth + 1)
                part = "(" + inner + ")"
            else:
                part = atoms[rng.between(0, len(atoms) - 1)]
            q = rng.between(0, 7)
            part += {0: "*", 1: "+", 2: "?", 3: "{1,2}"}.get(q, "")
            parts.append(part)
        return "".join(parts)

    ok = refused = 0
    for _ in range(400):
        rx = gen(0)
        try:
            _language_equals_regex(rx, b"ab1,", 6)
            ok += 1
        except wg.WgError as e:
            assert e.code == -2 and "regex" in str(e), rx
            refused += 1
    assert ok >= 60 and refused >= 60, (ok, refused)


@pytest.mark.parametrize("rx,frag", [
    (r"a*b*", "two repeated classes"),
    (r"(ab|cd|ef)", "three-way"),
    (r"(a|ab)", "same byte"),
    (r"(a*b)*c", "start with a single byte"),
    (r"a*a", "also matches"),
    (r"(a(bc)*)*d", "end of a repeated group"),
    (r"(ab)?(cd)?e", "followed by a single byte"),
    (r"(", "unbalanced"),
    (r"a{3,2}", "reversed"),
    (r"a+?", "lazy"),
    (r"\1", "back-references"),
    (r"[z-a]", "reversed range"),
    (r"*a", "nothing to repeat"),
    (r"a{2000}", "above 1000"),
    (r"[^\x00-\xff]", "no byte"),
])
def test_regex_lowering_refuses_what_the_operators_cannot_express(rx, frag):
    with pytest.raises(wg.WgError) as e:
        wg.regex_to_template(rx)
    assert e.value.code == -2 and frag in str(e.value), str(e.value)


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
])
def test_lowering_errors_are_reported_not_thrown(text, frag):
    with pytest.raises(wg.WgError) as e:
        wg.Table([text])
    assert e.value.code == -2 and frag in str(e.value)


def test_argument_checks_without_a_gpu():
    with pytest.raises(wg.WgError) as e:
        wg.Table([])
    assert e.value.code == -1
    with pytest.raises(wg.WgError):
        wg.Table(['Write("a")'], flags=8)
    with pytest.raises(ValueError):
        wg.Table(['Write("a")', 'Write("b")'], args=[{}])
    t = wg.Table(['Write($x)', 'Write($x)'], args=[{"x": b"ab"}, {"x": b"c"}])
    assert t.num_states == 1 + 3 + 2 and t.start_state(1) == 4
    with pytest.raises(wg.WgError):
        t.state(99)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
