"""The host code under AddressSanitizer and UndefinedBehaviorSanitizer: the library's operator
compiler, regular-expression translator and vocabulary index builder and the C oracle are built with
-fsanitize=address,undefined into one driver (tests/sanitize/host_check.cpp) and run over
workload templates with arguments, random operator trees, malformed templates, incremental
adds with a failing add in between, and regular expressions.  Nothing here touches the GPU."""
import os
import shutil
import subprocess

import pytest

import wg_synth as ws
from wg_synth.configs import TreeGen
from wg_synth.rng import Counter
from wg_synth.vocab import from_tokens, make_vocab, tiny_vocab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _hex(b):
    b = b.encode("utf-8") if isinstance(b, str) else bytes(b)
    return b.hex() if b else "-"


def _case_file(path):
    lines = []
    v = tiny_vocab(b"ab<.1,\"", 2)

    def vocab(v, eos_id=None):
        lines.append("V %s %s %d" % (_hex(bytes(v.bytes)), ",".join(str(int(x)) for x in v.offsets),
                                     v.eos_id if eos_id is None else eos_id))

    # the static indexes of several vocabularies: token ranges that are empty, ragged or whole,
    # multi-byte characters, duplicate and byte-less tokens, no end-of-sequence token
    for big, eos in ((make_vocab(5000, ("geometric", 4, 16), seed=3, utf8_tenths=2), None), (make_vocab(2048, ("uniform", 1, 9), seed=4), None),
                     (make_vocab(16385, ("geometric", 5, 24), seed=5), -1), (from_tokens([b"", b"a", b"a", b"ab", b"", b"\xff\xff\xff"], 0), None),
                     (from_tokens([b"", b""], 1), None)):
        vocab(big, eos)
        lines.append("I")
    vocab(v)
    lines.append("I")

    def case(texts, args, flags, lmax, chunks=None):
        lines.append("C %d %d" % (flags, lmax))
        order = chunks or [list(range(len(texts)))]
        for chunk in order:
            for i in chunk:
                lines.append("T " + _hex(texts[i]))
                for k, val in (args[i] if args else {}).items():
                    lines.append("A %s %s" % (k, _hex(val)))
            lines.append("G")

    for idx, kw in ((1, {}), (2, dict(B=4, V=1000)), (3, dict(B=4, V=1000)), (4, dict(B=12, V=1000)),
                    (5, dict(B=16, V=1000))):
        w = ws.make_workload(idx, **kw)
        n = len(w.texts)
        case(w.texts, w.args, 1, 24)
        case(w.texts, w.args, 0, 8, chunks=[[i] for i in range(n)])       # one add per instance
        case(w.texts, w.args, 3, 24 if idx != 4 else 6, chunks=[[i] for i in range(n)])   # states of equal futures share keys
    rng = Counter(5, 2)
    for _ in range(60):
        trees = [TreeGen(rng, alphabet=b"ab<.", max_depth=3, write_len=(0, 3), big=False).tree(1, 20)
                 for _ in range(rng.between(1, 3))]
        case([ws.to_text(t) for t in trees], None, rng.between(0, 3), 8)
    bad = ["Sequence(Write(\"a\")", "Frobnicate()", "Wait(allow={a})", "Write($missing)", "Wait(allow={a, <eos>}, wait={b})",
           "Sequence(Wait(allow={a}, wait={<eos>}), Write(\"b\"))", "Wait(allow={[z-a]}, wait={b})", "Write(\"\\x4\")",
           "IfElse(condition=Wait(allow={a}, true_waits={x}, false_waits={x}), if_body=None, else_body=None)", "", "(",
           "Wait(allow={a}, wait={b}, max=99999999999)", "Sequence(" * 40]
    good = "Sequence(Write(\"ab\"), Wait(allow={a}, wait={b}, max=3))"
    lines.append("C 3 8")
    for b in bad[:4]:                                        # the same with shared keys: what a failed add numbered is taken back
        lines += ["T " + _hex(good), "G", "T " + _hex(good), "T " + _hex(b), "G"]
    lines.append("C 1 8")
    for b in bad:                                            # a failing add between good ones
        lines += ["T " + _hex(good), "G", "T " + _hex(good), "T " + _hex(b), "G"]
    for rx in [r"\d+(\.\d+)*", r'"[^"]*"', r"(ab){1,3}c", r"a(bc|d(e)?)f", r"x{2,4}y", r"", r"a*b*", r"(ab|cd|ef)",
               r"(", r"[", r"a{", r"a{1,", r"\x4", r"[a-", r"(?", r"\\", "\\", r"a{1000}", r"(a{30}){30}b", r"((((((a))))))",
               r"[^\x00-\xff]", r"(a|b|c|d|e)+f", r"[\d-z]"]:
        lines.append("R " + _hex(rx))
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    return len(lines)


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("gcc") is None, reason="needs gcc and g++")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    csrc = os.path.join(ROOT, "paper_2507_16768_amd", "csrc")
    objs = []
    for cc, std, src in (("gcc", "-std=c11", os.path.join(ROOT, "oracle", "wg_oracle.c")),
                         ("g++", "-std=c++17", os.path.join(csrc, "wg_lower.cpp")),
                         ("g++", "-std=c++17", os.path.join(csrc, "wg_regex.cpp")),
                         ("g++", "-std=c++17", os.path.join(csrc, "wg_vocab_index.cpp")),
                         ("g++", "-std=c++17", os.path.join(ROOT, "tests", "sanitize", "host_check.cpp"))):
        obj = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([cc, std, "-Wall"] + san + ["-c", src, "-o", obj], check=True, cwd=ROOT)
        objs.append(obj)
    exe = str(tmp_path / "host_check")
    subprocess.run(["g++"] + san + objs + ["-o", exe], check=True)
    cases = str(tmp_path / "cases.txt")
    assert _case_file(cases) > 400
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe, cases], capture_output=True, text=True, env=env, timeout=600)
    tail = (r.stdout[-1500:] + "\n" + r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "failures 0" in r.stdout and "MISMATCH" not in r.stdout, tail
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr and "LeakSanitizer" not in r.stderr, tail
    assert r.stdout.count("index ok ") == 6 and "INDEX" not in r.stdout, tail
    assert r.stdout.count("\nok ") > 100 and r.stdout.count("err") > 15, tail
