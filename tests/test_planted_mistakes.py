"""The pins of the oracle are worth what they catch: each plausible mistake below is planted in
a copy of oracle/wg_oracle.c (never in the oracle itself, never on the GPU), the copy is built,
and the pin that is meant to catch that kind of mistake has to fail on it -- while it passes on an
untouched copy.  A mistake that no pin catches would fail this test."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "wg_oracle.c")

# (name, text in the source, what it becomes, -k expression of the pins that must catch it)
MISTAKES = [
    ("byte budget off by one",
     "(int64_t)aux < l->max)) {", "(int64_t)aux <= l->max)) {",
     "test_bounded_wait_budget"),
    ("allow tested before the terminator",
     """        if (set_has(&l->wait, x)) {                   /* terminator first: non-greedy */
            *nsid = (x == WGO_EOS) ? after_eos(h, l->tmpl) : l->next; return 1;
        }
        if (set_has(&l->allow, x) && (l->max < 0 || (int64_t)aux < l->max)) {
            *nsid = sid; *naux = l->max < 0 ? 0 : aux + 1; return 1;
        }""",
     """        if (set_has(&l->allow, x) && (l->max < 0 || (int64_t)aux < l->max)) {
            *nsid = sid; *naux = l->max < 0 ? 0 : aux + 1; return 1;
        }
        if (set_has(&l->wait, x)) {
            *nsid = (x == WGO_EOS) ? after_eos(h, l->tmpl) : l->next; return 1;
        }""",
     "test_terminator_wins_over_allow or test_worked_example_equals_regex"),
    ("DoWhile loops on false",
     """        l->tnext = first_of(n->body, n->cond->sid);   /* true: run the body again */
        l->fnext = cont;                              /* false: leave the loop */""",
     """        l->fnext = first_of(n->body, n->cond->sid);
        l->tnext = cont;""",
     "test_worked_example_equals_regex"),
    ("IfElse takes the else body on true",
     """        l->tnext = first_of(n->if_body, cont);
        l->fnext = first_of(n->else_body, cont);""",
     """        l->fnext = first_of(n->if_body, cont);
        l->tnext = first_of(n->else_body, cont);""",
     "test_worked_example_equals_regex"),
    ("a None body does not fall through to what follows",
     "        l->tnext = first_of(n->if_body, cont);\n", "        l->tnext = n->if_body ? first_of(n->if_body, cont) : n->cond->sid;\n",
     "test_worked_example_equals_regex or test_canonical_numbering"),
    ("the template's end takes any symbol",
     """    case L_END:
        if (x != WGO_EOS) return 0;""",
     """    case L_END:
        if (x < 0) return 0;""",
     "test_last_literal_admits_exactly_the_prefixes_of_its_remainder"),
    ("mask bits packed most significant first",
     "row[t >> 5] |= 1u << (t & 31);", "row[t >> 5] |= 1u << (31 - (t & 31));",
     "test_mask_packing_matches_numpy_packbits"),
    ("bf16 minus infinity without its sign",
     "((uint16_t *)logits)[(int64_t)b * row_stride + t] = 0xFF80u;", "((uint16_t *)logits)[(int64_t)b * row_stride + t] = 0x7F80u;",
     "test_apply_matches_numpy_where"),
    ("apply disallows where the bit is set",
     "            if (bit) continue;\n            if (dtype == 0) ((uint32_t *)logits)", "            if (!bit) continue;\n            if (dtype == 0) ((uint32_t *)logits)",
     "test_apply_matches_numpy_where"),
    ("the k best keep the higher id on ties",
     """                else better = !is_nan && v > best_v;
                if (better) { best = t; best_v = v; best_nan = is_nan; }
            }
            ids_out""",
     """                else better = !is_nan && v >= best_v;
                if (better) { best = t; best_v = v; best_nan = is_nan; }
            }
            ids_out""",
     "test_masked_topk"),
    ("a NaN is never replaced by a number in the greedy choice",
     "            else if (best_nan) better = !is_nan;                  /* any number beats a NaN */",
     "            else if (best_nan) better = 0;",
     "test_masked_argmax"),
    ("a forced run goes on through a condition",
     "h->leaf[sid].kind == L_LIT) {\n        out[n++]", "h->leaf[sid].kind != L_WAIT && h->leaf[sid].kind != L_END && h->leaf[sid].kind != L_FINAL) {\n        out[n++]",
     "test_forced_bytes"),
    ("a forced run is cut one byte early by its cap",
     "while (n < cap && sid != WGO_SID_ERROR", "while (n + 1 < cap && sid != WGO_SID_ERROR",
     "test_forced_bytes"),
    ("the budget key is not capped at the longest token",
     "return (uint32_t)(left < (int64_t)lmax ? left : (int64_t)lmax);", "return (uint32_t)left;",
     "test_trajectory_is_consistent_with_unmemoised_calls or test_budget_key_reduction_is_sound"),
]


def _run_pins(tmp_path, name, source_text, select):
    d = tmp_path / ("".join(c if c.isalnum() else "_" for c in name))
    d.mkdir()
    src = d / "wg_oracle.c"
    src.write_text(source_text)
    env = dict(os.environ, WG_ORACLE_SOURCE=str(src))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                        "-x", "-q", "-p", "no:cacheprovider", "-k", select],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:] + r.stderr[-500:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with open(SOURCE) as f:
        good = f.read()
    jobs = [("untouched copy", good, " or ".join("(%s)" % m[3] for m in MISTAKES))]
    for name, old, new, select in MISTAKES:
        assert good.count(old) == 1, "the text to replace for '%s' occurs %d times" % (name, good.count(old))
        jobs.append((name, good.replace(old, new), select))
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda j: _run_pins(tmp_path, *j), jobs))
    rc, out = results[0]
    assert rc == 0, "the pins do not pass on an untouched copy:\n" + out
    missed = []
    for (name, _, _), (rc, out) in zip(jobs[1:], results[1:]):
        # 1 = tests ran and some failed; anything else (no test selected, a copy that does not build) is no catch
        if rc != 1 or " failed" not in out:
            missed.append((name, rc, out[-400:]))
    assert not missed, "planted mistakes that no pin caught: %r" % (missed,)
