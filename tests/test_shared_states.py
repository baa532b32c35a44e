"""WG_SHARE_STATES: states with equal futures share their cache keys (the global cache of the section
"Mask Generation and Global Caching").  The bar for a shared key is exact: whatever states the
library gives one key must have, budget for budget, the same mask in the oracle, on a vocabulary
whose longest token is as long as the lowering was told.  The oracle does not know about keys:
its masks come from walking every token from every state."""
import itertools

import numpy as np
import pytest

import paper_2507_16768_amd as wg
import wg_synth as ws
from oracle import oracle as O
from wg_synth.configs import TreeGen
from wg_synth.rng import Counter
from wg_synth.vocab import from_tokens


def _vocab(alphabet, max_len):
    toks = [b""] + [bytes(t) for n in range(1, max_len + 1) for t in itertools.product(alphabet, repeat=n)]
    return from_tokens(toks, eos_id=0)


def _groups(table):
    by_key = {}
    for sid in range(table.num_states):
        by_key.setdefault(table.state(sid)["key"], []).append(sid)
    return by_key


def _check_shared_masks(texts, args, vocab, restart):
    """Every set of states with one key: equal masks in the oracle for every budget.  Returns the
    number of states and of distinct first keys."""
    flags = (wg.EOS_RESTART if restart else wg.EOS_STOP) | wg.SHARE_STATES
    t = wg.Table(texts, args, flags=flags, lmax=vocab.lmax)
    ov = O.OracleVocab(vocab.bytes, vocab.offsets, vocab.eos_id)
    o = O.Oracle(texts, args, ov, restart=restart)
    assert t.num_states == o.num_states
    groups = _groups(t)
    for key, sids in groups.items():
        infos = [t.state(s) for s in sids]
        assert len({(i["n_keys"], i["max"]) for i in infos}) == 1, (key, sids)
        if len(sids) < 2:
            continue
        d = o.describe(sids[0])
        auxes = range(0, d["max"] + 2) if d["kind"] == "WAIT" and d["max"] >= 0 else (0,)
        for aux in auxes:
            rows = [o.mask_row((s, aux)) for s in sids]
            for s, r in zip(sids[1:], rows[1:]):
                assert (r == rows[0]).all(), (key, sids[0], s, aux, texts)
    # keys are handed out without gaps and without overlap between groups
    spans = sorted((k, t.state(s[0])["n_keys"]) for k, s in groups.items())
    at = 0
    for k, n in spans:
        assert k == at, spans
        at += n
    return t.num_states, len(groups)


@pytest.mark.parametrize("restart", [False, True])
@pytest.mark.parametrize("max_len", [1, 2, 3, 4])
def test_states_with_one_key_have_one_mask_on_random_trees(restart, max_len):
    """Random operator trees (loops, conditions, None bodies, empty Writes, bounded Waits) over
    four letters, several per table; the vocabulary is every string of up to max_len letters, so
    the lowering looks max_len - 1 states ahead."""
    vocab = _vocab(b"ab<.", max_len)
    rng = Counter(77, 2, start=1000 * max_len + restart)
    states = keys = 0
    for _ in range(30):
        trees = [TreeGen(rng, alphabet=b"ab<.", max_depth=3, write_len=(0, 3), big=False).tree(1, 18)
                 for _ in range(rng.between(1, 4))]
        n, k = _check_shared_masks([ws.to_text(t) for t in trees], None, vocab, restart)
        states += n
        keys += k
    assert keys < states                                   # something was shared
    if max_len == 1:
        assert keys < 0.5 * states                         # one byte ahead: only a state's own part counts


def test_equal_tails_share_and_different_heads_do_not():
    """One template text with two arguments: instances that differ in the first argument only.  With
    tokens of up to 3 bytes a state shares its key across the instances exactly when no token
    starting there can reach a byte of the argument that differs."""
    vocab = _vocab(b"abxy", 3)
    text = 'Sequence(Write($head), Write("bbbb"), Wait(allow={a}, wait={x}), Write($tail), Write("yy"))'
    args = [{"head": b"aa", "tail": b"ab"}, {"head": b"ab", "tail": b"ab"}, {"head": b"aa", "tail": b"ab"}]
    n, k = _check_shared_masks([text] * 3, args, vocab, True)
    t = wg.Table([text] * 3, args, flags=wg.EOS_RESTART | wg.SHARE_STATES, lmax=3)
    per = (t.num_states - 1) // 3
    first = [1 + i * per for i in range(3)]
    key = lambda inst, off: t.state(first[inst] + off)["key"]
    # instance 2 equals instance 0 as a whole
    assert all(key(2, j) == key(0, j) for j in range(per))
    # heads "aa" / "ab": the first state differs at once, the second in the byte it expects
    assert key(1, 0) != key(0, 0) and key(1, 1) != key(0, 1)
    # from the literal "bbbb" on, nothing ahead differs any more
    assert all(key(1, j) == key(0, j) for j in range(2, per))
    # restart: the END state leads back to its own instance's start, which does not show in a mask
    assert t.state(first[1] + per - 1)["kind"] == 4 and key(1, per - 1) == key(0, per - 1)
    # and without the flag only the instances that are equal as a whole share
    p = wg.Table([text] * 3, args, flags=wg.EOS_RESTART, lmax=3)
    pk = lambda inst, off: p.state(first[inst] + off)["key"]
    assert all(pk(2, j) == pk(0, j) for j in range(per)) and all(pk(1, j) != pk(0, j) for j in range(per))


def test_states_inside_one_instance_share_too():
    vocab = _vocab(b"ab<", 2)
    text = 'Sequence(Write("ab"), Wait(allow={a}, wait={<}), Write("ab"), Wait(allow={a}, wait={<}), Write("ab"), Wait(allow={a}, wait={<}))'
    n, k = _check_shared_masks([text], None, vocab, False)
    t = wg.Table([text], None, flags=wg.EOS_STOP | wg.SHARE_STATES, lmax=2)
    # the first byte of each "ab" sees the same two states ahead ('b', then a Wait over the same sets)
    assert t.state(1)["key"] == t.state(4)["key"]
    assert k < n


def test_a_failed_add_leaves_the_keys_as_they_were():
    vocab = _vocab(b"ab<", 3)
    good = ['Sequence(Write("ab"), Wait(allow={a}, wait={<}, max=2), Write("b"))',
            'Sequence(Write("bb"), Wait(allow={a}, wait={<}, max=2), Write("b"))']
    whole = wg.Table(good, None, flags=wg.EOS_RESTART | wg.SHARE_STATES, lmax=3)
    step = wg.Table(good[:1], None, flags=wg.EOS_RESTART | wg.SHARE_STATES, lmax=3)
    with pytest.raises(wg.WgError):
        step.add_instances([good[1], "Sequence(Write(\"a\")"], None)     # the second text is cut off
    step.add_instances(good[1:], None)
    assert step.num_states == whole.num_states
    assert [step.state(s)["key"] for s in range(step.num_states)] == [whole.state(s)["key"] for s in range(whole.num_states)]


def test_workload_tables_share_little_but_exactly():
    """Config 4 in small: per-request arguments keep most futures apart 23 bytes ahead; what is shared
    is shared exactly (masks of a 1,000-token vocabulary with the workload's token lengths)."""
    w = ws.make_workload(4, B=8, V=1000)
    n, k = _check_shared_masks(w.texts, w.args, w.vocab, True)
    assert k <= n
