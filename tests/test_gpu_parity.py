"""GPU parity: the HIP path through the C ABI against the CPU oracle, bit for bit.

Masks, next states and masked logits are integer / bit-pattern results, so the bar is
exact equality everywhere (no tolerance)."""
import os

import numpy as np
import pytest

import wg_synth as ws
from oracle import oracle as O
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2507_16768_amd as wg
    wg.load_library()
    return torch


def _replay(torch, w, steps, check_logits_every=1, label="", fused=False, share=False):
    """Oracle generates the trajectory; the GPU replays it step by step (with fused=True through
    wg_advance_fill_masks instead of wg_advance + wg_fill_masks)."""
    import paper_2507_16768_amd as wg
    o = H.make_oracle(w)
    v, h = H.make_gpu(w, share=share)
    st0 = H.start_states(o, w)
    assert (h.start_states[w.request_template] == st0).all()
    V, W, B = w.vocab.V, (w.vocab.V + 31) // 32, w.B
    toks, sts, _ = o.trajectory(st0, w.token_draws(steps))
    d_states = H.dev_states(st0)
    d_mask = torch.empty((B, W), dtype=torch.int32, device="cuda")
    cur = st0.copy()
    seen = {}
    for k in range(steps):
        print("%s step %d" % (label, k), flush=True) if k % 16 == 0 else None
        if not fused or k == 0:
            h.fill_masks(d_states, d_mask)
        got = H.host_mask(d_mask)
        for b in range(B):
            key = (int(cur[b, 0]), int(cur[b, 1]))
            if key not in seen:
                seen[key] = o.mask_row(key)
            assert (got[b] == seen[key]).all(), (label, k, b, key)
        if k % check_logits_every == 0:
            host = H.logits_for(w, tag=k)
            d_log = H.dev_logits(host)
            wg.apply_mask(d_log, d_mask)
            want = O.apply_mask(host.copy(), np.stack([seen[(int(s[0]), int(s[1]))] for s in cur]))
            want_bits = want.view(np.uint32) if want.dtype == np.float32 else want
            assert (H.host_logit_bits(d_log) == want_bits).all(), (label, k)
        d_tok = torch.from_numpy(toks[k]).cuda()
        if fused and k + 1 < steps:
            d_mask.fill_(0x3C3C3C3C)
            h.advance_fill_masks(d_states, d_tok, d_mask)
        else:
            h.advance(d_states, d_tok)
        cur = o.advance(cur, toks[k])
        assert (cur == sts[k]).all()
        assert (H.host_states(d_states) == cur).all(), (label, k)
    assert h.error_count() == 0
    # the cache keys a bounded Wait by its remaining budget capped at the longest token
    return h, o, len({(k[0], o.key_rem(k)) for k in seen})


def test_config1_tiny_full(torch_cuda):
    """Config 1 as stated: V=32,000, one request, 64 steps, fp32 logits, argmax selection."""
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    w = ws.make_workload(1)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    cur = H.start_states(o, w)
    d_states = H.dev_states(cur)
    d_mask = torch.empty((1, h.W), dtype=torch.int32, device="cuda")
    visited = set()
    for k in range(w.steps):
        row = o.mask_row(tuple(cur[0]))
        h.fill_masks(d_states, d_mask)
        assert (H.host_mask(d_mask)[0] == row).all(), k
        host = H.logits_for(w, tag=k)
        d_log = H.dev_logits(host)
        wg.apply_mask(d_log, d_mask)
        want = O.apply_mask(host.copy(), row[None, :])
        assert (H.host_logit_bits(d_log) == want.view(np.uint32)).all(), k
        tok = int(np.argmax(want[0]))                      # lowest index on ties
        assert tok == int(torch.argmax(d_log[0]).item())
        d_tok = torch.tensor([tok], dtype=torch.int32, device="cuda")
        h.advance(d_states, d_tok)
        cur = o.advance(cur, [tok])
        assert (H.host_states(d_states) == cur).all(), k
        visited.add(int(cur[0, 0]))
    assert h.error_count() == 0 and len(visited) > 20


@pytest.mark.parametrize("idx,V,B,steps", [
    (2, 5003, 7, 96),        # V % 32 != 0: ragged last word and last 64-token slice
    (3, 4099, 9, 96),
    (4, 6001, 10, 64),
    (5, 7013, 33, 64),
])
def test_reduced_configs_every_step(torch_cuda, idx, V, B, steps):
    w = ws.make_workload(idx, V=V, B=B, steps=steps)
    h, o, nkeys = _replay(torch_cuda, w, steps, label="cfg%d-small" % idx)
    s = h.cache_stats()
    assert s["lookups"] == B * steps and s["builds"] == nkeys and 0 < s["hits"] <= B * steps - nkeys


@pytest.mark.parametrize("idx,V,B,steps", [(2, 5003, 7, 64), (3, 4099, 9, 64), (4, 6001, 10, 64), (5, 7013, 33, 48)])
def test_reduced_configs_with_states_of_equal_futures_sharing_keys(torch_cuda, idx, V, B, steps):
    """WG_SHARE_STATES: every mask, masked logit and state as without it; no more rows built than
    there are distinct (state, budget) pairs, and fewer keys in the handle than states ask for."""
    w = ws.make_workload(idx, V=V, B=B, steps=steps)
    h, o, nkeys = _replay(torch_cuda, w, steps, check_logits_every=8, label="cfg%d-shared" % idx, share=True)
    s = h.cache_stats()
    assert s["lookups"] == B * steps and 0 < s["builds"] <= nkeys
    v2, plain = H.make_gpu(w)
    assert s["keys"] <= plain.cache_stats()["keys"]
    if idx == 5:
        assert s["keys"] < plain.cache_stats()["keys"]


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("idx,V,B,steps", [(4, 6001, 10, 48), (5, 20011, 64, 24)])
def test_reduced_configs_under_other_seeds(torch_cuda, seed, idx, V, B, steps):
    """Other vocabularies, templates and token streams than the base seed's, through the
    separate calls and through the fused advance + fill."""
    for fused in (False, True):
        w = ws.make_workload(idx, seed=seed, V=V, B=B, steps=steps)
        _replay(torch_cuda, w, steps, check_logits_every=8, label="cfg%d-seed%d" % (idx, seed), fused=fused)


@pytest.mark.parametrize("idx,B,steps", [(2, 64, 24), (3, 128, 16), (4, 256, 8), (5, 1024, 6)])
def test_full_size_configs_sampled(torch_cuda, idx, B, steps):
    """Full V and B of configs 2-5; states every step, every distinct mask; the masked logits as raw
    bits on every step of config 2, on 8 steps of configs 3 and 4, on all 6 steps of config 5."""
    w = ws.make_workload(idx, steps=steps)
    assert w.B == B
    every = 1 if idx in (2, 5) else 2 if idx == 3 else 1
    _replay(torch_cuda, w, steps, check_logits_every=every, label="cfg%d-full" % idx)


@pytest.mark.parametrize("idx,V,B,steps", [(3, 3001, 8, 48), (5, 4099, 96, 24)])
def test_fused_advance_and_fill_match_the_separate_calls(torch_cuda, idx, V, B, steps):
    w = ws.make_workload(idx, V=V, B=B, steps=steps)
    h, o, nkeys = _replay(torch_cuda, w, steps, check_logits_every=8, label="fused cfg%d" % idx, fused=True)
    s = h.cache_stats()
    assert s["lookups"] == steps * B and s["builds"] == nkeys == s["rows_in_use"]
    # an illegal token in the fused call: the request goes to ERROR and gets a row of zeros
    torch = torch_cuda
    st = H.start_states(o, w)
    row = o.mask_row(tuple(st[0]))
    bad = next(t for t in range(w.vocab.V) if not (row[t >> 5] >> (t & 31)) & 1)
    good = O.select_bit(row, 0)
    d_states = H.dev_states(st[:2].copy() * 0 + st[0])
    d_mask = torch.empty((2, h.W), dtype=torch.int32, device="cuda")
    h.advance_fill_masks(d_states, torch.tensor([bad, good], dtype=torch.int32, device="cuda"), d_mask)
    got_s, got_m = H.host_states(d_states), H.host_mask(d_mask)
    nxt = o.advance(st[:1], [good])
    assert tuple(got_s[0]) == (0xFFFFFFFF, 0) and not got_m[0].any()
    assert (got_s[1] == nxt[0]).all() and (got_m[1] == o.mask_row(tuple(nxt[0]))).all()
    assert h.error_count() == 1


@pytest.mark.parametrize("idx,V,B,steps,rows,pad", [
    (3, 3001, 8, 40, 0, 0),        # V % 8 != 0: the separate apply kernels do the masking
    (4, 6008, 24, 40, 0, 0),       # bf16, 16-byte stores: masking inside the gather kernel
    (4, 6008, 24, 24, 0, 8),       # ... with padded logits rows
    (4, 6008, 24, 24, 0, 3),       # ... with a row stride that rules out 16-byte stores
    (5, 4104, 96, 24, 5, 0),       # five cache rows: most masks are built straight into the bitmask
    (2, 4096, 6, 30, 0, 0),
    (4, None, None, 6, 0, 0),      # full size: B=256, V=151,936, the shape the benchmark times
    (5, None, None, 3, 0, 0),      # full size: B=1,024
])
def test_decode_step_matches_the_oracle(torch_cuda, idx, V, B, steps, rows, pad):
    """wg_decode_step (advance + fill + apply in one call) against the oracle on every step:
    states, full bitmask and masked logits."""
    torch = torch_cuda
    w = ws.make_workload(idx, V=V, B=B, steps=steps) if V else ws.make_workload(idx, steps=steps)
    V, B = w.vocab.V, w.B
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    if rows:
        h.cache_resize(rows)
    cur = H.start_states(o, w)
    toks, sts, _ = o.trajectory(cur, w.token_draws(steps))
    d_states = H.dev_states(cur)
    d_mask = torch.empty((B, h.W), dtype=torch.int32, device="cuda")
    prev = None
    for k in range(steps):
        print("decode_step cfg%d step %d" % (idx, k), flush=True) if k % 8 == 0 else None
        host = H.logits_for(w, tag=k)
        d_log = H.dev_logits(host)
        if pad:
            buf = torch.zeros((B, V + pad), dtype=d_log.dtype, device="cuda")
            buf[:, :V] = d_log
            d_log = buf[:, :V]
        d_mask.fill_(0x77777777)
        h.decode_step(d_states, prev, d_mask, d_log)
        assert (H.host_states(d_states) == cur).all(), k
        want_mask = o.fill_masks(cur)
        assert (H.host_mask(d_mask) == want_mask).all(), k
        want = O.apply_mask(host.copy(), want_mask)
        want_bits = want.view(np.uint32) if want.dtype == np.float32 else want
        assert (H.host_logit_bits(d_log.contiguous()) == want_bits).all(), k
        if pad:
            assert (H.host_logit_bits(buf[:, V:].contiguous()) == 0).all()
        prev = torch.from_numpy(toks[k]).cuda()
        cur = sts[k]
    h.advance(d_states, prev)
    assert (H.host_states(d_states) == cur).all()
    s = h.cache_stats()
    assert s["lookups"] == steps * B and h.error_count() == 0
    assert (s["uncached_builds"] > 0) == bool(rows)


def test_decode_step_replayed_from_a_hip_graph(torch_cuda):
    """A decode step recorded once into a HIP graph and replayed for every later step, with the
    program's own eager copies and synchronisations between the replays: every replay (cache
    misses in the early ones, hits later) must give the oracle's states, masks and logits.  The
    step path launches kernels only (no allocation, no memset), and the number of the fill call,
    which tags claimed keys, lives in device memory, so a replay is a new call."""
    torch = torch_cuda
    w = ws.make_workload(4, V=6008, B=24, steps=20)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    B, V, steps = w.B, w.vocab.V, w.steps
    cur = H.start_states(o, w)
    toks, sts, _ = o.trajectory(cur, w.token_draws(steps))
    d_states = H.dev_states(cur)
    d_mask = torch.empty((B, h.W), dtype=torch.int32, device="cuda")
    d_log = H.dev_logits(H.logits_for(w, tag=0)).clone()
    d_tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()

    def check(k, host):
        assert (H.host_states(d_states) == cur).all(), k
        want_mask = o.fill_masks(cur)
        assert (H.host_mask(d_mask) == want_mask).all(), k
        assert (H.host_logit_bits(d_log) == O.apply_mask(host.copy(), want_mask)).all(), k

    # step 0 eagerly (no token yet); it also sizes the handle's per-call lists
    host = H.logits_for(w, tag=0)
    h.decode_step(d_states, None, d_mask, d_log)
    check(0, host)
    torch.cuda.synchronize()
    # record step 1 .. on a side stream: the recording itself runs nothing
    with torch.cuda.graph(graph, stream=side):
        h.decode_step(d_states, d_tok, d_mask, d_log, stream=side)
    for k in range(1, steps):
        print("graph replay for step %d" % k, flush=True) if k % 4 == 1 else None
        d_tok.copy_(torch.from_numpy(toks[k - 1]).cuda())
        cur = sts[k - 1]
        host = H.logits_for(w, tag=k)
        d_log.copy_(H.dev_logits(host))
        d_mask.fill_(0x11111111)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        check(k, host)
    s = h.cache_stats()
    assert s["lookups"] == steps * B and s["builds"] == s["rows_in_use"] > 0 and h.error_count() == 0


def test_long_tokens_take_the_generic_paths(torch_cuda):
    """Tokens of up to 40 bytes: longer than the three 8-byte chunks the fast paths hold."""
    import dataclasses
    base = ws.make_workload(4, V=3001, B=12, steps=48)
    vocab = ws.make_vocab(3001, ("geometric", 10, 40), seed=9, utf8_tenths=1)
    assert vocab.lmax == 40
    w = dataclasses.replace(base, vocab=vocab)
    h, o, nkeys = _replay(torch_cuda, w, 48, label="long-tokens")
    assert h.cache_stats()["builds"] == nkeys
    # and a bounded Wait whose budget binds below the longest token
    w2 = dataclasses.replace(base, vocab=vocab, B=3, request_template=np.zeros(3, dtype=np.int64),
                             texts=['Sequence(Wait(denies={}, wait={<}, max=30), Write("ab>"))'], args=[{}])
    o2 = H.make_oracle(w2)
    v2, h2 = H.make_gpu(w2)
    s = o2.start_state(0)
    st = np.array([[s, 0], [s, 11], [s, 27]], dtype=np.uint32)
    d_mask = torch_cuda.empty((3, h2.W), dtype=torch_cuda.int32, device="cuda")
    h2.fill_masks(H.dev_states(st), d_mask)
    assert (H.host_mask(d_mask) == o2.fill_masks(st)).all()


@pytest.mark.parametrize("idx", [2, 3, 4, 5])
def test_full_trajectories_reproduce_oracle_digests(torch_cuda, idx, golden_dir):
    """Every config at its full B, V and step count: the GPU draws the whole trajectory from its
    own masks (fill, pick the (draw mod popcount)-th allowed token, advance); tokens and states
    must hash, block by block, to the digests the oracle-only script wrote."""
    import hashlib
    import json
    import os
    import paper_2507_16768_amd as wg
    torch = torch_cuda
    with open(os.path.join(golden_dir, "trajectory_digests.json")) as f:
        gold = json.load(f)[str(idx)]
    w = ws.make_workload(idx)
    assert (gold["steps"], gold["B"], gold["V"]) == (w.steps, w.B, w.vocab.V) and gold["errors"] == 0
    v, h = H.make_gpu(w)
    states = H.dev_states(h.start_states[w.request_template])
    mask = torch.empty((w.B, h.W), dtype=torch.int32, device="cuda")
    draws = torch.from_numpy(w.token_draws().view(np.int64)).cuda()
    toks = torch.empty((w.steps, w.B), dtype=torch.int32, device="cuda")
    sts = torch.empty((w.steps, w.B, 2), dtype=torch.int32, device="cuda")
    for k in range(w.steps):
        if k % 512 == 0:
            print("cfg%d trajectory step %d" % (idx, k), flush=True)
        h.fill_masks(states, mask)
        wg.select_tokens(mask, w.vocab.V, draws[k], toks[k])
        h.advance(states, toks[k])
        sts[k].copy_(states)
    torch.cuda.synchronize()
    assert h.error_count() == 0
    toks_h, sts_h = toks.cpu().numpy(), sts.cpu().numpy().view(np.uint32)
    blk = gold["block"]
    for i, want in enumerate(gold["digests"]):
        d = hashlib.sha256()
        d.update(np.ascontiguousarray(toks_h[i * blk:(i + 1) * blk], dtype="<i4").tobytes())
        d.update(np.ascontiguousarray(sts_h[i * blk:(i + 1) * blk], dtype="<u4").tobytes())
        assert d.hexdigest()[:16] == want, "config %d diverges from the oracle in steps %d..%d" % (idx, i * blk, (i + 1) * blk - 1)
    s = h.cache_stats()
    assert s["builds"] == gold["distinct_masks"] and s["lookups"] == w.steps * w.B


def _all_states(o):
    out = [[O.SID_ERROR, 0]]
    for sid in range(o.num_states):
        d = o.describe(sid)
        auxes = range(0, d["max"] + 2) if d["kind"] == "WAIT" and d["max"] >= 0 else (0,)
        out += [[sid, a] for a in auxes]
    return np.array(out, dtype=np.uint32)


@pytest.mark.parametrize("restart", [False, True])
def test_random_trees_every_state_every_token(torch_cuda, restart):
    """Exhaustive on tiny inputs: every (state, budget) mask and every (state, token) advance of
    random operator trees (None bodies, empty Writes, max=0, nested loops) on a vocabulary of
    all strings up to length 3 over four letters, EOS in the middle of the id range."""
    from wg_synth.configs import TreeGen
    from wg_synth.rng import Counter
    from wg_synth.vocab import from_tokens
    import itertools
    import paper_2507_16768_amd as wg
    torch = torch_cuda
    alpha = b"ab<."
    toks = [bytes(t) for n in (1, 2, 3) for t in itertools.product(alpha, repeat=n)]
    toks.insert(17, b"")                                   # EOS is token 17
    toks.insert(40, b"")                                   # a byte-less token that is not EOS
    vocab = from_tokens(toks, eos_id=17)
    ov = O.OracleVocab(vocab.bytes, vocab.offsets, vocab.eos_id)
    gv = wg.Vocab(vocab.bytes, vocab.offsets, vocab.eos_id)
    rng = Counter(31, 2, start=500 * restart)
    V = vocab.V
    n_states = 0
    for case in range(40):
        trees = [TreeGen(rng, alphabet=alpha, max_depth=3, write_len=(0, 3), big=False).tree(1, 18)
                 for _ in range(rng.between(1, 3))]
        texts = [ws.to_text(t) for t in trees]
        o = O.Oracle(texts, None, ov, restart=restart)
        h = wg.Handle(texts, None, gv, flags=wg.EOS_RESTART if restart else wg.EOS_STOP)
        h.set_scan_batch((0, 8, 3)[case % 3])              # the class scan table by table, and several at a time
        st = _all_states(o)
        n_states += len(st)
        h.reserve_batch(len(st))
        d_mask = torch.empty((len(st), h.W), dtype=torch.int32, device="cuda")
        h.fill_masks(H.dev_states(st), d_mask)
        want = o.fill_masks(st)
        assert (H.host_mask(d_mask) == want).all(), texts
        rep = np.repeat(st, V, axis=0)
        tk = np.tile(np.arange(V, dtype=np.int32), len(st))
        d_st = H.dev_states(rep)
        h.advance(d_st, torch.from_numpy(tk).cuda())
        got = H.host_states(d_st)
        want_st = o.advance(rep, tk)
        bad = np.nonzero((got != want_st).any(axis=1))[0]
        assert len(bad) == 0, (texts, rep[bad[0]], toks[tk[bad[0]]], got[bad[0]], want_st[bad[0]])
        ok = got[:, 0] != O.SID_ERROR
        assert (ok.reshape(len(st), V) == np.stack([H.bits(r, V) for r in want])).all()
    assert n_states > 400


def test_templates_made_from_regular_expressions_run_on_the_device(torch_cuda):
    """Constraints given as regular expressions: translated on the host, then every state's mask
    and every (state, token) advance equals the oracle's, and a greedy decode of random logits
    under the masks produces a string the expression matches."""
    import itertools
    import re
    from wg_synth.vocab import from_tokens
    import paper_2507_16768_amd as wg
    torch = torch_cuda
    alpha = b"01.,[]x"
    toks = [bytes(t) for n in (1, 2, 3) for t in itertools.product(alpha, repeat=n)]
    toks.insert(5, b"")                                    # EOS is token 5
    vocab = from_tokens(toks, eos_id=5)
    V = vocab.V
    rxs = [r"\d+(\.\d+)*", r"\[\d+(,\d+)*\]", r"x{1,3}(\.|,)[01]?x"]
    texts = [wg.regex_to_template(rx) for rx in rxs]
    ov = O.OracleVocab(vocab.bytes, vocab.offsets, vocab.eos_id)
    o = O.Oracle(texts, None, ov, restart=False)
    gv = wg.Vocab(vocab.bytes, vocab.offsets, vocab.eos_id)
    h = wg.Handle(texts, None, gv, flags=wg.EOS_STOP)
    st = _all_states(o)
    h.reserve_batch(len(st))
    d_mask = torch.empty((len(st), h.W), dtype=torch.int32, device="cuda")
    h.fill_masks(H.dev_states(st), d_mask)
    assert (H.host_mask(d_mask) == o.fill_masks(st)).all()
    rep = np.repeat(st, V, axis=0)
    tk = np.tile(np.arange(V, dtype=np.int32), len(st))
    d_st = H.dev_states(rep)
    h.advance(d_st, torch.from_numpy(tk).cuda())
    assert (H.host_states(d_st) == o.advance(rep, tk)).all()
    # decode: 64 requests per expression, greedy on seeded logits until every request is FINAL
    errors_before = h.error_count()                         # from the illegal pairs fed above
    B = 64 * len(rxs)
    which = np.arange(B) % len(rxs)
    d_states = H.dev_states(h.start_states[which])
    d_mask = torch.empty((B, h.W), dtype=torch.int32, device="cuda")
    d_tok = torch.empty(B, dtype=torch.int32, device="cuda")
    outs = [b""] * B
    done = np.zeros(B, dtype=bool)
    for k in range(40):
        x = ws.make_logits(9, B, V, 1.0, tag=k)
        x[:, 5] += 0.5 * k - 4.0                            # EOS grows more likely with time
        h.fill_masks(d_states, d_mask)
        wg.masked_argmax(H.dev_logits(x), d_mask, d_tok)
        h.advance(d_states, d_tok)
        t_h, s_h = d_tok.cpu().numpy(), H.host_states(d_states)
        for b in range(B):
            if not done[b]:
                if t_h[b] == 5:
                    done[b] = True
                    assert s_h[b, 0] == O.SID_FINAL
                else:
                    assert t_h[b] >= 0
                    outs[b] += toks[t_h[b]]
        if done.all():
            break
    assert done.all()
    for b in range(B):
        assert re.fullmatch(rxs[which[b]].encode(), outs[b]), (rxs[which[b]], outs[b])
    print(sorted(set(outs))[:6], flush=True)
    assert len(set(outs)) > 20 and h.error_count() == errors_before


def test_tiny_shapes_and_no_eos(torch_cuda):
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    from wg_synth.vocab import from_tokens
    for V in (1, 31, 33, 64, 65):
        toks = [bytes([97 + (i % 3)]) * (1 + i % 5) for i in range(V)]
        vocab = from_tokens(toks, eos_id=-1)
        o = O.Oracle(['Sequence(Wait(allow={a}, wait={b}, max=3), Write("c"))'], None,
                     O.OracleVocab(vocab.bytes, vocab.offsets, -1), restart=True)
        gv = wg.Vocab(vocab.bytes, vocab.offsets, -1)
        h = wg.Handle(['Sequence(Wait(allow={a}, wait={b}, max=3), Write("c"))'], None, gv)
        st = _all_states(o)
        d_mask = torch.full((len(st), h.W), -1, dtype=torch.int32, device="cuda")
        h.fill_masks(H.dev_states(st), d_mask)
        assert (H.host_mask(d_mask) == o.fill_masks(st)).all(), V
        x = ws.make_logits(1, len(st), V, 1.0)
        d_log = H.dev_logits(x)
        wg.apply_mask(d_log, d_mask)
        assert (H.host_logit_bits(d_log) == O.apply_mask(x.copy(), o.fill_masks(st)).view(np.uint32)).all()


def test_cache_cold_warm_and_duplicates(torch_cuda):
    torch = torch_cuda
    w = ws.make_workload(3, V=4099, B=16, steps=4)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    st = H.start_states(o, w)                               # 16 requests in the same state
    d_states = H.dev_states(st)
    d_mask = torch.zeros((16, h.W), dtype=torch.int32, device="cuda")
    want = o.mask_row(tuple(st[0]))
    h.fill_masks(d_states, d_mask)
    s1 = h.cache_stats()
    assert (H.host_mask(d_mask) == want[None, :]).all()
    assert (s1["lookups"], s1["builds"], s1["hits"], s1["class_scans"]) == (16, 1, 0, 0)
    d_mask.zero_()
    h.fill_masks(d_states, d_mask)
    s2 = h.cache_stats()
    assert (H.host_mask(d_mask) == want[None, :]).all()
    assert (s2["lookups"], s2["builds"], s2["hits"]) == (32, 1, 16)
    h.cache_clear()
    d_mask.zero_()
    h.fill_masks(d_states, d_mask)
    s3 = h.cache_stats()
    assert (H.host_mask(d_mask) == want[None, :]).all()
    assert (s3["builds"], s3["hits"]) == (2, 16)
    # a Wait state needs its class table scanned once per cache epoch, however many keys use it
    wait_sid = next(s for s in range(h.num_states) if o.describe(s)["kind"] == "WAIT")
    two = H.dev_states(np.array([[wait_sid, 0]] * 16, dtype=np.uint32))
    h.fill_masks(two, d_mask)
    assert (H.host_mask(d_mask) == o.mask_row((wait_sid, 0))[None, :]).all()
    assert h.cache_stats()["class_scans"] == 1
    h.fill_masks(two, d_mask)
    assert h.cache_stats()["class_scans"] == 1
    assert s3["keys"] >= h.num_states and s3["arena_bytes"] >= s3["keys"] * h.W * 4


def test_batch_above_the_reservation_is_refused_until_reserved(torch_cuda):
    """A handle has room for 1,024 requests per call; a batch of 2,500 is refused by every
    per-step call (nothing is launched, nothing allocated) until wg_reserve_batch made room."""
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    w = ws.make_workload(5, V=3001, B=2500, steps=3)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    assert h.max_batch() == 1024
    cur = H.start_states(o, w)
    small = H.dev_states(cur[:100])
    d_small = torch.empty((100, h.W), dtype=torch.int32, device="cuda")
    h.fill_masks(small, d_small)                            # first a small call, then the large one
    toks, sts, _ = o.trajectory(cur, w.token_draws(3))
    d_states = H.dev_states(cur)
    d_mask = torch.full((2500, h.W), 0x13571357, dtype=torch.int32, device="cuda")
    d_log = torch.zeros((2500, w.vocab.V), dtype=torch.float32, device="cuda")
    d_tok = torch.from_numpy(toks[0]).cuda()
    for call in (lambda: h.fill_masks(d_states, d_mask), lambda: h.advance_fill_masks(d_states, d_tok, d_mask),
                 lambda: h.decode_step(d_states, None, d_mask, d_log)):
        with pytest.raises(wg.WgError, match="wg_reserve_batch"):
            call()
    assert (H.host_mask(d_mask) == 0x13571357).all() and (H.host_states(d_states) == cur).all()
    h.reserve_batch(2500)
    assert h.max_batch() == 2500
    h.reserve_batch(64)                                     # never shrinks
    assert h.max_batch() == 2500
    with pytest.raises(wg.WgError):
        h.reserve_batch(0)
    with pytest.raises(wg.WgError):
        h.reserve_batch(65536)
    for k in range(3):
        h.fill_masks(d_states, d_mask)
        assert (H.host_mask(d_mask) == o.fill_masks(cur)).all(), k
        h.advance(d_states, torch.from_numpy(toks[k]).cuda())
        cur = o.advance(cur, toks[k])
        assert (H.host_states(d_states) == cur).all()
    # the masks made before the reservation grew are still cached
    before = h.cache_stats()["builds"]
    h.fill_masks(small, d_small)
    assert (H.host_mask(d_small) == o.fill_masks(H.start_states(o, w)[:100])).all()
    assert h.cache_stats()["builds"] == before


def _pick_tokens(o_rows, draws):
    """The sampler stand-in on the host: the (draw mod popcount)-th allowed token of each row."""
    out = np.full(len(o_rows), -1, dtype=np.int32)
    for b, row in enumerate(o_rows):
        pop = int(np.unpackbits(row.view(np.uint8)).sum())
        if pop:
            out[b] = O.select_bit(row, int(draws[b]) % pop)
    return out


def test_small_cache_serves_overflow_keys_uncached(torch_cuda):
    """With fewer cache rows than distinct keys the surplus rows are built straight into the
    callers' bitmask (also for the other requests of the call that share the key) and every
    mask still equals the oracle's; a resize makes room again."""
    torch = torch_cuda
    w = ws.make_workload(5, V=3001, B=192, steps=10)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    h.cache_resize(7)
    cur = H.start_states(o, w)
    toks, sts, n_masks = o.trajectory(cur, w.token_draws(10))
    d_states = H.dev_states(cur)
    d_mask = torch.empty((w.B, h.W), dtype=torch.int32, device="cuda")
    for k in range(10):
        print("overflow step %d" % k, flush=True)
        d_mask.fill_(0x5A5A5A5A)
        h.fill_masks(d_states, d_mask)
        assert (H.host_mask(d_mask) == o.fill_masks(cur)).all(), k
        h.advance(d_states, torch.from_numpy(toks[k]).cuda())
        cur = sts[k]
    s = h.cache_stats()
    assert s["cache_rows"] == 7 and s["rows_in_use"] == 7
    assert s["uncached_builds"] > 0 and s["builds"] > n_masks       # overflow keys are rebuilt
    assert s["lookups"] == 10 * w.B
    # room for everything: every key is built once and then hit
    h.cache_resize(4096)
    cur = H.start_states(o, w)
    d_states = H.dev_states(cur)
    base = h.cache_stats()
    for k in range(10):
        h.fill_masks(d_states, d_mask)
        assert (H.host_mask(d_mask) == o.fill_masks(cur)).all(), k
        h.advance(d_states, torch.from_numpy(toks[k]).cuda())
        cur = sts[k]
    s2 = h.cache_stats()
    assert s2["uncached_builds"] == base["uncached_builds"]
    assert s2["builds"] - base["builds"] == s2["rows_in_use"] <= n_masks
    assert h.error_count() == 0


def test_instances_join_a_live_handle(torch_cuda):
    """Requests arrive while the batch is running: their instances are added to the handle, the
    running requests keep their states and cached rows, and every mask and state equals those of
    an oracle that compiled all instances at once.  Starting from one instance, the 64 instances
    outgrow the room reserved for states, keys and class tables, so the tables move as well."""
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    w = ws.make_workload(4, V=3001, B=64, steps=14)
    n_inst = len(w.texts)
    assert (np.asarray(w.request_template) == np.arange(w.B)).all() and n_inst == w.B
    o = H.make_oracle(w)
    gv = wg.Vocab(w.vocab.bytes, w.vocab.offsets, w.vocab.eos_id)
    h = wg.Handle(w.texts[:1], w.args[:1], gv)
    cur = H.start_states(o, w)
    assert (h.start_states[0] == cur[0]).all()
    draws = w.token_draws(14)
    joined = 1
    schedule = {2: 3, 4: 9, 5: 10, 7: 40, 10: 64}             # step -> instances present from then on
    d_mask = torch.empty((w.B, h.W), dtype=torch.int32, device="cuda")
    for k in range(14):
        print("join step %d, %d instances" % (k, joined), flush=True)
        if k in schedule:
            with pytest.raises(wg.WgError):                  # a request with a broken template is refused ...
                h.add_instances(["Sequence(Write(\"a\"), Wait(allow={b}))"], [{}])
            new = h.add_instances(w.texts[joined:schedule[k]], w.args[joined:schedule[k]])
            assert (new == cur[joined:schedule[k]]).all()    # ... and leaves the numbering alone
            joined = schedule[k]
            assert h.num_instances() == joined
        act = cur[:joined]
        d_states = H.dev_states(act)
        h.fill_masks(d_states, d_mask[:joined])
        want = o.fill_masks(act)
        assert (H.host_mask(d_mask[:joined]) == want).all(), k
        tok = _pick_tokens(want, draws[k])
        h.advance(d_states, torch.from_numpy(tok).cuda())
        nxt = o.advance(act, tok)
        assert (H.host_states(d_states) == nxt).all(), k
        cur[:joined] = nxt
    assert h.num_states == o.num_states and h.error_count() == 0
    # nothing was rebuilt because of the joins: as many builds as distinct keys were seen
    s = h.cache_stats()
    assert s["uncached_builds"] == 0 and s["builds"] == s["rows_in_use"]


def test_two_handles_share_one_vocabulary(torch_cuda):
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    w2, w3 = ws.make_workload(2, V=4099, B=4, steps=1), ws.make_workload(3, V=4099, B=4, steps=1)
    assert (w2.vocab.bytes == w3.vocab.bytes).all()
    gv = wg.Vocab(w2.vocab.bytes, w2.vocab.offsets, w2.vocab.eos_id)
    h2 = wg.Handle(w2.texts, w2.args, gv)
    h3 = wg.Handle(w3.texts, w3.args, gv)
    o2, o3 = H.make_oracle(w2), H.make_oracle(w3)
    for h, o, w in ((h2, o2, w2), (h3, o3, w3), (h2, o2, w2)):
        st = H.start_states(o, w)
        d_mask = torch.empty((4, h.W), dtype=torch.int32, device="cuda")
        h.fill_masks(H.dev_states(st), d_mask)
        assert (H.host_mask(d_mask) == o.fill_masks(st)).all()
    del h2
    st = H.start_states(o3, w3)
    d_mask = torch.empty((4, h3.W), dtype=torch.int32, device="cuda")
    h3.cache_clear()
    h3.fill_masks(H.dev_states(st), d_mask)
    assert (H.host_mask(d_mask) == o3.fill_masks(st)).all()


def test_error_states_and_illegal_tokens(torch_cuda):
    torch = torch_cuda
    w = ws.make_workload(2, V=5003, B=6, steps=1)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    s0 = int(o.start_state(0))
    st = np.array([[s0, 0], [O.SID_ERROR, 0], [h.num_states + 5, 0], [0, 0], [s0, 0], [s0, 0]], dtype=np.uint32)
    d_states = H.dev_states(st)
    d_mask = torch.full((6, h.W), -1, dtype=torch.int32, device="cuda")
    h.fill_masks(d_states, d_mask)
    got = H.host_mask(d_mask)
    want = o.fill_masks(st)
    assert (got == want).all()
    assert not got[1].any() and not got[2].any()           # ERROR / out of range: all-zero rows
    assert got[3].sum() == 1 and got[3][0] == 1            # FINAL admits only EOS (token 0)
    legal = int(np.nonzero(H.bits(want[0], w.vocab.V))[0][0])
    illegal = int(np.nonzero(~H.bits(want[0], w.vocab.V))[0][5])
    toks = np.array([legal, legal, legal, 0, illegal, w.vocab.V + 3], dtype=np.int32)
    h.advance(d_states, torch.from_numpy(toks).cuda())
    want_st = o.advance(st, toks)
    assert (H.host_states(d_states) == want_st).all()
    assert h.error_count() == 4
    toks2 = np.array([-1, 0, 0, 0, 0, 0], dtype=np.int32)
    h.advance(d_states, torch.from_numpy(toks2).cuda())
    assert (H.host_states(d_states) == o.advance(want_st, toks2)).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,stride_pad,offset", [(4096, 0, 0), (4104, 8, 0), (1000 + 13, 3, 0), (4096, 0, 1)])
def test_apply_shapes_strides_and_special_values(torch_cuda, dtype, V, stride_pad, offset):
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    B, W = 5, (V + 31) // 32
    x = ws.make_logits(3, B, V, 2.0)
    x[0, 3], x[1, 4], x[2, 5], x[3, 6] = np.nan, -0.0, np.inf, 1e-42
    m = ws.rng.draw(4, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[4, :] = 0xFFFFFFFF
    m[3, :] = 0
    host = x if dtype == "f32" else ws.to_bf16_bits(x)
    want = O.apply_mask(host.copy(), m)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    buf = torch.zeros(B * (V + stride_pad) + offset + 8, dtype=tdt, device="cuda")
    view = buf[offset:offset + B * (V + stride_pad)].view(B, V + stride_pad)[:, :V]
    view.copy_(H.dev_logits(host))
    d_mask = torch.from_numpy(m.view(np.int32)).cuda()
    wg.apply_mask(view, d_mask)
    got = H.host_logit_bits(view.contiguous())
    assert (got == (want.view(np.uint32) if dtype == "f32" else want)).all()
    if stride_pad:                                           # the padding between rows is untouched
        pad = buf[offset:offset + B * (V + stride_pad)].view(B, V + stride_pad)[:, V:]
        assert (H.host_logit_bits(pad.contiguous()) == 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,stride_pad,offset", [(151936, 0, 0), (4104, 8, 0), (1000 + 13, 3, 0), (4096, 0, 1)])
def test_masked_argmax_matches_oracle(torch_cuda, dtype, V, stride_pad, offset):
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    B, W = 9, (V + 31) // 32
    x = ws.make_logits(7, B, V, 2.0)
    x[0, 3], x[0, 4], x[1, 5], x[2, :] = np.nan, np.inf, -0.0, np.nan
    x[3, 100:200] = 7.5                                   # a long tie
    m = ws.rng.draw(8, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[:, -1] &= (1 << (V % 32)) - 1 if V % 32 else 0xFFFFFFFF
    m[4, :] = 0                                           # nothing allowed
    m[5, :] = 0
    m[5, W // 2] = 1 << 7                                 # a single allowed token
    m[6, :] = 0xFFFFFFFF
    m[6, -1] = m[0, -1] | 1
    host = x if dtype == "f32" else ws.to_bf16_bits(np.nan_to_num(x, nan=0.0)) | np.where(np.isnan(x), 0x7FC0, 0).astype(np.uint16)
    want = O.masked_argmax(host, m)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    buf = torch.zeros(B * (V + stride_pad) + offset + 8, dtype=tdt, device="cuda")
    view = buf[offset:offset + B * (V + stride_pad)].view(B, V + stride_pad)[:, :V]
    view.copy_(H.dev_logits(host))
    before = H.host_logit_bits(view.contiguous()).copy()
    d_tok = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    wg.masked_argmax(view, torch.from_numpy(m.view(np.int32)).cuda(), d_tok)
    assert d_tok.cpu().tolist() == want.tolist()
    assert want[4] == -1 and want[5] == (W // 2) * 32 + 7
    assert (H.host_logit_bits(view.contiguous()) == before).all()          # logits are only read


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V,stride_pad,offset,k", [(151936, 0, 0, 50), (20000, 0, 0, 64), (4104, 8, 0, 64),
                                                   (1000 + 13, 3, 0, 7), (4096, 0, 1, 1), (40, 0, 0, 64),
                                                   (500000, 0, 0, 64)])    # 62 slices: near the merge's limit
def test_masked_topk_matches_oracle(torch_cuda, dtype, V, stride_pad, offset, k):
    """The k best allowed tokens per row, ids and raw values, bit for bit; several 8,192-token
    slices and a ragged last one, rows with fewer than k allowed tokens, ties, NaNs, padded and
    misaligned rows."""
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    B, W = 11, (V + 31) // 32
    x = ws.make_logits(9, B, V, 2.0)
    x[0, 3], x[0, 4], x[1, 5], x[2, :] = np.nan, np.inf, -0.0, np.nan
    x[3, V // 3:V // 3 + 100] = 7.5                       # a long tie at the top
    x[7, :] = -np.arange(V, dtype=np.float32) / 64.0       # descending: the best tokens sit in few threads
    x[8, :] = 1.0                                          # all equal: the lowest ids win
    x[9, :] = np.arange(V, dtype=np.float32) / 64.0        # ascending: the best tokens are the row's last
    m = ws.rng.draw(10, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[:, -1] &= (1 << (V % 32)) - 1 if V % 32 else 0xFFFFFFFF
    m[4, :] = 0                                           # nothing allowed
    m[5, :] = 0
    m[5, W // 2] = 1 << 7                                 # a single allowed token
    m[6, :] = 0xFFFFFFFF
    m[6, -1] = m[0, -1] | 1
    m[10, :] = 0
    m[10, :: max(1, W // 5)] = 0x00010001                 # a dozen allowed tokens, far apart
    m[:, -1] &= (1 << (V % 32)) - 1 if V % 32 else 0xFFFFFFFF             # no bits at or above V
    host = x if dtype == "f32" else ws.to_bf16_bits(np.nan_to_num(x, nan=0.0)) | np.where(np.isnan(x), 0x7FC0, 0).astype(np.uint16)
    want_ids, want_vals = O.masked_topk(host, m, k)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    buf = torch.zeros(B * (V + stride_pad) + offset + 8, dtype=tdt, device="cuda")
    view = buf[offset:offset + B * (V + stride_pad)].view(B, V + stride_pad)[:, :V]
    view.copy_(H.dev_logits(host))
    before = H.host_logit_bits(view.contiguous()).copy()
    d_ids = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    d_vals = torch.zeros((B, k), dtype=tdt, device="cuda")
    work = torch.full((wg.masked_topk_workspace(B, V, k) // 8,), -1, dtype=torch.int64, device="cuda")
    d_mask = torch.from_numpy(m.view(np.int32)).cuda()
    for rep in range(2):                                   # the second call finds the workspace used
        wg.masked_topk(view, d_mask, d_ids, d_vals, work)
        assert (d_ids.cpu().numpy() == want_ids).all()
        got_vals = H.host_logit_bits(d_vals)
        assert (got_vals == (want_vals.view(np.uint32) if dtype == "f32" else want_vals)).all()
    assert (want_ids[4] == -1).all() and want_ids[5].tolist() == [(W // 2) * 32 + 7] + [-1] * (k - 1)
    assert (H.host_logit_bits(view.contiguous()) == before).all()          # logits are only read
    d_tok = torch.empty(B, dtype=torch.int32, device="cuda")
    wg.masked_argmax(view, d_mask, d_tok)
    assert (d_tok.cpu().numpy() == want_ids[:, 0]).all()                   # the best of the k is the greedy choice


def test_masked_topk_under_the_masks_of_a_decode_batch(torch_cuda):
    """Masks as the fill makes them (literal states with a handful of tokens, free-text Waits
    with most of the vocabulary), config 4 reduced."""
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    w = ws.make_workload(4, V=33003 - 3, B=24, steps=30)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    cur = H.start_states(o, w)
    toks, sts, _ = o.trajectory(cur, w.token_draws(30))
    d_states = H.dev_states(cur)
    d_mask = torch.empty((w.B, h.W), dtype=torch.int32, device="cuda")
    k = 40
    d_ids = torch.empty((w.B, k), dtype=torch.int32, device="cuda")
    d_vals = torch.empty((w.B, k), dtype=torch.bfloat16, device="cuda")
    work = torch.empty(wg.masked_topk_workspace(w.B, w.vocab.V, k), dtype=torch.uint8, device="cuda")
    for step in range(30):
        h.fill_masks(d_states, d_mask)
        if step % 6 == 5:
            host = H.logits_for(w, tag=step)
            wg.masked_topk(H.dev_logits(host), d_mask, d_ids, d_vals, work)
            want_ids, want_vals = O.masked_topk(host, o.fill_masks(cur), k)
            assert (d_ids.cpu().numpy() == want_ids).all(), step
            assert (H.host_logit_bits(d_vals) == want_vals).all(), step
        h.advance(d_states, torch.from_numpy(toks[step]).cuda())
        cur = o.advance(cur, toks[step])


def test_greedy_decoding_without_writing_logits(torch_cuda):
    """fill -> masked_argmax -> advance equals fill -> apply -> argmax -> advance (config 1)."""
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    w = ws.make_workload(1)
    o = H.make_oracle(w)
    v, h = H.make_gpu(w)
    cur = H.start_states(o, w)
    d_states = H.dev_states(cur)
    d_mask = torch.empty((1, h.W), dtype=torch.int32, device="cuda")
    d_tok = torch.empty(1, dtype=torch.int32, device="cuda")
    for k in range(w.steps):
        h.fill_masks(d_states, d_mask)
        host = H.logits_for(w, tag=k)
        wg.masked_argmax(H.dev_logits(host), d_mask, d_tok)
        masked = O.apply_mask(host.copy(), o.mask_row(tuple(cur[0]))[None, :])
        tok = int(np.argmax(masked[0]))
        assert int(d_tok.item()) == tok == int(O.masked_argmax(host, o.mask_row(tuple(cur[0]))[None, :])[0])
        h.advance(d_states, d_tok)
        cur = o.advance(cur, [tok])
        assert (H.host_states(d_states) == cur).all()


def test_select_tokens_matches_oracle(torch_cuda):
    torch = torch_cuda
    import paper_2507_16768_amd as wg
    B, V = 9, 5003
    W = (V + 31) // 32
    m = ws.rng.draw(5, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[:, -1] &= (1 << (V % 32)) - 1
    m[1, :] = 0
    m[2, :] = 0
    m[2, 77] = 1 << 9
    draws = ws.rng.draw(6, 9, np.arange(B))
    want = [O.select_bit(m[b], int(draws[b]) % max(1, int(H.bits(m[b], V).sum()))) if m[b].any() else -1
            for b in range(B)]
    d_tok = torch.zeros(B, dtype=torch.int32, device="cuda")
    wg.select_tokens(torch.from_numpy(m.view(np.int32)).cuda(), V,
                     torch.from_numpy(draws.view(np.int64)).cuda(), d_tok)
    assert d_tok.cpu().tolist() == want


def test_argument_errors_on_device_calls(torch_cuda):
    torch = torch_cuda
    import ctypes as C
    import paper_2507_16768_amd as wg
    w = ws.make_workload(1, V=2000)
    v, h = H.make_gpu(w)
    L = wg.load_library()
    assert L.wg_fill_masks(h._h, None, 1, None, None) == -1
    assert L.wg_fill_masks(h._h, C.c_void_p(16), 0, C.c_void_p(16), None) == -1
    assert L.wg_apply_mask(C.c_void_p(16), 7, 1, 32, 32, C.c_void_p(16), None) == -1
    assert L.wg_apply_mask(C.c_void_p(16), 0, 1, 32, 16, C.c_void_p(16), None) == -1
    assert L.wg_advance(None, None, None, 1, None) == -1
    assert b"null" in L.wg_last_error()
    assert L.wg_decode_step(h._h, C.c_void_p(16), None, 1, C.c_void_p(16), None, 0, 2000, None) == -1
    assert L.wg_decode_step(h._h, C.c_void_p(16), None, 1, C.c_void_p(16), C.c_void_p(16), 5, 2000, None) == -1
    assert L.wg_decode_step(h._h, C.c_void_p(16), None, 1, C.c_void_p(16), C.c_void_p(16), 0, 1999, None) == -1
    assert L.wg_decode_step(h._h, C.c_void_p(16), None, 0, C.c_void_p(16), C.c_void_p(16), 0, 2000, None) == -1
    assert L.wg_advance_fill_masks(h._h, C.c_void_p(16), None, 1, C.c_void_p(16), None) == -1
    assert L.wg_cache_resize(h._h, 0) == -1
    p16, ws_bytes = C.c_void_p(16), L.wg_masked_topk_workspace(1, 2000, 8)
    assert ws_bytes == 1 * 1 * 8 * 8 and L.wg_masked_topk_workspace(3, 8193, 64) == 3 * 2 * 64 * 8
    assert L.wg_masked_topk(p16, 0, 1, 2000, 2000, p16, 0, p16, p16, p16, ws_bytes, None) == -1      # k = 0
    assert L.wg_masked_topk(p16, 0, 1, 2000, 2000, p16, 65, p16, p16, p16, 1 << 20, None) == -1      # k > 64
    assert L.wg_masked_topk(p16, 0, 1, 2000, 2000, p16, 8, p16, p16, p16, ws_bytes - 1, None) == -1  # workspace too small
    assert b"workspace" in L.wg_last_error()
    assert L.wg_masked_topk(p16, 0, 1, 2000, 2000, p16, 8, p16, p16, C.c_void_p(20), ws_bytes, None) == -1
    assert L.wg_masked_topk(p16, 0, 1, 2000, 2000, p16, 8, p16, p16, None, ws_bytes, None) == -1
    assert L.wg_masked_topk(p16, 0, 1, 8192 * 129, 8192 * 129, p16, 64, p16, p16, p16, 1 << 30, None) == -1
    with pytest.raises(wg.WgError):
        wg.Vocab(np.zeros(4, np.uint8), np.array([0, 3, 2], np.uint64), 0)


def test_plain_c_client_of_the_abi(torch_cuda):
    """tests/abi/c_client.c: the calls of include/wg.h made from C (hipMalloc memory, a stream of its
    own, no Python in between) and compared with the C oracle inside the same program."""
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "abi", "c_client")
    if not os.path.exists(exe):                           # a second of gcc; the HIP library itself is never built here
        import __graft_entry__ as g
        g.build_c_client()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert r.returncode == 0 and r.stdout.strip().endswith("c_client ok"), (r.returncode, r.stdout[-500:], r.stderr[-1000:])
