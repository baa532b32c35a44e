"""The seeded input generators: reference values of the mixer, shapes, distributions."""
import numpy as np

import wg_synth as ws
from wg_synth.rng import draw, mix64


def test_mixer_reproduces_published_splitmix64_outputs():
    # SplitMix64 seeded with 0 emits mix(gamma), mix(2*gamma), mix(3*gamma); these three
    # values are the ones quoted with the reference implementation of the generator.
    g = 0x9E3779B97F4A7C15
    got = [int(mix64(np.uint64((k * g) % 2**64))) for k in range(3)]
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_draw_is_a_pure_function_of_its_counters():
    a = draw(0, 1, np.arange(1000))
    assert (a == draw(0, 1, np.arange(1000))).all()
    assert len(set(a.tolist())) == 1000
    assert (draw(0, 1, np.arange(8)) != draw(0, 2, np.arange(8))).all()
    assert (draw(1, 1, np.arange(8)) != draw(0, 1, np.arange(8))).all()
    assert int(draw(0, 1, 5)) == int(a[5])


def test_vocab_layout_and_length_distributions():
    v = ws.make_vocab(32000, ("uniform", 1, 8), seed=0)
    L = v.lengths()
    assert v.V == 32000 and L[0] == 0 and (L[1:257] == 1).all() and v.lmax == 8
    assert [v.token(i) for i in (1, 66, 256)] == [b"\x00", b"A", b"\xff"]
    assert abs(L[257:].mean() - 4.5) < 0.05 and L[257:].min() == 1
    body = v.bytes[256:]
    assert body.min() >= 0x20 and body.max() <= 0x7E
    g = ws.make_vocab(151936, ("geometric", 5, 24), seed=0, utf8_tenths=1)
    Lg = g.lengths()[257:]
    assert g.lmax == 24 and abs(Lg.mean() - 4.98) < 0.03
    assert abs((Lg == 1).mean() - 0.2) < 0.01 and abs((Lg > 8).mean() - 0.8**8) < 0.01
    first = g.bytes[g.offsets[257:-1].astype(np.int64)]
    assert abs((first >= 0x80).mean() - 0.10) < 0.01
    assert int(g.offsets[-1]) == len(g.bytes)


def test_utf8_tokens_are_valid_up_to_truncation():
    g = ws.make_vocab(20000, ("geometric", 4, 16), seed=2, utf8_tenths=1)
    n_multi = 0
    for t in range(257, g.V):
        b = g.token(t)
        if b[0] >= 0x80:
            n_multi += 1
            assert b.decode("utf-8", errors="ignore").encode("utf-8") in (b, b[:len(b) - 1], b[:len(b) - 2], b[:len(b) - 3])
    assert n_multi > 1000


def test_workloads_have_the_stated_shapes():
    for i, (V, B, steps, dt) in {1: (32000, 1, 64, "f32"), 2: (128256, 64, 512, "bf16"),
                                 3: (128256, 128, 1024, "f32"), 4: (151936, 256, 1024, "bf16"),
                                 5: (151936, 1024, 4096, "bf16")}.items():
        w = ws.make_workload(i)
        assert (w.vocab.V, w.B, w.steps, w.dtype) == (V, B, steps, dt)
        assert len(w.request_template) == B and w.request_template.max() == len(w.texts) - 1
    w4 = ws.make_workload(4)
    assert len(w4.texts) == 256 and len(set(w4.texts)) == 2        # static text, dynamic args
    assert len({a["t3"] for a in w4.args[0::2]}) == 128
    w5 = ws.make_workload(5)
    n = [ws.templates.count_leaves(a) for a in w5.asts]
    assert len(n) == 16 and min(n) >= 64 and max(n) <= 256
    assert max(ws.configs.nesting_depth(a) for a in w5.asts) == 4
    d = w4.token_draws(3)
    assert d.shape == (3, 256) and d.dtype == np.uint64


def test_logits_are_normal_and_bf16_rounding_is_nearest_even():
    x = ws.make_logits(0, 4, 50000, 2.0)
    assert x.dtype == np.float32 and abs(x.std() - 2.0) < 0.02 and abs(x.mean()) < 0.02
    assert not (ws.make_logits(0, 4, 50000, 2.0, tag=1) == x).all()
    f = np.array([1.0, 1.00390625, 1.01171875, -3.0, 0.0], dtype=np.float32)
    # 1.00390625 = 0x3F808000 is a tie -> even (0x3F80); 1.01171875 = 0x3F818000 tie -> 0x3F82
    assert ws.to_bf16_bits(f).tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC040, 0x0000]
