"""wg_masked_topk_static (the entry point that allocates nothing: its lists live in a device
array inside the library) against wg_masked_topk with a caller's workspace, through the C ABI."""
import numpy as np
import pytest

import wg_synth as ws
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _case(torch, wg, B, V, k, dtype, seed):
    W = (V + 31) // 32
    x = ws.make_logits(seed, B, V, 2.0)
    x[0, 3], x[0, 4] = np.nan, np.inf
    x[1, V // 3:V // 3 + 70] = 7.5                         # a long tie at the top
    m = ws.rng.draw(seed, 9, np.arange(B * W)).astype(np.uint32).reshape(B, W)
    m[2, :] = 0                                            # nothing allowed
    m[3, :] = 0
    m[3, W // 2] = 1 << 7                                  # a single allowed token
    m[:, -1] &= (1 << (V % 32)) - 1 if V % 32 else 0xFFFFFFFF
    host = x if dtype == "f32" else ws.to_bf16_bits(np.nan_to_num(x, nan=0.0)) | np.where(np.isnan(x), 0x7FC0, 0).astype(np.uint16)
    d_log = H.dev_logits(host)
    d_mask = torch.from_numpy(m.view(np.int32)).cuda()
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    want_ids = torch.full((B, k), -7, dtype=torch.int32, device="cuda")
    want_vals = torch.zeros((B, k), dtype=tdt, device="cuda")
    work = torch.empty(wg.masked_topk_workspace(B, V, k), dtype=torch.uint8, device="cuda")
    wg.masked_topk(d_log, d_mask, want_ids, want_vals, work)
    got_ids = torch.full((B, k), -9, dtype=torch.int32, device="cuda")
    got_vals = torch.ones((B, k), dtype=tdt, device="cuda")
    torch.cuda.synchronize()
    return d_log, d_mask, want_ids, want_vals, got_ids, got_vals


def test_masked_topk_static_matches_the_workspace_call_twice_in_a_row():
    import torch
    import paper_2507_16768_amd as wg
    assert torch.cuda.is_available(), "this test needs the GPU"
    L = wg.load_library()
    assert wg.masked_topk_static_capacity() == 4 << 20
    # first the shape the benchmark times (19 slices per row), then a smaller one that leaves
    # most of the array holding the first call's keys
    first = _case(torch, wg, 256, 151936, 50, "bf16", 21)
    second = _case(torch, wg, 7, 20000 + 13, 64, "f32", 22)
    for d_log, d_mask, want_ids, want_vals, got_ids, got_vals in (first, second):
        before = torch.cuda.memory_allocated()
        wg.masked_topk_static(d_log, d_mask, got_ids, got_vals)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        assert (got_ids.cpu().numpy() == want_ids.cpu().numpy()).all()
        assert (H.host_logit_bits(got_vals) == H.host_logit_bits(want_vals)).all()
        assert (want_ids[2] == -1).all() and (want_ids[3, 1:] == -1).all() and want_ids[3, 0] >= 0
    # and once more on the large shape: the array now holds the small call's keys in front
    d_log, d_mask, want_ids, want_vals, got_ids, got_vals = first
    got_ids.fill_(-9)
    wg.masked_topk_static(d_log, d_mask, got_ids, got_vals)
    assert (got_ids.cpu().numpy() == want_ids.cpu().numpy()).all()
    assert (H.host_logit_bits(got_vals) == H.host_logit_bits(want_vals)).all()
    # beyond the array: refused, nothing launched
    import ctypes as C
    p16 = C.c_void_p(16)
    assert 1024 * 19 * 64 * 8 > wg.masked_topk_static_capacity()
    assert L.wg_masked_topk_static(p16, 1, 1024, 151936, 151936, p16, 64, p16, p16, None) == -1
    assert b"workspace" in L.wg_last_error()
    assert L.wg_masked_topk_static(p16, 1, 1, 2000, 2000, p16, 0, p16, p16, None) == -1
    assert L.wg_masked_topk_static(None, 1, 1, 2000, 2000, p16, 8, p16, p16, None) == -1
