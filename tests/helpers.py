"""Shared plumbing of the tests: build both sides from one Workload, unpack rows."""
import numpy as np

import wg_synth as ws
from oracle import oracle as O


def bits(row, V):
    return np.unpackbits(np.ascontiguousarray(row).view(np.uint8), bitorder="little")[:V].astype(bool)


def make_oracle(w, restart=True):
    ov = O.OracleVocab(w.vocab.bytes, w.vocab.offsets, w.vocab.eos_id)
    return O.Oracle(w.texts, w.args, ov, restart=restart)


def start_states(o, w):
    return np.array([[o.start_state(int(t)), 0] for t in w.request_template], dtype=np.uint32)


def make_gpu(w, restart=True, share=False):
    import paper_2507_16768_amd as wg
    v = wg.Vocab(w.vocab.bytes, w.vocab.offsets, w.vocab.eos_id)
    h = wg.Handle(w.texts, w.args, v, flags=(wg.EOS_RESTART if restart else wg.EOS_STOP) | (wg.SHARE_STATES if share else 0))
    return v, h


def dev_states(st):
    import torch
    return torch.from_numpy(np.ascontiguousarray(st, dtype=np.uint32).view(np.int32).copy()).cuda()


def host_states(t):
    return t.cpu().numpy().view(np.uint32)


def host_mask(t):
    return t.cpu().numpy().view(np.uint32)


def logits_for(w, tag):
    """Host logits of the workload's dtype: float32 array, or uint16 bf16 bit patterns."""
    x = ws.make_logits(w.seed, w.B, w.vocab.V, w.sigma, tag=tag)
    return x if w.dtype == "f32" else ws.to_bf16_bits(x)


def dev_logits(host):
    import torch
    if host.dtype == np.float32:
        return torch.from_numpy(host.copy()).cuda()
    return torch.from_numpy(host.view(np.int16).copy()).cuda().view(torch.bfloat16)


def host_logit_bits(t):
    import torch
    if t.dtype == torch.float32:
        return t.cpu().numpy().view(np.uint32)
    return t.view(torch.int16).cpu().numpy().view(np.uint16)
