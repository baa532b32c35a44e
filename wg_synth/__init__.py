"""Seeded synthetic inputs: vocabularies, operator templates, logits, token draws.

This package only *generates inputs*.  It holds none of the structured-decoding
arithmetic (no FSM stepping, no masks): the CPU oracle and the HIP library each
implement that on their own and both are fed from here.
"""
from .rng import draw, draw_range            # noqa: F401
from .vocab import Vocab, make_vocab          # noqa: F401
from .templates import (                      # noqa: F401
    EOS, Hole, Write, Wait, CondWait, IfElse, DoWhile, Sequence,
    to_text, instantiate,
)
from .configs import Workload, make_workload, CONFIG_NAMES   # noqa: F401
from .logits import make_logits, to_bf16_bits                  # noqa: F401
