"""MI355X-native hot path of operator-based structured decoding (mask creation with a
device-resident cache, logit masking, state advance) behind a small C ABI.

`binding` wraps the shared library one-to-one; it marshals arguments and nothing else.
"""
from .binding import (  # noqa: F401
    WgError, Vocab, Handle, Table, apply_mask, masked_argmax, masked_topk, masked_topk_workspace, masked_topk_static, masked_topk_static_capacity, select_tokens, regex_to_template, marshal_templates,
    load_library, library_path,
    F32, BF16, EOS_STOP, EOS_RESTART, SHARE_STATES, SID_FINAL, SID_ERROR,
)
