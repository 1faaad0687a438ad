"""MI355X-native per-step device work of CTC-drafted speculative decoding.

The product is `libctcspec.so`, a C-ABI library of hand-written HIP kernels for gfx950 (see
`include/ctcspec.h`).  This package is the thin Python binding over it: it marshals torch device
tensors into the C calls and nothing else.  There is no CPU fallback: importing the binding without
the built library raises.
"""
from .binding import (  # noqa: F401
    Context,
    CtcspecError,
    accept_longest,
    ctc_collapse_tree,
    ctc_draft_topk,
    ctc_draft_topk_noalloc,
    ctc_loss,
    verify_sample_tokens,
    ctc_loss_workspace_bytes,
    ctc_raw_tree,
    ctc_sum_score,
    draft_layer_forward,
    draft_layer_workspace_bytes,
    kv_commit,
    layer_weights,
    library_path,
    load_library,
    prepared,
    tree_verify_attn,
    verify_head_argmax,
)
