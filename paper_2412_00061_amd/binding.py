"""ctypes binding of libctcspec.so.  Argument marshalling only: every step runs in the HIP kernels.

Each function has the name of the C entry point it calls and takes torch tensors that already live on
the GPU.  Output tensors are allocated with torch when the caller does not pass them in `out`.
"""
import ctypes
import os
from ctypes import POINTER, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = (
    "ctcspec_create", "ctcspec_destroy", "ctcspec_set_stream", "ctcspec_last_error",
    "ctcspec_workspace_bytes", "ctcspec_profile_draft_head", "ctcspec_draft_head_kernel_ms", "ctc_draft_topk", "ctc_collapse_tree", "tree_verify_attn",
    "accept_longest", "verify_head_argmax", "kv_commit", "draft_layer_workspace_bytes", "draft_layer_forward",
    "ctc_sum_score", "ctc_raw_tree", "ctc_loss_workspace_bytes", "ctc_loss", "verify_sample_tokens",
    "ctc_draft_topk_noalloc", "ctcspec_defer_topk_merge", "ctcspec_flush", "ctcspec_stream_probe",
)

CTCSPEC_F32, CTCSPEC_BF16 = 0, 1


class CtcspecError(RuntimeError):
    pass


class _Limits(ctypes.Structure):
    _fields_ = [(n, c_int) for n in ("max_batch", "max_slots", "max_topk", "max_vocab_rows",
                                     "max_nodes", "max_heads", "max_head_dim")]


class _LayerWeights(ctypes.Structure):
    _fields_ = [(n, c_void_p) for n in ("ln1", "wqkv", "wo", "ln2", "wgu", "wd")]


def library_path() -> str:
    return os.path.join(_HERE, "libctcspec.so")


def load_library():
    """Load the built library; fail loudly when it is missing (there is no fallback path)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise CtcspecError(
            f"{path} is missing: build it with `python -m paper_2412_00061_amd.build` "
            "(the HIP library is the only implementation; there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    lib.ctcspec_create.restype = c_int
    lib.ctcspec_create.argtypes = [POINTER(c_void_p), c_void_p, POINTER(_Limits)]
    lib.ctcspec_destroy.restype = None
    lib.ctcspec_destroy.argtypes = [c_void_p]
    lib.ctcspec_set_stream.restype = c_int
    lib.ctcspec_set_stream.argtypes = [c_void_p, c_void_p]
    lib.ctcspec_last_error.restype = c_char_p
    lib.ctcspec_last_error.argtypes = [c_void_p]
    lib.ctcspec_workspace_bytes.restype = c_size_t
    lib.ctcspec_workspace_bytes.argtypes = [c_void_p]
    lib.ctcspec_defer_topk_merge.restype = c_int
    lib.ctcspec_defer_topk_merge.argtypes = [c_void_p, c_int]
    lib.ctcspec_flush.restype = c_int
    lib.ctcspec_flush.argtypes = [c_void_p]
    lib.ctcspec_stream_probe.restype = c_int
    lib.ctcspec_stream_probe.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    lib.ctcspec_profile_draft_head.restype = c_int
    lib.ctcspec_profile_draft_head.argtypes = [c_void_p, c_int]
    lib.ctcspec_draft_head_kernel_ms.restype = c_int
    lib.ctcspec_draft_head_kernel_ms.argtypes = [c_void_p, POINTER(c_float)]
    lib.ctc_draft_topk.restype = c_int
    lib.ctc_draft_topk.argtypes = [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int,
                                   c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.ctc_draft_topk_noalloc.restype = c_int
    lib.ctc_draft_topk_noalloc.argtypes = list(lib.ctc_draft_topk.argtypes)
    lib.ctc_collapse_tree.restype = c_int
    lib.ctc_collapse_tree.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int32,
                                      c_int, c_int] + [c_void_p] * 10
    lib.tree_verify_attn.restype = c_int
    lib.tree_verify_attn.argtypes = [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                     c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int,
                                     c_int, c_float, c_void_p]
    lib.accept_longest.restype = c_int
    lib.accept_longest.argtypes = [c_void_p] * 6 + [c_int, c_int, c_int] + [c_void_p] * 4
    lib.verify_head_argmax.restype = c_int
    lib.verify_head_argmax.argtypes = [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int,
                                       c_void_p, c_void_p]
    lib.kv_commit.restype = c_int
    lib.kv_commit.argtypes = [c_void_p, c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_void_p,
                              c_int, c_int, c_int, c_int, c_int, c_void_p, c_void_p, c_void_p]
    lib.draft_layer_workspace_bytes.restype = c_size_t
    lib.draft_layer_workspace_bytes.argtypes = [c_int] * 5
    lib.draft_layer_forward.restype = c_int
    lib.draft_layer_forward.argtypes = ([c_void_p, c_int, c_void_p, POINTER(_LayerWeights)] + [c_void_p] * 5 +
                                        [c_int] * 6 + [c_float, c_float, c_void_p, c_size_t] + [c_void_p] * 5)
    lib.ctc_loss_workspace_bytes.restype = c_size_t
    lib.ctc_loss_workspace_bytes.argtypes = [c_int] * 3
    lib.verify_sample_tokens.restype = c_int
    lib.verify_sample_tokens.argtypes = [c_void_p] * 4 + [c_float] + [c_int] * 3 + [c_void_p]
    lib.ctc_loss.restype = c_int
    lib.ctc_loss.argtypes = [c_void_p] * 5 + [c_int] * 4 + [c_int32, c_void_p, c_size_t, c_void_p, c_void_p]
    lib.ctc_raw_tree.restype = c_int
    lib.ctc_raw_tree.argtypes = lib.ctc_collapse_tree.argtypes + [c_void_p]
    lib.ctc_sum_score.restype = c_int
    lib.ctc_sum_score.argtypes = [c_void_p] * 6 + [c_int, c_int, c_int, c_int32, c_int, c_void_p, c_void_p]
    _LIB = lib
    return lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CTCSPEC_F32
    if t.dtype == torch.bfloat16:
        return CTCSPEC_BF16
    raise CtcspecError(f"unsupported element type {t.dtype}")


def _ptr(t, dtype=None):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise CtcspecError("tensors must be contiguous GPU tensors")
    if dtype is not None and t.dtype != dtype:
        raise CtcspecError(f"expected {dtype}, got {t.dtype}")
    return c_void_p(t.data_ptr())


class Context:
    """Owns a ctcspec_ctx: the library's device workspace bound to one HIP stream."""

    def __init__(self, *, max_batch, max_slots, max_topk, max_vocab_rows, max_nodes, max_heads,
                 max_head_dim, stream=None):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise CtcspecError("no GPU visible: libctcspec runs on an MI355X only")
        lim = _Limits(max_batch, max_slots, max_topk, max_vocab_rows, max_nodes, max_heads, max_head_dim)
        stream = torch.cuda.current_stream() if stream is None else stream
        self.stream = stream
        handle = c_void_p()
        rc = self.lib.ctcspec_create(ctypes.byref(handle), c_void_p(stream.cuda_stream), ctypes.byref(lim))
        if rc != 0:
            raise CtcspecError(f"ctcspec_create failed ({rc}): {self.lib.ctcspec_last_error(None).decode()}")
        self.handle = handle

    @classmethod
    def for_config(cls, cfg, stream=None):
        return cls(max_batch=cfg.B, max_slots=cfg.T, max_topk=cfg.k, max_vocab_rows=cfg.Vp1,
                   max_nodes=cfg.max_nodes, max_heads=cfg.H, max_head_dim=cfg.dh, stream=stream)

    def set_stream(self, stream):
        self.stream = stream
        self._check(self.lib.ctcspec_set_stream(self.handle, c_void_p(stream.cuda_stream)), "ctcspec_set_stream")

    def workspace_bytes(self) -> int:
        return int(self.lib.ctcspec_workspace_bytes(self.handle))

    def defer_topk_merge(self, enable: bool):
        """Leave the merge of the draft head's partial results to the next ctc_collapse_tree call (see ctcspec.h)."""
        self._check(self.lib.ctcspec_defer_topk_merge(self.handle, 1 if enable else 0), "ctcspec_defer_topk_merge")

    def flush(self):
        self._check(self.lib.ctcspec_flush(self.handle), "ctcspec_flush")

    def profile_draft_head(self, enable: bool):
        self._check(self.lib.ctcspec_profile_draft_head(self.handle, 1 if enable else 0), "ctcspec_profile_draft_head")

    def draft_head_kernel_ms(self) -> float:
        ms = c_float()
        self._check(self.lib.ctcspec_draft_head_kernel_ms(self.handle, ctypes.byref(ms)), "ctcspec_draft_head_kernel_ms")
        return float(ms.value)

    def last_error(self) -> str:
        return self.lib.ctcspec_last_error(self.handle).decode()

    def _check(self, rc, what):
        if rc != 0:
            raise CtcspecError(f"{what} failed ({rc}): {self.last_error()}")

    def close(self):
        if getattr(self, "handle", None):
            self.lib.ctcspec_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def prepared(ctx, name, *args):
    """Marshal the arguments of C entry point `name` once and return a zero-argument callable that
    issues the call (for launch loops where per-call marshalling would dominate).  `args` follow the C
    parameter order after the context; tensors become device pointers, None becomes NULL."""
    fn = getattr(ctx.lib, name)
    keep, cargs = [], [ctx.handle]
    for a, ctype in zip(args, fn.argtypes[1:]):
        if isinstance(a, torch.Tensor):
            keep.append(a)
            cargs.append(_ptr(a))
        elif a is None:
            cargs.append(None)
        else:
            cargs.append(ctype(a))
    if len(cargs) != len(fn.argtypes):
        raise CtcspecError(f"{name}: expected {len(fn.argtypes) - 1} arguments, got {len(args)}")
    cargs = tuple(cargs)

    def call(_fn=fn, _args=cargs, _keep=keep, _ctx=ctx, _name=name):
        rc = _fn(*_args)
        if rc != 0:
            _ctx._check(rc, _name)

    return call


def _out(out, name, shape, dtype, device):
    if out is not None and name in out:
        t = out[name]
        if tuple(t.shape) != tuple(shape) or t.dtype != dtype:
            raise CtcspecError(f"out[{name!r}] must be {dtype} {tuple(shape)}")
        return t
    return torch.empty(shape, dtype=dtype, device=device)


def ctc_draft_topk(ctx, hidden, w, bias, k, *, want_logits=False, out=None):
    """hidden [B,T,D], w [V+1,D] (same dtype), bias [V+1] f32 or None -> dict(topk_id, topk_logp, lse[, logits])."""
    B, T, D = hidden.shape
    Vp1 = w.shape[0]
    if w.shape[1] != D or w.dtype != hidden.dtype:
        raise CtcspecError("w must be [V+1, D] with hidden's dtype")
    dev = hidden.device
    res = {
        "topk_id": _out(out, "topk_id", (B, T, k), torch.int32, dev),
        "topk_logp": _out(out, "topk_logp", (B, T, k), torch.float32, dev),
        "lse": _out(out, "lse", (B, T), torch.float32, dev),
    }
    if want_logits:
        res["logits"] = _out(out, "logits", (B, T, Vp1), torch.float32, dev)
    rc = ctx.lib.ctc_draft_topk(ctx.handle, _dtype_code(hidden), _ptr(hidden), _ptr(w),
                                _ptr(bias, torch.float32), B, T, D, Vp1, k, _ptr(res["topk_id"]),
                                _ptr(res["topk_logp"]), _ptr(res["lse"]), _ptr(res.get("logits")))
    ctx._check(rc, "ctc_draft_topk")
    return res


def ctc_draft_topk_noalloc(stream, hidden, w, bias, k, *, out, want_logits=False):
    """The same call without a context (the library's static scratch holds the partial results).  `stream`: a
    torch.cuda.Stream or None; `out` must hold every output tensor (this binding allocates nothing either)."""
    B, T, D = hidden.shape
    Vp1 = w.shape[0]
    if w.shape[1] != D or w.dtype != hidden.dtype:
        raise CtcspecError("w must be [V+1, D] with hidden's dtype")
    for name, shape, dtype in (("topk_id", (B, T, k), torch.int32), ("topk_logp", (B, T, k), torch.float32),
                               ("lse", (B, T), torch.float32)) + ((("logits", (B, T, Vp1), torch.float32),) if want_logits else ()):
        if name not in out or tuple(out[name].shape) != shape or out[name].dtype != dtype:
            raise CtcspecError(f"out[{name!r}] must be a {dtype} tensor of shape {shape}")
    lib = load_library()
    rc = lib.ctc_draft_topk_noalloc(c_void_p(stream.cuda_stream if stream is not None else 0), _dtype_code(hidden),
                                    _ptr(hidden), _ptr(w), _ptr(bias, torch.float32), B, T, D, Vp1, k,
                                    _ptr(out["topk_id"]), _ptr(out["topk_logp"]), _ptr(out["lse"]),
                                    _ptr(out["logits"]) if want_logits else None)
    if rc != 0:
        raise CtcspecError(f"ctc_draft_topk_noalloc failed ({rc}): {lib.ctcspec_last_error(None).decode()}")
    return out


def ctc_collapse_tree(ctx, topk_id, topk_logp, root_token, blank_id, beam, max_nodes, *, out=None):
    """topk_id/topk_logp [B,T,k], root_token [B] -> dict of the drafts, the tree and its ancestor mask."""
    B, T, k = topk_id.shape
    dev = topk_id.device
    words = (max_nodes + 63) // 64
    res = {
        "n_cand": _out(out, "n_cand", (B,), torch.int32, dev),
        "cand_tokens": _out(out, "cand_tokens", (B, beam, T), torch.int32, dev),
        "cand_len": _out(out, "cand_len", (B, beam), torch.int32, dev),
        "cand_score": _out(out, "cand_score", (B, beam), torch.float32, dev),
        "cand_leaf": _out(out, "cand_leaf", (B, beam), torch.int32, dev),
        "n_nodes": _out(out, "n_nodes", (B,), torch.int32, dev),
        "node_token": _out(out, "node_token", (B, max_nodes), torch.int32, dev),
        "node_parent": _out(out, "node_parent", (B, max_nodes), torch.int32, dev),
        "node_depth": _out(out, "node_depth", (B, max_nodes), torch.int32, dev),
        "anc_mask": _out(out, "anc_mask", (B, max_nodes, words), torch.int64, dev),
    }
    rc = ctx.lib.ctc_collapse_tree(
        ctx.handle, _ptr(topk_id, torch.int32), _ptr(topk_logp, torch.float32), _ptr(root_token, torch.int32),
        B, T, k, blank_id, beam, max_nodes, _ptr(res["n_cand"]), _ptr(res["cand_tokens"]),
        _ptr(res["cand_len"]), _ptr(res["cand_score"]), _ptr(res["cand_leaf"]), _ptr(res["n_nodes"]),
        _ptr(res["node_token"]), _ptr(res["node_parent"]), _ptr(res["node_depth"]), _ptr(res["anc_mask"]))
    ctx._check(rc, "ctc_collapse_tree")
    return res


def ctc_raw_tree(ctx, topk_id, topk_logp, root_token, blank_id, beam, max_nodes, *, out=None):
    """The literal layout: raw candidates at full length, removed positions masked.  Outputs of ctc_collapse_tree
    plus node_removed [B,max_nodes]."""
    B, T, k = topk_id.shape
    dev = topk_id.device
    words = (max_nodes + 63) // 64
    res = {
        "n_cand": _out(out, "n_cand", (B,), torch.int32, dev),
        "cand_tokens": _out(out, "cand_tokens", (B, beam, T), torch.int32, dev),
        "cand_len": _out(out, "cand_len", (B, beam), torch.int32, dev),
        "cand_score": _out(out, "cand_score", (B, beam), torch.float32, dev),
        "cand_leaf": _out(out, "cand_leaf", (B, beam), torch.int32, dev),
        "n_nodes": _out(out, "n_nodes", (B,), torch.int32, dev),
        "node_token": _out(out, "node_token", (B, max_nodes), torch.int32, dev),
        "node_parent": _out(out, "node_parent", (B, max_nodes), torch.int32, dev),
        "node_depth": _out(out, "node_depth", (B, max_nodes), torch.int32, dev),
        "anc_mask": _out(out, "anc_mask", (B, max_nodes, words), torch.int64, dev),
        "node_removed": _out(out, "node_removed", (B, max_nodes), torch.int32, dev),
    }
    rc = ctx.lib.ctc_raw_tree(
        ctx.handle, _ptr(topk_id, torch.int32), _ptr(topk_logp, torch.float32), _ptr(root_token, torch.int32),
        B, T, k, blank_id, beam, max_nodes, _ptr(res["n_cand"]), _ptr(res["cand_tokens"]),
        _ptr(res["cand_len"]), _ptr(res["cand_score"]), _ptr(res["cand_leaf"]), _ptr(res["n_nodes"]),
        _ptr(res["node_token"]), _ptr(res["node_parent"]), _ptr(res["node_depth"]), _ptr(res["anc_mask"]),
        _ptr(res["node_removed"]))
    ctx._check(rc, "ctc_raw_tree")
    return res


def tree_verify_attn(ctx, q, k_cache, v_cache, kv_off, ctx_len, kv_cap, k_tree, v_tree, n_nodes, anc_mask,
                     scale, *, out=None):
    """q/k_tree/v_tree [B,H,max_nodes,dh]; k_cache/v_cache flat buffers addressed through kv_off -> out f32."""
    B, H, max_nodes, dh = q.shape
    o = _out(None if out is None else {"out": out}, "out", (B, H, max_nodes, dh), torch.float32, q.device)
    rc = ctx.lib.tree_verify_attn(
        ctx.handle, _dtype_code(q), _ptr(q), _ptr(k_cache, q.dtype), _ptr(v_cache, q.dtype),
        _ptr(kv_off, torch.int64), _ptr(ctx_len, torch.int32), kv_cap, _ptr(k_tree, q.dtype),
        _ptr(v_tree, q.dtype), _ptr(n_nodes, torch.int32), _ptr(anc_mask, torch.int64), B, H, dh, max_nodes,
        c_float(scale), _ptr(o))
    ctx._check(rc, "tree_verify_attn")
    return o


def accept_longest(ctx, n_nodes, node_token, node_parent, node_depth, target_argmax, T, *, out=None):
    """Greedy acceptance walk -> dict(accept_len [B], accept_nodes [B,T+1], accept_tokens [B,T+1], next_token [B])."""
    B, max_nodes = node_token.shape
    dev = node_token.device
    res = {
        "accept_len": _out(out, "accept_len", (B,), torch.int32, dev),
        "accept_nodes": _out(out, "accept_nodes", (B, T + 1), torch.int32, dev),
        "accept_tokens": _out(out, "accept_tokens", (B, T + 1), torch.int32, dev),
        "next_token": _out(out, "next_token", (B,), torch.int32, dev),
    }
    rc = ctx.lib.accept_longest(
        ctx.handle, _ptr(n_nodes, torch.int32), _ptr(node_token, torch.int32), _ptr(node_parent, torch.int32),
        _ptr(node_depth, torch.int32), _ptr(target_argmax, torch.int32), B, T, max_nodes,
        _ptr(res["accept_len"]), _ptr(res["accept_nodes"]), _ptr(res["accept_tokens"]), _ptr(res["next_token"]))
    ctx._check(rc, "accept_longest")
    return res


def verify_head_argmax(ctx, node_hidden, w_base, n_nodes, *, want_logits=False, out=None):
    """node_hidden [B,max_nodes,D], w_base [V,D] (same dtype) -> dict(target_argmax [B,max_nodes][, logits])."""
    B, max_nodes, D = node_hidden.shape
    V = w_base.shape[0]
    dev = node_hidden.device
    res = {"target_argmax": _out(out, "target_argmax", (B, max_nodes), torch.int32, dev)}
    if want_logits:
        res["logits"] = _out(out, "logits", (B, max_nodes, V), torch.float32, dev)
    rc = ctx.lib.verify_head_argmax(ctx.handle, _dtype_code(node_hidden), _ptr(node_hidden),
                                    _ptr(w_base, node_hidden.dtype), _ptr(n_nodes, torch.int32), B, max_nodes, D, V,
                                    _ptr(res["target_argmax"]), _ptr(res.get("logits")))
    ctx._check(rc, "verify_head_argmax")
    return res


def kv_commit(ctx, k_tree, v_tree, accept_len, accept_nodes, kv_off, ctx_len, kv_cap, k_cache, v_cache, *,
              ctx_len_out=None):
    """Append the accepted path's K/V rows to the caches in place; ctx_len_out [B] int32 receives the new lengths."""
    B, H, max_nodes, dh = k_tree.shape
    T = accept_nodes.shape[1] - 1
    rc = ctx.lib.kv_commit(ctx.handle, _dtype_code(k_tree), _ptr(k_tree), _ptr(v_tree, k_tree.dtype),
                           _ptr(accept_len, torch.int32), _ptr(accept_nodes, torch.int32), T,
                           _ptr(kv_off, torch.int64), _ptr(ctx_len, torch.int32), kv_cap, B, H, dh, max_nodes,
                           _ptr(k_cache, k_tree.dtype), _ptr(v_cache, k_tree.dtype),
                           _ptr(ctx_len_out, torch.int32) if ctx_len_out is not None else None)
    ctx._check(rc, "kv_commit")


def layer_weights(ln1, wqkv, wo, ln2, wgu, wd):
    """The C struct of device pointers that draft_layer_forward takes (the tensors must outlive the calls)."""
    tensors = (ln1, wqkv, wo, ln2, wgu, wd)
    for t in tensors:
        _ptr(t, torch.bfloat16)
    st = _LayerWeights(*[t.data_ptr() for t in tensors])
    st._keep = tensors
    return st


def draft_layer_workspace_bytes(B, T, D, H, F) -> int:
    return int(load_library().draft_layer_workspace_bytes(B, T, D, H, F))


def draft_layer_forward(ctx, x, weights, pos0, k_cache, v_cache, kv_off, ctx_len, kv_cap, H, F, rms_eps, rope_theta,
                        *, workspace=None, want_f32=False, want_q=False, out=None):
    """x [B,T,D] bf16, weights from layer_weights() -> dict(out [B,T,D], k_new, v_new [B,H,T,dh][, out_f32][, q])."""
    B, T, D = x.shape
    dev = x.device
    need = draft_layer_workspace_bytes(B, T, D, H, F)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    res = {"out": _out(out, "out", (B, T, D), torch.bfloat16, dev),
           "k_new": _out(out, "k_new", (B, H, T, D // H), torch.bfloat16, dev),
           "v_new": _out(out, "v_new", (B, H, T, D // H), torch.bfloat16, dev)}
    if want_f32:
        res["out_f32"] = _out(out, "out_f32", (B, T, D), torch.float32, dev)
    if want_q:
        res["q"] = _out(out, "q", (B, H, T, D // H), torch.bfloat16, dev)
    rc = ctx.lib.draft_layer_forward(ctx.handle, _dtype_code(x), _ptr(x), ctypes.byref(weights),
                                     _ptr(pos0, torch.int32), _ptr(k_cache, x.dtype), _ptr(v_cache, x.dtype),
                                     _ptr(kv_off, torch.int64), _ptr(ctx_len, torch.int32), kv_cap, B, T, D, H, F,
                                     rms_eps, rope_theta, _ptr(workspace, torch.uint8), workspace.numel(),
                                     _ptr(res.get("q")), _ptr(res["k_new"]), _ptr(res["v_new"]), _ptr(res["out"]), _ptr(res.get("out_f32")))
    ctx._check(rc, "draft_layer_forward")
    return res


def ctc_sum_score(ctx, logits, lse, cand_tokens, cand_len, n_cand, blank_id, *, out=None):
    """logits [B,T,V+1] f32, lse [B,T] f32, candidates of ctc_collapse_tree -> dict(cand_logp_sum, cand_rank_sum)."""
    B, T, Vp1 = logits.shape
    beam = cand_tokens.shape[1]
    dev = logits.device
    res = {"cand_logp_sum": _out(out, "cand_logp_sum", (B, beam), torch.float32, dev),
           "cand_rank_sum": _out(out, "cand_rank_sum", (B, beam), torch.int32, dev)}
    rc = ctx.lib.ctc_sum_score(ctx.handle, _ptr(logits, torch.float32), _ptr(lse, torch.float32),
                               _ptr(cand_tokens, torch.int32), _ptr(cand_len, torch.int32), _ptr(n_cand, torch.int32),
                               B, T, Vp1, blank_id, beam, _ptr(res["cand_logp_sum"]), _ptr(res["cand_rank_sum"]))
    ctx._check(rc, "ctc_sum_score")
    return res


def ctc_loss_workspace_bytes(B, T, Lmax) -> int:
    return int(load_library().ctc_loss_workspace_bytes(B, T, Lmax))


def ctc_loss(ctx, logits, labels, label_len, frame_len, blank_id, *, want_grad=True, workspace=None, out=None):
    """logits [B,T,V+1] f32, labels [B,Lmax] i32 -> dict(loss [B][, grad [B,T,V+1]])."""
    B, T, Vp1 = logits.shape
    Lmax = labels.shape[1]
    dev = logits.device
    need = ctc_loss_workspace_bytes(B, T, Lmax)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    res = {"loss": _out(out, "loss", (B,), torch.float32, dev)}
    if want_grad:
        res["grad"] = _out(out, "grad", (B, T, Vp1), torch.float32, dev)
    rc = ctx.lib.ctc_loss(ctx.handle, _ptr(logits, torch.float32), _ptr(labels, torch.int32),
                          _ptr(label_len, torch.int32), _ptr(frame_len, torch.int32), B, T, Vp1, Lmax, blank_id,
                          _ptr(workspace, torch.uint8), workspace.numel(), _ptr(res["loss"]), _ptr(res.get("grad")))
    ctx._check(rc, "ctc_loss")
    return res


def verify_sample_tokens(ctx, logits, n_nodes, uniforms, temperature, *, out=None):
    """logits [B,N,V] f32, uniforms [B,N] f32 in [0,1) -> target_sampled [B,N] i32."""
    B, N, V = logits.shape
    res = _out(out, "target_sampled", (B, N), torch.int32, logits.device)
    rc = ctx.lib.verify_sample_tokens(ctx.handle, _ptr(logits, torch.float32), _ptr(n_nodes, torch.int32),
                                      _ptr(uniforms, torch.float32), float(temperature), B, N, V, _ptr(res))
    ctx._check(rc, "verify_sample_tokens")
    return res
