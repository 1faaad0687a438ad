"""Helpers shared by the GPU parity tests: upload of seeded inputs, error metric, oracle chaining."""
import functools

import numpy as np

import oracle
import workloads
from workloads.device import dev_f32, dev_i32, dev_i64, to_device  # noqa: F401


@functools.lru_cache(maxsize=2)
def cached_inputs(cfg_index: int, seed: int, variant: str):
    return workloads.make_inputs(workloads.get_config(cfg_index), seed, variant)


def rel_err_rms_floor(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - o_i| / max(|o_i|, rms(o)): relative error with an RMS floor (pure relative error is
    undefined where the reference crosses zero)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref ** 2)))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), max(rms, 1e-30))))


def rel_err_plain_above_rms(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - o_i| / |o_i| over the entries with |o_i| >= rms(o): the plain relative error where it is defined.
    It can never exceed rel_err_rms_floor (on these entries the two denominators are the same); the tests assert it
    next to the floored metric so that the plain 2e-3 figure is visible as such."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref ** 2)))
    big = np.abs(ref) >= max(rms, 1e-30)
    if not big.any():
        return 0.0
    return float(np.max(np.abs(got - ref)[big] / np.abs(ref)[big]))


def oracle_stage3(topk_id, topk_logp, root_token, cfg_blank, beam, max_nodes):
    """Run the oracle's collapse/tree stage for every sequence of a batch on (GPU-produced) top-k lists."""
    return [oracle.collapse_tree(topk_id[b], np.asarray(topk_logp[b], dtype=np.float32), int(root_token[b]),
                                 cfg_blank, beam, max_nodes) for b in range(topk_id.shape[0])]


STAGE3_INT_FIELDS = ("cand_tokens", "cand_len", "cand_leaf", "node_token", "node_parent", "node_depth")


def compare_stage3(gpu: dict, ref: list):
    """Bit-exact comparison of every stage-3 output against the oracle's (per sequence)."""
    g = {k: v.cpu().numpy() for k, v in gpu.items()}
    for b, r in enumerate(ref):
        assert int(g["n_cand"][b]) == r["n_cand"], (b, int(g["n_cand"][b]), r["n_cand"])
        assert int(g["n_nodes"][b]) == r["n_nodes"], (b, int(g["n_nodes"][b]), r["n_nodes"])
        for name in STAGE3_INT_FIELDS:
            assert np.array_equal(g[name][b], r[name]), (b, name, g[name][b], r[name])
        # scores are float32 on both sides: equal bit patterns
        assert np.array_equal(g["cand_score"][b].view(np.uint32), r["cand_score"].view(np.uint32)), \
            (b, g["cand_score"][b], r["cand_score"])
        assert np.array_equal(g["anc_mask"][b].view(np.uint64), r["anc_mask"]), (b, "anc_mask")
