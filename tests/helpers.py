"""Shared test helpers: small random parameter sets and pools for the CPU oracle."""
from __future__ import annotations

import dataclasses

import numpy as np


@dataclasses.dataclass(frozen=True)
class MiniShape:
    n_layers: int = 2
    hidden: int = 32
    n_q_heads: int = 4
    n_kv_heads: int = 2
    head_dim: int = 8
    ffn: int = 48
    vocab: int = 64
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    qk_norm: bool = False                 # RMSNorm over head_dim on q and k heads before the rotation
    rope_scaling: tuple = None            # (factor, low_freq_factor, high_freq_factor, original_max_position)
    qkv_bias: bool = False                # bias vectors on the q, k and v projections


def random_weights(shape, rng, dtype=np.float64, std=0.3, gains_random=True):
    """Dense numpy parameters; gains are random (not 1) so that a dropped gain shows."""
    def mat(r, c):
        return np.ascontiguousarray(rng.normal(0.0, std, size=(r, c)).astype(dtype))

    def gain():
        g = 1.0 + 0.2 * rng.normal(size=shape.hidden) if gains_random else np.ones(shape.hidden)
        return np.ascontiguousarray(g.astype(dtype))

    qd, kd = shape.n_q_heads * shape.head_dim, shape.n_kv_heads * shape.head_dim
    w = {"embed": mat(shape.vocab, shape.hidden)}
    for k in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd"):
        w[k] = []
    for _ in range(shape.n_layers):
        w["g1"].append(gain())
        w["wq"].append(mat(qd, shape.hidden))
        w["wk"].append(mat(kd, shape.hidden))
        w["wv"].append(mat(kd, shape.hidden))
        w["wo"].append(mat(shape.hidden, qd))
        w["g2"].append(gain())
        w["wg"].append(mat(shape.ffn, shape.hidden))
        w["wu"].append(mat(shape.ffn, shape.hidden))
        w["wd"].append(mat(shape.hidden, shape.ffn))
    w["gf"] = gain()
    w["wlm"] = mat(shape.vocab, shape.hidden)
    if getattr(shape, "qk_norm", False):
        w["qn"] = [np.ascontiguousarray((1.0 + 0.2 * rng.normal(size=shape.head_dim)).astype(dtype)) for _ in range(shape.n_layers)]
        w["kn"] = [np.ascontiguousarray((1.0 + 0.2 * rng.normal(size=shape.head_dim)).astype(dtype)) for _ in range(shape.n_layers)]
    if getattr(shape, "qkv_bias", False):
        for k, n in (("bq", qd), ("bk", kd), ("bv", kd)):
            w[k] = [np.ascontiguousarray(rng.normal(0.0, 0.5, size=n).astype(dtype)) for _ in range(shape.n_layers)]
    return w


def torch_weights_to_numpy(w):
    """Weights from workloads.make_weights (torch, CPU) -> numpy arrays the oracle reads
    (bf16 tensors become uint16 bit patterns)."""
    import torch

    def conv(t):
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).numpy().view(np.uint16)
        return t.numpy()

    out = {}
    for k, v in w.items():
        if isinstance(v, list):
            out[k] = [conv(t) for t in v]
        elif hasattr(v, "dtype") and hasattr(v, "detach"):
            out[k] = conv(v)
    return out
