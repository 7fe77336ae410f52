"""Seeded synthetic inputs for the shared-decode step.

This module only *draws* inputs (shapes, token ids, context lengths,
source-model ids, page tables, random weights and random KV contents).
It holds none of the decode step's arithmetic and is the one module that
both the CPU oracle's tests and the HIP path's tests/bench may import.

Traffic structure follows the paper's serving experiments: several
task-specific source models feed one shared decode batch, and per-model
load follows the Zipf split of Appendix A.2 ("Skewed workloads"):
P(i) = i^-a / sum_j j^-a over popularity rank i.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np
import torch

PAGE_TOKENS = 16
SEED_BASE = 0x5EED0000


@dataclasses.dataclass(frozen=True)
class Shape:
    """Architectural constants of one decoder (Llama-style block)."""
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    qk_norm: bool = False              # Qwen3-class option: RMSNorm over head_dim on q and k heads
    qkv_bias: bool = False             # Qwen2-class option: bias vectors on the q, k and v projections
    rope_scaling: Optional[tuple] = None  # LLaMA-3.1-class option: (factor, low_freq, high_freq, original_max_position)

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def body_params(self) -> int:
        h, f = self.hidden, self.ffn
        per_layer = h * (self.q_dim + 2 * self.kv_dim) + self.q_dim * h + 3 * h * f
        return self.n_layers * per_layer

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.kv_dim * 2


TINY = Shape("tiny", 2, 256, 4, 2, 64, 688, 1024)
# Tiny shape whose FFN width is a multiple of the 128-wide quantisation group.
TINY_Q = Shape("tiny_q", 2, 256, 4, 2, 64, 768, 1024)
# The tiny and small shapes with the backbone options of the paper's model families switched on.
TINY_BIAS = Shape("tiny_bias", 2, 256, 4, 2, 64, 768, 1024, qkv_bias=True)
SMALL_BIAS = Shape("small_bias", 2, 512, 8, 2, 128, 1024, 2048, qkv_bias=True)
TINY_QWEN = Shape("tiny_qwen", 2, 256, 4, 2, 64, 768, 1024, rms_eps=1e-6, rope_base=1000000.0, qk_norm=True)
SMALL_LLAMA31 = Shape("small_llama31", 2, 512, 8, 2, 128, 1024, 2048, rope_base=500000.0,
                      rope_scaling=(8.0, 1.0, 4.0, 256))
# A second small shape with head_dim 128 and GQA ratio 4 (the 8B head geometry).
SMALL128 = Shape("small128", 2, 512, 8, 2, 128, 1024, 2048)
# Small shape with the 14B head geometry (GQA ratio 5, head_dim 128).
SMALL_G5 = Shape("small_g5", 2, 1280, 10, 2, 128, 1024, 2048)
LLAMA_8B = Shape("llama8b", 32, 4096, 32, 8, 128, 14336, 128256)
QWEN_14B = Shape("qwen14b", 48, 5120, 40, 8, 128, 13824, 152064)

CFG5A_PAGES = 65600          # pool pages of the aliased 14B workload (206 GB at 196 608 B per cached token)
CFG5B_POOL_BYTES = 200e9     # pool budget of the unaliased 14B workload

SHAPES = {s.name: s for s in (TINY, TINY_Q, TINY_QWEN, SMALL128, SMALL_LLAMA31, SMALL_G5, LLAMA_8B, QWEN_14B)}


def zipf_probs(n_models: int, s: float) -> np.ndarray:
    """Zipf popularity split over ranks 1..n_models (Appendix A.2)."""
    ranks = np.arange(1, n_models + 1, dtype=np.float64)
    w = ranks ** (-float(s))
    return w / w.sum()


def draw_model_ids(batch: int, n_models: int, kind: str, rng: np.random.Generator,
                   s: float = 1.2) -> np.ndarray:
    """Source-model tag of every request.

    kind = "even":    batch split evenly over the ids, order shuffled.
    kind = "present": uniform draw, re-drawn until every id appears.
    kind = "zipf":    i.i.d. draws from zipf_probs(n_models, s).
    """
    if kind == "even":
        ids = np.arange(batch) % n_models
        rng.shuffle(ids)
    elif kind == "present":
        while True:
            ids = rng.integers(0, n_models, size=batch)
            if batch < n_models or len(np.unique(ids)) == n_models:
                break
    elif kind == "zipf":
        ids = rng.choice(n_models, size=batch, p=zipf_probs(n_models, s))
    else:
        raise ValueError(kind)
    return ids.astype(np.int32)


def draw_lengths(batch: int, kind: str, rng: np.random.Generator, lo: int, hi: int,
                 median: float = 1024.0, sigma: float = 1.0) -> np.ndarray:
    """Cached tokens per request *before* the step (L_i).

    kind = "uniform":   integers uniform in [lo, hi].
    kind = "lognormal": clip(round(exp(ln median + sigma z)), lo, hi); if the
                        draw has no request above hi/2 the largest is set to hi,
                        so that one long-tail request is always present.
    """
    if kind == "uniform":
        L = rng.integers(lo, hi + 1, size=batch)
    elif kind == "lognormal":
        z = rng.standard_normal(batch)
        L = np.clip(np.rint(np.exp(math.log(median) + sigma * z)), lo, hi).astype(np.int64)
        if L.max() < hi // 2:
            L[int(np.argmax(L))] = hi
    else:
        raise ValueError(kind)
    return L.astype(np.int32)


def pages_needed(lengths: np.ndarray, page_tokens: int = PAGE_TOKENS) -> np.ndarray:
    """Pages a request must own so that slot L_i (the one this step writes) exists."""
    return (lengths.astype(np.int64) + 1 + page_tokens - 1) // page_tokens


def deal_page_tables(lengths: np.ndarray, rng: np.random.Generator,
                     page_tokens: int = PAGE_TOKENS, spare_frac: float = 0.25,
                     n_pages: Optional[int] = None, max_pages: Optional[int] = None):
    """Shuffled page tables over one pool shared by all source models.

    Physical pages are a random permutation dealt to requests in order; unused
    table entries are -1.  If `n_pages` is given and smaller than the demand,
    each request's tail page (the one written this step) stays unique and its
    history pages are drawn with replacement from the remaining pages
    (read-only aliasing, used only to emulate a pool larger than memory).
    Returns (tables int32 [B, max_pages], n_pages).
    """
    need = pages_needed(lengths, page_tokens)
    total = int(need.sum())
    B = len(lengths)
    if max_pages is None:
        max_pages = int(need.max())
    tables = np.full((B, max_pages), -1, dtype=np.int32)
    if n_pages is None or n_pages >= total:
        if n_pages is None:
            n_pages = total + int(math.ceil(spare_frac * total))
        perm = rng.permutation(n_pages)[:total]
        o = 0
        for i in range(B):
            tables[i, :need[i]] = perm[o:o + need[i]]
            o += int(need[i])
    else:
        if n_pages < 2 * B:
            raise ValueError("pool too small for unique tail pages")
        perm = rng.permutation(n_pages)
        tails, shared = perm[:B], perm[B:]
        for i in range(B):
            hist = int(need[i]) - 1
            tables[i, :hist] = rng.choice(shared, size=hist, replace=True)
            tables[i, hist] = tails[i]
    return tables, int(n_pages)


def draw_tokens(batch: int, vocab: int, rng: np.random.Generator) -> np.ndarray:
    return rng.integers(0, vocab, size=batch).astype(np.int32)


def _torch_dtype(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64}[dtype]


def make_weights(shape: Shape, dtype: str, device: str, seed: int,
                 std: float = 0.02, layers: Optional[int] = None) -> Dict[str, object]:
    """Random decoder weights: every matrix and the embedding ~ N(0, std^2),
    rounded to `dtype`; RMSNorm gains ~ 1 + N(0, 0.1^2) (centred on 1 so that the
    activations keep their scale through the depth, spread so that a dropped,
    swapped or mis-indexed gain shows in the logits).  Matrices are row-major
    [out_features, in_features].  Returns a dict with per-layer lists."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    dt = _torch_dtype(dtype)
    nl = shape.n_layers if layers is None else layers

    def mat(rows, cols):
        w = torch.empty((rows, cols), dtype=torch.float32 if dtype == "f64" else dt, device=device)
        w.normal_(0.0, std, generator=g)
        return w.to(dt)

    def gain(n):
        v = torch.empty(n, dtype=torch.float32, device=device).normal_(1.0, 0.1, generator=g)
        return v.to(dt)

    w: Dict[str, object] = {"dtype": dtype, "shape": shape}
    w["embed"] = mat(shape.vocab, shape.hidden)
    for k in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd"):
        w[k] = []
    for _ in range(nl):
        w["g1"].append(gain(shape.hidden))
        w["wq"].append(mat(shape.q_dim, shape.hidden))
        w["wk"].append(mat(shape.kv_dim, shape.hidden))
        w["wv"].append(mat(shape.kv_dim, shape.hidden))
        w["wo"].append(mat(shape.hidden, shape.q_dim))
        w["g2"].append(gain(shape.hidden))
        w["wg"].append(mat(shape.ffn, shape.hidden))
        w["wu"].append(mat(shape.ffn, shape.hidden))
        w["wd"].append(mat(shape.hidden, shape.ffn))
    w["gf"] = gain(shape.hidden)
    w["wlm"] = mat(shape.vocab, shape.hidden)
    if shape.qk_norm:  # head-norm gains: 1 + N(0, 0.1^2), so that a dropped or swapped gain shows
        w["qn"] = [gain(shape.head_dim) for _ in range(nl)]
        w["kn"] = [gain(shape.head_dim) for _ in range(nl)]
    if shape.qkv_bias:  # N(0, 0.5^2): large enough that a dropped or misplaced bias shows in the logits
        def bias(n):
            return torch.empty(n, dtype=torch.float32, device=device).normal_(0.0, 0.5, generator=g).to(dt)
        w["bq"] = [bias(shape.q_dim) for _ in range(nl)]
        w["bk"] = [bias(shape.kv_dim) for _ in range(nl)]
        w["bv"] = [bias(shape.kv_dim) for _ in range(nl)]
    return w


def fill_kv_pool(pool: torch.Tensor, seed: int, chunk_elems: int = 1 << 28) -> None:
    """Fill a bf16 pool buffer (any layout) in place with N(0,1) values."""
    g = torch.Generator(device=pool.device)
    g.manual_seed(seed)
    flat = pool.view(-1)
    for o in range(0, flat.numel(), chunk_elems):
        flat[o:o + chunk_elems].normal_(0.0, 1.0, generator=g)


@dataclasses.dataclass
class Workload:
    """One synthetic mixed-model decode batch (host-side description)."""
    name: str
    shape: Shape
    dtype: str                 # "f32" | "bf16"
    batch: int
    n_models: int
    tokens: np.ndarray         # int32 [B]
    model_ids: np.ndarray      # int32 [B]
    seq_lens: np.ndarray       # int32 [B]   L_i, cached tokens before the step
    page_tables: np.ndarray    # int32 [B, max_pages]
    n_pages: int
    seed: int
    aliased: bool = False

    @property
    def max_pages(self) -> int:
        return int(self.page_tables.shape[1])

    @property
    def kv_tokens_read(self) -> int:
        return int((self.seq_lens.astype(np.int64) + 1).sum())


def make_workload(name: str, **over) -> Workload:
    """The benchmark/parity configurations.

    cfg1: tiny fp32, 8 requests, 3 source models, L ~ U[16,128].
    cfg2: 8B bf16, 64 requests even over 4 models, L ~ U[512,4096].
    cfg3: 8B bf16, 256 requests Zipf(1.2) over 8 models, log-normal lengths
          (median 1024, sigma 1, clipped to [64,16384]).
    cfg5: 14B bf16, 128 requests Zipf(1.2) over 16 models, L ~ U[2048,32768]; the
          caches of that draw would take 438 GB, so it comes in two forms that fit:
          cfg5a: all 128 requests over a pool of 65 600 pages (206 GB; more than
                 2^31 elements per layer): every request's tail page is its own,
                 its history pages are drawn with replacement from the rest of the
                 pool (read-only aliasing: the bytes read and the addresses are those
                 of the full batch, the memory is not);
          cfg5b: the first requests of the same draw whose pages fit 200 GB, no
                 aliasing (52 requests).
    Any field can be overridden (e.g. shape=SMALL128, batch=..., lo/hi=...).
    """
    if name == "cfg5a":
        over.setdefault("n_pages", CFG5A_PAGES)
        w = make_workload("cfg5", **over)
        w.name = "cfg5a"
        return w
    if name == "cfg5b":
        full = make_workload("cfg5", **{**over, "n_pages": 1 << 20})   # the whole draw (its own tables are not used)
        kv_tok = full.shape.kv_bytes_per_token()
        keep, tot = 0, 0
        for L in full.seq_lens:
            pages = int(pages_needed(np.array([L]))[0])
            if (tot + pages) * PAGE_TOKENS * kv_tok > CFG5B_POOL_BYTES:
                break
            tot += pages
            keep += 1
        n_pages = int(over.get("n_pages", CFG5B_POOL_BYTES // (PAGE_TOKENS * kv_tok)))   # the budget, whole pages
        L = full.seq_lens[:keep].copy()
        tables, n_pages = deal_page_tables(L, np.random.default_rng(full.seed + 1000), n_pages=n_pages)
        return Workload(name="cfg5b", shape=full.shape, dtype=full.dtype, batch=keep, n_models=full.n_models,
                        tokens=full.tokens[:keep].copy(), model_ids=full.model_ids[:keep].copy(), seq_lens=L,
                        page_tables=tables, n_pages=n_pages, seed=full.seed, aliased=False)
    presets = {
        "cfg1": dict(num=1, shape=TINY, dtype="f32", batch=8, n_models=3, ids="present",
                     lens="uniform", lo=16, hi=128),
        "cfg2": dict(num=2, shape=LLAMA_8B, dtype="bf16", batch=64, n_models=4, ids="even",
                     lens="uniform", lo=512, hi=4096),
        "cfg3": dict(num=3, shape=LLAMA_8B, dtype="bf16", batch=256, n_models=8, ids="zipf",
                     lens="lognormal", lo=64, hi=16384),
        "cfg5": dict(num=5, shape=QWEN_14B, dtype="bf16", batch=128, n_models=16, ids="zipf",
                     lens="uniform", lo=2048, hi=32768),
    }
    p = dict(presets[name])
    p.update(over)
    seed = int(p.get("seed", SEED_BASE + p["num"]))
    rng = np.random.default_rng(seed)
    shape: Shape = p["shape"]
    B = int(p["batch"])
    ids = draw_model_ids(B, p["n_models"], p["ids"], rng)
    L = draw_lengths(B, p["lens"], rng, p["lo"], p["hi"])
    tables, n_pages = deal_page_tables(L, rng, n_pages=p.get("n_pages"),
                                       max_pages=p.get("max_pages"))
    need = int(pages_needed(L).sum())
    toks = draw_tokens(B, shape.vocab, rng)
    return Workload(name=name, shape=shape, dtype=p["dtype"], batch=B, n_models=p["n_models"],
                    tokens=toks, model_ids=ids, seq_lens=L, page_tables=tables,
                    n_pages=n_pages, seed=seed, aliased=n_pages < need)
