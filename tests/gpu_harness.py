"""Test-side plumbing for GPU parity: builds one workload on the GPU, mirrors exactly the
bytes the GPU consumes into the CPU oracle, and compares.  The oracle is imported on first use only, so that
bench.py can share the case-building code without touching it outside its cpu_baseline leg."""
from __future__ import annotations

import sys
from typing import Dict, Optional, Sequence

import numpy as np
import torch

from paper_2603_02599_amd import binding as sun
from paper_2603_02599_amd import workloads as wl


def _orc():
    """The CPU oracle, imported on first use: building GPU cases (which bench.py also does) does not touch it."""
    from oracle import oracle as o
    return o


def __getattr__(name):  # H.orc for the tests
    if name == "orc":
        return _orc()
    raise AttributeError(name)


DEV = "cuda:0"


def say(msg: str):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def to_np(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def weights_to_np(w: Dict[str, object]) -> Dict[str, object]:
    out = {}
    for k, v in w.items():
        if isinstance(v, list):
            out[k] = [to_np(t) for t in v]
        elif isinstance(v, torch.Tensor):
            out[k] = to_np(v)
    return out


def oracle_triple(trip):
    """(codes, scales, zero points) as the oracle takes them; where the GPU side stores no zero points (the
    symmetric layout) the oracle gets the definition written out: 8.0 for every group."""
    q, s, z = trip
    sn = to_np(s)
    return to_np(q), sn, (to_np(z) if z is not None else np.full(sn.shape, 0x4800, np.uint16))


def layout_strides(lay) -> Dict[str, int]:
    keys = ["k_off", "k_layer", "k_page", "k_head", "k_token", "k_dim",
            "v_off", "v_layer", "v_page", "v_head", "v_token", "v_dim"]
    return {k: int(getattr(lay, k)) for k in keys}


class SharedWeights:
    """Decode weights on the GPU (dense, and optionally their 4-bit quantisation) with the library
    handle and a lazily built oracle mirror; shared by several workloads of the same shape."""

    def __init__(self, shape, dtype: str, seed: int, quant_mode: Optional[str] = None):
        self.shape, self.dtype = shape, dtype
        self.cfg = sun.make_cfg(shape, dtype)
        self.w = wl.make_weights(shape, dtype, DEV, seed)
        self.quant = None
        if quant_mode is None:
            self.handle = sun.sun_weights_create(self.cfg, self.w)
        else:
            self.quant = {k: [sun.sun_quantize_w4(m, 128, quant_mode) for m in self.w[k]] for k in sun.QUANT_KEYS}
            self.handle = sun.sun_qweights_create(self.cfg, self.w, self.quant)
        torch.cuda.synchronize()
        self._params = None

    def oracle_params(self):
        if self._params is None:
            wnp = weights_to_np(self.w)
            qnp = None
            if self.quant is not None:
                qnp = {k: [oracle_triple(trip) for trip in v] for k, v in self.quant.items()}
                for k, v in qnp.items():   # dense sources may have been released: only their width is needed
                    if k not in wnp:
                        wnp[k] = [np.empty((0, 2 * trip[0].shape[1]), np.float32) for trip in v]
            self._keep = (wnp, qnp)
            self._params = _orc().params_from_arrays(wnp, qnp)
        return self._params


class GpuCase:
    """One workload resident on the GPU with handles created through the C ABI."""

    def __init__(self, work: wl.Workload, weights: Optional[Dict[str, object]] = None, quant_mode: Optional[str] = None,
                 pool_seed: Optional[int] = None, weights_seed: Optional[int] = None,
                 shared: Optional[SharedWeights] = None):
        self.work = work
        shape = work.shape
        self.cfg = sun.make_cfg(shape, work.dtype)
        self.shared = shared
        if shared is not None:
            self.w = shared.w
        else:
            self.w = weights if weights is not None else wl.make_weights(shape, work.dtype, DEV, weights_seed or work.seed + 1)
        nbytes = sun.sun_kv_pool_bytes(self.cfg, work.n_pages)
        self.pool_mem = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=DEV)
        wl.fill_kv_pool(self.pool_mem, pool_seed or work.seed + 2)
        self.pool = sun.sun_kv_pool_create(self.cfg, self.pool_mem, 16, work.n_models)
        self.lay = self.pool.layout()
        assert self.lay.n_pages == work.n_pages
        self.quant = None
        if shared is not None:
            self.quant, self.weights = shared.quant, shared.handle
        elif quant_mode is None:
            self.weights = sun.sun_weights_create(self.cfg, self.w)
        else:
            self.quant = {k: [sun.sun_quantize_w4(m, 128, quant_mode) for m in self.w[k]] for k in sun.QUANT_KEYS}
            self.weights = sun.sun_qweights_create(self.cfg, self.w, self.quant)
        self.tokens = torch.from_numpy(work.tokens).to(DEV)
        self.tables = torch.from_numpy(work.page_tables).to(DEV)
        self.lens = torch.from_numpy(work.seq_lens).to(DEV)
        self.ids = torch.from_numpy(work.model_ids).to(DEV)
        self.ws = torch.empty(sun.sun_workspace_bytes(self.cfg, work.batch, work.max_pages), dtype=torch.uint8, device=DEV)
        self.logits = torch.empty((work.batch, shape.vocab), dtype=torch.float32, device=DEV)
        self.next = torch.empty(work.batch, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()

    def step(self, flags: int = 0, host_lens: bool = True, tokens=None, tables=None, lens=None, ids=None,
             logits=None, nxt=None):
        fn = sun.sun_qdecode_step if self.quant is not None else sun.sun_decode_step
        lens_t = self.lens if lens is None else lens
        fn(self.pool, self.weights, self.tokens if tokens is None else tokens,
           self.tables if tables is None else tables, lens_t, self.ids if ids is None else ids,
           self.logits if logits is None else logits, self.next if nxt is None else nxt, self.ws,
           seq_lens_host=(lens_t.cpu().numpy() if host_lens else None), flags=flags)
        torch.cuda.synchronize()

    # ---- oracle mirror ----
    def oracle_params(self):
        if self.shared is not None:
            return self.shared.oracle_params()
        wnp = weights_to_np(self.w)
        qnp = None
        if self.quant is not None:
            qnp = {k: [oracle_triple(trip) for trip in v] for k, v in self.quant.items()}
        self._keep = (wnp, qnp)
        return _orc().params_from_arrays(wnp, qnp)

    def extract_pool(self, rows: Sequence[int]):
        """Copies only the pages the given requests reference into a compact host pool with
        the same in-page layout; returns (host uint16 array, oracle pool, remapped tables)."""
        work, lay = self.work, self.lay
        tabs = work.page_tables[list(rows)]
        used = np.unique(tabs[tabs >= 0])
        remap = {int(p): i for i, p in enumerate(used)}
        new_tabs = np.vectorize(lambda p: remap.get(int(p), -1))(tabs).astype(np.int32)
        page_elems = int(lay.k_page)
        nl = work.shape.n_layers
        view = self.pool_mem.view(nl, int(lay.n_pages), page_elems)
        idx = torch.from_numpy(used.astype(np.int64)).to(DEV)
        small = view.index_select(1, idx).contiguous()
        host = to_np(small).reshape(-1).copy()
        st = layout_strides(lay)
        st["k_layer"] = st["v_layer"] = len(used) * page_elems
        pool = _orc().make_pool(host, len(used), 16, st)
        return host, pool, new_tabs, used

    def pool_pages_now(self, used: np.ndarray) -> np.ndarray:
        lay = self.lay
        view = self.pool_mem.view(self.work.shape.n_layers, int(lay.n_pages), int(lay.k_page))
        idx = torch.from_numpy(used.astype(np.int64)).to(DEV)
        return to_np(view.index_select(1, idx).contiguous()).reshape(-1)


def run_oracle(case: GpuCase, rows: Sequence[int], params=None, tokens=None, lens=None, ids=None, **kw):
    """Oracle step on the sampled requests, from the pool state *before* the GPU step
    (call this before case.step())."""
    work = case.work
    rows = list(rows)
    host, pool, tabs, used = case.extract_pool(rows)
    params = params if params is not None else case.oracle_params()
    ocfg = _orc().make_cfg(work.shape)
    toks = (work.tokens if tokens is None else tokens)[rows]
    ln = (work.seq_lens if lens is None else lens)[rows]
    mi = (work.model_ids if ids is None else ids)[rows]
    res = _orc().decode_step(ocfg, params, pool, toks, tabs, ln, mi, **kw)
    res["pool_after"] = host
    res["used_pages"] = used
    return res


def logits_report(got: np.ndarray, want: np.ndarray) -> Dict[str, float]:
    diff = np.abs(got.astype(np.float64) - want)
    return {"max_abs": float(diff.max()), "max_rel_excess": float((diff - 1e-2 * np.abs(want)).max()),
            "ref_std": float(want.std())}


def check_logits(got: np.ndarray, want: np.ndarray, dtype: str):
    """fp32: max-abs <= 1e-4.  bf16: |g - o| <= 2e-2 + 1e-2 |o| for every element."""
    diff = np.abs(got.astype(np.float64) - want)
    if dtype == "f32":
        assert diff.max() <= 1e-4, f"fp32 logits differ by {diff.max():.3e}"
    else:
        bound = 2e-2 + 1e-2 * np.abs(want)
        worst = float((diff - bound).max())
        assert worst <= 0, f"bf16 logits exceed 2e-2 + 1e-2|o| by {worst:.3e} (max abs {diff.max():.3e})"


def check_next_tokens(got: np.ndarray, want_logits: np.ndarray, tol: float):
    """Bit-exact unless the oracle's top two logits are closer than 2*tol (documented near-tie),
    in which case either of the two is accepted; returns the list of near-tie rows."""
    near = []
    for i in range(len(got)):
        order = np.argsort(-want_logits[i], kind="stable")
        top, second = int(order[0]), int(order[1])
        if int(got[i]) == top:
            continue
        gap = want_logits[i, top] - want_logits[i, second]
        assert gap < 2 * tol and int(got[i]) == second, \
            f"row {i}: gpu token {int(got[i])}, oracle {top} (gap to runner-up {gap:.3e})"
        near.append(i)
    return near


def appended_mask(shape, strides: Dict[str, int], n_elems: int, tabs: np.ndarray, lens: np.ndarray) -> np.ndarray:
    """Boolean mask over a (compact) pool: the elements Eq. 4 says this step writes."""
    m = np.zeros(n_elems, dtype=bool)
    d = shape.head_dim
    for i, L in enumerate(lens):
        page, slot = int(tabs[i, int(L) // 16]), int(L) % 16
        for l in range(shape.n_layers):
            for h in range(shape.n_kv_heads):
                for kv in ("k", "v"):
                    o = (strides[kv + "_off"] + l * strides[kv + "_layer"] + page * strides[kv + "_page"] +
                         h * strides[kv + "_head"] + slot * strides[kv + "_token"])
                    m[o + np.arange(d) * strides[kv + "_dim"]] = True
    return m


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def check_appended_kv(gpu_after: np.ndarray, orc_after: np.ndarray, before: np.ndarray, mask: np.ndarray, dtype: str,
                      abs_tol: float = 2e-6):
    """Eq. 4: only the predicted slots change.  fp32 path: values equal the oracle's bf16
    rounding up to 1 bf16 ulp (an fp32 and an fp64 projection can round apart), or, for an element
    that cancels to nearly zero, where one bf16 ulp is smaller than the fp32 accumulation error of
    the projection that produced it, up to abs_tol absolute (2e-6 for one step over a given cache);
    bf16 path: within the logits tolerance.
    Returns (#elements off by one ulp or more, #elements written)."""
    assert np.array_equal(gpu_after[~mask], before[~mask]), "GPU wrote outside the appended slots"
    assert np.array_equal(orc_after[~mask], before[~mask])
    a, b = gpu_after[mask].astype(np.int32), orc_after[mask].astype(np.int32)

    def ordered(u):  # monotone integer code of a bf16 bit pattern
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)

    ulp = np.abs(ordered(a) - ordered(b))
    ga, oa = bf16_to_f64(gpu_after[mask]), bf16_to_f64(orc_after[mask])
    if dtype == "f32":
        bad = (ulp > 1) & (np.abs(ga - oa) > abs_tol)
        assert not bad.any(), f"appended K/V differs by {ulp[bad].max()} bf16 ulps ({np.abs(ga - oa)[bad].max():.2e})"
    else:
        worst = float((np.abs(ga - oa) - (2e-2 + 1e-2 * np.abs(oa))).max())
        assert worst <= 0, f"appended K/V exceeds the bf16 tolerance by {worst:.3e}"
    return int((ulp >= 1).sum()), int(mask.sum())
