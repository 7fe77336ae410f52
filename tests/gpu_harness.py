"""Test-side plumbing for GPU parity: on top of the package's device-side case (pool, weights, inputs on the
GPU) it mirrors exactly the bytes the GPU consumes into the CPU oracle, and compares.  The oracle is imported on
first use only."""
from __future__ import annotations

import sys
from typing import Dict, Optional, Sequence

import numpy as np
import torch

from paper_2603_02599_amd import binding as sun
from paper_2603_02599_amd import workloads as wl
from paper_2603_02599_amd.device_case import DEV, DeviceCase, DeviceWeights, layout_strides, say, to_np, weights_to_np  # noqa: F401


def _orc():
    """The CPU oracle, imported on first use: building GPU cases (which bench.py also does) does not touch it."""
    from oracle import oracle as o
    return o


def __getattr__(name):  # H.orc for the tests
    if name == "orc":
        return _orc()
    raise AttributeError(name)


def oracle_triple(trip):
    """(codes, scales, zero points) as the oracle takes them; where the GPU side stores no zero points (the
    symmetric layout) the oracle gets the definition written out: 8.0 for every group."""
    q, s, z = trip
    sn = to_np(s)
    return to_np(q), sn, (to_np(z) if z is not None else np.full(sn.shape, 0x4800, np.uint16))


def weights_oracle_params(sw: DeviceWeights):
    """Oracle mirror of shared device weights, built once per object."""
    if getattr(sw, "_params", None) is None:
        wnp = weights_to_np(sw.w)
        qnp = None
        if sw.quant is not None:
            qnp = {k: [oracle_triple(trip) for trip in v] for k, v in sw.quant.items()}
            for k, v in qnp.items():   # dense sources may have been released: only their width is needed
                if k not in wnp:
                    wnp[k] = [np.empty((0, 2 * trip[0].shape[1]), np.float32) for trip in v]
        sw._keep = (wnp, qnp)
        sw._params = _orc().params_from_arrays(wnp, qnp)
    return sw._params


def case_oracle_params(case: DeviceCase):
    if case.shared is not None:
        return weights_oracle_params(case.shared)
    wnp = weights_to_np(case.w)
    qnp = None
    if case.quant is not None:
        qnp = {k: [oracle_triple(trip) for trip in v] for k, v in case.quant.items()}
    case._keep = (wnp, qnp)
    return _orc().params_from_arrays(wnp, qnp)


def case_extract_pool(case: DeviceCase, rows: Sequence[int]):
    """Copies only the pages the given requests reference into a compact host pool with
    the same in-page layout; returns (host uint16 array, oracle pool, remapped tables, page ids)."""
    work, lay = case.work, case.lay
    tabs = work.page_tables[list(rows)]
    used = np.unique(tabs[tabs >= 0])
    remap = {int(p): i for i, p in enumerate(used)}
    new_tabs = np.vectorize(lambda p: remap.get(int(p), -1))(tabs).astype(np.int32)
    page_elems = int(lay.k_page)
    nl = work.shape.n_layers
    view = case.pool_mem.view(nl, int(lay.n_pages), page_elems)
    idx = torch.from_numpy(used.astype(np.int64)).to(DEV)
    small = view.index_select(1, idx).contiguous()
    host = to_np(small).reshape(-1).copy()
    st = layout_strides(lay)
    st["k_layer"] = st["v_layer"] = len(used) * page_elems
    pool = _orc().make_pool(host, len(used), 16, st)
    return host, pool, new_tabs, used


class SharedWeights(DeviceWeights):
    """Decode weights on the GPU with a lazily built oracle mirror."""

    def oracle_params(self):
        return weights_oracle_params(self)


class GpuCase(DeviceCase):
    """One workload resident on the GPU, with the oracle mirrors the parity tests need."""

    def oracle_params(self):
        return case_oracle_params(self)

    def extract_pool(self, rows: Sequence[int]):
        return case_extract_pool(self, rows)


def run_oracle(case: DeviceCase, rows: Sequence[int], params=None, tokens=None, lens=None, ids=None, **kw):
    """Oracle step on the sampled requests, from the pool state *before* the GPU step
    (call this before case.step())."""
    work = case.work
    rows = list(rows)
    host, pool, tabs, used = case_extract_pool(case, rows)
    params = params if params is not None else case_oracle_params(case)
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
                      abs_tol: float = None, max_off_frac: float = None, quant: bool = False):
    """Eq. 4: only the predicted slots change, and each stored value is the oracle's round-to-nearest-even
    bf16 value, or its neighbour: the projections that produce it differ from the oracle's fp64 ones by much
    less than a bf16 ulp, so the two roundings can fall apart by one ulp and no more.  An element that cancels
    to nearly zero is the exception (one bf16 ulp there is smaller than the error the path is allowed before the
    rounding); it is held to an absolute bound instead: 2e-6 for the fp32 path (its accumulation error); 2e-3
    for the bf16 path (a tenth of the logit tolerance: what reaches a deep layer's projection input through the
    layers before it; measured up to 1.1e-3 at 48 layers); 1e-2 + 5e-3|o| for the 4-bit path (half its logit
    tolerance: there the projection inputs are rounded to 16-bit fixed point per group, and the measured
    difference of a deep layer's entries reaches 8e-3, the same as its logits').  A store that does not round
    to nearest (truncation) would still be within one ulp everywhere but off by one in about half of the
    elements, so the fraction of elements that differ at all is bounded too (max_off_frac: 0.15, measured
    0.4 to 3.5 per cent at 2 to 48 layers and 0 to 3 elements on the fp32 path; 0.3 for the 4-bit path, measured
    up to 0.18 at 48 layers: the store is the same kernel on all three paths).
    Returns (#elements off by one ulp or more, #elements written)."""
    abs_tol = max(abs_tol or 0.0, 2e-6 if dtype == "f32" else 2e-3)   # a caller may widen the floor, not narrow it
    if max_off_frac is None:
        max_off_frac = 0.3 if quant else 0.15
    assert np.array_equal(gpu_after[~mask], before[~mask]), "GPU wrote outside the appended slots"
    assert np.array_equal(orc_after[~mask], before[~mask])
    a, b = gpu_after[mask].astype(np.int32), orc_after[mask].astype(np.int32)

    def ordered(u):  # monotone integer code of a bf16 bit pattern
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)

    ulp = np.abs(ordered(a) - ordered(b))
    ga, oa = bf16_to_f64(gpu_after[mask]), bf16_to_f64(orc_after[mask])
    bound = np.maximum(abs_tol, 1e-2 + 5e-3 * np.abs(oa)) if quant else abs_tol
    bad = (ulp > 1) & (np.abs(ga - oa) > bound)
    assert not bad.any(), (f"appended K/V differs by {ulp[bad].max()} bf16 ulps ({np.abs(ga - oa)[bad].max():.2e} absolute) "
                           f"in {int(bad.sum())} of {int(mask.sum())} elements")
    off = int((ulp >= 1).sum())
    assert off <= max_off_frac * max(int(mask.sum()), 1) + 3, \
        f"{off} of {int(mask.sum())} appended K/V elements differ from the oracle's rounding: not round-to-nearest?"
    return off, int(mask.sum())


def appended_kv_stats(gpu_after: np.ndarray, orc_after: np.ndarray, mask: np.ndarray) -> Dict[str, float]:
    """For the log: the largest difference (absolute, and in bf16 ulps) among the written elements."""
    a, b = gpu_after[mask].astype(np.int32), orc_after[mask].astype(np.int32)
    oa_, ob_ = np.where(a & 0x8000, -(a & 0x7FFF), a & 0x7FFF), np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    ulp = np.abs(oa_ - ob_)
    d = np.abs(bf16_to_f64(gpu_after[mask]) - bf16_to_f64(orc_after[mask]))
    multi = ulp > 1
    return {"max_ulp": int(ulp.max()) if ulp.size else 0, "n_multi_ulp": int(multi.sum()),
            "max_abs_where_multi_ulp": float(d[multi].max()) if multi.any() else 0.0,
            "off_frac": float((ulp >= 1).mean()) if ulp.size else 0.0}


def replay_steps_on_gpu_cache(case: DeviceCase, used: np.ndarray, after: np.ndarray, tabs: np.ndarray, lens0: np.ndarray,
                              tokens_per_step, ids: np.ndarray, quant: bool = False):
    """Several decode steps of the same requests, each compared on its own: step s of the oracle starts from the
    cache the GPU holds (`after`: the compact copy of the used pages after all steps; step s reads positions
    below lens0 + s only, which later steps do not touch), is fed the token the GPU was fed, computes position
    lens0 + s next to the GPU's entry for it (decode_step_peer: see oracle_step_next_to_gpu_cache) and returns
    its logits.  Each step is thereby held to the single-step bar.  tokens_per_step[s]: the tokens fed at
    step s.  Returns (list of per-step logits, summed peer counts)."""
    work = case.work
    st = layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    ocfg, params = _orc().make_cfg(work.shape), case_oracle_params(case)
    tol_abs, tol_rel, max_off = kv_bound(work.dtype, quant)
    peer = _orc().make_pool(after, len(used), 16, st)
    logits, tot = [], {"equal": 0, "neighbour": 0, "by_value": 0, "rejected": 0}
    for s, toks in enumerate(tokens_per_step):
        host = after.copy()
        pool = _orc().make_pool(host, len(used), 16, st)
        ln = (lens0 + s).astype(np.int32)
        res = _orc().decode_step_peer(ocfg, params, pool, peer, np.asarray(toks, np.int32), tabs, ln, ids, tol_abs, tol_rel)
        for k2, v in res["peer"].items():
            tot[k2] += v
        assert res["peer"]["rejected"] == 0, f"step {s}: {res['peer']}"
        assert np.array_equal(host, after), "the oracle stored something else than the GPU's accepted entries"
        logits.append(res["logits"])
    n = sum(tot.values())
    assert tot["neighbour"] + tot["by_value"] <= max_off * n + 3, f"{tot}: too many entries differ for a round-to-nearest store"
    return logits, tot


def kv_bound(dtype: str, quant: bool):
    """(tol_abs, tol_rel, max share of entries that may differ at all) of the appended-K/V comparison: see
    check_appended_kv."""
    if dtype == "f32":
        return 2e-6, 0.0, 0.15
    return (1e-2, 5e-3, 0.3) if quant else (2e-3, 0.0, 0.15)


def oracle_step_next_to_gpu_cache(case: DeviceCase, rows: Sequence[int], extracted, after: np.ndarray, tokens=None,
                                  lens=None, ids=None, quant: bool = False):
    """The oracle's step for the sampled requests, run after the GPU's from the cache as it was before
    (`extracted` = case_extract_pool(case, rows) taken before the GPU step), next to the GPU's cache after its
    step (`after`, the same pages): every new entry is computed and rounded by the oracle and compared with the
    GPU's; a GPU entry that is that rounding, its neighbour, or within the bound is what the oracle then attends
    over (a stored bf16 code is a rounding decision, and the fp32 path may legitimately take the other side of
    a boundary; carried through 32 to 48 layers such a flip would otherwise show up in everything compared
    after it, a request that puts much attention weight on its own new position being the worst case).  Asserts
    that no entry is rejected, that the share of entries that differ at all stays under the bound (a store
    that truncates instead of rounding would differ in half of them), and that nothing else in the cache
    moved.  Returns the oracle's result dict (logits, next, peer counts)."""
    work = case.work
    rows = list(rows)
    host, pool, tabs, used = extracted
    before = host.copy()
    st = layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    peer = _orc().make_pool(after, len(used), 16, st)
    toks = (work.tokens if tokens is None else tokens)[rows]
    ln = (work.seq_lens if lens is None else lens)[rows]
    mi = (work.model_ids if ids is None else ids)[rows]
    tol_abs, tol_rel, max_off = kv_bound(work.dtype, quant)
    res = _orc().decode_step_peer(_orc().make_cfg(work.shape), case_oracle_params(case), pool, peer, toks, tabs, ln, mi,
                                  tol_abs, tol_rel)
    cnt = res["peer"]
    total = sum(cnt.values())
    mask = appended_mask(work.shape, st, after.size, tabs, ln)
    assert total == int(mask.sum())
    assert np.array_equal(after[~mask], before[~mask]), "GPU wrote outside the appended slots"
    assert np.array_equal(host[~mask], before[~mask])
    assert cnt["rejected"] == 0, f"{cnt['rejected']} of {total} appended K/V entries are neither the oracle's rounding, its neighbour, nor within the bound"
    assert np.array_equal(host[mask], after[mask])
    assert cnt["neighbour"] + cnt["by_value"] <= max_off * total + 3, f"{cnt} of {total}: too many entries differ for a round-to-nearest store"
    return res
