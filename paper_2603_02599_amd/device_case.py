"""Device-side plumbing shared by bench.py and the GPU tests: one synthetic workload resident on the GPU (pool,
weights, inputs, workspace) with handles created through the C ABI.  No arithmetic of the method lives here
and nothing here touches the CPU oracle; the tests add the oracle mirrors on top (tests/gpu_harness.py)."""
from __future__ import annotations

import sys
from typing import Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as sun
from . import workloads as wl

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


def layout_strides(lay) -> Dict[str, int]:
    keys = ["k_off", "k_layer", "k_page", "k_head", "k_token", "k_dim",
            "v_off", "v_layer", "v_page", "v_head", "v_token", "v_dim"]
    return {k: int(getattr(lay, k)) for k in keys}


class DeviceWeights:
    """Decode weights on the GPU (dense, and optionally their 4-bit quantisation) with the library
    handle; shared by several workloads of the same shape."""

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


class DeviceCase:
    """One workload resident on the GPU with handles created through the C ABI."""

    def __init__(self, work: wl.Workload, weights: Optional[Dict[str, object]] = None, quant_mode: Optional[str] = None,
                 pool_seed: Optional[int] = None, weights_seed: Optional[int] = None,
                 shared: Optional[DeviceWeights] = None):
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

    def pool_pages_now(self, used: np.ndarray) -> np.ndarray:
        lay = self.lay
        view = self.pool_mem.view(self.work.shape.n_layers, int(lay.n_pages), int(lay.k_page))
        idx = torch.from_numpy(used.astype(np.int64)).to(DEV)
        return to_np(view.index_select(1, idx).contiguous()).reshape(-1)
