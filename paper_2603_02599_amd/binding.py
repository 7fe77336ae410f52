"""Thin ctypes binding of libsun (argument marshalling only; every step of the decode path
runs in the HIP kernels).  Function names follow include/sun.h.  PyTorch tensors are used
as device-memory owners; their data_ptr() is what crosses the boundary.

There is no CPU fallback: if the HIP library is missing the import of a function fails."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SUN_LIB_PATH", os.path.join(_HERE, "libsun.so"))  # override: another build of libsun

SUN_F32, SUN_BF16 = 0, 1
SUN_VALIDATE, SUN_PROFILE, SUN_SERVE_RESET = 1, 2, 4
STATUS = {0: "SUN_OK", 1: "SUN_ERR_NULL", 2: "SUN_ERR_SHAPE", 3: "SUN_ERR_POOL_SIZE", 4: "SUN_ERR_WORKSPACE",
          5: "SUN_ERR_PAGE_RANGE", 6: "SUN_ERR_SEQ_LEN", 7: "SUN_ERR_MODEL_ID", 8: "SUN_ERR_HIP", 9: "SUN_ERR_TOKEN"}
PROFILE_KINDS = ("attn_split", "attn_combine", "qkv_proj", "o_proj", "gate_up_proj", "down_proj", "lm_head", "other")

EXPORTS = [
    "sun_kv_pool_bytes", "sun_kv_pool_create", "sun_kv_pool_layout", "sun_kv_pool_destroy",
    "sun_kv_pool_ingest", "sun_kv_pool_model_tokens",
    "sun_weights_pack_bytes", "sun_weights_create", "sun_weights_destroy",
    "sun_qweights_pack_bytes", "sun_qweights_create", "sun_quantize_w4",
    "sun_workspace_bytes", "sun_decode_step", "sun_qdecode_step", "sun_decode_run",
    "sun_prefill_workspace_bytes", "sun_prefill", "sun_serve_workspace_bytes", "sun_decode_serve",
    "sun_paged_attention", "sun_paged_attention_static", "sun_paged_attention_static_bytes",
    "sun_paged_attention_static_limit", "sun_linear",
    "sun_hbm_read_probe", "sun_profile_read", "sun_profile_reset", "sun_last_error", "sun_version",
]


class ServeState(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("token_ids", "page_tables", "seq_lens", "model_ids", "slot_req", "slot_left",
                                          "w_req", "w_token", "w_tables", "w_lens", "w_model", "w_budget", "ring",
                                          "counters")] + \
               [(n, C.c_int32) for n in ("n_wait", "ring_cap", "idle_page", "eos_id")]


class SunError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("act_dtype", C.c_int32), ("qk_norm", C.c_int32), ("rope_scaling", C.c_int32),
                ("rope_original_max_position", C.c_int32), ("rope_factor", C.c_float),
                ("rope_low_freq_factor", C.c_float), ("rope_high_freq_factor", C.c_float), ("qkv_bias", C.c_int32)]


class KvLayout(C.Structure):
    _fields_ = [("n_pages", C.c_int64), ("page_tokens", C.c_int32), ("reserved", C.c_int32),
                ("k_off", C.c_int64), ("k_layer", C.c_int64), ("k_page", C.c_int64), ("k_head", C.c_int64),
                ("k_token", C.c_int64), ("k_dim", C.c_int64),
                ("v_off", C.c_int64), ("v_layer", C.c_int64), ("v_page", C.c_int64), ("v_head", C.c_int64),
                ("v_token", C.c_int64), ("v_dim", C.c_int64), ("total_elems", C.c_int64)]


class WeightPtrs(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + [(k, C.POINTER(C.c_void_p)) for k in
                                          ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")] + \
               [("gf", C.c_void_p), ("wlm", C.c_void_p), ("q_norm", C.POINTER(C.c_void_p)), ("k_norm", C.POINTER(C.c_void_p)),
                ("bq", C.POINTER(C.c_void_p)), ("bk", C.POINTER(C.c_void_p)), ("bv", C.POINTER(C.c_void_p))]


class QMat(C.Structure):
    _fields_ = [("q", C.c_void_p), ("s", C.c_void_p), ("z", C.c_void_p)]


class QWeightPtrs(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("g1", C.POINTER(C.c_void_p)),
                ("wq", C.POINTER(QMat)), ("wk", C.POINTER(QMat)), ("wv", C.POINTER(QMat)), ("wo", C.POINTER(QMat)),
                ("g2", C.POINTER(C.c_void_p)),
                ("wg", C.POINTER(QMat)), ("wu", C.POINTER(QMat)), ("wd", C.POINTER(QMat)),
                ("gf", C.c_void_p), ("wlm", C.c_void_p),
                ("q_norm", C.POINTER(C.c_void_p)), ("k_norm", C.POINTER(C.c_void_p)),
                ("bq", C.POINTER(C.c_void_p)), ("bk", C.POINTER(C.c_void_p)), ("bv", C.POINTER(C.c_void_p))]


_lib = None


def lib() -> C.CDLL:
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_02599_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.sun_last_error.restype = C.c_char_p
        L.sun_version.restype = C.c_char_p
        for f in ("sun_kv_pool_bytes", "sun_weights_pack_bytes", "sun_qweights_pack_bytes", "sun_workspace_bytes",
                  "sun_prefill_workspace_bytes", "sun_serve_workspace_bytes", "sun_paged_attention_static_bytes",
                  "sun_paged_attention_static_limit"):
            getattr(L, f).restype = C.c_size_t
        L.sun_kv_pool_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int64, C.c_int]
        L.sun_kv_pool_create.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_size_t, C.c_int, C.c_int,
                                         C.POINTER(C.c_void_p)]
        L.sun_kv_pool_layout.argtypes = [C.c_void_p, C.POINTER(KvLayout)]
        L.sun_kv_pool_destroy.argtypes = [C.c_void_p]
        L.sun_kv_pool_destroy.restype = None
        L.sun_weights_pack_bytes.argtypes = [C.POINTER(ModelCfg)]
        L.sun_weights_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(WeightPtrs), C.c_void_p, C.c_size_t,
                                         C.c_void_p, C.POINTER(C.c_void_p)]
        L.sun_weights_destroy.argtypes = [C.c_void_p]
        L.sun_weights_destroy.restype = None
        L.sun_qweights_pack_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int]
        L.sun_qweights_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(QWeightPtrs), C.c_int, C.c_void_p,
                                          C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
        L.sun_quantize_w4.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.sun_kv_pool_ingest.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p,
                                         C.c_int, C.c_void_p, C.c_uint]
        L.sun_kv_pool_model_tokens.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int64)]
        L.sun_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int]
        step_args = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p,
                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint]
        L.sun_decode_step.argtypes = step_args
        L.sun_qdecode_step.argtypes = step_args
        L.sun_decode_run.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint]
        L.sun_serve_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int]
        L.sun_decode_serve.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(ServeState),
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint]
        L.sun_prefill_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int]
        L.sun_prefill.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                  C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint]
        L.sun_paged_attention.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.sun_paged_attention_static.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_int,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.sun_paged_attention_static_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int]
        L.sun_paged_attention_static_limit.argtypes = []
        L.sun_linear.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.c_size_t, C.c_void_p]
        L.sun_hbm_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.sun_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.sun_profile_reset.restype = None
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise SunError(rc, lib().sun_last_error().decode())


def _p(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        assert t.is_contiguous()
        return t.data_ptr()
    return int(t)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def make_cfg(shape, act_dtype: str) -> ModelCfg:
    """shape: object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, rms_eps, rope_base and
    optionally qk_norm (bool), qkv_bias (bool) and rope_scaling = (factor, low_freq_factor, high_freq_factor, original_max_position)."""
    rs = getattr(shape, "rope_scaling", None)
    return ModelCfg(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                    shape.vocab, float(shape.rms_eps), float(shape.rope_base),
                    {"f32": SUN_F32, "bf16": SUN_BF16}[act_dtype], int(bool(getattr(shape, "qk_norm", False))),
                    1 if rs else 0, int(rs[3]) if rs else 0, float(rs[0]) if rs else 0.0, float(rs[1]) if rs else 0.0,
                    float(rs[2]) if rs else 0.0, int(bool(getattr(shape, "qkv_bias", False))))


# ------------------------------------------------------------------ pool
def sun_kv_pool_bytes(cfg: ModelCfg, n_pages: int, page_tokens: int = 16) -> int:
    return int(lib().sun_kv_pool_bytes(C.byref(cfg), n_pages, page_tokens))


class KvPool:
    """Owner of the pool handle; `mem` (a torch uint8/bf16 CUDA tensor) is borrowed and kept alive."""

    def __init__(self, handle: int, mem: torch.Tensor):
        self.handle, self.mem = handle, mem

    def layout(self) -> KvLayout:
        return sun_kv_pool_layout(self)

    def __del__(self):
        # at interpreter shutdown the module globals may already be gone; the handle is host memory only
        if getattr(self, "handle", None) and _lib is not None:
            _lib.sun_kv_pool_destroy(self.handle)
            self.handle = None


def sun_kv_pool_create(cfg: ModelCfg, mem: torch.Tensor, page_tokens: int = 16, n_source_models: int = 1) -> KvPool:
    out = C.c_void_p()
    nbytes = mem.numel() * mem.element_size() if isinstance(mem, torch.Tensor) else 0
    _check(lib().sun_kv_pool_create(C.byref(cfg), _p(mem), nbytes, page_tokens, n_source_models, C.byref(out)))
    return KvPool(out.value, mem)


def sun_kv_pool_layout(pool: KvPool) -> KvLayout:
    lay = KvLayout()
    _check(lib().sun_kv_pool_layout(pool.handle, C.byref(lay)))
    return lay


# ------------------------------------------------------------------ weights
LAYER_KEYS = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")
QUANT_KEYS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")


class Weights:
    def __init__(self, handle: int, keep: list, quant: bool):
        self.handle, self.keep, self.quant = handle, keep, quant

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.sun_weights_destroy(self.handle)
            self.handle = None


def _ptr_array(tensors: Sequence[torch.Tensor]):
    arr = (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    return arr


def _set_head_norms(ptrs, w, cfg: ModelCfg, keep: List[object]):
    """Per-layer vectors of the backbone options: head-norm gains (w["qn"], w["kn"]) and projection biases
    (w["bq"], w["bk"], w["bv"])."""
    fields = ((("q_norm", "qn"), ("k_norm", "kn")) if cfg.qk_norm else ()) + \
             ((("bq", "bq"), ("bk", "bk"), ("bv", "bv")) if cfg.qkv_bias else ())
    for field, key in fields:
        arr = _ptr_array(w[key])
        keep.extend([arr, w[key]])
        setattr(ptrs, field, C.cast(arr, C.POINTER(C.c_void_p)))


def sun_weights_pack_bytes(cfg: ModelCfg) -> int:
    return int(lib().sun_weights_pack_bytes(C.byref(cfg)))


def sun_weights_create(cfg: ModelCfg, w: Dict[str, object], stream=None, keep_sources: bool = True) -> Weights:
    """w: dict from workloads.make_weights (torch CUDA tensors).  Allocates the pack buffer with torch."""
    ptrs = WeightPtrs()
    keep: List[object] = []
    ptrs.embed = w["embed"].data_ptr()
    for k in LAYER_KEYS:
        arr = _ptr_array(w[k])
        keep.append(arr)
        setattr(ptrs, k, C.cast(arr, C.POINTER(C.c_void_p)))
    ptrs.gf, ptrs.wlm = w["gf"].data_ptr(), w["wlm"].data_ptr()
    _set_head_norms(ptrs, w, cfg, keep)
    nbytes = sun_weights_pack_bytes(cfg)
    pack = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=w["embed"].device) if cfg.act_dtype == SUN_BF16 else None
    out = C.c_void_p()
    _check(lib().sun_weights_create(C.byref(cfg), C.byref(ptrs), _p(pack), nbytes, _stream(stream), C.byref(out)))
    keep.append(pack)
    if keep_sources or cfg.act_dtype == SUN_F32:
        keep.append(w)
    else:
        keep.extend([w["embed"], w["g1"], w["g2"], w["gf"], w.get("qn"), w.get("kn")])
    return Weights(out.value, keep, False)


def sun_qweights_pack_bytes(cfg: ModelCfg, group: int = 128) -> int:
    return int(lib().sun_qweights_pack_bytes(C.byref(cfg), group))


def sun_qweights_create(cfg: ModelCfg, w: Dict[str, object], quant: Dict[str, list], group: int = 128,
                        stream=None) -> Weights:
    """quant[key][layer] = (q uint8 [out, in/2], s fp16 [out, in/128], z fp16 [out, in/128]) CUDA tensors;
    w supplies embed, g1, g2, gf, wlm."""
    ptrs = QWeightPtrs()
    keep: List[object] = [w["embed"], w["g1"], w["g2"], w["gf"], w["wlm"], quant]
    ptrs.embed = w["embed"].data_ptr()
    for k in ("g1", "g2"):
        arr = _ptr_array(w[k])
        keep.append(arr)
        setattr(ptrs, k, C.cast(arr, C.POINTER(C.c_void_p)))
    for k in QUANT_KEYS:
        arr = (QMat * len(quant[k]))(*[QMat(q.data_ptr(), s.data_ptr(), z.data_ptr() if z is not None else None)
                                       for (q, s, z) in quant[k]])
        keep.append(arr)
        setattr(ptrs, k, C.cast(arr, C.POINTER(QMat)))
    ptrs.gf, ptrs.wlm = w["gf"].data_ptr(), w["wlm"].data_ptr()
    _set_head_norms(ptrs, w, cfg, keep)
    nbytes = sun_qweights_pack_bytes(cfg, group)
    pack = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=w["embed"].device) if cfg.act_dtype == SUN_BF16 else None
    out = C.c_void_p()
    _check(lib().sun_qweights_create(C.byref(cfg), C.byref(ptrs), group, _p(pack), nbytes, _stream(stream), C.byref(out)))
    keep.append(pack)
    return Weights(out.value, keep, True)


def sun_quantize_w4(w: torch.Tensor, group: int = 128, mode: str = "asym", stream=None):
    """Returns (q uint8 [rows, cols/2], s fp16 [rows, cols/group], z fp16 [rows, cols/group]); mode "sym_noz" is
    the symmetric grid without stored zero points (z is None: 8 everywhere)."""
    rows, cols = w.shape
    dt = {torch.float32: SUN_F32, torch.bfloat16: SUN_BF16}[w.dtype]
    q = torch.empty((rows, cols // 2), dtype=torch.uint8, device=w.device)
    s = torch.empty((rows, cols // group), dtype=torch.float16, device=w.device)
    z = torch.empty_like(s) if mode != "sym_noz" else None
    _check(lib().sun_quantize_w4(_p(w), dt, rows, cols, group, {"asym": 0, "sym": 1, "sym_noz": 1}[mode], _p(q), _p(s),
                                 _p(z), _stream(stream)))
    return q, s, z


# ------------------------------------------------------------------ step
def sun_workspace_bytes(cfg: ModelCfg, max_batch: int, max_pages: int) -> int:
    return int(lib().sun_workspace_bytes(C.byref(cfg), max_batch, max_pages))


def _host_i32(a):
    if a is None:
        return None, None
    import numpy as np
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data


def _step(fn, pool, weights, token_ids, page_tables, seq_lens, model_ids, logits_out, next_tokens_out, workspace,
          seq_lens_host, stream, flags):
    batch, max_pages = page_tables.shape
    keep, host_ptr = _host_i32(seq_lens_host)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(fn(pool.handle if pool is not None else None, weights.handle if weights is not None else None, batch,
              _p(token_ids), _p(page_tables), max_pages, _p(seq_lens), host_ptr, _p(model_ids), _p(logits_out),
              _p(next_tokens_out), _p(workspace), ws_bytes, _stream(stream), flags))


def sun_decode_step(pool, weights, token_ids, page_tables, seq_lens, model_ids, logits_out, next_tokens_out,
                    workspace, seq_lens_host=None, stream=None, flags: int = 0):
    _step(lib().sun_decode_step, pool, weights, token_ids, page_tables, seq_lens, model_ids, logits_out,
          next_tokens_out, workspace, seq_lens_host, stream, flags)


def sun_qdecode_step(pool, weights, token_ids, page_tables, seq_lens, model_ids, logits_out, next_tokens_out,
                     workspace, seq_lens_host=None, stream=None, flags: int = 0):
    _step(lib().sun_qdecode_step, pool, weights, token_ids, page_tables, seq_lens, model_ids, logits_out,
          next_tokens_out, workspace, seq_lens_host, stream, flags)


def sun_kv_pool_ingest(pool, model_id: int, k_src, v_src, first_pos: int, page_table_row, stream=None, flags: int = 0):
    """k_src, v_src: bf16 tensors [n_layers, n_tokens, n_kv_heads, head_dim]; page_table_row: int32 [max_pages]."""
    _check(lib().sun_kv_pool_ingest(pool.handle, model_id, _p(k_src), _p(v_src), int(k_src.shape[1]), first_pos,
                                    _p(page_table_row), int(page_table_row.numel()), _stream(stream), flags))


def sun_kv_pool_model_tokens(pool, model_id: int) -> int:
    n = C.c_int64()
    _check(lib().sun_kv_pool_model_tokens(pool.handle, model_id, C.byref(n)))
    return int(n.value)


def sun_decode_run(pool, weights, n_steps: int, token_ids, page_tables, seq_lens, model_ids, free_pages, free_head,
                   run_status, tokens_out, logits_out, workspace, stream=None, flags: int = 0):
    """n_steps greedy steps in a row; token_ids, page_tables, seq_lens and free_head are updated on the device."""
    batch, max_pages = page_tables.shape
    n_free = int(free_pages.numel()) if free_pages is not None else 0
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().sun_decode_run(pool.handle if pool is not None else None,
                                weights.handle if weights is not None else None, batch, n_steps, _p(token_ids),
                                _p(page_tables), max_pages, _p(seq_lens), _p(model_ids), _p(free_pages), n_free,
                                _p(free_head), _p(run_status), _p(tokens_out), _p(logits_out), _p(workspace), ws_bytes,
                                _stream(stream), flags))


def sun_serve_workspace_bytes(cfg: ModelCfg, slots: int, max_pages: int) -> int:
    return int(lib().sun_serve_workspace_bytes(C.byref(cfg), slots, max_pages))


class ServeTensors:
    """Device tensors of a continuous-batching decode worker (the fields of sun_serve_state), kept alive
    together with the struct handed to the library."""

    def __init__(self, slots: int, max_pages: int, waiting, ring_pages, ring_cap: int, idle_page: int,
                 eos_id: int = -1, device="cuda"):
        import torch
        i32 = dict(dtype=torch.int32, device=device)
        self.slots, self.max_pages = slots, max_pages
        self.token_ids = torch.zeros(slots, **i32)
        self.page_tables = torch.full((slots, max_pages), -1, **i32)
        self.seq_lens = torch.zeros(slots, **i32)
        self.model_ids = torch.zeros(slots, **i32)
        self.slot_req = torch.full((slots,), -1, **i32)
        self.slot_left = torch.zeros(slots, **i32)
        n = len(waiting["req"])
        self.n_wait = n
        self.w = {k: torch.as_tensor(waiting[k], dtype=torch.int32).to(device).contiguous()
                  for k in ("req", "token", "tables", "lens", "model", "budget")}
        assert self.w["tables"].shape == (n, max_pages) or n == 0
        ring = torch.zeros(ring_cap, **i32)
        ring[:len(ring_pages)] = torch.as_tensor(ring_pages, dtype=torch.int32)
        self.ring, self.ring_cap = ring, ring_cap
        self.counters = torch.zeros(8, **i32)
        self.counters[2] = len(ring_pages)
        self.idle_page, self.eos_id = idle_page, eos_id

    def struct(self) -> "ServeState":
        s = ServeState()
        for name in ("token_ids", "page_tables", "seq_lens", "model_ids", "slot_req", "slot_left", "ring", "counters"):
            setattr(s, name, _p(getattr(self, name)))
        for k in ("req", "token", "tables", "lens", "model", "budget"):
            setattr(s, "w_" + k, _p(self.w[k]) if self.n_wait else None)
        s.n_wait, s.ring_cap, s.idle_page, s.eos_id = self.n_wait, self.ring_cap, self.idle_page, self.eos_id
        return s


def sun_decode_serve(pool, weights, n_steps: int, state: ServeTensors, tokens_out, req_out, logits_out, workspace,
                     stream=None, flags: int = 0):
    """n_steps iterations of decode + retire/advance/admit on the device; `state` is updated in place."""
    st = state.struct()
    _check(lib().sun_decode_serve(pool.handle, weights.handle, state.slots, state.max_pages, n_steps, C.byref(st),
                                  _p(tokens_out), _p(req_out), _p(logits_out), _p(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream), flags))


def sun_prefill_workspace_bytes(cfg: ModelCfg, n_tokens: int, max_pages: int) -> int:
    return int(lib().sun_prefill_workspace_bytes(C.byref(cfg), n_tokens, max_pages))


def sun_prefill(pool, weights, token_ids, page_table_row, first_pos: int, model_id: int, logits_out, next_token_out,
                workspace, stream=None, flags: int = 0):
    """Causal forward of `weights` over the prompt tokens (int32 [n_tokens]) of one request; fills its pages."""
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    n_tokens = int(token_ids.numel()) if token_ids is not None else 0
    max_pages = int(page_table_row.numel()) if page_table_row is not None else 0
    _check(lib().sun_prefill(pool.handle if pool is not None else None,
                             weights.handle if weights is not None else None, n_tokens, _p(token_ids),
                             _p(page_table_row), max_pages, first_pos, model_id, _p(logits_out), _p(next_token_out),
                             _p(workspace), ws_bytes, _stream(stream), flags))


def sun_paged_attention(pool, layer: int, q, page_tables, n_tokens, out, workspace, n_tokens_host=None, stream=None):
    batch, max_pages = page_tables.shape
    keep, host_ptr = _host_i32(n_tokens_host)
    _check(lib().sun_paged_attention(pool.handle, layer, batch, _p(q), _p(page_tables), max_pages, _p(n_tokens),
                                     host_ptr, _p(out), _p(workspace), workspace.numel() * workspace.element_size(),
                                     _stream(stream)))


def sun_paged_attention_static(pool, layer: int, q, page_tables, n_tokens, out, n_tokens_host=None, stream=None):
    batch, max_pages = page_tables.shape
    keep, host_ptr = _host_i32(n_tokens_host)
    _check(lib().sun_paged_attention_static(pool.handle, layer, batch, _p(q), _p(page_tables), max_pages, _p(n_tokens),
                                            host_ptr, _p(out), _stream(stream)))


def sun_paged_attention_static_bytes(cfg, batch: int, max_pages: int) -> int:
    return int(lib().sun_paged_attention_static_bytes(C.byref(cfg), batch, max_pages))


def sun_paged_attention_static_limit() -> int:
    return int(lib().sun_paged_attention_static_limit())


def sun_linear(weights, layer: int, mat: int, x, out, workspace, stream=None):
    _check(lib().sun_linear(weights.handle, layer, mat, x.shape[0], _p(x), _p(out), _p(workspace),
                            workspace.numel() * workspace.element_size(), _stream(stream)))


def sun_hbm_read_probe(src, block_bytes: int, perm, workgroups: int, sink, streaming_loads: bool = False, stream=None):
    _check(lib().sun_hbm_read_probe(_p(src), src.numel() * src.element_size(), block_bytes, _p(perm) if perm is not None else None,
                                    workgroups, 1 if streaming_loads else 0, _p(sink), _stream(stream)))


def sun_profile_reset():
    lib().sun_profile_reset()


def sun_profile_read() -> Dict[str, Dict[str, float]]:
    out = {}
    for k, name in enumerate(PROFILE_KINDS):
        ms, n = C.c_double(), C.c_int64()
        _check(lib().sun_profile_read(k, C.byref(ms), C.byref(n)))
        out[name] = {"ms": ms.value, "launches": int(n.value)}
    return out


def sun_version() -> str:
    return lib().sun_version().decode()
