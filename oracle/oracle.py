"""ctypes front end of the CPU oracle (oracle/sun_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu-baseline leg.  The GPU library never imports this module and
this module never imports the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sun_oracle.c")
_LIB = os.path.join(_HERE, "libsun_oracle.so")

F32, BF16, F64, W4 = 0, 1, 2, 3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP across independent rows/requests)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Cfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("rms_eps", C.c_double), ("rope_base", C.c_double),
                ("act_bf16", C.c_int32), ("qk_norm", C.c_int32), ("rope_scaling", C.c_int32),
                ("rope_orig_max", C.c_int32), ("rope_factor", C.c_double), ("rope_low_freq", C.c_double),
                ("rope_high_freq", C.c_double), ("qkv_bias", C.c_int32), ("pad_", C.c_int32)]


class Mat(C.Structure):
    _fields_ = [("kind", C.c_int32), ("rows", C.c_int32), ("cols", C.c_int32), ("group", C.c_int32),
                ("data", C.c_void_p), ("q", C.c_void_p), ("s", C.c_void_p), ("z", C.c_void_p)]


class Pool(C.Structure):
    _fields_ = [("base", C.c_void_p), ("n_pages", C.c_int64), ("page_tokens", C.c_int32), ("pad_", C.c_int32),
                ("k_off", C.c_int64), ("k_layer", C.c_int64), ("k_page", C.c_int64), ("k_head", C.c_int64),
                ("k_token", C.c_int64), ("k_dim", C.c_int64),
                ("v_off", C.c_int64), ("v_layer", C.c_int64), ("v_page", C.c_int64), ("v_head", C.c_int64),
                ("v_token", C.c_int64), ("v_dim", C.c_int64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_silu.restype = C.c_double
        _lib.orc_silu.argtypes = [C.c_double]
        _lib.orc_bf16_to_double.restype = C.c_double
        _lib.orc_bf16_to_double.argtypes = [C.c_uint16]
        _lib.orc_double_to_bf16.restype = C.c_uint16
        _lib.orc_double_to_bf16.argtypes = [C.c_double]
        _lib.orc_float_to_half.restype = C.c_uint16
        _lib.orc_float_to_half.argtypes = [C.c_float]
        _lib.orc_half_to_float.restype = C.c_float
        _lib.orc_half_to_float.argtypes = [C.c_uint16]
        _lib.orc_argmax.restype = C.c_int32
    return _lib


def threads() -> int:
    return int(lib().orc_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def make_cfg(shape, act_bf16: bool = False) -> Cfg:
    """shape: any object with the Shape fields (n_layers, hidden, ...).  act_bf16 selects the
    16-bit configuration, in which every projection consumes bf16-rounded activations."""
    rs = getattr(shape, "rope_scaling", None)  # (factor, low_freq_factor, high_freq_factor, original_max_position)
    return Cfg(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
               shape.ffn, shape.vocab, float(shape.rms_eps), float(shape.rope_base), int(act_bf16),
               int(bool(getattr(shape, "qk_norm", False))), 1 if rs else 0, int(rs[3]) if rs else 0,
               float(rs[0]) if rs else 1.0, float(rs[1]) if rs else 1.0, float(rs[2]) if rs else 1.0,
               int(bool(getattr(shape, "qkv_bias", False))), 0)


_KIND = {np.dtype(np.float32): F32, np.dtype(np.uint16): BF16, np.dtype(np.float64): F64}


def dense_mat(a: np.ndarray) -> Mat:
    """Dense parameter; a uint16 array is read as bfloat16 bit patterns."""
    assert a.flags["C_CONTIGUOUS"]
    if a.ndim == 1:
        rows, cols = 1, a.shape[0]
    else:
        rows, cols = a.shape
    return Mat(_KIND[a.dtype], rows, cols, 0, _ptr(a), None, None, None)


def w4_mat(q: np.ndarray, s: np.ndarray, z: np.ndarray, cols: int, group: int) -> Mat:
    """Quantised parameter: q uint8 [rows, cols/2], s/z uint16 (fp16 bits) [rows, groups]."""
    assert q.dtype == np.uint8 and s.dtype == np.uint16 and z.dtype == np.uint16
    assert q.flags["C_CONTIGUOUS"] and s.flags["C_CONTIGUOUS"] and z.flags["C_CONTIGUOUS"]
    return Mat(W4, q.shape[0], cols, group, None, _ptr(q), _ptr(s), _ptr(z))


class Params:
    """Parameter table in the order the C side expects; keeps the arrays alive."""

    def __init__(self, n_layers: int):
        self.n_layers = n_layers
        self.mats = (Mat * (3 + PER_LAYER * n_layers))()
        self.keep: List[object] = []

    def set(self, idx: int, m: Mat, *arrays):
        self.mats[idx] = m
        self.keep.extend(arrays)


LAYER_KEYS = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")
HEAD_NORM_KEYS = ("qn", "kn")   # gains of the optional q/k head norm, length head_dim; absent -> ones (unused)
BIAS_KEYS = ("bq", "bk", "bv")  # biases of the optional q/k/v projection bias; absent -> a dummy (unused)
PER_LAYER = len(LAYER_KEYS) + len(HEAD_NORM_KEYS) + len(BIAS_KEYS)
QUANT_KEYS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")


def params_from_arrays(w: Dict[str, object], quant: Optional[Dict[str, list]] = None,
                       group: int = 128) -> Params:
    """w: dict of numpy arrays (float32 / float64 / uint16-as-bf16): 'embed', 'gf', 'wlm'
    and per-layer lists under LAYER_KEYS.  quant: optional dict key -> list of (q, s, z)
    per layer replacing the dense matrices of QUANT_KEYS (QSUN, Appendix A.1)."""
    nl = len(w["wq"])
    p = Params(nl)
    p.set(0, dense_mat(w["embed"]), w["embed"])
    for l in range(nl):
        for j, k in enumerate(LAYER_KEYS):
            if quant is not None and k in quant:
                q, s, z = quant[k][l]
                cols = w[k][l].shape[1]
                p.set(1 + PER_LAYER * l + j, w4_mat(q, s, z, cols, group), q, s, z)
            else:
                p.set(1 + PER_LAYER * l + j, dense_mat(w[k][l]), w[k][l])
        for j, k in enumerate(HEAD_NORM_KEYS + BIAS_KEYS):
            g = w[k][l] if k in w else np.ones(1, dtype=np.float64)
            p.set(1 + PER_LAYER * l + len(LAYER_KEYS) + j, dense_mat(g), g)
    p.set(1 + PER_LAYER * nl, dense_mat(w["gf"]), w["gf"])
    p.set(2 + PER_LAYER * nl, dense_mat(w["wlm"]), w["wlm"])
    return p


def make_pool(base: np.ndarray, n_pages: int, page_tokens: int, strides: Dict[str, int]) -> Pool:
    """base: uint16 array holding the bf16 pool.  strides: element strides with keys
    k_off,k_layer,k_page,k_head,k_token,k_dim and the same for v_."""
    assert base.dtype == np.uint16 and base.flags["C_CONTIGUOUS"]
    p = Pool()
    p.base = _ptr(base)
    p.n_pages = n_pages
    p.page_tokens = page_tokens
    for k, v in strides.items():
        setattr(p, k, int(v))
    p._keep = base
    return p


def default_strides(shape, n_pages: int, page_tokens: int = 16) -> Dict[str, int]:
    """A plain layout for CPU-only tests: [layer][page][k|v][head][token][dim]."""
    d, hkv = shape.head_dim, shape.n_kv_heads
    blk = page_tokens * d
    page = 2 * hkv * blk
    return dict(k_off=0, k_layer=n_pages * page, k_page=page, k_head=blk, k_token=d, k_dim=1,
                v_off=hkv * blk, v_layer=n_pages * page, v_page=page, v_head=blk, v_token=d, v_dim=1)


def pool_elems(shape, n_pages: int, page_tokens: int = 16) -> int:
    return shape.n_layers * n_pages * 2 * shape.n_kv_heads * page_tokens * shape.head_dim


def kv_ingest(base: np.ndarray, strides: Dict[str, int], k_src: np.ndarray, v_src: np.ndarray, first_pos: int,
              page_table, page_tokens: int = 16) -> None:
    """Places a cache computed elsewhere (Eq. 2: the prefill module's C_T for a prompt, or a later chunk of
    it) into the pages a request owns: token t of the source becomes position first_pos + t, which lives in
    slot (first_pos + t) % page_tokens of page page_table[(first_pos + t) // page_tokens].  k_src, v_src:
    uint16 bf16 bit patterns [n_layers, n_tokens, n_kv_heads, head_dim]; base: the pool as a flat uint16
    array, addressed through `strides` (element strides and offsets as in make_pool).  Nothing is converted:
    a byte-exact scatter."""
    assert k_src.dtype == np.uint16 and v_src.dtype == np.uint16 and k_src.shape == v_src.shape
    nl, nt, hkv, d = k_src.shape
    for l in range(nl):
        for t in range(nt):
            pos = first_pos + t
            page, slot = int(page_table[pos // page_tokens]), pos % page_tokens
            if page < 0:
                raise ValueError(f"position {pos} has no page")
            for h in range(hkv):
                for kv, src in (("k", k_src), ("v", v_src)):
                    o = (strides[kv + "_off"] + l * strides[kv + "_layer"] + page * strides[kv + "_page"] +
                         h * strides[kv + "_head"] + slot * strides[kv + "_token"])
                    base[o + np.arange(d) * strides[kv + "_dim"]] = src[l, t, h]


def decode_step(cfg: Cfg, params: Params, pool: Pool, tokens, page_tables, seq_lens, model_ids,
                mode: int = 0, want_rowsums: bool = False, want_attn: bool = False):
    """Runs one decode step; mutates the pool (appends the new K/V).  Returns a dict."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    page_tables = np.ascontiguousarray(page_tables, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    model_ids = np.ascontiguousarray(model_ids, dtype=np.int32)
    B = tokens.shape[0]
    logits = np.empty((B, cfg.vocab), dtype=np.float64)
    nxt = np.empty(B, dtype=np.int32)
    rows = np.empty((B, cfg.n_layers, cfg.n_q_heads), dtype=np.float64) if want_rowsums else None
    attn = np.empty((B, cfg.n_layers, cfg.n_q_heads * cfg.head_dim), dtype=np.float64) if want_attn else None
    rc = lib().orc_decode_step(C.byref(cfg), params.mats, C.byref(pool), C.c_int(B), _ptr(tokens),
                               _ptr(page_tables), C.c_int(page_tables.shape[1]), _ptr(seq_lens),
                               _ptr(model_ids), C.c_int(mode), _ptr(logits), _ptr(nxt), _ptr(rows), _ptr(attn))
    if rc != 0:
        raise ValueError(f"orc_decode_step failed with status {rc}")
    return {"logits": logits, "next": nxt, "rowsums": rows, "attn": attn}


def decode_step_peer(cfg: Cfg, params: Params, pool: Pool, peer: Pool, tokens, page_tables, seq_lens, model_ids,
                     tol_abs: float, tol_rel: float = 0.0, mode: int = 0):
    """One decode step next to another implementation's cache after the same step (`peer`, same page ids):
    every new K/V value is computed and rounded here; where the peer's stored bf16 code is that rounding, its
    neighbour, or within tol_abs + tol_rel |value| of it, the peer's code is what this step stores and attends
    over (a stored code is a rounding decision that a correct fp32 implementation may take one step away),
    otherwise its own.  Returns the dict of decode_step plus "peer": counts of entries (equal, adopted as
    neighbour, adopted by value, kept own = peer rejected)."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    page_tables = np.ascontiguousarray(page_tables, dtype=np.int32)
    seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
    model_ids = np.ascontiguousarray(model_ids, dtype=np.int32)
    B = tokens.shape[0]
    logits = np.empty((B, cfg.vocab), dtype=np.float64)
    nxt = np.empty(B, dtype=np.int32)
    stats = np.zeros(4, dtype=np.int64)
    rc = lib().orc_decode_step_peer(C.byref(cfg), params.mats, C.byref(pool), C.c_int(B), _ptr(tokens),
                                    _ptr(page_tables), C.c_int(page_tables.shape[1]), _ptr(seq_lens),
                                    _ptr(model_ids), C.c_int(mode), _ptr(logits), _ptr(nxt), C.byref(peer),
                                    C.c_double(tol_abs), C.c_double(tol_rel), _ptr(stats))
    if rc != 0:
        raise ValueError(f"orc_decode_step_peer failed with status {rc}")
    return {"logits": logits, "next": nxt, "peer": {"equal": int(stats[0]), "neighbour": int(stats[1]),
                                                    "by_value": int(stats[2]), "rejected": int(stats[3])}}


def decode_run(cfg: Cfg, params: Params, pool: Pool, tokens, page_tables, seq_lens, model_ids, free_pages,
               free_head: int, n_steps: int, page_tokens: int = 16, mode: int = 0, forced_tokens=None,
               keep_logits: bool = False):
    """Greedy decoding as the repeated application of the decode step (Section 3.1, Eq. 3 applied for
    t = T+1, T+2, ...; every step extends each cache by one entry, Eq. 4), for a fixed set of requests.

    After a step, a request's generated token becomes its next input and its length grows by one.  When
    the position it will write next opens a new page (length % page_tokens == 0) and its table has no
    page there yet, it takes the next unused entry of `free_pages`; requests are served in index order.
    A request that finds the free list empty, or whose table is full, is frozen: its token is still
    replaced, its length is not advanced, so it re-decodes the same position; bit 0 (free list empty)
    or bit 1 (table full) of the returned status is set.

    forced_tokens [n_steps, B], if given, replaces the fed-back tokens (teacher forcing); the step's own
    argmax is still what is recorded.  Mutates pool, page_tables and seq_lens copies; returns a dict with
    tokens [n_steps, B], the last step's logits (every step's, [n_steps, B, V], under keep_logits), final
    page_tables, seq_lens, free_head, status."""
    tokens = np.array(tokens, dtype=np.int32, copy=True)
    tables = np.array(page_tables, dtype=np.int32, copy=True)
    lens = np.array(seq_lens, dtype=np.int32, copy=True)
    model_ids = np.ascontiguousarray(model_ids, dtype=np.int32)
    free_pages = np.ascontiguousarray(free_pages, dtype=np.int32)
    B, max_pages = tables.shape
    out = np.empty((n_steps, B), dtype=np.int32)
    status, head, logits, every = 0, int(free_head), None, []
    for s in range(n_steps):
        res = decode_step(cfg, params, pool, tokens, tables, lens, model_ids, mode=mode)
        out[s] = res["next"]
        logits = res["logits"]
        if keep_logits:
            every.append(logits)
        tokens = np.array(out[s] if forced_tokens is None else forced_tokens[s], dtype=np.int32)
        for i in range(B):
            new_len = int(lens[i]) + 1
            slot_page = new_len // page_tokens
            if slot_page >= max_pages:
                status |= 2
                continue
            if new_len % page_tokens == 0 and tables[i, slot_page] < 0:
                if head >= len(free_pages):
                    status |= 1
                    continue
                tables[i, slot_page] = free_pages[head]
                head += 1
            lens[i] = new_len
    if keep_logits:
        logits = np.stack(every)
    return {"tokens": out, "logits": logits, "page_tables": tables, "seq_lens": lens, "free_head": head,
            "status": status}


def serve_run(cfg: Cfg, params: Params, pool: Pool, slots: int, max_pages: int, n_steps: int, waiting, ring_pages,
              idle_page: int, eos_id: int = -1, page_tokens: int = 16, mode: int = 0, forced_tokens=None,
              state=None, keep_logits: bool = False, bookkeeping_only: bool = False):
    """A decode worker that admits and retires requests between steps (the continuous batching of
    Section 2.1.1): `slots` batch rows, each idle or occupied by one request, the decode step of Eq. 3
    over the occupied rows every iteration, and between iterations, in this order and in row order
    within each:
      1. an occupied row records its token and has one token less to generate; it is finished when none
         is left or the token is eos_id;
      2. finished rows retire: their pages go to the tail of the list of free pages (column order) and
         the row becomes idle;
      3. the others feed their token back and grow by one position, taking the page at the head of the
         free list when the next position opens a page their table lacks;
      4. idle rows take waiting requests first in, first out, while the head of the queue fits: the
         pages it may still need, (len + budget - 1) // page_tokens + 1 minus those its table holds,
         must be free beyond what the rows already admitted may still need.  A budget running past the
         table is cut to fit (status bit 1).
    Idle rows are not decoded here: a request's tokens depend on nothing but its own cache and input.

    waiting: list of dicts {req, token, table (int32 [max_pages]), len, model, budget}, already prefilled.
    forced_tokens [n_steps, slots], if given, is taken as the token of every occupied row instead of the
    row's own argmax (recorded, tested against eos_id and fed back), so that a replay follows another
    implementation through a near-tie; the row's own logits are kept for the comparison.  state: the dict a
    previous call returned (continues it) or None (all rows idle, then admission, before the first step).
    bookkeeping_only (needs forced_tokens): the decode step is not run at all; what remains is the schedule
    and the page accounting, which depend on the tokens through eos_id only.
    Returns the state dict: rows, ring (list, head first), counters, plus tokens/reqs [n_steps, slots]
    (-1 for idle rows), writes (step, row, request, page, slot of every position appended, Eq. 4) and the logits of every step under keep_logits (rows of idle slots are NaN)."""
    if state is None:
        st = {"req": [-1] * slots, "left": [0] * slots, "token": [0] * slots, "len": [0] * slots,
              "model": [0] * slots, "tables": np.full((slots, max_pages), -1, np.int32),
              "ring": [int(p) for p in ring_pages], "whead": 0, "status": 0, "retired": 0, "admitted": 0,
              "generated": 0, "steps": 0}
        st["tables"][:, 0] = idle_page
    else:
        st = {k: (v.copy() if isinstance(v, np.ndarray) else (list(v) if isinstance(v, list) else v))
              for k, v in state.items() if k not in ("tokens", "reqs", "logits", "writes")}

    def held(row):
        return int((np.asarray(row) >= 0).sum())

    def admit():
        outstanding = sum(max(0, (st["len"][i] + st["left"][i] - 1) // page_tokens + 1 - held(st["tables"][i]))
                          for i in range(slots) if st["req"][i] >= 0)
        avail = len(st["ring"]) - outstanding
        for i in range(slots):
            if st["req"][i] >= 0:
                continue
            if st["whead"] >= len(waiting):
                break
            w = waiting[st["whead"]]
            budget = int(w["budget"])
            room = max_pages * page_tokens - int(w["len"])
            cut = budget > room
            budget = max(1, min(budget, room))
            need = max(0, (int(w["len"]) + budget - 1) // page_tokens + 1 - held(w["table"]))
            if need > avail:
                break                      # the head of the queue blocks those behind it
            avail -= need
            if cut:
                st["status"] |= 2
            st["req"][i], st["left"][i], st["token"][i] = int(w["req"]), budget, int(w["token"])
            st["len"][i], st["model"][i] = int(w["len"]), int(w["model"])
            st["tables"][i] = np.asarray(w["table"], np.int32)
            st["whead"] += 1
            st["admitted"] += 1

    if state is None:
        admit()
    toks_out = np.full((n_steps, slots), -1, np.int32)
    reqs_out = np.full((n_steps, slots), -1, np.int32)
    every, writes = [], []
    for s in range(n_steps):
        rows = [i for i in range(slots) if st["req"][i] >= 0]
        writes += [(s, i, st["req"][i], int(st["tables"][i, st["len"][i] // page_tokens]), st["len"][i] % page_tokens)
                   for i in rows]
        lg_all = np.full((slots, cfg.vocab), np.nan) if not bookkeeping_only else None
        nxt = {}
        if rows and not bookkeeping_only:
            res = decode_step(cfg, params, pool, np.array([st["token"][i] for i in rows], np.int32),
                              st["tables"][rows], np.array([st["len"][i] for i in rows], np.int32),
                              np.array([st["model"][i] for i in rows], np.int32), mode=mode)
            for j, i in enumerate(rows):
                nxt[i] = int(res["next"][j])
                lg_all[i] = res["logits"][j]
        if keep_logits:
            every.append(lg_all)
        finished = []
        for i in rows:                                   # 1
            tok = nxt[i] if forced_tokens is None else int(forced_tokens[s][i])
            toks_out[s, i], reqs_out[s, i] = tok, st["req"][i]
            st["left"][i] -= 1
            st["generated"] += 1
            st["token"][i] = tok
            if st["left"][i] == 0 or tok == eos_id:
                finished.append(i)
        for i in finished:                               # 2
            st["ring"].extend(int(p) for p in st["tables"][i] if p >= 0)
            st["tables"][i] = -1
            st["tables"][i, 0] = idle_page
            st["req"][i], st["left"][i], st["token"][i], st["len"][i], st["model"][i] = -1, 0, 0, 0, 0
            st["retired"] += 1
        for i in rows:                                   # 3
            if i in finished:
                continue
            new_len = st["len"][i] + 1
            col = new_len // page_tokens
            if col >= max_pages:
                st["status"] |= 2
                continue
            if new_len % page_tokens == 0 and st["tables"][i, col] < 0:
                if not st["ring"]:
                    st["status"] |= 1
                    continue
                st["tables"][i, col] = st["ring"].pop(0)
            st["len"][i] = new_len
        admit()                                          # 4
        st["steps"] += 1
    st["tokens"], st["reqs"], st["writes"] = toks_out, reqs_out, writes
    if keep_logits:
        st["logits"] = np.stack(every) if every else None
    return st


def decode_contig_f64(cfg: Cfg, params: Params, token: int, L: int, Kc: np.ndarray, Vc: np.ndarray,
                      round_kv: bool = False):
    """Kc, Vc: float64 [NL, cap, Hkv, d]; writes position L.  Returns (logits, next)."""
    assert Kc.dtype == np.float64 and Kc.flags["C_CONTIGUOUS"] and Vc.flags["C_CONTIGUOUS"]
    logits = np.empty(cfg.vocab, dtype=np.float64)
    nxt = C.c_int32(0)
    rc = lib().orc_decode_contig_f64(C.byref(cfg), params.mats, C.c_int32(token), C.c_int64(L),
                                     C.c_int64(Kc.shape[1]), _ptr(Kc), _ptr(Vc), C.c_int(int(round_kv)),
                                     _ptr(logits), C.byref(nxt))
    if rc != 0:
        raise ValueError(f"orc_decode_contig_f64 failed with status {rc}")
    return logits, int(nxt.value)


def full_forward(cfg: Cfg, params: Params, tokens, round_kv: bool = False, want_kv: bool = False):
    """Causal forward over the whole sequence (no cache). Returns logits [T,V] (and K,V)."""
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    T = tokens.shape[0]
    logits = np.empty((T, cfg.vocab), dtype=np.float64)
    K = V = None
    if want_kv:
        K = np.empty((cfg.n_layers, T, cfg.n_kv_heads, cfg.head_dim), dtype=np.float64)
        V = np.empty_like(K)
    rc = lib().orc_full_forward(C.byref(cfg), params.mats, C.c_int(T), _ptr(tokens), C.c_int(int(round_kv)),
                                _ptr(logits), _ptr(K), _ptr(V))
    if rc != 0:
        raise ValueError(f"orc_full_forward failed with status {rc}")
    return (logits, K, V) if want_kv else logits


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float64)
    h = np.empty_like(x)
    lib().orc_rmsnorm(_ptr(x), _ptr(g), C.c_int(x.shape[0]), C.c_double(eps), _ptr(h))
    return h


def rope(u: np.ndarray, pos: int, base: float) -> np.ndarray:
    out = np.array(u, dtype=np.float64, copy=True)
    lib().orc_rope(_ptr(out), C.c_int(out.shape[0]), C.c_int64(pos), C.c_double(base))
    return out


def rope_freq(cfg: Cfg, j: int) -> float:
    lib().orc_rope_freq.restype = C.c_double
    return float(lib().orc_rope_freq(C.byref(cfg), C.c_int(j)))


def silu(z: float) -> float:
    return float(lib().orc_silu(z))


def linear(m: Mat, X: np.ndarray) -> np.ndarray:
    X = np.ascontiguousarray(X, dtype=np.float64)
    Y = np.empty((X.shape[0], m.rows), dtype=np.float64)
    lib().orc_linear(C.byref(m), _ptr(X), C.c_int(X.shape[0]), _ptr(Y))
    return Y


def argmax(v: np.ndarray) -> int:
    v = np.ascontiguousarray(v, dtype=np.float64)
    return int(lib().orc_argmax(_ptr(v), C.c_int(v.shape[0])))


def attention_paged(cfg: Cfg, pool: Pool, layer: int, page_table: np.ndarray, q: np.ndarray, n: int):
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    q = np.ascontiguousarray(q, dtype=np.float64)
    a = np.empty(cfg.n_q_heads * cfg.head_dim, dtype=np.float64)
    rs = np.empty(cfg.n_q_heads, dtype=np.float64)
    rc = lib().orc_attention_paged(C.byref(cfg), C.byref(pool), C.c_int(layer), _ptr(page_table), _ptr(q),
                                   C.c_int64(n), _ptr(a), _ptr(rs))
    assert rc == 0
    return a, rs


def quantize_w4(w: np.ndarray, group: int = 128, mode: str = "asym"):
    """Returns (q uint8 [rows, cols/2], s uint16 [rows, groups], z uint16 [rows, groups])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    rows, cols = w.shape
    ng = (cols + group - 1) // group
    q = np.empty((rows, cols // 2), dtype=np.uint8)
    s = np.empty((rows, ng), dtype=np.uint16)
    z = np.empty((rows, ng), dtype=np.uint16)
    rc = lib().orc_quantize_w4(_ptr(w), C.c_int(rows), C.c_int(cols), C.c_int(group),
                               C.c_int({"asym": 0, "sym": 1}[mode]), _ptr(q), _ptr(s), _ptr(z))
    if rc != 0:
        raise ValueError(f"orc_quantize_w4 failed with status {rc}")
    return q, s, z


def dequantize_w4(q: np.ndarray, s: np.ndarray, z: np.ndarray, cols: int, group: int = 128) -> np.ndarray:
    m = w4_mat(q, s, z, cols, group)
    out = np.empty((q.shape[0], cols), dtype=np.float32)
    lib().orc_dequantize_w4(C.byref(m), _ptr(out))
    return out


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 values to bf16 (nearest even) and return the bit patterns."""
    f = lib().orc_double_to_bf16
    flat = np.asarray(x, dtype=np.float64).ravel()
    return np.array([f(float(v)) for v in flat], dtype=np.uint16).reshape(np.shape(x))


def bf16_values(bits: np.ndarray) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32).astype(np.float64)
