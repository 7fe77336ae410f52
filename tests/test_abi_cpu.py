"""Boundary checks that need no GPU: the library loads, exports every symbol the header
declares, and rejects bad arguments before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

from paper_2603_02599_amd import binding as sun
from paper_2603_02599_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2603_02599_amd.build import build_lib
    build_lib()
    return sun.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "sun.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(sun_[a-z0-9_]+)\s*\(", header))
    assert len(names) >= 19
    for n in names:
        assert hasattr(lib, n), f"{n} declared in sun.h but not exported"
    assert set(sun.EXPORTS) == names
    assert b"gfx950" in lib.sun_version()


def test_struct_sizes_match_the_header(tmp_path):
    """The ctypes mirrors against the header itself: a C program that includes sun.h prints the sizes."""
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text('#include <stdio.h>\n#include "sun.h"\nint main(void) { printf("%zu %zu %zu %zu %zu %zu\\n", '
                   'sizeof(sun_model_cfg), sizeof(sun_kv_layout), sizeof(sun_qmat), sizeof(sun_weight_ptrs), '
                   'sizeof(sun_qweight_ptrs), sizeof(sun_serve_state)); return 0; }\n')
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-std=c11", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    sizes = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert sizes == [C.sizeof(sun.ModelCfg), C.sizeof(sun.KvLayout), C.sizeof(sun.QMat), C.sizeof(sun.WeightPtrs),
                     C.sizeof(sun.QWeightPtrs), C.sizeof(sun.ServeState)]
    assert C.sizeof(sun.ModelCfg) == 68 and C.sizeof(sun.KvLayout) == 8 + 8 + 12 * 8 + 8 and C.sizeof(sun.QMat) == 24


FAKE = 0x7F0000000000  # aligned, never dereferenced: these calls fail (or only store it) before any GPU work


def _pool(lib, cfg, n_pages=4, nsrc=3):
    out = C.c_void_p()
    nbytes = lib.sun_kv_pool_bytes(C.byref(cfg), n_pages, 16)
    rc = lib.sun_kv_pool_create(C.byref(cfg), FAKE, nbytes, 16, nsrc, C.byref(out))
    return rc, out


def test_pool_create_and_layout(lib):
    cfg = sun.make_cfg(wl.TINY, "f32")
    rc, pool = _pool(lib, cfg, 5)
    assert rc == 0
    lay = sun.KvLayout()
    assert lib.sun_kv_pool_layout(pool, C.byref(lay)) == 0
    assert lay.n_pages == 5 and lay.page_tokens == 16
    per_page = 2 * wl.TINY.n_kv_heads * 16 * wl.TINY.head_dim
    assert lay.total_elems == wl.TINY.n_layers * 5 * per_page == lib.sun_kv_pool_bytes(C.byref(cfg), 5, 16) // 2
    # K is [token][dim], V is [dim][token] inside a (layer, page, head) block; blocks do not overlap
    assert (lay.k_token, lay.k_dim, lay.v_token, lay.v_dim) == (64, 1, 1, 16)
    assert lay.v_off - lay.k_off == wl.TINY.n_kv_heads * 16 * 64 and lay.k_page == per_page
    lib.sun_kv_pool_destroy(pool)


def test_pool_create_errors(lib):
    cfg = sun.make_cfg(wl.TINY, "f32")
    out = C.c_void_p()
    assert lib.sun_kv_pool_create(C.byref(cfg), None, 1 << 20, 16, 1, C.byref(out)) == 1       # NULL memory
    assert lib.sun_kv_pool_create(C.byref(cfg), FAKE, 1 << 20, 8, 1, C.byref(out)) == 2        # page size
    assert lib.sun_kv_pool_create(C.byref(cfg), FAKE, 100, 16, 1, C.byref(out)) == 3           # no page fits
    assert lib.sun_kv_pool_create(C.byref(cfg), FAKE + 4, 1 << 20, 16, 1, C.byref(out)) == 3   # misaligned
    assert lib.sun_kv_pool_create(C.byref(cfg), FAKE, 1 << 20, 16, 0, C.byref(out)) == 7       # no source model
    assert b"source" in lib.sun_last_error()
    bad = sun.make_cfg(wl.TINY, "f32")
    bad.head_dim = 48
    assert lib.sun_kv_pool_create(C.byref(bad), FAKE, 1 << 20, 16, 1, C.byref(out)) == 2
    bad = sun.make_cfg(wl.TINY, "bf16")      # ffn 688 is not a multiple of 128
    assert lib.sun_kv_pool_create(C.byref(bad), FAKE, 1 << 20, 16, 1, C.byref(out)) == 2
    assert lib.sun_kv_pool_create(None, FAKE, 1 << 20, 16, 1, C.byref(out)) == 1


def _f32_weights(lib, cfg, shape):
    nl = shape.n_layers
    arrs = [(C.c_void_p * nl)(*([FAKE] * nl)) for _ in range(9)]
    ptrs = sun.WeightPtrs()
    ptrs.embed = ptrs.gf = ptrs.wlm = FAKE
    for k, a in zip(sun.LAYER_KEYS, arrs):
        setattr(ptrs, k, C.cast(a, C.POINTER(C.c_void_p)))
    out = C.c_void_p()
    rc = lib.sun_weights_create(C.byref(cfg), C.byref(ptrs), None, 0, None, C.byref(out))
    return rc, out, (arrs, ptrs)


def test_weights_create_errors_and_sizes(lib):
    cfg = sun.make_cfg(wl.TINY, "f32")
    rc, w, keep = _f32_weights(lib, cfg, wl.TINY)
    assert rc == 0 and w.value
    lib.sun_weights_destroy(w)
    ptrs = keep[1]
    ptrs.wlm = None
    out = C.c_void_p()
    assert lib.sun_weights_create(C.byref(cfg), C.byref(ptrs), None, 0, None, C.byref(out)) == 1
    # bf16 needs pack memory
    cfg_b = sun.make_cfg(wl.SMALL128, "bf16")
    assert lib.sun_weights_pack_bytes(C.byref(cfg_b)) == 2 * (wl.SMALL128.body_params + wl.SMALL128.vocab * wl.SMALL128.hidden)
    rc, _, _ = _f32_weights(lib, cfg_b, wl.SMALL128)
    assert rc == 1
    cfg8 = sun.make_cfg(wl.LLAMA_8B, "bf16")
    assert lib.sun_weights_pack_bytes(C.byref(cfg8)) == 2 * (wl.LLAMA_8B.body_params + 128256 * 4096)
    qb = lib.sun_qweights_pack_bytes(C.byref(cfg8), 128)
    assert qb == int(wl.LLAMA_8B.body_params * 0.53125) + 2 * 128256 * 4096      # 4 bits + fp16 scale and zero per 128
    assert lib.sun_qweights_pack_bytes(C.byref(cfg8), 64) == 0
    # quantised tables (fp32 activations: nothing is packed, so fake device pointers are only stored): zero points
    # for every matrix or for none
    cfg_q = sun.make_cfg(wl.TINY_Q, "f32")
    nl = wl.TINY_Q.n_layers

    def qcreate(z_of):
        qp = sun.QWeightPtrs()
        arrs = []
        qp.embed, qp.gf, qp.wlm = FAKE, FAKE, FAKE
        for k in ("g1", "g2"):
            a = (C.c_void_p * nl)(*[FAKE] * nl)
            arrs.append(a)
            setattr(qp, k, C.cast(a, C.POINTER(C.c_void_p)))
        for k in sun.QUANT_KEYS:
            a = (sun.QMat * nl)(*[sun.QMat(FAKE, FAKE, z_of(k, l)) for l in range(nl)])
            arrs.append(a)
            setattr(qp, k, C.cast(a, C.POINTER(sun.QMat)))
        out = C.c_void_p()
        rc = lib.sun_qweights_create(C.byref(cfg_q), C.byref(qp), 128, None, 0, None, C.byref(out))
        if rc == 0:
            lib.sun_weights_destroy(out)
        return rc

    assert qcreate(lambda k, l: FAKE) == 0 and qcreate(lambda k, l: None) == 0
    assert qcreate(lambda k, l: None if (k, l) == ("wo", 1) else FAKE) == 1 and b"zero points" in lib.sun_last_error()


def test_step_rejects_bad_arguments_before_enqueueing(lib):
    cfg = sun.make_cfg(wl.TINY, "f32")
    rc, pool = _pool(lib, cfg)
    assert rc == 0
    rc, w, keep = _f32_weights(lib, cfg, wl.TINY)
    assert rc == 0
    need = lib.sun_workspace_bytes(C.byref(cfg), 8, 9)
    assert need > 0 and lib.sun_workspace_bytes(C.byref(cfg), 0, 9) == 0

    def step(fn=lib.sun_decode_step, pool=pool, w=w, batch=8, tok=FAKE, pt=FAKE, mp=9, lens=FAKE, ids=FAKE, nxt=FAKE,
             ws=FAKE, wsb=need):
        return fn(pool, w, batch, tok, pt, mp, lens, None, ids, None, nxt, ws, wsb, None, 0)

    assert step(pool=None) == 1 and step(w=None) == 1
    assert step(tok=None) == 1 and step(pt=None) == 1 and step(lens=None) == 1 and step(ids=None) == 1
    assert step(nxt=None) == 1 and step(ws=None) == 1
    assert step(batch=0) == 2 and step(batch=257) == 2 and step(mp=0) == 2
    assert step(wsb=need - 1) == 4 and b"workspace" in lib.sun_last_error()
    assert step(ws=FAKE + 8) == 4
    assert step(fn=lib.sun_qdecode_step) == 2          # dense weights handed to the QSUN entry point

    def run(pool=pool, w=w, batch=8, steps=3, tok=FAKE, head=FAKE, status=FAKE, out=FAKE, free=FAKE, n_free=4, wsb=need):
        return lib.sun_decode_run(pool, w, batch, steps, tok, FAKE, 9, FAKE, FAKE, free, n_free, head, status, out, None,
                                  FAKE, wsb, None, 0)

    assert run(pool=None) == 1 and run(w=None) == 1 and run(head=None) == 1 and run(status=None) == 1
    assert run(out=None) == 1 and run(free=None) == 1
    assert run(steps=0) == 2 and run(batch=0) == 2 and run(n_free=-1) == 1
    assert run(wsb=need - 1) == 4 and run(tok=None) == 1
    pneed = lib.sun_prefill_workspace_bytes(C.byref(cfg), 40, 9)
    assert pneed > lib.sun_workspace_bytes(C.byref(cfg), 40, 9) and lib.sun_prefill_workspace_bytes(C.byref(cfg), 0, 9) == 0

    def prefill(pool=pool, w=w, n=40, tok=FAKE, pt=FAKE, mp=9, first=0, mid=0, ws=FAKE, wsb=pneed):
        return lib.sun_prefill(pool, w, n, tok, pt, mp, first, mid, None, None, ws, wsb, None, 0)

    assert prefill(pool=None) == 1 and prefill(w=None) == 1 and prefill(tok=None) == 1 and prefill(pt=None) == 1
    assert prefill(ws=None) == 1 and prefill(mid=-1) == 7 and prefill(mid=3) == 7
    assert prefill(n=0) == 6 and prefill(first=-1) == 6 and prefill(first=9 * 16 - 39) == 6   # last position needs a 10th page
    assert prefill(wsb=pneed - 1) == 4 and prefill(ws=FAKE + 8) == 4
    sneed = lib.sun_serve_workspace_bytes(C.byref(cfg), 8, 9)
    assert sneed > need

    def serve(pool=pool, w=w, slots=8, mp=9, steps=2, wsb=sneed, ws=FAKE, out=FAKE, **fields):
        st = sun.ServeState()
        for name, _ in sun.ServeState._fields_[:14]:
            setattr(st, name, FAKE)
        st.n_wait, st.ring_cap, st.idle_page, st.eos_id = 3, 16, 0, -1
        for k, v in fields.items():
            setattr(st, k, v)
        return lib.sun_decode_serve(pool, w, slots, mp, steps, C.byref(st), out, FAKE, None, ws, wsb, None, 0)

    assert serve(pool=None) == 1 and serve(w=None) == 1 and serve(out=None) == 1 and serve(ws=None) == 1
    assert serve(ring=None) == 1 and serve(counters=None) == 1 and serve(slot_left=None) == 1 and serve(w_budget=None) == 1
    assert lib.sun_decode_serve(pool, w, 8, 9, 2, None, FAKE, FAKE, None, FAKE, sneed, None, 0) == 1
    assert serve(slots=0) == 2 and serve(slots=257) == 2 and serve(steps=0) == 2 and serve(n_wait=-1) == 2
    assert serve(ring_cap=0) == 2 and serve(wsb=sneed - 1) == 4 and serve(ws=FAKE + 8) == 4
    other = sun.make_cfg(wl.TINY_Q, "f32")
    rc, pool2 = _pool(lib, other)
    assert rc == 0 and step(pool=pool2) == 2           # pool and weights of different shapes
    assert prefill(pool=pool2) == 2 and serve(pool=pool2) == 2
    lib.sun_kv_pool_destroy(pool2)
    lib.sun_weights_destroy(w)
    lib.sun_kv_pool_destroy(pool)


def test_single_op_argument_checks(lib):
    cfg = sun.make_cfg(wl.TINY, "f32")
    rc, pool = _pool(lib, cfg)
    ing = lib.sun_kv_pool_ingest
    assert ing(None, 0, FAKE, FAKE, 4, 0, FAKE, 2, None, 0) == 1 and ing(pool, 0, None, FAKE, 4, 0, FAKE, 2, None, 0) == 1
    assert ing(pool, 0, FAKE, FAKE, 4, 0, None, 2, None, 0) == 1
    assert ing(pool, -1, FAKE, FAKE, 4, 0, FAKE, 2, None, 0) == 7 and ing(pool, 99, FAKE, FAKE, 4, 0, FAKE, 2, None, 0) == 7
    assert ing(pool, 0, FAKE, FAKE, 0, 0, FAKE, 2, None, 0) == 6 and ing(pool, 0, FAKE, FAKE, 4, -1, FAKE, 2, None, 0) == 6
    assert ing(pool, 0, FAKE, FAKE, 4, 30, FAKE, 2, None, 0) == 6      # positions 30..33 need a third table entry
    assert ing(pool, 0, FAKE + 2, FAKE, 4, 0, FAKE, 2, None, 0) == 2   # misaligned source
    n = C.c_int64(-1)
    assert lib.sun_kv_pool_model_tokens(pool, 0, C.byref(n)) == 0 and n.value == 0
    assert lib.sun_kv_pool_model_tokens(pool, 0, None) == 1 and lib.sun_kv_pool_model_tokens(pool, 7, C.byref(n)) == 7
    assert lib.sun_paged_attention(pool, 5, 1, FAKE, FAKE, 4, FAKE, None, FAKE, FAKE, 1 << 30, None) == 2
    assert lib.sun_paged_attention(pool, 0, 1, None, FAKE, 4, FAKE, None, FAKE, FAKE, 1 << 30, None) == 1
    assert lib.sun_paged_attention(pool, 0, 1, FAKE, FAKE, 4, FAKE, None, FAKE, FAKE, 16, None) == 4
    # the attention entry point that allocates nothing: same checks, and the size limit before any launch
    st = lib.sun_paged_attention_static
    assert st(None, 0, 1, FAKE, FAKE, 4, FAKE, None, FAKE, None) == 1 and st(pool, 0, 1, None, FAKE, 4, FAKE, None, FAKE, None) == 1
    assert st(pool, 5, 1, FAKE, FAKE, 4, FAKE, None, FAKE, None) == 2 and st(pool, 0, 0, FAKE, FAKE, 4, FAKE, None, FAKE, None) == 2
    limit = lib.sun_paged_attention_static_limit()
    assert limit == 16 << 20 and 0 < lib.sun_paged_attention_static_bytes(C.byref(cfg), 8, 8) < limit
    assert lib.sun_paged_attention_static_bytes(C.byref(cfg), 1024, 1 << 16) > limit
    assert lib.sun_paged_attention_static_bytes(None, 8, 8) == 0 and lib.sun_paged_attention_static_bytes(C.byref(cfg), 0, 8) == 0
    assert st(pool, 0, 1024, FAKE, FAKE, 1 << 16, FAKE, None, FAKE, None) == 4
    assert b"scratch" in lib.sun_last_error()
    # the read probe
    pr = lib.sun_hbm_read_probe
    assert pr(None, 1 << 20, 4096, None, 256, 0, FAKE, None) == 1 and pr(FAKE, 1 << 20, 4096, None, 256, 1, None, None) == 1
    assert pr(FAKE, 1 << 20, 1000, None, 256, 0, FAKE, None) == 2 and pr(FAKE, 1 << 20, 0, None, 256, 0, FAKE, None) == 2
    assert pr(FAKE, 1024, 4096, None, 256, 0, FAKE, None) == 2 and pr(FAKE, 1 << 20, 4096, None, 0, 0, FAKE, None) == 2
    assert pr(FAKE + 8, 1 << 20, 4096, None, 256, 1, FAKE, None) == 2
    assert lib.sun_quantize_w4(FAKE, 0, 4, 256, 64, 0, FAKE, FAKE, FAKE, None) == 2
    assert lib.sun_quantize_w4(FAKE, 0, 4, 200, 128, 0, FAKE, FAKE, FAKE, None) == 2
    assert lib.sun_quantize_w4(None, 0, 4, 256, 128, 0, FAKE, FAKE, FAKE, None) == 1
    lib.sun_kv_pool_destroy(pool)


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(sun, "_lib", None)
    monkeypatch.setattr(sun, "LIB_PATH", "/nonexistent/libsun.so")
    with pytest.raises(FileNotFoundError):
        sun.lib()
