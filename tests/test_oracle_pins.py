"""Pins of the CPU oracle against things other than itself (CPU only).

Each test names what fixes the expected value: a library routine of torch/numpy
on a special case, a closed form, an identity from the paper (Eq. 1 == Eq. 2+3
when prefill and decode share parameters; Eq. 4 cache concatenation), or brute
force on a tiny input.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from helpers import MiniShape, random_weights

PT = 16


def _pool_for(orc, shape, n_pages, rng=None, fill=True):
    n = orc.pool_elems(shape, n_pages, PT)
    if fill and rng is not None:
        vals = rng.normal(size=n)
        base = orc.bf16_bits(vals) if n < 200000 else _fast_bf16(vals)
    else:
        base = np.zeros(n, dtype=np.uint16)
    return base, orc.make_pool(base, n_pages, PT, orc.default_strides(shape, n_pages, PT))


def _fast_bf16(vals):
    t = torch.from_numpy(np.asarray(vals, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


# --------------------------------------------------------------------------
# library-built causal forward (Eq. 1) in float64 torch
# --------------------------------------------------------------------------

def _rope_complex(x, pos, base):
    """Rotation written as a complex product: (x_j + i x_{j+d/2}) * exp(i pos theta_j).
    cos/sin are rounded to float32 as the oracle's reading prescribes."""
    d = x.shape[-1]
    j = torch.arange(d // 2, dtype=torch.float64)
    theta = torch.tensor(base, dtype=torch.float64) ** (-2.0 * j / d)
    ang = pos.to(torch.float64)[:, None] * theta[None, :]
    rot = torch.complex(torch.cos(ang).float().double(), torch.sin(ang).float().double())
    z = torch.complex(x[..., : d // 2], x[..., d // 2:])
    z = z * rot[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def torch_causal_forward(shape, w, tokens, act_bf16=False):
    """tokens: list of ints. Returns logits [T, V] (float64) using only torch library ops.
    act_bf16: the input of every projection is rounded to bfloat16 by torch's own conversion."""
    rb = (lambda t: t.to(torch.bfloat16).to(torch.float64)) if act_bf16 else (lambda t: t)
    tw = {k: ([torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in v] if isinstance(v, list)
              else torch.from_numpy(np.asarray(v, dtype=np.float64))) for k, v in w.items()}
    T = len(tokens)
    Hq, Hkv, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = tw["embed"][torch.tensor(tokens, dtype=torch.long)]
    pos = torch.arange(T)
    for l in range(shape.n_layers):
        h = rb(F.rms_norm(x, (shape.hidden,), tw["g1"][l], eps=shape.rms_eps))
        q = F.linear(h, tw["wq"][l]).view(T, Hq, d)
        k = F.linear(h, tw["wk"][l]).view(T, Hkv, d)
        v = F.linear(h, tw["wv"][l]).view(T, Hkv, d)
        q, k = _rope_complex(q, pos, shape.rope_base), _rope_complex(k, pos, shape.rope_base)
        kr = k.repeat_interleave(Hq // Hkv, dim=1)
        vr = v.repeat_interleave(Hq // Hkv, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kr.transpose(0, 1)[None],
                                           vr.transpose(0, 1)[None], is_causal=True)[0]
        a = rb(a.transpose(0, 1).reshape(T, Hq * d))
        x = x + F.linear(a, tw["wo"][l])
        h = rb(F.rms_norm(x, (shape.hidden,), tw["g2"][l], eps=shape.rms_eps))
        x = x + F.linear(rb(F.silu(F.linear(h, tw["wg"][l])) * F.linear(h, tw["wu"][l])), tw["wd"][l])
    h = rb(F.rms_norm(x, (shape.hidden,), tw["gf"], eps=shape.rms_eps))
    return F.linear(h, tw["wlm"]).numpy()


@pytest.mark.parametrize("shape", [MiniShape(), MiniShape(n_layers=1, n_q_heads=2, n_kv_heads=2),
                                   MiniShape(n_layers=3, hidden=40, n_q_heads=6, n_kv_heads=2, head_dim=4, ffn=56)])
def test_full_forward_equals_torch_library_forward(orc, shape):
    """Eq. 1 evaluated by the oracle's brute-force routine == the same network
    assembled from torch's rms_norm / linear / scaled_dot_product_attention /
    silu and a complex-number rotary."""
    rng = np.random.default_rng(11)
    w = random_weights(shape, rng)
    toks = rng.integers(0, shape.vocab, size=21).tolist()
    got = orc.full_forward(orc.make_cfg(shape), orc.params_from_arrays(w), toks)
    want = torch_causal_forward(shape, w, toks)
    assert np.abs(got - want).max() < 1e-10
    assert np.abs(want).max() > 0.05  # not a vacuous comparison


def test_sixteen_bit_configuration_rounds_projection_inputs(orc):
    """16-bit configuration: the vectors fed to the projections are bf16 values.  Pinned to the
    torch-library forward with torch's own bfloat16 conversion at the same five places, through
    the brute-force forward and through prefill + contiguous decode."""
    shape = MiniShape()
    rng = np.random.default_rng(31)
    w = random_weights(shape, rng)
    toks = rng.integers(0, shape.vocab, size=19)
    cfg, params = orc.make_cfg(shape, act_bf16=True), orc.params_from_arrays(w)
    want = torch_causal_forward(shape, w, toks.tolist(), act_bf16=True)
    got = orc.full_forward(cfg, params, toks)
    assert np.abs(got - want).max() < 1e-10
    plain = orc.full_forward(orc.make_cfg(shape), params, toks)
    assert 1e-5 < np.abs(got - plain).max() < 0.3        # the rounding is really applied, and is small
    L = len(toks) - 1
    _, K, V = orc.full_forward(cfg, params, toks[:L], want_kv=True)
    Kc = np.zeros((shape.n_layers, L + 1, shape.n_kv_heads, shape.head_dim))
    Vc = np.zeros_like(Kc)
    Kc[:, :L], Vc[:, :L] = K, V
    logits, _ = orc.decode_contig_f64(cfg, params, int(toks[L]), L, Kc, Vc)
    assert np.abs(logits - want[-1]).max() < 1e-10


@pytest.mark.parametrize("L", [0, 1, 15, 16, 17, 37])
def test_prefill_then_decode_equals_full_forward(orc, L):
    """Eq. 2+3 with theta_p = theta_d is the same function as Eq. 1: prefill the
    first L tokens (full forward capturing K/V), decode token L at position L."""
    shape = MiniShape()
    rng = np.random.default_rng(100 + L)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    toks = rng.integers(0, shape.vocab, size=L + 1)
    want = torch_causal_forward(shape, w, toks.tolist())[-1]
    cap = L + 1
    Kc = np.zeros((shape.n_layers, cap, shape.n_kv_heads, shape.head_dim))
    Vc = np.zeros_like(Kc)
    if L > 0:
        _, K, V = orc.full_forward(cfg, params, toks[:L], want_kv=True)
        Kc[:, :L], Vc[:, :L] = K, V
    logits, nxt = orc.decode_contig_f64(cfg, params, int(toks[L]), L, Kc, Vc)
    assert np.abs(logits - want).max() < 1e-10
    assert nxt == int(np.argmax(want))


def _prefill_into_pool(orc, shape, cfg, params, toks, n_pages, table, rng):
    """Full forward with bf16-rounded K/V; scatter K/V of toks into pool pages of `table`."""
    base, pool = _pool_for(orc, shape, n_pages, rng)
    st = orc.default_strides(shape, n_pages, PT)
    if len(toks):
        _, K, V = orc.full_forward(cfg, params, toks, round_kv=True, want_kv=True)
        kb, vb = orc.bf16_bits(K), orc.bf16_bits(V)
        assert np.array_equal(orc.bf16_values(kb), K)  # already on the bf16 grid
        orc.kv_ingest(base, st, kb, vb, 0, table, PT)
    return base, pool


@pytest.mark.parametrize("L", [0, 5, 15, 16, 31, 33])
@pytest.mark.parametrize("mode", [0, 1])
def test_paged_decode_step_equals_full_forward_with_bf16_cache(orc, L, mode):
    """Same identity through the paged bf16 pool: a causal forward whose K/V are
    rounded to bf16 must equal prefill-into-pages + one paged decode step; two
    chained steps must equal the forward over L+2 tokens (Eq. 4)."""
    shape = MiniShape()
    rng = np.random.default_rng(200 + L)
    w = random_weights(shape, rng)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    toks = rng.integers(0, shape.vocab, size=L + 2)
    n_pages = 9
    table = rng.permutation(n_pages)[: (L + 2 + PT - 1) // PT + 1].astype(np.int32)
    base, pool = _prefill_into_pool(orc, shape, cfg, params, toks[:L], n_pages, table, rng)
    want = orc.full_forward(cfg, params, toks, round_kv=True)
    ids = np.zeros(1, np.int32)
    r1 = orc.decode_step(cfg, params, pool, toks[L:L + 1], table[None], [L], ids, mode=mode)
    assert np.abs(r1["logits"][0] - want[L]).max() < 1e-10
    r2 = orc.decode_step(cfg, params, pool, toks[L + 1:L + 2], table[None], [L + 1], ids, mode=mode)
    assert np.abs(r2["logits"][0] - want[L + 1]).max() < 1e-10
    # and the library-built forward agrees when nothing is rounded (sanity of the flag)
    lib = torch_causal_forward(shape, w, toks.tolist())
    assert np.abs(want - lib).max() < 0.2 and np.abs(want - lib).max() > 0  # rounding changes it, slightly


# --------------------------------------------------------------------------
# paged == contiguous, append, softmax rows, batch-mix invariance
# --------------------------------------------------------------------------

def _random_batch(orc, shape, rng, lens, n_models=3, spare=3):
    lens = np.asarray(lens, dtype=np.int32)
    need = (lens.astype(np.int64) + 1 + PT - 1) // PT
    n_pages = int(need.sum()) + spare
    perm = rng.permutation(n_pages)
    tables = np.full((len(lens), int(need.max()) + 1), -1, np.int32)
    o = 0
    for i, n in enumerate(need):
        tables[i, :n] = perm[o:o + n]
        o += int(n)
    base, pool = _pool_for(orc, shape, n_pages, rng)
    toks = rng.integers(0, shape.vocab, size=len(lens)).astype(np.int32)
    ids = rng.integers(0, n_models, size=len(lens)).astype(np.int32)
    return dict(base=base, pool=pool, tables=tables, toks=toks, ids=ids, lens=lens, n_pages=n_pages)


def test_paged_equals_contiguous_bitwise(orc):
    shape = MiniShape()
    rng = np.random.default_rng(5)
    w = random_weights(shape, rng, dtype=np.float32)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    lens = [0, 1, 15, 16, 17, 31, 32, 47, 63, 100]
    b = _random_batch(orc, shape, rng, lens)
    base0 = b["base"].copy()
    r0 = orc.decode_step(cfg, params, b["pool"], b["toks"], b["tables"], b["lens"], b["ids"], mode=0)
    after0 = b["base"].copy()
    b["base"][:] = base0
    r1 = orc.decode_step(cfg, params, b["pool"], b["toks"], b["tables"], b["lens"], b["ids"], mode=1)
    assert np.array_equal(r0["logits"], r1["logits"])
    assert np.array_equal(r0["next"], r1["next"])
    assert np.array_equal(after0, b["base"])


def test_append_touches_exactly_the_predicted_slots(orc):
    """Eq. 4: after the step the pool differs from before only in slot L_i of the
    tail page of each request, for every layer and both K and V."""
    shape = MiniShape()
    rng = np.random.default_rng(6)
    w = random_weights(shape, rng, dtype=np.float32)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    lens = [3, 15, 16, 40]
    b = _random_batch(orc, shape, rng, lens)
    before = b["base"].copy()
    orc.decode_step(cfg, params, b["pool"], b["toks"], b["tables"], b["lens"], b["ids"])
    st = orc.default_strides(shape, b["n_pages"], PT)
    allowed = np.zeros(before.shape, dtype=bool)
    for i, L in enumerate(lens):
        page, slot = int(b["tables"][i, L // PT]), L % PT
        for l in range(shape.n_layers):
            for h in range(shape.n_kv_heads):
                o = l * st["k_layer"] + page * st["k_page"] + h * st["k_head"] + slot * st["k_token"]
                allowed[st["k_off"] + o: st["k_off"] + o + shape.head_dim] = True
                allowed[st["v_off"] + o: st["v_off"] + o + shape.head_dim] = True
    changed = before != b["base"]
    assert allowed.sum() == len(lens) * shape.n_layers * 2 * shape.n_kv_heads * shape.head_dim
    assert not np.any(changed & ~allowed)
    assert changed[allowed].mean() > 0.95  # random values: nearly every allowed element differs


def test_softmax_rows_sum_to_one_and_single_key_returns_value(orc):
    shape = MiniShape()
    rng = np.random.default_rng(7)
    w = random_weights(shape, rng, dtype=np.float32)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    b = _random_batch(orc, shape, rng, [0, 7, 64, 129])
    r = orc.decode_step(cfg, params, b["pool"], b["toks"], b["tables"], b["lens"], b["ids"],
                        want_rowsums=True, want_attn=True)
    assert np.abs(r["rowsums"] - 1.0).max() < 1e-12
    # request 0 has L = 0: one key, so the attention output is the (rounded) new V itself
    st = orc.default_strides(shape, b["n_pages"], PT)
    page = int(b["tables"][0, 0])
    G = shape.n_q_heads // shape.n_kv_heads
    for l in range(shape.n_layers):
        for h in range(shape.n_q_heads):
            o = st["v_off"] + l * st["v_layer"] + page * st["v_page"] + (h // G) * st["v_head"]
            v0 = orc.bf16_values(b["base"][o:o + shape.head_dim])
            assert np.array_equal(r["attn"][0, l, h * shape.head_dim:(h + 1) * shape.head_dim], v0)


def test_output_is_invariant_to_batch_mates_and_model_ids(orc):
    """The property SUN relies on (Section 3.2.1): decode parameters are the same for
    every task, so a request's result cannot depend on its own or its batch-mates'
    source-model ids, nor on which other requests share the batch."""
    shape = MiniShape()
    rng = np.random.default_rng(8)
    w = random_weights(shape, rng, dtype=np.float32)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    b = _random_batch(orc, shape, rng, [20, 33, 5, 64, 17])
    base0 = b["base"].copy()
    full = orc.decode_step(cfg, params, b["pool"], b["toks"], b["tables"], b["lens"], b["ids"])
    for i in range(len(b["lens"])):
        b["base"][:] = base0
        alone = orc.decode_step(cfg, params, b["pool"], b["toks"][i:i + 1], b["tables"][i:i + 1],
                                b["lens"][i:i + 1], np.array([2 - b["ids"][i]], np.int32))
        assert np.array_equal(alone["logits"][0], full["logits"][i])
        assert alone["next"][0] == full["next"][i]
    # relabel ids, reverse order
    b["base"][:] = base0
    rev = orc.decode_step(cfg, params, b["pool"], b["toks"][::-1], b["tables"][::-1], b["lens"][::-1],
                          (b["ids"][::-1] + 1) % 3)
    assert np.array_equal(rev["logits"][::-1], full["logits"])


def test_page_out_of_range_and_bad_token_are_rejected(orc):
    shape = MiniShape()
    rng = np.random.default_rng(9)
    w = random_weights(shape, rng, dtype=np.float32)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    b = _random_batch(orc, shape, rng, [20])
    bad = b["tables"].copy()
    bad[0, 1] = b["n_pages"]
    with pytest.raises(ValueError):
        orc.decode_step(cfg, params, b["pool"], b["toks"], bad, b["lens"], b["ids"])
    bad[0, 1] = -1
    with pytest.raises(ValueError):
        orc.decode_step(cfg, params, b["pool"], b["toks"], bad, b["lens"], b["ids"])
    with pytest.raises(ValueError):
        orc.decode_step(cfg, params, b["pool"], [shape.vocab], b["tables"], b["lens"], b["ids"])


# --------------------------------------------------------------------------
# single operations against library routines / closed forms
# --------------------------------------------------------------------------

def test_attention_special_case_equals_torch_sdpa(orc):
    """G = 1, one page: paged attention is softmax(q K^T / sqrt d) V."""
    shape = MiniShape(n_layers=1, n_q_heads=3, n_kv_heads=3, head_dim=16)
    rng = np.random.default_rng(10)
    n_pages, n = 4, 16
    base, pool = _pool_for(orc, shape, n_pages, rng)
    st = orc.default_strides(shape, n_pages, PT)
    page = 2
    q = rng.normal(size=shape.n_q_heads * shape.head_dim)
    a, rs = orc.attention_paged(orc.make_cfg(shape), pool, 0, np.array([page], np.int32), q, n)
    d = shape.head_dim
    K = np.stack([orc.bf16_values(base[st["k_off"] + page * st["k_page"] + h * st["k_head"]:][: n * d]).reshape(n, d)
                  for h in range(3)])
    V = np.stack([orc.bf16_values(base[st["v_off"] + page * st["v_page"] + h * st["v_head"]:][: n * d]).reshape(n, d)
                  for h in range(3)])
    want = F.scaled_dot_product_attention(torch.from_numpy(q.reshape(3, 1, d))[None], torch.from_numpy(K)[None],
                                          torch.from_numpy(V)[None])[0, :, 0].numpy().ravel()
    assert np.abs(a - want).max() < 1e-12
    assert np.abs(rs - 1).max() < 1e-12


def test_gqa_head_mapping_by_brute_force(orc):
    """Query head h reads KV head h // G (checked with a hand-rolled loop, G = 3)."""
    shape = MiniShape(n_layers=2, n_q_heads=6, n_kv_heads=2, head_dim=4)
    rng = np.random.default_rng(12)
    n_pages = 5
    base, pool = _pool_for(orc, shape, n_pages, rng)
    st = orc.default_strides(shape, n_pages, PT)
    pt = np.array([3, 0, 4], np.int32)
    n, d, layer = 35, 4, 1
    q = rng.normal(size=6 * d)
    a, _ = orc.attention_paged(orc.make_cfg(shape), pool, layer, pt, q, n)
    for h in range(6):
        kvh = h // 3
        s = np.empty(n)
        vals = np.empty((n, d))
        for t in range(n):
            o = layer * st["k_layer"] + int(pt[t // PT]) * st["k_page"] + kvh * st["k_head"] + (t % PT) * st["k_token"]
            s[t] = q[h * d:(h + 1) * d] @ orc.bf16_values(base[st["k_off"] + o: st["k_off"] + o + d]) / 2.0
            vals[t] = orc.bf16_values(base[st["v_off"] + o: st["v_off"] + o + d])
        p = np.exp(s - s.max())
        p /= p.sum()
        assert np.abs(a[h * d:(h + 1) * d] - p @ vals).max() < 1e-12


def test_rmsnorm_closed_form_and_library(orc):
    g = np.linspace(0.5, 1.5, 24)
    c, eps = 3.0, 1e-5
    got = orc.rmsnorm(np.full(24, c), g, eps)
    assert np.abs(got - g * c / math.sqrt(c * c + eps)).max() < 1e-14
    x = np.random.default_rng(1).normal(size=24)
    want = F.rms_norm(torch.from_numpy(x), (24,), torch.from_numpy(g), eps=eps).numpy()
    assert np.abs(orc.rmsnorm(x, g, eps) - want).max() < 1e-14


def test_rope_properties(orc):
    rng = np.random.default_rng(2)
    d, base = 16, 10000.0
    u, v = rng.normal(size=d), rng.normal(size=d)
    assert np.array_equal(orc.rope(u, 0, base), u)                       # identity at position 0
    r = orc.rope(u, 1234, base)
    assert np.abs((r[:8] ** 2 + r[8:] ** 2) - (u[:8] ** 2 + u[8:] ** 2)).max() < 1e-6  # per-pair norm
    dots = [orc.rope(u, m, base) @ orc.rope(v, m - 7, base) for m in (7, 50, 900)]
    assert max(dots) - min(dots) < 1e-5                                   # depends on m - n only
    # explicit angles: pair j rotates by pos * base^(-2j/d), counter-clockwise
    pos = 3
    for j in range(8):
        ang = pos * base ** (-2.0 * j / d)
        want = (u[j] * math.cos(ang) - u[j + 8] * math.sin(ang), u[j + 8] * math.cos(ang) + u[j] * math.sin(ang))
        got = orc.rope(u, pos, base)
        assert abs(got[j] - want[0]) < 1e-6 and abs(got[j + 8] - want[1]) < 1e-6
    # first pair has theta = 1: position pi/2-ish check of the sign convention
    e = np.zeros(d)
    e[0] = 1.0
    r = orc.rope(e, 1, base)
    assert abs(r[0] - math.cos(1.0)) < 1e-7 and abs(r[8] - math.sin(1.0)) < 1e-7


def test_silu_linear_argmax(orc):
    assert orc.silu(0.0) == 0.0
    for z in (-3.0, -0.5, 0.7, 4.0):
        assert abs(orc.silu(z) - float(F.silu(torch.tensor(z, dtype=torch.float64)))) < 1e-15
    rng = np.random.default_rng(3)
    W, X = rng.normal(size=(7, 13)), rng.normal(size=(3, 13))
    assert np.abs(orc.linear(orc.dense_mat(np.ascontiguousarray(W)), X) - X @ W.T).max() < 1e-13
    W32 = np.ascontiguousarray(W.astype(np.float32))
    assert np.abs(orc.linear(orc.dense_mat(W32), X) - X @ W32.astype(np.float64).T).max() < 1e-13
    assert orc.argmax(np.array([1.0, 5.0, 5.0, 2.0, 5.0])) == 1            # lowest index on ties
    assert orc.argmax(np.array([-1.0, -1.0])) == 0


def test_number_formats_against_numpy_and_torch(orc):
    rng = np.random.default_rng(4)
    xs = np.concatenate([rng.normal(size=2000), rng.normal(size=500) * 1e-3, [0.0, -0.0, 1.0, 65504.0, 1e-8, 6e-5, 3e-5]])
    xs32 = xs.astype(np.float32)
    L = orc.lib()
    half_got = np.array([L.orc_float_to_half(float(v)) for v in xs32], dtype=np.uint16)
    assert np.array_equal(half_got, xs32.astype(np.float16).view(np.uint16))
    back = np.array([L.orc_half_to_float(int(h)) for h in half_got], dtype=np.float32)
    assert np.array_equal(back, half_got.view(np.float16).astype(np.float32))
    # bf16: on float32 inputs, torch's conversion is round-to-nearest-even
    want = torch.from_numpy(xs32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.bf16_bits(xs32.astype(np.float64)), want)
    # ties and a double that float32 double-rounding would get wrong
    one_ulp = 2.0 ** -7
    assert orc.bf16_values(orc.bf16_bits(np.array([1.0 + one_ulp / 2])))[0] == 1.0            # tie -> even
    assert orc.bf16_values(orc.bf16_bits(np.array([1.0 + 3 * one_ulp / 2])))[0] == 1.0 + 2 * one_ulp
    assert orc.bf16_values(orc.bf16_bits(np.array([1.0 + one_ulp / 2 + 2.0 ** -40])))[0] == 1.0 + one_ulp


def test_bf16_and_f32_weights_are_read_at_stored_value(orc):
    rng = np.random.default_rng(13)
    W = rng.normal(size=(5, 8)).astype(np.float32)
    bits = _fast_bf16(W)
    X = rng.normal(size=(2, 8))
    want = X @ orc.bf16_values(bits).reshape(5, 8).T
    assert np.abs(orc.linear(orc.dense_mat(bits.reshape(5, 8)), X) - want).max() < 1e-14


def test_step_next_to_a_peer_cache_adopts_valid_neighbours_only(orc):
    """decode_step_peer: the step stores, and attends over, the peer's bf16 code where that code is its own
    rounding, the neighbouring value, or within the given bound of it; its own rounding otherwise.
    Pinned by (a) a peer that is the plain step's own cache (nothing changes, logits bit-identical),
    (b) a one-layer model whose peer entries are nudged: the stored entries follow the rule element by
    element, and the logits equal what the oracle's primitives (norm, projections, rotation, paged attention
    over the pool as stored) give when chained by hand, i.e. attention really read the adopted entries."""
    shape = MiniShape(n_layers=1)
    rng = np.random.default_rng(61)
    w = random_weights(shape, rng, dtype=np.float32)
    cfg, params = orc.make_cfg(shape), orc.params_from_arrays(w)
    lens = [0, 5, 16, 33]
    b = _random_batch(orc, shape, rng, lens)
    before = b["base"].copy()
    plain = orc.decode_step(cfg, params, b["pool"], b["toks"], b["tables"], b["lens"], b["ids"])
    own_after = b["base"].copy()
    written = own_after != before
    st = orc.default_strides(shape, b["n_pages"], PT)
    # (a) the peer is the plain step's result
    b["base"][:] = before
    peer_base = own_after.copy()
    peer = orc.make_pool(peer_base, b["n_pages"], PT, st)
    r = orc.decode_step_peer(cfg, params, b["pool"], peer, b["toks"], b["tables"], b["lens"], b["ids"], tol_abs=0.0)
    n_new = len(lens) * 2 * shape.n_kv_heads * shape.head_dim
    assert r["peer"] == {"equal": n_new, "neighbour": 0, "by_value": 0, "rejected": 0}
    assert np.array_equal(r["logits"], plain["logits"]) and np.array_equal(b["base"], own_after)
    # (b) nudge the peer's new entries: +1 code (neighbour), +3 codes on a large value (rejected), +3 codes on a value
    # tiny enough to be within tol_abs (adopted by value)
    def ordered(u):
        return np.where(u & 0x8000, -(u & 0x7FFF).astype(np.int64), (u & 0x7FFF).astype(np.int64))
    def from_ordered(o):
        return np.where(o < 0, 0x8000 | (-o), o).astype(np.uint16)
    idx = np.flatnonzero(written)
    vals = (own_after[idx].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    rng2 = np.random.default_rng(62)
    pick = rng2.permutation(len(idx))
    nb, far = pick[:40], pick[40:60]
    peer_base[:] = own_after
    peer_base[idx[nb]] = from_ordered(ordered(own_after[idx[nb]]) + rng2.choice([-1, 1], size=len(nb)))
    peer_base[idx[far]] = from_ordered(ordered(own_after[idx[far]]) + 3 * rng2.choice([-1, 1], size=len(far)))
    tol = 1e-3
    far_vals = (peer_base[idx[far]].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    by_value = np.abs(far_vals - vals[far]) <= tol
    assert by_value.any() and (~by_value).any(), "the draw should hold both kinds"
    b["base"][:] = before
    r = orc.decode_step_peer(cfg, params, b["pool"], peer, b["toks"], b["tables"], b["lens"], b["ids"], tol_abs=tol)
    assert r["peer"] == {"equal": n_new - 60, "neighbour": 40, "by_value": int(by_value.sum()), "rejected": int((~by_value).sum())}
    expect = peer_base.copy()
    expect[idx[far[~by_value]]] = own_after[idx[far[~by_value]]]          # rejected: the step's own rounding stays
    assert np.array_equal(b["base"], expect)
    assert not np.array_equal(r["logits"], plain["logits"])
    # the chain by hand over the pool as stored
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    for i, L in enumerate(lens):
        x0 = f64(w["embed"][b["toks"][i]])
        h = orc.rmsnorm(x0, f64(w["g1"][0]), shape.rms_eps)
        q = orc.linear(orc.dense_mat(np.ascontiguousarray(w["wq"][0])), h[None])[0].reshape(shape.n_q_heads, shape.head_dim)
        qr = np.concatenate([orc.rope(q[hh], L, shape.rope_base) for hh in range(shape.n_q_heads)])
        a, _ = orc.attention_paged(cfg, b["pool"], 0, b["tables"][i], qr, L + 1)
        x1 = x0 + orc.linear(orc.dense_mat(np.ascontiguousarray(w["wo"][0])), a[None])[0]
        h2 = orc.rmsnorm(x1, f64(w["g2"][0]), shape.rms_eps)
        gate = orc.linear(orc.dense_mat(np.ascontiguousarray(w["wg"][0])), h2[None])[0]
        up = orc.linear(orc.dense_mat(np.ascontiguousarray(w["wu"][0])), h2[None])[0]
        u = np.array([orc.silu(float(g)) for g in gate]) * up
        x2 = x1 + orc.linear(orc.dense_mat(np.ascontiguousarray(w["wd"][0])), u[None])[0]
        hf = orc.rmsnorm(x2, f64(w["gf"]), shape.rms_eps)
        logits = orc.linear(orc.dense_mat(np.ascontiguousarray(w["wlm"])), hf[None])[0]
        assert np.abs(logits - r["logits"][i]).max() < 1e-11
