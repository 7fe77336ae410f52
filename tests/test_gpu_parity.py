"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on identical
seeded inputs.  fp32 logits: max-abs <= 1e-4.  bf16 / QSUN logits: |g - o| <= 2e-2 + 1e-2 |o|.
Next tokens: exact, except documented near-ties (oracle top-2 gap below twice the tolerance)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2603_02599_amd import binding as sun  # noqa: E402
from paper_2603_02599_amd import workloads as wl  # noqa: E402


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sun.lib()
    return gpu_harness


def _full_step_parity(H, case, rows=None, tol=None):
    from oracle import oracle as orc
    work = case.work
    rows = list(range(work.batch)) if rows is None else list(rows)
    before_host, _, tabs, used = case.extract_pool(rows)
    ref = H.run_oracle(case, rows)
    case.step(flags=sun.SUN_VALIDATE)
    got_logits = case.logits.cpu().numpy()[rows]
    got_next = case.next.cpu().numpy()[rows]
    rep = H.logits_report(got_logits, ref["logits"])
    H.say(f"{work.name}/{work.shape.name}/{work.dtype} B={work.batch} rows={len(rows)} logits {rep}")
    H.check_logits(got_logits, ref["logits"], work.dtype)
    tol = tol if tol is not None else (1e-4 if work.dtype == "f32" else 2e-2)
    near = H.check_next_tokens(got_next, ref["logits"], tol)
    st = H.layout_strides(case.lay)
    st["k_layer"] = st["v_layer"] = len(used) * int(case.lay.k_page)
    mask = H.appended_mask(work.shape, st, before_host.size, tabs, work.seq_lens[rows])
    after = case.pool_pages_now(used)
    if work.dtype != "f32":
        H.say(f"   appended K/V {H.appended_kv_stats(after, ref['pool_after'], mask)}")
    off, total = H.check_appended_kv(after, ref["pool_after"], before_host, mask, work.dtype, quant=case.quant is not None)
    H.say(f"   next-token near-ties {near}; appended K/V elements off by >=1 bf16 ulp: {off} of {total}")
    return rep


# ------------------------------------------------------------------ fp32 parity configuration
def test_cfg1_tiny_fp32_full_step(H):
    H.say("cfg1 tiny fp32")
    case = H.GpuCase(wl.make_workload("cfg1"))
    rep = _full_step_parity(H, case)
    assert rep["ref_std"] > 0.05


@pytest.mark.parametrize("lens", [[0, 1, 15, 16, 17, 31, 32, 62, 63, 64, 127, 128, 255, 256, 257, 510, 511, 512, 600, 767, 768, 1100]])
def test_fp32_edge_lengths(H, lens):
    """Empty cache, page boundaries, small-chunk (64) and full-chunk (256) boundaries of the attention
    work split, the first lengths that get a full chunk (n = L+1 >= 512), multi-chunk requests."""
    H.say(f"fp32 edge lengths {lens}")
    work = wl.make_workload("cfg1", batch=len(lens), seed=77)
    rng = np.random.default_rng(5)
    work.seq_lens = np.array(lens, np.int32)
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    case = H.GpuCase(work)
    _full_step_parity(H, case)


def test_fp32_single_request_and_no_logits_output(H):
    H.say("fp32 batch 1, logits_out NULL")
    work = wl.make_workload("cfg1", batch=1, n_models=1, seed=78)
    case = H.GpuCase(work)
    ref = H.run_oracle(case, [0])
    fn = sun.sun_decode_step
    fn(case.pool, case.weights, case.tokens, case.tables, case.lens, case.ids, None, case.next, case.ws)
    torch.cuda.synchronize()
    assert int(case.next.cpu()[0]) == int(ref["next"][0])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_argmax_ties_take_the_lowest_index(H, dtype):
    """LM head rows 0..99 are -v and all later rows +v: every request's logits are two exact plateaus,
    so greedy decoding must return token 100 (v.h > 0) or token 0 (v.h < 0) on both sides."""
    H.say(f"argmax ties {dtype}")
    shape = wl.TINY if dtype == "f32" else wl.SMALL128
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=16, seed=91)
    w = wl.make_weights(shape, dtype, "cuda", 92)
    v = w["wlm"][0].clone()
    w["wlm"][:100] = -v
    w["wlm"][100:] = v
    case = H.GpuCase(work, weights=w)
    ref = H.run_oracle(case, list(range(work.batch)))
    case.step()
    got = case.next.cpu().numpy()
    lg = case.logits.cpu().numpy()
    assert set(np.unique(ref["next"])) <= {0, 100} and len(set(ref["next"])) == 2, "both plateaus should occur"
    assert np.array_equal(got, ref["next"])
    for i in range(work.batch):  # the plateaus are exact on the GPU as well: identical rows give identical logits
        assert len(np.unique(lg[i, 100:])) == 1 and len(np.unique(lg[i, :100])) == 1


def test_fp32_qsun_tiny(H):
    """QSUN with fp32 activations: tight check of the dequantised projections (1e-4)."""
    for mode in ("asym", "sym", "sym_noz"):
        H.say(f"fp32 QSUN tiny_q {mode}")
        work = wl.make_workload("cfg1", shape=wl.TINY_Q, seed=79)
        case = H.GpuCase(work, quant_mode=mode)
        _full_step_parity(H, case)


# ------------------------------------------------------------------ kernel-level parity
def test_quantiser_matches_oracle_bit_for_bit(H):
    from oracle import oracle as orc
    g = torch.Generator(device=H.DEV).manual_seed(3)
    for dtype in (torch.float32, torch.bfloat16):
        w = (torch.randn((96, 1024), generator=g, device=H.DEV) * 0.02).to(dtype)
        w[0, :128] = 0          # an all-zero group
        w[1, :128] = 0.5        # a constant group
        for mode in ("asym", "sym"):
            H.say(f"quantiser {dtype} {mode}")
            q, s, z = sun.sun_quantize_w4(w, 128, mode)
            torch.cuda.synchronize()
            qo, so, zo = orc.quantize_w4(w.float().cpu().numpy(), 128, mode)
            assert int((H.to_np(q) != qo).sum()) == 0
            assert int((H.to_np(s) != so).sum()) == 0
            assert int((H.to_np(z) != zo).sum()) == 0
            if mode == "sym":       # without stored zero points: same codes and scales, and the grid's zero is 8
                q2, s2, z2 = sun.sun_quantize_w4(w, 128, "sym_noz")
                torch.cuda.synchronize()
                assert z2 is None and torch.equal(q2, q) and torch.equal(s2, s) and (zo == 0x4800).all()


_GQA_SHAPES = [wl.Shape(f"gqa{g}_d128", 1, 256, g, 1, 128, 256, 256) for g in (1, 3, 6, 7, 8)] + \
              [wl.Shape(f"gqa{g}_d64", 1, 256, 2 * g, 2, 64, 256, 256) for g in (1, 3, 8)]


@pytest.mark.parametrize("shape,dtype", [(wl.TINY, "f32"), (wl.SMALL128, "bf16"), (wl.TINY_Q, "bf16")] +
                         [(s, "bf16") for s in _GQA_SHAPES], ids=lambda v: v.name if hasattr(v, "name") else v)
def test_paged_attention_op(H, shape, dtype):
    """Attention sub-step alone against the oracle's paged attention (ragged lengths, shuffled tables)."""
    _attention_op_case(H, shape, dtype, [1, 2, 16, 17, 33, 255, 256, 257, 511, 513, 1000, 31])


@pytest.mark.parametrize("shape,dtype", [(wl.TINY, "f32"), (wl.SMALL128, "bf16")], ids=lambda v: v.name if hasattr(v, "name") else v)
def test_paged_attention_op_more_requests_than_a_step_takes(H, shape, dtype):
    """The attention operation alone takes up to 1024 requests (the step: 256): 700 short ragged ones."""
    rng = np.random.default_rng(90)
    _attention_op_case(H, shape, dtype, [int(v) for v in rng.integers(1, 120, size=700)])


def _attention_op_case(H, shape, dtype, lens):
    from oracle import oracle as orc
    H.say(f"paged attention {shape.name} {dtype}, {len(lens)} requests")
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=len(lens), seed=80)
    rng = np.random.default_rng(6)
    work.seq_lens = np.array(lens, np.int32) - 1
    work.page_tables, work.n_pages = wl.deal_page_tables(work.seq_lens, rng)
    case = H.GpuCase(work)
    B, QD = len(lens), shape.n_q_heads * shape.head_dim
    q = torch.randn((B, QD), device=H.DEV, generator=torch.Generator(device=H.DEV).manual_seed(4)) * 2.0
    n = torch.tensor(lens, dtype=torch.int32, device=H.DEV)
    out = torch.empty_like(q)
    layer = shape.n_layers - 1
    for host in (np.array(lens, np.int32), None):
        out.zero_()
        sun.sun_paged_attention(case.pool, layer, q, case.tables, n, out, case.ws, n_tokens_host=host)
        torch.cuda.synchronize()
        host_pool, pool, tabs, used = case.extract_pool(range(B))
        ocfg = orc.make_cfg(shape)
        worst = 0.0
        for i in range(B):
            a, rs = orc.attention_paged(ocfg, pool, layer, tabs[i], q[i].double().cpu().numpy(), lens[i])
            assert abs(rs - 1).max() < 1e-12
            worst = max(worst, float(np.abs(out[i].double().cpu().numpy() - a).max()))
        H.say(f"   max abs diff {worst:.3e} (host lengths {'given' if host is not None else 'absent'})")
        assert worst < (2e-5 if dtype == "f32" else 2e-4)


@pytest.mark.parametrize("batch", [1, 8, 33, 64, 100, 200, 256])
def test_linear_op_bf16(H, batch):
    """Every projection of the step (stacked QKV, O, fused SwiGLU, down, lm_head) alone."""
    from oracle import oracle as orc
    shape = wl.SMALL128
    H.say(f"linear bf16 batch {batch}")
    cfg = sun.make_cfg(shape, "bf16")
    w = wl.make_weights(shape, "bf16", H.DEV, 11, std=0.05)
    W = sun.sun_weights_create(cfg, w)
    ws = torch.empty(sun.sun_workspace_bytes(cfg, batch, 4), dtype=torch.uint8, device=H.DEV)
    g = torch.Generator(device=H.DEV).manual_seed(batch)
    wn = H.weights_to_np(w)
    for mat, K, N in ((0, 512, 1536), (1, 1024, 512), (2, 512, 1024), (3, 1024, 512), (4, 512, 2048)):
        x = torch.randn((batch, K), device=H.DEV, generator=g)
        out = torch.full((batch, N), float("nan"), device=H.DEV)
        sun.sun_linear(W, 1, mat, x, out, ws)
        torch.cuda.synchronize()
        xr = x.double().cpu().numpy()       # activations enter the matrix cores as hi+lo bf16 (16 significant bits)
        lin = lambda key: orc.linear(orc.dense_mat(wn[key][1] if isinstance(wn[key], list) else wn[key]), xr)
        if mat == 0:
            want = np.concatenate([lin("wq"), lin("wk"), lin("wv")], axis=1)
        elif mat == 2:
            gate, up = lin("wg"), lin("wu")
            want = gate / (1 + np.exp(-gate)) * up
        else:
            want = lin({1: "wo", 3: "wd", 4: "wlm"}[mat])
        got = out.double().cpu().numpy()
        tol = 1e-2 * np.abs(want) + 2e-3 if mat == 2 else 2e-4 + 1e-5 * np.abs(want)   # mat 2 output is bf16
        assert np.all(np.abs(got - want) <= tol), f"mat {mat}: max diff {np.abs(got - want).max():.3e}"


@pytest.mark.parametrize("batch", [8, 64, 130, 256])
def test_linear_op_w4(H, batch):
    from oracle import oracle as orc
    shape = wl.SMALL128
    H.say(f"linear W4 batch {batch}")
    cfg = sun.make_cfg(shape, "bf16")
    w = wl.make_weights(shape, "bf16", H.DEV, 12, std=0.05)
    quant = {k: [sun.sun_quantize_w4(m, 128, "asym") for m in w[k]] for k in sun.QUANT_KEYS}
    W = sun.sun_qweights_create(cfg, w, quant)
    ws = torch.empty(sun.sun_workspace_bytes(cfg, batch, 4), dtype=torch.uint8, device=H.DEV)
    g = torch.Generator(device=H.DEV).manual_seed(100 + batch)

    def qlin(key, xr):
        q, s, z = (H.to_np(t) for t in quant[key][0])
        return orc.linear(orc.w4_mat(q, s, z, w[key][0].shape[1], 128), xr)

    for mat, K, N in ((0, 512, 1536), (1, 1024, 512), (2, 512, 1024), (3, 1024, 512)):
        x = torch.randn((batch, K), device=H.DEV, generator=g)
        out = torch.full((batch, N), float("nan"), device=H.DEV)
        sun.sun_linear(W, 0, mat, x, out, ws)
        torch.cuda.synchronize()
        xr = x.double().cpu().numpy()
        if mat == 0:
            want = np.concatenate([qlin("wq", xr), qlin("wk", xr), qlin("wv", xr)], axis=1)
        elif mat == 2:
            gate, up = qlin("wg", xr), qlin("wu", xr)
            want = gate / (1 + np.exp(-gate)) * up
        else:
            want = qlin({1: "wo", 3: "wd"}[mat], xr)
        got = out.double().cpu().numpy()
        tol = 1e-2 * np.abs(want) + 2e-3 if mat == 2 else 1e-3 + 1e-4 * np.abs(want)
        assert np.all(np.abs(got - want) <= tol), f"mat {mat}: max diff {np.abs(got - want).max():.3e}"


def test_linear_op_w4_fixed_point_bound_with_outliers_and_empty_groups(H):
    """The 4-bit projections take their input as 16-bit fixed point per row and 128-wide group.  Rows with
    outliers 100x the rest, groups that are all zero, an all-zero row and a row of tiny values: the result stays
    within the bound the format implies, sum over groups of (max|x| of the group / 32639 / 2) * sum|w_hat|, plus
    fp32 rounding; rows and groups without outliers are not affected by the outliers elsewhere."""
    from oracle import oracle as orc
    shape = wl.SMALL128
    H.say("linear W4 with outliers and empty groups")
    cfg = sun.make_cfg(shape, "bf16")
    w = wl.make_weights(shape, "bf16", H.DEV, 13, std=0.05)
    quant = {k: [sun.sun_quantize_w4(m, 128, "asym") for m in w[k]] for k in sun.QUANT_KEYS}
    W = sun.sun_qweights_create(cfg, w, quant)
    batch = 40
    ws = torch.empty(sun.sun_workspace_bytes(cfg, batch, 4), dtype=torch.uint8, device=H.DEV)
    rng = np.random.default_rng(14)
    for mat, key, K, N in ((1, "wo", 1024, 512), (3, "wd", 1024, 512)):
        x = rng.standard_normal((batch, K)).astype(np.float32)
        x[0, rng.integers(0, K, size=5)] *= 100.0          # outliers in a few groups of row 0
        x[1, 128:384] = 0.0                                 # two empty groups
        x[2, :] = 0.0                                       # an empty row
        x[3, :] *= 1e-20                                    # tiny values: the scale is tiny, not zero
        x[4, 5] = 3.0e4                                     # one huge value
        xd = torch.from_numpy(x).to(H.DEV)
        out = torch.full((batch, N), float("nan"), device=H.DEV)
        sun.sun_linear(W, 0, mat, xd, out, ws)
        torch.cuda.synchronize()
        q, sc, z = (H.to_np(t) for t in quant[key][0])
        what = orc.dequantize_w4(q, sc, z, K, 128).astype(np.float64)
        want = orc.linear(orc.w4_mat(q, sc, z, K, 128), x.astype(np.float64))
        got = out.double().cpu().numpy()
        assert np.isfinite(got).all()
        amax = np.abs(x.astype(np.float64)).reshape(batch, K // 128, 128).max(axis=2)              # [b, g]
        wabs = np.abs(what).reshape(N, K // 128, 128).sum(axis=2)                                   # [n, g]
        bound = (amax / 32639.0 / 2.0) @ wabs.T                                                     # [b, n]
        slack = 4e-6 * (np.abs(x.astype(np.float64)) @ np.abs(what).T) + 1e-30                      # fp32 rounding of sums and scales
        err = np.abs(got - want)
        assert np.all(err <= 1.05 * bound + slack), f"mat {mat}: worst excess {(err - bound - slack).max():.3e}"
        assert np.all(got[2] == 0.0)
        H.say(f"   mat {mat}: max err / bound = {(err / (bound + slack)).max():.3f}; row 0 max err {err[0].max():.2e}, "
              f"other rows {err[5:].max():.2e}")
        assert err[5:].max() < 2e-4      # rows without outliers keep their usual accuracy


# ------------------------------------------------------------------ bf16 and QSUN full steps, small shapes
@pytest.mark.parametrize("batch", [8, 48, 100])
def test_bf16_small_full_step(H, batch):
    H.say(f"bf16 small128 batch {batch}")
    work = wl.make_workload("cfg2", shape=wl.SMALL128, batch=batch, lo=1, hi=700, seed=81 + batch)
    case = H.GpuCase(work)
    _full_step_parity(H, case)


@pytest.mark.parametrize("mode", ["asym", "sym", "sym_noz"])
def test_qsun_small_full_step(H, mode):
    H.say(f"QSUN small128 {mode}")
    work = wl.make_workload("cfg2", shape=wl.SMALL128, batch=40, lo=1, hi=700, seed=91)
    case = H.GpuCase(work, quant_mode=mode)
    _full_step_parity(H, case)


def test_bf16_and_qsun_gqa_ratio_5(H):
    """The 14B head geometry (5 query heads per KV head) on a small shape, dense and 4-bit."""
    for quant in (None, "asym"):
        H.say(f"bf16 small_g5 quant={quant}")
        work = wl.make_workload("cfg2", shape=wl.SMALL_G5, batch=20, n_models=4, lo=1, hi=900, seed=95)
        case = H.GpuCase(work, quant_mode=quant)
        _full_step_parity(H, case)


@pytest.mark.parametrize("dtype,quant", [("f32", None), ("bf16", None), ("bf16", "asym")])
def test_qkv_bias_option(H, dtype, quant):
    """Qwen2-class block: bias vectors on the q, k and v projections, added before the rotation."""
    H.say(f"q/k/v bias {dtype} quant={quant}")
    shape = wl.TINY_BIAS if dtype == "f32" else wl.SMALL_BIAS
    work = wl.make_workload("cfg2", shape=shape, dtype=dtype, batch=14, lo=1, hi=700, seed=98)
    _full_step_parity(H, H.GpuCase(work, quant_mode=quant))
    if quant is None:       # the option is live: the same weights without the biases give different logits
        import dataclasses
        plain = dataclasses.replace(shape, qkv_bias=False)
        work2 = wl.make_workload("cfg2", shape=plain, dtype=dtype, batch=14, lo=1, hi=700, seed=98)
        c1, c2 = H.GpuCase(work), H.GpuCase(work2)
        c1.step()
        c2.step()
        assert (c1.logits - c2.logits).abs().max() > 1e-2


def test_symmetric_layout_without_zero_points_equals_the_one_with(H):
    """Scales only (two groups per dword, zero point 8 implied) against the same grid with stored zero points:
    the same arithmetic on the same values, so the logits are bit-identical; odd and even group counts, and the
    14B width whose 80 groups per row split unevenly over the K splits."""
    for shape, batch in ((wl.SMALL128, 40), (wl.TINY_Q, 9), (wl.SMALL_G5, 70)):
        H.say(f"QSUN {shape.name}: sym with and without stored zero points")
        work = wl.make_workload("cfg2", shape=shape, batch=batch, lo=1, hi=500, seed=96)
        a, b = H.GpuCase(work, quant_mode="sym"), H.GpuCase(work, quant_mode="sym_noz")
        assert all(trip[2] is None for v in b.quant.values() for trip in v)
        a.step()
        b.step()
        assert torch.equal(a.logits, b.logits) and torch.equal(a.next, b.next)
        assert torch.equal(a.pool_mem, b.pool_mem)


def test_bf16_head_dim_64(H):
    H.say("bf16 tiny_q (head_dim 64, G=2)")
    work = wl.make_workload("cfg1", shape=wl.TINY_Q, dtype="bf16", batch=12, lo=1, hi=400, seed=92)
    case = H.GpuCase(work)
    _full_step_parity(H, case)


# ------------------------------------------------------------------ the SUN property on the GPU
@pytest.mark.parametrize("dtype,shape", [("f32", wl.TINY), ("bf16", wl.SMALL128)])
def test_batch_mix_invariance_is_bitwise(H, dtype, shape):
    """Relabelling model ids, and replacing every *other* request of the batch, must leave a
    request's logits bit-identical (same batch size and row index)."""
    H.say(f"batch-mix invariance {dtype}")
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=8, lo=1, hi=600, seed=93)
    case = H.GpuCase(work)
    pool0 = case.pool_mem.clone()
    case.step()
    base = case.logits.clone()
    base_next = case.next.clone()
    # (a) relabel the source models
    case.pool_mem.copy_(pool0)
    ids2 = ((case.ids + 1) % work.n_models).contiguous()
    case.step(ids=ids2)
    assert torch.equal(case.logits, base) and torch.equal(case.next, base_next)
    # (b) keep request 3, swap tokens / lengths / tables of all the others for different ones
    keep = 3
    rng = np.random.default_rng(9)
    lens2 = work.seq_lens.copy()
    toks2 = work.tokens.copy()
    for i in range(work.batch):
        if i != keep:
            lens2[i] = rng.integers(0, int(work.seq_lens[i]) + 1)     # shorter prefixes of their own pages
            toks2[i] = rng.integers(0, shape.vocab)
    case.pool_mem.copy_(pool0)
    case.step(tokens=torch.from_numpy(toks2).to(H.DEV), lens=torch.from_numpy(lens2).to(H.DEV))
    assert torch.equal(case.logits[keep], base[keep]) and case.next[keep] == base_next[keep]
    assert not torch.equal(case.logits[0], base[0])
    # (c) the same step twice gives the same bits (no atomics, fixed reduction order)
    case.pool_mem.copy_(pool0)
    case.step(host_lens=False)
    assert torch.equal(case.logits, base)


def test_validation_errors(H):
    H.say("SUN_VALIDATE error paths")
    work = wl.make_workload("cfg1", seed=94)
    case = H.GpuCase(work)
    bad = case.tables.clone()
    bad[2, 0] = work.n_pages
    with pytest.raises(sun.SunError) as e:
        case.step(flags=sun.SUN_VALIDATE, tables=bad)
    assert e.value.status == 5
    dup = case.tables.clone()
    need = wl.pages_needed(work.seq_lens)
    dup[1, need[1] - 1] = dup[0, need[0] - 1]
    with pytest.raises(sun.SunError) as e:
        case.step(flags=sun.SUN_VALIDATE, tables=dup)
    assert e.value.status == 5
    with pytest.raises(sun.SunError) as e:
        case.step(flags=sun.SUN_VALIDATE, lens=torch.full_like(case.lens, work.max_pages * 16))
    assert e.value.status == 6
    with pytest.raises(sun.SunError) as e:
        case.step(flags=sun.SUN_VALIDATE, ids=torch.full_like(case.ids, work.n_models))
    assert e.value.status == 7
    with pytest.raises(sun.SunError) as e:
        case.step(flags=sun.SUN_VALIDATE, tokens=torch.full_like(case.tokens, -1))
    assert e.value.status == 9
    case.step(flags=sun.SUN_VALIDATE)   # and the good call still works afterwards


# ------------------------------------------------------------------ backbone options of the paper's model families
def test_fp32_head_norm_option(H):
    """Qwen3-class block: RMSNorm over head_dim on q and k heads before the rotation (rms_eps 1e-6, base 1e6)."""
    H.say("fp32 tiny with q/k head norm")
    work = wl.make_workload("cfg1", shape=wl.TINY_QWEN, seed=95)
    rep = _full_step_parity(H, H.GpuCase(work))
    # the option is live: the same inputs through the plain block give different logits
    import dataclasses
    plain = dataclasses.replace(wl.TINY_QWEN, qk_norm=False)
    work2 = wl.make_workload("cfg1", shape=plain, seed=95)
    c1, c2 = H.GpuCase(work), H.GpuCase(work2)
    c1.step()
    c2.step()
    assert (c1.logits - c2.logits).abs().max() > 1e-3


@pytest.mark.parametrize("quant", [None, "asym"])
def test_bf16_head_norm_option(H, quant):
    import dataclasses
    shape = dataclasses.replace(wl.SMALL128, name="small128_qknorm", qk_norm=True, rms_eps=1e-6)
    H.say(f"bf16 small128 with q/k head norm, quant={quant}")
    work = wl.make_workload("cfg2", shape=shape, batch=24, lo=20, hi=700, seed=96)
    _full_step_parity(H, H.GpuCase(work, quant_mode=quant))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scaled_rotary_option(H, dtype):
    """LLaMA-3.1-class rotary scaling (factor 8, low 1, high 4) with a short original length (256), so that at
    these positions (up to 2000) kept, blended and slowed pairs all occur."""
    H.say(f"{dtype} small with scaled rotary frequencies")
    work = wl.make_workload("cfg2", shape=wl.SMALL_LLAMA31, dtype=dtype, batch=12, lo=300, hi=2000, seed=97)
    rep = _full_step_parity(H, H.GpuCase(work))
    import dataclasses
    plain = dataclasses.replace(wl.SMALL_LLAMA31, rope_scaling=None)
    c1 = H.GpuCase(work)
    c2 = H.GpuCase(wl.make_workload("cfg2", shape=plain, dtype=dtype, batch=12, lo=300, hi=2000, seed=97))
    c1.step()
    c2.step()
    assert (c1.logits - c2.logits).abs().max() > 1e-3


def test_tied_embeddings(H):
    """Small models of the Qwen3 family tie the LM head to the embedding: the same pointer serves as both."""
    H.say("fp32 tiny, lm_head tied to the embedding")
    work = wl.make_workload("cfg1", seed=98)
    w = wl.make_weights(wl.TINY, "f32", "cuda", 99)
    w["wlm"] = w["embed"]
    _full_step_parity(H, H.GpuCase(work, weights=w))


@pytest.mark.parametrize("dtype,shape,quant", [("f32", wl.TINY, None), ("bf16", wl.SMALL128, None), ("bf16", wl.SMALL128, "asym")])
def test_every_rmsnorm_gain_is_live(H, dtype, shape, quant):
    """The gains of the two norms of every layer and of the final norm are drawn around 1, not equal to 1, so
    the parity tests above already pin their wiring; here each one is shown to reach the logits on the GPU:
    scaling one gain vector changes them."""
    H.say(f"gains live {dtype} quant={quant}")
    work = wl.make_workload("cfg1", shape=shape, dtype=dtype, batch=6, lo=1, hi=200, seed=120)
    w = wl.make_weights(shape, dtype, "cuda", 121)
    assert all((g.float() - 1).abs().max() > 0.05 for g in w["g1"] + w["g2"] + [w["gf"]])
    base_case = H.GpuCase(work, weights=w, quant_mode=quant)
    pool0 = base_case.pool_mem.clone()
    base_case.step()
    base = base_case.logits.clone()
    for key, layer in (("g1", 0), ("g1", 1), ("g2", 0), ("g2", 1), ("gf", None)):
        w2 = {k: (list(v) if isinstance(v, list) else v) for k, v in w.items()}
        if layer is None:
            w2[key] = (w[key].float() * 1.5).to(w[key].dtype)
        else:
            w2[key][layer] = (w[key][layer].float() * 1.5).to(w[key][layer].dtype)
        c = H.GpuCase(work, weights=w2, quant_mode=quant)
        c.pool_mem.copy_(pool0)
        c.step()
        assert (c.logits - base).abs().max() > 1e-3, f"{key}[{layer}] does not reach the logits"


@pytest.mark.parametrize("batch", [65, 100, 128, 129, 200, 256])
def test_linear_op_bf16_above_64_rows_ragged_columns(H, batch):
    """The projection kernel for more than 64 rows (a wave owns two 32-column strips, a workgroup up to four
    such pairs) on widths that leave the last workgroup partly empty and the last wave with one strip only:
    20 and 65 strips; every projection of the step, alone."""
    from oracle import oracle as orc
    shape = wl.Shape("ragged_cols", 2, 640, 5, 1, 128, 1152, 2080)
    H.say(f"linear bf16 batch {batch}, ragged column counts")
    cfg = sun.make_cfg(shape, "bf16")
    w = wl.make_weights(shape, "bf16", H.DEV, 14, std=0.05)
    W = sun.sun_weights_create(cfg, w)
    ws = torch.empty(sun.sun_workspace_bytes(cfg, batch, 4), dtype=torch.uint8, device=H.DEV)
    g = torch.Generator(device=H.DEV).manual_seed(1000 + batch)
    wn = H.weights_to_np(w)
    for mat, K, N in ((0, 640, 896), (1, 640, 640), (2, 640, 1152), (3, 1152, 640), (4, 640, 2080)):
        x = torch.randn((batch, K), device=H.DEV, generator=g)
        out = torch.full((batch, N), float("nan"), device=H.DEV)
        sun.sun_linear(W, 1, mat, x, out, ws)
        torch.cuda.synchronize()
        xr = x.double().cpu().numpy()
        lin = lambda key: orc.linear(orc.dense_mat(wn[key][1] if isinstance(wn[key], list) else wn[key]), xr)
        if mat == 0:
            want = np.concatenate([lin("wq"), lin("wk"), lin("wv")], axis=1)
        elif mat == 2:
            gate, up = lin("wg"), lin("wu")
            want = gate / (1 + np.exp(-gate)) * up
        else:
            want = lin({1: "wo", 3: "wd", 4: "wlm"}[mat])
        got = out.double().cpu().numpy()
        tol = 1e-2 * np.abs(want) + 2e-3 if mat == 2 else 2e-4 + 1e-5 * np.abs(want)   # mat 2 output is bf16
        assert np.all(np.abs(got - want) <= tol), f"mat {mat}: max diff {np.abs(got - want).max():.3e}"
