"""Shared machinery of the GPU parity tests: run the HIP path through the C ABI and compare with the oracle."""
import numpy as np
import torch

from paper_2512_14082_amd import api
from paper_2512_14082_amd import workloads as W

MASK_AGREE_MIN = 0.999      # fraction of valid block decisions that must agree
CUT_TOL = 1e-3              # a mismatch must lie within this of the cut (normalised score / cumulative share)
OUT_MAX_ABS = 2e-2
OUT_MEAN_ABS = 5e-3


def device_tensors(w: W.Workload, layout="htd"):
    q, k, v = (api.bits_to_device(x) for x in (w.q, w.k, w.v))
    if layout == "thd":
        q, k, v = (x.transpose(0, 1).contiguous() for x in (q, k, v))
    return q, k, v


def to_htd(x: torch.Tensor, layout):
    return x if layout == "htd" else x.transpose(0, 1)


def problem_of(w: W.Workload, scale=0.0):
    return api.Problem(w.cu_seqlens, w.n_heads_q, w.n_heads_kv, w.block_size, w.causal, scale, w.head_dim)


def select_of(w: W.Workload):
    dev = lambda r: None if r is None else torch.from_numpy(r).cuda()
    return api.Select(w.c_q, w.c_k, w.c_h, w.mode, w.param if w.mode == W.TOP_P else 0.9,
                      w.param if w.mode == W.TOP_K else 0.25, w.pool, dev(w.rand_q), dev(w.rand_k))


def rand_of(w: W.Workload):
    return None if w.rand_q is None else (w.rand_q, w.rand_k)


def row_geometry(cu, S):
    loc, nb = [], []
    for b in range(len(cu) - 1):
        n = -(-(cu[b + 1] - cu[b]) // S)
        loc += list(range(n))
        nb += [n] * n
    return np.array(loc), np.array(nb)


def check_mask_against_oracle(m_gpu, m_ref, score_ref, cu, S, causal, mode, param, rows=None, counts=None):
    """>= 99.9 % of valid decisions equal; every mismatch admissible: the oracle's normalised score of the
    block lies within 1e-3 of the row's cut, or (Top-P) the cumulative share next to it lies within 1e-3 of P.
    ``counts`` (a two-element list) accumulates [mismatches, valid decisions] over several calls; the agreement
    bound is then the caller's to assert on the total."""
    loc, nb = row_geometry(cu, S)
    H, NQ, NK = m_ref.shape
    c_h = H // score_ref.shape[0]
    n_valid = n_bad = 0
    rr = range(NQ) if rows is None else rows
    for h in range(H):
        for r in rr:
            nv = loc[r] + 1 if causal else nb[r]
            a, b = m_gpu[h, r, :nv], m_ref[h, r, :nv]
            assert not m_gpu[h, r, nv:].any(), "bit outside the valid set"
            assert a.any(), "empty mask row"
            n_valid += nv
            diff = np.nonzero(a != b)[0]
            if len(diff) == 0:
                continue
            n_bad += len(diff)
            sc = score_ref[h // c_h, r, :nv]
            p = sc / sc.sum()
            tau = p[b == 1].min()
            order = np.lexsort((np.arange(nv), -p))
            cum = np.cumsum(p[order])
            pos = np.empty(nv, dtype=int)
            pos[order] = np.arange(nv)
            for j in diff:
                ok = abs(p[j] - tau) <= CUT_TOL
                if mode == W.TOP_P:
                    before = cum[pos[j] - 1] if pos[j] > 0 else 0.0
                    ok = ok or abs(before - param) <= CUT_TOL or abs(cum[pos[j]] - param) <= CUT_TOL
                assert ok, f"inadmissible mask mismatch h={h} row={r} j={j} p={p[j]:.3e} tau={tau:.3e}"
    agree = 1.0 - n_bad / max(1, n_valid)
    if counts is not None:
        counts[0] += n_bad
        counts[1] += n_valid
        return agree
    assert agree >= MASK_AGREE_MIN, f"mask agreement {agree:.5f}"
    return agree


def check_output(o_gpu, o_ref, what=""):
    sel = ~np.isnan(o_ref)
    d = np.abs(o_gpu[sel].astype(np.float64) - o_ref[sel])
    if not d.max() <= OUT_MAX_ABS:
        full = np.where(sel, np.abs(o_gpu.astype(np.float64) - np.nan_to_num(o_ref)), 0.0)
        bad_rows = np.argwhere(full.max(-1) > OUT_MAX_ABS)
        raise AssertionError(f"{what} max-abs {d.max():.4f}; {len(bad_rows)} bad (head, token) rows of "
                             f"{int(sel[..., 0].sum())}; first {bad_rows[:12].tolist()} last {bad_rows[-3:].tolist()}")
    assert d.mean() <= OUT_MEAN_ABS, f"{what} mean-abs {d.mean():.5f}"
    return d.max(), d.mean()


def full_pipeline_check(ctx, oracle, w: W.Workload, layout="htd", check_dense=True, rows=None, score_rtol=2e-3):
    """Pool, scores, mask, selection, sparse and dense attention of one workload against the oracle."""
    q, k, v = device_tensors(w, layout)
    qf, kf, vf = w.f32()
    p, s = problem_of(w), select_of(w)
    param = w.param
    # -- pooling: bit exact
    qt = ctx.pool_seq_varlen(p, q, w.c_q, layout, w.pool, s.rand_q)  # equals the flat entry point when every window is whole
    if w.pool == 0 and w.head_dim == 128 and all((w.cu_seqlens[b + 1] - w.cu_seqlens[b]) % w.c_q == 0 for b in range(len(w.cu_seqlens) - 1)):
        assert torch.equal(qt, ctx.avgpool_seq(q, w.c_q, layout))
    torch.cuda.synchronize()
    qt_bits = qt.view(torch.int16).cpu().numpy().view(np.uint16)
    off = oracle.composite_offsets(w.cu_seqlens, w.c_q)
    for h in range(w.n_heads_q):
        ref = np.concatenate([oracle.pool_seq(qf[h, w.cu_seqlens[b]:w.cu_seqlens[b + 1]], w.c_q, w.pool,
                                              None if w.rand_q is None else w.rand_q[h, off[b]:off[b + 1]])
                              for b in range(len(w.cu_seqlens) - 1)])
        assert np.array_equal(qt_bits[h], W.f32_to_bf16_bits(ref)), f"pooling mismatch head {h}"
    # -- scores and mask, in both forms of the score computation: two sweeps over the composite keys (the least
    #    workspace), then one sweep (the workspace the size query asks for); the latter's mask feeds the attention
    m_ref, sc_ref = oracle.build_mask(qf, kf, w.cu_seqlens, w.block_size, w.c_q, w.c_k, w.causal, w.mode, param,
                                      c_h=w.c_h, rows=rows, pool=w.pool, rand=rand_of(w))
    rr = slice(None) if rows is None else list(rows)
    # (the one-sweep form is offered when a key block holds at least 8 composite keys; else both runs are two sweeps)
    assert (ctx.workspace_bytes(p, s) > ctx.workspace_bytes_min(p, s)) == (w.block_size // w.c_k >= 8)
    for minimal in (True, False):
        form = "two sweeps" if minimal else "one sweep"
        ws = ctx.alloc_workspace(p, s, minimal=minimal)
        m_dev, sc_dev = ctx.build_mask(p, s, q, k, layout, workspace=ws, want_score=True)
        torch.cuda.synchronize()
        m_gpu = api.unpack_mask(m_dev, p.n_cols)
        sc_gpu = sc_dev.cpu().numpy()
        np.testing.assert_allclose(sc_gpu[:, rr], sc_ref[:, rr], rtol=score_rtol, atol=1e-6, err_msg=form)
        # -- the score kernel's two tilings (one or two 32-row tiles per wavefront) do the same arithmetic per row
        if w.head_dim == 128 and w.block_size // w.c_q <= 32:
            for tiles in (1, 2):
                s_t = select_of(w)
                s_t.proxy_tiles = tiles
                m_t, sc_t = ctx.build_mask(p, s_t, q, k, layout, workspace=ws, want_score=True)
                torch.cuda.synchronize()
                assert torch.equal(sc_t, sc_dev) and torch.equal(m_t, m_dev), f"{form}: proxy_tiles={tiles} changes the result"
        # -- averaged queries are pooled inside the score kernel unless head pooling follows: the same arithmetic as
        #    the pooling pass (checked bit for bit above), so the same scores as with that pass forced
        if w.pool == 0 and w.c_h == 1:
            s_p = select_of(w)
            s_p.query_pool_pass = 1
            m_p, sc_p = ctx.build_mask(p, s_p, q, k, layout, workspace=ws, want_score=True)
            torch.cuda.synchronize()
            assert torch.equal(sc_p, sc_dev) and torch.equal(m_p, m_dev), f"{form}: pooling the queries on the fly changes the result"
        agree = check_mask_against_oracle(m_gpu, m_ref, sc_ref, w.cu_seqlens, w.block_size, w.causal, w.mode, param, rows)
        # -- selection alone is index work: on the GPU's own scores it must match the oracle bit for bit
        m_sel = oracle.select_mask(sc_gpu, w.cu_seqlens, w.block_size, w.causal, w.mode, param, rows)
        m_sel = np.repeat(m_sel, w.c_h, axis=0)
        assert np.array_equal(m_gpu[:, rr], m_sel[:, rr]), f"{form}: selection differs from the oracle on identical scores"
    # -- sparse attention on the GPU's own mask
    o_dev, lse_dev = ctx.sparse_attn(p, q, k, v, m_dev, layout, want_lse=True)
    torch.cuda.synchronize()
    o_gpu = to_htd(o_dev, layout).float().cpu().numpy()
    o_ref, lse_ref = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, w.block_size, w.causal, m_gpu, rows=rows)
    check_output(o_gpu, o_ref, "sparse")
    ls = ~np.isnan(lse_ref)
    np.testing.assert_allclose(lse_dev.cpu().numpy()[ls], lse_ref[ls], rtol=1e-3, atol=2e-3)
    if check_dense:
        od_dev, _ = ctx.full_attn(p, q, k, v, layout)
        torch.cuda.synchronize()
        od_ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, w.block_size, w.causal, None, rows=rows)
        check_output(to_htd(od_dev, layout).float().cpu().numpy(), od_ref, "dense")
    return agree


def say(msg):
    """Progress line of a long test (visible with -s; flushed so that a run that dies still names its step)."""
    print(msg, flush=True)


def sampled_rows(w: W.Workload, pop_h, rng, n_random):
    """Query-block rows one head is checked on at full size: the first and last row of every sequence, the rows
    with the fewest and the most selected blocks, and ``n_random`` seeded rows."""
    rows, base = set(), 0
    for n in w.n_blocks():
        if n > 0:
            rows.update((base, base + n - 1))
        base += n
    rows.update((int(np.argmin(pop_h)), int(np.argmax(pop_h))))
    rows.update(int(x) for x in rng.integers(0, len(pop_h), n_random))
    return sorted(rows)


def sampled_config_check(ctx, oracle, w: W.Workload, seed, n_random=16, attn_heads=(0,), attn_random=1,
                         dense_heads=(0,), extra_thresholds=()):
    """A benchmark configuration at its own shape: the whole GPU path exactly as bench.py launches it (mask with
    workspace, block-sparse attention, dense attention), the oracle on sampled outputs.

    Mask and scores: per query head, the rows of ``sampled_rows``.  Selection: bit-exact against the oracle's
    selection applied to the GPU's own scores on EVERY row.  Attention: for the heads of ``attn_heads`` the first
    and last row of every sequence, the head's rows of least and most selected blocks and ``attn_random`` seeded rows;
    dense attention on the last row and one seeded row of ``dense_heads``.  ``extra_thresholds``: further Top-P
    thresholds run through unisparse_select_blocks on the same score buffer, checked the same way.
    Returns {"agreement", "density", "densities": {P: density}}."""
    rng = np.random.default_rng(seed)
    S, H, G = w.block_size, w.n_heads_q, w.n_heads_q // w.n_heads_kv
    q, k, v = device_tensors(w)
    qf, kf, vf = w.f32()
    p, s = problem_of(w), select_of(w)
    ws, m_dev = ctx.alloc_workspace(p, s), ctx.alloc_mask(p)
    ctx.build_mask(p, s, q, k, workspace=ws, mask=m_dev)                  # as the benchmark calls it
    _, sc_dev = ctx.build_mask(p, s, q, k, workspace=ws, mask=ctx.alloc_mask(p), want_score=True)
    o_dev, lse_dev = ctx.sparse_attn(p, q, k, v, m_dev, want_lse=True, workspace=ws)     # as the benchmark calls it
    o_plain, lse_plain = ctx.sparse_attn(p, q, k, v, m_dev, want_lse=True)                # default work order
    od_dev, _ = ctx.full_attn(p, q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(o_dev, o_plain) and torch.equal(lse_dev, lse_plain), "the ranked work order changes the output"
    del o_plain, lse_plain
    s_p = select_of(w)
    s_p.query_pool_pass = 1                 # the queries pooled in a pass of their own instead of inside the score kernel
    m_p, sc_p = ctx.build_mask(p, s_p, q, k, workspace=ws, want_score=True)
    torch.cuda.synchronize()
    assert torch.equal(sc_p, sc_dev) and torch.equal(m_p, m_dev), "pooling the queries on the fly changes the result"
    del m_p, sc_p
    m_gpu = api.unpack_mask(m_dev, p.n_cols)
    sc_gpu = sc_dev.cpu().numpy()
    loc, nb = row_geometry(w.cu_seqlens, S)
    NQ, NK = m_gpu.shape[1], m_gpu.shape[2]
    valid = (np.arange(NK)[None, :] <= loc[:, None]) if w.causal else (np.arange(NK)[None, :] < nb[:, None])
    n_valid_head = int(valid.sum())
    # -- structure that holds on every row
    assert not (m_gpu & ~valid[None]).any(), "bit outside the valid set"
    assert m_gpu.any(-1).all(), "empty mask row"
    assert not (sc_gpu * ~valid[None]).any(), "score outside the valid set"
    whole = np.array([all((w.cu_seqlens[b + 1] - w.cu_seqlens[b]) % S == 0 for b in range(len(w.cu_seqlens) - 1))])
    if whole.all():
        np.testing.assert_allclose(sc_gpu.sum(-1), S / w.c_q, rtol=1e-3)       # every composite row of A~ sums to 1
    density = float(m_gpu.sum()) / (H * n_valid_head)
    say(f"{w.name}: GPU path done, density {density:.4f}")
    # -- selection is index work: on the GPU's own scores it must equal the oracle's on every row
    m_sel = oracle.select_mask(sc_gpu, w.cu_seqlens, S, w.causal, w.mode, w.param)
    assert np.array_equal(m_gpu, m_sel), "selection differs from the oracle on identical scores"
    # -- scores and mask against the oracle's own scores, sampled rows per head
    pop = m_gpu.sum(-1)
    counts = [0, 0]
    ref = {}
    for h in range(H):
        rows = sampled_rows(w, pop[h], rng, n_random)
        m_ref, sc_ref = oracle.build_mask(qf[h:h + 1], kf[h // G:h // G + 1], w.cu_seqlens, S, w.c_q, w.c_k, w.causal,
                                          w.mode, w.param, rows=rows)
        np.testing.assert_allclose(sc_gpu[h, rows], sc_ref[0, rows], rtol=2e-3, atol=1e-6)
        check_mask_against_oracle(m_gpu[h:h + 1], m_ref, sc_ref, w.cu_seqlens, S, w.causal, w.mode, w.param, rows, counts)
        ref[h] = (rows, sc_ref)
    agree = 1.0 - counts[0] / counts[1]
    say(f"{w.name}: mask agreement {agree:.6f} over {counts[1]} sampled decisions ({counts[0]} admissible mismatches)")
    assert agree >= MASK_AGREE_MIN, f"mask agreement {agree:.5f}"
    result = {"agreement": agree, "density": density, "densities": {w.param: density}}
    # -- the other form of the score computation (two sweeps, the least workspace) on the same sampled rows
    m2_dev, sc2_dev = ctx.build_mask(p, s, q, k, workspace=ctx.alloc_workspace(p, s, minimal=True), want_score=True)
    torch.cuda.synchronize()
    m2, sc2 = api.unpack_mask(m2_dev, p.n_cols), sc2_dev.cpu().numpy()
    del m2_dev, sc2_dev
    assert np.array_equal(m2, oracle.select_mask(sc2, w.cu_seqlens, S, w.causal, w.mode, w.param)), \
        "two sweeps: selection differs from the oracle on identical scores"
    cnt2 = [0, 0]
    for h in range(H):
        rows, sc_ref = ref[h]
        np.testing.assert_allclose(sc2[h, rows], sc_ref[0, rows], rtol=2e-3, atol=1e-6)
        m_ref = oracle.select_mask(sc_ref, w.cu_seqlens, S, w.causal, w.mode, w.param, rows)
        check_mask_against_oracle(m2[h:h + 1], m_ref, sc_ref, w.cu_seqlens, S, w.causal, w.mode, w.param, rows, cnt2)
    agree2 = 1.0 - cnt2[0] / cnt2[1]
    between = float((m2 == m_gpu).mean())
    say(f"{w.name}: two-sweep form: mask agreement {agree2:.6f} with the oracle, {between:.6f} of all bits equal to the one-sweep mask")
    assert agree2 >= MASK_AGREE_MIN and between >= MASK_AGREE_MIN
    del m2, sc2
    # -- further thresholds on the same score buffer (selection only)
    for P in extra_thresholds:
        s_p = select_of(w)
        s_p.threshold = P
        m_p = api.unpack_mask(ctx.select_blocks(p, s_p, sc_dev.clone()), p.n_cols)
        torch.cuda.synchronize()
        assert np.array_equal(m_p, oracle.select_mask(sc_gpu, w.cu_seqlens, S, w.causal, w.mode, P)), f"P={P}"
        cnt = [0, 0]
        for h in range(H):
            rows, sc_ref = ref[h]
            m_ref = oracle.select_mask(sc_ref, w.cu_seqlens, S, w.causal, w.mode, P, rows)
            check_mask_against_oracle(m_p[h:h + 1], m_ref, sc_ref, w.cu_seqlens, S, w.causal, w.mode, P, rows, cnt)
        a_p = 1.0 - cnt[0] / cnt[1]
        result["densities"][P] = float(m_p.sum()) / (H * n_valid_head)
        say(f"{w.name}: P = {P}: density {result['densities'][P]:.4f}, mask agreement {a_p:.6f}")
        assert a_p >= MASK_AGREE_MIN, f"P={P}: mask agreement {a_p:.5f}"
    # -- attention on the GPU's own mask, sampled (head, row) outputs
    o_gpu = o_dev.float().cpu().numpy()
    lse_gpu = lse_dev.cpu().numpy()
    for h in attn_heads:
        rows = sampled_rows(w, pop[h], rng, attn_random)
        o_ref, lse_ref = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, S, w.causal, m_gpu, rows=rows, heads=[h])
        mx, mean = check_output(o_gpu[h:h + 1], o_ref[h:h + 1], f"{w.name} sparse head {h}")
        ls = ~np.isnan(lse_ref[h])
        np.testing.assert_allclose(lse_gpu[h][ls], lse_ref[h][ls], rtol=1e-3, atol=2e-3)
        say(f"{w.name}: sparse attention head {h} rows {rows}: max-abs {mx:.4f} mean-abs {mean:.5f}")
    od_gpu = od_dev.float().cpu().numpy()
    for h in dense_heads:
        rows = sorted({NQ - 1, int(rng.integers(0, NQ))})
        od_ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, S, w.causal, None, rows=rows, heads=[h])
        mx, mean = check_output(od_gpu[h:h + 1], od_ref[h:h + 1], f"{w.name} dense head {h}")
        say(f"{w.name}: dense attention head {h} rows {rows}: max-abs {mx:.4f} mean-abs {mean:.5f}")
    return result
