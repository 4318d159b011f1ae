"""Headline benchmark: ms per attention layer at 128K context for the UniSparse hot path
(composite-token proxy + block selection + block-sparse attention) on one MI355X, and the
speedup over this library's own dense attention kernel.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg3|cfg2|cfg1|cfg4|cfg5]

A step = one pass of the whole hot path (pool -> compressed scores -> selection -> row ranking -> sparse attention)
over one synthetic layer already resident in HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def _profiled_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel, as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    written down in profiles/ (a line `traffic_bytes_per_launch <workload> <bytes>`); None when there is no such line."""
    path = os.path.join(ROOT, "profiles", "bench_cfg3_hbm_traffic.md")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == workload:
                    return float(parts[2])
    except OSError:
        pass
    return None


def _events(n):
    import torch
    return [torch.cuda.Event(enable_timing=True) for _ in range(n)]


def _time_ms(fn, reps, warm=1):
    """Average duration of fn() over reps launches, HIP events on the launch stream."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    a, b = _events(2)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def cpu_baseline(w, m_gpu, valid_pairs_per_head, budget_s=20.0):
    """Time the oracle (as it stands) on a bounded sample of the same workload and scale to one layer."""
    import numpy as np
    from oracle import reference as oracle
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    qf, kf, vf = w.f32()
    H = w.n_heads_q
    NQ = m_gpu.shape[1]
    G = H // w.n_heads_kv
    # proxy sample: every 2nd query-block row of head 0
    rows_p = list(range(NQ - 1, -1, -2))
    t0 = time.time()
    oracle.build_mask(qf[:1], kf[:1], w.cu_seqlens, w.block_size, w.c_q, w.c_k, w.causal, w.mode, w.param,
                      rows=rows_p)
    t_proxy = time.time() - t0
    seq_loc = []
    for b in range(len(w.cu_seqlens) - 1):
        seq_loc += list(range((w.cu_seqlens[b + 1] - w.cu_seqlens[b]) // w.block_size))
    work = lambda r: (seq_loc[r] + 1) if w.causal else max(seq_loc) + 1
    proxy_scale = H * sum(work(r) for r in range(NQ)) / sum(work(r) for r in rows_p)
    # attention sample: a few rows of head 0, scaled by selected block pairs
    pairs_total = float(m_gpu.sum())
    rows_a, t_attn, pairs_s = [], 0.0, 0.0
    step = max(1, NQ // 64)
    for r in range(NQ - 1 - step // 2, -1, -step):
        t0 = time.time()
        oracle.masked_attention(qf, kf, vf, w.cu_seqlens, w.block_size, w.causal, m_gpu, rows=[r], heads=[0])
        t_attn += time.time() - t0
        pairs_s += float(m_gpu[0, r].sum())
        rows_a.append(r)
        if t_attn > budget_s:
            break
    est_ms = (t_proxy * proxy_scale + t_attn * pairs_total / max(pairs_s, 1.0)) * 1e3
    return {"value": est_ms, "unit": "ms/layer (extrapolated from the sample)", "cores": threads, "kind": "oracle",
            "sample": f"mask oracle on {len(rows_p)} query-block rows of head 0 ({t_proxy:.1f} s) + attention oracle on "
                      f"{len(rows_a)} query-block rows of head 0 ({t_attn:.1f} s), scaled by valid / selected block pairs"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg3",
                    help="cfg1 .. cfg5 (cfg3 is the headline), or rand32k_d64 / rand32k_d128 / rand32k_d256: random "
                         "GQA 32/8 layer at L = 32K with that head dimension and a fixed 25 %% budget")
    ap.add_argument("--gain", type=float, default=4.0)
    ap.add_argument("--layout", default="htd", choices=["htd", "thd"])
    ap.add_argument("--c-h", type=int, default=0, help="head compression factor (Eq. (2)); 0 = the workload's own (1)")
    ap.add_argument("--c", type=int, default=0, help="sequence compression factor c_q = c_k; 0 = the workload's own (8)")
    ap.add_argument("--param", type=float, default=0.0,
                    help="selection threshold P (Top-P workloads) or kept fraction f (budget workloads); 0 = the workload's own")
    ap.add_argument("--dense-reps", type=int, default=2)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--profile-copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (one MI355X holds the whole layer); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_14082_amd import api
    from paper_2512_14082_amd import workloads as W

    kw = {} if args.workload == "cfg4" or args.workload.startswith("rand32k") else {"gain": args.gain}
    t0 = time.time()
    w = W.by_name(args.workload, **kw)
    t_gen = time.time() - t0
    if args.c_h > 0:
        w.c_h = args.c_h
    if args.c > 0:
        w.c_q = w.c_k = args.c
    if args.param > 0:
        w.param = args.param
    ctx = api.Context(0)
    q, k, v = (api.bits_to_device(x) for x in (w.q, w.k, w.v))
    if args.layout == "thd":
        q, k, v = (x.transpose(0, 1).contiguous() for x in (q, k, v))
    p = api.Problem(w.cu_seqlens, w.n_heads_q, w.n_heads_kv, w.block_size, w.causal, head_dim=w.head_dim)
    s = api.Select(w.c_q, w.c_k, w.c_h, w.mode, w.param if w.mode == W.TOP_P else 0.9,
                   w.param if w.mode == W.TOP_K else 0.25)
    ws = ctx.alloc_workspace(p, s)
    mask = ctx.alloc_mask(p)
    o = torch.empty_like(q)
    od = torch.empty_like(q)
    score = torch.empty((p.n_heads_q // s.c_h, p.n_rows, p.n_cols), dtype=torch.float32, device="cuda")
    lay = args.layout

    # HIP events around the dominant kernel's launch inside every step (torch's current stream is the launch stream)
    ev = []

    def step(timed=False):
        ctx.build_mask(p, s, q, k, lay, workspace=ws, mask=mask)
        if timed:
            ev.append(_events(2))
            ev[-1][0].record()
        ctx.sparse_attn(p, q, k, v, mask, lay, out=o, workspace=ws)      # unisparse_sparse_attn_ws: ranked work order
        if timed:
            ev[-1][1].record()

    if args.profile_copy_mb > 0:
        src = torch.empty(args.profile_copy_mb << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step(timed=True)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t1) * 1e3 / args.steps
    ms_sparse_in_step = sum(a.elapsed_time(b) for a, b in ev) / len(ev)

    # ---- per-kernel timings (HIP events on the launch stream) ------------------------------------
    reps = max(3, args.steps)
    if w.head_dim == 128:
        ms_pool = _time_ms(lambda: (ctx.avgpool_seq(q, s.c_q, lay), ctx.avgpool_seq(k, s.c_k, lay)), reps)
    else:
        ms_pool = _time_ms(lambda: (ctx.pool_seq_varlen(p, q, s.c_q, lay), ctx.pool_seq_varlen(p, k, s.c_k, lay)), reps)
    ms_build = _time_ms(lambda: ctx.build_mask(p, s, q, k, lay, workspace=ws, mask=mask), reps)
    # scores for the selection-only timing
    _, sc = ctx.build_mask(p, s, q, k, lay, workspace=ws, mask=mask, want_score=True)
    ms_select = _time_ms(lambda: ctx.select_blocks(p, s, sc, mask=mask), reps)
    ms_sparse = _time_ms(lambda: ctx.sparse_attn(p, q, k, v, mask, lay, out=o, workspace=ws), reps)
    # the dense baseline in the same setting as the sparse launch of a step: after the mask kernels, not back to back
    # with itself (the device clock depends on what ran just before)
    ctx.full_attn(p, q, k, v, lay, out=od)
    evd = []
    for _ in range(args.dense_reps):
        ctx.build_mask(p, s, q, k, lay, workspace=ws, mask=mask)
        evd.append(_events(2))
        evd[-1][0].record()
        ctx.full_attn(p, q, k, v, lay, out=od)
        evd[-1][1].record()
    torch.cuda.synchronize()
    ms_dense = sum(a.elapsed_time(b) for a, b in evd) / len(evd)
    torch.cuda.synchronize()

    m_gpu = api.unpack_mask(mask, p.n_cols)
    nnz = float(m_gpu.sum())
    valid = float(w.valid_pairs() * w.n_heads_q)
    S, d = w.block_size, w.head_dim
    flop_pair = 4.0 * S * S * d
    sparse_tflops = nnz * flop_pair / (ms_sparse_in_step * 1e-3) / 1e12      # the launches of the timed steps
    dense_tflops = valid * flop_pair / (ms_dense * 1e-3) / 1e12
    pool_bytes = (w.q.size + w.k.size) * 2 * (1 + 1.0 / s.c_q)
    out = {
        "metric": "ms/layer at 128K ctx (proxy + sparse attn); speedup vs own dense HIP attn",
        "value": ms_step, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "heads_q": w.n_heads_q, "heads_kv": w.n_heads_kv, "head_dim": d,
                   "tokens": w.total_tokens, "block_size": S, "causal": w.causal, "c_q": s.c_q, "c_k": s.c_k,
                   "c_h": s.c_h, "selection": "top_p" if w.mode == W.TOP_P else "top_k", "param": w.param,
                   "gain": w.gain, "layout": lay},
        "speedup_vs_dense": ms_dense / ms_step,
        "mask_density": nnz / valid,
        # (sparse_attn: HIP events around the launch inside the timed steps, row ranking included; the other entries
        #  are timed after them, each launch repeated back to back.  scores_and_select: the one-sweep score kernel plus
        #  the selection kernel that normalises its row sums; select_given_scores: unisparse_select_blocks alone on a
        #  score buffer, for reference)
        "kernels_ms": {"pool": ms_pool, "scores_and_select": ms_build - ms_pool, "select_given_scores": ms_select,
                       "build_mask": ms_build, "sparse_attn": ms_sparse_in_step, "sparse_attn_back_to_back": ms_sparse,
                       "dense_attn": ms_dense},
        "effective_tflops": valid * flop_pair / (ms_step * 1e-3) / 1e12,
        "dense_tflops": dense_tflops,
        "pool_gbs": pool_bytes / (ms_pool * 1e-3) / 1e9,
        "roofline": {"kernel": "attention_kernel (block-sparse)", "bound": "mfma", "achieved": sparse_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": sparse_tflops / PEAK_BF16_TFLOPS,
                     "traffic": _profiled_traffic(w.name)},
        "host_gen_s": t_gen,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, m_gpu, w.valid_pairs())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
