"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from paper_2512_14082_amd import api
from paper_2512_14082_amd import workloads as W

import parity_utils as PU

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    return api.Context(0)


def test_config1_single_head(ctx, oracle):
    """Configuration 1 in full: one head, L = 2048, S = 64, top-25 % budget."""
    w = W.single_head_planted()
    agree = PU.full_pipeline_check(ctx, oracle, w)
    print("cfg1 mask agreement", agree)


@pytest.mark.parametrize("layout", ["htd", "thd"])
@pytest.mark.parametrize("S,causal,mode,param", [
    (128, True, W.TOP_P, 0.9),
    (128, False, W.TOP_K, 0.3),
    (64, True, W.TOP_K, 0.25),
    (64, False, W.TOP_P, 0.8),
])
def test_small_gqa_varlen(ctx, oracle, layout, S, causal, mode, param):
    """Several tiles, ragged sequence mix (1, 3 and 5 blocks), GQA 4:2 heads."""
    w = W.random_small(H=4, Hkv=2, lengths=(S, 3 * S, 5 * S), S=S, causal=causal, mode=mode, param=param, seed=11)
    PU.full_pipeline_check(ctx, oracle, w, layout)


@pytest.mark.parametrize("S,causal,mode,param,layout", [
    (128, True, W.TOP_P, 0.9, "htd"),
    (128, False, W.TOP_K, 0.4, "thd"),
    (64, True, W.TOP_K, 0.5, "thd"),
    (64, False, W.TOP_P, 0.8, "htd"),
])
def test_ragged_last_blocks(ctx, oracle, S, causal, mode, param, layout):
    """Sequence lengths that are not multiples of S (whole pooling windows): a block and a bit, several blocks and
    most of one, less than one block, two and a half blocks."""
    w = W.random_small(H=4, Hkv=2, lengths=(S + 8, 3 * S - 16, 40, 2 * S + S // 2), S=S, causal=causal, mode=mode,
                       param=param, seed=13)
    PU.full_pipeline_check(ctx, oracle, w, layout)


@pytest.mark.parametrize("S,causal,cq,ck,layout", [
    (128, True, 8, 8, "htd"),
    (128, False, 4, 16, "thd"),
    (64, True, 16, 4, "htd"),
    (64, False, 8, 8, "thd"),
])
def test_partial_pooling_windows(ctx, oracle, S, causal, cq, ck, layout):
    """Lengths that neither S nor c divides: the last pooling window of a sequence is partial."""
    w = W.random_small(H=4, Hkv=2, lengths=(S + 5, 3 * S - 13, 37, 2 * S + S // 2 + 3, 1), S=S, causal=causal,
                       mode=W.TOP_P, param=0.85, seed=17)
    w.c_q, w.c_k = cq, ck
    PU.full_pipeline_check(ctx, oracle, w, layout)


def test_dense_attention_any_length(ctx, oracle):
    """Attention alone needs no pooling windows: any length works."""
    w = W.random_small(H=2, Hkv=1, lengths=(203, 1, 129), S=128, causal=True, seed=14)
    q, k, v = PU.device_tensors(w)
    qf, kf, vf = w.f32()
    p = PU.problem_of(w)
    o, lse = ctx.full_attn(p, q, k, v, want_lse=True)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, 128, True, None)
    assert not np.isnan(o_ref).any()
    PU.check_output(o.float().cpu().numpy(), o_ref, "dense")
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=1e-3, atol=2e-3)


@pytest.mark.parametrize("kind", ["rising", "falling", "spikes", "ramp"])
@pytest.mark.parametrize("S,causal", [(128, True), (128, False), (64, True)])
def test_attention_with_logits_spanning_hundreds_of_units(ctx, oracle, kind, S, causal):
    steep_logits_check(ctx, oracle, kind, S, causal, 128)


@pytest.mark.parametrize("d", [64, 256])
@pytest.mark.parametrize("kind,S,causal", [("rising", 128, True), ("spikes", 128, False), ("ramp", 64, True),
                                           ("falling", 128, True)])
def test_attention_with_steep_logits_other_head_dims(ctx, oracle, d, kind, S, causal):
    """The same at head dimensions 64 and 256 (at 256 a block is walked in two stages of 64 keys)."""
    steep_logits_check(ctx, oracle, kind, S, causal, d)


@pytest.mark.parametrize("kind", ["rising", "falling", "spikes", "ramp"])
@pytest.mark.parametrize("S,causal,cq,ck,d", [(128, True, 8, 8, 128), (128, False, 8, 8, 128), (64, True, 4, 4, 128),
                                              (128, True, 32, 32, 128), (128, True, 4, 16, 64), (128, False, 16, 2, 256)])
def test_scores_with_logits_spanning_hundreds_of_units(ctx, oracle, kind, S, causal, cq, ck, d):
    """The compressed-space softmax on the same inputs, in both forms of the score kernel.  The one-sweep form
    stores sums of exponentials relative to a per-row reference that is fixed early and moves only when a tile's sum
    would pass 2^40: "rising" moves it after values were stored (the workgroup then repeats its sweep), "spikes" and
    "ramp" move it inside a tile and from tile to tile, "falling" makes later terms vanish against the first."""
    w = W.steep_logits(kind, H=4, Hkv=2, lengths=(8 * S + 40, 3 * S), S=S, causal=causal, seed=170 + S + cq, d=d)
    w.c_q, w.c_k, w.mode, w.param = cq, ck, W.TOP_P, 0.9
    q, k, _ = PU.device_tensors(w)
    qf, kf, _ = w.f32()
    p, s = PU.problem_of(w), PU.select_of(w)
    m_ref, sc_ref = oracle.build_mask(qf, kf, w.cu_seqlens, S, cq, ck, causal, w.mode, w.param)
    for minimal in (True, False):
        m_dev, sc_dev = ctx.build_mask(p, s, q, k, workspace=ctx.alloc_workspace(p, s, minimal=minimal), want_score=True)
        torch.cuda.synchronize()
        m_gpu, sc_gpu = api.unpack_mask(m_dev, p.n_cols), sc_dev.cpu().numpy()
        assert np.isfinite(sc_gpu).all()
        np.testing.assert_allclose(sc_gpu, sc_ref, rtol=2e-3, atol=1e-6, err_msg=f"minimal={minimal}")
        PU.check_mask_against_oracle(m_gpu, m_ref, sc_ref, w.cu_seqlens, S, causal, w.mode, w.param)
        assert np.array_equal(m_gpu, oracle.select_mask(sc_gpu, w.cu_seqlens, S, causal, w.mode, w.param))


def steep_logits_check(ctx, oracle, kind, S, causal, d):
    """Rows whose logits differ by up to ~190 natural-log units: the attention kernels keep one reference value per
    row for their exponentials and move it only when a probability would grow past a bound, so these inputs drive
    that path (a new reference in every block, in the middle of tiles, in nearly every tile) and its opposite (terms
    that vanish against an early reference).  Dense and block-sparse (random half of the blocks) against the oracle,
    ragged last block included."""
    w = W.steep_logits(kind, H=2, Hkv=1, lengths=(8 * S + 40, 3 * S), S=S, causal=causal, seed=70 + S, d=d)
    q, k, v = PU.device_tensors(w)
    qf, kf, vf = w.f32()
    p = PU.problem_of(w)
    o, lse = ctx.full_attn(p, q, k, v, want_lse=True)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, S, causal, None)
    PU.check_output(o.float().cpu().numpy(), o_ref, f"dense {kind}")
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=1e-3, atol=2e-3)
    rng = np.random.default_rng(5)
    nq, nk = p.n_rows, p.n_cols
    m = (rng.random((2, nq, nk)) < 0.5).astype(np.uint8)
    loc, nb = PU.row_geometry(w.cu_seqlens, S)
    m[:, np.arange(nq), loc] = 1                                   # keep the diagonal so that no row is empty
    if causal:
        m &= (np.arange(nk)[None, :] <= loc[:, None]).astype(np.uint8)[None]
    m &= (np.arange(nk)[None, :] < nb[:, None]).astype(np.uint8)[None]
    o, lse = ctx.sparse_attn(p, q, k, v, api.pack_mask(m), want_lse=True)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, S, causal, m)
    PU.check_output(o.float().cpu().numpy(), o_ref, f"sparse {kind}")
    np.testing.assert_allclose(lse.cpu().numpy(), lse_ref, rtol=1e-3, atol=2e-3)


def test_planted_gqa_4k(ctx, oracle):
    w = W.gqa_planted(L=4096, H=8, Hkv=2, S=128, P=0.95, seed=21)
    PU.full_pipeline_check(ctx, oracle, w)


@pytest.mark.parametrize("cq,ck", [(4, 4), (16, 16), (4, 16), (16, 4), (32, 2), (2, 32), (32, 32), (2, 2)])
def test_other_granularities(ctx, oracle, cq, ck):
    w = W.gqa_planted(L=2048, H=4, Hkv=2, S=128, P=0.9, seed=31)
    w.c_q, w.c_k = cq, ck
    PU.full_pipeline_check(ctx, oracle, w, check_dense=False)


@pytest.mark.parametrize("c_h", [2, 4, 8])
def test_head_compression(ctx, oracle, c_h):
    """c_h inside a GQA group (2, 4) and spanning two key heads (8)."""
    w = W.gqa_planted(L=1024, H=8, Hkv=2, S=128, P=0.9, seed=41)
    w.c_h = c_h
    PU.full_pipeline_check(ctx, oracle, w, check_dense=False)


def test_full_mask_equals_dense_and_empty_rows(ctx, oracle):
    w = W.random_small(H=2, Hkv=1, lengths=(512,), S=128, causal=True, seed=5)
    q, k, v = PU.device_tensors(w)
    p = PU.problem_of(w)
    N = 4
    full = np.tril(np.ones((2, N, N), np.uint8))
    o_s, _ = ctx.sparse_attn(p, q, k, v, api.pack_mask(full))
    o_d, _ = ctx.full_attn(p, q, k, v)
    torch.cuda.synchronize()
    # all blocks selected = dense attention (the two kernels order their softmax arithmetic differently, so equal
    # up to the rounding of the bf16 output, and both within tolerance of the oracle)
    assert (o_s.float() - o_d.float()).abs().max().item() <= 2.0 ** -6
    qf, kf, vf = w.f32()
    o_ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, 128, True, None)
    PU.check_output(o_s.float().cpu().numpy(), o_ref, "sparse with a full mask")
    PU.check_output(o_d.float().cpu().numpy(), o_ref, "dense")
    # garbage bits above the diagonal / beyond the sequence are ignored
    noisy = np.ones((2, N, 64), np.uint8)
    o_n, _ = ctx.sparse_attn(p, q, k, v, api.pack_mask(noisy))
    torch.cuda.synchronize()
    assert torch.equal(o_n, o_s)
    # an empty row gives zeros and lse = -inf, other rows are untouched
    hole = full.copy()
    hole[0, 2, :] = 0
    o_h, lse = ctx.sparse_attn(p, q, k, v, api.pack_mask(hole), want_lse=True)
    torch.cuda.synchronize()
    assert torch.all(o_h[0, 256:384] == 0) and torch.all(torch.isinf(lse[0, 256:384]))
    assert torch.equal(o_h[1], o_s[1]) and torch.equal(o_h[0, :256], o_s[0, :256])


def test_rows_sum_to_one_and_determinism(ctx, oracle):
    w = W.gqa_planted(L=2048, H=4, Hkv=2, S=128, P=0.9, seed=51)
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w), PU.select_of(w)
    m1, sc1 = ctx.build_mask(p, s, q, k, want_score=True)
    m2, sc2 = ctx.build_mask(p, s, q, k, want_score=True)
    ones = torch.ones_like(v)
    o1, _ = ctx.sparse_attn(p, q, k, ones, m1)
    o2, _ = ctx.sparse_attn(p, q, k, v, m1)
    o3, _ = ctx.sparse_attn(p, q, k, v, m2)
    torch.cuda.synchronize()
    assert torch.equal(m1, m2) and torch.equal(sc1, sc2) and torch.equal(o2, o3)      # bit-reproducible
    assert torch.allclose(o1.float(), torch.ones_like(o1, dtype=torch.float32), atol=8e-3)   # weights sum to 1
    np.testing.assert_allclose(sc1.sum(-1).cpu().numpy(), 128 / 8, rtol=1e-4)     # score rows sum to S / c_q


def test_softmax_scale_and_threshold_one(ctx, oracle):
    w = W.random_small(H=2, Hkv=2, lengths=(384,), S=128, causal=True, mode=W.TOP_P, param=1.0, seed=9)
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w, scale=0.05), PU.select_of(w)
    m, _ = ctx.build_mask(p, s, q, k)
    torch.cuda.synchronize()
    assert np.array_equal(api.unpack_mask(m, 3), np.tril(np.ones((2, 3, 3), np.uint8)))   # P = 1 keeps all valid
    o, _ = ctx.full_attn(p, q, k, v)
    torch.cuda.synchronize()
    qf, kf, vf = w.f32()
    ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, 128, True, None, scale=0.05)
    PU.check_output(o.float().cpu().numpy(), ref, "scaled dense")


def test_error_paths(ctx):
    w = W.random_small(H=2, Hkv=1, lengths=(256,), S=128)
    q, k, v = PU.device_tensors(w)
    bad = api.Problem([0, 256], 3, 2, 128, True)                 # query heads not a multiple of key heads
    with pytest.raises(api.UnisparseError) as e:
        ctx.full_attn(bad, q, k, v)
    assert e.value.code == 2
    p = PU.problem_of(w)
    with pytest.raises(api.UnisparseError) as e:
        ctx.build_mask(p, api.Select(c_q=3), q, k)
    assert e.value.code == 2
    overlapping = torch.as_strided(q, q.shape, (q.stride(0), 64, 1))   # token rows 64 elements apart: they overlap
    with pytest.raises(api.UnisparseError) as e:
        ctx.full_attn(p, overlapping, k, v)
    assert e.value.code == 2
    with pytest.raises(api.UnisparseError) as e:
        ctx.build_mask(p, api.Select(c_q=1), q, k)               # S / c = 128: no kernel
    assert e.value.code == 4
    with pytest.raises(api.UnisparseError) as e:
        ctx.build_mask(p, api.Select(threshold=1.5), q, k)
    assert e.value.code == 3
    with pytest.raises(api.UnisparseError) as e:
        ctx.build_mask(p, api.Select(pool=2), q, k)              # stochastic pooling without its uniform numbers
    assert e.value.code == 1
    with pytest.raises(api.UnisparseError) as e:
        ctx.build_mask(p, api.Select(pool=3), q, k)
    assert e.value.code == 3
    with pytest.raises(api.UnisparseError) as e:
        ctx.build_mask(p, api.Select(), q, k, workspace=torch.empty(1024, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 5


def test_config2_shape_sampled_rows(ctx, oracle):
    """Llama-3-8B-shaped layer at L = 32K (GQA 32/8, Top-P 0.95): full GPU run, oracle on sampled outputs."""
    r = PU.sampled_config_check(ctx, oracle, W.gqa_planted(), seed=1, attn_heads=(0, 13, 31), dense_heads=(5,))
    assert 0.2 < r["density"] < 0.8


def test_config3_headline_shape_sampled_rows(ctx, oracle):
    """The benchmarked configuration itself (GQA 32/8, L = 128K, S = 128, Top-P 0.9): the mask, the block-sparse and
    the dense kernel as bench.py launches them; selection bit-exact on all 32768 rows, scores / mask on ~20 rows of
    every head, attention on 5-6 rows of three heads (sparse) and two rows of two heads (dense)."""
    r = PU.sampled_config_check(ctx, oracle, W.gqa_zipf(), seed=3, attn_heads=(0, 13, 31), dense_heads=(2, 29))
    assert 0.2 < r["density"] < 0.5


def test_config4_video_shape_sampled_rows(ctx, oracle):
    """Configuration 4 at its own shape: 40 heads without grouping, 64K tokens of a 16 x 64 x 64 grid, non-causal,
    fixed 20 % budget (512 key blocks per row: eight mask words, every key block valid on every row)."""
    w = W.video_field()
    r = PU.sampled_config_check(ctx, oracle, w, seed=4, attn_heads=(0, 17, 39), dense_heads=(21,))
    assert abs(r["density"] - np.ceil(0.2 * 512) / 512) < 1e-9            # the budget is met exactly on every row


def test_config5_packed_shape_threshold_sweep(ctx, oracle):
    """Configuration 5 at its own shape: four packed causal sequences of 8K, 16K, 32K and 64K tokens (GQA 32/8) in one
    launch, and the threshold sweep P in {0.8, 0.9, 0.95, 0.99} through unisparse_select_blocks on one score buffer:
    density must grow with P."""
    w = W.gqa_varlen()
    r = PU.sampled_config_check(ctx, oracle, w, seed=5, attn_heads=(0, 14, 31), attn_random=3, dense_heads=(9,),
                                extra_thresholds=(0.8, 0.95, 0.99))
    d = r["densities"]
    assert d[0.8] < d[0.9] < d[0.95] < d[0.99] <= 1.0


def test_empty_sequences_in_the_batch(ctx, oracle):
    """Zero-length sequences take no rows and change nothing for their neighbours."""
    w = W.random_small(H=4, Hkv=2, lengths=(128, 0, 256, 0), S=128, causal=True, mode=W.TOP_P, param=0.9, seed=15)
    PU.full_pipeline_check(ctx, oracle, w)
    w2 = W.random_small(H=4, Hkv=2, lengths=(128, 256), S=128, causal=True, mode=W.TOP_P, param=0.9, seed=15)
    assert np.array_equal(w.q, w2.q)                                  # same tokens, only the sequence table differs
    q, k, v = PU.device_tensors(w)
    m1, _ = ctx.build_mask(PU.problem_of(w), PU.select_of(w), q, k)
    m2, _ = ctx.build_mask(PU.problem_of(w2), PU.select_of(w2), q, k)
    o1, _ = ctx.sparse_attn(PU.problem_of(w), q, k, v, m1)
    o2, _ = ctx.sparse_attn(PU.problem_of(w2), q, k, v, m2)
    torch.cuda.synchronize()
    assert torch.equal(m1, m2) and torch.equal(o1, o2)


def test_maximum_block_count(ctx, oracle):
    """One head at the largest supported sequence: 4096 blocks of 128 tokens (L = 512K).  Oracle on sampled rows."""
    S, N = 128, 4096
    w = W.random_small(H=1, Hkv=1, lengths=(N * S,), S=S, causal=True, mode=W.TOP_K, param=0.02, seed=16)
    rows = [0, 1, 2047, N - 1]
    q, k, v = PU.device_tensors(w)
    qf, kf, vf = w.f32()
    p, s = PU.problem_of(w), PU.select_of(w)
    m_dev, sc_dev = ctx.build_mask(p, s, q, k, want_score=True)
    torch.cuda.synchronize()
    m_gpu = api.unpack_mask(m_dev, p.n_cols)
    m_ref, sc_ref = oracle.build_mask(qf, kf, w.cu_seqlens, S, w.c_q, w.c_k, True, w.mode, w.param, rows=rows)
    np.testing.assert_allclose(sc_dev.cpu().numpy()[:, rows], sc_ref[:, rows], rtol=2e-3, atol=1e-6)
    PU.check_mask_against_oracle(m_gpu, m_ref, sc_ref, w.cu_seqlens, S, True, w.mode, w.param, rows)
    k_i = np.maximum(1, np.ceil(0.02 * np.arange(1, N + 1)))
    assert np.array_equal(m_gpu[0].sum(-1), k_i)                      # the budget is met exactly on every row
    o_dev, _ = ctx.sparse_attn(p, q, k, v, m_dev)
    torch.cuda.synchronize()
    o_ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, S, True, m_gpu, rows=[0, N - 1])
    PU.check_output(o_dev.float().cpu().numpy(), o_ref, "max-size sparse")


@pytest.mark.parametrize("lengths", [(256, 384), (133, 37, 300)])
def test_max_pooling_option(ctx, oracle, lengths):
    """The max-pooling alternative of the compression-strategy ablation, whole and partial windows."""
    w = W.random_small(H=4, Hkv=2, lengths=lengths, S=128, causal=True, mode=W.TOP_P, param=0.85, seed=18)
    w.pool = 1
    PU.full_pipeline_check(ctx, oracle, w, check_dense=False)


@pytest.mark.parametrize("lengths,S,cq,ck,layout", [((256, 384), 128, 8, 8, "htd"), ((133, 37, 300), 128, 16, 4, "thd"),
                                                     ((192, 70), 64, 2, 16, "htd"), ((512,), 128, 32, 32, "htd")])
def test_stochastic_pooling_option(ctx, oracle, lengths, S, cq, ck, layout):
    """Stochastic pooling of the compression-strategy ablation: the token drawn in every window equals the oracle's
    bit for bit (same uniform numbers, same fp32 inversion), whole and clipped windows, then the usual pipeline."""
    w = W.random_small(H=4, Hkv=2, lengths=lengths, S=S, causal=True, mode=W.TOP_P, param=0.85, seed=23)
    w.c_q, w.c_k = cq, ck
    w.draw_pool_uniforms()
    PU.full_pipeline_check(ctx, oracle, w, layout=layout, check_dense=False)
    # key side alone (its own uniform numbers), and magnitudes spread over four orders so the draw is far from uniform
    rng = np.random.default_rng(5)
    kf = w.f32()[1] * np.exp(rng.uniform(-4.0, 4.0, size=(w.n_heads_kv, w.total_tokens, 1))).astype(np.float32)
    kb = W.f32_to_bf16_bits(kf)
    kf = W.bf16_bits_to_f32(kb)
    p = PU.problem_of(w)
    kt = ctx.pool_seq_varlen(p, api.bits_to_device(kb), ck, "htd", 2, torch.from_numpy(w.rand_k).cuda())
    torch.cuda.synchronize()
    kt_bits = kt.view(torch.int16).cpu().numpy().view(np.uint16)
    off = oracle.composite_offsets(w.cu_seqlens, ck)
    for h in range(w.n_heads_kv):
        ref = np.concatenate([oracle.stochpool_seq(kf[h, w.cu_seqlens[b]:w.cu_seqlens[b + 1]], ck,
                                                   w.rand_k[h, off[b]:off[b + 1]]) for b in range(len(lengths))])
        assert np.array_equal(kt_bits[h], W.f32_to_bf16_bits(ref))


def test_one_call_entry_point_equals_two_calls(ctx, oracle):
    """unisparse_attn = build_mask + sparse_attn on the same stream: same mask, same output, bit for bit."""
    w = W.gqa_planted(L=2048, H=4, Hkv=2, S=128, P=0.9, seed=61)
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w), PU.select_of(w)
    m2, _ = ctx.build_mask(p, s, q, k)
    o2, _ = ctx.sparse_attn(p, q, k, v, m2)
    o1, m1 = ctx.attn(p, s, q, k, v)
    torch.cuda.synchronize()
    assert torch.equal(m1, m2) and torch.equal(o1, o2)
    qf, kf, vf = w.f32()
    o_ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, 128, True, api.unpack_mask(m1, p.n_cols))
    PU.check_output(o1.float().cpu().numpy(), o_ref, "one-call")


def test_ranked_work_order_gives_identical_output(ctx, oracle):
    """unisparse_sparse_attn_ws ranks the rows of every head by their number of selected blocks and changes nothing
    but the order rows are worked on: output and LSE equal unisparse_sparse_attn bit for bit - packed ragged batches,
    every head dimension and block size, grouped and ungrouped heads, a single row, a mask with an empty row - and
    a workspace that is too small is refused."""
    # (rows are ranked when heads x query-block rows pass 512, what the device holds at once: all cases but the fourth)
    cases = [
        dict(H=8, Hkv=2, lengths=(16384,), S=128, causal=True, d=128),
        dict(H=8, Hkv=4, lengths=(3000, 770, 10000, 0, 1290), S=128, causal=True, d=128),
        dict(H=6, Hkv=6, lengths=(6400, 640), S=64, causal=False, d=128),
        dict(H=4, Hkv=1, lengths=(100,), S=128, causal=True, d=128),
        dict(H=8, Hkv=4, lengths=(9000, 3330), S=128, causal=True, d=256),
        dict(H=8, Hkv=4, lengths=(9000, 3330), S=64, causal=False, d=64),
    ]
    for n, c in enumerate(cases):
        w = W.random_small(H=c["H"], Hkv=c["Hkv"], lengths=c["lengths"], S=c["S"], causal=c["causal"], mode=W.TOP_P,
                           param=0.7, seed=300 + n, d=c["d"])
        q, k, v = PU.device_tensors(w)
        p, s = PU.problem_of(w), PU.select_of(w)
        m, _ = ctx.build_mask(p, s, q, k)
        if n == 1:
            m[1, 3] = 0                                        # an empty mask row among the others
        ws = torch.empty(ctx.attn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        o1, l1 = ctx.sparse_attn(p, q, k, v, m, want_lse=True)
        o2, l2 = ctx.sparse_attn(p, q, k, v, m, want_lse=True, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2), f"case {n}"
    with pytest.raises(api.UnisparseError) as e:
        ctx.sparse_attn(p, q, k, v, m, workspace=torch.empty(64, dtype=torch.uint8, device="cuda"))
    assert e.value.code == 5
    # ungrouped heads whose K/V pass the last-level cache eight heads at a time: chunks ordered key head by key head
    w = W.random_small(H=8, Hkv=8, lengths=(262144,), S=128, causal=True, mode=W.TOP_K, param=0.01, seed=320, d=128)
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w), PU.select_of(w)
    m, _ = ctx.build_mask(p, s, q, k)
    ws = torch.empty(ctx.attn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
    o1, l1 = ctx.sparse_attn(p, q, k, v, m, want_lse=True)
    o2, l2 = ctx.sparse_attn(p, q, k, v, m, want_lse=True, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2), "key-head-major order"
    del q, k, v, o1, o2, w
    # the largest row count that is ranked (8192 rows: the whole sort buffer) and the first that is not
    for nq, lengths in ((8192, (4096 * 64, 4096 * 64)), (8200, (4096 * 64, 4096 * 64, 8 * 64))):
        w = W.random_small(H=1, Hkv=1, lengths=lengths, S=64, causal=True, mode=W.TOP_K, param=0.004, seed=310, d=64)
        q, k, v = PU.device_tensors(w)
        p, s = PU.problem_of(w), PU.select_of(w)
        m, _ = ctx.build_mask(p, s, q, k)
        ws = torch.empty(ctx.attn_workspace_bytes(p), dtype=torch.uint8, device="cuda")
        o1, l1 = ctx.sparse_attn(p, q, k, v, m, want_lse=True)
        o2, l2 = ctx.sparse_attn(p, q, k, v, m, want_lse=True, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2), f"{nq} rows"


def test_strided_views(ctx, oracle):
    """Q, K, V and O as views into larger buffers: padded token and head strides, non-zero storage offset."""
    w = W.random_small(H=4, Hkv=2, lengths=(256, 100), S=128, causal=True, mode=W.TOP_P, param=0.9, seed=19)
    q, k, v = PU.device_tensors(w)                         # [H, T, d] contiguous
    T = w.total_tokens

    def padded(x):
        big = torch.zeros((x.shape[0] + 1, T + 3, 128 + 24), dtype=torch.bfloat16, device="cuda")
        view = big[1:, 2:2 + T, 8:136]                     # head stride, token stride 152, offset 8 elements
        view.copy_(x)
        return view

    qp, kp, vp = padded(q), padded(k), padded(v)
    p, s = PU.problem_of(w), PU.select_of(w)
    m1, sc1 = ctx.build_mask(p, s, q, k, want_score=True)
    m2, sc2 = ctx.build_mask(p, s, qp, kp, want_score=True)
    o1, l1 = ctx.sparse_attn(p, q, k, v, m1, want_lse=True)
    out = padded(torch.zeros_like(q))
    o2, l2 = ctx.sparse_attn(p, qp, kp, vp, m2, out=out, want_lse=True)
    d1, _ = ctx.full_attn(p, q, k, v)
    d2, _ = ctx.full_attn(p, qp, kp, vp)
    torch.cuda.synchronize()
    assert torch.equal(m1, m2) and torch.equal(sc1, sc2)
    assert torch.equal(o1, o2.contiguous()) and torch.equal(l1, l2) and torch.equal(d1, d2.contiguous())


def test_randomised_small_problems(ctx, oracle):
    """Sixty seeded draws over everything a call can vary -- block size, both compression factors, head counts and
    head compression, 1-3 packed sequences of arbitrary lengths, causal or not, Top-P or budget, pooling strategy,
    memory layout -- each through the whole pipeline check."""
    for it in range(60):
        rng = np.random.default_rng(4000 + it)
        S = int(rng.choice([64, 128]))
        cs = [c for c in (1, 2, 4, 8, 16, 32) if S // c in (4, 8, 16, 32, 64)]
        cq, ck = int(rng.choice(cs)), int(rng.choice(cs))
        Hkv, G = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4]))
        H = Hkv * G
        ch = int(rng.choice([c for c in (1, 2, 4, 8) if H % c == 0 and (G % c == 0 or c % G == 0)]))
        nseq = int(rng.integers(1, 4))
        lengths = tuple(int(x) for x in rng.integers(1, int(rng.choice([300, 900])), nseq))
        if rng.random() < 0.3:
            lengths = tuple(int(S * rng.integers(1, 6)) for _ in range(nseq))
        causal = bool(rng.random() < 0.7)
        mode = W.TOP_P if rng.random() < 0.6 else W.TOP_K
        param = float(rng.choice([0.5, 0.8, 0.9, 0.95, 1.0] if mode == W.TOP_P else [0.1, 0.25, 0.5, 1.0]))
        pool = int(rng.choice([0, 0, 1, 2]))
        layout = str(rng.choice(["htd", "thd"]))
        w = W.random_small(H=H, Hkv=Hkv, lengths=lengths, S=S, causal=causal, mode=mode, param=param, seed=900 + it,
                           scale=float(rng.choice([0.5, 1.0, 1.5])))
        w.c_q, w.c_k, w.c_h, w.pool = cq, ck, ch, pool
        if pool == 2:
            w.draw_pool_uniforms()
        try:
            PU.full_pipeline_check(ctx, oracle, w, layout=layout)
        except AssertionError as e:
            raise AssertionError(f"draw {it}: S={S} c=({cq},{ck},{ch}) H={H}/{Hkv} lengths={lengths} causal={causal} "
                                 f"mode={mode} param={param} pool={pool} {layout}: {e}") from e


@pytest.mark.parametrize("lengths,S,cq,ck,ch,causal", [
    ((1000, 77, 300), 128, 8, 8, 1, True), ((513, 2049), 128, 8, 8, 1, False), ((700, 131), 64, 4, 16, 2, True),
    ((333,), 128, 2, 2, 1, True), ((900, 260), 128, 16, 2, 4, False), ((1500,), 64, 8, 8, 1, True)])
def test_nothing_is_read_from_the_workspace_before_it_is_written(ctx, oracle, lengths, S, cq, ck, ch, causal):
    """build_mask and sparse_attn_ws leave the same bits whether the workspace held zeros or 0xFF bytes (NaN as
    floats, -1 as integers) before the call, in both forms of the score computation: every value they read from it
    they wrote earlier in the same call (rows past a sequence's end, key blocks past a row's valid set and padding
    included)."""
    w = W.random_small(H=4, Hkv=2, lengths=lengths, S=S, causal=causal, mode=W.TOP_P, param=0.9, seed=31 + S + cq)
    w.c_q, w.c_k, w.c_h = cq, ck, ch
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w), PU.select_of(w)
    for minimal in (False, True):
        res = []
        for fill in (0, 255):
            ws = ctx.alloc_workspace(p, s, minimal=minimal)
            ws.fill_(fill)
            m = ctx.alloc_mask(p)
            m.fill_(-1 if fill else 0)
            m, sc = ctx.build_mask(p, s, q, k, workspace=ws, mask=m, want_score=True)
            o, lse = ctx.sparse_attn(p, q, k, v, m, want_lse=True, workspace=ws)
            torch.cuda.synchronize()
            res.append((m.clone(), sc.clone(), o.clone(), lse.clone()))
        for a, b in zip(*res):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"minimal={minimal}"
        assert torch.isfinite(res[0][1]).all()


def test_randomised_medium_problems(ctx, oracle):
    """Twenty-four seeded problems of 2K-14K tokens per sequence (many key stages per sweep of the score kernel, several
    workgroups per head, all head dimensions), a third of them with logits that rise, fall, spike or ramp over hundreds
    of units; scores, mask and attention against the oracle on sampled query-block rows."""
    for it in range(24):
        rng = np.random.default_rng(52000 + it)
        d = int(rng.choice([128, 128, 64, 256]))
        S = int(rng.choice([64, 128]))
        cs = [c for c in (2, 4, 8, 16, 32) if S // c in (4, 8, 16, 32, 64)]
        cq, ck = int(rng.choice(cs)), int(rng.choice(cs))
        Hkv, G = int(rng.choice([1, 2])), int(rng.choice([1, 2, 4]))
        H = Hkv * G
        ch = int(rng.choice([1, 1] + [c for c in (1, 2, 4) if H % c == 0 and (G % c == 0 or c % G == 0)]))
        nseq = int(rng.integers(1, 4))
        lengths = tuple(int(x) for x in rng.integers(2000, 14000, nseq))
        causal = bool(rng.random() < 0.7)
        mode = W.TOP_P if rng.random() < 0.6 else W.TOP_K
        param = float(rng.choice([0.5, 0.8, 0.9, 0.95] if mode == W.TOP_P else [0.1, 0.25, 0.5]))
        layout = str(rng.choice(["htd", "thd"]))
        kind = str(rng.choice(["random", "random", "rising", "spikes", "ramp", "falling"]))
        if kind == "random":
            w = W.random_small(H=H, Hkv=Hkv, lengths=lengths, S=S, causal=causal, mode=mode, param=param,
                               seed=2900 + it, scale=float(rng.choice([0.5, 1.0, 1.5])), d=d)
        else:
            step = float(rng.choice([2.0, 8.0, 16.0])) / (max(lengths) // S / 8 + 1)
            w = W.steep_logits(kind, H=H, Hkv=Hkv, lengths=lengths, S=S, causal=causal, seed=2900 + it, d=d, step=step)
            w.mode, w.param = mode, param
        w.c_q, w.c_k, w.c_h = cq, ck, ch
        NQ = sum(-(-L // S) for L in lengths)
        rows = sorted(set(int(x) for x in rng.integers(0, NQ, 5)) | {NQ - 1, 0})
        try:
            PU.full_pipeline_check(ctx, oracle, w, layout=layout, check_dense=(it % 4 == 0), rows=rows)
        except AssertionError as e:
            raise AssertionError(f"draw {it}: {kind} d={d} S={S} c=({cq},{ck},{ch}) H={H}/{Hkv} lengths={lengths} "
                                 f"causal={causal} mode={mode} param={param} {layout} rows={rows}: {e}") from e


@pytest.mark.parametrize("d", [64, 256])
@pytest.mark.parametrize("S,lengths,cq,ck,ch,causal,mode,param,pool,layout", [
    (128, (512, 384), 8, 8, 1, True, W.TOP_P, 0.9, 0, "htd"),
    (128, (300, 77, 1000), 16, 4, 2, True, W.TOP_K, 0.3, 0, "thd"),
    (64, (448,), 4, 4, 1, False, W.TOP_P, 0.8, 1, "htd"),
    (64, (130, 257), 2, 16, 4, True, W.TOP_P, 0.95, 2, "thd"),
    (128, (640,), 32, 2, 1, False, W.TOP_K, 0.5, 0, "htd"),
])
def test_other_head_dims(ctx, oracle, d, S, lengths, cq, ck, ch, causal, mode, param, pool, layout):
    """Head dimensions 64 and 256: every stage against the oracle (whole and ragged sequences, every pooling strategy,
    head compression, both layouts), sparse and dense attention."""
    w = W.random_small(H=4, Hkv=2, lengths=lengths, S=S, causal=causal, mode=mode, param=param, seed=29, d=d)
    w.c_q, w.c_k, w.c_h, w.pool = cq, ck, ch, pool
    if pool == 2:
        w.draw_pool_uniforms()
    PU.full_pipeline_check(ctx, oracle, w, layout=layout)


def test_other_head_dims_randomised(ctx, oracle):
    """Forty seeded random small problems at head dimensions 64 and 256 (same draws as the test above for 128)."""
    for it in range(40):
        rng = np.random.default_rng(7000 + it)
        d = int(rng.choice([64, 256]))
        S = int(rng.choice([64, 128]))
        cs = [c for c in (1, 2, 4, 8, 16, 32) if S // c in (4, 8, 16, 32, 64)]
        cq, ck = int(rng.choice(cs)), int(rng.choice(cs))
        Hkv, G = int(rng.choice([1, 2])), int(rng.choice([1, 2, 4]))
        H = Hkv * G
        ch = int(rng.choice([c for c in (1, 2, 4, 8) if H % c == 0 and (G % c == 0 or c % G == 0)]))
        nseq = int(rng.integers(1, 4))
        lengths = tuple(int(x) for x in rng.integers(1, 700, nseq))
        causal = bool(rng.random() < 0.7)
        mode = W.TOP_P if rng.random() < 0.6 else W.TOP_K
        param = float(rng.choice([0.5, 0.8, 0.9, 1.0] if mode == W.TOP_P else [0.1, 0.25, 1.0]))
        pool = int(rng.choice([0, 0, 1, 2]))
        layout = str(rng.choice(["htd", "thd"]))
        w = W.random_small(H=H, Hkv=Hkv, lengths=lengths, S=S, causal=causal, mode=mode, param=param, seed=950 + it,
                           scale=float(rng.choice([0.5, 1.0])), d=d)
        w.c_q, w.c_k, w.c_h, w.pool = cq, ck, ch, pool
        if pool == 2:
            w.draw_pool_uniforms()
        try:
            PU.full_pipeline_check(ctx, oracle, w, layout=layout)
        except AssertionError as e:
            raise AssertionError(f"draw {it}: d={d} S={S} c=({cq},{ck},{ch}) H={H}/{Hkv} lengths={lengths} "
                                 f"causal={causal} mode={mode} param={param} pool={pool} {layout}: {e}") from e


@pytest.mark.parametrize("N,causal", [(5, True), (64, True), (65, False), (200, True), (1024, False), (4096, True)])
def test_selection_on_crafted_scores(ctx, oracle, N, causal):
    """unisparse_select_blocks on hand-made score rows where ties, zeros and the position of the cut are under
    control: heavy ties (scores quantised to a few levels), uniform rows, all-zero rows, one dominant block,
    a cut that falls exactly on a level boundary; every threshold / budget; bit-exact against the oracle."""
    S, H = 64, 3
    rng = np.random.default_rng(N)
    p = api.Problem([0, N * S], H, 1, S, causal)
    score = np.zeros((H, N, N), dtype=np.float32)
    kinds = ["levels", "uniform", "zeros", "dominant", "random", "pow2", "sparse"]
    for h in range(H):
        for r in range(N):
            kind = kinds[(r + h) % len(kinds)]
            if kind == "levels":
                row = rng.integers(0, 4, N).astype(np.float32) / 8.0           # exact in fp32/fp64: ties everywhere
            elif kind == "uniform":
                row = np.full(N, 0.25, np.float32)
            elif kind == "zeros":
                row = np.zeros(N, np.float32)
            elif kind == "dominant":
                row = np.full(N, 2.0 ** -20, np.float32)
                row[rng.integers(0, N)] = 1.0
            elif kind == "pow2":
                row = (2.0 ** -rng.integers(0, 12, N)).astype(np.float32)      # sums exact: cuts land on boundaries
            elif kind == "sparse":
                row = np.where(rng.random(N) < 0.1, rng.random(N), 0.0).astype(np.float32)
            else:
                row = rng.random(N).astype(np.float32) ** 4
            score[h, r] = row
    rows = None if N <= 1024 else sorted({0, 1, 63, 64, 65, N - 1, *[int(x) for x in rng.integers(0, N, 40)]})
    for mode, params in ((W.TOP_P, (0.25, 0.5, 0.75, 0.9, 1.0)), (W.TOP_K, (0.01, 0.25, 0.5, 1.0))):
        for param in params:
            s = api.Select(mode=mode, threshold=param if mode == W.TOP_P else 0.9,
                           budget_frac=param if mode == W.TOP_K else 0.25)
            sc_dev = torch.from_numpy(score).cuda()
            m_dev = ctx.select_blocks(p, s, sc_dev)
            torch.cuda.synchronize()
            m_gpu = api.unpack_mask(m_dev, p.n_cols)
            m_ref = oracle.select_mask(score, [0, N * S], S, causal, mode, param, rows)
            rr = slice(None) if rows is None else rows
            bad = np.argwhere(m_gpu[:, rr] != m_ref[:, rr])
            assert len(bad) == 0, f"mode {mode} param {param}: first mismatches (head, row, col) {bad[:5].tolist()}"
            if causal:                                   # the call also clears the scores outside the valid set
                assert not np.triu(sc_dev.cpu().numpy(), 1).any()


def test_maximum_sequence_count(ctx, oracle):
    """Sixty-four packed sequences (the limit), some empty, some shorter than a block or a pooling window; one more
    is refused."""
    rng = np.random.default_rng(33)
    lengths = [int(x) for x in rng.integers(1, 300, 64)]
    lengths[3] = 0
    lengths[9] = 5
    lengths[40] = 1
    lengths[63] = 0
    w = W.random_small(H=4, Hkv=2, lengths=lengths, S=64, causal=True, mode=W.TOP_P, param=0.9, seed=34)
    w.c_q, w.c_k = 8, 4
    PU.full_pipeline_check(ctx, oracle, w, layout="thd")
    q, k, v = PU.device_tensors(w)
    too_many = api.Problem([0] + list(np.cumsum([8] * 65)), 4, 2, 64, True)
    with pytest.raises(api.UnisparseError) as e:
        ctx.full_attn(too_many, q, k, v)
    assert e.value.code == 2


def test_graph_capture_and_replay(ctx, oracle):
    """After one ordinary call the entry points only launch kernels, so mask + sparse attention can be captured in
    a HIP graph; three replays, with eager work and synchronisation in between, reproduce the eager result bit
    for bit."""
    w = W.gqa_planted(L=2048, H=4, Hkv=2, S=128, P=0.9, seed=62)
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w), PU.select_of(w)
    ws = ctx.alloc_workspace(p, s)
    m_e, o_e = ctx.alloc_mask(p), torch.empty_like(q)
    ctx.build_mask(p, s, q, k, workspace=ws, mask=m_e)
    ctx.sparse_attn(p, q, k, v, m_e, out=o_e)
    torch.cuda.synchronize()
    m_g, o_g = ctx.alloc_mask(p), torch.empty_like(q)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.build_mask(p, s, q, k, workspace=ws, mask=m_g)
        ctx.sparse_attn(p, q, k, v, m_g, out=o_g)
    for rep in range(3):
        m_g.fill_(-1)
        o_g.fill_(7.0)
        od, _ = ctx.full_attn(p, q, k, v)                  # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(m_g, m_e), f"replay {rep}: mask differs"
        assert torch.equal(o_g, o_e), f"replay {rep}: output differs"
    qf, kf, vf = w.f32()
    o_ref, _ = oracle.masked_attention(qf, kf, vf, w.cu_seqlens, 128, True, api.unpack_mask(m_g, p.n_cols))
    PU.check_output(o_g.float().cpu().numpy(), o_ref, "graph replay")


def test_tuning_picks_a_tiling_and_keeps_the_mask(ctx, oracle):
    w = W.gqa_planted(L=4096, H=4, Hkv=2, S=128, P=0.9, seed=63)
    q, k, v = PU.device_tensors(w)
    p, s = PU.problem_of(w), PU.select_of(w)
    m0, _ = ctx.build_mask(p, s, q, k)
    ctx.tune(p, s, q, k)
    assert s.proxy_tiles in (1, 2)
    m1, _ = ctx.build_mask(p, s, q, k)
    torch.cuda.synchronize()
    assert torch.equal(m0, m1)
