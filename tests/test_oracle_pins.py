"""Pins for the CPU oracle: each oracle function is checked against something that is not
itself -- hand-worked fixtures, closed forms, invariants, brute force on tiny inputs, and
special cases that reduce to a library routine (torch softmax / scaled_dot_product_attention /
avg_pool1d / bfloat16 casts).  None of these tests needs a GPU."""
import itertools
import os

import numpy as np
import pytest
import torch

from paper_2512_14082_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16_values(rng, shape, scale=1.0):
    x = (scale * rng.standard_normal(shape)).astype(np.float32)
    return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()


# ----------------------------------------------------------------------------- bf16 rounding

def test_bf16_rounding_matches_torch_cast(oracle):
    lib = oracle._load()
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.standard_normal(2000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 2000),
                         np.array([1.00390625, 1.01171875, 1.005859375, 0.0, -0.0, 3.0e38, 1e-40], np.float32)])
    ref = torch.from_numpy(xs).to(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([lib.oracle_bf16_round_scalar(float(x)) for x in xs], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32))


def test_generator_bf16_helpers_match_torch_cast():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(4096).astype(np.float32)
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits, ref.view(torch.int16).numpy().view(np.uint16))
    assert np.array_equal(W.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())


# ----------------------------------------------------------------------------- pooling, Eq. (1)

def test_pool_identity_constant_and_ramp(oracle):
    rng = np.random.default_rng(2)
    x = bf16_values(rng, (64, 16))
    assert np.array_equal(oracle.avgpool_seq(x, 1), x)                       # c = 1 is the identity
    c = np.full((64, 16), 0.71875, np.float32)
    assert np.array_equal(oracle.avgpool_seq(c, 8), c[:8])                   # mean of a constant
    ramp = np.repeat(np.arange(64, dtype=np.float32)[:, None], 4, axis=1)    # token index as value
    out = oracle.avgpool_seq(ramp, 8)
    assert np.array_equal(out[:, 0], np.arange(8) * 8 + 3.5)                 # window mid-points, 0-based windows


@pytest.mark.parametrize("c", [2, 4, 8, 16, 32])
def test_pool_matches_torch_avg_pool_on_bf16(oracle, c):
    rng = np.random.default_rng(3 + c)
    x = bf16_values(rng, (256, 128))
    ref = torch.nn.functional.avg_pool1d(torch.from_numpy(x).T[None], c, c)[0].T
    ref = ref.to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.avgpool_seq(x, c), ref)


def test_head_pool_matches_mean(oracle):
    rng = np.random.default_rng(5)
    x = bf16_values(rng, (8, 32, 16))
    ref = torch.from_numpy(x).reshape(4, 2, 32, 16).mean(1).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.avgpool_head(x, 2), ref)


# ----------------------------------------------------------------------------- scores, Eq. (3)-(4)

def brute_block_mass(q, k, S, causal):
    """Textbook softmax attention matrix (torch, fp64) summed over S x S blocks."""
    q = torch.from_numpy(q).double()
    k = torch.from_numpy(k).double()
    L, d = q.shape
    p = q @ k.T / np.sqrt(d)
    if causal:
        p = p.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    a = torch.softmax(p, dim=-1)
    N = L // S
    return a.reshape(N, S, N, S).sum(dim=(1, 3)).numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_scores_c1_equal_exact_attention_block_mass(oracle, causal):
    """With c_q = c_k = 1 the proxy *is* the attention matrix: pins logits, scale, causal rule,
    softmax and the R_x index mapping against torch."""
    rng = np.random.default_rng(10)
    q = bf16_values(rng, (96, 32), 1.5)
    k = bf16_values(rng, (96, 32), 1.5)
    sc = oracle.block_scores_head(q, k, S=16, c_q=1, c_k=1, causal_mode=int(causal), scale=1 / np.sqrt(32))
    np.testing.assert_allclose(sc, brute_block_mass(q, k, 16, causal), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("c", [2, 8])
def test_scores_equal_attention_over_torch_pooled_tokens(oracle, causal, c):
    """For c_q = c_k = c the proxy is exact attention between the pooled tokens with block S / c."""
    rng = np.random.default_rng(11)
    L, d, S = 512, 64, 64
    q = bf16_values(rng, (1, L, d), 1.3)
    k = bf16_values(rng, (1, L, d), 1.3)
    pool = lambda x: torch.nn.functional.avg_pool1d(torch.from_numpy(x).T[None], c, c)[0].T \
        .to(torch.bfloat16).to(torch.float32).numpy()
    ref = brute_block_mass(pool(q[0]), pool(k[0]), S // c, causal) * 1.0
    # brute_block_mass scales by 1/sqrt(d): same d, so directly comparable
    got = oracle.block_scores(q, k, [0, L], S, c, c, causal)[0]
    if causal:
        ref = np.tril(ref)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-13)


def test_scores_asymmetric_noncausal_matches_torch(oracle):
    rng = np.random.default_rng(12)
    L, d, S = 256, 32, 64
    q = bf16_values(rng, (L, d))
    k = bf16_values(rng, (L, d))
    cq, ck = 4, 16
    pool = lambda x, c: torch.nn.functional.avg_pool1d(torch.from_numpy(x).T[None], c, c)[0].T \
        .to(torch.bfloat16).double()
    a = torch.softmax(pool(q, cq) @ pool(k, ck).T / np.sqrt(d), -1)
    N = L // S
    ref = a.reshape(N, S // cq, N, S // ck).sum(dim=(1, 3)).numpy()
    got = oracle.block_scores(q[None], k[None], [0, L], S, cq, ck, False)[0]
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("cq,ck", [(8, 8), (4, 16), (16, 4), (2, 32)])
def test_score_rows_sum_to_composites_per_block(oracle, cq, ck):
    """Every composite row of A~ sums to 1, so a score row sums to S / c_q; the causal cut keeps all of
    it because a key window that starts after the query window's last token is never visible."""
    rng = np.random.default_rng(13)
    L, d, S = 512, 32, 64
    q = bf16_values(rng, (2, L, d))
    k = bf16_values(rng, (1, L, d))
    for causal in (False, True):
        sc = oracle.block_scores(q, k, [0, L], S, cq, ck, causal)
        np.testing.assert_allclose(sc.sum(-1), S / cq, rtol=1e-12)
        if causal:
            assert np.all(np.triu(sc[0], 1) == 0)
        assert np.all(sc >= 0)


def token_window_visibility(L, cq, ck):
    """Composite-level causal visibility stated on TOKENS, not on composite indices: take the textbook
    token-level causal matrix (key s may be seen by query t iff s <= t) and call composite key s'
    visible to composite query t' iff ANY (query token, key token) pair of their two windows is
    causally allowed.  Windows are the clipped, non-overlapping ones of Eq. (1)."""
    tok = np.tril(np.ones((L, L), dtype=bool))                 # [query token, key token]
    Lq, Lk = -(-L // cq), -(-L // ck)
    vis = np.zeros((Lq, Lk), dtype=bool)
    for t in range(Lq):
        for s in range(Lk):
            vis[t, s] = tok[t * cq:min(L, (t + 1) * cq), s * ck:min(L, (s + 1) * ck)].any()
    return vis


def torch_asymmetric_causal_scores(q, k, S, cq, ck, vis):
    """Eq. (3)-(4) over a torch softmax of the torch-pooled logits restricted to ``vis``."""
    L, d = q.shape
    pool = lambda x, c: torch.nn.functional.avg_pool1d(torch.from_numpy(x).T[None], c, c, ceil_mode=True)[0].T \
        .to(torch.bfloat16).double()
    p = pool(q, cq) @ pool(k, ck).T / np.sqrt(d)
    p = p.masked_fill(~torch.from_numpy(vis), float("-inf"))
    a = torch.softmax(p, dim=-1).numpy()
    N = -(-L // S)
    ref = np.zeros((N, N))
    for t in range(a.shape[0]):
        for s in range(a.shape[1]):
            ref[(t * cq) // S, (s * ck) // S] += a[t, s]          # t' in R_q(i), s' in R_k(j)
    return np.tril(ref)                                           # block-level cut of Alg. 1 step 4


@pytest.mark.parametrize("S", [64, 128])
@pytest.mark.parametrize("cq,ck", [(32, 2), (16, 4), (4, 16), (2, 32)])
def test_scores_asymmetric_causal_match_token_window_visibility(oracle, cq, ck, S):
    """Pins the valid attention range of a composite query when c_q != c_k (Sec. 5 "Fused Kernel
    Optimization"; the shapes of the ablation "Q-K Compression Ratio Allocation") against a visibility
    matrix built from explicit token windows.  Two other plausible rules are shown to give different
    scores on the same input, so the pin is sensitive to the choice."""
    rng = np.random.default_rng(17 + cq)
    L, d = 4 * S, 32
    q = bf16_values(rng, (L, d), 1.3)
    k = bf16_values(rng, (L, d), 1.3)
    vis = token_window_visibility(L, cq, ck)
    ref = torch_asymmetric_causal_scores(q, k, S, cq, ck, vis)
    got = oracle.block_scores(q[None], k[None], [0, L], S, cq, ck, True)[0]
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-13)
    # alternative rules, again on token windows: (a) the key window must start no later than the FIRST
    # token of the query window; (b) the key window must END no later than the query window's last token
    tok = np.tril(np.ones((L, L), dtype=bool))
    Lq, Lk = L // cq, L // ck
    vis_a = np.array([[tok[t * cq, s * ck] for s in range(Lk)] for t in range(Lq)])
    vis_b = np.array([[tok[(t + 1) * cq - 1, (s + 1) * ck - 1] for s in range(Lk)] for t in range(Lq)])
    vis_b[:, 0] |= ~vis_b.any(axis=1)                             # keep rule (b) free of empty rows
    # with nested windows (a) can differ only when the query window is the longer one, (b) only when the
    # key window is: each is the plausible mistake for one half of the table's shapes
    other = vis_a if cq > ck else vis_b
    assert (other != vis).any()
    alt = torch_asymmetric_causal_scores(q, k, S, cq, ck, other)
    assert np.abs(alt - got).max() > 1e-3


def test_scores_asymmetric_causal_ragged_length(oracle):
    """Same pin with a length that neither S nor the compression factors divide."""
    rng = np.random.default_rng(18)
    L, d, S = 203, 32, 64
    q = bf16_values(rng, (L, d), 1.3)
    k = bf16_values(rng, (L, d), 1.3)
    for cq, ck in [(4, 16), (16, 4)]:
        ref = torch_asymmetric_causal_scores(q, k, S, cq, ck, token_window_visibility(L, cq, ck))
        got = oracle.block_scores(q[None], k[None], [0, L], S, cq, ck, True)[0]
        np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-13)


def test_scores_asymmetric_causal_constant_input_hand_worked(oracle):
    """Constant Q = K: every visible composite key of a row gets the same weight, so the scores are
    counts worked out by hand from the token windows (L = 16, S = 8, two blocks).

    c_q = 4, c_k = 2: query windows end at tokens 3, 7, 11, 15; key windows start at 0, 2, ..., 14.
      visible keys per composite query: 2, 4, 6, 8.  Block 1 holds queries 2 and 3, block 0 keys 0..3:
      Score(1,0) = 4/6 + 4/8 = 7/6,  Score(1,1) = 2/6 + 4/8 = 5/6,  Score(0,0) = 2/2 + 4/4 = 2.
    c_q = 2, c_k = 4: query windows end at 1, 3, 5, ..., 15; key windows start at 0, 4, 8, 12.
      visible keys per composite query: 1, 1, 2, 2, 3, 3, 4, 4.  Block 1 holds queries 4..7, block 0 keys 0, 1:
      Score(1,0) = 2/3 + 2/3 + 2/4 + 2/4 = 7/3,  Score(1,1) = 1/3 + 1/3 + 2/4 + 2/4 = 5/3,  Score(0,0) = 4.
    ("starts no later than the first query token" would give 4/5 + 4/7 in the first case; "ends no later than
    the last query token" would leave composite query 0 of the second case without any key.)"""
    x = np.full((1, 16, 8), 0.5, np.float32)
    sc = oracle.block_scores(x, x, [0, 16], 8, 4, 2, True)[0]
    np.testing.assert_allclose(sc, [[2.0, 0.0], [7.0 / 6.0, 5.0 / 6.0]], rtol=1e-12)
    sc = oracle.block_scores(x, x, [0, 16], 8, 2, 4, True)[0]
    np.testing.assert_allclose(sc, [[4.0, 0.0], [7.0 / 3.0, 5.0 / 3.0]], rtol=1e-12)


def test_scores_constant_input_closed_form(oracle):
    L, d, S, c = 256, 16, 32, 4
    x = np.full((1, L, d), 0.5, np.float32)
    sc = oracle.block_scores(x, x, [0, L], S, c, c, False)[0]
    np.testing.assert_allclose(sc, (S / c) / (L / S), rtol=1e-12)            # n_q / N everywhere
    # causal: composite row t' sees t'+1 equal keys -> mass 1/(t'+1) each
    sc = oracle.block_scores(x, x, [0, L], S, c, c, True)[0]
    n = S // c
    i, j = 3, 1
    want = sum(n / (t + 1) for t in range(i * n, (i + 1) * n))
    np.testing.assert_allclose(sc[i, j], want, rtol=1e-12)
    want_diag = sum((t - i * n + 1) / (t + 1) for t in range(i * n, (i + 1) * n))
    np.testing.assert_allclose(sc[i, i], want_diag, rtol=1e-12)


def test_scores_causal_ignore_future_keys(oracle):
    rng = np.random.default_rng(14)
    L, d, S, c = 256, 32, 64, 8
    q = bf16_values(rng, (1, L, d))
    k = bf16_values(rng, (1, L, d))
    k2 = k.copy()
    k2[0, 128:] = bf16_values(rng, (128, d), 5.0)                            # perturb blocks 2, 3
    a = oracle.block_scores(q, k, [0, L], S, c, c, True)[0]
    b = oracle.block_scores(q, k2, [0, L], S, c, c, True)[0]
    assert np.array_equal(a[:2], b[:2])
    assert not np.array_equal(a[2:], b[2:])


def test_literal_alg1_variant_differs_only_by_future_mass(oracle):
    """Softmax over all composite keys followed by the block-level cut (the literal order of Alg. 1)
    gives row sums below S/c_q; the two readings agree when there are no future keys (last row, upper part empty)."""
    rng = np.random.default_rng(15)
    L, d, S, c = 256, 32, 64, 8
    q = bf16_values(rng, (1, L, d))
    k = bf16_values(rng, (1, L, d))
    lit = oracle.block_scores(q, k, [0, L], S, c, c, True, literal_alg1=True)[0]
    assert np.all(lit.sum(-1)[:-1] < S / c)
    non = oracle.block_scores(q, k, [0, L], S, c, c, False)[0]
    np.testing.assert_allclose(lit, np.tril(non), rtol=1e-12)


def test_gqa_and_head_compression_mapping(oracle):
    rng = np.random.default_rng(16)
    L, d, S, c = 128, 32, 32, 4
    q = bf16_values(rng, (4, L, d))
    k = bf16_values(rng, (2, L, d))
    sc = oracle.block_scores(q, k, [0, L], S, c, c, True)
    for h in range(4):                                                       # query head h <-> KV head h // 2
        one = oracle.block_scores(q[h:h + 1], k[h // 2:h // 2 + 1], [0, L], S, c, c, True)[0]
        assert np.array_equal(sc[h], one)
    # c_h = 2 inside a GQA group: pooled queries against the (unchanged) shared key head
    sc2 = oracle.block_scores(q, k, [0, L], S, c, c, True, c_h=2)
    assert sc2.shape[0] == 2
    qt = np.stack([oracle.avgpool_seq(q[h], c) for h in range(4)])
    qh = torch.from_numpy(qt).reshape(2, 2, L // c, d).mean(1).to(torch.bfloat16).to(torch.float32).numpy()
    kt = oracle.avgpool_seq(k[1], c)
    ref = np.tril(brute_block_mass(qh[1], kt, S // c, True))
    np.testing.assert_allclose(sc2[1], ref * 1.0, rtol=1e-10, atol=1e-13)


# ----------------------------------------------------------------------------- selection, Eq. (5)

def _read_top_p_fixture():
    rows = []
    with open(os.path.join(GOLDEN, "top_p_worked_examples.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p, sc, sel = [x.strip() for x in line.split("|")]
            rows.append((float(p), [float(x) for x in sc.split()], [int(x) for x in sel.split()]))
    return rows


def test_top_p_hand_worked_examples(oracle):
    rows = _read_top_p_fixture()
    assert len(rows) >= 12
    for P, sc, want in rows:
        sel = oracle.select_row(np.array(sc), oracle.TOP_P, P)
        assert list(np.nonzero(sel)[0]) == want, (P, sc)


def test_top_p_is_minimal_prefix_bruteforce(oracle):
    """Among all subsets with mass >= P*tot the selected one has the fewest blocks, and the largest mass
    among those of that size (= a prefix of the descending order)."""
    rng = np.random.default_rng(20)
    for trial in range(60):
        n = int(rng.integers(1, 9))
        sc = rng.random(n) ** 3 + 1e-3
        P = float(rng.choice([0.3, 0.5, 0.8, 0.9, 0.95, 0.99]))
        sel = oracle.select_row(sc, oracle.TOP_P, P)
        tot = sc.sum()
        best = None
        for r in range(1, n + 1):
            feas = [s for s in itertools.combinations(range(n), r) if sc[list(s)].sum() >= P * tot - 1e-15]
            if feas:
                best = (r, max(sc[list(s)].sum() for s in feas))
                break
        idx = np.nonzero(sel)[0]
        assert len(idx) == best[0]
        np.testing.assert_allclose(sc[idx].sum(), best[1], rtol=1e-12)
        assert sc[idx].min() >= np.delete(sc, idx).max() if len(idx) < n else True


def test_top_p_uniform_and_full(oracle):
    for n, P in [(16, 0.5), (16, 0.3), (10, 0.75), (7, 0.9)]:
        sel = oracle.select_row(np.ones(n), oracle.TOP_P, P)
        kk = int(np.ceil(P * n - 1e-12))
        assert list(np.nonzero(sel)[0]) == list(range(kk))
    sc = np.array([0.0, 3.0, 0.0, 1.0])
    assert oracle.select_row(sc, oracle.TOP_P, 1.0).sum() == 4               # P = 1 keeps every valid block
    assert list(np.nonzero(oracle.select_row(sc, oracle.TOP_P, 0.999))[0]) == [1, 3]


def test_top_k_budget(oracle):
    rng = np.random.default_rng(21)
    for n in [1, 2, 5, 32, 100]:
        for f in [0.25, 0.2, 0.5, 1.0]:
            sc = rng.random(n)
            sel = oracle.select_row(sc, oracle.TOP_K, f)
            kk = max(1, int(np.ceil(f * n)))
            assert sel.sum() == kk
            if kk < n:
                assert sc[sel == 1].min() >= sc[sel == 0].max()
    sel = oracle.select_row(np.array([1.0, 2.0, 2.0, 2.0]), oracle.TOP_K, 0.5)
    assert list(np.nonzero(sel)[0]) == [1, 2]                                # tie -> lower index


def test_mask_structure_and_varlen_independence(oracle):
    w = W.random_small(H=2, Hkv=1, lengths=(128, 256, 64), S=32, causal=True, seed=3)
    q, k, _ = w.f32()
    m, sc = oracle.build_mask(q, k, w.cu_seqlens, 32, 4, 4, True, oracle.TOP_P, 0.8)
    assert m.shape == (2, 14, 8)
    row = 0
    for b, nb in enumerate(w.n_blocks()):
        t0, t1 = w.cu_seqlens[b], w.cu_seqlens[b + 1]
        alone, _ = oracle.build_mask(q[:, t0:t1], k[:, t0:t1], [0, t1 - t0], 32, 4, 4, True, oracle.TOP_P, 0.8)
        assert np.array_equal(m[:, row:row + nb, :nb], alone)
        assert np.all(m[:, row:row + nb, nb:] == 0)                          # no bit beyond the sequence
        for i in range(nb):
            assert np.all(m[:, row + i, i + 1:] == 0)                        # causal: nothing above the diagonal
            assert np.all(m[:, row + i].sum(-1) >= 1)
        row += nb


def test_sparsity_hand_worked_examples(oracle):
    with open(os.path.join(GOLDEN, "sparsity_worked_examples.txt")) as f:
        lines = [l.strip() for l in f if l.strip() and not l.startswith("#")]
    assert len(lines) >= 3
    for line in lines:
        n, rows, frac = [x.strip() for x in line.split("|")]
        n = int(n)
        m = np.zeros((1, n, n), np.uint8)
        for i, r in enumerate(rows.split("/")):
            vals = [int(x) for x in r.split()]
            m[0, i, :len(vals)] = vals
        num, den = [int(x) for x in frac.split()]
        assert abs(oracle.sparsity(m, [0, n * 16], 16, True) - num / den) < 1e-15


# ----------------------------------------------------------------------------- attention, Sec. 2.2

def torch_masked_attention(q, k, v, S, causal, mask):
    """Library routine: scaled_dot_product_attention in fp64 with the token-level expansion of the block mask."""
    q, k, v = [torch.from_numpy(x).double() for x in (q, k, v)]
    L = q.shape[0]
    allowed = torch.from_numpy(np.kron(mask, np.ones((S, S), dtype=np.uint8))).bool()
    if causal:
        allowed &= torch.tril(torch.ones(L, L, dtype=torch.bool))
    o = torch.nn.functional.scaled_dot_product_attention(q[None], k[None], v[None], attn_mask=allowed[None])[0]
    p = (q @ k.T / np.sqrt(q.shape[1])).masked_fill(~allowed, float("-inf"))
    return o.numpy(), torch.logsumexp(p, -1).numpy()


@pytest.mark.parametrize("causal", [False, True])
def test_masked_attention_matches_torch_sdpa(oracle, causal):
    rng = np.random.default_rng(30)
    L, d, S = 128, 32, 16
    N = L // S
    q, k, v = [bf16_values(rng, (1, L, d)) for _ in range(3)]
    mask = (rng.random((1, N, N)) < 0.4).astype(np.uint8)
    mask[0, np.arange(N), np.arange(N)] = 1
    if causal:
        mask = np.tril(mask)
    O, lse = oracle.masked_attention(q, k, v, [0, L], S, causal, mask)
    ro, rl = torch_masked_attention(q[0], k[0], v[0], S, causal, mask[0])
    np.testing.assert_allclose(O[0], ro, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(lse[0], rl, rtol=1e-9, atol=1e-12)


def test_all_blocks_selected_equals_dense_sdpa(oracle):
    rng = np.random.default_rng(31)
    L, d, S = 192, 64, 32
    q, v = bf16_values(rng, (4, L, d)), bf16_values(rng, (2, L, d))
    k = bf16_values(rng, (2, L, d))
    N = L // S
    full = np.tril(np.ones((4, N, N), np.uint8))
    O, _ = oracle.masked_attention(q, k, v, [0, L], S, True, full)
    Od, _ = oracle.masked_attention(q, k, v, [0, L], S, True, None)
    assert np.array_equal(O, Od)
    tq, tk, tv = [torch.from_numpy(x).double() for x in (q, k, v)]
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[None], tk.repeat_interleave(2, 0)[None], tv.repeat_interleave(2, 0)[None], is_causal=True)[0]
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-9, atol=1e-12)        # also pins the GQA head mapping


def test_attention_rows_sum_to_one_and_masking_is_respected(oracle):
    rng = np.random.default_rng(32)
    L, d, S = 128, 32, 32
    N = L // S
    q, k, v = [bf16_values(rng, (1, L, d)) for _ in range(3)]
    mask = np.array([[[1, 0, 0, 0], [0, 1, 0, 0], [1, 0, 1, 0], [0, 1, 0, 1]]], np.uint8)
    ones = np.ones_like(v)
    O1, _ = oracle.masked_attention(q, k, ones, [0, L], S, True, mask)
    np.testing.assert_allclose(O1, 1.0, rtol=1e-12)                          # weights sum to 1
    O, _ = oracle.masked_attention(q, k, v, [0, L], S, True, mask)
    k2, v2 = k.copy(), v.copy()
    k2[0, 32:64] += 3.0                                                      # block 1 is not selected by rows 0 and 2
    v2[0, 32:64] -= 2.0
    O2, _ = oracle.masked_attention(q, k2, v2, [0, L], S, True, mask)
    assert np.array_equal(O[0, :32], O2[0, :32]) and np.array_equal(O[0, 64:96], O2[0, 64:96])
    assert not np.array_equal(O[0, 32:64], O2[0, 32:64])
    # causality inside the diagonal block: changing token t+1.. never changes row t
    k3, v3 = k.copy(), v.copy()
    k3[0, 10:] += 1.0
    v3[0, 10:] += 1.0
    O3, _ = oracle.masked_attention(q, k3, v3, [0, L], S, True, mask)
    assert np.array_equal(O[0, :10], O3[0, :10])


def test_planted_pattern_is_recovered(oracle):
    """Generator and proxy agree: the planted sink / band / hot blocks are what the proxy ranks first."""
    w = W.single_head_planted()
    q, k, _ = w.f32()
    m, sc = oracle.build_mask(q, k, w.cu_seqlens, w.block_size, 8, 8, True, oracle.TOP_K, 0.25)
    np.testing.assert_allclose(1 - oracle.sparsity(m, w.cu_seqlens, w.block_size, True), 144 / 528, rtol=1e-12)
    rec = []
    for i, hs in enumerate(w.planted["hot"]):
        sel = set(np.nonzero(m[0, i])[0])
        rec.append(len(sel & set(hs)) / min(len(hs), len(sel)))
    assert np.mean(rec) > 0.9


def test_proxy_ranking_tracks_exact_block_mass(oracle):
    """Sec. 4.1: rankings from the c = 8 compressed space follow the token-level ones (the paper reports
    Spearman > 0.98 on its data; the planted synthetic data gives the same picture)."""
    from scipy.stats import spearmanr
    w = W.gqa_planted(L=4096, H=1, Hkv=1, S=128, seed=5)
    q, k, _ = w.f32()
    proxy = oracle.block_scores(q, k, w.cu_seqlens, 128, 8, 8, True)[0]
    exact = oracle.block_scores(q, k, w.cu_seqlens, 128, 1, 1, True)[0] / 8.0
    rhos = [spearmanr(proxy[i, :i + 1], exact[i, :i + 1])[0] for i in range(8, 32)]
    assert np.mean(rhos) > 0.9


# ----------------------------------------------------------------------------- ragged last block (S does not divide L)

@pytest.mark.parametrize("causal", [False, True])
def test_ragged_scores_c1_equal_exact_block_mass(oracle, causal):
    """L = 5 blocks and a remainder: with c = 1 the scores are the exact attention mass of the (clipped) blocks."""
    rng = np.random.default_rng(50)
    L, S, d = 88, 16, 32                                  # 5 full blocks + 8 tokens
    q = bf16_values(rng, (L, d), 1.5)
    k = bf16_values(rng, (L, d), 1.5)
    sc = oracle.block_scores_head(q, k, S=S, c_q=1, c_k=1, causal_mode=int(causal), scale=1 / np.sqrt(d))
    p = torch.from_numpy(q).double() @ torch.from_numpy(k).double().T / np.sqrt(d)
    if causal:
        p = p.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    a = torch.softmax(p, -1)
    N = -(-L // S)
    pad = torch.zeros(N * S, N * S, dtype=torch.float64)
    pad[:L, :L] = a
    ref = pad.reshape(N, S, N, S).sum(dim=(1, 3)).numpy()
    assert sc.shape == (N, N)
    np.testing.assert_allclose(sc, ref, rtol=1e-10, atol=1e-13)


def test_ragged_score_rows_sum_to_existing_composites(oracle):
    rng = np.random.default_rng(51)
    L, S, c = 200, 64, 8                                  # 3 full blocks + 8 tokens = one composite token
    q = bf16_values(rng, (1, L, 32))
    k = bf16_values(rng, (1, L, 32))
    sc = oracle.block_scores(q, k, [0, L], S, c, c, causal=False)
    np.testing.assert_allclose(sc[0].sum(-1), [8, 8, 8, 1], rtol=1e-12)
    m, _ = oracle.build_mask(q, k, [0, L], S, c, c, True, 1, 0.5)
    assert m.shape == (1, 4, 4) and not np.triu(m[0], 1).any() and m[0].any(-1).all()


@pytest.mark.parametrize("causal", [False, True])
def test_ragged_masked_attention_matches_torch_sdpa(oracle, causal):
    rng = np.random.default_rng(52)
    L, d, S = 108, 32, 16                                 # 6 full blocks + 12 tokens
    N = -(-L // S)
    q, k, v = [bf16_values(rng, (1, L, d)) for _ in range(3)]
    mask = (rng.random((1, N, N)) < 0.4).astype(np.uint8)
    mask[0, np.arange(N), np.arange(N)] = 1
    if causal:
        mask = np.tril(mask)
    O, lse = oracle.masked_attention(q, k, v, [0, L], S, causal, mask)
    tq, tk, tv = [torch.from_numpy(x[0]).double() for x in (q, k, v)]
    allowed = torch.from_numpy(np.kron(mask[0], np.ones((S, S), dtype=np.uint8))[:L, :L].copy()).bool()
    if causal:
        allowed &= torch.tril(torch.ones(L, L, dtype=torch.bool))
    ro = torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None], attn_mask=allowed[None])[0]
    rl = torch.logsumexp((tq @ tk.T / np.sqrt(d)).masked_fill(~allowed, float("-inf")), -1)
    assert not np.isnan(O).any()
    np.testing.assert_allclose(O[0], ro.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(lse[0], rl.numpy(), rtol=1e-9, atol=1e-12)


def test_ragged_packed_sequences_are_independent(oracle):
    rng = np.random.default_rng(53)
    S, d = 16, 32
    lens = [40, 16, 56]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    q, k, v = [bf16_values(rng, (2, T, d)) for _ in range(3)]
    m, sc = oracle.build_mask(q, k, cu, S, 8, 8, True, 0, 0.8)
    assert m.shape[1] == 3 + 1 + 4
    O, _ = oracle.masked_attention(q, k, v, cu, S, True, m)
    assert not np.isnan(O).any()
    r0 = 0
    for b, Lb in enumerate(lens):
        sl = slice(int(cu[b]), int(cu[b + 1]))
        nb = -(-Lb // S)
        mb, _ = oracle.build_mask(q[:, sl], k[:, sl], [0, Lb], S, 8, 8, True, 0, 0.8)
        assert np.array_equal(mb, m[:, r0:r0 + nb, :nb])
        Ob, _ = oracle.masked_attention(q[:, sl], k[:, sl], v[:, sl], [0, Lb], S, True, mb)
        assert np.array_equal(Ob, O[:, sl])
        r0 += nb


# ----------------------------------------------------------------------------- partial pooling windows (c does not divide L)

@pytest.mark.parametrize("c,L", [(8, 43), (4, 9), (16, 17), (32, 100)])
def test_partial_window_pool_matches_torch_ceil_mode(oracle, c, L):
    """The last window averages the tokens that exist: torch's avg_pool1d with ceil_mode (divisor = clipped window)."""
    rng = np.random.default_rng(60 + c)
    x = bf16_values(rng, (L, 128))
    ref = torch.nn.functional.avg_pool1d(torch.from_numpy(x).T[None], c, c, ceil_mode=True)[0].T
    ref = ref.to(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.avgpool_seq(x, c)
    assert got.shape == (-(-L // c), 128)
    assert np.array_equal(got, ref)
    tail = x[(L // c) * c:].astype(np.float32)
    if len(tail):                                                      # and by hand for the clipped window
        acc = np.zeros(128, np.float32)
        for row in tail:
            acc = acc + row
        hand = torch.from_numpy(acc / np.float32(len(tail))).to(torch.bfloat16).float().numpy()
        assert np.array_equal(got[-1], hand)


@pytest.mark.parametrize("causal", [False, True])
def test_partial_window_scores_equal_attention_over_torch_pooled_tokens(oracle, causal):
    """L = 2 blocks + 20 tokens with c = 8: 2 whole windows and one of 4 tokens in the last block."""
    rng = np.random.default_rng(61)
    L, d, S, c = 148, 64, 64, 8
    q = bf16_values(rng, (1, L, d), 1.3)
    k = bf16_values(rng, (1, L, d), 1.3)
    pool = lambda x: torch.nn.functional.avg_pool1d(torch.from_numpy(x).T[None], c, c, ceil_mode=True)[0].T \
        .to(torch.bfloat16).double()
    pq, pk = pool(q[0]), pool(k[0])                                  # 19 composite tokens
    p = pq @ pk.T / np.sqrt(d)
    if causal:                                                       # c_q = c_k: composite key s' visible iff s' <= t'
        p = p.masked_fill(torch.triu(torch.ones(19, 19, dtype=torch.bool), 1), float("-inf"))
    a = torch.softmax(p, -1)
    n, N = S // c, 3
    pad = torch.zeros(N * n, N * n, dtype=torch.float64)
    pad[:19, :19] = a
    ref = pad.reshape(N, n, N, n).sum(dim=(1, 3)).numpy()
    got = oracle.block_scores(q, k, [0, L], S, c, c, causal)[0]
    if causal:
        ref = np.tril(ref)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(got.sum(-1), [8, 8, 3], rtol=1e-12)


def test_partial_windows_packed_sequences_are_independent(oracle):
    rng = np.random.default_rng(62)
    S, d, c = 16, 32, 8
    lens = [37, 5, 50]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k = [bf16_values(rng, (2, int(cu[-1]), d)) for _ in range(2)]
    assert oracle.composite_offsets(cu, c) == [0, 5, 6, 13]
    m, sc = oracle.build_mask(q, k, cu, S, c, c, True, 0, 0.8)
    r0 = 0
    for b, Lb in enumerate(lens):
        sl = slice(int(cu[b]), int(cu[b + 1]))
        nb = -(-Lb // S)
        mb, sb = oracle.build_mask(q[:, sl], k[:, sl], [0, Lb], S, c, c, True, 0, 0.8)
        assert np.array_equal(mb, m[:, r0:r0 + nb, :nb]) and np.array_equal(sb, sc[:, r0:r0 + nb, :nb])
        r0 += nb


# ----------------------------------------------------------------------------- max pooling (ablation "Compression Strategy")

@pytest.mark.parametrize("c,L", [(8, 64), (8, 43), (4, 9), (32, 100)])
def test_max_pool_matches_torch_max_pool(oracle, c, L):
    rng = np.random.default_rng(70 + c)
    x = bf16_values(rng, (L, 128))
    ref = torch.nn.functional.max_pool1d(torch.from_numpy(x).T[None], c, c, ceil_mode=True)[0].T.numpy()
    got = oracle.maxpool_seq(x, c)
    assert np.array_equal(got, ref)
    assert np.array_equal(oracle.maxpool_seq(x, 1), x)                        # c = 1 is the identity


def test_max_pool_scores_equal_attention_over_torch_pooled_tokens(oracle):
    rng = np.random.default_rng(71)
    L, d, S, c = 256, 64, 64, 8
    q = bf16_values(rng, (1, L, d), 1.3)
    k = bf16_values(rng, (1, L, d), 1.3)
    pool = lambda x: torch.nn.functional.max_pool1d(torch.from_numpy(x).T[None], c, c)[0].T.numpy()
    ref = np.tril(brute_block_mass(pool(q[0]), pool(k[0]), S // c, True))
    got = oracle.block_scores(q, k, [0, L], S, c, c, True, pool=oracle.POOL_MAX)[0]
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-13)
    avg = oracle.block_scores(q, k, [0, L], S, c, c, True)[0]
    assert np.abs(avg - got).max() > 1e-3                                     # the option really changes the proxy


# ---- stochastic pooling (ablation "Compression Strategy"): one token per window, drawn by its share of the L2 norms

def test_stochastic_pool_picks_tokens_in_proportion_to_their_norms(oracle):
    # A window of tokens with norms 1, 2, 3, 6: over a fine grid of uniform numbers the choice frequencies are the
    # normalised norms 1/12, 2/12, 3/12, 6/12 (squared norms would give 1/50, 4/50, 9/50, 36/50).
    d, c, n = 16, 4, 12000
    base = np.zeros((c, d), dtype=np.float32)
    for m, w in enumerate((1.0, 2.0, 3.0, 6.0)):
        base[m, m] = w                                                         # distinct directions, exact norms
    x = np.tile(base, (n, 1))
    u = ((np.arange(n) + 0.5) / n).astype(np.float32)
    out, sel = oracle.stochpool_seq(x, c, u, return_choice=True)
    freq = np.bincount(sel, minlength=c) / n
    np.testing.assert_allclose(freq, np.array([1, 2, 3, 6]) / 12.0, atol=2.0 / n)
    assert np.array_equal(out, base[sel])                                      # the composite IS the chosen token
    # inversion: the chosen offsets are non-decreasing in u, ties broken towards the earlier token
    assert np.all(np.diff(sel) >= 0)
    assert sel[0] == 0 and sel[-1] == c - 1


def test_stochastic_pool_closed_forms(oracle):
    rng = np.random.default_rng(81)
    d, c = 32, 8
    # equal norms -> token floor(u c)
    dirs = np.eye(d, dtype=np.float32)[:c] * 4.0
    u = np.array([0.0, 0.124, 0.126, 0.5, 0.874, 0.876, 0.9999], dtype=np.float32)
    x = np.tile(dirs, (len(u), 1))
    _, sel = oracle.stochpool_seq(x, c, u, return_choice=True)
    assert sel.tolist() == [0, 0, 1, 4, 6, 7, 7]
    # all the magnitude on one token -> always that token; zero tokens are never drawn, whatever u
    x = np.zeros((3 * c, d), dtype=np.float32)
    x[5], x[c + 0], x[2 * c + 7] = 1.0, -2.0, 0.5
    _, sel = oracle.stochpool_seq(x, c, np.array([0.0, 0.7, 0.3], dtype=np.float32), return_choice=True)
    assert sel.tolist() == [5, 0, 7]
    # the norm is over all channels and sign-blind: a token of many small channels outweighs one large channel
    x = np.zeros((2, d), dtype=np.float32)
    x[0, 3] = 3.0                                                              # norm 3
    x[1, :] = -1.0                                                             # norm sqrt(32) = 5.66
    share0 = 3.0 / (3.0 + np.sqrt(32.0))
    _, sel = oracle.stochpool_seq(x, 2, np.array([share0 - 1e-3], dtype=np.float32), return_choice=True)
    assert sel[0] == 0
    _, sel = oracle.stochpool_seq(x, 2, np.array([share0 + 1e-3], dtype=np.float32), return_choice=True)
    assert sel[0] == 1
    # c = 1 is the identity; an all-zero window returns a zero token
    y = bf16_values(rng, (20, d), 1.0)
    assert np.array_equal(oracle.stochpool_seq(y, 1, rng.random(20).astype(np.float32)), y)
    assert not oracle.stochpool_seq(np.zeros((8, d), np.float32), 4, np.array([0.3, 0.9], np.float32)).any()


@pytest.mark.parametrize("L,c", [(37, 8), (64, 16), (5, 8)])
def test_stochastic_pool_matches_fp64_inversion_and_clips_last_window(oracle, L, c):
    # Independent statement in float64 numpy: cumulative norms against u * total.  A draw may differ only when u sits
    # within fp32 rounding of a boundary between two tokens, which these seeded numbers avoid by a wide margin.
    rng = np.random.default_rng(L * 100 + c)
    d = 64
    x = bf16_values(rng, (L, d), 1.0)
    Lc = -(-L // c)
    u = rng.random(Lc).astype(np.float32)
    out, sel = oracle.stochpool_seq(x, c, u, return_choice=True)
    for t in range(Lc):
        win = x[t * c:min(L, (t + 1) * c)].astype(np.float64)
        cum = np.cumsum(np.sqrt((win ** 2).sum(axis=1)))
        margin = np.abs(cum / cum[-1] - float(u[t])).min()
        assert margin > 1e-5
        pick = int(np.searchsorted(cum, float(u[t]) * cum[-1], side="right"))
        assert sel[t] == pick and pick < len(win)
        assert np.array_equal(out[t], x[t * c + pick])


def test_stochastic_pool_feeds_the_proxy_per_head_and_sequence(oracle):
    # composite tokens of a packed batch: every (head, sequence) window uses its own uniform number, laid out like
    # the packed composite tokens; scores equal exact attention over the tokens picked by hand.
    rng = np.random.default_rng(83)
    cu, d, S, c = [0, 128, 320], 32, 64, 8
    T = cu[-1]
    q = bf16_values(rng, (2, T, d), 1.2)
    k = bf16_values(rng, (1, T, d), 1.2)
    off = oracle.composite_offsets(cu, c)
    rq = rng.random((2, off[-1])).astype(np.float32)
    rk = rng.random((1, off[-1])).astype(np.float32)
    Qt, Kt = oracle.composite_tokens(q, k, cu, c, c, 1, oracle.POOL_STOCHASTIC, (rq, rk))
    for h in range(2):
        for b in range(2):
            ref = oracle.stochpool_seq(q[h, cu[b]:cu[b + 1]], c, rq[h, off[b]:off[b + 1]])
            assert np.array_equal(Qt[h, off[b]:off[b + 1]], ref)
    assert np.array_equal(Kt[0], Kt[1])                                        # one KV head serves both query heads
    got = oracle.block_scores(q, k, cu, S, c, c, True, pool=oracle.POOL_STOCHASTIC, rand=(rq, rk))
    for b in range(2):
        nb = (cu[b + 1] - cu[b]) // S
        ref = np.tril(brute_block_mass(Qt[0, off[b]:off[b + 1]], Kt[0, off[b]:off[b + 1]], S // c, True))
        np.testing.assert_allclose(got[0, cu[b] // S:cu[b] // S + nb, :nb], ref, rtol=1e-10, atol=1e-13)
