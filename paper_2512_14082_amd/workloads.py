"""Seeded synthetic inputs for the five benchmark configurations.

This module only *draws inputs*: it holds none of the method's arithmetic (no pooling,
scoring, selection or attention) and is the single piece of code that both the HIP path
and the CPU oracle are fed from.  The paper measures on public long-context suites run
through trained models; neither is available offline, so these inputs reproduce their
*shapes* (grouped-query 32/8 heads, head_dim 128, up to 128K tokens, a 16x64x64 video
token grid) and the *structure* attention maps of such models are known to have: an
attention sink on the first key block, a local band, and a few "vertical" hot key blocks.

Everything is generated with numpy from one integer seed, rounded to bf16 (round to
nearest even) and returned as uint16 bit patterns, head-major:
    q : uint16 [H, T, d]     k, v : uint16 [H_kv, T, d]

A gain ``g`` multiplies every planted term (queries get ``g * dir``, keys ``3 g * dir``).
g = 1 is the literal amplitude; at head_dim 128 that boosts a planted logit by only
3/sqrt(128) = 0.27, which leaves a cumulative-threshold selection with nothing to prune,
so the default is g = 4 (logit boost 4.2), which lands in the mask-density range the
paper's sparsity tables report.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

BASE_SEED = 251214082
HEAD_DIM = 128
TOP_P = 0
TOP_K = 1


# --------------------------------------------------------------------------- bf16 I/O helpers

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even. Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    name: str
    q: np.ndarray                 # uint16 [H, T, d]
    k: np.ndarray                 # uint16 [H_kv, T, d]
    v: np.ndarray                 # uint16 [H_kv, T, d]
    cu_seqlens: List[int]
    block_size: int
    causal: bool
    c_q: int = 8
    c_k: int = 8
    c_h: int = 1
    pool: int = 0                 # 0 average pooling (the method), 1 max / 2 stochastic pooling (ablation)
    rand_q: Optional[np.ndarray] = None   # stochastic pooling: float32 uniforms [H, composite queries]
    rand_k: Optional[np.ndarray] = None   # and [H_kv, composite keys], see draw_pool_uniforms
    mode: int = TOP_P
    param: float = 0.9            # threshold P (TOP_P) or kept fraction f (TOP_K)
    gain: float = 4.0
    seed: int = BASE_SEED
    planted: Dict = field(default_factory=dict)   # what was planted, for recall checks

    @property
    def n_heads_q(self) -> int:
        return self.q.shape[0]

    @property
    def n_heads_kv(self) -> int:
        return self.k.shape[0]

    @property
    def total_tokens(self) -> int:
        return self.q.shape[1]

    @property
    def head_dim(self) -> int:
        return self.q.shape[2]

    def n_blocks(self) -> List[int]:
        return [-(-(self.cu_seqlens[b + 1] - self.cu_seqlens[b]) // self.block_size)
                for b in range(len(self.cu_seqlens) - 1)]

    def valid_pairs(self) -> int:
        """Valid (query block, key block) pairs per query head."""
        tot = 0
        for n in self.n_blocks():
            tot += n * (n + 1) // 2 if self.causal else n * n
        return tot

    def f32(self):
        return bf16_bits_to_f32(self.q), bf16_bits_to_f32(self.k), bf16_bits_to_f32(self.v)

    def n_composite(self, c: int) -> int:
        """Composite tokens of the packed batch at compression factor c (one per started window)."""
        return sum(-(-(self.cu_seqlens[b + 1] - self.cu_seqlens[b]) // c) for b in range(len(self.cu_seqlens) - 1))

    def draw_pool_uniforms(self, seed: Optional[int] = None) -> "Workload":
        """Switch to stochastic pooling and draw the uniform numbers in [0, 1) that it consumes, one per
        (head, composite token), laid out like the composite tokens."""
        rng = np.random.default_rng(self.seed + 977 if seed is None else seed)
        self.pool = 2
        self.rand_q = rng.random((self.n_heads_q, self.n_composite(self.c_q)), dtype=np.float32)
        self.rand_k = rng.random((self.n_heads_kv, self.n_composite(self.c_k)), dtype=np.float32)
        return self


def _unit(rng, d):
    x = rng.standard_normal(d)
    return (x / np.linalg.norm(x)).astype(np.float64)


def _normal_bits(rng, shape) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


# --------------------------------------------------------------------------- config 1

def single_head_planted(L: int = 2048, S: int = 64, frac: float = 0.25, gain: float = 4.0,
                        seed: int = BASE_SEED + 0, d: int = HEAD_DIM, n_hot: int = 8) -> Workload:
    """One causal head with a row-specific planted pattern.

    Orthonormal directions u, r_0..r_{N-1} (QR of a Gaussian matrix).  Every query gets
    +g u and key block 0 gets +3g u (sink).  Query block i also gets +g r_i, and the key
    blocks of Hot(i) = {i, i-1} + ``n_hot`` distinct earlier blocks get +3g r_i.
    """
    rng = np.random.default_rng(seed)
    N = L // S
    assert N + 1 <= d
    basis, _ = np.linalg.qr(rng.standard_normal((d, N + 1)))
    u, r = basis[:, 0], basis[:, 1:].T
    q = rng.standard_normal((L, d))
    k = rng.standard_normal((L, d))
    v = rng.standard_normal((L, d))
    q += gain * u
    k[:S] += 3.0 * gain * u
    hot = []
    for i in range(N):
        hs = {i}
        if i >= 1:
            hs.add(i - 1)
        cand = np.arange(0, i)
        picks = rng.choice(cand, size=min(n_hot, len(cand)), replace=False) if len(cand) else []
        hs.update(int(x) for x in picks)
        hot.append(sorted(hs))
        q[i * S:(i + 1) * S] += gain * r[i]
        for j in hs:
            k[j * S:(j + 1) * S] += 3.0 * gain * r[i]
    to = lambda a: f32_to_bf16_bits(a.astype(np.float32))[None]
    return Workload("cfg1_single_head_L2048", to(q), to(k), to(v), [0, L], S, True, mode=TOP_K, param=frac,
                    gain=gain, seed=seed, planted={"hot": hot, "sink": 0})


# --------------------------------------------------------------------------- configs 2, 3, 5

_HEAD_MULT = (0.7, 0.9, 1.1, 1.3)


def _gqa_sequence(rng, L, S, H, Hkv, gain, hot_sets, d=HEAD_DIM, n_freq=16, q_out=None, k_out=None,
                  v_out=None, t0=0):
    """Fill q_out[:, t0:t0+L], k_out, v_out for one sequence with sink + local band + hot key blocks.

    Per KV head: a unit direction u; key blocks of its hot set (block 0 is always hot: the sink) get
    +3g u; the G query heads of the group get +g m_h u with m_h in (0.7, 0.9, 1.1, 1.3) so that masks
    differ inside a group.  Local band: a random-Fourier positional code with Gaussian kernel of width
    sigma = 2S tokens, in 2*n_freq directions orthogonal to u; keys +3g F_t, queries +g m_h F_t.
    """
    G = H // Hkv
    pos = np.arange(L, dtype=np.float64)
    sigma = 2.0 * S
    for g in range(Hkv):
        u = _unit(rng, d)
        basis, _ = np.linalg.qr(np.column_stack([u, rng.standard_normal((d, 2 * n_freq))]))
        E = basis[:, 1:]                                     # d x 2n_freq, orthogonal to u
        omega = rng.standard_normal(n_freq) / sigma
        ang = pos[:, None] * omega[None, :]
        F = np.concatenate([np.cos(ang), np.sin(ang)], axis=1) / np.sqrt(n_freq)   # L x 2n_freq
        FE = (F @ E.T).astype(np.float32)                    # L x d
        kk = rng.standard_normal((L, d), dtype=np.float32)
        kk += np.float32(3.0 * gain) * FE
        hot_vec = (3.0 * gain * u).astype(np.float32)
        for j in hot_sets[g]:
            kk[j * S:(j + 1) * S] += hot_vec
        k_out[g, t0:t0 + L] = f32_to_bf16_bits(kk)
        v_out[g, t0:t0 + L] = _normal_bits(rng, (L, d))
        for m in range(G):
            h = g * G + m
            mh = _HEAD_MULT[m % 4]
            qq = rng.standard_normal((L, d), dtype=np.float32)
            qq += np.float32(gain * mh) * (FE + u.astype(np.float32))
            q_out[h, t0:t0 + L] = f32_to_bf16_bits(qq)


def gqa_planted(L: int = 32768, H: int = 32, Hkv: int = 8, S: int = 128, P: float = 0.95,
                gain: float = 4.0, seed: int = BASE_SEED + 1, hot_frac: float = 0.05,
                name: Optional[str] = None) -> Workload:
    """Llama-3-8B-shaped causal layer: sink, local band of ~4 blocks, ~5 % uniformly drawn hot key blocks per KV head."""
    rng = np.random.default_rng(seed)
    N = L // S
    n_hot = int(np.ceil(hot_frac * N))
    hot_sets = []
    for g in range(Hkv):
        picks = rng.choice(np.arange(1, N), size=min(n_hot, N - 1), replace=False) if N > 1 else []
        hot_sets.append(sorted({0, *[int(x) for x in picks]}))
    q = np.empty((H, L, HEAD_DIM), np.uint16)
    k = np.empty((Hkv, L, HEAD_DIM), np.uint16)
    v = np.empty((Hkv, L, HEAD_DIM), np.uint16)
    _gqa_sequence(rng, L, S, H, Hkv, gain, hot_sets, q_out=q, k_out=k, v_out=v)
    return Workload(name or f"cfg2_gqa32x8_L{L}", q, k, v, [0, L], S, True, mode=TOP_P, param=P, gain=gain,
                    seed=seed, planted={"hot": hot_sets})


def gqa_zipf(L: int = 131072, H: int = 32, Hkv: int = 8, S: int = 128, P: float = 0.9,
             gain: float = 4.0, seed: int = BASE_SEED + 2, hot_frac: float = 0.05,
             name: Optional[str] = None) -> Workload:
    """As gqa_planted, but hot key blocks follow a Zipf(1.1) popularity shared by all heads.

    One seeded permutation ranks the key blocks [1, N); rank r has weight r^-1.1.  KV head g draws
    ceil(hot_frac * N * 2^((g mod 4) - 1)) blocks with replacement and de-duplicates, so the hot-set
    size (hence the mask density) differs between heads while popular blocks recur across heads.
    """
    rng = np.random.default_rng(seed)
    N = L // S
    perm = rng.permutation(np.arange(1, N)) if N > 1 else np.array([], dtype=np.int64)
    w = np.arange(1, N, dtype=np.float64) ** -1.1
    w = w / w.sum() if len(w) else w
    hot_sets = []
    for g in range(Hkv):
        draws = int(np.ceil(hot_frac * N * 2.0 ** ((g % 4) - 1)))
        picks = rng.choice(perm, size=draws, replace=True, p=w) if N > 1 else []
        hot_sets.append(sorted({0, *[int(x) for x in picks]}))
    q = np.empty((H, L, HEAD_DIM), np.uint16)
    k = np.empty((Hkv, L, HEAD_DIM), np.uint16)
    v = np.empty((Hkv, L, HEAD_DIM), np.uint16)
    _gqa_sequence(rng, L, S, H, Hkv, gain, hot_sets, q_out=q, k_out=k, v_out=v)
    return Workload(name or f"cfg3_gqa32x8_zipf_L{L}", q, k, v, [0, L], S, True, mode=TOP_P, param=P, gain=gain,
                    seed=seed, planted={"hot": hot_sets})


def gqa_varlen(lengths: Sequence[int] = (8192, 16384, 32768, 65536), H: int = 32, Hkv: int = 8, S: int = 128,
               P: float = 0.9, gain: float = 4.0, seed: int = BASE_SEED + 4, hot_frac: float = 0.05,
               name: Optional[str] = None) -> Workload:
    """Packed causal sequences (cu_seqlens), each generated like gqa_planted with its own hot sets."""
    rng = np.random.default_rng(seed)
    cu = [0]
    for L in lengths:
        cu.append(cu[-1] + int(L))
    T = cu[-1]
    q = np.empty((H, T, HEAD_DIM), np.uint16)
    k = np.empty((Hkv, T, HEAD_DIM), np.uint16)
    v = np.empty((Hkv, T, HEAD_DIM), np.uint16)
    planted = []
    for b, L in enumerate(lengths):
        N = L // S
        n_hot = int(np.ceil(hot_frac * N))
        hot_sets = []
        for g in range(Hkv):
            picks = rng.choice(np.arange(1, N), size=min(n_hot, N - 1), replace=False) if N > 1 else []
            hot_sets.append(sorted({0, *[int(x) for x in picks]}))
        planted.append(hot_sets)
        _gqa_sequence(rng, L, S, H, Hkv, gain, hot_sets, q_out=q, k_out=k, v_out=v, t0=cu[b])
    return Workload(name or "cfg5_gqa32x8_varlen", q, k, v, cu, S, True, mode=TOP_P, param=P, gain=gain, seed=seed,
                    planted={"hot": planted})


# --------------------------------------------------------------------------- config 4

def video_field(grid=(16, 64, 64), H: int = 40, S: int = 128, frac: float = 0.20, sigma: float = 2.0,
                noise_var: float = 0.5, seed: int = BASE_SEED + 3, name: Optional[str] = None) -> Workload:
    """Video-DiT-shaped bidirectional layer: tokens on a (t, h, w) raster grid.

    Per head a random field F (white noise smoothed by a separable 3-D Gaussian, sigma tokens per
    axis, periodic boundary, rescaled to unit variance per channel) is shared by queries and keys:
    Q = F + e_q, K = F + e_k with independent N(0, noise_var) noise, so attention is spatially local.
    """
    from scipy.ndimage import gaussian_filter1d
    rng = np.random.default_rng(seed)
    L = int(np.prod(grid))
    q = np.empty((H, L, HEAD_DIM), np.uint16)
    k = np.empty((H, L, HEAD_DIM), np.uint16)
    v = np.empty((H, L, HEAD_DIM), np.uint16)
    sd = np.float32(np.sqrt(noise_var))
    for h in range(H):
        F = rng.standard_normal((*grid, HEAD_DIM), dtype=np.float32)
        for ax in range(3):
            F = gaussian_filter1d(F, sigma=sigma, axis=ax, mode="wrap", truncate=4.0)
        F = F.reshape(L, HEAD_DIM)
        F /= F.std(axis=0, keepdims=True)
        q[h] = f32_to_bf16_bits(F + sd * rng.standard_normal((L, HEAD_DIM), dtype=np.float32))
        k[h] = f32_to_bf16_bits(F + sd * rng.standard_normal((L, HEAD_DIM), dtype=np.float32))
        v[h] = _normal_bits(rng, (L, HEAD_DIM))
    return Workload(name or f"cfg4_video_H{H}_L{L}", q, k, v, [0, L], S, False, mode=TOP_K, param=frac, gain=1.0,
                    seed=seed, planted={"grid": tuple(grid)})


# --------------------------------------------------------------------------- small unstructured case

def random_small(H: int = 4, Hkv: int = 2, lengths: Sequence[int] = (256,), S: int = 64, causal: bool = True,
                 mode: int = TOP_P, param: float = 0.9, seed: int = 7, scale: float = 1.0,
                 d: int = HEAD_DIM) -> Workload:
    """Plain i.i.d. N(0, scale^2) tensors for unit tests."""
    rng = np.random.default_rng(seed)
    cu = [0]
    for L in lengths:
        cu.append(cu[-1] + int(L))
    T = cu[-1]
    mk = lambda n: f32_to_bf16_bits((scale * rng.standard_normal((n, T, d))).astype(np.float32))
    return Workload(f"random_H{H}x{Hkv}_T{T}", mk(H), mk(Hkv), mk(Hkv), cu, S, causal, mode=mode, param=param,
                    gain=0.0, seed=seed)


def steep_logits(kind: str = "rising", H: int = 2, Hkv: int = 1, lengths: Sequence[int] = (1024,), S: int = 128,
                 causal: bool = True, step: float = 16.0, seed: int = 77, d: int = HEAD_DIM) -> Workload:
    """Inputs whose attention logits span hundreds of natural-log units inside one row: the case in which a streaming
    softmax has to move its reference value again and again (or sees later terms vanish against it).

    Queries are N(0,1) + 6 u for a unit vector u, keys are 0.5 N(0,1) + b u with the key's boost b chosen so that the
    logit q.k / sqrt(d) is about `step` * level: "rising": level = key-block index (every block dwarfs the ones before
    it); "falling": level = -(key-block index); "spikes": level 0 except for 2 % of the keys, which get a random level in
    [1, 12] (a new maximum in the middle of a tile, at random places); "ramp": level grows by 1/8 per key inside
    every block and restarts (a new maximum in nearly every 32-key tile)."""
    rng = np.random.default_rng(seed)
    cu = [0]
    for L in lengths:
        cu.append(cu[-1] + int(L))
    T = cu[-1]
    u = _unit(rng, d).astype(np.float32)
    q = rng.standard_normal((H, T, d), dtype=np.float32) + 6.0 * u
    k = 0.5 * rng.standard_normal((Hkv, T, d), dtype=np.float32)
    v = rng.standard_normal((Hkv, T, d), dtype=np.float32)
    level = np.zeros((Hkv, T), np.float32)
    for b in range(len(lengths)):
        pos = np.arange(cu[b + 1] - cu[b])
        if kind == "rising":
            lv = (pos // S).astype(np.float32)
        elif kind == "falling":
            lv = -(pos // S).astype(np.float32)
        elif kind == "ramp":
            lv = (pos % S).astype(np.float32) / 8.0
        elif kind == "spikes":
            lv = None
        else:
            raise ValueError(kind)
        for g in range(Hkv):
            if lv is None:
                x = np.where(rng.random(len(pos)) < 0.02, rng.integers(1, 13, len(pos)), 0).astype(np.float32)
            else:
                x = lv
            level[g, cu[b]:cu[b + 1]] = x
    boost = level * np.float32(step * np.sqrt(d) / 6.0)
    k += boost[..., None] * u
    return Workload(f"steep_{kind}_T{T}", f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v), cu, S, causal,
                    mode=TOP_K, param=0.5, gain=0.0, seed=seed)


def random_32k(d: int = HEAD_DIM, seed: int = BASE_SEED + 9, **_unused) -> Workload:
    """GQA 32/8 layer at L = 32K with i.i.d. Gaussian tensors and a fixed 25 % budget: the timing shape for the
    head dimensions other than 128 (no planted structure; selection at a fixed budget keeps the density known)."""
    w = random_small(H=32, Hkv=8, lengths=(32768,), S=128, causal=True, mode=TOP_K, param=0.25, seed=seed, d=d)
    w.name = f"rand32k_gqa32x8_d{d}"
    return w


def by_name(name: str, **kw) -> Workload:
    if name.startswith("rand32k_d"):
        return random_32k(d=int(name[len("rand32k_d"):]), **kw)
    table = {
        "cfg1": single_head_planted,
        "cfg2": gqa_planted,
        "cfg3": gqa_zipf,
        "cfg4": video_field,
        "cfg5": gqa_varlen,
    }
    return table[name](**kw)
