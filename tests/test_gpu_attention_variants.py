"""GPU parity of the tree-attention kernels called on their own, shape by shape: every kernel variant
(narrow / wide query blocks, head size 64 / 128, bf16 / 8-bit prefix) with ragged prefixes, several key
chunks, two mask words and a partly filled cache, and score profiles chosen to drive the softmax through
its reference updates (scores that keep rising along the prefix, scores that fall, single keys far above
the rest).  Each output row is compared with the float64 oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import eagle2_oracle as orc
from oracle import fp8_kv_oracle as f8
from paper_2406_16858_amd import DraftRound
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _cfg(name, **kw):
    base = dict(name=name, index=0, dtype="bf16", batch=1, vocab=4096, hidden=512, depth=4, topk=5, n_tree=24,
                n_q_heads=8, n_kv_heads=2, head_dim=64, prefix_lo=0, prefix_hi=0, n_layers=1, w_std=0.05,
                accept="greedy", temperature=1.0, seed=777)
    base.update(kw)
    return wl.RoundConfig(**base)


def _random_tree_mask(n, rng):
    """Ancestor-or-self matrix of a random tree on n nodes (node 0 is the root, parent[i] < i)."""
    mask = np.zeros((n, n), dtype=bool)
    mask[0, 0] = True
    for i in range(1, n):
        p = int(rng.integers(0, i))
        mask[i] = mask[p]
        mask[i, i] = True
    return mask


def _mask_words(mask):
    n = mask.shape[0]
    words = (n + 63) // 64
    out = np.zeros((n, words), dtype=np.uint64)
    for i in range(n):
        for j in np.flatnonzero(mask[i]):
            out[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return out


def _run(cfg, region, fp8=False, key_gain=None, spikes=0, filled=None, seed=0, zero_k_scale_head=None):
    """region: allocated prefix rows per sequence; filled: rows in use per sequence (a pre-allocated cache)
    or None; key_gain(t, P) -> factor applied to prefix key t of a P-key prefix; spikes: number of prefix
    keys per sequence replaced by a multiple of one of the sequence's queries (a score far above the rest)."""
    rng = np.random.default_rng(1000 + seed)
    B, N, Hq, Hkv, dh = cfg.batch, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    g = Hq // Hkv
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda", prefix_lens=region)
    offs = off.cpu().numpy()
    used = list(region) if filled is None else list(filled)
    if key_gain is not None or spikes:
        Kf = Kp.float()
        for b in range(B):
            lo, P = int(offs[b]), used[b]
            if key_gain is not None and P:
                gain = torch.tensor([key_gain(t, P) for t in range(P)], dtype=torch.float32, device=Kf.device)
                Kf[lo:lo + P] *= gain[:, None, None]
            for _ in range(spikes if P else 0):
                t, n, h = int(rng.integers(0, P)), int(rng.integers(0, N)), int(rng.integers(0, Hq))
                Kf[lo + t, h // g] = 2.5 * Q[b, n, h].float()
        Kp = Kf.to(Kp.dtype)
    masks = [_random_tree_mask(N, rng) for _ in range(B)]
    rnd = DraftRound(B, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, N, cfg.dtype, Hq, Hkv, dh, total_prefix=sum(region))
    rnd.mask_bits.copy_(torch.from_numpy(np.stack([_mask_words(m) for m in masks]).view(np.int64)))
    O = torch.full_like(Q, float("nan"))
    lse = torch.full((B, N, Hq), float("nan"), dtype=torch.float32, device="cuda")
    plen = None if filled is None else torch.tensor(filled, dtype=torch.int32, device="cuda")
    if fp8:
        K8, V8, ks, vs = wl.make_fp8_prefix(Kp, Vp)
        if zero_k_scale_head is not None:
            ks[zero_k_scale_head] = 0.0                # every prefix key of that head reads as zero
        rnd.tree_attn_fp8kv(Q, K8, V8, ks, vs, off, Kt, Vt, O, lse, prefix_len=plen)
        Kd = torch.from_numpy(f8.dequantize(K8.cpu().numpy(), ks.cpu().numpy()))
        Vd = torch.from_numpy(f8.dequantize(V8.cpu().numpy(), vs.cpu().numpy()))
    else:
        rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, lse, prefix_len=plen)
        Kd, Vd = Kp, Vp
    torch.cuda.synchronize()
    tol = pu.REL_TOL["bf16"]
    worst = 0.0
    for b in range(B):
        lo = int(offs[b])
        hi = lo + used[b]
        ref, ref_lse = orc.tree_attn(pu.f64(Q[b]), pu.f64(Kd[lo:hi]), pu.f64(Vd[lo:hi]), pu.f64(Kt[b]), pu.f64(Vt[b]), masks[b])
        got = pu.f64(O[b])
        assert np.isfinite(got).all(), f"seq {b}: non-finite output"
        for h in range(Hq):
            e = pu.rel_err(got[:, h], ref[:, h])
            worst = max(worst, e)
            assert e <= tol, f"seq {b} head {h}: attention rel err {e:.3e} > {tol}"
        le = float(np.max(np.abs(pu.f64(lse[b]) - ref_lse)))
        assert le <= tol * max(1.0, float(np.abs(ref_lse).max())), f"seq {b}: lse err {le:.3e}"
    return worst


# rows per KV head = (Hq / Hkv) * N; more than 256 selects the wide kernels
SHAPES = {
    "narrow_dh64": dict(batch=3, n_tree=24, n_q_heads=8, n_kv_heads=2, head_dim=64),
    "narrow_dh128": dict(batch=2, n_tree=60, n_q_heads=8, n_kv_heads=2, head_dim=128),
    "wide_dh64": dict(batch=3, n_tree=40, n_q_heads=16, n_kv_heads=2, head_dim=64),
    "wide_dh128": dict(batch=2, n_tree=60, n_q_heads=16, n_kv_heads=2, head_dim=128),
    "wide_dh64_two_mask_words": dict(batch=2, n_tree=128, topk=16, depth=3, n_q_heads=8, n_kv_heads=2, head_dim=64),
    "wide_dh128_ragged_rows": dict(batch=1, n_tree=37, n_q_heads=8, n_kv_heads=1, head_dim=128),   # 296 rows: last block partly used
}
REGIONS = {1: [[700], [63], [0]], 2: [[999, 65], [64, 0], [1, 129]], 3: [[130, 700, 0], [65, 64, 63], [2049, 1, 300]]}


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16_prefix", "fp8_prefix"])
@pytest.mark.parametrize("shape", list(SHAPES))
def test_shapes_and_ragged_prefixes(shape, fp8):
    cfg = _cfg(shape, **SHAPES[shape])
    for i, region in enumerate(REGIONS[cfg.batch]):
        _run(cfg, region, fp8=fp8, seed=i)


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16_prefix", "fp8_prefix"])
@pytest.mark.parametrize("shape", ["narrow_dh128", "wide_dh64", "wide_dh128"])
def test_several_key_chunks_and_partly_filled_cache(shape, fp8):
    cfg = _cfg(shape, **SHAPES[shape])
    region = [9000, 2500, 4097][:cfg.batch]
    _run(cfg, region, fp8=fp8, seed=5)
    _run(cfg, region, fp8=fp8, filled=[5000, 0, 4096][:cfg.batch], seed=6)


PROFILES = {
    # the row maximum keeps climbing along the prefix: the reference is moved again and again
    "rising": lambda t, P: 0.2 + 4.0 * t / max(P - 1, 1),
    # the first tile holds the maximum: everything after it is far below the reference
    "falling": lambda t, P: 4.2 - 4.0 * t / max(P - 1, 1),
    # quiet stretches between loud ones
    "bursts": lambda t, P: 4.0 if (t // 97) % 3 == 2 else 0.3,
}


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16_prefix", "fp8_prefix"])
@pytest.mark.parametrize("profile", list(PROFILES))
@pytest.mark.parametrize("shape", ["narrow_dh64", "narrow_dh128", "wide_dh64", "wide_dh128"])
def test_score_profiles_that_move_the_softmax_reference(shape, profile, fp8):
    cfg = _cfg(shape, **SHAPES[shape])
    region = [1500, 700, 333][:cfg.batch]
    _run(cfg, region, fp8=fp8, key_gain=PROFILES[profile], seed=7)


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16_prefix", "fp8_prefix"])
@pytest.mark.parametrize("shape", ["narrow_dh128", "wide_dh64", "wide_dh128"])
def test_single_keys_far_above_the_rest(shape, fp8):
    """A few prefix keys aligned with one query each: that row's score jumps by tens of log2 units in
    the middle of the stream while the other rows of the wave stay where they were."""
    cfg = _cfg(shape, **SHAPES[shape])
    region = [1500, 700, 333][:cfg.batch]
    _run(cfg, region, fp8=fp8, spikes=6, seed=8)


@pytest.mark.parametrize("shape", ["narrow_dh128", "wide_dh64"])
def test_key_scale_of_zero(shape):
    """An all-zero key head stored with scale 0: its prefix scores are all 0 (uniform weights), the
    tree keys of the same launch keep their own scale."""
    cfg = _cfg(shape, **SHAPES[shape])
    _run(cfg, [700, 130, 64][:cfg.batch], fp8=True, zero_k_scale_head=1, seed=9)


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16_prefix", "fp8_prefix"])
@pytest.mark.parametrize("shape", ["narrow_dh128", "wide_dh64", "wide_dh128"])
@pytest.mark.parametrize("log2_factor", [100, -100])
def test_values_scaled_by_a_power_of_two_scale_the_output_exactly(shape, log2_factor, fp8):
    """Multiplying every value row by 2^k multiplies every product, sum and rounding step by 2^k exactly (no
    overflow, no subnormals), so the output must be the unscaled output times 2^k bit for bit -- including through
    the split-KV partial outputs, which leave the workgroups as 16-bit floats under a per-row power-of-two scale
    (a fixed 16-bit format would overflow at 2^100 and flush to zero at 2^-100).  Several key chunks per sequence."""
    cfg = _cfg("pow2_" + shape, **SHAPES[shape])
    region = [700, 2049, 300][:cfg.batch]
    B, N, Hq, Hkv, dh = cfg.batch, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda", prefix_lens=region)
    rng = np.random.default_rng(4242)
    masks = [_random_tree_mask(N, rng) for _ in range(B)]
    rnd = DraftRound(B, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, N, cfg.dtype, Hq, Hkv, dh, total_prefix=sum(region))
    rnd.mask_bits.copy_(torch.from_numpy(np.stack([_mask_words(m) for m in masks]).view(np.int64)))
    f = 2.0 ** log2_factor
    outs = []
    for factor in (1.0, f):
        O = torch.full_like(Q, float("nan"))
        Vts = (Vt.float() * factor).to(Vt.dtype)
        if fp8:
            K8, V8, ks, vs = wl.make_fp8_prefix(Kp, Vp)
            rnd.tree_attn_fp8kv(Q, K8, V8, ks, vs * factor, off, Kt, Vts, O, None)     # the value scale carries the factor
        else:
            rnd.tree_attn(Q, Kp, (Vp.float() * factor).to(Vp.dtype), off, Kt, Vts, O, None)
        torch.cuda.synchronize()
        outs.append(O.float())
    assert torch.isfinite(outs[1]).all()
    assert float(outs[0].abs().max()) > 0.0
    assert torch.equal(outs[0] * f, outs[1]), "the output did not scale exactly with the values"
