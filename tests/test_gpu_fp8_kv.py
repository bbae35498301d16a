"""GPU parity of the 8-bit prefix KV cache variant (eagle2_tree_attn_fp8kv, eagle2_commit_kv_fp8)
against the oracle: attention over the dequantised prefix within the bf16 tolerance, codes written
by the quantising commit bit-exact."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import eagle2_oracle as orc
from oracle import fp8_kv_oracle as f8
from tests import parity_utils as pu

pytestmark = pytest.mark.gpu


def _cfg(name, **kw):
    base = dict(name=name, index=0, dtype="bf16", batch=1, vocab=4096, hidden=512, depth=4, topk=5, n_tree=24,
                n_q_heads=8, n_kv_heads=2, head_dim=64, prefix_lo=130, prefix_hi=130, n_layers=1, w_std=0.05,
                accept="greedy", temperature=1.0, seed=4321)
    base.update(kw)
    return wl.RoundConfig(**base)


def _round(cfg, total_prefix):
    from paper_2406_16858_amd import DraftRound
    return DraftRound(cfg.batch, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, cfg.n_tree, cfg.dtype, cfg.n_q_heads,
                      cfg.n_kv_heads, cfg.head_dim, total_prefix=total_prefix)


def _random_tree_masks(rng, B, N):
    """Per sequence a random tree on N rows (row 0 the root): boolean masks and their bit words."""
    words = (N + 63) // 64
    masks, bits = [], np.zeros((B, N, words), dtype=np.uint64)
    for b in range(B):
        m = np.zeros((N, N), dtype=bool)
        for i in range(N):
            if i > 0:
                m[i] = m[int(rng.integers(0, i))]
            m[i, i] = True
            for j in np.flatnonzero(m[i]):
                bits[b, i, j >> 6] |= np.uint64(1) << np.uint64(j & 63)
        masks.append(m)
    return masks, bits


def test_every_code_decodes_exactly():
    """With zero queries every visible key weighs the same; a row that sees one prefix key and itself
    (value 0) returns half the prefix value, so a value scale of 2 hands back the decoded codes."""
    cfg = _cfg("codes", batch=2, n_tree=2, n_q_heads=1, n_kv_heads=1, head_dim=128)
    rnd = _round(cfg, 2)
    codes = np.arange(256, dtype=np.uint8).reshape(2, 1, 128).copy()
    codes[codes == 0x7f] = 0x00                         # the two NaN codes are not allowed in a cache
    codes[codes == 0xff] = 0x80
    V8 = torch.from_numpy(codes).cuda()
    K8 = torch.from_numpy(np.flip(codes, 2).copy()).cuda()
    Q = torch.zeros((2, 2, 1, 128), dtype=torch.bfloat16, device="cuda")
    Kt = torch.ones((2, 2, 1, 128), dtype=torch.bfloat16, device="cuda")
    Vt = torch.zeros_like(Kt)
    off = torch.tensor([0, 1, 2], dtype=torch.int64, device="cuda")
    rnd.mask_bits.copy_(torch.tensor([[[1], [3]], [[1], [3]]], dtype=torch.int64))
    ks = torch.tensor([0.37], dtype=torch.float32, device="cuda")
    vs = torch.tensor([2.0], dtype=torch.float32, device="cuda")
    O = torch.full_like(Q, float("nan"))
    rnd.tree_attn_fp8kv(Q, K8, V8, ks, vs, off, Kt, Vt, O)
    torch.cuda.synchronize()
    got = pu.f64(O[:, 0, 0])
    assert np.array_equal(got, f8.e4m3_decode(codes[:, 0]))


@pytest.mark.parametrize("shape", ["narrow_dh64", "narrow_dh128", "wide_dh128", "wide_dh64", "partly_filled", "two_mask_words",
                                   "no_prefix"])
def test_fp8_prefix_attention_parity(shape):
    kw = dict(narrow_dh64=dict(batch=4, n_tree=24, n_q_heads=8, n_kv_heads=2, head_dim=64),
              narrow_dh128=dict(batch=3, n_tree=60, n_q_heads=8, n_kv_heads=2, head_dim=128),
              wide_dh128=dict(batch=2, n_tree=40, n_q_heads=16, n_kv_heads=2, head_dim=128),
              wide_dh64=dict(batch=2, n_tree=80, n_q_heads=16, n_kv_heads=2, head_dim=64),
              partly_filled=dict(batch=4, n_tree=24, n_q_heads=8, n_kv_heads=2, head_dim=128),
              two_mask_words=dict(batch=2, n_tree=128, topk=16, depth=3, n_q_heads=8, n_kv_heads=2, head_dim=128),
              no_prefix=dict(batch=3, n_tree=24, n_q_heads=8, n_kv_heads=2, head_dim=128))[shape]
    cfg = _cfg("fp8_" + shape, seed=91, **kw)
    B, N = cfg.batch, cfg.n_tree
    region = {4: [0, 77, 2300, 64], 3: [513, 1, 190], 2: [700, 129]}[B]
    if shape == "no_prefix":
        region = [0, 0, 0]
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda", prefix_lens=region)
    K8, V8, ks, vs = wl.make_fp8_prefix(Kp, Vp)
    plen = None
    filled = list(region)
    if shape == "partly_filled":
        filled = [0, 40, 2300, 63]
        plen = torch.tensor(filled, dtype=torch.int32, device="cuda")
        K8[int(off[1]) + 40: int(off[2])] = 0x7f        # unfilled rows hold garbage (NaN codes)
        V8[int(off[1]) + 40: int(off[2])] = 0x7f
    rnd = _round(cfg, sum(region))
    rng = np.random.default_rng(17)
    masks, bits = _random_tree_masks(rng, B, N)
    rnd.mask_bits.copy_(torch.from_numpy(bits.view(np.int64)))
    O = torch.full_like(Q, float("nan"))
    lse = torch.full((B, N, cfg.n_q_heads), float("nan"), dtype=torch.float32, device="cuda")
    rnd.tree_attn_fp8kv(Q, K8, V8, ks, vs, off, Kt, Vt, O, lse, prefix_len=plen)
    torch.cuda.synchronize()
    assert not torch.isnan(O.float()).any()
    offs = off.cpu().numpy()
    k8, v8 = K8.cpu().numpy(), V8.cpu().numpy()
    ksn, vsn = ks.cpu().numpy(), vs.cpu().numpy()
    worst = 0.0
    for b in range(B):
        lo = int(offs[b])
        kd = f8.dequantize(k8[lo:lo + filled[b]], ksn)
        vd = f8.dequantize(v8[lo:lo + filled[b]], vsn)
        ref, ref_lse = orc.tree_attn(pu.f64(Q[b]), kd, vd, pu.f64(Kt[b]), pu.f64(Vt[b]), masks[b])
        e = pu.rel_err(pu.f64(O[b]), ref)
        worst = max(worst, e)
        assert e <= pu.REL_TOL["bf16"], f"seq {b}: rel err {e:.2e}"
        assert np.max(np.abs(pu.f64(lse[b]) - ref_lse)) <= pu.REL_TOL["bf16"] * max(1.0, np.abs(ref_lse).max())
    print(f"fp8 prefix {shape}: max rel err {worst:.2e}")


def test_commit_kv_fp8_bit_exact_and_next_round_reads_it():
    cfg = _cfg("fp8_commit", batch=3, depth=4, topk=5, n_tree=24, n_q_heads=8, n_kv_heads=2, head_dim=128, seed=5)
    B, N, D, Hkv, dh, L = cfg.batch, cfg.n_tree, cfg.depth, cfg.n_kv_heads, cfg.head_dim, 3
    region = [40, 12, 30]
    plen = [17, 9, 30]                                   # sequence 1 has room for 3 rows only, sequence 2 for none
    rng = np.random.default_rng(23)
    Kt = torch.randn((L, B, N, Hkv, dh), dtype=torch.float32).to(torch.bfloat16)
    Vt = torch.randn((L, B, N, Hkv, dh), dtype=torch.float32).to(torch.bfloat16)
    ks = torch.tensor(rng.uniform(0.004, 0.02, (L, Hkv)), dtype=torch.float32)
    vs = torch.tensor([[2.0 ** -7, 2.0 ** -6]] * L, dtype=torch.float32)          # exact quotients: half-way cases are hit
    # planted values: beyond the largest code, half-way points between codes, tiny, signed zeros
    halfway = (f8.e4m3_decode(np.arange(126)) + f8.e4m3_decode(np.arange(1, 127))) / 2
    special = np.concatenate([halfway, -halfway, [8192.0, -8192.0, 0.0, -0.0, 2.0 ** -11, 448.0, 464.0, 480.0]])
    for h in range(Hkv):
        vals = torch.tensor(special * float(vs[0, h]), dtype=torch.float32).to(torch.bfloat16)
        assert np.array_equal(pu.f64(vals), special * float(vs[0, h]))             # all on the bf16 grid
        Vt[0, 0, 0, h, :] = vals[:dh]
        Vt[0, 0, 3, h, :] = vals[dh:2 * dh]
        Vt[1, 0, 5, h, : len(special) - 2 * dh] = vals[2 * dh:]
    total = sum(region)
    off = torch.zeros(B + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.tensor(region), 0)
    Kc = torch.full((L, total, Hkv, dh), 0x55, dtype=torch.uint8)
    Vc = torch.full((L, total, Hkv, dh), 0x55, dtype=torch.uint8)
    paths = [[0, 3, 5, 11], [0, 1, 2, 7, 9], [0, 4]]
    rnd = _round(cfg, total)
    ap = np.full((B, D + 1), -1, dtype=np.int32)
    for b, p in enumerate(paths):
        ap[b, : len(p)] = p
    rnd.accept_path.copy_(torch.from_numpy(ap))
    rnd.accept_len.copy_(torch.tensor([len(p) - 1 for p in paths], dtype=torch.int32))
    Kc_d, Vc_d = Kc.cuda(), Vc.cuda()
    rnd.commit_kv_fp8(off.cuda(), torch.tensor(plen, dtype=torch.int32, device="cuda"), Kt.cuda(), Vt.cuda(), Kc_d, Vc_d,
                      ks.cuda(), vs.cuda(), n_layers=L, tree_layer_stride=B * N * Hkv * dh, cache_layer_stride=total * Hkv * dh)
    torch.cuda.synchronize()
    Kw, Vw = Kc.numpy().copy(), Vc.numpy().copy()
    new_len = []
    for layer in range(L):
        for b in range(B):
            n = f8.commit_kv_fp8(Kw[layer], Vw[layer], int(off[b]), int(off[b + 1]), plen[b], pu.f64(Kt[layer, b]),
                                 pu.f64(Vt[layer, b]), paths[b], ks[layer].numpy(), vs[layer].numpy())
            if layer == 0:
                new_len.append(n)
    assert new_len == [21, 12, 30]
    assert np.array_equal(Kc_d.cpu().numpy(), Kw)
    assert np.array_equal(Vc_d.cpu().numpy(), Vw)

    # the next round's attention over the grown 8-bit cache (layer 1) equals the oracle over its dequantised rows
    Q, _, _, Kt2, Vt2, _ = wl.make_attention_inputs(cfg, "cuda", prefix_lens=region)
    masks, bits = _random_tree_masks(rng, B, N)
    rnd.mask_bits.copy_(torch.from_numpy(bits.view(np.int64)))
    O = torch.full_like(Q, float("nan"))
    rnd.tree_attn_fp8kv(Q, Kc_d[1], Vc_d[1], ks[1].cuda(), vs[1].cuda(), off.cuda(), Kt2, Vt2, O,
                        prefix_len=torch.tensor(new_len, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    for b in range(B):
        lo = int(off[b])
        kd = f8.dequantize(Kw[1][lo:lo + new_len[b]], ks[1].numpy())
        vd = f8.dequantize(Vw[1][lo:lo + new_len[b]], vs[1].numpy())
        ref, _ = orc.tree_attn(pu.f64(Q[b]), kd, vd, pu.f64(Kt2[b]), pu.f64(Vt2[b]), masks[b])
        assert pu.rel_err(pu.f64(O[b]), ref) <= pu.REL_TOL["bf16"]


def test_fp8_entry_points_reject_float32_and_missing_scales():
    from paper_2406_16858_amd import Eagle2Error
    cfg32 = wl.get_config(1)
    rnd = _round(cfg32, 128)
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg32, "cuda", prefix_lens=[128])
    K8 = torch.zeros(Kp.shape, dtype=torch.uint8, device="cuda")
    s = torch.ones(cfg32.n_kv_heads, dtype=torch.float32, device="cuda")
    O = torch.zeros_like(Q)
    with pytest.raises(Eagle2Error):
        rnd.tree_attn_fp8kv(Q, K8, K8, s, s, off, Kt, Vt, O)
    cfg = _cfg("fp8_args")
    rnd = _round(cfg, 130)
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda")
    K8 = torch.zeros(Kp.shape, dtype=torch.uint8, device="cuda")
    s = torch.ones(cfg.n_kv_heads, dtype=torch.float32, device="cuda")
    O = torch.full_like(Q, 7.0)
    with pytest.raises(Eagle2Error):
        rnd.tree_attn_fp8kv(Q, K8, K8, s, None, off, Kt, Vt, O)
    with pytest.raises(Eagle2Error):
        rnd.commit_kv_fp8(off, torch.zeros(1, dtype=torch.int32, device="cuda"), Kt, Vt, K8, K8, None, s)
    torch.cuda.synchronize()
    assert torch.all(O == 7.0)                           # nothing was enqueued
