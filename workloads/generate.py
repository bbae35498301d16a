"""Seeded random tensors with the shapes and value distributions of the configurations.

Every tensor comes from its own generator stream, keyed by (config seed, stream
id, layer), so the order in which tensors are requested does not change their
values.  Tensors are returned in the configuration's storage type (bf16 values
are produced by rounding fp32 normals to nearest-even), on the requested device;
both the CPU oracle's tests and the HIP path read exactly these rounded values.
No arithmetic of the method lives here.
"""
from __future__ import annotations

from typing import List, Optional, Tuple

import torch

from .configs import DraftLayerConfig, RoundConfig

# stream ids
_S_W, _S_H, _S_Q, _S_KP, _S_VP, _S_KT, _S_VT, _S_TL, _S_SPIKE, _S_UA, _S_UB, _S_PLEN = range(12)


def _torch_dtype(cfg: RoundConfig) -> torch.dtype:
    return torch.float32 if cfg.dtype == "fp32" else torch.bfloat16


class SeededStream:
    """A generator for one tensor: seed = f(config seed, stream id, layer)."""

    def __init__(self, cfg: RoundConfig, stream: int, layer: int = 0, device="cpu"):
        self.device = torch.device(device)
        self.gen = torch.Generator(device=self.device)
        self.gen.manual_seed(cfg.seed * 4096 + layer * 16 + stream)

    def normal(self, shape, std: float, dtype: torch.dtype, chunk_rows: int = 1 << 15) -> torch.Tensor:
        """N(0, std) drawn in fp32 and rounded to `dtype`, generated in row chunks
        so that the fp32 staging buffer stays small for multi-GB tensors."""
        shape = tuple(int(s) for s in shape)
        out = torch.empty(shape, dtype=dtype, device=self.device)
        if out.numel() == 0:
            return out
        flat = out.view(shape[0], -1) if len(shape) > 1 else out.view(-1, 1)
        for r0 in range(0, flat.shape[0], chunk_rows):
            r1 = min(flat.shape[0], r0 + chunk_rows)
            blk = torch.randn((r1 - r0, flat.shape[1]), generator=self.gen,
                              device=self.device, dtype=torch.float32)
            flat[r0:r1] = (blk * std).to(dtype)
        return out

    def uniform(self, shape) -> torch.Tensor:
        """fp32 uniforms in [0, 1)."""
        return torch.rand(tuple(shape), generator=self.gen, device=self.device, dtype=torch.float32)

    def integers(self, lo: int, hi: int, shape) -> torch.Tensor:
        """int64 uniform in [lo, hi] inclusive."""
        return torch.randint(lo, hi + 1, tuple(shape), generator=self.gen, device=self.device)


def make_lm_head(cfg: RoundConfig, device="cpu") -> torch.Tensor:
    """W [V, Hd], N(0, w_std), row-major."""
    return SeededStream(cfg, _S_W, 0, device).normal((cfg.vocab, cfg.hidden), cfg.w_std, _torch_dtype(cfg))


def make_hidden_states(cfg: RoundConfig, device="cpu", scale: float = 1.0) -> torch.Tensor:
    """H [B, D, k, Hd], N(0, scale): one hidden state per (sequence, pass, frontier
    slot).  Pass 0 uses slot 0 only.  `scale` > 1 gives the peaked family used for
    parity coverage (draft distributions with confident tokens)."""
    return SeededStream(cfg, _S_H, 0, device).normal(
        (cfg.batch, cfg.depth, cfg.topk, cfg.hidden), scale, _torch_dtype(cfg))


def make_prefix_lengths(cfg: RoundConfig) -> List[int]:
    """Per-sequence KV prefix lengths, uniform in [prefix_lo, prefix_hi]."""
    if cfg.prefix_lo == cfg.prefix_hi:
        return [cfg.prefix_lo] * cfg.batch
    g = SeededStream(cfg, _S_PLEN, 0, "cpu")
    return [int(v) for v in g.integers(cfg.prefix_lo, cfg.prefix_hi, (cfg.batch,))]


def make_attention_inputs(cfg: RoundConfig, device="cpu", layer: int = 0,
                          prefix_lens: Optional[List[int]] = None):
    """Q [B,N,Hq,dh]; K/V prefix [sum P,Hkv,dh]; K/V tree [B,N,Hkv,dh], all N(0,1);
    kv_offsets [B+1] int64 (token offsets of each sequence's prefix)."""
    dt = _torch_dtype(cfg)
    if prefix_lens is None:
        prefix_lens = make_prefix_lengths(cfg)
    total = int(sum(prefix_lens))
    B, N, Hq, Hkv, dh = cfg.batch, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    q = SeededStream(cfg, _S_Q, layer, device).normal((B, N, Hq, dh), 1.0, dt)
    kp = SeededStream(cfg, _S_KP, layer, device).normal((total, Hkv, dh), 1.0, dt)
    vp = SeededStream(cfg, _S_VP, layer, device).normal((total, Hkv, dh), 1.0, dt)
    kt = SeededStream(cfg, _S_KT, layer, device).normal((B, N, Hkv, dh), 1.0, dt)
    vt = SeededStream(cfg, _S_VT, layer, device).normal((B, N, Hkv, dh), 1.0, dt)
    off = torch.zeros(B + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(torch.tensor(prefix_lens, dtype=torch.int64), 0)
    return q, kp, vp, kt, vt, off.to(device)


def make_fp8_prefix(kp: torch.Tensor, vp: torch.Tensor):
    """8-bit image of a prefix K/V pair [T, Hkv, dh] for the quantised-cache variant: per-KV-head scales
    max|x| / 448 (the whole E4M3 range is used; 1 for an empty or all-zero head) and the codes PyTorch's own
    float8_e4m3fn conversion gives for x / scale.  Returns (K codes, V codes) uint8 and (k_scale, v_scale)
    float32 [Hkv], on the tensors' device."""
    def one(x):
        xf = x.detach().to("cpu", torch.float32)
        amax = xf.abs().amax(dim=(0, 2)) if xf.shape[0] else torch.zeros(xf.shape[1])
        scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax)).to(torch.float32)
        q = (xf / scale[None, :, None]).clamp(-448.0, 448.0)
        codes = q.to(torch.float8_e4m3fn).view(torch.uint8)
        return codes.to(x.device), scale.to(x.device)
    k8, ks = one(kp)
    v8, vs = one(vp)
    return k8, v8, ks, vs


def make_target_logits(cfg: RoundConfig, device="cpu", std: float = 3.0,
                       spike: float = 8.0) -> Tuple[torch.Tensor, torch.Tensor]:
    """Target logits [B,N,V] fp32 ~ N(0, std) with `spike` added at one seeded
    token per row.  Returns (logits, spike_token [B,N] int64)."""
    B, N, V = cfg.batch, cfg.n_tree, cfg.vocab
    tl = SeededStream(cfg, _S_TL, 0, device).normal((B * N, V), std, torch.float32).view(B, N, V)
    tok = SeededStream(cfg, _S_SPIKE, 0, device).integers(0, V - 1, (B, N))
    tl.view(B * N, V)[torch.arange(B * N, device=tl.device), tok.view(-1)] += spike
    return tl, tok


def make_uniforms(cfg: RoundConfig, device="cpu") -> Tuple[torch.Tensor, torch.Tensor]:
    """u_accept, u_bonus [B,N] fp32 in [0,1): the random numbers the sampling
    acceptance draws, supplied per tree row."""
    ua = SeededStream(cfg, _S_UA, 0, device).uniform((cfg.batch, cfg.n_tree))
    ub = SeededStream(cfg, _S_UB, 0, device).uniform((cfg.batch, cfg.n_tree))
    return ua, ub


def make_draft_weights(cfg: RoundConfig, dl: DraftLayerConfig, device="cpu") -> dict:
    """Random weights of the draft layer, [out, in] row-major in the configuration's type:
    N(0, 1/sqrt(fan_in)) matrices (activations keep unit scale), gains 1 + N(0, 0.1),
    embeddings N(0, 1)."""
    dt = _torch_dtype(cfg)
    Hd, V = cfg.hidden, cfg.vocab
    qd, kvd, inter = dl.n_q_heads * dl.head_dim, dl.n_kv_heads * dl.head_dim, dl.intermediate

    def mat(stream, rows, cols):
        return SeededStream(cfg, 32 + stream, 0, device).normal((rows, cols), cols ** -0.5, dt)

    def gain(stream):
        g = SeededStream(cfg, 32 + stream, 0, device).normal((Hd,), 0.1, torch.float32) + 1.0
        return g.to(dt)

    return {"embed": SeededStream(cfg, 32, 0, device).normal((V, Hd), 1.0, dt), "fc": mat(1, Hd, 2 * Hd), "g_attn": gain(2),
            "wqkv": mat(3, qd + 2 * kvd, Hd), "wo": mat(4, Hd, qd), "g_mlp": gain(5), "wgu": mat(6, 2 * inter, Hd),
            "wdown": mat(7, Hd, inter)}
