"""ctypes binding of libeagle2_hip.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "_lib", "libeagle2_hip.so")
_lib = None

DTYPE_F32, DTYPE_BF16 = 0, 1
MODE_GREEDY, MODE_SAMPLE = 0, 1
FLAG_RANK_BY_CONFIDENCE, FLAG_NO_RERANK, FLAG_STATIC_TREE = 1, 2, 4


class Eagle2Error(RuntimeError):
    pass


class RoundCfg(C.Structure):
    """Mirror of eagle2_cfg."""
    _fields_ = [("batch", C.c_int32), ("vocab", C.c_int32), ("hidden", C.c_int32), ("depth", C.c_int32),
                ("topk", C.c_int32), ("n_tree", C.c_int32), ("dtype", C.c_int32), ("flags", C.c_int32),
                ("static_tree", C.c_void_p)]

    @property
    def n_cand(self) -> int:
        return self.topk + (self.depth - 1) * self.topk * self.topk

    @property
    def n_draft_rows(self) -> int:
        return 1 + (self.depth - 1) * self.topk


class AttnCfg(C.Structure):
    """Mirror of eagle2_attn_cfg."""
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("scale", C.c_float), ("total_prefix", C.c_int64)]


class DraftCfg(C.Structure):
    """Mirror of eagle2_draft_cfg."""
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("intermediate", C.c_int32),
                ("eps", C.c_float), ("rope_theta", C.c_float)]


class DraftWeights(C.Structure):
    """Mirror of eagle2_draft_weights (device pointers)."""
    _fields_ = [(n, C.c_void_p) for n in ("embed", "fc", "g_attn", "wqkv", "wo", "g_mlp", "wgu", "wdown")]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built library; raises if it is missing (there is no other code path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise Eagle2Error(f"{_LIB_PATH} not found: build it with `python -m paper_2406_16858_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    lib.eagle2_version.restype = C.c_int
    lib.eagle2_last_error.restype = C.c_char_p
    lib.eagle2_workspace_bytes.restype = sz
    lib.eagle2_workspace_bytes.argtypes = [C.POINTER(RoundCfg), C.POINTER(AttnCfg)]
    lib.eagle2_expand.restype = C.c_int
    lib.eagle2_expand.argtypes = [C.POINTER(RoundCfg), i32, vp, i64, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.eagle2_rerank.restype = C.c_int
    lib.eagle2_rerank.argtypes = [C.POINTER(RoundCfg)] + [vp] * 12 + [vp, sz, vp]
    lib.eagle2_tree_attn.restype = C.c_int
    lib.eagle2_tree_attn.argtypes = [C.POINTER(RoundCfg), C.POINTER(AttnCfg)] + [vp] * 10 + [vp, sz, vp]
    lib.eagle2_tree_attn_fp8kv.restype = C.c_int
    lib.eagle2_tree_attn_fp8kv.argtypes = [C.POINTER(RoundCfg), C.POINTER(AttnCfg)] + [vp] * 12 + [vp, sz, vp]
    lib.eagle2_accept.restype = C.c_int
    lib.eagle2_accept.argtypes = [C.POINTER(RoundCfg)] + [vp] * 12 + [vp, sz, vp]
    lib.eagle2_accept_noalloc.restype = C.c_int
    lib.eagle2_accept_noalloc.argtypes = [C.POINTER(RoundCfg)] + [vp] * 12 + [vp]
    lib.eagle2_accept_noalloc_scratch_bytes.restype = sz
    lib.eagle2_accept_noalloc_scratch_bytes.argtypes = []
    lib.eagle2_commit_kv.restype = C.c_int
    lib.eagle2_commit_kv.argtypes = [C.POINTER(RoundCfg), C.POINTER(AttnCfg), i32, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, vp]
    lib.eagle2_commit_kv_fp8.restype = C.c_int
    lib.eagle2_commit_kv_fp8.argtypes = [C.POINTER(RoundCfg), C.POINTER(AttnCfg), i32, vp, vp, vp, vp, vp, vp, i64, vp, vp, i64, vp, vp, vp]
    lib.eagle2_commit_round.restype = C.c_int
    lib.eagle2_commit_round.argtypes = [C.POINTER(RoundCfg)] + [vp] * 9 + [vp]
    lib.eagle2_draft_workspace_bytes.restype = sz
    lib.eagle2_draft_workspace_bytes.argtypes = [C.POINTER(RoundCfg), C.POINTER(DraftCfg), i64]
    lib.eagle2_draft_forward.restype = C.c_int
    lib.eagle2_draft_forward.argtypes = ([C.POINTER(RoundCfg), C.POINTER(DraftCfg), C.POINTER(DraftWeights), i32] + [vp] * 9 +
                                         [i64] + [vp] * 4 + [vp, sz, vp])
    lib.eagle2_kernel_timing_enable.restype = C.c_int
    lib.eagle2_kernel_timing_enable.argtypes = [i32]
    lib.eagle2_kernel_timing_read.restype = C.c_int
    lib.eagle2_kernel_timing_read.argtypes = [i32, C.POINTER(C.c_double), C.POINTER(i32)]
    _lib = lib
    return lib


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None, name: str = "tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise Eagle2Error(f"{name} must live in device memory")
    if not t.is_contiguous():
        raise Eagle2Error(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise Eagle2Error(f"{name} must be {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check(rc: int):
    if rc != 0:
        raise Eagle2Error(f"eagle2 error {rc}: {load_library().eagle2_last_error().decode()}")


def _ws(workspace: Optional[torch.Tensor]):
    if workspace is None:
        return None, 0
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def _elem(cfg: RoundCfg) -> torch.dtype:
    return torch.float32 if cfg.dtype == DTYPE_F32 else torch.bfloat16


def eagle2_version() -> int:
    return load_library().eagle2_version()


def eagle2_workspace_bytes(cfg: RoundCfg, attn: Optional[AttnCfg] = None) -> int:
    return int(load_library().eagle2_workspace_bytes(C.byref(cfg), C.byref(attn) if attn is not None else None))


def eagle2_expand(cfg: RoundCfg, d: int, H: torch.Tensor, W: torch.Tensor, cand_token, cand_score, cand_parent,
                  frontier, draft_logits, workspace, h_seq_stride: int = 0, stream=None):
    lib = load_library()
    el = _elem(cfg)
    # H may be a strided view over sequences; only its first element's address and the stride are passed
    if not H.is_cuda or H.dtype != el:
        raise Eagle2Error("H must be a device tensor of the configured dtype")
    wp, wb = _ws(workspace)
    _check(lib.eagle2_expand(C.byref(cfg), d, C.c_void_p(H.data_ptr()), h_seq_stride, _ptr(W, el, "W"),
                             _ptr(cand_token, torch.int32, "cand_token"), _ptr(cand_score, torch.float64, "cand_score"),
                             _ptr(cand_parent, torch.int32, "cand_parent"), _ptr(frontier, torch.int32, "frontier"),
                             _ptr(draft_logits, torch.float32, "draft_logits"), wp, wb, _stream(stream)))


def eagle2_rerank(cfg: RoundCfg, cand_token, cand_score, cand_parent, frontier, root_token, prefix_len,
                  tree_token, tree_parent, tree_depth, tree_cand, position_ids, mask_bits, workspace=None, stream=None):
    lib = load_library()
    wp, wb = _ws(workspace)
    i32 = torch.int32
    _check(lib.eagle2_rerank(C.byref(cfg), _ptr(cand_token, i32, "cand_token"), _ptr(cand_score, torch.float64, "cand_score"),
                             _ptr(cand_parent, i32, "cand_parent"), _ptr(frontier, i32, "frontier"),
                             _ptr(root_token, i32, "root_token"),
                             _ptr(prefix_len, i32, "prefix_len"), _ptr(tree_token, i32, "tree_token"),
                             _ptr(tree_parent, i32, "tree_parent"), _ptr(tree_depth, i32, "tree_depth"),
                             _ptr(tree_cand, i32, "tree_cand"), _ptr(position_ids, i32, "position_ids"),
                             _ptr(mask_bits, torch.int64, "mask_bits"), wp, wb, _stream(stream)))


def eagle2_tree_attn(cfg: RoundCfg, attn: AttnCfg, Q, K_prefix, V_prefix, kv_offsets, K_tree, V_tree, mask_bits,
                     O, lse, workspace, stream=None, prefix_len=None):
    lib = load_library()
    el = _elem(cfg)
    wp, wb = _ws(workspace)
    _check(lib.eagle2_tree_attn(C.byref(cfg), C.byref(attn), _ptr(Q, el, "Q"), _ptr(K_prefix, el, "K_prefix"),
                                _ptr(V_prefix, el, "V_prefix"), _ptr(kv_offsets, torch.int64, "kv_offsets"),
                                _ptr(prefix_len, torch.int32, "prefix_len"), _ptr(K_tree, el, "K_tree"), _ptr(V_tree, el, "V_tree"),
                                _ptr(mask_bits, torch.int64, "mask_bits"), _ptr(O, el, "O"),
                                _ptr(lse, torch.float32, "lse"), wp, wb, _stream(stream)))


def eagle2_tree_attn_fp8kv(cfg: RoundCfg, attn: AttnCfg, Q, K_prefix8, V_prefix8, k_scale, v_scale, kv_offsets, K_tree, V_tree,
                           mask_bits, O, lse, workspace, stream=None, prefix_len=None):
    lib = load_library()
    el, u8, f32 = _elem(cfg), torch.uint8, torch.float32
    wp, wb = _ws(workspace)
    _check(lib.eagle2_tree_attn_fp8kv(C.byref(cfg), C.byref(attn), _ptr(Q, el, "Q"), _ptr(K_prefix8, u8, "K_prefix8"),
                                      _ptr(V_prefix8, u8, "V_prefix8"), _ptr(k_scale, f32, "k_scale"), _ptr(v_scale, f32, "v_scale"),
                                      _ptr(kv_offsets, torch.int64, "kv_offsets"), _ptr(prefix_len, torch.int32, "prefix_len"),
                                      _ptr(K_tree, el, "K_tree"), _ptr(V_tree, el, "V_tree"),
                                      _ptr(mask_bits, torch.int64, "mask_bits"), _ptr(O, el, "O"),
                                      _ptr(lse, torch.float32, "lse"), wp, wb, _stream(stream)))


def eagle2_accept(cfg: RoundCfg, mode, target_logits, draft_logits, temperature, u_accept, u_bonus,
                  tree_token, tree_parent, tree_cand, accept_len, accept_path, bonus_token, workspace, stream=None):
    lib = load_library()
    wp, wb = _ws(workspace)
    i32, f32 = torch.int32, torch.float32
    _check(lib.eagle2_accept(C.byref(cfg), _ptr(mode, i32, "mode"), _ptr(target_logits, f32, "target_logits"),
                             _ptr(draft_logits, f32, "draft_logits"), _ptr(temperature, f32, "temperature"),
                             _ptr(u_accept, f32, "u_accept"), _ptr(u_bonus, f32, "u_bonus"),
                             _ptr(tree_token, i32, "tree_token"), _ptr(tree_parent, i32, "tree_parent"),
                             _ptr(tree_cand, i32, "tree_cand"), _ptr(accept_len, i32, "accept_len"),
                             _ptr(accept_path, i32, "accept_path"), _ptr(bonus_token, i32, "bonus_token"),
                             wp, wb, _stream(stream)))


def eagle2_accept_noalloc(cfg: RoundCfg, mode, target_logits, draft_logits, temperature, u_accept, u_bonus,
                          tree_token, tree_parent, tree_cand, accept_len, accept_path, bonus_token, stream=None):
    """eagle2_accept without a workspace argument: the scratch is a fixed device array inside the library."""
    lib = load_library()
    i32, f32 = torch.int32, torch.float32
    _check(lib.eagle2_accept_noalloc(C.byref(cfg), _ptr(mode, i32, "mode"), _ptr(target_logits, f32, "target_logits"),
                                     _ptr(draft_logits, f32, "draft_logits"), _ptr(temperature, f32, "temperature"),
                                     _ptr(u_accept, f32, "u_accept"), _ptr(u_bonus, f32, "u_bonus"),
                                     _ptr(tree_token, i32, "tree_token"), _ptr(tree_parent, i32, "tree_parent"),
                                     _ptr(tree_cand, i32, "tree_cand"), _ptr(accept_len, i32, "accept_len"),
                                     _ptr(accept_path, i32, "accept_path"), _ptr(bonus_token, i32, "bonus_token"),
                                     _stream(stream)))


def eagle2_accept_noalloc_scratch_bytes() -> int:
    return int(load_library().eagle2_accept_noalloc_scratch_bytes())


def eagle2_commit_kv(cfg: RoundCfg, attn: AttnCfg, n_layers: int, accept_len, accept_path, kv_offsets, prefix_len,
                     K_tree, V_tree, tree_layer_stride: int, K_cache, V_cache, cache_layer_stride: int, stream=None):
    lib = load_library()
    el, i32 = _elem(cfg), torch.int32
    _check(lib.eagle2_commit_kv(C.byref(cfg), C.byref(attn), n_layers, _ptr(accept_len, i32, "accept_len"),
                                _ptr(accept_path, i32, "accept_path"), _ptr(kv_offsets, torch.int64, "kv_offsets"),
                                _ptr(prefix_len, i32, "prefix_len"), _ptr(K_tree, el, "K_tree"), _ptr(V_tree, el, "V_tree"),
                                tree_layer_stride, _ptr(K_cache, el, "K_cache"), _ptr(V_cache, el, "V_cache"),
                                cache_layer_stride, _stream(stream)))


def eagle2_commit_kv_fp8(cfg: RoundCfg, attn: AttnCfg, n_layers: int, accept_len, accept_path, kv_offsets, prefix_len,
                         K_tree, V_tree, tree_layer_stride: int, K_cache8, V_cache8, cache_layer_stride: int,
                         k_scale, v_scale, stream=None):
    lib = load_library()
    el, i32, u8, f32 = _elem(cfg), torch.int32, torch.uint8, torch.float32
    _check(lib.eagle2_commit_kv_fp8(C.byref(cfg), C.byref(attn), n_layers, _ptr(accept_len, i32, "accept_len"),
                                    _ptr(accept_path, i32, "accept_path"), _ptr(kv_offsets, torch.int64, "kv_offsets"),
                                    _ptr(prefix_len, i32, "prefix_len"), _ptr(K_tree, el, "K_tree"), _ptr(V_tree, el, "V_tree"),
                                    tree_layer_stride, _ptr(K_cache8, u8, "K_cache8"), _ptr(V_cache8, u8, "V_cache8"),
                                    cache_layer_stride, _ptr(k_scale, f32, "k_scale"), _ptr(v_scale, f32, "v_scale"),
                                    _stream(stream)))


def eagle2_commit_round(cfg: RoundCfg, accept_len, accept_path, tree_token, bonus_token, target_hidden,
                        out_tokens, root_token, prefix_len, next_hidden, stream=None):
    lib = load_library()
    el, i32 = _elem(cfg), torch.int32
    _check(lib.eagle2_commit_round(C.byref(cfg), _ptr(accept_len, i32, "accept_len"), _ptr(accept_path, i32, "accept_path"),
                                   _ptr(tree_token, i32, "tree_token"), _ptr(bonus_token, i32, "bonus_token"),
                                   _ptr(target_hidden, el, "target_hidden"), _ptr(out_tokens, i32, "out_tokens"),
                                   _ptr(root_token, i32, "root_token"), _ptr(prefix_len, i32, "prefix_len"),
                                   _ptr(next_hidden, el, "next_hidden"), _stream(stream)))


def eagle2_draft_workspace_bytes(cfg: RoundCfg, draft: DraftCfg, total_prefix: int) -> int:
    return int(load_library().eagle2_draft_workspace_bytes(C.byref(cfg), C.byref(draft), total_prefix))


def draft_weights(cfg: RoundCfg, tensors: dict) -> DraftWeights:
    """Packs device tensors (keys as the struct's fields) into eagle2_draft_weights; the caller keeps them alive."""
    el = _elem(cfg)
    return DraftWeights(**{n: _ptr(tensors[n], el, n).value for n, _ in DraftWeights._fields_})


def eagle2_draft_forward(cfg: RoundCfg, draft: DraftCfg, weights: DraftWeights, d: int, cand_token, cand_parent, frontier,
                         root_token, root_feature, prefix_len, K_prefix, V_prefix, kv_offsets, total_prefix: int,
                         draft_feature, K_draft, V_draft, draft_mask, workspace, stream=None):
    lib = load_library()
    el, i32 = _elem(cfg), torch.int32
    wp, wb = _ws(workspace)
    _check(lib.eagle2_draft_forward(C.byref(cfg), C.byref(draft), C.byref(weights), d, _ptr(cand_token, i32, "cand_token"),
                                    _ptr(cand_parent, i32, "cand_parent"), _ptr(frontier, i32, "frontier"),
                                    _ptr(root_token, i32, "root_token"), _ptr(root_feature, el, "root_feature"),
                                    _ptr(prefix_len, i32, "prefix_len"), _ptr(K_prefix, el, "K_prefix"),
                                    _ptr(V_prefix, el, "V_prefix"), _ptr(kv_offsets, torch.int64, "kv_offsets"), total_prefix,
                                    _ptr(draft_feature, el, "draft_feature"), _ptr(K_draft, el, "K_draft"),
                                    _ptr(V_draft, el, "V_draft"), _ptr(draft_mask, torch.int64, "draft_mask"), wp, wb, _stream(stream)))


def eagle2_kernel_timing_enable(enable: bool):
    _check(load_library().eagle2_kernel_timing_enable(1 if enable else 0))


def eagle2_kernel_timing_read(which: int):
    ms, n = C.c_double(0.0), C.c_int32(0)
    _check(load_library().eagle2_kernel_timing_read(which, C.byref(ms), C.byref(n)))
    return ms.value, n.value
