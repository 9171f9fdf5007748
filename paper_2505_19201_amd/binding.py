"""ctypes binding of libdream.so: same names and argument order as include/dream.h.

Device buffers are torch tensors (only their data_ptr() crosses the boundary); sizes are Python
ints; `stream` is a torch.cuda.Stream or None (= torch's current stream).  Every wrapper raises
DreamError on a non-zero status.  Nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch

F32, BF16 = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdream.so")

EXPORTED_SYMBOLS = (
    "dream_init", "dream_tree_verify_attn_workspace", "dream_tree_verify_attn",
    "dream_draft_xattn_workspace", "dream_draft_xattn", "dream_visual_compress_workspace",
    "dream_visual_compress", "dream_accept_path_workspace", "dream_accept_path",
    "dream_tree_validate_host", "dream_last_error", "dream_set_kv_splits", "dream_set_q_tiles", "dream_set_tile_waves", "dream_attn_variants",
    "dream_attn_plan_describe", "dream_stream_read", "dream_kv_commit",
    "dream_tree_expand_workspace", "dream_tree_expand_level", "dream_tree_finalize",
    "dream_attention_entropy_workspace", "dream_attention_entropy", "dream_spec_accept_workspace", "dream_spec_accept",
    "dream_project_rows", "dream_project_rows_multi", "dream_accept_path_static", "dream_accept_static_init",
)


class DreamError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libdream status {status}: {message}")
        self.status = status


class AttnDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float), ("s_max", C.c_int64)]


def attn_desc(batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, s_max: int,
              scale: float = 0.0) -> AttnDesc:
    return AttnDesc(batch, n_q_heads, n_kv_heads, head_dim, dtype, scale, s_max)


_lib: Optional[C.CDLL] = None


def library_path() -> str:
    return _LIB_PATH


def load() -> C.CDLL:
    """Load libdream.so.  Raises if it has not been built (python -m paper_2505_19201_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_19201_amd.build`; "
                                    "there is no fallback path")
        lib = C.CDLL(_LIB_PATH)
        for name in EXPORTED_SYMBOLS:
            getattr(lib, name)
        for name in ("dream_tree_verify_attn_workspace", "dream_draft_xattn_workspace",
                     "dream_visual_compress_workspace", "dream_accept_path_workspace", "dream_tree_expand_workspace",
                     "dream_attention_entropy_workspace", "dream_spec_accept_workspace"):
            getattr(lib, name).restype = C.c_size_t
        lib.dream_last_error.restype = C.c_char_p
        lib.dream_set_kv_splits.restype = None
        lib.dream_set_q_tiles.restype = None
        lib.dream_set_tile_waves.restype = None
        _lib = lib
    return _lib


def _dev(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check(status: int) -> None:
    if status != 0:
        raise DreamError(status, load().dream_last_error().decode())


def dream_last_error() -> str:
    return load().dream_last_error().decode()


def dream_set_kv_splits(n_splits: int) -> None:
    load().dream_set_kv_splits(C.c_int32(n_splits))


def dream_set_q_tiles(q_tiles: int) -> None:
    load().dream_set_q_tiles(C.c_int32(q_tiles))


def dream_set_tile_waves(waves: int) -> None:
    load().dream_set_tile_waves(C.c_int32(waves))


def dream_stream_read(src: torch.Tensor, nbytes: int, sink: torch.Tensor, offset_bytes: int = 0, stream=None) -> None:
    if offset_bytes < 0 or offset_bytes + nbytes > src.numel() * src.element_size():
        raise ValueError("range outside the source tensor")
    _check(load().dream_stream_read(C.c_void_p(src.data_ptr() + offset_bytes), C.c_size_t(nbytes), _dev(sink), _stream(stream)))


def dream_attn_variants() -> list:
    buf = C.create_string_buffer(4096)
    _check(load().dream_attn_variants(buf, C.c_size_t(4096)))
    return buf.value.decode().split(";")


def dream_attn_plan_describe(desc: "AttnDesc", n_q: int, max_kv_len: int) -> str:
    buf = C.create_string_buffer(256)
    _check(load().dream_attn_plan_describe(C.byref(desc), C.c_int32(n_q), C.c_int64(max_kv_len), buf, C.c_size_t(256)))
    return buf.value.decode()


def dream_init() -> None:
    _check(load().dream_init())


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch of at least nbytes (allocation is the caller's job in C; the content needs no initialisation)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def to_device(a: np.ndarray, dtype: Optional[str] = None, device="cuda") -> torch.Tensor:
    """Upload a host array; uint16 arrays tagged "bf16" become torch.bfloat16 views of the same bits."""
    if dtype == "bf16" or (dtype is None and a.dtype == np.uint16):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(device).view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def dream_tree_verify_attn_workspace(desc: AttnDesc, n_tree: int, max_kv_len: int) -> int:
    return int(load().dream_tree_verify_attn_workspace(C.byref(desc), C.c_int32(n_tree), C.c_int64(max_kv_len)))


def dream_tree_verify_attn(desc: AttnDesc, q, k_cache, v_cache, prefix_len, n_tree: int, parent, tree_mask,
                           max_kv_len: int, out, lse, workspace, stream=None) -> None:
    _check(load().dream_tree_verify_attn(C.byref(desc), _dev(q), _dev(k_cache), _dev(v_cache), _dev(prefix_len),
                                         C.c_int32(n_tree), _dev(parent), _dev(tree_mask), C.c_int64(max_kv_len),
                                         _dev(out), _dev(lse), _dev(workspace),
                                         C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def dream_draft_xattn_workspace(desc: AttnDesc, n_q: int, max_kv_len: int) -> int:
    return int(load().dream_draft_xattn_workspace(C.byref(desc), C.c_int32(n_q), C.c_int64(max_kv_len)))


def dream_draft_xattn(desc: AttnDesc, q, kx_cache, vx_cache, prefix_len, n_tree: int, parent, n_q: int, q_node,
                      max_kv_len: int, out, workspace, stream=None) -> None:
    _check(load().dream_draft_xattn(C.byref(desc), _dev(q), _dev(kx_cache), _dev(vx_cache), _dev(prefix_len),
                                    C.c_int32(n_tree), _dev(parent), C.c_int32(n_q), _dev(q_node),
                                    C.c_int64(max_kv_len), _dev(out), _dev(workspace),
                                    C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def dream_visual_compress_workspace(desc: AttnDesc, n_q: int, vis_len: int) -> int:
    return int(load().dream_visual_compress_workspace(C.byref(desc), C.c_int32(n_q), C.c_int32(vis_len)))


def dream_visual_compress(desc: AttnDesc, q, q_pos, n_q: int, k_cache, n_keys: int, vis_start: int, vis_len: int,
                          keep_num: int, keep_den: int, scores_in, scores_out, kept_idx, gather_src, n_rows_src: int,
                          gather_dst, row_elems: int, workspace, stream=None, row_lse_in=None) -> int:
    """Returns k, the kept count the library reports through its host out-parameter."""
    n_kept = C.c_int32(-1)
    _check(load().dream_visual_compress(C.byref(desc), _dev(q), _dev(q_pos), C.c_int32(n_q), _dev(k_cache),
                                        C.c_int32(n_keys), C.c_int32(vis_start), C.c_int32(vis_len),
                                        C.c_int32(keep_num), C.c_int32(keep_den), _dev(scores_in), _dev(row_lse_in), _dev(scores_out),
                                        _dev(kept_idx), C.byref(n_kept), _dev(gather_src), C.c_int64(n_rows_src),
                                        _dev(gather_dst), C.c_int64(row_elems), _dev(workspace),
                                        C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))
    return int(n_kept.value)


def dream_accept_path_workspace(batch: int, n_tree: int, vocab: int) -> int:
    return int(load().dream_accept_path_workspace(C.c_int32(batch), C.c_int32(n_tree), C.c_int32(vocab)))


def dream_accept_path(logits, logits_dtype: int, batch: int, n_tree: int, vocab: int, token, parent, max_depth: int,
                      node_argmax, accept_len, accept_path, bonus_token, workspace, stream=None) -> None:
    _check(load().dream_accept_path(_dev(logits), C.c_int32(logits_dtype), C.c_int32(batch), C.c_int32(n_tree),
                                    C.c_int32(vocab), _dev(token), _dev(parent), C.c_int32(max_depth),
                                    _dev(node_argmax), _dev(accept_len), _dev(accept_path), _dev(bonus_token),
                                    _dev(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                                    _stream(stream)))


def dream_accept_static_init() -> None:
    _check(load().dream_accept_static_init())


def dream_accept_path_static(logits, logits_dtype: int, batch: int, n_tree: int, vocab: int, token, parent, max_depth: int,
                             node_argmax, accept_len, accept_path, bonus_token, stream=None) -> None:
    _check(load().dream_accept_path_static(_dev(logits), C.c_int32(logits_dtype), C.c_int32(batch), C.c_int32(n_tree),
                                           C.c_int32(vocab), _dev(token), _dev(parent), C.c_int32(max_depth),
                                           _dev(node_argmax), _dev(accept_len), _dev(accept_path), _dev(bonus_token),
                                           _stream(stream)))


def dream_kv_commit(desc: AttnDesc, caches: Sequence[torch.Tensor], prefix_len: torch.Tensor, n_tree: int,
                    accept_path: torch.Tensor, accept_len: torch.Tensor, prefix_len_out: Optional[torch.Tensor] = None,
                    stream=None) -> None:
    ptrs = (C.c_void_p * len(caches))(*[_dev(c).value for c in caches])
    _check(load().dream_kv_commit(C.byref(desc), ptrs, C.c_int32(len(caches)), _dev(prefix_len), C.c_int32(n_tree),
                                  _dev(accept_path), C.c_int32(accept_path.shape[-1]), _dev(accept_len),
                                  _dev(prefix_len_out), _stream(stream)))


def dream_project_rows(desc: AttnDesc, x, n_rows: int, hidden: int, w, n_heads: int, row_base, row_index, out, stream=None) -> None:
    _check(load().dream_project_rows(C.byref(desc), _dev(x), C.c_int32(n_rows), C.c_int32(hidden), _dev(w), C.c_int32(n_heads),
                                     _dev(row_base), _dev(row_index), _dev(out), _stream(stream)))


class ProjJob(C.Structure):
    _fields_ = [("x", C.c_void_p), ("w", C.c_void_p), ("n_heads", C.c_int32), ("row_base", C.c_void_p),
                ("row_index", C.c_void_p), ("out", C.c_void_p)]


def dream_project_rows_multi(desc: AttnDesc, jobs, n_rows: int, hidden: int, stream=None) -> None:
    """jobs: sequence of (x, w, n_heads, row_base, row_index, out)."""
    arr = (ProjJob * len(jobs))(*[ProjJob(_dev(x), _dev(w), n_heads, _dev(rb), _dev(ri), _dev(out))
                                  for x, w, n_heads, rb, ri, out in jobs])
    _check(load().dream_project_rows_multi(C.byref(desc), arr, C.c_int32(len(jobs)), C.c_int32(n_rows), C.c_int32(hidden),
                                           _stream(stream)))


def dream_spec_accept_workspace(batch: int, n_tree: int, vocab: int) -> int:
    return int(load().dream_spec_accept_workspace(C.c_int32(batch), C.c_int32(n_tree), C.c_int32(vocab)))


def dream_spec_accept(target_logits, draft_logits, logits_dtype: int, batch: int, n_tree: int, vocab: int, token, parent,
                      u_accept, u_bonus, max_depth: int, temperature: float, accept_len, accept_path, bonus_token, workspace,
                      stream=None) -> None:
    _check(load().dream_spec_accept(_dev(target_logits), _dev(draft_logits), C.c_int32(logits_dtype), C.c_int32(batch),
                                    C.c_int32(n_tree), C.c_int32(vocab), _dev(token), _dev(parent), _dev(u_accept), _dev(u_bonus),
                                    C.c_int32(max_depth), C.c_float(temperature), _dev(accept_len), _dev(accept_path),
                                    _dev(bonus_token), _dev(workspace), C.c_size_t(workspace.numel() * workspace.element_size()),
                                    _stream(stream)))


def dream_attention_entropy_workspace(desc: AttnDesc, n_q: int) -> int:
    return int(load().dream_attention_entropy_workspace(C.byref(desc), C.c_int32(n_q)))


def dream_attention_entropy(desc: AttnDesc, q, q_pos, n_q: int, k_cache, n_keys: int, row_entropy, ae, workspace, stream=None) -> None:
    _check(load().dream_attention_entropy(C.byref(desc), _dev(q), _dev(q_pos), C.c_int32(n_q), _dev(k_cache), C.c_int32(n_keys),
                                          _dev(row_entropy), _dev(ae), _dev(workspace),
                                          C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def dream_tree_expand_workspace(batch: int, n_frontier: int, vocab: int, k: int) -> int:
    return int(load().dream_tree_expand_workspace(C.c_int32(batch), C.c_int32(n_frontier), C.c_int32(vocab), C.c_int32(k)))


def dream_tree_expand_level(logits: torch.Tensor, logits_dtype: int, batch: int, n_frontier: int, vocab: int,
                            cum_in: torch.Tensor, k: int, cand_token: torch.Tensor, cand_score: torch.Tensor,
                            next_frontier: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    _check(load().dream_tree_expand_level(_dev(logits), C.c_int32(logits_dtype), C.c_int32(batch), C.c_int32(n_frontier),
                                          C.c_int32(vocab), _dev(cum_in), C.c_int32(k), _dev(cand_token), _dev(cand_score),
                                          _dev(next_frontier), _dev(workspace),
                                          C.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream)))


def dream_tree_finalize(pool_score: torch.Tensor, pool_parent: torch.Tensor, pool_token: torch.Tensor, batch: int, n_pool: int,
                        budget: int, tree_parent: torch.Tensor, tree_token: torch.Tensor, tree_pool_index: torch.Tensor,
                        stream=None) -> int:
    n_tree = C.c_int32(0)
    _check(load().dream_tree_finalize(_dev(pool_score), _dev(pool_parent), _dev(pool_token), C.c_int32(batch), C.c_int32(n_pool),
                                      C.c_int32(budget), _dev(tree_parent), _dev(tree_token), _dev(tree_pool_index),
                                      C.byref(n_tree), _stream(stream)))
    return int(n_tree.value)


def dream_tree_validate_host(parent_host: np.ndarray) -> int:
    """Host-side validation of one parent array; returns the maximum depth."""
    p = np.ascontiguousarray(parent_host, dtype=np.int32)
    depth = C.c_int32(0)
    _check(load().dream_tree_validate_host(p.ctypes.data_as(C.c_void_p), C.c_int32(p.shape[0]), C.byref(depth)))
    return int(depth.value)
