"""Host<->device plumbing around the binding: numpy in, C-ABI call on cuda:0, numpy out.

Used by the GPU parity tests, the smoke check and examples; holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import dream_inputs as di
from . import binding as dream

DT = {"f32": dream.F32, "bf16": dream.BF16}
TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


def desc_for(x: di.AttnInputs, scale: float = 0.0):
    B, _, Hq, D = x.q.shape
    return dream.attn_desc(B, Hq, x.k.shape[1], D, DT[x.dtype], x.s_max, scale)


class DeviceAttn:
    """Uploaded attention operands (kept resident so several calls can reuse them)."""

    def __init__(self, x: di.AttnInputs):
        self.x = x
        self.q = dream.to_device(x.q, x.dtype)
        self.k = dream.to_device(x.k, x.dtype)
        self.v = dream.to_device(x.v, x.dtype)
        self.prefix_len = dream.to_device(x.prefix_len)
        self.parent = dream.to_device(x.parent)
        self.n_tree = x.parent.shape[1]
        self.max_kv = int(x.prefix_len.max()) + self.n_tree


def verify_plan(x: di.AttnInputs) -> str:
    """The launch plan run_verify(x) will get (host-only)."""
    return dream.dream_attn_plan_describe(desc_for(x), x.parent.shape[1], int(x.prefix_len.max()) + x.parent.shape[1])


def xattn_plan(x: di.AttnInputs, n_q: int) -> str:
    """The launch plan run_xattn(x, rows with n_q columns, ...) will get (host-only)."""
    return dream.dream_attn_plan_describe(desc_for(x), n_q, int(x.prefix_len.max()) + x.parent.shape[1])


def run_verify(x: di.AttnInputs, tree_mask=None, scale: float = 0.0, want_lse: bool = True, dev: DeviceAttn = None):
    dev = dev or DeviceAttn(x)
    desc = desc_for(x, scale)
    B, T, Hq, D = x.q.shape
    out = torch.full((B, T, Hq, D), float("nan"), dtype=TORCH_DT[x.dtype], device="cuda")
    lse = torch.full((B, Hq, T), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    ws = dream.alloc_workspace(dream.dream_tree_verify_attn_workspace(desc, T, dev.max_kv))
    tm = None if tree_mask is None else dream.to_device(tree_mask)
    dream.dream_tree_verify_attn(desc, dev.q, dev.k, dev.v, dev.prefix_len, T, dev.parent, tm, dev.max_kv, out, lse, ws)
    torch.cuda.synchronize()
    return out_to_f64(out), (None if lse is None else lse.cpu().numpy().astype(np.float64))


def run_xattn(x: di.AttnInputs, rows: np.ndarray, q_node, scale: float = 0.0, dev: DeviceAttn = None):
    """rows: [B, n_q] indices into x.q's row axis giving the query rows of this call; q_node: [B, n_q] or None."""
    dev = dev or DeviceAttn(x)
    desc = desc_for(x, scale)
    B, _, Hq, D = x.q.shape
    n_q = rows.shape[1]
    qsel = np.stack([x.q[b, rows[b]] for b in range(B)])
    q = dream.to_device(qsel, x.dtype)
    out = torch.full((B, n_q, Hq, D), float("nan"), dtype=TORCH_DT[x.dtype], device="cuda")
    ws = dream.alloc_workspace(dream.dream_draft_xattn_workspace(desc, n_q, dev.max_kv))
    qn = None if q_node is None else dream.to_device(np.ascontiguousarray(q_node, dtype=np.int32))
    dream.dream_draft_xattn(desc, q, dev.k, dev.v, dev.prefix_len, dev.n_tree, dev.parent, n_q, qn, dev.max_kv, out, ws)
    torch.cuda.synchronize()
    return out_to_f64(out), qsel


def run_accept(logits: np.ndarray, dtype: str, token: np.ndarray, parent: np.ndarray, max_depth: int):
    B, T, V = logits.shape
    lg = dream.to_device(logits, dtype)
    tok, par = dream.to_device(token), dream.to_device(parent)
    am = torch.full((B, T), -7, dtype=torch.int32, device="cuda")
    alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    path = torch.full((B, max_depth + 1), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_accept_path_workspace(B, T, V))
    dream.dream_accept_path(lg, DT[dtype], B, T, V, tok, par, max_depth, am, alen, path, bonus, ws)
    torch.cuda.synchronize()
    return am.cpu().numpy(), alen.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy()


def run_compress(dtype: str, q, k, n_keys, vis_start, vis_len, keep_num, keep_den, q_pos=None, scores_in=None,
                 gather_src=None, scale: float = 0.0, want_scores: bool = True, row_lse=None):
    """Returns (scores [B,v] float32 or None, kept [B,k] int32, gathered or None)."""
    if scores_in is None:
        B, n_q, Hq, D = q.shape
        Hkv, s_max = k.shape[1], k.shape[2]
        desc = dream.attn_desc(B, Hq, Hkv, D, DT[dtype], s_max, scale)
        dq, dk = dream.to_device(q, dtype), dream.to_device(k, dtype)
    else:
        B = scores_in.shape[0]
        n_q = 1
        desc = dream.attn_desc(B, 1, 1, 64, DT[dtype], max(n_keys, 1), scale)
        dq = dk = None
    k_keep = (vis_len * keep_num + keep_den // 2) // keep_den
    kept = torch.full((B, max(k_keep, 1)), -7, dtype=torch.int32, device="cuda")
    sc_out = torch.full((B, max(vis_len, 1)), float("nan"), dtype=torch.float32, device="cuda") if want_scores else None
    dpos = None if q_pos is None else dream.to_device(np.ascontiguousarray(q_pos, dtype=np.int32))
    dsi = None if scores_in is None else dream.to_device(np.ascontiguousarray(scores_in, dtype=np.float32))
    gsrc = gdst = None
    n_rows_src = row_elems = 0
    if gather_src is not None:
        gsrc = dream.to_device(gather_src, dtype)
        n_rows_src, row_elems = gather_src.shape[1], gather_src.shape[2]
        gdst = torch.zeros((B, max(k_keep, 1), row_elems), dtype=TORCH_DT[dtype], device="cuda")
    ws = dream.alloc_workspace(dream.dream_visual_compress_workspace(desc, n_q, vis_len))
    dlse = None if row_lse is None else dream.to_device(np.ascontiguousarray(row_lse, dtype=np.float32))
    k_rep = dream.dream_visual_compress(desc, dq, dpos, n_q, dk, n_keys, vis_start, vis_len, keep_num, keep_den, dsi,
                                        sc_out, kept, gsrc, n_rows_src, gdst, row_elems, ws, row_lse_in=dlse)
    torch.cuda.synchronize()
    assert k_rep == k_keep
    scores = None if sc_out is None else sc_out.cpu().numpy()[:, :vis_len]
    g = None
    if gdst is not None:
        g = gdst[:, :k_keep]
        g = g.view(torch.int16).cpu().numpy().view(np.uint16) if dtype == "bf16" else g.cpu().numpy()
    return scores, kept.cpu().numpy()[:, :k_keep], g


def run_commit(caches, dtype: str, prefix_len, n_tree: int, path, accept_len):
    """caches: list of numpy [B,Hkv,s_max,D]; returns (list of committed numpy caches as raw bit views, new_len)."""
    B, Hkv, s_max, D = caches[0].shape
    desc = dream.attn_desc(B, 1, Hkv, D, DT[dtype], s_max)
    dev = [dream.to_device(c, dtype) for c in caches]
    pl = dream.to_device(np.ascontiguousarray(prefix_len, dtype=np.int32))
    pth = dream.to_device(np.ascontiguousarray(path, dtype=np.int32))
    al = dream.to_device(np.ascontiguousarray(accept_len, dtype=np.int32))
    new_len = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    dream.dream_kv_commit(desc, dev, pl, n_tree, pth, al, new_len)
    torch.cuda.synchronize()
    view = torch.int32 if dtype == "f32" else torch.int16
    return [t.view(view).cpu().numpy() for t in dev], new_len.cpu().numpy()


def run_expand(logits: np.ndarray, dtype: str, cum: np.ndarray, k: int):
    """Returns (cand_token [B,F,k], cand_score [B,F,k] float32, next_frontier [B,min(k,F*k)])."""
    B, F, V = logits.shape
    lg = dream.to_device(logits, dtype)
    cm = dream.to_device(np.ascontiguousarray(cum, dtype=np.float32))
    kf = min(k, F * k)
    tok = torch.full((B, F, k), -7, dtype=torch.int32, device="cuda")
    sc = torch.full((B, F, k), float("nan"), dtype=torch.float32, device="cuda")
    nxt = torch.full((B, kf), -7, dtype=torch.int32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_tree_expand_workspace(B, F, V, k))
    dream.dream_tree_expand_level(lg, DT[dtype], B, F, V, cm, k, tok, sc, nxt, ws)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), sc.cpu().numpy(), nxt.cpu().numpy()


def run_finalize(pool_score: np.ndarray, pool_parent: np.ndarray, pool_token: np.ndarray, budget: int):
    B, N = pool_score.shape
    T = 1 + min(budget, N - 1)
    par = torch.full((B, T), -7, dtype=torch.int32, device="cuda")
    tok = torch.full((B, T), -7, dtype=torch.int32, device="cuda")
    pidx = torch.full((B, T), -7, dtype=torch.int32, device="cuda")
    n_tree = dream.dream_tree_finalize(dream.to_device(np.ascontiguousarray(pool_score, dtype=np.float32)),
                                       dream.to_device(np.ascontiguousarray(pool_parent, dtype=np.int32)),
                                       dream.to_device(np.ascontiguousarray(pool_token, dtype=np.int32)), B, N, budget, par, tok, pidx)
    torch.cuda.synchronize()
    return n_tree, par.cpu().numpy(), tok.cpu().numpy(), pidx.cpu().numpy()


def run_entropy(dtype: str, q: np.ndarray, k: np.ndarray, n_keys: int, q_pos=None, scale: float = 0.0):
    """Returns (row_entropy [B,Hq,n_q] float32, ae [B] float32)."""
    B, n_q, Hq, D = q.shape
    Hkv, s_max = k.shape[1], k.shape[2]
    desc = dream.attn_desc(B, Hq, Hkv, D, DT[dtype], s_max, scale)
    dq, dk = dream.to_device(q, dtype), dream.to_device(k, dtype)
    qp = None if q_pos is None else dream.to_device(np.ascontiguousarray(q_pos, dtype=np.int32))
    row = torch.full((B, Hq, n_q), float("nan"), dtype=torch.float32, device="cuda")
    ae = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_attention_entropy_workspace(desc, n_q))
    dream.dream_attention_entropy(desc, dq, qp, n_q, dk, n_keys, row, ae, ws)
    torch.cuda.synchronize()
    return row.cpu().numpy(), ae.cpu().numpy()


def run_spec_accept(tlogits: np.ndarray, dlogits: np.ndarray, dtype: str, token, parent, u_accept, u_bonus, max_depth: int,
                    temperature: float = 1.0):
    B, T, V = tlogits.shape
    tl, dl = dream.to_device(tlogits, dtype), dream.to_device(dlogits, dtype)
    tok = dream.to_device(np.ascontiguousarray(token, dtype=np.int32))
    par = dream.to_device(np.ascontiguousarray(parent, dtype=np.int32))
    ua = dream.to_device(np.ascontiguousarray(u_accept, dtype=np.float32))
    ub = dream.to_device(np.ascontiguousarray(u_bonus, dtype=np.float32))
    alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    path = torch.full((B, max_depth + 1), -7, dtype=torch.int32, device="cuda")
    bonus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_spec_accept_workspace(B, T, V))
    dream.dream_spec_accept(tl, dl, DT[dtype], B, T, V, tok, par, ua, ub, max_depth, temperature, alen, path, bonus, ws)
    torch.cuda.synchronize()
    return alen.cpu().numpy(), path.cpu().numpy(), bonus.cpu().numpy()


def run_project(x: np.ndarray, w: np.ndarray, n_heads: int, head_dim: int, row_base=None, row_index=None, cache: np.ndarray = None):
    """bf16 bit-pattern inputs.  Dense mode returns [B,R,H,D] float64; cache mode returns the whole cache as int16 bits."""
    B, R, hidden = x.shape
    s_max = 1 if cache is None else cache.shape[2]
    desc = dream.attn_desc(B, n_heads, n_heads, head_dim, dream.BF16, s_max)
    dx, dw = dream.to_device(x, "bf16"), dream.to_device(w, "bf16")
    if cache is None:
        out = torch.full((B, R, n_heads, head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
        dream.dream_project_rows(desc, dx, R, hidden, dw, n_heads, None, None, out)
        torch.cuda.synchronize()
        return out_to_f64(out)
    out = dream.to_device(cache, "bf16")
    rb = dream.to_device(np.ascontiguousarray(row_base, dtype=np.int32))
    ri = None if row_index is None else dream.to_device(np.ascontiguousarray(row_index, dtype=np.int32))
    dream.dream_project_rows(desc, dx, R, hidden, dw, n_heads, rb, ri, out)
    torch.cuda.synchronize()
    return out.view(torch.int16).cpu().numpy()


def run_project_qkv(e: np.ndarray, s: np.ndarray, wq, wk, wv, n_q_heads, n_kv_heads, head_dim, row_base, row_index, k_cache, v_cache):
    """One launch for a draft level: Q dense from e, K and V from s into the caches.  Returns (q f64, k bits, v bits)."""
    B, R, hidden = e.shape
    desc = dream.attn_desc(B, n_q_heads, n_kv_heads, head_dim, dream.BF16, k_cache.shape[2])
    de, ds = dream.to_device(e, "bf16"), dream.to_device(s, "bf16")
    dwq, dwk, dwv = (dream.to_device(w, "bf16") for w in (wq, wk, wv))
    q = torch.full((B, R, n_q_heads, head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    kc, vc = dream.to_device(k_cache, "bf16"), dream.to_device(v_cache, "bf16")
    rb = dream.to_device(np.ascontiguousarray(row_base, dtype=np.int32))
    ri = dream.to_device(np.ascontiguousarray(row_index, dtype=np.int32))
    dream.dream_project_rows_multi(desc, [(de, dwq, n_q_heads, None, None, q), (ds, dwk, n_kv_heads, rb, ri, kc),
                                          (ds, dwv, n_kv_heads, rb, ri, vc)], R, hidden)
    torch.cuda.synchronize()
    return out_to_f64(q), kc.view(torch.int16).cpu().numpy(), vc.view(torch.int16).cpu().numpy()
