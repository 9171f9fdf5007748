"""ctypes front-end of the float64 CPU oracle (oracle/dream_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package; it
shares no code with the HIP path and never imports it.  The C file is compiled with gcc on first
use (or by `python -m oracle.build`).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dream_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP for the batched loops)."""
    if os.environ.get("DREAM_ORACLE_UBSAN") == "1":
        return build_sanitized()["library"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(run_selftest: bool = False) -> dict:
    """Host-side sanitizer builds of the oracle (gcc; nothing here touches a GPU):
    - oracle/selftest_asan: dream_oracle.c + selftest.c as an executable under -fsanitize=address,undefined; it calls
      every entry point on exact-size heap buffers (an AddressSanitizer library cannot be loaded into an interpreter
      that was not started with it, hence the separate executable);
    - oracle/liboracle_ubsan.so: the shared library under -fsanitize=undefined with errors fatal; the test suite uses it
      when DREAM_ORACLE_UBSAN=1 is set in the environment."""
    exe = os.path.join(_HERE, "selftest_asan")
    ubsan = os.path.join(_HERE, "liboracle_ubsan.so")
    common = ["-O1", "-g", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-fno-omit-frame-pointer"]
    subprocess.check_call(["gcc", *common, "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", exe,
                           _SRC, os.path.join(_HERE, "selftest.c"), "-lm"])
    tmp = ubsan + ".tmp.%d" % os.getpid()
    subprocess.check_call(["gcc", *common, "-fPIC", "-shared", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                           "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, ubsan)
    out = {"selftest": exe, "library": ubsan}
    if run_selftest:
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
        p = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out["selftest_output"] = p.stdout
        if p.returncode != 0:
            raise RuntimeError("oracle selftest under AddressSanitizer/UBSan failed:\n" + p.stdout)
    return out


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_keep_count.restype = C.c_int
        _lib.oracle_topk_keep.restype = C.c_int
        _lib.oracle_tree_attn.restype = C.c_int
        _lib.oracle_visual_scores.restype = C.c_int
        _lib.oracle_accept_path.restype = C.c_int
        _lib.oracle_attention_entropy.restype = C.c_int
        _lib.oracle_kv_commit.restype = C.c_int
        _lib.oracle_get_threads.restype = C.c_int
        _lib.oracle_hw_threads.restype = C.c_int
    return _lib


def set_threads(n: int) -> None:
    lib().oracle_set_threads(C.c_int(int(n)))


def hw_threads() -> int:
    return int(lib().oracle_hw_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(a: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    assert a.dtype == want, (a.dtype, dtype)
    return np.ascontiguousarray(a)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def tree_attn(q, k, v, dtype: str, prefix_len, parent, include_self: bool,
              q_node=None, scale: Optional[float] = None) -> Tuple[np.ndarray, np.ndarray]:
    """q [B,Tq,Hq,D], k/v [B,Hkv,s_max,D], parent [B,T] -> (out [B,Tq,Hq,D] f64, lse [B,Hq,Tq] f64)."""
    q, k, v = _check(q, dtype), _check(k, dtype), _check(v, dtype)
    B, Tq, Hq, D = q.shape
    _, Hkv, s_max, _ = k.shape
    parent = _i32(parent).reshape(B, -1)
    prefix_len = _i32(prefix_len).reshape(B)
    qn = None if q_node is None else _i32(q_node).reshape(B, Tq)
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.zeros((B, Tq, Hq, D), dtype=np.float64)
    lse = np.zeros((B, Hq, Tq), dtype=np.float64)
    rc = lib().oracle_tree_attn(_ptr(q), _ptr(k), _ptr(v), C.c_int(_DT[dtype]), C.c_int(B), C.c_int(Tq),
                                C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int64(s_max), _ptr(prefix_len),
                                C.c_int(parent.shape[1]), _ptr(parent), _ptr(qn), C.c_int(int(include_self)),
                                C.c_double(scale), _ptr(out), _ptr(lse))
    assert rc == 0
    return out, lse


def attn_row(q, k, v, dtype: str, prefix_len, parent, include_self: bool, b: int, h: int, row: int,
             node: Optional[int] = None, scale: Optional[float] = None) -> Tuple[np.ndarray, float]:
    """One output row (sequence b, query head h, query row `row` belonging to tree node `node`)."""
    q, k, v = _check(q, dtype), _check(k, dtype), _check(v, dtype)
    B, Tq, Hq, D = q.shape
    _, Hkv, s_max, _ = k.shape
    parent = _i32(parent).reshape(B, -1)
    node = row if node is None else node
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.zeros(D, dtype=np.float64)
    lse = C.c_double(0.0)
    par_b = np.ascontiguousarray(parent[b])
    q_row = ((b * Tq + row) * Hq + h) * D
    kv_base = (b * Hkv + h // (Hq // Hkv)) * s_max * D
    lib().oracle_attn_row(_ptr(q), _ptr(k), _ptr(v), C.c_int(_DT[dtype]), C.c_int(D), C.c_int64(q_row),
                          C.c_int64(kv_base), C.c_int(int(np.asarray(prefix_len).reshape(-1)[b])), _ptr(par_b),
                          C.c_int(node), C.c_int(int(include_self)), C.c_double(scale), _ptr(out), C.byref(lse))
    return out, float(lse.value)


def visual_scores(q, k, dtype: str, vis_start: int, vis_len: int, q_pos=None,
                  scale: Optional[float] = None, include_diag: bool = True) -> np.ndarray:
    """q [B,Nq,Hq,D], k [B,Hkv,s_max,D] -> scores [B, vis_len] f64."""
    q, k = _check(q, dtype), _check(k, dtype)
    B, n_q, Hq, D = q.shape
    _, Hkv, s_max, _ = k.shape
    qp = None if q_pos is None else _i32(q_pos).reshape(B, n_q)
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    scores = np.zeros((B, vis_len), dtype=np.float64)
    rc = lib().oracle_visual_scores(_ptr(q), _ptr(qp), C.c_int(n_q), _ptr(k), C.c_int(_DT[dtype]), C.c_int(B),
                                    C.c_int(Hq), C.c_int(Hkv), C.c_int(D), C.c_int64(s_max), C.c_int(vis_start),
                                    C.c_int(vis_len), C.c_double(scale), C.c_int(int(include_diag)), _ptr(scores))
    assert rc == 0
    return scores


def keep_count(vis_len: int, keep_num: int, keep_den: int) -> int:
    return int(lib().oracle_keep_count(C.c_int(vis_len), C.c_int(keep_num), C.c_int(keep_den)))


def topk_keep(scores, vis_start: int, keep_num: int, keep_den: int) -> np.ndarray:
    """scores [B, v] (any float dtype; widened exactly to f64) -> kept absolute positions [B, k], ascending."""
    s = np.ascontiguousarray(np.asarray(scores), dtype=np.float64)
    B, v = s.shape
    k = keep_count(v, keep_num, keep_den)
    kept = np.zeros((B, k), dtype=np.int32)
    k2 = lib().oracle_topk_keep(_ptr(s), C.c_int(B), C.c_int(vis_start), C.c_int(v), C.c_int(keep_num),
                                C.c_int(keep_den), _ptr(kept))
    assert k2 == k
    return kept


def gather_rows(src, dtype: str, kept) -> np.ndarray:
    """src [B, n_rows, row_elems], kept [B, k] -> [B, k, row_elems] (byte copy)."""
    src = _check(src, dtype)
    kept = _i32(kept)
    B, n_rows, row_elems = src.shape
    k = kept.shape[1]
    dst = np.zeros((B, k, row_elems), dtype=src.dtype)
    lib().oracle_gather_rows(_ptr(src), C.c_int(_DT[dtype]), C.c_int(B), C.c_int64(n_rows), C.c_int64(row_elems),
                             _ptr(kept), C.c_int(k), _ptr(dst))
    return dst


def accept_path(logits, dtype: str, token, parent, max_depth: int):
    """logits [B,T,V] -> (node_argmax [B,T], accept_len [B], accept_path [B,max_depth+1], bonus [B])."""
    logits = _check(logits, dtype)
    B, T, V = logits.shape
    token, parent = _i32(token).reshape(B, T), _i32(parent).reshape(B, T)
    am = np.zeros((B, T), dtype=np.int32)
    alen = np.zeros(B, dtype=np.int32)
    path = np.zeros((B, max_depth + 1), dtype=np.int32)
    bonus = np.zeros(B, dtype=np.int32)
    rc = lib().oracle_accept_path(_ptr(logits), C.c_int(_DT[dtype]), C.c_int(B), C.c_int(T), C.c_int(V), _ptr(token),
                                  _ptr(parent), C.c_int(max_depth), _ptr(am), _ptr(alen), _ptr(path), _ptr(bonus))
    assert rc == 0
    return am, alen, path, bonus


def kv_commit(cache, dtype: str, prefix_len, n_tree: int, path, accept_len):
    """cache [B,Hkv,s_max,D] -> (committed copy, new_len [B]); path [B, stride] root first."""
    cache = _check(cache, dtype).copy()
    B, Hkv, s_max, D = cache.shape
    prefix_len, accept_len = _i32(prefix_len), _i32(accept_len)
    path = _i32(path).reshape(B, -1)
    new_len = np.zeros(B, dtype=np.int32)
    rc = lib().oracle_kv_commit(_ptr(cache), C.c_int(_DT[dtype]), C.c_int(B), C.c_int(Hkv), C.c_int64(s_max), C.c_int(D),
                                _ptr(prefix_len), C.c_int(n_tree), _ptr(path), C.c_int(path.shape[1]), _ptr(accept_len),
                                _ptr(new_len))
    if rc != 0:
        raise ValueError("kv_commit: path entry or length out of range")
    return cache, new_len


def project(x, w, dtype: str, n_heads: int, head_dim: int) -> np.ndarray:
    """x [B,R,hidden], w [n_heads*head_dim, hidden] -> y [B,R,n_heads,head_dim] f64 (Eq. 1's linear maps)."""
    x, w = _check(x, dtype), _check(w, dtype)
    B, R, hidden = x.shape
    assert w.shape == (n_heads * head_dim, hidden)
    out = np.zeros((B, R, n_heads, head_dim), dtype=np.float64)
    rc = lib().oracle_project(_ptr(x), _ptr(w), C.c_int(_DT[dtype]), C.c_int(B), C.c_int(R), C.c_int(hidden), C.c_int(n_heads),
                              C.c_int(head_dim), _ptr(out))
    assert rc == 0
    return out


def attention_entropy(q, k, dtype: str, q_pos=None, scale: Optional[float] = None):
    """q [B,Nq,Hq,D], k [B,Hkv,s_max,D] -> (row_entropy [B,Hq,Nq] f64, ae [B] f64), Eq. 2."""
    q, k = _check(q, dtype), _check(k, dtype)
    B, n_q, Hq, D = q.shape
    _, Hkv, s_max, _ = k.shape
    qp = None if q_pos is None else _i32(q_pos).reshape(B, n_q)
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    row = np.zeros((B, Hq, n_q), dtype=np.float64)
    ae = np.zeros(B, dtype=np.float64)
    rc = lib().oracle_attention_entropy(_ptr(q), _ptr(qp), C.c_int(n_q), _ptr(k), C.c_int(_DT[dtype]), C.c_int(B), C.c_int(Hq),
                                        C.c_int(Hkv), C.c_int(D), C.c_int64(s_max), C.c_double(scale), _ptr(row), _ptr(ae))
    assert rc == 0
    return row, ae


from .tree_build import expand_level, finalize_tree, build_tree  # noqa: E402,F401  (float64 numpy, same rules as the C part)
from .spec_accept import spec_accept  # noqa: E402,F401
