"""No-GPU checks of the boundary: the library loads, exports every function include/dream.h declares,
and rejects bad arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2505_19201_amd as dream
from paper_2505_19201_amd import build as dream_build


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dream.library_path()):
        dream_build.build(verbose=False)
    return dream.load()


def _declared_functions():
    """Every function any header under include/ declares (the boundary in dream.h, the test switches in dream_tuning.h)."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    names = set()
    for header in sorted(os.listdir(os.path.join(root, "include"))):
        text = open(os.path.join(root, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(dream_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_function_is_exported(lib):
    names = _declared_functions()
    assert {"dream_tree_verify_attn", "dream_draft_xattn", "dream_visual_compress", "dream_accept_path"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(dream.EXPORTED_SYMBOLS) == names


def test_binding_never_imports_the_oracle():
    import sys
    src = open(dream.binding.__file__).read() + open(dream.__file__).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
    assert "oracle" not in [m.split(".")[0] for m in sys.modules if m.startswith("paper_2505_19201_amd")]


def test_tree_validation_on_host(lib):
    assert dream.dream_tree_validate_host(np.array([-1, 0, 0, 1, 3, 4])) == 4
    assert dream.dream_tree_validate_host(np.array([-1])) == 0
    for bad in ([0, 0], [-1, 1], [-1, 0, 3], [-1, -1]):
        with pytest.raises(dream.DreamError) as e:
            dream.dream_tree_validate_host(np.array(bad))
        assert e.value.status == -1


def test_host_side_argument_errors(lib):
    d = dream.attn_desc(1, 4, 4, 64, dream.BF16, 128)
    one = C.c_void_p(16)      # never dereferenced: every call below fails validation first
    f = lib.dream_tree_verify_attn
    args = lambda desc, n_tree=8, maxkv=100, ws=one, wsb=1 << 30, q=one: (  # noqa: E731
        C.byref(desc), q, one, one, one, C.c_int32(n_tree), one, None, C.c_int64(maxkv), one, None, ws, C.c_size_t(wsb), None)
    assert f(*args(d, q=None)) == -1
    assert f(*args(dream.attn_desc(1, 6, 4, 64, dream.BF16, 128))) == -1          # Hq % Hkv
    assert f(*args(dream.attn_desc(1, 4, 4, 96, dream.BF16, 128))) == -2          # head_dim
    assert f(*args(d, n_tree=257)) == -2
    assert f(*args(d, n_tree=0)) == -2
    assert f(*args(d, maxkv=129)) == -1                                           # beyond s_max
    big = dream.attn_desc(1, 32, 8, 128, dream.BF16, 4200)                        # a long cache with few KV heads: key splits need a workspace
    assert dream.dream_tree_verify_attn_workspace(big, 60, 4156) > 65536
    assert f(*args(big, n_tree=60, maxkv=4156, wsb=65536)) == -3                   # workspace too small
    assert "workspace" in dream.dream_last_error()
    g = lib.dream_accept_path
    assert g(one, C.c_int32(1), C.c_int32(1), C.c_int32(2000), C.c_int32(100), one, one, C.c_int32(6), one, one, one, one,
             one, C.c_size_t(1 << 30), None) == -2
    assert g(one, C.c_int32(5), C.c_int32(1), C.c_int32(8), C.c_int32(100), one, one, C.c_int32(6), one, one, one, one,
             one, C.c_size_t(1 << 30), None) == -1
    h = lib.dream_visual_compress
    base = [C.byref(d), one, None, C.c_int32(64), one, C.c_int32(64), C.c_int32(0), C.c_int32(32), C.c_int32(1), C.c_int32(2),
            None, None, None, one, None, None, C.c_int64(0), None, C.c_int64(0), one, C.c_size_t(1 << 30), None]
    bad = list(base); bad[9] = C.c_int32(0)
    assert h(*bad) == -1                                                          # keep_den
    bad = list(base); bad[8] = C.c_int32(3)
    assert h(*bad) == -1                                                          # keep_num > keep_den
    bad = list(base); bad[6] = C.c_int32(40)
    assert h(*bad) == -1                                                          # span beyond keys
    bad = list(base); bad[20] = C.c_size_t(16)
    assert h(*bad) == -3


def test_workspace_sizes_are_monotone(lib):
    d = dream.attn_desc(1, 32, 32, 128, dream.BF16, 800)
    a = dream.dream_tree_verify_attn_workspace(d, 60, 764)
    assert a >= 256
    dream.dream_set_kv_splits(4)
    try:
        assert dream.dream_tree_verify_attn_workspace(d, 60, 764) > a            # forced splits need room for their states
    finally:
        dream.dream_set_kv_splits(0)
    assert dream.dream_accept_path_workspace(1, 60, 32000) >= 2 * 60 * 4 * 4
    assert dream.dream_visual_compress_workspace(d, 704, 576) >= 32 * 704 * 4 + 32 * 576 * 4


def test_launch_plans_of_the_paper_shapes(lib):
    """The plan is host logic: one sequence with a short cache takes the single-launch wave kernel with its output
    columns split over workgroups (MHA, and GQA groups of up to 4 heads), a long cache or a batch of sequences the
    shared-tile kernel, with key splits and a merge launch where the streams are few."""
    def plan(B, hq, hkv, d, n_q, s):
        return dream.dream_attn_plan_describe(dream.attn_desc(B, hq, hkv, d, dream.BF16, s), n_q, s)
    llava = plan(1, 32, 32, 128, 60, 764)
    assert llava.startswith("attn_wave_kernel<128,8,2,1>") and "workgroups=256" in llava and "merge_launch=0" in llava
    level = plan(1, 32, 32, 128, 16, 764)            # one drafted tree level: a single query tile per head
    assert level.startswith("attn_wave_kernel<128,8,4,1>") and "workgroups=128" in level
    pixtral = plan(1, 32, 8, 128, 60, 1340)
    assert pixtral.startswith("attn_wave_kernel<128,8,2,1>") and "workgroups=256" in pixtral and "merge_launch=0" in pixtral
    gemma3 = plan(1, 16, 8, 256, 60, 1340)
    assert gemma3.startswith("attn_wave_kernel<256,4,4,1>") and "workgroups=256" in gemma3
    long_cache = plan(1, 32, 8, 128, 60, 4156)        # more than 64 key tiles
    assert long_cache.startswith("attn_bf16_kernel<128,1,") and "splits=8" in long_cache and "merge_launch=1" in long_cache
    batch = plan(32, 32, 32, 64, 60, 1660)
    assert batch.startswith("attn_bf16_kernel<64,1,") and "splits=1 " in batch and "merge_launch=0" in batch
    f32 = dream.dream_attn_plan_describe(dream.attn_desc(1, 4, 4, 64, dream.F32, 104), 8, 104)
    assert f32.startswith("attn_f32_kernel")
    with pytest.raises(dream.DreamError):
        dream.dream_attn_plan_describe(dream.attn_desc(1, 32, 32, 96, dream.BF16, 764), 60, 764)


def test_every_attention_kernel_variant_has_a_parity_case(lib):
    """The GPU suite runs tests/attn_cases.VARIANT_CASES all elements against the oracle; here, without a GPU: the
    list names every variant the library can dispatch to, and each case's shape really plans its variant."""
    import dream_inputs as di
    from tests.attn_cases import (EXTRA_W8_CASES, FULL_VERIFY_PLANS, FULL_XATTN_PLANS, STREAMING_PLANS, VARIANT_CASES, variant_config,
                                  variant_prefix_lens)
    built = dream.dream_attn_variants()
    assert len(built) == len(set(built))
    assert sorted(c.variant for c in VARIANT_CASES) == sorted(built)
    for case in VARIANT_CASES + EXTRA_W8_CASES:
        cfg = variant_config(case)
        pl = variant_prefix_lens(case)
        assert max(pl) == pl[0] == case.kv_len - case.n_tree and min(pl) >= 0
        dream.dream_set_kv_splits(case.splits)
        dream.dream_set_q_tiles(case.q_tiles)
        dream.dream_set_tile_waves(case.waves)
        try:
            desc = dream.attn_desc(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dream.BF16, case.kv_len + 5)
            plan = dream.dream_attn_plan_describe(desc, case.n_tree, case.kv_len)
        finally:
            dream.dream_set_kv_splits(0)
            dream.dream_set_q_tiles(0)
            dream.dream_set_tile_waves(0)
        assert plan.startswith(case.variant + " "), (case, plan)
    for name, want in FULL_VERIFY_PLANS.items():
        cfg = di.CONFIGS[name]
        S = cfg.prefix + cfg.n_tree
        desc = dream.attn_desc(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dream.BF16, S + 5)
        assert dream.dream_attn_plan_describe(desc, cfg.n_tree, S) == want, name
        for n_q, want_x in zip((1, 10), FULL_XATTN_PLANS[name]):
            assert dream.dream_attn_plan_describe(desc, n_q, S) == want_x, (name, n_q)
        assert want.split(" ")[0] in built
    for name, want in STREAMING_PLANS.items():
        cfg = di.CONFIGS[name].with_batch(32)
        S = cfg.prefix + cfg.n_tree
        desc = dream.attn_desc(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, dream.BF16, S)
        assert dream.dream_attn_plan_describe(desc, cfg.n_tree, S) == want, name


def test_kv_commit_argument_errors(lib):
    """Host-side checks of dream_kv_commit return before any launch."""
    import ctypes as C
    desc = dream.attn_desc(1, 4, 4, 128, dream.BF16, 100)
    ptrs = (C.c_void_p * 1)(0x1000)
    fake = C.c_void_p(0x2000)

    def call(d=desc, caches=ptrs, n=1, pl=fake, n_tree=8, path=fake, stride=7, alen=fake, out=None):
        return lib.dream_kv_commit(C.byref(d), caches, C.c_int32(n), pl, C.c_int32(n_tree), path, C.c_int32(stride), alen,
                                   out, None)
    assert call(caches=None) == -1
    assert call(n=0) == -1
    assert call(n_tree=0) == -1
    assert call(n_tree=101) == -1                  # the tree rows must fit the cache
    assert call(stride=0) == -1
    assert call(out=fake) == -1                    # aliases prefix_len
    assert "alias" in dream.dream_last_error()
    assert call(caches=(C.c_void_p * 1)(0x1008)) == -1   # not 16-byte aligned
    assert call(caches=(C.c_void_p * 1)(None)) == -1
    wide = dream.attn_desc(1, 4, 4, 1024, dream.F32, 1000)   # 4 KB rows: 64 of them exceed 64 KB
    assert call(d=wide, n_tree=64, stride=64) == -2
    odd = dream.attn_desc(1, 4, 4, 60, dream.BF16, 100)      # 120-byte rows
    assert call(d=odd) == -2


def test_tree_build_argument_errors(lib):
    """Host-side checks of the tree-construction entry points return before any launch."""
    import ctypes as C
    fake = C.c_void_p(0x1000)

    def expand(logits=fake, dt=dream.BF16, B=1, F=4, V=32000, cum=fake, k=4, tok=fake, sc=fake, nxt=fake, ws=fake, nb=1 << 30):
        return lib.dream_tree_expand_level(logits, C.c_int32(dt), C.c_int32(B), C.c_int32(F), C.c_int32(V), cum, C.c_int32(k), tok, sc,
                                           nxt, ws, C.c_size_t(nb), None)
    assert expand(logits=None) == -1 and expand(cum=None) == -1 and expand(nxt=None) == -1
    assert expand(dt=7) == -1
    assert expand(F=0) == -1 and expand(F=17) == -1
    assert expand(k=0) == -1 and expand(k=17) == -1 and expand(V=3, k=4) == -1
    assert expand(B=0) == -1 and expand(B=5000, F=16) == -1
    need = dream.dream_tree_expand_workspace(1, 4, 32000, 4)
    assert need > 256 and expand(nb=need - 1) == -3 and expand(ws=None) == -3
    assert dream.dream_tree_expand_workspace(1, 4, 262144, 4) > need
    assert dream.dream_tree_expand_workspace(2, 4, 32000, 4) > need

    def finalize(score=fake, parent=fake, token=fake, B=1, N=85, budget=32, tp=fake, tt=fake, ti=fake):
        n = C.c_int32(-1)
        return lib.dream_tree_finalize(score, parent, token, C.c_int32(B), C.c_int32(N), C.c_int32(budget), tp, tt, ti, C.byref(n), None), n.value
    assert finalize(score=None)[0] == -1 and finalize(ti=None)[0] == -1
    assert finalize(N=0)[0] == -1 and finalize(N=1025)[0] == -1 and finalize(budget=-1)[0] == -1 and finalize(B=0)[0] == -1


def test_attention_entropy_argument_errors(lib):
    import ctypes as C
    fake = C.c_void_p(0x1000)
    desc = dream.attn_desc(1, 32, 32, 128, dream.BF16, 764)

    def call(d=desc, q=fake, n_q=704, k=fake, n_keys=704, ae=fake, ws=fake, nb=1 << 30):
        return lib.dream_attention_entropy(C.byref(d), q, None, C.c_int32(n_q), k, C.c_int32(n_keys), None, ae, ws, C.c_size_t(nb), None)
    assert call(q=None) == -1 and call(k=None) == -1 and call(ae=None) == -1
    assert call(n_q=0) == -1 and call(n_keys=0) == -1 and call(n_keys=765) == -1
    assert call(n_q=705) == -1                       # rows at positions 0..704 but 704 keys
    assert call(d=dream.attn_desc(1, 32, 32, 96, dream.BF16, 764)) == -2
    assert call(d=dream.attn_desc(1, 32, 5, 128, dream.BF16, 764)) == -1
    need = dream.dream_attention_entropy_workspace(desc, 704)
    assert need > 256 and call(nb=need - 1) == -3 and call(ws=None) == -3


def test_spec_accept_argument_errors(lib):
    import ctypes as C
    fake = C.c_void_p(0x1000)

    def call(tl=fake, dl=fake, dt=dream.BF16, B=1, T=60, V=32000, tok=fake, par=fake, ua=fake, ub=fake, depth=6, temp=1.0, al=fake,
             ap=fake, bt=fake, ws=fake, nb=1 << 30):
        return lib.dream_spec_accept(tl, dl, C.c_int32(dt), C.c_int32(B), C.c_int32(T), C.c_int32(V), tok, par, ua, ub, C.c_int32(depth),
                                     C.c_float(temp), al, ap, bt, ws, C.c_size_t(nb), None)
    assert call(tl=None) == -1 and call(dl=None) == -1 and call(ua=None) == -1 and call(ub=None) == -1 and call(bt=None) == -1
    assert call(dt=9) == -1 and call(B=0) == -1 and call(V=0) == -1 and call(depth=-1) == -1 and call(depth=1024) == -1
    assert call(T=0) == -2 and call(T=1025) == -2
    assert call(temp=0.0) == -1 and call(temp=-1.0) == -1
    assert "greedy" in dream.dream_last_error()
    need = dream.dream_spec_accept_workspace(1, 60, 32000)
    assert need == 256 + 3 * 32000 * 4 + 3 * 2048 + 1024 and call(nb=need - 1) == -3 and call(ws=None) == -3
    assert call(B=1100, T=60) == -2                  # more than 65535 rows


def test_project_rows_argument_errors(lib):
    import ctypes as C
    fake = C.c_void_p(0x1000)
    desc = dream.attn_desc(1, 32, 32, 128, dream.BF16, 764)

    def call(d=desc, x=fake, R=10, hid=4096, w=fake, H=32, rb=None, ri=None, out=fake):
        return lib.dream_project_rows(C.byref(d), x, C.c_int32(R), C.c_int32(hid), w, C.c_int32(H), rb, ri, out, None)
    assert call(x=None) == -1 and call(w=None) == -1 and call(out=None) == -1
    assert call(R=0) == -1 and call(H=0) == -1 and call(R=(1 << 20) + 1) == -1
    assert call(hid=0) == -2 and call(hid=4000) == -2
    assert call(d=dream.attn_desc(1, 32, 32, 72, dream.BF16, 764)) == -2
    assert call(d=dream.attn_desc(1, 32, 32, 128, dream.F32, 764)) == -2
    assert call(ri=fake) == -1                        # a row index needs a row base
    assert call(x=C.c_void_p(0x1008)) == -1 and "aligned" in dream.dream_last_error()

    from paper_2505_19201_amd.binding import ProjJob

    def multi(n=1, job=None):
        arr = (ProjJob * 5)(*[job or ProjJob(0x1000, 0x2000, 8, None, None, 0x3000)] * 5)
        return lib.dream_project_rows_multi(C.byref(desc), arr, C.c_int32(n), C.c_int32(10), C.c_int32(4096), None)
    assert multi(0) == -1 and multi(5) == -1
    assert multi(2, ProjJob(0x1000, None, 8, None, None, 0x3000)) == -1
    assert multi(1, ProjJob(0x1000, 0x2000, 0, None, None, 0x3000)) == -1
    assert lib.dream_project_rows_multi(C.byref(desc), None, C.c_int32(1), C.c_int32(10), C.c_int32(4096), None) == -1


def test_header_compiles_as_c_and_host_calls_work(lib, tmp_path):
    """include/dream.h is a C header: a C99 program built against it with gcc calls the host-only entry points."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(dream.library_path())
    exe = str(tmp_path / "abi_check")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                    os.path.join(root, "tests", "c", "abi_check.c"), "-o", exe, "-L", libdir, "-ldream", "-Wl,-rpath," + libdir],
                   check=True, capture_output=True, text=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    assert out.startswith("attn_wave_kernel<128,8,2,1>")


def test_every_plan_names_a_built_variant(lib):
    """Host-only sweep of shapes (batch, heads, grouping, head_dim, rows, key range): whatever the launch plan chooses,
    the variant exists (dream_attn_plan_describe fails with 'not built' otherwise) and its name is in the variant list."""
    built = set(dream.dream_attn_variants())
    seen = set()
    for D in (64, 128, 256):
        for hkv, g in ((1, 1), (2, 4), (8, 1), (8, 2), (8, 4), (32, 1), (4, 8)):
            for B in (1, 2, 3, 4, 7, 8, 16, 32, 64, 100):
                for n_q in (1, 10, 16, 17, 33, 60, 64, 65, 130, 256):
                    for kv in (n_q, 40, 150, 700, 1340, 2600, 9000):
                        if kv < n_q:
                            continue
                        desc = dream.attn_desc(B, hkv * g, hkv, D, dream.BF16, kv + 3)
                        plan = dream.dream_attn_plan_describe(desc, n_q, kv)
                        name = plan.split(" ")[0]
                        assert name in built, (D, hkv, g, B, n_q, kv, plan)
                        assert dream.dream_tree_verify_attn_workspace(desc, n_q, kv) >= 256
                        seen.add(name)
    assert len(seen) >= 25, sorted(built - seen)   # the sweep reaches most of the table without any override
