"""GPU: the whole path captured in one HIP graph gives, on every replay, exactly what the eager calls give.

The library enqueues kernels only (no memset nodes, no allocation, no synchronisation), so a captured step must be
bit-identical to the eager step however often it is replayed and whatever runs between the replays; the inputs
are rewritten between replays so that a replay cannot pass by leaving old results in place."""
import numpy as np
import pytest

import dream_inputs as di

pytestmark = pytest.mark.gpu


def test_captured_step_matches_eager_on_every_replay():
    import torch
    import paper_2505_19201_amd as dream
    assert torch.cuda.is_available(), "this test needs the MI355X"
    cfg = di.Config("graph", "bf16", 2, 8, 4, 128, 512, 96, 40, 60, 6, 1, 4, 4096, 1, 55)
    B, T, Hq, Hkv, D, P, V = cfg.batch, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.prefix, cfg.vocab
    S = P + T
    x = di.verify_inputs(cfg)
    s_max = x.s_max
    dev = torch.device("cuda")
    q, k, v = (dream.to_device(a, "bf16") for a in (x.q, x.k, x.v))
    prefix_len, parent = dream.to_device(x.prefix_len), dream.to_device(x.parent)
    desc = dream.attn_desc(B, Hq, Hkv, D, dream.BF16, s_max)
    out = torch.empty(B, T, Hq, D, dtype=torch.bfloat16, device=dev)
    lse = torch.empty(B, Hq, T, dtype=torch.float32, device=dev)
    ws_v = dream.alloc_workspace(dream.dream_tree_verify_attn_workspace(desc, T, S))
    pq = dream.to_device(di.prefill_q(cfg), "bf16")
    feats = dream.to_device(di.feature_rows(cfg), "bf16")
    n_keep = (cfg.n_visual * cfg.keep_num + cfg.keep_den // 2) // cfg.keep_den
    scores = torch.empty(B, cfg.n_visual, dtype=torch.float32, device=dev)
    kept = torch.empty(B, n_keep, dtype=torch.int32, device=dev)
    gathered = torch.empty(B, n_keep, cfg.hidden, dtype=torch.bfloat16, device=dev)
    ws_c = dream.alloc_workspace(dream.dream_visual_compress_workspace(desc, P, cfg.n_visual))
    lg_np, tok_np, _, _ = di.accept_inputs(cfg)
    logits, token = dream.to_device(lg_np, "bf16"), dream.to_device(tok_np)
    dlogits = (logits.float() + 0.5 * torch.randn(B, T, V, device=dev)).to(torch.bfloat16)
    ua, ub = torch.rand(B, T, device=dev), torch.rand(B, device=dev)
    am = torch.empty(B, T, dtype=torch.int32, device=dev)
    alen, bonus = torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev)
    path = torch.empty(B, cfg.depth + 1, dtype=torch.int32, device=dev)
    alen2, bonus2, path2 = torch.empty_like(alen), torch.empty_like(bonus), torch.empty_like(path)
    ws_a = dream.alloc_workspace(dream.dream_accept_path_workspace(B, T, V))
    ws_s = dream.alloc_workspace(dream.dream_spec_accept_workspace(B, T, V))
    ent_row = torch.empty(B, Hq, P, dtype=torch.float32, device=dev)
    ae = torch.empty(B, dtype=torch.float32, device=dev)
    ws_e = dream.alloc_workspace(dream.dream_attention_entropy_workspace(desc, P))
    wk = (torch.randn(Hkv * D, cfg.hidden, device=dev) * cfg.hidden ** -0.5).to(torch.bfloat16)
    new_len = torch.empty_like(prefix_len)
    tree_feats = feats[:, :T].contiguous()
    k2 = k.clone()

    def step():
        dream.dream_tree_verify_attn(desc, q, k, v, prefix_len, T, parent, None, S, out, lse, ws_v)
        dream.dream_visual_compress(desc, pq, None, P, k, P, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den, None, scores, kept,
                                    feats, P, gathered, cfg.hidden, ws_c)
        dream.dream_attention_entropy(desc, pq, None, P, k, P, ent_row, ae, ws_e)
        dream.dream_accept_path(logits, dream.BF16, B, T, V, token, parent, cfg.depth, am, alen, path, bonus, ws_a)
        dream.dream_spec_accept(logits, dlogits, dream.BF16, B, T, V, token, parent, ua, ub, cfg.depth, 1.0, alen2, path2, bonus2, ws_s)
        dream.dream_project_rows(desc, tree_feats, T, cfg.hidden, wk, Hkv, prefix_len, None, k2)      # append T rows after the prefix
        dream.dream_kv_commit(desc, [k2], prefix_len, T, path, alen, new_len)

    outputs = (out, lse, scores, kept, gathered, ent_row, ae, am, alen, path, bonus, alen2, path2, bonus2, k2, new_len)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in outputs]

    def scramble(seed):
        """New inputs where that keeps the shapes valid, garbage in every output."""
        g = torch.Generator(device=dev)
        g.manual_seed(seed)
        q.copy_(torch.randn(q.shape, device=dev, generator=g).to(torch.bfloat16))
        ua.copy_(torch.rand(ua.shape, device=dev, generator=g))
        ub.copy_(torch.rand(ub.shape, device=dev, generator=g))
        k2.copy_(k)
        for t in outputs:
            if t is not k2:
                t.fill_(-3)

    scramble(1)
    step()
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    scramble(1)
    with torch.cuda.graph(graph, stream=stream):
        step()
    for seed in (1, 2, 3, 4):
        scramble(seed)
        step()
        want = snapshot()
        scramble(seed)
        (torch.randn(1 << 20, device=dev) * 2).sum().item()      # unrelated eager work and a synchronisation in between
        graph.replay()
        got = snapshot()
        for i, (g_, w_) in enumerate(zip(got, want)):
            assert torch.equal(g_.view(torch.uint8) if g_.dtype != torch.bfloat16 else g_.view(torch.int16),
                               w_.view(torch.uint8) if w_.dtype != torch.bfloat16 else w_.view(torch.int16)), (seed, i)
    assert int(alen.min()) >= 0 and bool((new_len == prefix_len + alen + 1).all())
