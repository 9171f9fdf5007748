"""Shapes that reach every bf16 attention kernel variant of the launch plan, and the plans of the full-size
configurations.  Host data only: tests/test_abi.py checks (without a GPU) that the list is complete and that
every case really plans the variant it names; tests/test_gpu_attention.py runs each case against the oracle,
all elements."""
from collections import namedtuple

import dream_inputs as di

# kv_len = prefix + n_tree is the longest sequence of the case; shorter ones are mixed in by the GPU test.
# splits / q_tiles / waves are the launch-shape overrides the case needs (0 = automatic).
VariantCase = namedtuple("VariantCase", "variant batch n_q_heads n_kv_heads head_dim n_tree depth kv_len splits q_tiles waves", defaults=(0,))

VARIANT_CASES = [
    VariantCase("attn_bf16_kernel<64,1,2,1>", 1, 2, 2, 64, 17, 4, 150, 0, 0),
    VariantCase("attn_bf16_kernel<64,1,3,1>", 1, 2, 2, 64, 17, 4, 150, 2, 0),
    VariantCase("attn_bf16_kernel<64,1,4,1>", 1, 2, 2, 64, 17, 4, 200, 2, 0),
    VariantCase("attn_bf16_kernel<64,1,2,2>", 1, 4, 2, 64, 60, 6, 150, 1, 1),
    VariantCase("attn_bf16_kernel<128,1,2,1>", 1, 2, 2, 128, 17, 4, 150, 0, 0),
    VariantCase("attn_bf16_kernel<128,1,3,1>", 1, 2, 2, 128, 17, 4, 150, 2, 0),
    VariantCase("attn_bf16_kernel<128,1,4,1>", 1, 2, 2, 128, 17, 4, 200, 2, 0),
    VariantCase("attn_bf16_kernel<128,1,1,2>", 1, 4, 2, 128, 60, 6, 150, 1, 1),
    VariantCase("attn_bf16_kernel<256,1,1,2>", 1, 4, 2, 256, 60, 6, 150, 0, 1),
    # the same three with one query group per KV head: K/V loads with the nontemporal hint (waves = 4: not the two-key-group form)
    VariantCase("attn_bf16_kernel<64,1,2,2,4,1,1>", 1, 2, 2, 64, 17, 4, 150, 1, 0, 4),
    VariantCase("attn_bf16_kernel<128,1,1,2,4,1,1>", 1, 2, 2, 128, 17, 4, 150, 1, 0, 4),
    VariantCase("attn_bf16_kernel<256,1,1,2,4,1,1>", 1, 2, 2, 256, 17, 4, 150, 0, 0),
    VariantCase("attn_bf16_kernel<64,2,1,2>", 1, 2, 2, 64, 60, 6, 150, 0, 2),
    VariantCase("attn_bf16_kernel<64,4,1,2>", 2, 8, 2, 64, 60, 6, 150, 0, 4),
    VariantCase("attn_bf16_kernel<128,2,1,2>", 1, 2, 2, 128, 60, 6, 150, 0, 2),
    VariantCase("attn_bf16_kernel<128,4,1,1>", 2, 8, 2, 128, 60, 6, 150, 0, 4),
    VariantCase("attn_bf16_kernel<256,2,1,1>", 1, 4, 2, 256, 60, 6, 150, 0, 2),
    # 8 waves as two key groups (multi-head shapes with few streams per CU)
    VariantCase("attn_bf16_kernel<64,1,2,2,8,1,1,2>", 2, 4, 4, 64, 60, 6, 333, 1, 0, 8),
    VariantCase("attn_bf16_kernel<128,1,1,2,8,1,1,2>", 2, 4, 4, 128, 60, 6, 333, 1, 0, 8),
    # 8 waves per workgroup: 8 query tiles of a KV head (one per wave), 16 (two per wave), head_dim 256
    VariantCase("attn_bf16_kernel<128,1,1,2,8>", 2, 4, 2, 128, 60, 6, 150, 0, 0, 8),
    VariantCase("attn_bf16_kernel<128,2,1,2,8>", 2, 8, 2, 128, 60, 6, 150, 0, 0, 8),
    VariantCase("attn_bf16_kernel<256,1,1,2,8>", 2, 4, 2, 256, 60, 6, 150, 0, 0, 8),
    # trees of 65-256 nodes (four mask words per node): 100, 200 and 256 nodes
    VariantCase("attn_bf16_kernel<64,1,2,2,4,4>", 2, 4, 4, 64, 100, 7, 333, 0, 0),
    VariantCase("attn_bf16_kernel<128,1,1,2,4,4>", 2, 4, 2, 128, 200, 9, 410, 0, 0),
    VariantCase("attn_bf16_kernel<256,1,1,2,4,4>", 1, 4, 2, 256, 256, 12, 300, 0, 0),
    VariantCase("attn_wave_kernel<64,8,1,1>", 3, 24, 8, 64, 17, 4, 1340, 0, 0),
    VariantCase("attn_wave_kernel<64,8,2,1>", 8, 2, 2, 64, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<64,4,1,1>", 3, 24, 8, 64, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<64,8,1,2>", 6, 24, 8, 64, 17, 4, 1340, 0, 0),
    VariantCase("attn_wave_kernel<64,4,1,2>", 6, 24, 8, 64, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<128,8,1,1>", 3, 24, 8, 128, 17, 4, 1340, 0, 0),
    VariantCase("attn_wave_kernel<128,8,2,1>", 3, 12, 4, 128, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<128,8,4,1>", 8, 2, 2, 128, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<128,4,1,1>", 3, 24, 8, 128, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<128,8,1,2>", 6, 24, 8, 128, 17, 4, 1340, 0, 0),
    VariantCase("attn_wave_kernel<128,4,1,2>", 6, 24, 8, 128, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<256,4,1,1>", 3, 24, 8, 256, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<256,4,2,1>", 3, 12, 4, 256, 17, 4, 150, 0, 0),
    VariantCase("attn_wave_kernel<256,4,4,1>", 8, 2, 2, 256, 17, 4, 150, 0, 0),
]

# The launch the benchmark times: dream_tree_verify_attn at each full-size configuration.
FULL_VERIFY_PLANS = {
    "llava": "attn_wave_kernel<128,8,2,1> workgroups=256 splits=1 merge_launch=0",
    "pixtral": "attn_wave_kernel<128,8,2,1> workgroups=256 splits=1 merge_launch=0",
    "gemma3": "attn_wave_kernel<256,4,4,1> workgroups=256 splits=1 merge_launch=0",
    "smolvlm_b1": "attn_wave_kernel<64,8,2,1> workgroups=256 splits=1 merge_launch=0",
    "smolvlm_b8": "attn_bf16_kernel<64,1,2,2,8,1,1,2> workgroups=256 splits=1 merge_launch=0",
    "smolvlm_b32": "attn_bf16_kernel<64,1,2,2,4,1,1> workgroups=1024 splits=1 merge_launch=0",
}

# 8-wave shapes beyond the one-case-per-variant list: idle waves (6 query tiles), idle tile slots (12 query tiles, two
# per wave), and a long ragged key range
EXTRA_W8_CASES = [
    # two key groups: idle query-tile waves, sequences whose key range is shorter than one step, an odd number of tiles
    VariantCase("attn_bf16_kernel<64,1,2,2,8,1,1,2>", 3, 2, 2, 64, 17, 4, 170, 1, 0, 8),
    VariantCase("attn_bf16_kernel<128,1,1,2,8,1,1,2>", 2, 2, 2, 128, 33, 5, 225, 1, 0, 8),
    VariantCase("attn_bf16_kernel<128,1,1,2,8>", 2, 6, 2, 128, 17, 4, 700, 0, 0, 8),
    VariantCase("attn_bf16_kernel<128,2,1,2,8>", 1, 6, 2, 128, 60, 6, 333, 0, 0, 8),
    VariantCase("attn_bf16_kernel<256,1,1,2,8>", 3, 4, 2, 256, 33, 5, 410, 0, 0, 8),
]

# The 32-sequence launches bench.py times as the streaming regime of the grouped-query configurations
STREAMING_PLANS = {
    "llava": "attn_bf16_kernel<128,1,1,2,4,1,1> workgroups=1024 splits=1 merge_launch=0",
    "pixtral": "attn_bf16_kernel<128,2,1,2,8> workgroups=256 splits=1 merge_launch=0",
    "gemma3": "attn_bf16_kernel<256,1,1,2,8> workgroups=256 splits=1 merge_launch=0",
}

# dream_draft_xattn at each full-size configuration: (plan of the root call, plan of a 10-row level call)
FULL_XATTN_PLANS = {
    "llava": ("attn_wave_kernel<128,8,4,1> workgroups=128 splits=1 merge_launch=0",) * 2,
    "pixtral": ("attn_wave_kernel<128,8,4,1> workgroups=128 splits=1 merge_launch=0",) * 2,
    "gemma3": ("attn_bf16_kernel<256,1,1,2,4,1,1> workgroups=64 splits=8 merge_launch=1",) * 2,
    "smolvlm_b1": ("attn_wave_kernel<64,8,2,1> workgroups=64 splits=1 merge_launch=0",) * 2,
    "smolvlm_b8": ("attn_wave_kernel<64,8,1,1> workgroups=256 splits=1 merge_launch=0",) * 2,
    "smolvlm_b32": ("attn_bf16_kernel<64,1,2,2,4,1,1> workgroups=1024 splits=1 merge_launch=0",) * 2,
}


def variant_config(case: VariantCase) -> di.Config:
    prefix = case.kv_len - case.n_tree
    n_visual = (prefix * 3) // 4
    return di.Config("variant", "bf16", case.batch, case.n_q_heads, case.n_kv_heads, case.head_dim,
                     case.n_q_heads * case.head_dim, n_visual, prefix - n_visual, case.n_tree, case.depth, 1, 4, 1000, 1, 47)


def variant_prefix_lens(case: VariantCase):
    """Ragged lengths: the first sequence has the full prefix (it fixes the plan), the others are shorter."""
    prefix = case.kv_len - case.n_tree
    return [prefix - (b * 37) % max(prefix // 2, 1) for b in range(case.batch)]
