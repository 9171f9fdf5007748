/*
 * dream_tuning.h - launch-shape overrides of libdream for experiments and tests.  NOT part of the stable
 * boundary in dream.h: these switches are process-wide (one atomic integer each), so they are for a
 * single-threaded harness that sweeps launch shapes or wants a test to reach a particular kernel variant.
 * A production caller never needs them: the attention calls choose their launch shape themselves.
 */
#ifndef DREAM_TUNING_H
#define DREAM_TUNING_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* 0 = choose automatically (the default).  dream_set_kv_splits: number of key-range splits the attention
 * calls use (1 = never split; any value also switches the single-launch wave kernel off).
 * dream_set_q_tiles: 16-row query tiles one wave serves in the shared-tile kernel (1, 2 or 4).
 * Results are identical up to floating-point summation order.  The workspace size depends on both: query
 * it again after changing either, and change neither while another thread is inside an attention call. */
void dream_set_kv_splits(int32_t n_splits);
void dream_set_q_tiles(int32_t q_tiles);
/* Waves per workgroup of the shared-tile kernel: 4 = never the 8-wave form, 8 = the 8-wave form wherever it exists
 * (bf16, head_dim >= 128, unsplit key range), 0 = automatic. */
void dream_set_tile_waves(int32_t waves);

/* Host-only: the names of all bf16 attention kernel variants the launch plan can choose, separated by ';', in the
 * spelling dream_attn_plan_describe uses ("attn_wave_kernel<128,8,2,1>": head_dim, waves, column slices, query tiles
 * per workgroup; "attn_bf16_kernel<128,1,1,2>": head_dim, query tiles per wave, key tiles per step, steps in flight;
 * a fifth argument 8 marks the form with 8 waves per workgroup).
 * The tests use it to make sure every variant has a parity case.  0, or -1 if buf is too small. */
int dream_attn_variants(char *buf, size_t buf_bytes);

#ifdef __cplusplus
}
#endif
#endif /* DREAM_TUNING_H */
