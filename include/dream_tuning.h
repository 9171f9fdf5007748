/*
 * dream_tuning.h - launch-shape overrides of libdream for experiments and tests.  NOT part of the stable
 * boundary in dream.h: these two switches are process-wide (one atomic integer each), so they are for a
 * single-threaded harness that sweeps launch shapes or wants a test to reach a particular kernel variant.
 * A production caller never needs them: the attention calls choose their launch shape themselves.
 */
#ifndef DREAM_TUNING_H
#define DREAM_TUNING_H

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

#ifdef __cplusplus
}
#endif
#endif /* DREAM_TUNING_H */
