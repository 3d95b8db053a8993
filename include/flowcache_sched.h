/*
 * flowcache_sched.h -- host-side tick scheduler for chunk-autoregressive denoising with a
 * budgeted clean KV cache.  No GPU work, no allocation: the caller provides the state block.
 *
 * It produces, tick by tick, what the device calls of flowcache.h need: which units (video
 * chunks, or blocks inside a chunk) are being denoised, how many steps each has taken, where
 * their K/V slots are in the per-head cache, how long the clean region is, and when a unit
 * finishes and has to be committed to the clean region (appended while the cache is filling,
 * merged and compressed back to the budget afterwards).
 *
 * Schedule (Sec. 3.1, Eq. (3) and the sliding window of Sec. 4.1): unit i starts at tick
 * i*stagger and takes `steps` ticks; with a window of l units and stagger = steps/l this is
 * the range t in [(i-1)T/l, (i+l-1)T/l] of Eq. (3) (units counted from 1 there).  The
 * hierarchical variant of Sec. 4.1 (blocks inside a chunk, each block starting a fixed number
 * of steps after the previous one) is the same schedule with stagger = that number of steps;
 * consecutive chunks are separate schedules whose `prefix_tokens` are the overlap frames.
 *
 * Cache layout per head (token positions):
 *   [0, budget + L_c)                         clean region (only its first L_clean rows valid)
 *   [budget + L_c + s*L_c, ... + L_c)         slot s of the active ring, s = unit % window
 * Cache phases (App. C.1): while L_clean + L_c <= budget a finished unit is appended;
 * afterwards [clean | finished unit] is compressed to `budget` rows.
 */
#ifndef FLOWCACHE_SCHED_H
#define FLOWCACHE_SCHED_H

#include <stddef.h>
#include <stdint.h>

#include "flowcache.h"

#ifdef __cplusplus
extern "C" {
#endif

#define FC_SCHED_DONE 5 /* flowcache_sched_next: the schedule is complete, *out untouched */

typedef struct {
    int32_t n_units;       /* units to generate, >= 1                                          */
    int32_t steps;         /* denoising steps per unit (T), >= 1                               */
    int32_t stagger;       /* ticks between the starts of consecutive units, in [1, steps]     */
    int32_t window;        /* active-ring slots; 0 = ceil(steps / stagger); must cover it and  */
                           /* be <= FC_MAX_ACTIVE                                              */
    int32_t L_c;           /* tokens per unit                                                  */
    int32_t budget;        /* clean-cache budget in tokens, >= 0 (0: nothing is kept)          */
    int32_t prefix_tokens; /* clean tokens present before the first tick, <= budget            */
} fc_sched_config;

typedef struct {
    int32_t tick;                      /* 0-based                                              */
    int32_t A;                         /* active units this tick, causal order (oldest first)  */
    int32_t unit[FC_MAX_ACTIVE];       /* their indices                                        */
    int32_t step_idx[FC_MAX_ACTIVE];   /* steps each has already taken (0 = just initialised)  */
    int32_t active_off[FC_MAX_ACTIVE]; /* first cache position of each unit's slot             */
    int32_t L_clean;                   /* clean rows visible to attention during this tick     */
    int32_t commit_unit;               /* unit taking its last step this tick, else -1         */
    int32_t commit_src_off;            /* its slot: rows to move to the clean region ...       */
    int32_t commit_dst_off;            /* ... starting here (= L_clean)                        */
    int32_t merged_len;                /* L_clean + L_c: length of the set to compress         */
    int32_t compress;                  /* 1: compress [0, merged_len) to budget; 0: append     */
    int32_t L_clean_after;             /* clean rows after the commit (next tick's L_clean)    */
} fc_tick;

/* Bytes of caller-provided state (host memory, any alignment of 8). */
size_t flowcache_sched_state_bytes(void);

/* Validates cfg and initialises the state.  FC_INVALID_ARGUMENT for null pointers, a state
 * block that is too small, or a configuration outside the ranges stated above. */
int flowcache_sched_init(void* state, size_t state_bytes, const fc_sched_config* cfg);

/* Token positions per head the caches must hold: budget + L_c + window*L_c (0 on bad state). */
int64_t flowcache_sched_capacity(const void* state);

/* Number of ticks of the whole schedule: (n_units - 1)*stagger + steps (0 on bad state). */
int64_t flowcache_sched_total_ticks(const void* state);

/* Writes the next tick and advances.  FC_OK, FC_SCHED_DONE after the last tick, or
 * FC_INVALID_ARGUMENT for null / uninitialised state. */
int flowcache_sched_next(void* state, fc_tick* out);

#ifdef __cplusplus
}
#endif
#endif /* FLOWCACHE_SCHED_H */
