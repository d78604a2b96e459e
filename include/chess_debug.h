/*
 * Test hooks of libchess: ways to force launch shapes and code paths that the library otherwise chooses by
 * itself, so that tests can reach every one of them.  Not part of the product interface (include/chess.h).
 */
#ifndef CHESS_DEBUG_H
#define CHESS_DEBUG_H

#include "chess.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test hook: force the number of workgroups that cooperate on one (sequence, KV head) in
 * chess_select and chess_decode_step (1..32, capped by what can be resident at once); 0 restores the automatic choice. */
int chess_debug_force_cluster(chess_ctx* ctx, int32_t cluster);

/* Test hook: the schedule of the selection levels in chess_select and chess_decode_step: 1 = lazy (grids, chunks
 * of kept grids, pages of kept chunks: three memory phases), 2 = merged (all chunks scored together with the grids:
 * two phases); 0 restores the automatic choice.  The selected pages are the same either way. */
int chess_debug_force_schedule(chess_ctx* ctx, int32_t schedule);

/* Test hook: on = 1 makes every level of chess_select find its cut by the general path (radix select
 * on the keys in LDS) that otherwise only serves tied or very large levels; 0 restores the automatic
 * choice.  The selected pages are the same either way. */
int chess_debug_force_general_cut(chess_ctx* ctx, int32_t on);

/* Test hook: the number of polls after which a workgroup of chess_select / chess_decode_step gives up waiting for
 * the keys of the other members of its cluster (0 restores the default, 32768, about 30 ms).  With a negative value
 * every such wait is given up before its first poll, on purpose: every workgroup still leaves normally, the
 * workspace's error flag is raised, the results are undefined and the workspace must be re-initialised. */
int chess_debug_set_poll_limit(chess_ctx* ctx, int32_t polls);

/* Test hook: force the split-K shape of the decode entry points (n_splits in [1, 256] with n_splits * G <= 1024,
 * waves in {1, 4}); n_splits = 0 restores the automatic choice.  CHESS_EINVAL if the forced shape would
 * not fit the workspace for max_batch sequences. */
int chess_debug_force_splits(chess_ctx* ctx, int32_t n_splits, int32_t waves);

#ifdef __cplusplus
}
#endif
#endif /* CHESS_DEBUG_H */
