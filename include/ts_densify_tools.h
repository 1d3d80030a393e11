/*
 * ts_densify_tools -- calls for tests, benchmarks and tuning.  None of them is needed to use
 * the library (ts_densify.h); they are kept apart because they synchronise, or read back the
 * library's working arrays, or change process-wide settings that every later call sees.
 *
 * The settings are plain process-wide variables: set them while no call is in flight.
 * ts_set_piece_tokens changes the order in which a row's pairs are added and therefore the
 * bits of later results (each setting is still deterministic); the other settings change
 * only how the work is spread over the launches, never a result.
 */
#ifndef TS_DENSIFY_TOOLS_H
#define TS_DENSIFY_TOOLS_H

#include "ts_densify.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * What ts_last_views points at, copied to host arrays: waits for `stream`, then copies
 * count [V] and row_start [V + 1] (int32), the first n_valid sorted records
 * (TS_SORTED_PAIR_BYTES each) and the two scalars.  Any out-pointer may be NULL.  V is that
 * of the most recent call (the number of rows of the range for ts_densify_range), which the
 * library knows and the caller states: count_out holds rows_capacity int32 and row_start_out
 * rows_capacity + 1; TS_ERR_CAPACITY, with nothing written, if the last call's V exceeds
 * rows_capacity, and likewise if n_valid exceeds sorted_capacity records.  This call
 * synchronises.
 */
int ts_read_views(int32_t* count_out, int32_t* row_start_out, int64_t rows_capacity, void* sorted_out,
                  int64_t sorted_capacity, int32_t* n_valid_out, int32_t* n_bad_ids_out, void* stream);

/*
 * Host arithmetic: the bytes of workspace that a call of exactly this shape uses (n_total pairs
 * of row_dtype, d columns, V rows), under the current tuning settings.  ts_workspace_bytes(n, d, V)
 * is an upper bound of it for every shape with at most n pairs, d columns and V rows.
 */
int ts_call_workspace_bytes(int64_t n_total, int32_t row_dtype, int32_t d, int32_t V, int64_t* bytes);

/*
 * How the most recent call was split over its launches, for byte accounting in
 * benchmarks.  Writes 8 int32 to info (host): [0] piece_tokens C; [1] X: dense rows
 * [0, X) were copied beside the sort launches; [2] T = V: untouched rows in [X, T) were
 * copied by the row-reduce kernel; [3] sort slices; [4] ids per sort work-group;
 * [5] pieces; [6] levels of the tree in which the shares of a cut row are added up;
 * [7] bit 0: the call was in place; bits 1-2: how rows with at most C pairs were added up
 * (0 in the pieces, 1 row by row with the long rows by lone wavefronts, 2 row by row with the
 * long rows by work-groups).
 */
int ts_last_launch_info(int32_t* info);

/*
 * Per-kernel timing for benchmarks.  ts_profile_begin(capacity) makes each of the
 * next `capacity` densify calls stamp a HIP event pair with the begin and the end of
 * its row-reduce kernel (the launch variant that takes events) on the caller's stream; ts_profile_end waits for those events and writes
 * up to `capacity` durations in milliseconds to ms_out (host) and how many to
 * *n_out (host), then stops recording.  capacity <= 4096.
 */
int ts_profile_begin(int32_t capacity);
int ts_profile_end(float* ms_out, int32_t capacity, int32_t* n_out);

/*
 * Tuning.  piece_tokens: sorted positions handled by one wavefront item of the
 * row-reduce kernel (8, 16 or 32; 0 = choose from n and the row type).  Changes the fixed
 * summation order (still deterministic) and the workspace size.
 */
int ts_set_piece_tokens(int32_t piece_tokens);

/*
 * Tuning.  The sort launches are latency-bound, so work-groups that copy dense rows run
 * beside them to keep HBM busy.  sort_bytes: dense bytes (read + write) copied from dense_in
 * to dense_out beside each sort launch, before it is known which rows receive pairs (those
 * are overwritten afterwards).  -1 = default, 0 = none.  Results do not depend on it.
 */
int ts_set_overlap_bytes(int64_t sort_bytes);

/*
 * Tuning.  Output rows with at most piece_tokens pairs are added up either by the pieces
 * that hold their pairs (mode 0) or row by row, by the wavefront that would otherwise copy
 * the row (mode 1).  -1 = choose from the number of pairs, the rows' width and type and the size
 * of the dense operand.  Results do not depend on it.
 */
int ts_set_short_rows(int32_t mode);

/* Tuning.  Ids owned by one sort work-group (64 .. 2048, power of two; 0 = choose from V and n). */
int ts_set_sort_part(int32_t part);

#ifdef __cplusplus
}
#endif
#endif /* TS_DENSIFY_TOOLS_H */
