/*
 * turbo_serving.h - host-side planning routines of the TurboTransformers paper, C ABI.
 *
 * These two run on the CPU between inferences; all pointers are HOST pointers owned by the caller, nothing is
 * allocated beyond the call, nothing touches the GPU.  Return values are the TURBO_* codes of turbo_reduce.h.
 */
#ifndef TURBO_SERVING_H
#define TURBO_SERVING_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Sequence-length-aware batch scheduler (Section 5, Algorithm 2, Equation 2): split n variable-length requests
 * into batches so that the total inference time is minimal, each batch being zero-padded to its longest request.
 * Requests are sorted by length (stable), and a dynamic program over prefixes of the sorted list chooses where
 * batches end:  states[i] = min_j ( states[j] + cached_cost[len_i][i-j] * (i-j) ),  len_i the longest (= last)
 * request of the batch (j, i].
 *
 *   lengths      [n] sequence lengths, each in 1..max_len.
 *   cached_cost  dense table [(max_len+1) * (max_batch+1)]; entry [len*(max_batch+1) + b] is the cost PER REQUEST
 *                of one inference with b requests padded to length len (the paper's warm-up table).  Entries with
 *                b = 0 or len = 0 are ignored.  Batches larger than max_batch are never formed.
 *   order        [n] out: request indices in scheduling order (sorted by length; ties keep input order).
 *   batch_end    [n] out: batch k consists of order[batch_end[k-1] .. batch_end[k]-1] (batch_end[-1] = 0); the
 *                first *n_batches entries are valid.
 *   total_cost   out: the minimal total cost, sum over batches of cached_cost[longest][size] * size.
 * Among schedules of equal cost the one the algorithm's strict comparison finds first (smaller last batch) wins.
 * Errors: TURBO_ERR_NULL, TURBO_ERR_SHAPE (n <= 0, max_len <= 0, max_batch <= 0, a length outside 1..max_len).
 */
int turbo_batch_schedule(const int *lengths, int n, const double *cached_cost, int max_len, int max_batch, int *order,
                         int *batch_end, int *n_batches, double *total_cost);

/*
 * Cost table from samples (Section 6.3 describes two ways to obtain cached_cost: measure every (length, batch)
 * pair in a warm-up phase, or, when there are too many, measure a sample of them and interpolate; entries may
 * later be overwritten with measured values).  This call is the second way; the paper does not name the
 * interpolation, the reading here is: the samples lie on a grid sample_len x sample_batch (both strictly
 * increasing, values >= 1), the table entry for (len, b) is the bilinear interpolation of the four surrounding
 * samples, and outside the grid the outermost cell's bilinear form is continued (a grid of one line is constant
 * along that axis); results below zero are raised to zero.  At a sample point the entry equals the sample.
 *
 *   sample_cost  [n_len * n_batch], entry [i*n_batch + j] = cost PER REQUEST at (sample_len[i], sample_batch[j]).
 *   cached_cost  out, dense [(max_len+1) * (max_batch+1)] as turbo_batch_schedule reads it; row 0 and column 0
 *                are set to 0.  Overwriting single entries afterwards with measured costs is the caller's business
 *                (the table is the caller's memory).
 * Errors: TURBO_ERR_NULL, TURBO_ERR_SHAPE (empty or non-increasing grids, values < 1, max_len or max_batch <= 0).
 */
int turbo_cost_table_fill(const int *sample_len, int n_len, const int *sample_batch, int n_batch,
                          const double *sample_cost, int max_len, int max_batch, double *cached_cost);

/*
 * Sequence-length-aware allocator (Section 4.2, Algorithm 1): given the life time (first and last operator index
 * in topological order) and the size of every intermediate tensor of one inference, place each tensor at an offset
 * inside a chunk so that tensors whose life times overlap never share bytes, reusing the chunks kept from earlier
 * inferences and appending new ones only when nothing fits.  Tensors are taken in non-increasing order of size
 * (ties: input order); inside a chunk the smallest sufficient gap between life-time-overlapping tensors wins, else
 * the space after the last of them; a new chunk has size max(default_chunk_size, ceil(size * k_scale)).  Chunks
 * that end up unused are released (removed from the list; indices refer to the list after removal).
 *
 *   first_op, last_op, size   [n] per tensor; first_op <= last_op, size > 0 (bytes or any unit).
 *   chunk_sizes               [max_chunks] in/out: sizes of the *n_chunks chunks held on entry; on return the
 *                             chunks in use after this plan.
 *   n_chunks                  in/out.
 *   assigned_chunk, assigned_offset   [n] out, indexed like the input tensors.
 * Errors: TURBO_ERR_NULL, TURBO_ERR_SHAPE (bad sizes or life times, k_scale < 1, more than max_chunks needed).
 */
int turbo_mem_plan(const int *first_op, const int *last_op, const long long *size, int n, long long *chunk_sizes,
                   int *n_chunks, int max_chunks, long long default_chunk_size, double k_scale, int *assigned_chunk,
                   long long *assigned_offset);

#ifdef __cplusplus
}
#endif
#endif /* TURBO_SERVING_H */
