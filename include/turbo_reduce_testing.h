/*
 * turbo_reduce_testing.h - testing, tuning and measurement hooks of the batch-reduction library.
 *
 * None of this is part of the method (the operations are declared in turbo_reduce.h).  The hooks are process-wide
 * switches and probes for the test suite, tuning sweeps and the benchmark: they never change WHAT is computed, only
 * which kernel variant computes it, and they must not be changed while another host thread is inside the library.
 */
#ifndef TURBO_REDUCE_TESTING_H
#define TURBO_REDUCE_TESTING_H

#include "turbo_reduce.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * turbo_set_override(key, value): value < 0 restores the built-in choice.
 *   TURBO_OVR_PATH          force a kernel family of the two reductions: 0 wave (a group of lanes per row),
 *                           1 block (a workgroup per row, LDS combine), 2 stream (a workgroup per row, row
 *                           re-read from memory).  A forced family that cannot hold the row falls back to the
 *                           built-in choice.  For the head permutations and bias+GELU, 2 selects the flat kernel
 *                           (no grouping of rows that share a bias column).
 *   TURBO_OVR_MAX_VEC_BYTES cap the width of one load/store (2..16 bytes); any cap also selects the aligned
 *                           narrow kernels instead of element-aligned 16-byte accesses for odd row lengths
 *   TURBO_OVR_GRID_WAVES    cap on resident workgroups (of 4 wavefronts) per compute unit used to size the grid
 *                           of the looping kernels
 *   TURBO_OVR_GRID_BLOCKS   exact number of workgroups of the kernels that loop over tiles or rows (all softmax
 *                           kernels, the workgroup-per-row and two-sweep LayerNorm), never more than there are tiles or rows
 *   TURBO_OVR_BLOCK_WAVES   wavefronts per row (2..16) of the block family, used when the row then fits the
 *                           registers of that many wavefronts and is accessed with 16-byte vectors; otherwise the
 *                           built-in choice stands
 * Returns TURBO_OK, or TURBO_ERR_SHAPE for an unknown key.
 *
 * turbo_describe_plan(op, rows, row_len, dtype, aligned16, buf, buf_len): writes
 * a short text such as "wave vec=4 lanes=32 nv=1 rows=8" naming the variant the
 * dispatcher would pick for `rows` rows of `row_len` elements (op 0 = softmax,
 * 1 = layernorm).  `buf` is a HOST buffer.  Returns TURBO_OK or an error code.
 *
 * turbo_debug_fastdiv(n, d): the library's multiply-shift division n / d as the
 * kernels compute it (host evaluation; n < 2^31, d >= 1), for host-side tests.
 *
 * turbo_stream_probe(in0, in1, out, n_bytes, stream): measurement aid, not part of
 * the method: the plain stream that the kernels above are compared with.  Treats
 * the DEVICE buffers as n_bytes/4 binary32 values and writes out = in0 + in1, or
 * out = in0 when in1 is NULL, with the same access shape as the element-wise
 * kernels (16-byte non-temporal accesses).  out == in0 with in1 == NULL is the
 * one-read-one-write mix of the in-place softmax; two inputs and a separate
 * output are the two-reads-one-write mix of add-bias-LayerNorm.  Pointers must be
 * 16-byte aligned (TURBO_ERR_ALIGN) and n_bytes a positive multiple of 16
 * (TURBO_ERR_SHAPE); out may equal in0 or in1 exactly, other overlap is undefined.
 * Asynchronous on `stream`; allocates nothing.
 */
enum turbo_override { TURBO_OVR_PATH = 0, TURBO_OVR_MAX_VEC_BYTES = 1, TURBO_OVR_GRID_WAVES = 2, TURBO_OVR_BLOCK_WAVES = 3,
                      TURBO_OVR_GRID_BLOCKS = 4, TURBO_OVR_COUNT_ = 5 };
int turbo_set_override(int key, int value);
int turbo_describe_plan(int op, int rows, int row_len, int dtype, int aligned16, char *buf, int buf_len);
unsigned turbo_debug_fastdiv(unsigned n, unsigned d);
int turbo_stream_probe(const void *in0, const void *in1, void *out, long long n_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TURBO_REDUCE_TESTING_H */
