/*
 * cq_bench.h - measurement aids and test switches of libcq.  NOT part of the product ABI
 * (that is cq.h): a deployment ships cq.h only.  The benchmark and the test-suite use these
 * to time reference traffic patterns and to force a kernel family or a row split that the
 * library would not pick by itself.
 *
 * The two switches are THREAD-LOCAL: they change what later calls on the calling thread select
 * and are invisible to every other thread.  Both start at "automatic".
 */
#ifndef CQ_BENCH_H_
#define CQ_BENCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Kernel selection for cq_quantize_kv / cq_decode_attn* on this thread.  AUTO picks the tuned
 * kernels when the shape allows and the shape-agnostic ones otherwise; GENERIC forces the
 * shape-agnostic kernels; TUNED returns CQ_ERR_UNSUPPORTED instead of falling back.
 * Returns the previous value, or CQ_ERR_UNSUPPORTED (-3) for an unknown one. */
enum { CQ_PATH_AUTO = 0, CQ_PATH_GENERIC = 1, CQ_PATH_TUNED = 2 };
int cq_bench_set_kernel_path(int path);

/* Chunks per (batch, KV head) row of the tuned decode on this thread: 0 = the library's own
 * choice (the fewest that fit on chip), n >= 1 = at least n (clamped to what the row allows).
 * cq_decode_workspace_bytes follows the switch.  Returns the previous value, or
 * CQ_ERR_SHAPE (-2) for a negative one. */
int cq_bench_set_decode_chunks(int n_chunks);

/* Enqueue a plain streaming read of `bytes` bytes at `buf` (device, 16-byte aligned).  `sink`
 * is a device float that is practically never written (may be NULL).  The benchmark times it
 * to report the practical read ceiling of the box next to the published HBM peak. */
int cq_bench_stream_read(const void *buf, size_t bytes, void *sink, void *stream);
/* Plain device-to-device copy of `bytes` bytes (both 16-byte aligned): the kernel of known
 * traffic that hardware byte counters are scaled with. */
int cq_bench_stream_copy(void *dst, const void *src, size_t bytes, void *stream);
/* The memory traffic of the tuned quantizer without its arithmetic.  One block per tile of
 * 128 tokens x 128 fp16 values reads the tile's 32 KB of `x_f16` (device, n_tiles * 32 KB,
 * 16-byte aligned) with the quantizer's load pattern and writes `code_bytes_per_tile` (a
 * multiple of 16) to `codes` (device, 16-byte aligned) and `meta_bytes_per_tile` (a multiple of
 * 4) to `meta` (device, 4-byte aligned), both tile after tile.  What is written is
 * meaningless.  CQ_ERR_NULL for null pointers, CQ_ERR_ALIGN for misaligned ones, CQ_ERR_SHAPE
 * for sizes that are not such multiples. */
int cq_bench_tile_traffic(const void *x_f16, void *codes, void *meta, size_t n_tiles,
                          int code_bytes_per_tile, int meta_bytes_per_tile, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CQ_BENCH_H_ */
