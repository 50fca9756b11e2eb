/*
 * inferturbo_aids.h -- measurement aids of libinferturbo_hip.  Not part of the
 * method and not needed to use the library: the benchmark and the profiles
 * use them to calibrate hardware counters, to measure what the memory system
 * delivers for a gather's access pattern, and to switch between kernel
 * variants for A/B timings.  Conventions as in inferturbo.h (device pointers
 * unless marked host, status codes, `stream` = hipStream_t as void*).
 */
#ifndef INFERTURBO_AIDS_H
#define INFERTURBO_AIDS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Plain device copy of n_bytes (multiple of 16) with one 16-byte load and
 * store per lane: the known-size kernel that hardware byte counters are
 * scaled against, and the streaming rate of this machine. */
int32_t itb_copy_bytes(const void *src, void *dst, int64_t n_bytes, void *stream);

/* Random-row read probe: for every i < n_idx the row idx[i] of `table`
 * ([n_rows x row_bytes], row_bytes in {16, 32, ..., 1024}, 16-byte aligned) is
 * read once, 16 bytes per lane, with the index stream read sequentially --
 * the memory traffic of a gather (Sec. IV-B gather_nbrs over a CSR row) with
 * no arithmetic and every SIMD full.  Its rate is the practical ceiling for
 * a gather of rows of that size over a table of that size on this machine.
 * idx entries must lie in [0, n_rows) (trusted); `sink` receives one word per
 * launched thread (2048 blocks x 256 threads x 4 bytes, sink_bytes is checked). */
int32_t itb_random_row_read(const void *table, int64_t n_rows, int32_t row_bytes, const int32_t *idx, int64_t n_idx,
                            void *sink, int64_t sink_bytes, void *stream);

/* Process-wide switches for A/B measurements.  key 0 = in-degree up to which
 * gather processes one row per lane group instead of per wavefront (-1 =
 * built-in choice); 2 = XCD-contiguous tile order in the radix passes (1 =
 * on); 3 = in-degree above which a non-hub row gets a whole block (512); 4 =
 * resident wavefronts per SIMD of the row gather (-1 = built-in choice); 5 =
 * out-degrees from a keys-only sort instead of partition + bucket counts; 6 =
 * helper-stream overlap (hub passes of a gather, out-degree branch of the CSR
 * build; 1 = on); 7 = row loads in flight per lane of the gather loops (-1 =
 * built-in choice); 8 = loads of the randomly addressed source rows: 0 plain,
 * 1 non-temporal, -1 by table size (non-temporal from 3 GiB on: measured 10 %
 * faster on a 12.8 GB table, 5-10 % slower on tables of 1 GB and less; the
 * probe itb_random_row_read follows the same switch); 9 = the update of a
 * layer feeds the projection of a following narrowing layer in the same
 * launch (1 = on); 10 = attention scores of a projection taken in its
 * epilogue instead of by an extra score tile (1 = where the head width allows
 * it and d_in >= 256, 2 = wherever the head width allows it, 0 = never). */
int32_t itb_set_tuning(int32_t key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* INFERTURBO_AIDS_H */
