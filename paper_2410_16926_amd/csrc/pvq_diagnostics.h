/* Host-only diagnostics of libpvq.  Not part of the public interface (include/pvq.h): the symbols are
 * exported so that the tests can call them through ctypes. */
#ifndef PVQ_DIAGNOSTICS_H
#define PVQ_DIAGNOSTICS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The table-driven decoder that the kernels use for D = 8 when N(8,K) fits a 32-bit word and the tables
 * fit LDS: rebuilds those tables and replays the kernels' table walk on the host for the indices
 * [first, first + count) (clipped to N(8,K)), comparing every decoded point with the
 * coordinate-by-coordinate walk of App. B.3.  *mismatches (host) receives the number of indices that
 * differ (0 when the tables are right).  PVQ_E_UNSUPPORTED if (8,K) has no such tables.
 */
int pvq_fast_tables_selftest(int K, uint64_t first, uint64_t count, uint64_t *mismatches);

/*
 * The coordinate-by-coordinate decoder with one table probe per coordinate (groups of 16 and 32, multi-word
 * indices): builds its tables for (D, K) and replays the kernels' walk on the host for `count` indices (the
 * first and last index, two in the middle, then seeded random ones, a third of them near the start of the
 * range), comparing every decoded point with the magnitude-by-magnitude walk of App. B.3.  *mismatches (host)
 * receives the number that differ; schedule (host, 2 ints, may be NULL) the width schedule chosen (the
 * dimensions from which on half- and quarter-width integers are used, 0 = none), *table_bytes (may be NULL)
 * the size of the tables.  PVQ_E_UNSUPPORTED for D outside {8, 16, 32} or indices beyond 128 bits.
 */
int pvq_walk_tables_selftest(int D, int K, uint64_t seed, uint64_t count, uint64_t *mismatches, int *schedule,
                             uint32_t *table_bytes);

/*
 * Which kernels pvq_decode_gemv would launch for a rows x cols matrix of this context and `batch` vectors,
 * without launching anything: kinds[i] and nvecs[i] (host arrays of max_passes entries) receive the kind of
 * pass i (0 generic coordinate-by-coordinate kernel, 1 table-driven vector-ALU kernel, 2 the same with whole
 * rows per wave, 3 the 16-vector vector-ALU kernel, 4 the matrix-core kernel) and the number of vectors it
 * takes; *passes the number of passes.  For reports (a benchmark line that says which path a batch size
 * took).  PVQ_E_INVALID_ARG for NULL pointers, a batch outside 1..16 or max_passes < the passes needed.
 */
struct pvq_ctx;
int pvq_decode_gemv_plan(const struct pvq_ctx *ctx, int64_t rows, int64_t cols, int batch, int *kinds, int *nvecs,
                         int max_passes, int *passes);

/*
 * pvq_correct chooses per launch who applies the panel before's update to the panel's own columns: a launch of
 * its own, or, from *tiles* update tiles in the launch on, the panel's workgroups themselves (default 1536, which
 * small test matrices never reach).  Sets that number for the process and returns the one in force before in
 * *previous (may be NULL); results do not depend on it.  PVQ_E_INVALID_ARG for tiles < 0.
 */
int pvq_correct_set_front_tiles(int64_t tiles, int64_t *previous);

/*
 * pvq_decode for groups of 8 with 24-bit indices has two decoders: the table decoder, whose tables take most of a
 * unit's LDS and some microseconds to copy there, and the coordinate-by-coordinate one, which starts at once and
 * takes longer per group.  Matrices of fewer than *groups* groups (rows x cols / 8; default 1 572 864) go to the
 * second.  Sets that number for the process and returns the one in force before in *previous (may be NULL).  Both
 * decoders give the same pulses; their float32 gains can differ in the last place (one divides the amplitude by
 * sqrt(sum y^2), the other multiplies by a tabulated reciprocal).  PVQ_E_INVALID_ARG for groups < 0.
 */
int pvq_decode_set_table_decoder_min_groups(int64_t groups, int64_t *previous);

#ifdef __cplusplus
}
#endif
#endif
