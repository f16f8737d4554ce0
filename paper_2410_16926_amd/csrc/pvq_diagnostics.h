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

#ifdef __cplusplus
}
#endif
#endif
