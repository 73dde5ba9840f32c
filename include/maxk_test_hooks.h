/*
 * libmaxk -- host-side introspection for the library's own tests.  Not part of the API: these symbols may change
 * or disappear between versions, and no caller needs them to use the path.
 */
#ifndef MAXK_TEST_HOOKS_H
#define MAXK_TEST_HOOKS_H

#include "maxk.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The number of private output-row copies the forward kernel (Alg. 1's on-chip output row) keeps in LDS for
 * MaxK k: entries that share one 64-lane instruction must map to different copies.  Negative maxk_status for k < 1. */
MAXK_API int32_t maxk_fwd_private_copies(int32_t k);

/* How many regroupings of A^T the handle holds: slab tables (one per slab height ever needed) and visit lists of the
 * LDS-tiled backward kernel (one per destination-set size and k / 4).  They are built once and kept, so the counts
 * never go down and a repeated shape never adds one.  Either out pointer may be NULL. */
MAXK_API maxk_status maxk_graph_cached_tables(const maxk_graph* g, int32_t* n_slab_tables, int32_t* n_tiled_tables);

#ifdef __cplusplus
}
#endif
#endif /* MAXK_TEST_HOOKS_H */
