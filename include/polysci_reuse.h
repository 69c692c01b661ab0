/*
 * polysci_reuse.h -- C ABI of the host-side data-reuse analysis (no GPU involved; all pointers are HOST pointers
 * owned by the caller).
 *
 * The three calls are Section 4 of the paper for perfectly nested rectangular loop nests with a single statement:
 * Algorithm 1 (working-set sizes of every dependence), Algorithm 2 (which cache level can hold each working set)
 * and Eq. 1 (the cost that ranks code variants).  The polyhedral machinery of the paper is replaced by direct
 * enumeration of the iteration space, which is exact for such nests.
 */
#ifndef POLYSCI_REUSE_H
#define POLYSCI_REUSE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_REUSE_MAX_LOOPS 8
#define PS_REUSE_MAX_DIMS 4

/* Loops 0 .. n_loops-1, outermost first, iterator l running over 0 .. extent[l]-1; the schedule is the
 * lexicographic order of the iterators (Section 3). */
typedef struct {
    int32_t n_loops;
    int32_t extent[PS_REUSE_MAX_LOOPS];
} ps_loop_nest;

/* One array reference of the statement: array[ f_0 ][ f_1 ] ... with f_d = sum_l coef[d][l] * iter_l + offset[d]
 * (the read and write relations of Section 3).  elem_bytes weights every element of this reference's array when
 * working sets are counted (use 1 to count elements as the paper does); it must agree between references to the
 * same array. */
typedef struct {
    int32_t array;      /* array id, 0 .. 31 */
    int32_t n_dims;     /* 1 .. PS_REUSE_MAX_DIMS */
    int32_t is_write;   /* 0 = read, 1 = write */
    int32_t elem_bytes; /* >= 1 */
    int32_t coef[PS_REUSE_MAX_DIMS][PS_REUSE_MAX_LOOPS];
    int32_t offset[PS_REUSE_MAX_DIMS];
} ps_array_ref;

/* One dependence that exists in the nest, and its two working-set sizes (Algorithm 1). */
typedef struct {
    int32_t src_ref, tgt_ref; /* indices into the reference list */
    int64_t ws_min, ws_max;   /* distinct data touched from the first source iteration up to and including its
                                 first / last target iteration, in elem_bytes units */
} ps_reuse_dep;

/* Algorithm 1.  Considers every ordered pair of references to the same array (read/read, write/read, read/write,
 * write/write; a reference paired with itself included) whose accesses meet in two different iterations.  Writes
 * up to `cap` entries to `out` (may be NULL if cap == 0) and returns the number of dependences found, or a negative
 * ps_status: PS_EINVAL for malformed arguments, PS_EUNSUPPORTED if the iteration space exceeds 2^24 iterations or
 * an array's bounding box exceeds 2^28 elements. */
int ps_reuse_working_sets(const ps_loop_nest *nest, const ps_array_ref *refs, int n_refs, ps_reuse_dep *out, int cap);

/* Algorithm 2.  `ws` holds n_ws working-set sizes (duplicates are dropped: WS_all is a set); cache_sizes[0..n_levels)
 * are the capacities from the fastest level outwards, in the same unit.  Sizes are taken in ascending order; each is
 * added to the first level whose accumulated size still admits it, else to *mem_ws.  level_ws receives n_levels
 * sums.  Returns PS_OK or PS_EINVAL. */
int ps_reuse_assign(const int64_t *ws, int n_ws, const int64_t *cache_sizes, int n_levels, int64_t *level_ws,
                    int64_t *mem_ws);

/* Eq. 1: sum_i level_ws[i] * lat[i] / bw[i] + mem_ws * lat[n_levels] / bw[n_levels].  lat and bw hold
 * n_levels + 1 entries (the last is main memory).  Returns a negative value on invalid arguments. */
double ps_reuse_cost(const int64_t *level_ws, int n_levels, int64_t mem_ws, const double *lat, const double *bw);

#ifdef __cplusplus
}
#endif
#endif /* POLYSCI_REUSE_H */
