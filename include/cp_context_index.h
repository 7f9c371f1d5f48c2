/*
 * cp_context_index: the paper's context index on the host (C ABI).
 *
 * A tree of contexts (ordered lists of distinct context-block ids) in which every node holds a
 * prefix shared by everything below it (paper, Section 4.1, Figure "construction"):
 *   - construction from a batch: pairwise distances (Eq. 1), hierarchical clustering, one
 *     virtual node per merge holding the blocks its two children share, removal of empty virtual
 *     nodes, top-down prefix alignment, search paths (appendix algorithm "Context Index
 *     Construction via Hierarchical Clustering");
 *   - search: greedy descent to the node with the longest shared prefix (Section 4.2, appendix
 *     algorithm "Context Index Tree Search");
 *   - insertion with alignment: the new context inherits the matched node's context as its
 *     prefix and keeps the order of its other blocks (Section 5.1, appendix algorithm "Context
 *     Alignment for Prefix Sharing");
 *   - scheduling: execution order from search paths (Section 5.2, appendix algorithm
 *     "Search-Path-Based Request Grouping and Scheduling").
 *
 * Choices the paper leaves open, as taken here:
 *   - clustering is average linkage; of several pairs at the smallest distance the one with the
 *     smallest lower cluster id is merged, then the smallest higher id (points are 0..m-1, the
 *     cluster made by step t is m + t); cluster distances are combined in double precision;
 *   - identical contexts (same ids, same order) share one leaf whose frequency counts them;
 *     clustering runs over the distinct contexts in order of first appearance;
 *   - a virtual node lists the shared blocks in ascending id order (then aligned to its
 *     parent); children are listed larger subtree first, equal sizes in id order;
 *   - the search goes down only while the best child shares more blocks with the query than the
 *     node it is at, and ends at a leaf or at a child that holds blocks the query lacks; among
 *     children at equal distance the first is taken;
 *   - inserting under a leaf or a partial match puts a new virtual node in its place (shared
 *     blocks in the matched node's order); cached nodes are never reordered.
 *
 * Everything is host memory; no GPU call is made.  The distance matrix may come from
 * cp_context_distance (copied back by the caller) or be left to this library.  All functions
 * return 0 on success, -1 for a NULL pointer, -2 for an argument out of range (including an
 * output buffer that is too small: the needed length is still stored).  An index is not
 * thread-safe.
 */
#ifndef CP_CONTEXT_INDEX_H
#define CP_CONTEXT_INDEX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cp_index cp_index;

/*
 * Which contexts are identical to an earlier one.
 * contexts  HOST [n][stride] int32, row i holds lens[i] distinct ids >= 0 in rank order
 * lens      HOST [n] int32, 0 <= lens[i] <= stride
 * first_of  HOST [n] int32 out: rank (0..m-1, order of first appearance) of the distinct
 *           context that row i equals
 * m         out: number of distinct contexts
 */
int cp_index_distinct(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride,
                      int32_t *first_of, int32_t *m);

/*
 * Builds the index over a batch.
 * alpha     weight of the positional term of Eq. 1, finite and >= 0
 * dist      HOST [m][m] float32 distances between the DISTINCT contexts (see above), row-major,
 *           symmetric; or NULL: Eq. 1 is then evaluated here in double precision
 * m         number of distinct contexts, as cp_index_distinct reports; checked
 * out       receives the index; release with cp_index_free
 * Stored context i (see the accessors) is input row i.
 */
int cp_index_build(const int32_t *contexts, const int32_t *lens, int32_t n, int32_t stride,
                   double alpha, const float *dist, int32_t m, cp_index **out);
void cp_index_free(cp_index *index);

/* Stored contexts (batch rows, then inserted ones) and nodes ever created. */
int32_t cp_index_num_contexts(const cp_index *index);
int32_t cp_index_num_nodes(const cp_index *index);

/* Aligned ids / search path (child positions from the root) of stored context i. */
int cp_index_aligned(const cp_index *index, int32_t i, int32_t *ids, int32_t cap, int32_t *len);
int cp_index_path(const cp_index *index, int32_t i, int32_t *path, int32_t cap, int32_t *len);
/* Node handle of the leaf of stored context i. */
int cp_index_leaf(const cp_index *index, int32_t i, int32_t *node);

/*
 * Tree inspection.  Node handles are stable; handle 0 is the root (empty context).
 * cp_index_node: parent handle (-1 for the root), leaf flag, frequency, clustering distance at
 * which a virtual node was made (0 for leaves and the root), number of children, context.
 * cp_index_children: the child handles in order.
 */
int cp_index_node(const cp_index *index, int32_t node, int32_t *parent, int32_t *is_leaf,
                  int32_t *freq, double *created_at, int32_t *num_children, int32_t *ids,
                  int32_t cap, int32_t *len);
int cp_index_children(const cp_index *index, int32_t node, int32_t *children, int32_t cap,
                      int32_t *len);

/*
 * Search without changing the index: the path to the matched node and its handle.
 */
int cp_index_search(const cp_index *index, const int32_t *ids, int32_t len, int32_t *path,
                    int32_t cap, int32_t *path_len, int32_t *node);

/*
 * Search, align and store a new context (it becomes stored context cp_index_num_contexts()-1).
 * aligned   out [len]: the context to run, a permutation of ids
 * path      out: its search path; cap entries available, path_len receives the length
 * The index is changed only when 0 is returned.  The path of the stored context has at most one
 * entry more than the path cp_index_search reports for the same ids; when cap is below that
 * bound the call returns -2 with the bound in path_len and stores nothing.
 */
int cp_index_insert(cp_index *index, const int32_t *ids, int32_t len, int32_t *aligned,
                    int32_t *path, int32_t cap, int32_t *path_len);

/*
 * Execution order for n contexts from their search paths.
 * paths     HOST [n][stride] int32, row i holds path_lens[i] entries
 * order     HOST [n] int32 out: indices 0..n-1 in execution order
 */
int cp_index_schedule(const int32_t *paths, const int32_t *path_lens, int32_t n, int32_t stride,
                      int32_t *order);

#ifdef __cplusplus
}
#endif
#endif /* CP_CONTEXT_INDEX_H */
