/*
 * bb.h - C ABI of the load balancer (same library, libsc_mi355x.so; host code only).
 *
 * Algorithm CREATE-BALANCED-BATCHES of arXiv 2504.10700 (Section 3, the subsection on the iterative
 * multi-objective bin packing): distributes N graphs with given sizes (vertex counts) over
 * bins (mini-batches) of capacity C, the number of bins a multiple of the number of GPUs G,
 * by dealing the graphs in descending size order to the bins in descending order of remaining
 * capacity, one graph per bin and sweep; bins that cannot take the current graph are set
 * aside as full and get a second chance when an active bin has become fuller than they are;
 * graphs left over when no bin remains are packed the same way into a fresh set of bins.
 *
 * Readings where the paper is open or at odds with itself: the bins are sorted as the listing
 * says (stable, remaining capacity descending - the prose speaks of fuller bins first); ties
 * keep the previous order, bins returned by the second chance are appended behind the active
 * ones; bins are numbered in creation order (first call 0..M-1, then the bins of every
 * further call for left-over graphs) and bins that stay empty are kept, so every call
 * contributes a multiple of G bins; a graph larger than C is an error.
 */
#ifndef BB_MI355X_H
#define BB_MI355X_H

#include "sc.h"

#ifdef __cplusplus
extern "C" {
#endif

/* sizes        host int32 [n_graphs], 0 <= sizes[i] <= capacity
 * bin_of_graph host int32 [n_graphs] (out): the bin every graph was put into
 * slot_of_graph host int32 [n_graphs] (out, may be NULL): its position inside that bin
 *              (the order in which the bin received its graphs)
 * n_bins       host (out): number of bins created (a multiple of n_gpus; 0 for no graphs)
 * Runs on the calling thread, allocates host memory only, touches no device.
 * SC_ERR_INVALID_ARG: null pointer, capacity < 1, n_gpus < 1, n_graphs < 0 or a size
 * outside [0, capacity].  Deterministic: equal inputs give equal outputs. */
sc_status bb_create_balanced_batches(const int32_t* sizes, int64_t n_graphs, int64_t capacity, int32_t n_gpus,
                                     int32_t* bin_of_graph, int32_t* slot_of_graph, int64_t* n_bins);

#ifdef __cplusplus
}
#endif
#endif /* BB_MI355X_H */
