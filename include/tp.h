/*
 * tp.h - C ABI of the MI355X channelwise tensor product (same library, libsc_mi355x.so).
 *
 * The operation is the message construction of MACE (channelwise tensor product), Algorithm 1 of
 * arXiv 2504.10700 (Section 4.1), fused with the pooling over the neighbours of the
 * receiving atom that the same section describes before Algorithm 2: for every atom i,
 * channel k and output component (l3,m3)
 *
 *   A[i,k,(l3,m3)] = sum_{edges ji with receiver i} sum_{(l1,m1),(l2,m2)}
 *                    C(l1,l2,l3)[m1,m2,m3] * R[ji, p(l1,l2,l3), k] * Y[ji,(l1,m1)] * h[j,k,(l2,m2)]
 *
 * with j the sender of edge ji, Y the spherical harmonics of the edge direction
 * (l1 = 0..l_Y), h the sender's features (l2 = 0..l_h), R the per-edge, per-channel radial
 * weights and C the real-basis coupling tensors of sc.h (sc_coupling_tensor).  All three
 * carry the real basis with component index l*l + l + m and parity (-1)^l.
 *
 * Paths (the index of R): every (l1,l2,l3) with |l1-l2| <= l3 <= l1+l2 (triangle rule,
 * Section 4.2), l3 <= L_max and l1+l2+l3 even (parity), ordered by (l1,l2,l3) ascending.
 * Contributions of different paths to one (l3,m3) are summed (accumulation line of
 * Algorithm 1).
 *
 * Graph layout.  Edges are stored grouped by receiver, receivers ascending (the order in
 * which neighbour lists are built): row_ptr[i] .. row_ptr[i+1] are the edges received by
 * atom i.  The backward additionally needs the edges grouped by sender: send_ptr[j] ..
 * send_ptr[j+1] index send_edge[], which lists the ids of the edges sent by atom j
 * (ascending within a sender, so that results are reproducible).  Per-edge messages
 * without pooling (the literal output of Algorithm 1) are obtained by passing
 * row_ptr = 0,1,..,E with n_nodes_out = E.
 *
 * Conventions: as in sc.h (device pointers for tensors and index arrays, dense row-major,
 * 16-byte aligned tensors, 4-byte aligned index arrays; calls enqueue on the given HIP
 * stream and never synchronise; outputs are overwritten; errors by return code with
 * sc_last_error()).  Index arrays are not validated (they live on the device and the calls do
 * not synchronise): sender values outside [0, n_nodes_in), a row_ptr that is not ascending
 * from 0 to n_edges, or a send_edge that is not a permutation of the edge ids give undefined
 * VALUES; every index is clamped into its range where the kernels read it, so such a list never
 * makes them touch memory outside the buffers.
 * No entry point allocates; no workspace is needed except for tp_backward (see there).
 */
#ifndef TP_MI355X_H
#define TP_MI355X_H

#include "sc.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tp_plan tp_plan; /* opaque */

#define TP_MAX_L 3 /* largest l_Y, l_h and L_max */

typedef struct {
  int32_t struct_size;  /* = sizeof(tp_config), ABI guard                              */
  int32_t num_channels; /* K >= 1                        (N_channels of Algorithm 1)   */
  int32_t l_Y;          /* Y carries l1 = 0..l_Y, 0..TP_MAX_L                          */
  int32_t l_h;          /* h carries l2 = 0..l_h, 0..TP_MAX_L                          */
  int32_t L_max;        /* A carries l3 = 0..L_max, 0..TP_MAX_L (L_max of Algorithm 1) */
  int32_t dtype;        /* sc_dtype of Y, h, R, A and the gradients                    */
  int32_t device;       /* HIP device ordinal (ignored with SC_PLAN_HOST_ONLY)         */
  uint32_t flags;       /* SC_PLAN_HOST_ONLY, SC_PLAN_FORCE_GENERIC                    */
} tp_config;

typedef struct {
  int32_t n_Y;         /* (l_Y+1)^2   */
  int32_t n_h;         /* (l_h+1)^2   */
  int32_t n_out;       /* (L_max+1)^2 */
  int32_t num_paths;   /* P: second extent of R */
  int32_t specialised; /* 1 if generated straight-line kernels serve this plan */
  /* generated kernels only (else 0): vector instructions / floating-point operations (a fused
   * multiply-add counts as two) per (edge, channel) of the forward, the backward and the
   * second-order kernel */
  int32_t ops[3];
  int32_t flops[3];
} tp_info;

/* Section 4.1, inputs of Algorithm 1: fixes K and the three l ranges, derives the sparse
 * coupling terms on the host and uploads them.  Fails with SC_ERR_UNSUPPORTED beyond
 * TP_MAX_L; never later. */
sc_status tp_plan_create(const tp_config* cfg, tp_plan** out_plan);
sc_status tp_plan_destroy(tp_plan* plan);
sc_status tp_plan_info(const tp_plan* plan, tp_info* out);

/* paths: host buffer of num_paths rows {l1, l2, l3} in the order of the second index of R. */
sc_status tp_plan_paths(const tp_plan* plan, int32_t* paths);

/* Non-zero coupling terms of the plan (host buffers, for tests and the kernel generator):
 * term t says  msg[c[t]] += coef[t] * R[path[t]] * Y[a[t]] * h[b[t]].  Call with
 * capacity 0 to query the count. */
sc_status tp_plan_terms(const tp_plan* plan, int32_t capacity, int32_t* n_terms, int32_t* path, int32_t* a,
                        int32_t* b, int32_t* c, double* coef);

/* Forward of Algorithm 1 with pooling.
 *   Y       dev [n_edges][n_Y]            h       dev [n_nodes_in][K][n_h]
 *   R       dev [n_edges][num_paths][K]   sender  dev int32 [n_edges], values in [0, n_nodes_in)
 *   row_ptr dev int32 [n_nodes_out + 1]   A       dev [n_nodes_out][K][n_out]   (overwritten;
 *                                                  rows of atoms without incoming edges are zero)
 * n_nodes_out == 0 or n_edges == 0 are valid (A, if any, is zeroed). */
sc_status tp_forward(tp_plan* plan, int64_t n_nodes_in, int64_t n_nodes_out, int64_t n_edges, const void* Y,
                     const void* h, const void* R, const int32_t* sender, const int32_t* row_ptr, void* A,
                     void* hip_stream);

/* Bytes of device workspace tp_backward and tp_double_backward need (partial sums of dY per 64-channel block and
 * the per-edge shares of dh or d2h: about n_edges * (K * n_h + ceil(K/64) * n_Y) elements; the backward of the
 * generated kernels keeps only the edges' receiver indices where the shares would be). */
sc_status tp_workspace_bytes(const tp_plan* plan, int64_t n_edges, size_t* bytes);

/* Backward of tp_forward for an upstream gradient dA [n_nodes_out][K][n_out] (training by
 * gradient descent, Section 2.2; dY feeds the forces):
 *   dY dev [n_edges][n_Y]   dh dev [n_nodes_in][K][n_h]   dR dev [n_edges][num_paths][K]   (overwritten)
 * send_ptr dev int32 [n_nodes_in + 1] and send_edge dev int32 [n_edges] group the edges by
 * sender (see the header comment).  workspace: device memory, 256-byte aligned, at least
 * tp_workspace_bytes(plan, n_edges).  All sums have a fixed order: results are bitwise
 * reproducible for identical inputs.  Generated kernels: one launch walks the edges grouped by
 * sender, in the order of send_edge (dR and the partial dY of every edge; dh of an atom is summed
 * in registers and written once, zero for an atom that sends nothing), one sums the dY partials.
 * dR and dY of an edge are written by the walk of the sender under which send_edge lists it: an
 * edge that send_edge omits keeps whatever dR and dY held.  Table-driven kernels walk by receiver,
 * write every edge's share of dh into the workspace and sum the shares per sender in a third launch. */
sc_status tp_backward(tp_plan* plan, int64_t n_nodes_in, int64_t n_nodes_out, int64_t n_edges, const void* Y,
                      const void* h, const void* R, const int32_t* sender, const int32_t* row_ptr,
                      const int32_t* send_ptr, const int32_t* send_edge, const void* dA, void* dY, void* dh,
                      void* dR, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Second-order pass (Section 2.2: forces are derivatives of the energy and reach a force loss
 * through dY, so that loss differentiates tp_backward once more).  With (dY, dh, dR) as
 * returned by tp_backward for dA and
 *   psi = sum(HY * dY) + sum(Hh * dh) + sum(HR * dR)
 * it returns the gradients of psi with respect to the four arguments of the backward:
 *   HY  dev [n_edges][n_Y]   Hh dev [n_nodes_in][K][n_h]   HR dev [n_edges][num_paths][K]   (cotangents, inputs)
 *   ddA dev [n_nodes_out][K][n_out]   d2Y dev [n_edges][n_Y]   d2h dev [n_nodes_in][K][n_h]
 *   d2R dev [n_edges][num_paths][K]                                                   (all overwritten)
 * Everything else (graph arrays, workspace of tp_workspace_bytes, zero rows for atoms without
 * edges, fixed summation orders) is as for tp_backward. */
sc_status tp_double_backward(tp_plan* plan, int64_t n_nodes_in, int64_t n_nodes_out, int64_t n_edges, const void* Y,
                             const void* h, const void* R, const int32_t* sender, const int32_t* row_ptr,
                             const int32_t* send_ptr, const int32_t* send_edge, const void* dA, const void* HY,
                             const void* Hh, const void* HR, void* ddA, void* d2Y, void* d2h, void* d2R,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* Measurement helper as in sc.h: while enabled, tp_forward / tp_backward bracket their
 * main kernels with HIP events; tp_profile_read returns the durations in milliseconds of
 * the forward kernel, the edge-walking backward kernel (with the generated kernels: the
 * receiver indices and the walk by sender) and the per-sender sum of dh (table-driven kernels;
 * the generated backward has no such launch and reports the time between two events with
 * nothing in between) of the most recent calls (negative if none). */
sc_status tp_profile_enable(tp_plan* plan, int32_t on);
sc_status tp_profile_read(tp_plan* plan, float* forward_ms, float* backward_ms, float* dh_sum_ms);
/* Same for the edge-walking kernel of the most recent tp_double_backward call. */
sc_status tp_profile_read_double_backward(tp_plan* plan, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* TP_MI355X_H */
