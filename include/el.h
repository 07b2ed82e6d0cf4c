/*
 * el.h - C ABI of the per-order channel-mixing linear (same library, libsc_mi355x.so).
 *
 * Section 4.1 of arXiv 2504.10700 (the paragraph before Algorithm 2): after the pooling over
 * the neighbours the channels k that belong to one order l are mixed linearly once more, and the
 * result is what the symmetric contraction takes.  For every atom i, output
 * channel k', order l = 0..l_max and component m
 *
 *   Y[i,k',(l,m)] = sum_k W[l,k,k'] * X[i,k,(l,m)]
 *
 * one K_in x K_out matrix per order l, shared by the 2l+1 components of that order; component
 * index l*l + l + m as in sc.h.  No bias and no normalisation factor inside the operation.
 * This is a dense contraction: the kernels run on the matrix cores (MFMA, fp32 or fp64
 * inputs and accumulation) when K_in and K_out are multiples of 64 (forward alone: K_in a
 * multiple of 16), and on plain vector kernels otherwise.
 *
 * Conventions as in sc.h: device pointers, dense row-major, 16-byte aligned; calls enqueue on
 * the given HIP stream and never synchronise; outputs are overwritten; errors by return code
 * with sc_last_error().  Layouts:
 *   X  [n_nodes][K_in][(l_max+1)^2]     W  [l_max+1][K_in][K_out]     Y  [n_nodes][K_out][(l_max+1)^2]
 */
#ifndef EL_MI355X_H
#define EL_MI355X_H

#include "sc.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t struct_size; /* = sizeof(el_config), ABI guard */
  int32_t k_in;        /* K_in >= 1                        */
  int32_t k_out;       /* K_out >= 1                       */
  int32_t l_max;       /* 0..SC_MAX_L                      */
  int32_t dtype;       /* sc_dtype of X, W, Y and the gradients */
  int32_t device;      /* HIP device ordinal               */
} el_config;

/* Forward.  n_nodes == 0 is valid and does nothing. */
sc_status el_forward(const el_config* cfg, int64_t n_nodes, const void* X, const void* W, void* Y, void* hip_stream);

/* Bytes of device workspace el_backward needs (W transposed for the dX product, partial sums of dW per range of atoms). */
sc_status el_workspace_bytes(const el_config* cfg, int64_t n_nodes, size_t* bytes);

/* Backward for an upstream gradient dY [n_nodes][K_out][(l_max+1)^2] (training, Section 2.2):
 *   dX [n_nodes][K_in][(l_max+1)^2] = sum_k' W[l,k,k'] dY[.,k',.]          (overwritten)
 *   dW [l_max+1][K_in][K_out]       = sum over atoms and m of X[.,k,.] dY[.,k',.]   (overwritten)
 * workspace: device memory, 256-byte aligned, at least el_workspace_bytes().  dW is summed in a
 * fixed order (per range of atoms, then over the ranges): bitwise reproducible.
 * n_nodes == 0 zeroes dW. */
sc_status el_backward(const el_config* cfg, int64_t n_nodes, const void* X, const void* W, const void* dY, void* dX,
                      void* dW, void* workspace, size_t workspace_bytes, void* hip_stream);

/* The linear and the contraction as one forward call (Section 4.1: the channel mixing and
 * Algorithm 2 are consecutive steps on the receiving atom):
 *
 *   B = sc_forward(A, z, W)   with   A[i,k',(l,m)] = sum_k W_lin[l,k,k'] X[i,k,(l,m)]
 *
 * plan: a contraction plan (sc.h); its num_channels is K_out of the linear, its l_max the l_max
 * of X, its dtype the dtype of every tensor.  k_in: input channels of the linear.
 *   X [n_nodes][k_in][(l_max+1)^2]   W_lin [l_max+1][k_in][K]   z [n_nodes] int32   W [Z][num_paths][K]
 *   B [n_nodes][K][n_LM]  (overwritten)
 * For fp32 plans served by the generated 0e+1o kernel with K a multiple of 128 and k_in a multiple
 * of 16, one kernel computes the tile of A on the matrix cores and evaluates the contraction from
 * the accumulators: A is never written (el_sc_is_fused returns 1).  Every other plan runs
 * el_forward into the workspace and then sc_forward, with the same result up to rounding.
 * workspace: device memory, 256-byte aligned, at least el_sc_workspace_bytes().  Same conventions
 * as sc_forward (stream, no synchronisation); z is not validated: an index outside 0..Z-1 gives an
 * undefined B row for that atom, never an access outside the buffers.  n_nodes == 0 does nothing. */
int32_t el_sc_is_fused(const sc_plan* plan, int32_t k_in);
sc_status el_sc_workspace_bytes(const sc_plan* plan, int32_t k_in, int64_t n_nodes, size_t* bytes);
sc_status el_sc_forward(sc_plan* plan, int32_t k_in, int64_t n_nodes, const void* X, const void* W_lin,
                        const int32_t* z, const void* W, void* B, void* workspace, size_t workspace_bytes,
                        void* hip_stream);

/* Backward of el_sc_forward for an upstream gradient dB [n_nodes][K][n_LM] (training, Section 2.2):
 *   dX     [n_nodes][k_in][(l_max+1)^2]   gradient with respect to X        (overwritten)
 *   dW_lin [l_max+1][k_in][K]             gradient with respect to W_lin    (overwritten)
 *   dW     [Z][num_paths][K]              gradient with respect to W        (overwritten)
 * Three steps through the workspace, not one kernel: A is computed again (the fused forward never
 * wrote it), sc_backward gives dA and dW, el_backward gives dX and dW_lin.  dW needs the atoms
 * grouped by element and dW_lin a sum over all atoms, so A and dA pass through memory in any
 * arrangement of this backward; what one kernel could save is one read of A.
 * workspace: device memory, 256-byte aligned, at least el_sc_backward_workspace_bytes() (A and dA
 * plus the larger of the two inner workspaces).  Same conventions and reproducibility as
 * sc_backward and el_backward.  n_nodes == 0 zeroes dW and dW_lin.  Plans with bfloat16 rows are
 * not served. */
sc_status el_sc_backward_workspace_bytes(const sc_plan* plan, int32_t k_in, int64_t n_nodes, size_t* bytes);
sc_status el_sc_backward(sc_plan* plan, int32_t k_in, int64_t n_nodes, const void* X, const void* W_lin,
                         const int32_t* z, const void* W, const void* dB, void* dX, void* dW_lin, void* dW,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EL_MI355X_H */
