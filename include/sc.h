/*
 * sc.h - C ABI of the MI355X symmetric tensor contraction library (libsc_mi355x.so).
 *
 * The operation is the product-basis step of MACE (symmetric contraction), Algorithm 2 of
 * arXiv 2504.10700 (Section 4.1) together with the message equation of Section 2.2:
 * for every atom i, channel k and output component (L,M)
 *
 *   B[i,k,(L,M)] = sum_{nu=1..nu_max} sum_{eta} W[z_i, p(nu,L,eta), k]
 *                  * sum_{a_1..a_nu} U^{(nu,L,eta)}[M; a_1..a_nu] * prod_{xi=1..nu} A[i,k,a_xi]
 *
 * where A are the atomic-basis features in the real spherical-harmonic basis
 * (component index a = l*l + l + m, l = 0..l_max, parity (-1)^l), z_i the element
 * index of atom i, W the element-dependent per-channel weights and U the generalized
 * Clebsch-Gordan coefficients of the coupling path eta.  The backward entry point
 * returns the gradients of sum(dB * B) with respect to A and W.
 *
 * Coupling paths (the paper's eta; it indexes weights by the l-tuple only, which is
 * ambiguous for nu = 3): a path is an ORDERED l-tuple plus, for nu = 3, the
 * intermediate L2 of the chain ((l1 x l2) -> L2) x l3 -> L.  Every path the triangle
 * rule (Section 4.2) and parity allow is present.  Global path index p: nu ascending,
 * then output irrep in the order given in sc_config, then (l1, l2, L2, l3) ascending.
 * U chains real-basis coupling tensors C(l1,l2,l3) - the unique rotation-invariant
 * tensor of the three irreps, unit Frobenius norm, first non-zero entry in row-major
 * (m1,m2,m3) order positive - with no further factor:
 *   nu=1: U[M;a] = delta(a, L*L+L+M)      nu=2: U[M;a1,a2] = C(l1,l2,L)[m1,m2,M]
 *   nu=3: U[M;a1,a2,a3] = sum_M2 C(l1,l2,L2)[m1,m2,M2] * C(L2,l3,L)[M2,m3,M].
 *
 * Conventions for every entry point
 *  - All tensor arguments of sc_forward / sc_backward are DEVICE pointers owned by the
 *    caller: dense, row-major, no strides, 16-byte aligned.  Arguments of the plan /
 *    info / table helpers are HOST pointers.
 *  - sc_forward / sc_backward only enqueue work on the given HIP stream (NULL = the
 *    default stream) and never synchronise.  The plan is immutable after creation and
 *    may be used from several streams; a workspace must not be shared by calls that
 *    can overlap in time.
 *  - Outputs are overwritten (never accumulated into); inputs are never modified;
 *    outputs must not alias inputs or each other.
 *  - Errors are reported by return code only; sc_last_error() gives a thread-local
 *    message for the last failing call of the calling thread.  Argument errors are
 *    found on the host before anything is launched.  Element indices outside
 *    [0, num_elements) are NOT detected: such nodes are skipped by the grouping
 *    pass (their rows of B / dA are left unwritten); no out-of-bounds access results.
 */
#ifndef SC_MI355X_H
#define SC_MI355X_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sc_plan sc_plan; /* opaque; created and destroyed only by this library */

typedef enum {
  SC_OK = 0,
  SC_ERR_INVALID_ARG = 1, /* null pointer, bad size, misaligned pointer, bad struct_size   */
  SC_ERR_UNSUPPORTED = 2, /* configuration outside what the library implements             */
  SC_ERR_WORKSPACE = 3,   /* workspace missing or smaller than sc_workspace_bytes()        */
  SC_ERR_HIP = 4,         /* a HIP runtime call failed (message has the HIP error string)  */
  SC_ERR_ALLOC = 5        /* host or device allocation failed                              */
} sc_status;

/* SC_BF16: the per-node tensors (A, B, dB, dA, H, ddB, dA2) are stored as bfloat16 (halving the
 * bytes the operation must move), W and dW stay fp32 and all arithmetic is fp32; results are
 * rounded to nearest-even on the way out.  Served by the generated kernels only (plans they do
 * not cover fail with SC_ERR_UNSUPPORTED at creation); the channel count must be a multiple of 8. */
typedef enum { SC_F32 = 0, SC_F64 = 1, SC_BF16 = 2 } sc_dtype;

#define SC_MAX_OUT 4       /* output irreps per plan                                       */
#define SC_MAX_L 3         /* largest l_max and largest output L                           */
#define SC_MAX_NU 3        /* largest correlation order                                    */
#define SC_MAX_ELEMENTS 1024

/* sc_config.flags */
#define SC_PLAN_HOST_ONLY 1u     /* build tables only; no device is touched, compute calls fail   */
#define SC_PLAN_FORCE_GENERIC 2u /* use the table-driven kernels even if a specialised one exists */
#define SC_PLAN_WINDOW_ORDER 4u  /* tuning: let sc_forward order its visits by element inside windows of
                                    the batch for every batch size (default: from SC_WINDOW_ORDER_MIN_NODES
                                    nodes on, below which the ordering costs more than it saves).  Results
                                    do not depend on it.                                              */
#define SC_WINDOW_ORDER_MIN_NODES 8192

/* flags of sc_forward / sc_backward / sc_double_backward */
#define SC_REUSE_GROUPING 1u /* the workspace still holds the grouping written by the previous
                                compute call of this plan with the same n_nodes and the
                                same z contents: skip regrouping                           */
#define SC_Z_GROUPED 4u      /* the caller's batch is already grouped by element: z is non-decreasing.
                                The permutation pass is skipped and the backward passes read their
                                rows in batch order.  Pass it to every call on that batch (also to
                                the calls that reuse the grouping).  With a z that is not
                                non-decreasing the results are wrong (never an access outside the
                                buffers).  The table-driven kernels ignore it.                   */
#define SC_REUSE_WEIGHTS 2u  /* the workspace still holds the weights as the previous compute
                                call of this plan prepared them, and W has the same contents
                                (the backward of a step after its forward): skip that step   */

#define SC_COMPONENT_MAJOR 8u /* the per-node tensors (A, B, dB, dA, and H, ddB, dA2 of the second-order
                                 pass) are laid out [n_nodes][component][K] (channel fastest) instead
                                 of [n_nodes][K][component]; W and dW keep their layout.  Served for
                                 plans with a generated kernel (sc_info.specialised) and fp32 or fp64
                                 rows; otherwise the call fails with SC_ERR_UNSUPPORTED and launches
                                 nothing.  The per-node results are those of the default layout,
                                 bit for bit, transposed.                                         */

typedef struct {
  int32_t struct_size;            /* = sizeof(sc_config), ABI guard                                  */
  int32_t num_channels;           /* K >= 1                          (N_channels of Algorithm 2)     */
  int32_t l_max;                  /* A carries l = 0..l_max, 0..SC_MAX_L     (L_max of Algorithm 2)  */
  int32_t nu_max;                 /* correlation order 1..SC_MAX_NU          (nu_max of Algorithm 2) */
  int32_t num_elements;           /* Z: z values lie in [0, Z), 1..SC_MAX_ELEMENTS                   */
  int32_t num_out;                /* number of output irreps, 1..SC_MAX_OUT                          */
  int32_t out_l[SC_MAX_OUT];      /* L of each output irrep, 0..SC_MAX_L                             */
  int32_t out_parity[SC_MAX_OUT]; /* +1 = even ("e"), -1 = odd ("o")                                 */
  int32_t dtype;                  /* sc_dtype of A, W, B, dB, dA, dW (SC_BF16: see sc_dtype)         */
  int32_t device;                 /* HIP device ordinal (ignored with SC_PLAN_HOST_ONLY)             */
  uint32_t flags;                 /* SC_PLAN_*                                                       */
  int32_t tile_nodes;             /* tuning: nodes per tile of the grouping pass; 0 = chosen by the
                                     library from the batch size and the chip's compute-unit count  */
} sc_config;

typedef struct {
  int32_t n_lm;        /* (l_max+1)^2 components of A per (node, channel)          */
  int32_t n_LM;        /* sum of (2L+1) over the output irreps                     */
  int32_t num_paths;   /* P: second extent of W and dW                             */
  int32_t specialised; /* 1 if a generated straight-line kernel serves this plan   */
  /* generated kernels only (else 0): vector instructions and floating-point operations
   * (a fused multiply-add counts as two) per (node, channel) of the forward, backward and
   * second-order main kernels, for roofline accounting */
  int32_t ops[3];
  int32_t flops[3];
} sc_info;

/* Section 4.1, inputs of Algorithm 2: fixes K, l_max, nu_max, the element range and
 * the output irreps; derives the coupling tables (host, Wigner 3j by the Racah sum,
 * moved to the real basis) and uploads them to cfg->device.
 * On success *out_plan owns host and device memory until sc_plan_destroy.
 * Fails with SC_ERR_UNSUPPORTED for parameters beyond the SC_MAX_* limits or output
 * irreps no path can reach; never later. */
sc_status sc_plan_create(const sc_config* cfg, sc_plan** out_plan);

/* Frees the plan (NULL is a no-op returning SC_OK).  The caller must make sure no
 * enqueued work still uses it. */
sc_status sc_plan_destroy(sc_plan* plan);

sc_status sc_plan_info(const sc_plan* plan, sc_info* out);

/* paths: host buffer of num_paths rows {nu, out_index, l1, l2, l3, L2}, unused = -1,
 * in the global path order defined above (the eta of Section 2.2's message equation). */
sc_status sc_plan_paths(const sc_plan* plan, int32_t* paths);

/* Sparse form of one path's generalized coupling tensor after merging slot
 * permutations (the same A enters every slot of the product, Section 4.1, so terms that
 * differ only by a permutation of the slots are one term): term t says  P_{p,M[t]}(a) += coef[t] * a[i1[t]] * a[i2[t]] * a[i3[t]]
 * with i1 <= i2 <= i3 and unused slots = -1.  Call with capacity 0 to query the
 * count (*n_terms); host buffers.  Exists for tests and the kernel generator. */
sc_status sc_plan_path_terms(const sc_plan* plan, int32_t path, int32_t capacity, int32_t* n_terms,
                             int32_t* M, int32_t* i1, int32_t* i2, int32_t* i3, double* coef);

/* C(l1,l2,l3) of the header comment (Clebsch-Gordan coefficients of the paper's
 * notation table in the real basis), row-major [2l1+1][2l2+1][2l3+1] doubles into a
 * host buffer; all zero when the triangle rule fails.  0 <= l <= 2*SC_MAX_L. */
sc_status sc_coupling_tensor(int32_t l1, int32_t l2, int32_t l3, double* out);

/* Bytes of device workspace sc_forward / sc_backward need for a call with exactly
 * n_nodes nodes (a caller that sizes one buffer for several batch sizes takes the
 * maximum over them). */
sc_status sc_workspace_bytes(const sc_plan* plan, int64_t n_nodes, size_t* bytes);

/* Forward of Algorithm 2.
 *   A  dev [n_nodes][K][n_lm]         z  dev int32 [n_nodes]
 *   W  dev [Z][num_paths][K]          B  dev [n_nodes][K][n_LM]   (overwritten)
 * workspace: device memory, 256-byte aligned, >= sc_workspace_bytes(plan, n_nodes).
 * It receives the grouping of nodes by element (reusable by the backward of the
 * same batch, see SC_REUSE_GROUPING).  n_nodes == 0 is valid and does nothing. */
sc_status sc_forward(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W,
                     void* B, void* workspace, size_t workspace_bytes, uint32_t flags, void* hip_stream);

/* For callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): sc_forward with its scratch (the weights
 * prepared for the kernels, the grouping of the table-driven kernels) kept in a fixed device
 * array inside the library instead of a caller's workspace.  Same arguments, same kernels,
 * same results bit for bit as sc_forward without flags.  Calls no hipMalloc, hipFree or other
 * allocating routine.
 * Limits: n_nodes <= SC_NOALLOC_MAX_NODES, and the plan's forward scratch for n_nodes must fit
 * SC_NOALLOC_SCRATCH_BYTES (about 1.9 MB for 89 elements x 128 channels in fp32, 5.1 MB for
 * 256 channels with 0e+1o+2e outputs, plus 8 bytes per node); beyond them the call fails with
 * SC_ERR_WORKSPACE and launches nothing.
 * Every GPU holds ONE such array (SC_NOALLOC_SCRATCH_BYTES of device memory per GPU the
 * library is loaded on, until the process ends), shared by all plans and streams: calls of
 * sc_forward_noalloc that can overlap in time on one GPU race on it and must be ordered by
 * the caller (one stream, or events). */
#define SC_NOALLOC_MAX_NODES 65536
#define SC_NOALLOC_SCRATCH_BYTES (8u << 20)
sc_status sc_forward_noalloc(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W,
                             void* B, void* hip_stream);

/* Backward of Algorithm 2 for an upstream gradient dB (training, Section 2.2: energies
 * and forces are trained by gradient descent through this operation).
 *   dB dev [n_nodes][K][n_LM]
 *   dA dev [n_nodes][K][n_lm]  (overwritten)   dA[i,k,a] = sum_LM dB * dB[i,k,LM]/dA[i,k,a]
 *   dW dev [Z][num_paths][K]   (overwritten)   dW[e,p,k] = sum_{i: z_i = e} sum_M dB[i,k,(L_p,M)] * P_{p,M}(A[i,k,:])
 * Rows of dW for elements that do not occur are zero.  n_nodes == 0 zeroes dW.
 * dW is reduced per element in a fixed order (no floating-point atomics): results
 * are bitwise reproducible for identical inputs. */
sc_status sc_backward(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W,
                      const void* dB, void* dA, void* dW, void* workspace, size_t workspace_bytes,
                      uint32_t flags, void* hip_stream);

/* Second-order pass of Algorithm 2 (Section 2.2: forces are derivatives of the total energy,
 * so a loss on forces differentiates the backward pass once more).  With
 *   psi = sum_{i,k,a} H[i,k,a] * dA[i,k,a](A, W, dB)        (dA as returned by sc_backward)
 * it returns the gradients of psi with respect to the three arguments of the backward pass:
 *   H   dev [n_nodes][K][n_lm]   cotangent of dA (input)
 *   ddB dev [n_nodes][K][n_LM]   (overwritten)  d psi / d dB = directional derivative of B along H
 *   dA2 dev [n_nodes][K][n_lm]   (overwritten)  d psi / d A  = (Hessian of sum(dB*B) in A) . H
 *   dW2 dev [Z][num_paths][K]    (overwritten)  d psi / d W
 * A, z, W, dB, workspace, flags, stream, the zero rows of absent elements, n_nodes == 0 and
 * reproducibility are as for sc_backward (dW2 is reduced exactly like dW). */
sc_status sc_double_backward(sc_plan* plan, int64_t n_nodes, const void* A, const int32_t* z, const void* W,
                             const void* dB, const void* H, void* ddB, void* dA2, void* dW2, void* workspace,
                             size_t workspace_bytes, uint32_t flags, void* hip_stream);

/* Measurement helper (benchmarks only; not part of the operation).  While enabled,
 * sc_forward / sc_backward / sc_double_backward bracket their main kernel - the fused forward
 * kernel, or the fused dA + per-tile dW kernel; not the grouping pass and not the dW reduction - with
 * HIP events on the call's stream.  sc_profile_read blocks until the most recent
 * bracketed call of each kind has finished and returns that kernel's duration in
 * milliseconds (negative if no such call was made).  While enabled the plan must be used
 * from one thread and one stream at a time. */
sc_status sc_profile_enable(sc_plan* plan, int32_t on);
sc_status sc_profile_read(sc_plan* plan, float* forward_ms, float* backward_ms);
/* Same for the main kernel of the most recent sc_double_backward call. */
sc_status sc_profile_read_double_backward(sc_plan* plan, float* ms);

/* Measurement helper (benchmarks only; not part of the operation): streaming kernels without
 * arithmetic that move a known number of bytes, so that a benchmark can state the bandwidth
 * the machine attains in the same run as the contraction kernels.  Enqueues one kernel on the
 * stream, on the current device; all pointers are device memory, 16-byte aligned.
 *   SC_PROBE_READ   reads n bytes of src (dst: 4 bytes, never written for finite data)
 *   SC_PROBE_WRITE  writes n bytes of dst
 *   SC_PROBE_COPY   copies n bytes from src to dst
 *   SC_PROBE_ROWS   the access pattern of the fused backward kernel: for each of n rows, taken
 *                   in the order perm[0..n) (int32, values in [0, n); clamped), reads 4096 bytes
 *                   of src (64 B per lane) and 1024 bytes of src2 (16 B per lane) and writes
 *                   4096 bytes of dst; moves n * 9216 bytes
 *   SC_PROBE_ROWS_FORWARD  the same walk with the forward kernel's traffic: per row 4096 bytes of
 *                   src in and 1024 bytes of dst out (src2 unused); moves n * 5120 bytes
 * n bytes must be a multiple of 16.  src2 and perm are used by the row patterns only. */
#define SC_PROBE_READ 0
#define SC_PROBE_WRITE 1
#define SC_PROBE_COPY 2
#define SC_PROBE_ROWS 3
#define SC_PROBE_ROWS_FORWARD 4
sc_status sc_probe_stream(int32_t kind, const void* src, const void* src2, void* dst, const int32_t* perm,
                          int64_t n, void* hip_stream);

/* Thread-local message of the last failing call on this thread; never NULL. */
const char* sc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SC_MI355X_H */
