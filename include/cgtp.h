/*
 * cgtp.h - C ABI of the Clebsch-Gordan tensor product library for AMD MI355X (gfx950).
 *
 * The library computes, on one GPU,
 *
 *     z = TP(P, x, y, W) = W . P . (x (x) y)                       (paper Eq. 1)
 *
 * for a block-sparse Clebsch-Gordan tensor P described by irreps strings and a path
 * list (paper Sec. 2.1, Sec. 2.4 / Eq. 2), its three gradients (paper Sec. 3.3), and the
 * same operation fused into a graph convolution z_j = sum_{e=(j,k)} TP(P, x_k, y_e, W_e)
 * (paper Sec. 3.5, Eq. 4, Alg. 4) with its gradients.
 *
 * A plan is created once per problem: the planner analyses the irreps and paths, builds
 * the nonzero lists of every P^(l1,l2,l3) block, emits HIP source specialised to the
 * problem (coefficients as literals, contraction fully unrolled; paper Sec. 3.2) and
 * compiles it at run time.  Compute calls enqueue kernels on the caller's stream and
 * return without synchronising.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer to caller-owned memory, 16-byte aligned,
 *     row-major [rows, dim] with no padding.  Inputs are never modified; outputs are
 *     overwritten (never accumulated into).
 *   - Inside a row, irreps segments follow the irreps string; inside a segment of
 *     multiplicity mul and degree l the index is u*(2l+1) + (m+l) (layout CGTP_MUL_IR, the
 *     default: the layout the models themselves use, which the paper keeps, Sec. 4) or
 *     (m+l)*mul + u (layout CGTP_IR_MUL, the transposed layout the paper's Sec. 4 discusses
 *     as the alternative), u < mul, m = -l..l, in
 *     the real spherical-harmonic basis in which degree 1 reads (y, z, x).  The CG blocks
 *     are normalised so that sum_{m1 m2} C[m1,m2,k] C[m1,m2,k'] = delta_{kk'} and signed
 *     so that their first nonzero entry in (m1,m2,m3) order is positive.
 *   - Paths are sorted by (ix, iy, iz).  Weights are stored compressed (no structural
 *     zeros, paper Sec. 3): a uvu path (the paper's kernel B) owns mul_x words, a uvw
 *     path (kernel C) a row-major [mul_x, mul_z] tile; tiles are concatenated in path
 *     order.  Per-sample weights are [rows, n_w]; shared weights are [n_w].
 *   - Graphs: edges are given in CSR order by receiver.  row_ptr[j]..row_ptr[j+1] are
 *     the edges entering node j (the row of z they add into) and col[e] is the sender
 *     (the row of x they read).  Row e of y_edges / W_edges belongs to CSR position e.
 *     t_perm lists CSR positions grouped by sender (stable), t_row_ptr indexes it by
 *     sender: the transpose permutation the backward pass needs (paper Sec. 3.5).
 *   - Every function returns a cgtp_status; cgtp_last_error() gives the message of the
 *     last failure on the calling thread.  Nothing throws or aborts across the ABI.
 *   - Zero rows (B == 0, E == 0) are valid: nothing is launched, except that conv
 *     outputs indexed by node are still zero-filled.  Nodes without edges get exact zeros.
 */
#ifndef CGTP_H
#define CGTP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cgtp_plan cgtp_plan; /* opaque; owned by the library until cgtp_plan_destroy */

typedef enum {
  CGTP_OK = 0,
  CGTP_EINVAL = 1,       /* malformed irreps, forbidden path, null pointer, negative size */
  CGTP_EUNSUPPORTED = 2, /* valid problem outside what the kernels cover */
  CGTP_ECOMPILE = 3,     /* run-time compilation of the generated source failed, or the compiled code was refused
                            (see cgtp_check_code_object) */
  CGTP_ERUNTIME = 4,     /* a HIP call failed */
  CGTP_ENOMEM = 5
} cgtp_status;

typedef enum { CGTP_F32 = 0, CGTP_F64 = 1 } cgtp_dtype;
typedef enum { CGTP_UVU = 0, CGTP_UVW = 1 } cgtp_mode;
/* Plan flags.  Bit 0 selects the layout inside the irreps segments of x, z and their gradients (paper Sec. 4,
 * "data layout"): CGTP_MUL_IR (0, default) index u*(2l+1) + (m+l); CGTP_IR_MUL (1) index (m+l)*mul + u.  y (mul = 1)
 * and the weights are the same in both.  IR_MUL is implemented for uvu plans (every entry point); uvw plans answer
 * CGTP_EUNSUPPORTED.  All other bits must be zero (CGTP_EINVAL). */
enum { CGTP_MUL_IR = 0u, CGTP_IR_MUL = 1u };

/* One instruction of the problem description (paper Eq. 2): segment indices into the three
 * irreps lists, the weight structure, and an extra scale alpha applied to the path. */
typedef struct {
  int32_t ix, iy, iz;
  int32_t mode;  /* cgtp_mode */
  double coeff;  /* alpha_p, 1.0 for the plain tensor product */
} cgtp_path;

/* Which kernel of a plan (for cgtp_plan_source / cgtp_plan_kernel_info). */
typedef enum {
  CGTP_K_TP_FWD = 0,
  CGTP_K_TP_BWD = 1,
  CGTP_K_CONV_FWD = 2,
  CGTP_K_CONV_BWD = 3,
  CGTP_K_CONV_FWD_ATOMIC = 4,
  CGTP_K_CONV_BWD_ATOMIC = 5,
  CGTP_K_TP_DBL_BWD = 6,    /* the fused second-order kernel (uvw with per-sample weights, two-kernel variant: its backward-like half) */
  CGTP_K_CONV_DBL_FWD = 7,  /* uvw plans with per-sample weights, two-kernel variant: the forward-like half of tp_double_backward */
  CGTP_K_CONV_DBL_BWD = 8
} cgtp_kernel;

/* ---- planning (host side, synchronous; paper Sec. 3.1-3.2) ------------------------- */

/* Build a plan.  paths == NULL / n_paths == 0 enumerates every path allowed by the
 * triangle rule and the parity rule over the three irreps lists, in `default_mode`.
 * shared_weights != 0 means one weight vector for all rows (uvw plans only; the contraction then runs on the
 * matrix cores, fp32, mul_x % 4 == 0 and mul_z % 16 == 0).  uvw plans with shared_weights == 0 take a weight
 * tile per row (the paper's kernel C as DiffDock-like models use it): fp32 and fp64, multiplicities up to 64.
 * `device` is the HIP device ordinal the kernels are compiled and loaded for; a negative
 * value plans and generates source without touching any GPU (no kernel can be launched
 * from such a plan).  Fails with CGTP_EINVAL (bad string, forbidden path, uvu with
 * mul_x != mul_z, unknown flag bit), CGTP_EUNSUPPORTED (mul_y != 1, l > 8, mixed uvu/uvw, CGTP_IR_MUL with a
 * uvw plan), CGTP_ECOMPILE.  `flags`: see CGTP_MUL_IR / CGTP_IR_MUL above. */
cgtp_status cgtp_plan_create(const char* irreps_x, const char* irreps_y, const char* irreps_z,
                             const cgtp_path* paths, int32_t n_paths, int32_t default_mode,
                             int32_t shared_weights, int32_t dtype, int32_t device, uint32_t flags,
                             cgtp_plan** out);
/* Optional settings of a plan.  struct_size = sizeof(cgtp_options) as the caller knows it (fields beyond it
 * keep their defaults).  kahan_conv != 0: the convolution kernels (conv_forward, conv_backward,
 * conv_forward_atomic) add the per-edge results of a row with compensated (Kahan) summation, the extension
 * the paper's Sec. 5 proposes for stable neighbourhood sums; costs four extra additions per output word and
 * edge and twice the accumulator registers. */
typedef struct {
  int32_t struct_size;
  int32_t kahan_conv;
} cgtp_options;

/* cgtp_plan_create with options (NULL = defaults). */
cgtp_status cgtp_plan_create_ex(const char* irreps_x, const char* irreps_y, const char* irreps_z,
                                const cgtp_path* paths, int32_t n_paths, int32_t default_mode,
                                int32_t shared_weights, int32_t dtype, int32_t device, uint32_t flags,
                                const cgtp_options* options, cgtp_plan** out);
cgtp_status cgtp_plan_destroy(cgtp_plan* plan);

/* Introspection.  which: 0 = dim_x, 1 = dim_y, 2 = dim_z, 3 = number of weights n_w. */
int64_t cgtp_plan_dim(const cgtp_plan* plan, int32_t which);
int32_t cgtp_plan_num_paths(const cgtp_plan* plan);
/* Path p in weight order: the instruction, its (l1,l2,l3), the number of nonzeros of its CG
 * block and the offset of its weight tile.  Any output pointer may be NULL. */
cgtp_status cgtp_plan_get_path(const cgtp_plan* plan, int32_t p, cgtp_path* path, int32_t* l1l2l3,
                               int32_t* nnz, int64_t* w_offset);
/* Nonzeros of path p's CG block, lexicographic in (i,j,k), including the normalisation but not
 * alpha.  Writes at most `cap` entries to each non-NULL array, returns the total count. */
int32_t cgtp_plan_path_nonzeros(const cgtp_plan* plan, int32_t p, int32_t cap, int32_t* i, int32_t* j,
                                int32_t* k, double* v);
/* Nonzero-FLOP model per row (sample or edge): which 0 = forward, 1 = backward, 2 = second-order pass as the
 * fused kernels evaluate it.  Forward counts 2 per nonzero per channel plus the weight multiply; backward 3x the
 * contraction + 1.5x the weight part (2x for uvw plans, whose backward is two GEMMs of the forward's size); the
 * second-order pass 8x the contraction + 3x the weight part (the seven separate dispatches of the paper would be
 * 3 forward + 4 backward = 15x + 9x); for uvw plans with per-sample weights 7x + 5x (seven dispatches: 15x + 11x). */
int64_t cgtp_plan_flops(const cgtp_plan* plan, int32_t which);
/* Generated HIP source of a kernel (NUL-terminated, owned by the plan), or NULL. */
const char* cgtp_plan_source(const cgtp_plan* plan, int32_t kernel);
/* Compiled-kernel facts: info[0] = vector registers (both kinds), [1] = SGPRs, [2] = static LDS bytes,
 * [3] = private (spill) bytes per lane, [4] = workgroup size, [5] = resident workgroups per CU (0 when the
 * plan was compiled without a device).  Available once the kernel has been compiled (device >= 0 or -2). */
cgtp_status cgtp_plan_kernel_info(const cgtp_plan* plan, int32_t kernel, int32_t info[6]);

/* ---- batched tensor product (paper Alg. 1-2) and its backward (Alg. 3) --------------- */

/* z[b] = TP(P, x[b], y[b], W[b]) for b < B.  x [B,dim_x], y [B,dim_y], W [B,n_w] or [n_w]
 * when the plan has shared weights, z [B,dim_z]. */
cgtp_status tp_forward(cgtp_plan* plan, const void* x, const void* y, const void* W, void* z,
                       int64_t B, void* hip_stream);

/* Given gz = dE/dz [B,dim_z]: gx = dE/dx [B,dim_x], gy = dE/dy [B,dim_y], gW = dE/dW, all three
 * computed in one pass (paper Sec. 3.3, Alg. 3).  uvu plans and uvw plans with per-row weights: gW is
 * [B,n_w].  uvw plans with shared weights (needs mul_x and mul_z multiples of 16): gW is [n_w], summed over
 * the batch in a fixed order (deterministic) through a plan-owned workspace that grows on demand; calls on
 * one plan must not overlap. */
cgtp_status tp_backward(cgtp_plan* plan, const void* x, const void* y, const void* W, const void* gz,
                        void* gx, void* gy, void* gW, int64_t B, void* hip_stream);

/* Second-order pass (paper Sec. 3.4).  With (a, b, C) = (dE/dx, dE/dy, dE/dW) as tp_backward returns
 * them and a scalar L(a, b, C): given La = dL/da [B,dim_x], Lb = dL/db [B,dim_y], LC = dL/dC [B,n_w],
 * writes Lx = dL/dx [B,dim_x], Ly = dL/dy [B,dim_y], LW = dL/dW [B,n_w], Lgz = dL/dgz [B,dim_z].
 * Equal to the paper's linear combination of seven forward / backward dispatches.  uvu plans: evaluated in
 * one fused kernel that reads every operand once; no workspace.  uvw plans with per-sample weights: also one
 * kernel, which forms Lgz from the W and LC tiles while it holds them for Lx, Ly, LW (every operand read once, no
 * workspace); plans created with CGTP_UVWPS_DBL_ONE=0 in the environment use a forward-like kernel for Lgz and a
 * backward-like one for the rest instead.
 * With CGTP_UVWPS_DBL_FUSED=0 in the environment such plans run the seven dispatches themselves instead (three
 * tp_forward, four tp_backward on permuted operands, sums formed in place; B * (dim_x + dim_y + dim_z + n_w)
 * elements of temporaries in the plan's workspace, grown on first use, CGTP_ENOMEM if that fails): a second route
 * to the same result, kept for verification.  uvw plans with shared weights: CGTP_EUNSUPPORTED.  All pointers are
 * device pointers, 16-byte aligned, row-major. */
cgtp_status tp_double_backward(cgtp_plan* plan, const void* x, const void* y, const void* W, const void* gz,
                               const void* La, const void* Lb, const void* LC, void* Lx, void* Ly, void* LW,
                               void* Lgz, int64_t B, void* hip_stream);

/* ---- fused tensor product + graph convolution (paper Eq. 4, Alg. 4) ------------------ */

/* z_nodes[j] = sum over CSR row j of TP(P, x_nodes[col[e]], y_edges[e], W_edges[e]).
 * x_nodes [V,dim_x], y_edges [E,dim_y], W_edges [E,n_w], z_nodes [V,dim_z]; row_ptr [V+1] and
 * col [E] are int64 device arrays.  Deterministic: no atomics, run-to-run bit-identical.
 * Uses a plan-owned workspace that grows on demand (hipMalloc on the first call and when
 * a larger problem arrives); calls on one plan must not overlap.  uvu plans only. */
cgtp_status conv_forward(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                         void* z_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                         void* hip_stream);

/* conv_forward for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels and bit-identical results; the side buffer for rows
 * split between edge ranges is a static device array of the library (32 MiB per GPU, held from the moment the library
 * is loaded on that GPU until the process ends) instead of the plan's workspace, so the call allocates nothing - not
 * on its first use either.  Needs (edge ranges) * 2 * dim_z * sizeof(element) bytes, where the number of edge ranges
 * is min(E, waves of the kernel resident on the GPU); CGTP_EINVAL with the figures in cgtp_last_error() if that
 * exceeds the array (the MACE-shaped benchmark plan needs exactly 32 MiB in either precision).  The plan's device
 * must be the current device.  All calls on one GPU share the array: calls that overlap in time on one GPU (different
 * streams, different plans, different threads) race; calls on one stream are ordered and safe. */
cgtp_status conv_forward_static(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                void* z_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                                void* hip_stream);

/* Gradients of conv_forward given gz_nodes [V,dim_z]: gx_nodes [V,dim_x] (summed over the edges
 * leaving each node), gy_edges [E,dim_y], gW_edges [E,n_w] (CSR order).  t_row_ptr [V+1] and
 * t_perm [E] are the transpose permutation described above.  Same workspace rule. */
cgtp_status conv_backward(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                          const void* gz_nodes, void* gx_nodes, void* gy_edges, void* gW_edges, int64_t V,
                          int64_t E, const int64_t* row_ptr, const int64_t* col, const int64_t* t_row_ptr,
                          const int64_t* t_perm, void* hip_stream);

/* Second-order pass of the convolution (paper Sec. 3.4 applied to Eq. 4).  With (a, b, C) = conv_backward's
 * (gx_nodes, gy_edges, gW_edges) and a scalar L(a, b, C): given La_nodes = dL/da [V,dim_x], Lb_edges = dL/db
 * [E,dim_y], LC_edges = dL/dC [E,n_w], writes Lx_nodes = dL/dx [V,dim_x], Ly_edges = dL/dy [E,dim_y], LW_edges =
 * dL/dW [E,n_w], Lgz_nodes = dL/dgz [V,dim_z].  Equal to the paper's combination of seven convolution forward /
 * backward dispatches; evaluated by two fused kernels (one walk over receiver rows for dL/dgz, one over sender
 * rows for the rest).  Deterministic; same graph arrays, layouts, workspace rule and errors as conv_backward. */
cgtp_status conv_double_backward(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                 const void* gz_nodes, const void* La_nodes, const void* Lb_edges,
                                 const void* LC_edges, void* Lx_nodes, void* Ly_edges, void* LW_edges,
                                 void* Lgz_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                                 const int64_t* t_row_ptr, const int64_t* t_perm, void* hip_stream);

/* conv_forward / conv_backward for edge data that stays in the caller's own (unsorted) order: y_edges / W_edges /
 * gy_edges / gW_edges row edge_perm[c] belongs to CSR position c, with edge_perm the `perm` array that
 * cgtp_csr_from_coo returns (int64 device array [E]; NULL = identity, i.e. conv_forward / conv_backward).
 * Together with cgtp_csr_from_coo this serves unsorted edge lists deterministically and without moving the
 * per-edge tensors; on MI355X it is several times faster than the atomic variant below. */
cgtp_status conv_forward_perm(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                              void* z_nodes, int64_t V, int64_t E, const int64_t* row_ptr, const int64_t* col,
                              const int64_t* edge_perm, void* hip_stream);
cgtp_status conv_backward_perm(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                               const void* gz_nodes, void* gx_nodes, void* gy_edges, void* gW_edges, int64_t V,
                               int64_t E, const int64_t* row_ptr, const int64_t* col, const int64_t* t_row_ptr,
                               const int64_t* t_perm, const int64_t* edge_perm, void* hip_stream);

/* ---- nondeterministic convolution on unsorted edges (paper Sec. 3.5, second algorithm) -- */

/* Same results as conv_forward / conv_backward up to the order of the floating-point sums, for an
 * edge list in ANY order: edge e goes from node send[e] (row of x) to node recv[e] (row of z);
 * y_edges / W_edges / gy_edges / gW_edges row e belongs to edge e.  Needs neither CSR order nor
 * the transpose permutation.  The node-indexed output (z_nodes, resp. gx_nodes) is zero-filled
 * and then accumulated with one hardware float atomic per word and edge, so results are not
 * bit-reproducible from run to run.  recv, send: int64 device arrays [E].  uvu plans only; no
 * workspace is used. */
cgtp_status conv_forward_atomic(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                void* z_nodes, int64_t V, int64_t E, const int64_t* recv, const int64_t* send,
                                void* hip_stream);
cgtp_status conv_backward_atomic(cgtp_plan* plan, const void* x_nodes, const void* y_edges, const void* W_edges,
                                 const void* gz_nodes, void* gx_nodes, void* gy_edges, void* gW_edges, int64_t V,
                                 int64_t E, const int64_t* recv, const int64_t* send, void* hip_stream);

/* ---- graph preparation (integer work; paper Sec. 3.5 requires row-sorted edges) ------ */

/* Stable sort of E COO edges (recv[e], send[e]), 0 <= index < V, by (receiver, sender, original
 * position).  All pointers are device pointers to int64; outputs: row_ptr [V+1], col [E],
 * perm [E] (original index of the edge at each CSR position), t_row_ptr [V+1], t_perm [E].
 * Scratch memory belongs to the library (one buffer per device and stream, grown when a larger graph than any
 * before arrives, kept until the process ends).  The range check of the indices is part of the return value
 * (CGTP_EINVAL), so this call waits for the stream once before it returns; cgtp_csr_from_coo_async does not. */
cgtp_status cgtp_csr_from_coo(const int64_t* recv, const int64_t* send, int64_t E, int64_t V,
                              int64_t* row_ptr, int64_t* col, int64_t* perm, int64_t* t_row_ptr,
                              int64_t* t_perm, void* hip_stream);

/* The same preparation as an ordinary asynchronous call (paper Sec. 3.5 needs it once per graph; models that rebuild
 * their neighbour list every step need it on the stream like any other kernel): everything is enqueued on hip_stream,
 * nothing is allocated, nothing waits.  `workspace` is caller-owned device memory of at least
 * cgtp_csr_workspace_bytes(E, V) bytes, 256-byte aligned (CGTP_EINVAL if it is smaller); its contents are scratch.
 * bad_flag (device int32, may be NULL) receives 1 if any index lies outside [0, V) - such edges are then treated as
 * (0, 0) - else 0.  t_row_ptr and t_perm may both be NULL: the transpose (needed by the backward pass only) is skipped. */
size_t cgtp_csr_workspace_bytes(int64_t E, int64_t V);
cgtp_status cgtp_csr_from_coo_async(const int64_t* recv, const int64_t* send, int64_t E, int64_t V,
                                    int64_t* row_ptr, int64_t* col, int64_t* perm, int64_t* t_row_ptr,
                                    int64_t* t_perm, void* workspace, size_t workspace_bytes, int32_t* bad_flag,
                                    void* hip_stream);

/* Message of the last error on this thread (valid until the next failing call on it). */
const char* cgtp_last_error(void);

/* The check every freshly compiled kernel passes before it is cached or loaded, applied to a code object in a file
 * (host path): the code is disassembled and searched for vector instructions placed between the exit of a
 * lane-divergent loop and the next write to the execution mask, where no lane is active (register-allocator spill
 * code has been seen there; a kernel with such code is refused at plan creation, CGTP_ECOMPILE).  Writes the first
 * such instruction as a C string into found[0..capacity) (empty string: none).  CGTP_EINVAL if the file cannot be
 * read or is no gfx950 code object.  No GPU needed. */
cgtp_status cgtp_check_code_object(const char* path, char* found, size_t capacity);

#ifdef __cplusplus
}
#endif
#endif /* CGTP_H */
