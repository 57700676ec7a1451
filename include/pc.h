/*
 * libpc -- forward (log-likelihood) and backward (PC flows) passes of a compiled probabilistic
 * circuit on one AMD gfx950 GPU.  Plain C ABI: raw pointers and sizes, no C++/torch types.
 *
 * Conventions used by every entry point
 *   - "device" pointers are hipMalloc-style GPU addresses owned by the caller; "host" pointers are
 *     ordinary CPU memory.  theta, tables, their flow arrays and the workspace must be 16-byte aligned
 *     (PC_ERR_ARG otherwise).  The handle (pc_circuit) owns only its compiled int32 tables and a few
 *     KB of reduction scratch.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Forward, backward
 *     and the EM step only enqueue kernels (no memset or copy nodes, no allocation); they never
 *     synchronise the device, so a caller may capture them into a HIP graph and replay it.  A kernel
 *     fault surfaces as PC_ERR_HIP from the next call that checks the runtime's error state.
 *   - Every call returns a pc_status; pc_last_error() gives a thread-local message for the last
 *     non-OK status.  No exceptions cross this boundary.
 *   - Node blocks hold K node slots.  The compiled node offset of user block u is (u+1)*K; rows
 *     0..K-1 are a reserved null block (log-probability 0, flow 0).  Parameter block p lives at
 *     theta[(p+1)*K*K ...]; theta[0 .. K*K) must be all zero (it backs the padding entries of the
 *     index tables, the "pseudo blocks with probability 0" of Sec. 4.3).  Inside a parameter block
 *     element (i, j) is at i*K + j, i = sum node in its block, j = child node in its block
 *     (the view(K_M, K_N) of Alg. 1).
 *   - tables[t][c][k]: probability of category c under node k of an input block that uses table t
 *     (category-major so that one (sample, variable) lookup reads K contiguous floats; the paper
 *     gives no input-layer layout).
 *   - Precision: fp32 data and fp32 accumulation everywhere.  Sum layers of K = 64 / 128 whose rows reduce over at least
 *     2048 child nodes, and parameter flows reduced over at least 4096 samples per parameter block, take each product
 *     as three bf16 MFMAs on operands split into a bf16 pair (hi + lo; the dropped lo x lo term is 2^-16 relative).
 *   - Environment switches, read once per process, for measurements and cross-checks (results stay within the same
 *     tolerances): PC_BF16=0 keeps every contraction on the fp32 matrix cores; PC_BF16_CT=1|2 forces the 64 x 32 or
 *     64 x 64 tile form of the bf16 sum kernels; PC_FORCE_GENERIC=1 (read by pc_compile) routes every block size
 *     through the one-thread-per-output kernels.
 */
#ifndef PC_H_
#define PC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pc_circuit pc_circuit;

typedef enum {
    PC_OK = 0,
    PC_ERR_ARG,              /* null pointer, negative size, id out of range, unsupported K      */
    PC_ERR_CYCLE,            /* the block graph is not a DAG                                    */
    PC_ERR_NOT_ALTERNATING,  /* sum block with a non-product child, product with a product child */
    PC_ERR_NOT_BLOCK_SPARSE, /* duplicate (parent, child) block pair, or an inner block w/o child */
    PC_ERR_TIE,              /* two sum blocks share some but not all of their parameter blocks  */
    PC_ERR_TOO_LARGE,        /* an index does not fit in int32                                  */
    PC_ERR_WORKSPACE,        /* workspace smaller than pc_workspace_bytes                       */
    PC_ERR_STATE,            /* pc_backward without a matching pc_forward                       */
    PC_ERR_HIP               /* the HIP runtime reported an error                               */
} pc_status;

/* Block-level DAG handed to pc_compile (all host pointers, read only, not retained).
 * Def. 1: input blocks carry a categorical distribution per node, product blocks multiply their
 * child blocks element-wise (node k of the block has node k of every child block as children),
 * sum blocks are fully connected to each of their child blocks through one K x K parameter block
 * (Sec. 4.2: every block pair is fully connected or unconnected). */
typedef struct {
    int32_t K;                 /* node block size K_M = K_N (Sec. 4.1), 1 <= K <= 128 (larger: PC_ERR_ARG); the matrix-core
                                  kernels serve K % 32 == 0, vector kernels every other K */
    int32_t n_blocks;
    int32_t root_block;        /* a sum block; its node 0 is the root n_r                        */
    const uint8_t *type;       /* [n_blocks] 0 input, 1 product, 2 sum                           */
    const int32_t *n_real;     /* [n_blocks] real nodes in the block, 1..K; slots n_real..K-1 are placeholders (Sec. 4.1
                                  footnote) of probability 0: the caller keeps their theta rows and table columns at 0.  A
                                  product node over a placeholder slot of any child has probability 0 as well, so a
                                  product block has no more useful nodes than its smallest child; equality of the
                                  counts is not required */
    const int64_t *child_ptr;  /* [n_blocks+1] CSR offsets into child / param_blk                */
    const int32_t *child;      /* [n_edges] child block ids                                      */
    const int32_t *param_blk;  /* [n_edges] parameter block id of a sum edge (equal ids = tied parameters,
                                  App. A.3); ignored for product edges                           */
    int32_t n_param_blocks;
    const int32_t *in_var;     /* [n_blocks] variable read by an input block                     */
    const int32_t *in_table;   /* [n_blocks] categorical table used by an input block            */
    int32_t n_vars, n_cats, n_tables;
    int32_t max_groups;        /* G of Alg. 2 (App. A.1)                                         */
    int32_t tol_permille;      /* tol of Alg. 2 in 1/1000                                        */
    int32_t product_scratch;   /* 0: every node's log-probability is kept for the backward pass.
                                  1: the memory-saving mode of Sec. 5 -- the log-probabilities of product blocks live in one
                                  scratch sized for the largest product layer and are recomputed in the backward pass just
                                  before the sum layer that reads them.  Needs the block order of pc_order_for_scratch. */
} pc_dag;

/* Compile once, reuse for every batch (Sec. 6.1).  Layers by longest-path depth (Sec. 3), groups by
 * the dynamic programme of App. A.1, forward index tensors sum_ids / prod_ids / param_ids (Sec. 4.3)
 * and backward index tensors ch_ids / par_ids / par_param_ids (App. A.2), for sum and product layers
 * alike.  Validation, depths and Alg. 2 run on the host; the graph transpose, the sorting of neighbour lists and
 * the filling of every table run as HIP kernels on `stream`; the call waits for them.  *out is set only on PC_OK. */
pc_status pc_compile(const pc_dag *dag, void *stream, pc_circuit **out);
/* The host half of pc_compile alone (validation, layering, Alg. 2, tables); touches no GPU.  The handle
 * serves pc_get_sizes / pc_get_layer / pc_copy_group / pc_workspace_*; forward, backward and the EM
 * step return PC_ERR_STATE on it, and pc_get_group reports NULL device pointers. */
pc_status pc_compile_host(const pc_dag *dag, pc_circuit **out);
void pc_destroy(pc_circuit *c);
const char *pc_last_error(void);

/* Collapse of consecutive sum / sum and product / product blocks (footnote to Def. 2): pc_compile accepts only DAGs
 * in which sum blocks have product children and product blocks have sum or input children (PC_ERR_NOT_ALTERNATING
 * otherwise); this optional pre-pass rewrites any other DAG of sum, product and input blocks into that form.  A
 * product block takes over the children of its product children; a sum block takes over the children of its sum
 * children with the K x K weight blocks multiplied (sum_j A[i][j] sum_k B[j][k] c_k = sum_k (A B)[i][k] c_k), several
 * paths to one child add up.  The circuit computes the same function; its parameters are those of the collapsed
 * circuit.  Host only; `theta` is a host array [n_param_blocks + 1][K][K].  Canonical form of the result:
 *   - edges keep the order of the original edges, a replaced edge expanding in place into its child's edges; a child
 *     reached twice keeps its first position (product blocks: PC_ERR_NOT_BLOCK_SPARSE);
 *   - blocks no longer reachable from the root are dropped, the others keep their order (block_map: old id -> new id, -1);
 *   - a sum block none of whose edges changed keeps its parameter blocks (and its ties), a changed one gets fresh
 *     blocks for all its edges; parameter blocks are renumbered in order of first use.
 * A sum block with an input child remains an error of pc_compile.  The handle owns every array it hands out
 * (pc_collapsed_dag: ready for pc_compile; max_groups, tol_permille, n_vars, n_cats, n_tables are copied). */
typedef struct pc_collapsed pc_collapsed;
pc_status pc_collapse(const pc_dag *dag, const float *theta, pc_collapsed **out);
/* Block order for product_scratch = 1 (Sec. 5, product values recomputed): the same DAG with its blocks renumbered --
 * input and sum blocks first (relative order kept), then the product blocks grouped by the depth of the sum blocks
 * that read them, so that the product blocks a sum layer reads are one contiguous range of ids.  A product block read
 * by sum blocks of several depths is copied, one copy per depth (it is then evaluated once for each of them; product
 * blocks carry no parameters, so log-likelihoods and parameter flows are those of the original circuit).  Parameter
 * block ids do not change; the result (pc_collapsed_dag; pc_collapsed_block_map: old id -> new id, for a copied block
 * its first copy; product_scratch already set) is owned by the handle. */
pc_status pc_order_for_scratch(const pc_dag *dag, pc_collapsed **out);
const pc_dag *pc_collapsed_dag(const pc_collapsed *r);
const float *pc_collapsed_theta(const pc_collapsed *r, int64_t *len);   /* [n_param_blocks + 1][K][K], block 0 zero */
const int32_t *pc_collapsed_block_map(const pc_collapsed *r);            /* [n_blocks of the input DAG]            */
void pc_collapsed_destroy(pc_collapsed *r);

typedef struct {
    int32_t K, n_blocks, n_layers;
    int64_t n_rows;            /* (n_blocks+1)*K rows of the node buffers                        */
    int64_t theta_len;         /* floats in theta / theta_flow: (n_param_blocks+1)*K*K           */
    int64_t tables_len;        /* floats in tables / table_flow: n_tables*n_cats*K               */
    int32_t n_vars, n_cats, n_tables;
} pc_sizes;
pc_status pc_get_sizes(const pc_circuit *c, pc_sizes *out);

/* Compiled layers, for inspection and bit-exact checks.  Layer 0 is the input layer. */
typedef struct {
    int32_t kind;              /* 0 input, 1 product, 2 sum                                      */
    int32_t depth;
    int32_t n_fwd_groups;      /* input layer: 1                                                 */
    int32_t n_bwd_groups;      /* input layer: 0                                                 */
} pc_layer_desc;
pc_status pc_get_layer(const pc_circuit *c, int32_t layer, pc_layer_desc *out);

/* One group of a layer.  dir 0 = forward tables, 1 = backward tables.
 *   sum / product layer, forward : ids = sum_ids [n_rows] (node offsets), nbr = prod_ids,
 *                                   par = param_ids [n_rows x width] (parameter offsets; product: zeros)
 *   sum / product layer, backward: ids = ch_ids, nbr = par_ids, par = par_param_ids
 *   input layer (dir 0, group 0) : ids = node offsets, nbr = variable per block, par = table per block, width 1
 * Pointers are device addresses owned by the handle. */
typedef struct {
    int32_t n_rows, width;
    const int32_t *ids, *nbr, *par;
} pc_group_desc;
pc_status pc_get_group(const pc_circuit *c, int32_t layer, int32_t dir, int32_t group, pc_group_desc *out);
/* Same tables copied to host arrays sized from pc_get_group (any of the three may be NULL). */
pc_status pc_copy_group(const pc_circuit *c, int32_t layer, int32_t dir, int32_t group,
                        int32_t *ids_host, int32_t *nbr_host, int32_t *par_host);

/* Workspace (device, caller-owned) for batches of up to B samples.  It holds three node buffers
 * of n_rows x stride floats, row = node offset, samples contiguous (l in R^{N x B} of Sec. 4.3):
 *   l  log-probability residuals, F  node flows, N  log(F) - l of sum rows (the log_nf of Alg. 3 / 4),
 * one block buffer R of (n_blocks+1) x stride floats, row = node offset / K, and small per-batch
 * scratch.  The log-probability of node row n in sample b is  R[n / K][b] + l[n][b]  (R holds
 * integers; keeping the bulk of a large log-probability there leaves l accurate to ~1e-6).
 * stride = B rounded up to a multiple of 32; columns >= B behave as fully marginalised samples with
 * root flow 0. */
#define PC_MAX_BATCH 2097152   /* samples per call: kernels address a batch row with 32-bit byte offsets (else PC_ERR_TOO_LARGE) */
typedef struct {
    int64_t stride;            /* floats between consecutive rows                               */
    size_t l_offset, f_offset, n_offset, r_offset;   /* byte offsets into the workspace         */
    size_t total_bytes;
    int64_t l_rows;            /* rows of l and F: n_rows, or with product_scratch the null, input and sum blocks followed by
                                  the window of the largest product layer (product rows are not kept; N then has the
                                  null, input and sum rows only)                                           */
} pc_ws_layout;
pc_status pc_workspace_layout(const pc_circuit *c, int32_t B, pc_ws_layout *out);
pc_status pc_workspace_bytes(const pc_circuit *c, int32_t B, size_t *bytes);

/* Forward pass, Eq. (1) in log space: ll[b] = log p_root(x_b).
 *   theta  device [theta_len] fp32;  tables device [tables_len] fp32
 *   x      device int32 [B, n_vars] category per variable
 *   mask   device uint8 [B, n_vars] or NULL; non-zero marginalises that variable (Sec. 2)
 *   ll     device fp32 [B] (out).  A sample of probability 0 gives -inf.
 * Leaves every node's log-probability in the workspace for pc_backward. */
pc_status pc_forward(pc_circuit *c, const float *theta, const float *tables, const int32_t *x,
                     const uint8_t *mask, int32_t B, void *workspace, size_t workspace_bytes,
                     float *ll, void *stream);

/* pc_forward for callers that cannot allocate device memory or pass a workspace along: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and same result as
 * pc_forward, but the workspace is a fixed array of PC_STATIC_SCRATCH_BYTES inside the library's device image (every
 * GPU the library runs on holds its copy until the process ends).  The call allocates nothing and records no timing
 * events; it only enqueues kernels on `stream`.  PC_ERR_WORKSPACE if pc_workspace_bytes(c, B) exceeds
 * PC_STATIC_SCRATCH_BYTES.  All calls on one GPU share that array: calls that overlap in time on one GPU (two streams,
 * two threads, two circuits) race; the array keeps the last call's contents, and every call writes what it reads.  It
 * leaves no state for pc_backward (which returns PC_ERR_STATE after it). */
#define PC_STATIC_SCRATCH_BYTES (64u << 20)
pc_status pc_forward_static(pc_circuit *c, const float *theta, const float *tables, const int32_t *x,
                            const uint8_t *mask, int32_t B, float *ll, void *stream);

/* Backward pass, Def. 2: node flows with F_root = 1, then
 *   theta_flow[param(n,c)] += sum_b theta_{n,c} p_c / p_n F_n        (Alg. 3; tied edges add up, App. A.3)
 *   table_flow[t][x_b,v][k] += sum_b F_n                              for observed variables
 * Both flow arrays are device fp32 with the layouts of theta / tables and are ACCUMULATED into
 * (mini-batch and full-batch EM, Sec. 6.1 / 6.3); either may be NULL to skip that part.
 * Must follow pc_forward on the same workspace, B, theta, tables, x, mask (else PC_ERR_STATE).
 * Samples of probability 0 contribute no flow. */
pc_status pc_backward(pc_circuit *c, const float *theta, const float *tables, const int32_t *x,
                      const uint8_t *mask, int32_t B, void *workspace, size_t workspace_bytes,
                      float *theta_flow, float *table_flow, void *stream);

/* EM update (Sec. 2; step size of App. C.3): per sum node, with Z = sum of its accumulated edge flows
 * and n_ch its number of real children,
 *   theta_new = (flow + pseudocount / n_ch) / (Z + pseudocount);  theta <- (1 - step) theta + step theta_new
 * (row unchanged if Z + pseudocount == 0; placeholder rows / columns unchanged); the same per table
 * column over the categories.  Sum blocks with tied parameters are normalised once over their summed
 * flows.  Zeroes theta_flow and table_flow afterwards. */
pc_status pc_em_step(pc_circuit *c, float *theta, float *tables, float *theta_flow, float *table_flow,
                     float step, float pseudocount, void *stream);

/* Per-kernel timing for benchmarks (the measurement protocol, not an operation of the paper).  While enabled,
 * every kernel launch of forward / backward / EM is bracketed by two HIP events on the launch stream.
 * pc_profile_read waits for the recorded events (it synchronises with the work launched so far) and returns
 * the running totals per kernel class since pc_profile_enable; class names: pc_kernel_class_name(i),
 * i < n_classes ("sum_fwd", "sum_bwd_child", "sum_bwd_param", "prod_fwd", ...). */
#define PC_MAX_KERNEL_CLASSES 16
typedef struct {
    int32_t n_classes;
    int64_t launches[PC_MAX_KERNEL_CLASSES];
    double ms[PC_MAX_KERNEL_CLASSES];
    int64_t bf16_launches[PC_MAX_KERNEL_CLASSES];   /* of those, launches whose contraction ran as bf16-split products */
} pc_profile;
pc_status pc_profile_enable(pc_circuit *c, int32_t on);
pc_status pc_profile_read(pc_circuit *c, pc_profile *out);
const char *pc_kernel_class_name(int32_t cls);

/* Achievable peaks of the device the calling thread has current, for quoting beside the published ones (measurement
 * protocol).  Both time `reps` launches of a plain kernel with HIP events on `stream` and wait for them.
 *   pc_measure_copy      16-byte streaming copy of `bytes` from src to dst (device, 16-byte aligned, not overlapping);
 *                        *gb_per_s = (bytes read + bytes written) / time
 *   pc_measure_mfma_f32  register-only loop of v_mfma_f32_32x32x2_f32 on every SIMD; `out` is a device buffer of at
 *                        least 2 MiB that receives the accumulators; *tflops = multiply-add flops / time */
pc_status pc_measure_copy(const void *src, void *dst, size_t bytes, int32_t reps, void *stream, double *gb_per_s);
pc_status pc_measure_mfma_f32(void *out, size_t out_bytes, int32_t reps, void *stream, double *tflops);

#ifdef __cplusplus
}
#endif
#endif /* PC_H_ */
