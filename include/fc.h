/*
 * fc.h -- C ABI of the fused-combinator library for AMD MI355X (gfx950).
 *
 * The library executes array-combinator programs (paper section 2, "Language")
 * as fused clusters (section 3, "Fusion"): map / zipWith / generate producers
 * are evaluated in registers, pushed through gathers, and consumed by a fold, a
 * segmented fold, a single-pass scan or a scatter, so that no intermediate
 * array reaches memory.  Which combinators share a loop is described by a
 * clustering (section 4.1: pi, x, m; section 4.2: traversal orders) that
 * fc_plan() chooses by solving the paper's integer linear program exactly.
 *
 * Everything here is plain C: POD structs, raw pointers, sizes.  No exception
 * crosses the boundary; every function returns FC_OK (0) or a negative error
 * code and leaves a message for fc_last_error().
 *
 * Pointers are HOST pointers unless a comment says DEVICE.
 */
#ifndef FC_H
#define FC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------- error codes */
#define FC_OK                   0
#define FC_E_BADGRAPH          -1  /* cycle / arity / dtype / shape mismatch, unknown function  */
#define FC_E_ILLEGAL_PARTITION -2  /* breaks a rule of section 3.4 or a constraint of Fig. "Total ILP formulation" */
#define FC_E_UNSUPPORTED       -3  /* legal cluster, but no kernel is built for its combination of consumers (e.g. three
                                      folds of flattened arrays, a scan of f32 that feeds a fold in its cluster), or its element
                                      programs exceed the limits (24 nodes, 7 external arrays, gathers nested 3 deep).
                                      Element programs of maps, generates and gathers as such always run: compiled for
                                      the shapes of the paper's programs, interpreted otherwise */
#define FC_E_UNBOUND           -4  /* an input or manifest array has no device buffer, or it is too small / misaligned */
#define FC_E_SCRATCH           -5  /* scratch missing, misaligned or smaller than fc_scratch_bytes() */
#define FC_E_HIP               -6  /* a HIP runtime call failed (message holds hipGetErrorString) */
#define FC_E_ARG               -7  /* NULL / out-of-range argument, capacity too small */
#define FC_E_LIMIT             -8  /* graph too large for the exact chooser, or a size above 2^31-1 elements */
#define FC_E_DEVICE_WAIT       -9  /* fc_check: a kernel of an earlier call gave up a bounded wait (see fc_check) */

/* ---------------------------------------------------------------- vocabulary */
/* Combinators of the language (section 2; Table 1 gives their cluster signatures).
 * One node = one combinator = the array it produces. */
typedef enum fc_kind {
  FC_INPUT    = 0,  /* array handed in by the caller; every edge out of it is infusible (section 3.4) */
  FC_MAP      = 1,  /* n-ary map: zipWith after the SoA transformation (section 2, last paragraph) */
  FC_GENERATE = 2,  /* ys[i] = f(i) */
  FC_GATHER   = 3,  /* ys[j] = src[idx[j]]; arg0 = idx (read in output order), arg1 = src (read in the gather's own order) */
  FC_FOLD     = 4,  /* shape (1): fold of the flattened argument; else fold of the innermost dimension */
  FC_FOLDSEG  = 5,  /* arg0 = flat values, arg1 = offsets[R+1] (infusible); y[r] = fold of values[off[r], off[r+1]) */
  FC_SCANL    = 6,  /* exclusive prefix combine (+), identity seeded; traversal order 0; a rank-2 array is scanned row
                       by row.  i32: exact.  f32: summed in a fixed tree order (the same bits on every launch), so
                       a prefix differs from the sequentially rounded sum by rounding only; an f32 scan can be
                       stored (also together with the array it scans) but not fused with a scatter or a fold
                       (FC_E_UNSUPPORTED) */
  FC_SCANR    = 7,  /* exclusive suffix combine; traversal order 1 */
  FC_SCATTER  = 8,  /* arg0 = dest (infusible, updated in place; none of the other arguments may be the same array:
                       FC_E_BADGRAPH), arg1 = index, arg2 = value, arg3 = flag (optional);
                       fn = OVERWRITE (kept indices distinct) or ADD (colliding indices combine: exact for i32,
                       in an unspecified order for f32) */
  FC_FORCE    = 9   /* identity; every edge out of it is infusible */
} fc_kind;

typedef enum fc_dtype { FC_F32 = 0, FC_I32 = 1 } fc_dtype;

/* Element functions (the paper allows arbitrary lambdas; the kernels here are
 * hand written, so the lambdas form a closed vocabulary). */
typedef enum fc_fn {
  FC_FN_NONE = 0,
  /* map functions; fp32 arithmetic is rounded operation by operation (never contracted) */
  FC_FN_IDENT = 1,        /* x                                           */
  FC_FN_AFFINE = 2,       /* fparam[0]*x + fparam[1]                     */
  FC_FN_SIN_X_MUL_X = 3,  /* sin(x)*x                                    */
  FC_FN_SQ_PLUS_ONE = 4,  /* x*x + 1                                     */
  FC_FN_MUL2 = 5,         /* a*b                                         */
  FC_FN_ADD2 = 6,         /* a+b                                         */
  FC_FN_ADD3 = 7,         /* (a+b)+c                                     */
  FC_FN_ADD5 = 8,         /* (((a+b)+c)+d)+e                             */
  FC_FN_EXP_NEG = 9,      /* exp(-x)                                     */
  FC_FN_MOD_EQ = 10,      /* i32 -> i32: (x mod iparam[0] == iparam[1]) ? 1 : 0 for x >= 0; iparam[0] > 0;
                             a residue outside [0, iparam[0]) matches no x */
  /* generate functions (index -> i32) */
  FC_FN_IOTA = 32,            /* i                                                       */
  FC_FN_IOTA_REV = 33,        /* n-1-i                                                   */
  FC_FN_CLAMP_SHIFT_2D = 34,  /* (i,j) -> clamp(i+iparam[0],0,H-1)*W + clamp(j+iparam[1],0,W-1) */
  FC_FN_ROW_OF_2D = 35,       /* (i,j) -> i                                              */
  FC_FN_CONST_I32 = 36,       /* iparam[0]                                               */
  /* reducers of fold / foldSeg / scan and combination functions of scatter */
  FC_OP_ADD = 64,
  FC_OP_MAX = 65,
  FC_OP_MUL = 66,
  FC_OP_OVERWRITE = 67        /* scatter only: the new value wins (section 2.1) */
} fc_fn;

#define FC_MAX_ARGS 6

/* node flags */
#define FC_NODE_OUTPUT 1u   /* a result of the program: must be manifest (m = 0) */
#define FC_NODE_SINGLE_PASS 2u /* on a fold or foldSeg node: its cluster must run as ONE pass over the arrays it reads,
                                  every gather issued at the position that asks for it (section 2: a fold inside a
                                  cluster is one stage of a parallel reduction).  Without the flag the library may, for
                                  a gathered table larger than the L2 of an XCD, run a kernel that visits the positions
                                  in another order and in more than one kernel (elements sorted by table range in a
                                  first kernel and gathered from on-chip memory; for small inputs the streams of a
                                  segmented fold read once per column range), which is faster and, the reducers
                                  being commutative, gives the same result up to rounding */

typedef struct fc_node {
  int32_t  kind;              /* fc_kind  */
  int32_t  dtype;             /* fc_dtype of the produced array */
  int32_t  fn;                /* fc_fn    */
  float    fparam[2];
  int32_t  iparam[4];
  int32_t  nargs;
  int32_t  arg[FC_MAX_ARGS];  /* indices of the producing nodes; each < own index (topological order) */
  int32_t  rank;              /* 1 or 2 */
  int64_t  shape[2];          /* row-major extents; unused extents are 1 */
  uint32_t flags;
  uint32_t infusible_args;    /* bit k set: the edge from arg[k] is infusible whatever the kinds say
                                 (the argument is indexed with `!`, wrapped in force, or passed to foreign code) */
} fc_node;

/* The data dependence graph (n, N, F, I) of section 4.1.  Edges are implied by
 * the argument lists; edge e is the e-th (consumer ascending, slot ascending)
 * argument reference.  Fusible / infusible follows from the kinds (inputs,
 * force, scatter destination and scatter result, foldSeg offsets are infusible). */
typedef struct fc_graph {
  int32_t        n;
  const fc_node *nodes;
} fc_graph;

/* A clustering in the variables of Fig. "Total ILP formulation".  All arrays are
 * caller allocated: n_nodes entries for the per-node arrays, n_edges for the
 * per-edge array. */
typedef struct fc_partition {
  int32_t  n_nodes;       /* capacity of pi / fused_away / order_out (in) */
  int32_t  n_edges;       /* capacity of edge_unfused (in)                */
  int32_t *pi;            /* cluster number; clusters run in ascending order           */
  uint8_t *fused_away;    /* m_a: 1 = the array never reaches memory, 0 = manifest      */
  int32_t *order_out;     /* d^o_a: 0, 1 or the label (2 + ordinal) of a gather         */
  uint8_t *edge_unfused;  /* x_ab: 0 = fused over, 1 = not                              */
  int32_t  n_clusters;    /* (out) clusters after the connected-component split         */
  double   cost;          /* (out) value of the requested cost function                 */
  int32_t  proven;        /* (out, fc_plan and fc_plan_weighted) 1: the clustering is optimal; 0: it is the
                             best one found when the search budget of FC_PLAN_ANYTIME ran out */
} fc_partition;

/* cost functions of section 4.1 ("Cost function"), evaluated on the ILP solution */
typedef enum fc_cost {
  FC_COST_CLUSTERS    = 0,  /* (a) largest cluster number + 1                                  */
  FC_COST_FUSED_EDGES = 1,  /* (b) sum of x over fusible edges                                 */
  FC_COST_ARRAYS      = 2,  /* (c) number of manifest non-input arrays                         */
  FC_COST_READS       = 3,  /* (d) array reads: one per (array, consuming cluster, order)      */
  FC_COST_READS_WRITES= 4,  /* (e) reads + manifest arrays                                     */
  FC_COST_BYTES       = 5   /* (e) with every read / write weighted by the array's bytes       */
} fc_cost;

/* plan flags */
#define FC_PLAN_NO_SPLIT 1u  /* keep the raw ILP solution (skip the connected-component split) */
#define FC_PLAN_EXECUTABLE 2u /* choose among the clusterings fc_run_fused has kernels for: the kernels are a fixed
                                 set of cluster shapes, and the optimum of the ILP may contain a legal cluster that
                                 is not among them (fc_run_fused would answer FC_E_UNSUPPORTED).  With this flag the
                                 result is the cheapest clustering that runs; FC_E_UNSUPPORTED if there is none,
                                 i.e. some combinator has no kernel even on its own */
#define FC_PLAN_ANYTIME 4u    /* the chooser is an exact branch and bound: its time grows exponentially with the
                                 number of combinators (seconds up to 24, half a minute at 30, much longer from 36 on).
                                 With this flag it starts from a clustering built greedily and improved by
                                 moving combinators between neighbouring clusters, searches for 1.2 seconds at
                                 most, spends what is left of two seconds on further (random) moves if the search
                                 had not finished, and returns the best clustering found, which is legal at any
                                 moment; fc_partition.proven says whether the search had finished.  Programs of
                                 more than 64 combinators get the greedy clustering improved by two seconds of moves.
                                 Without the flag a search that exceeds its (much larger) budget, or a program
                                 of more than 64 combinators, ends in FC_E_LIMIT */

typedef struct fc_buffer {
  void   *ptr;    /* DEVICE pointer, 16-byte aligned; NULL = not bound */
  int64_t bytes;
} fc_buffer;

/* ---------------------------------------------------------------- planning (host only) */

/* Number of edges of the graph (length of fc_partition.edge_unfused). */
int fc_num_edges(const fc_graph *g, int32_t *n_edges);

/* Choose the clustering that minimises `cost_fn` subject to the constraints of
 * Fig. "Total ILP formulation" (sections 4.1, 4.2), by exact branch and bound over
 * the edge variables x, then split clusters into connected components (section
 * 4.1, "Performance and correctness").  Fills every array of *out, n_clusters, cost
 * and proven.  Graphs of more than 64 non-input nodes, and searches that exceed their
 * budget, are refused (FC_E_LIMIT) unless FC_PLAN_ANYTIME is set. */
int fc_plan(const fc_graph *g, int cost_fn, uint32_t flags, fc_partition *out);

/* fc_plan for a linear combination of the cost functions: minimises
 * sum_k weights[k] * cost_k, k over the FC_COST_COUNT values of fc_cost (section 5.1,
 * "Runtime analysis", proposes such a combination with coefficients found by tuning as
 * the way to a cost function that models run time on a given machine).  weights: HOST,
 * FC_COST_COUNT entries, none negative, not all zero (else FC_E_ARG).  out->cost is the
 * weighted sum for the chosen clustering.  Same outputs and limits as fc_plan. */
#define FC_COST_COUNT 6
int fc_plan_weighted(const fc_graph *g, const double *weights, uint32_t flags, fc_partition *out);

/* The greedy comparison arms of section 5 ("Greedy"): direction 0 walks the fusible edges
 * from the top of the graph, 1 from the bottom, and fuses an edge whenever a legal
 * clustering still exists that fuses it together with the edges already taken.  The
 * result is locally maximal, not optimal.  Same outputs and limits as fc_plan; cost is the
 * value of cost_fn for the returned clustering. */
int fc_plan_greedy(const fc_graph *g, int direction, int cost_fn, uint32_t flags, fc_partition *out);

/* The clustering with every combinator in a cluster of its own (no fusion). */
int fc_partition_trivial(const fc_graph *g, fc_partition *out);

/* Check a clustering against the rules of section 3.4 and the ILP constraints;
 * only pi is read, the other arrays and n_clusters are (re)derived and written.
 * *cost receives the value of cost_fn for it (may be NULL). */
int fc_partition_check(const fc_graph *g, fc_partition *p, int cost_fn, double *cost);

/* Work duplication (named in sections 1 and 6, outside the paper's ILP): clone
 * every map / generate node that a gather reads as its source and that has other
 * consumers, once per such gather, so that each clone has a single traversal
 * order.  Writes the rewritten graph to out_nodes (capacity entries), its size to
 * *out_n, and for each new node the index of the node it came from to origin. */
int fc_duplicate(const fc_graph *g, fc_node *out_nodes, int32_t capacity, int32_t *out_n, int32_t *origin);

/* ---------------------------------------------------------------- execution (device work) */

/* Bytes of device scratch fc_run_* needs for this graph and clustering
 * (p == NULL: the unfused clustering): the control block, the manifest
 * intermediates, and the workspace of the cluster kernel that asks for the most. */
int fc_scratch_bytes(const fc_graph *g, const fc_partition *p, size_t *bytes);

/* Execute the program cluster by cluster, one kernel launch per cluster (two for a
 * fold over a gather from a table larger than the L2 of an XCD), on `hip_stream`
 * (a hipStream_t; NULL = the default stream).  The call only enqueues work and
 * returns; results are valid after the stream is synchronised.
 *
 * bufs[i] is the DEVICE buffer of node i.  Inputs and manifest arrays (m = 0) of
 * the clustering must be bound, fused-away arrays are ignored.  Arrays made
 * manifest by the clustering but not bound by the caller are placed in scratch.
 * A scatter updates its destination buffer in place (section 2, scatter), its own
 * buffer must be NULL or equal to the destination's.  Scalar results (fold of
 * shape (1)) are 4-byte device buffers.  Gather and scatter indices out of range
 * are undefined behaviour, as in the paper.
 *
 * scratch: DEVICE, 256-byte aligned, at least fc_scratch_bytes().  Its first
 * FC_SCRATCH_CONTROL_BYTES must be zero the first time a buffer is used; every
 * call leaves them ready for the next one.  Two calls that overlap in time must
 * not share a scratch buffer. */
int fc_run_fused(const fc_graph *g, const fc_partition *p, const fc_buffer *bufs,
                 void *scratch, size_t scratch_bytes, void *hip_stream);

/* fc_run_fused for callers that cannot allocate device memory or bring a scratch buffer:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, checks, kernels and results as fc_run_fused, but the scratch is a buffer
 * of FC_STATIC_SCRATCH_BYTES inside the library's code object (one copy per device, zero
 * when the library is loaded, kept until the process ends).  The call allocates nothing,
 * on the device or through any library.  The first call on a device looks the buffer's
 * address up (make that call outside a graph capture).
 *
 * Programs whose fc_scratch_bytes() exceeds FC_STATIC_SCRATCH_BYTES (manifest
 * intermediates the caller did not bind, or a kernel workspace, too large) are refused
 * with FC_E_LIMIT before anything is enqueued: bind the intermediates, or use fc_run_fused.
 * All calls on one device share the one buffer: calls that overlap in time on a device
 * (two streams, two host threads) race, as two fc_run_fused calls on one scratch buffer
 * would.  Nothing has to be cleared between calls: words left by earlier calls carry
 * older launch tags.  fc_check(NULL, stream) reports on this buffer. */
#define FC_STATIC_SCRATCH_BYTES (32u << 20)
int fc_run_fused_static(const fc_graph *g, const fc_partition *p, const fc_buffer *bufs, void *hip_stream);

/* Same program, no fusion: one kernel per combinator, every intermediate array
 * (generated index arrays included) materialised in scratch unless bound. */
int fc_run_unfused(const fc_graph *g, const fc_buffer *bufs,
                   void *scratch, size_t scratch_bytes, void *hip_stream);

/* Status of the device work enqueued so far by fc_run_* calls that used `scratch`.
 *
 * Kernels whose workgroups hand partial results to each other (the last stage of a fold,
 * the tiles of a single-pass scan, the teams of the column-blocked segmented fold; section
 * 2 asks of a fold or scan inside a cluster only that it is one pass, and names the chained
 * scan) never wait without bound: a workgroup polls for a word of another workgroup of its
 * launch at most a fixed number of times (about a second), then takes the operator's
 * identity in place of the missing value, sets word 1 of the control block at the start of
 * scratch (word 0 counts the launches that used the block) and goes on, so that no launch
 * can hang the device.  The results of such a launch are wrong.  It cannot happen while the
 * assumptions the kernels rest on hold (workgroups of a launch start in index order; the
 * device is not shared with work that holds compute units for seconds), and fc_run_* does
 * not look: it only enqueues.  A caller that wants the guarantee calls fc_check after the
 * calls whose results it is about to use.
 *
 * fc_check waits until the work enqueued on `hip_stream` has finished (it synchronises the
 * stream), reads the word, and returns FC_OK if it is zero.  Otherwise it clears the word
 * and returns FC_E_DEVICE_WAIT: every result produced with this scratch buffer since the
 * last check is to be discarded.  scratch: DEVICE, the buffer given to fc_run_*; NULL: the
 * buffer fc_run_fused_static uses on the current device.  Allocates nothing.
 * Errors: FC_E_SCRATCH (misaligned), FC_E_HIP. */
int fc_check(void *scratch, void *hip_stream);

/* Name of the kernel instance chosen for cluster `cluster` of the clustering
 * (p == NULL: the unfused clustering), for reports and profiles. */
int fc_cluster_kernel(const fc_graph *g, const fc_partition *p, int32_t cluster,
                      char *name, size_t capacity);

#define FC_SCRATCH_CONTROL_BYTES (1u << 23)

/* Message of the last error on the calling thread; valid until the next call. */
const char *fc_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FC_H */
