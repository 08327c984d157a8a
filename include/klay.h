/*
 * klay.h -- C ABI of the MI355X (gfx950) layered arithmetic-circuit evaluator.
 *
 * The library evaluates a negation-normal-form circuit DAG (paper Section 2, Eq. 1: leaves
 * are literals, inner nodes AND / OR gates) on a batch of leaf-weight vectors, layer by
 * layer (Section 3.1, Eq. 2; Section 4, Alg. 1; Appendix C, Alg. 2-4), and differentiates
 * the root values with respect to the leaf weights.
 *
 * Conventions
 *   - Plain C, no exceptions.  Every call returns a klay_status; klay_last_error() gives a
 *     thread-local message for the last failing call on the calling thread.
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP device memory on
 *     the circuit's device.  The library never takes ownership of caller buffers.
 *   - klay_forward / klay_backward only enqueue work on the caller's stream; they do not
 *     synchronise the host with the device.  A handle must not be used from two streams at
 *     once (its activation workspace is shared between calls).
 */
#ifndef KLAY_H
#define KLAY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct klay_circuit klay_circuit;   /* opaque; owns index arrays and (unless set) a workspace */

typedef enum {
    KLAY_OK = 0,
    KLAY_EINVAL = 1,   /* malformed argument or circuit (index out of range, empty gate, ...) */
    KLAY_ECYCLE = 2,   /* the node graph is not acyclic */
    KLAY_ENOMEM = 3,   /* host or device allocation failed, or caller workspace too small */
    KLAY_EHIP = 4,     /* a HIP runtime call failed */
    KLAY_ESTATE = 5    /* call order violated (backward before forward, host-only handle, ...) */
} klay_status;

/* Semiring of the evaluation (Section 4): REAL = (+, x) on probabilities, LOG = (logsumexp, +)
 * on log-probabilities (Alg. 4 with epsilon = 0).  Section 4 closes by noting that any semiring
 * whose operations are reductions will do; MAXLOG = (max, +) on log-probabilities is the one
 * offered beyond the paper's two: the log weight of the heaviest proof tree (for a smooth d-DNNF
 * the most probable model).  MAXLOG is evaluated forward only. */
typedef enum { KLAY_REAL = 0, KLAY_LOG = 1, KLAY_MAXLOG = 2 } klay_semiring;

/* node_type codes of the input DAG */
enum { KLAY_LIT = 0, KLAY_AND = 1, KLAY_OR = 2, KLAY_TRUE = 3, KLAY_FALSE = 4 };

/* Build-time options; zero-initialise and override.  0 means "library default". */
typedef struct klay_options {
    int32_t no_reorder;      /* 1: keep nodes of a layer in input-id order (no locality sort)     */
    int32_t heavy_fan;       /* rows with more sources than this are split (default 48); a pass that
                                splits rows anyway and whose unsplit rows are few (under 2e5 entries) with a
                                tenth or more of them in rows longer than half of it splits from half on */
    int32_t min_segment;     /* smallest split segment, in edges (default 24)                     */
    int32_t no_tail;         /* 1: one launch per layer also for the narrow top layers            */
    int32_t unary_chains;    /* 1: the paper's layerization throughout: an edge that skips layers goes through
                                one unary chain node per layer (Section 3.1).  Default (0): padding-free
                                below the narrow top of the circuit.  Chain nodes only copy a value, so in
                                the layers 1 .. A (A = klay_info_t.alias_top_layer) none are made and an edge
                                reads the child's own row wherever it lives; layer A is complete (it holds
                                a stand-in for every node read from above), and the layers above it, the
                                ones the persistent kernels may take, are as in the paper.  Same values
                                and gradients, fewer rows and edges.  klay_layer_csr returns, for the layers
                                up to A, rows of the whole activation buffer (layer 0 first).  A = 0 when
                                the whole circuit is narrow, A = L when no layer is (or with no_tail)   */
    int32_t no_merge;        /* 1: do not identify structurally identical gates (Section 3.2)         */
    int32_t small_batch_edges; /* 1: batches of at most 32 columns run the lanes = edges kernel (a wave takes
                                64 / B index entries per step and reduces the entries of a row across its
                                lanes with a segmented scan) instead of the default, a lane group per row,
                                which measures about twice as fast at B = 1 and B = 4; same results        */
    int32_t tail_rows_cap;   /* > 0: layers with more nodes than this are no candidates for the persistent
                                kernels (at most 20000, the default; smaller values move the boundary
                                between the two parts of the layerization up: for tests)                 */
    int32_t no_fusion;       /* 1: every AND node's value is written.  Default (0): in the padding-free part an
                                AND node with at most one child that is not a leaf, few children and parents,
                                and only short OR rows above it is fused into those rows when the batch has more
                                than 64 columns: they read its children and combine them themselves, so a forward
                                pass does not write its value.  klay_backward, which needs every value, evaluates
                                the fused rows first when it follows such a pass, and the forward pass of a handle
                                whose previous forward pass was followed by klay_backward writes every value.
                                Same results                                                              */
} klay_options;

typedef struct klay_info_t {
    int32_t num_vars;
    int32_t num_roots;
    int32_t num_layers;       /* L: gate layers 1..L above the leaf layer 0                        */
    int32_t device;           /* -1 for a host-only handle                                        */
    int64_t num_nodes;        /* nodes of the layered circuit, all layers, unary chain nodes incl. */
    int64_t num_edges;        /* edges of the layered circuit = sum over layers of |S_l|           */
    int64_t dag_nodes;        /* input nodes reachable from the roots                              */
    int64_t dag_edges;        /* their child edges                                                 */
    int64_t num_pad_nodes;    /* unary chain nodes inserted by layerization                        */
    int64_t max_layer_nodes;
    int64_t max_fan_in;
    int64_t max_fan_out;
    int64_t num_split_rows;   /* rows (forward) and columns (backward) evaluated by split passes   */
    int64_t index_bytes;      /* device bytes held by index arrays                                 */
    int64_t tail_first_layer; /* first layer that may run in the persistent top-of-circuit kernel
                                 (0: none); the layers actually taken depend on the batch size       */
    int64_t num_merged_nodes; /* input gates identified with a structurally identical gate          */
    int64_t alias_top_layer;  /* A: the layers 1 .. A are padding-free (see klay_options.unary_chains)  */
    int64_t num_fused_rows;   /* AND rows that the fused plans do not evaluate (see klay_options.no_fusion) */
} klay_info_t;

/* Per-kernel-class timing of the most recent forward / backward call, filled only while
 * profiling is enabled.  Durations come from HIP events recorded on the caller's stream around
 * every single launch.  FWD_x / BWD_x are the main-row launches of a layer (one kernel each:
 * the streaming kernel for B > 32), SPLIT the segment launches of split rows, COMBINE their
 * combine launches, MAIN_COMBINE (any operation) the launches that take the main rows and the combine
 * rows of a layer together (32 < B <= 64, where the segments run in a launch of their own first),
 * FWD_OR_FUSED the forward launches of OR layers that read the children of fused AND rows (klay_options.no_fusion),
 * PROD_EDGES the per-parent pass of the real-semiring reverse sweep over a product layer (adjoint
 * times the product of the non-zero children, in place), BWD_PROD the by-child pass that follows
 * it, BWD_SUM_MUL / BWD_PROD_MUL the passes into a product layer, whose rows leave multiplied by
 * the nodes' own values (so that PROD_EDGES only has to repair columns whose value is zero).
 * Log-semiring reverse sweep: BWD_SOFTMAX_ONE is the step through an OR layer that gathers one
 * row per edge, BWD_SUM_ENC the step through an AND layer that leaves the adjoints of the OR layer
 * below in the form that step reads; BWD_SOFTMAX, the two-gather step, only runs where that form
 * cannot be used. */
enum { KLAY_K_LEAF = 0, KLAY_K_FWD_SUM, KLAY_K_FWD_PROD, KLAY_K_FWD_LSE, KLAY_K_ROOT,
       KLAY_K_SEED, KLAY_K_BWD_SUM, KLAY_K_BWD_SOFTMAX, KLAY_K_BWD_LEAF, KLAY_K_TAIL_FWD,
       KLAY_K_TAIL_BWD, KLAY_K_SPLIT, KLAY_K_PROD_EDGES, KLAY_K_FWD_MAX, KLAY_K_BWD_SUM_ENC,
       KLAY_K_BWD_SOFTMAX_ONE, KLAY_K_BWD_PROD, KLAY_K_BWD_SUM_MUL, KLAY_K_BWD_PROD_MUL,
       KLAY_K_COMBINE, KLAY_K_MAIN_COMBINE, KLAY_K_FWD_OR_FUSED, KLAY_K_COUNT };
typedef struct klay_profile_t {
    float   ms[KLAY_K_COUNT];          /* summed device time of the class's launches       */
    int32_t launches[KLAY_K_COUNT];
    double  alg_bytes[KLAY_K_COUNT];   /* algorithmic bytes moved by those launches (no-reuse model:
                                          every index entry gathers its row from memory)             */
    double  min_bytes[KLAY_K_COUNT];   /* compulsory bytes of those launches: every distinct source row
                                          read once, every output row written once, plus the indices */
} klay_profile_t;

/*
 * klay_build -- layerize and tensorize a circuit (Section 3.1 Eq. 2, Section 3.2, Alg. 2, Alg. 3)
 * and upload the per-layer index arrays.
 *
 *   num_vars      V; literals name variables 0..V-1
 *   num_nodes     number of nodes of the input DAG
 *   node_type     host [num_nodes], KLAY_LIT .. KLAY_FALSE
 *   node_lit      host [num_nodes]; for KLAY_LIT +(v+1) (positive) or -(v+1) (negated), else ignored
 *   child_ptr     host [num_nodes+1]; children of node i are child_idx[child_ptr[i] .. child_ptr[i+1])
 *   child_idx     host [child_ptr[num_nodes]] node ids, in any order
 *   num_roots, roots   host [num_roots] node ids; out[:, r] of klay_forward is roots[r]'s value
 *   device        HIP device ordinal, or -1 for a host-only handle (layerization only: the
 *                 inspection calls work, forward/backward return KLAY_ESTATE)
 *   out           receives the handle
 *
 * All arrays are borrowed for the duration of the call only.  Nodes not reachable from a root
 * are dropped.  Leaves carrying the same literal and gates with the same type and the same
 * children are identified bottom-up (Section 3.2, Eq. 3, Theorem 1; child lists are compared on
 * a hash hit, so a collision never merges different gates); values are unchanged by it.  Gates of the wrong parity for their height (an OR directly over leaves, an AND
 * under an AND) are lifted one layer so that odd layers hold AND and even layers OR (Section 3.1).
 * Layer-skipping edges get one chain of unary nodes per (child, layer); all roots are extended to
 * the height of the tallest (Section 3.2).
 * Errors: KLAY_EINVAL (bad sizes, index or literal out of range, a gate without children, a gate of the
 * circuit that lists the same node id twice, a leaf with children, no roots), KLAY_ECYCLE, KLAY_ENOMEM,
 * KLAY_EHIP.  Two different leaf nodes with the same literal under one gate, or two gates that turn out
 * identical, are two children and count twice (Eq. 1).
 */
klay_status klay_build(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type,
                       const int32_t* node_lit, const int64_t* child_ptr, const int32_t* child_idx,
                       int32_t num_roots, const int32_t* roots, int32_t device, klay_circuit** out);

/* Same with explicit options (opts may be NULL). */
klay_status klay_build_ex(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type,
                          const int32_t* node_lit, const int64_t* child_ptr, const int32_t* child_idx,
                          int32_t num_roots, const int32_t* roots, int32_t device,
                          const klay_options* opts, klay_circuit** out);

/*
 * klay_forward -- evaluate all layers (Alg. 1 for KLAY_REAL, Alg. 4 for KLAY_LOG).
 *   leaf_weights  device [B, V] row-major fp32: p_v (REAL) or log p_v (LOG, MAXLOG).  The negated literal
 *                 of v gets 1 - p_v resp. log(1 - exp(x_v)).
 *   B             batch size >= 1
 *   out           device [B, R] row-major fp32; out[b, r] = value of roots[r] on sample b
 *   stream        hipStream_t (as void*), may be NULL for the default stream
 * Keeps the layers' values in the workspace for klay_backward (all but those of fused AND rows, which
 * klay_backward then evaluates itself: see klay_options.no_fusion).  Grows the library-owned
 * workspace (hipMalloc, which synchronises) when B exceeds what earlier calls needed, unless a
 * caller workspace was set.  Errors: KLAY_EINVAL, KLAY_ENOMEM, KLAY_EHIP, KLAY_ESTATE.
 */
klay_status klay_forward(klay_circuit* c, const float* leaf_weights, int32_t B, float* out,
                         klay_semiring semiring, void* stream);

/*
 * klay_forward_static -- klay_forward for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same results as
 * klay_forward, but the layer values, the partial rows of split rows and the transposed leaf weights
 * live in a fixed array in device memory that is part of the library image (KLAY_STATIC_WORKSPACE_BYTES
 * per GPU, held until the process ends) instead of the handle's workspace.  The call allocates
 * nothing (no hipMalloc / hipFree, no events: profiling is not recorded) and only enqueues kernels.
 *   - A circuit / batch size whose forward workspace, klay_workspace_bytes(c, B, 0), exceeds
 *     KLAY_STATIC_WORKSPACE_BYTES is refused with KLAY_ENOMEM before anything is launched.
 *   - Forward only: nothing is kept for klay_backward, and the handle's own state (a previous
 *     klay_forward that is still to be differentiated) is left untouched.
 *   - All handles on one GPU share the one array: calls that overlap in time on the same GPU (two
 *     streams, two threads, two handles) race.  Calls on one stream are ordered and safe; nothing in
 *     the array has to survive from one call to the next, and nothing is assumed to start at zero.
 * Errors: as klay_forward.
 */
#define KLAY_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
klay_status klay_forward_static(klay_circuit* c, const float* leaf_weights, int32_t B, float* out,
                                klay_semiring semiring, void* stream);

/*
 * klay_backward -- reverse-mode derivative of the most recent klay_forward on this handle
 * (the paper obtains it from autograd, Section 6; here it is a reverse sweep over the layers).
 *   dout          device [B, R] fp32, adjoint of `out`
 *   dleaf         device [B, V] fp32, receives sum_r dout[b,r] * d out[b,r] / d leaf_weights[b,v];
 *                 every entry is written (0 for variables the circuit does not use)
 * Uses B, the semiring and the activations of that forward call; the caller must not have run
 * another forward in between.  The first real-semiring call on a handle uploads extra index
 * arrays (hipMalloc, which synchronises); later calls only enqueue.
 * MAXLOG is not differentiated (KLAY_EINVAL).  A literal whose adjoint is exactly 0 contributes 0 even where the
 * derivative of its weight is infinite (log-domain negated literal at p = 1).
 * Errors: KLAY_ESTATE if no forward was run, KLAY_EINVAL, KLAY_EHIP.
 */
klay_status klay_backward(klay_circuit* c, const float* dout, float* dleaf, void* stream);

/*
 * klay_forward_lits / klay_backward_lits -- the same two passes with weights of their own for the
 * negated literals (weighted model counting with arbitrary literal weights, Section 2: every leaf
 * of the arithmetic circuit carries a weight).
 *   pos_weights   device [B, V]: weight of literal v (probability, or its log in the log-domain semirings)
 *   neg_weights   device [B, V]: weight of literal -v, same domain; NULL makes the call klay_forward
 *   dpos, dneg    device [B, V]: adjoints of the two arrays, treated as independent inputs; dneg may
 *                 be NULL when only dpos is wanted.  Every entry is written.
 * A forward pass with neg_weights must be differentiated by klay_backward_lits and one without by
 * klay_backward (KLAY_ESTATE otherwise).  Everything else is as for klay_forward / klay_backward.
 */
klay_status klay_forward_lits(klay_circuit* c, const float* pos_weights, const float* neg_weights, int32_t B,
                              float* out, klay_semiring semiring, void* stream);
klay_status klay_backward_lits(klay_circuit* c, const float* dout, float* dpos, float* dneg, void* stream);

/*
 * klay_forward_f64 / klay_backward_f64 -- the same evaluation in double precision, for circuits whose
 * log-values outgrow what fp32 resolves and as an on-device accuracy reference for the fp32 kernels.
 * Same launch plans, a plain (untuned) gather-reduce kernel, the full-precision exp / log.
 *   pos_weights, neg_weights, out, dout, dpos, dneg   as for klay_forward_lits / klay_backward_lits,
 *                 in double; neg_weights = NULL derives the negated literals from pos_weights, and
 *                 dneg must then be NULL as well.
 * All three semirings are evaluated; KLAY_LOG and KLAY_REAL are differentiated (KLAY_MAXLOG is not:
 * KLAY_EINVAL).  In double the real semiring reaches circuits whose values underflow fp32.
 * The activations live in a library-owned workspace of their own (klay_set_workspace and
 * klay_workspace_bytes do not cover it) and are independent of the fp32 state: a handle can hold
 * one fp32 and one double-precision forward pass at the same time.  Profiling does not cover
 * these calls.
 */
klay_status klay_forward_f64(klay_circuit* c, const double* pos_weights, const double* neg_weights, int32_t B,
                             double* out, klay_semiring semiring, void* stream);
klay_status klay_backward_f64(klay_circuit* c, const double* dout, double* dpos, double* dneg, void* stream);

/* Structure of the layered circuit. */
klay_status klay_info(const klay_circuit* c, klay_info_t* info);

/* nodes[l], edges[l] for l = 0..L (host arrays of num_layers+1 entries; edges[0] = 0). */
klay_status klay_layer_sizes(const klay_circuit* c, int64_t* nodes, int64_t* edges);

/*
 * Host copy of layer l's index vectors (Section 4 / Alg. 3), 1 <= l <= L, in CSR form:
 * row_ptr [n_l + 1], child [e_l].  child is the paper's S_l (position in layer l-1); the paper's
 * R_l is row_ptr expanded (edge j belongs to parent r iff row_ptr[r] <= j < row_ptr[r+1]).
 * For l <= klay_info_t.alias_top_layer child holds rows of the whole activation buffer instead
 * (the rows of layer 0, then those of layer 1, ...), always of a layer below l.
 */
klay_status klay_layer_csr(const klay_circuit* c, int32_t layer, int64_t* row_ptr, int32_t* child);

/*
 * Host copy of what each node of layer l (0 <= l <= L) stands for: origin[i] is the input node id
 * whose value row i holds (for a unary chain node: the id of the node the chain starts from),
 * is_pad[i] is 1 for chain nodes.
 */
klay_status klay_layer_nodes(const klay_circuit* c, int32_t layer, int32_t* origin, uint8_t* is_pad);

/*
 * position[r] (host array of num_roots entries) = row of the top layer L that holds roots[r]'s value
 * (Section 3.2: all roots sit in the last layer, a root of lower height through a stand-in).
 */
klay_status klay_root_positions(const klay_circuit* c, int32_t* position);

/* Bytes of device workspace a forward (and, if need_backward, backward) call with batch B needs.  A handle built
 * with device = -1 answers for a device that grants a workgroup the whole 160 KB LDS of a compute unit (the
 * persistent kernels' buffers depend on which layers fit). */
size_t klay_workspace_bytes(const klay_circuit* c, int32_t B, int need_backward);

/* Use caller device memory (256-byte aligned) as workspace instead of library-owned memory;
 * dev_ptr = NULL returns to library-owned memory.  The caller keeps ownership. */
klay_status klay_set_workspace(klay_circuit* c, void* dev_ptr, size_t bytes);

/* Enable (1) / disable (0) per-kernel-class event timing; klay_get_profile synchronises on the
 * recorded events and returns the figures of the most recent forward and backward calls. */
klay_status klay_set_profiling(klay_circuit* c, int32_t enable);
klay_status klay_get_profile(klay_circuit* c, klay_profile_t* profile);

/*
 * Incremental construction of a multi-rooted circuit (Section 3.2: circuits that share variables
 * are merged into one layered circuit, one after the other, and share every node they have in
 * common).  A builder collects circuits; klay_builder_finish layerizes all of them together, so
 * identical sub-circuits of different circuits become one set of rows and all roots reach the
 * height of the tallest circuit.
 *
 *   klay_builder_create   num_vars = V of the leaf-weight array all circuits are evaluated on.
 *   klay_builder_add      same arrays as klay_build (node ids are local to this circuit; borrowed
 *                         for the call).  first_root (may be NULL) receives the column of `out`
 *                         that this circuit's roots[0] will occupy; its roots take consecutive
 *                         columns, circuits in the order they were added.  Range errors are
 *                         reported here (KLAY_EINVAL) and leave the builder unchanged; structural
 *                         errors (cycle, empty gate, repeated child) are reported by finish.
 *   klay_builder_finish   layerize what has been added so far (as klay_build_ex).  The builder
 *                         stays valid: more circuits may be added and finish called again, each
 *                         call returning an independent handle.  KLAY_ESTATE if nothing was added.
 *   klay_builder_destroy  NULL is allowed.
 */
typedef struct klay_builder klay_builder;
klay_status klay_builder_create(int32_t num_vars, klay_builder** out);
klay_status klay_builder_add(klay_builder* b, int64_t num_nodes, const uint8_t* node_type,
                             const int32_t* node_lit, const int64_t* child_ptr, const int32_t* child_idx,
                             int32_t num_roots, const int32_t* roots, int32_t* first_root);
klay_status klay_builder_finish(const klay_builder* b, int32_t device, const klay_options* opts,
                                klay_circuit** out);
void klay_builder_destroy(klay_builder* b);

/* Frees index arrays and library-owned workspace.  NULL is allowed. */
void klay_destroy(klay_circuit* c);

/* Message of the last failing call on this thread ("" if none). */
const char* klay_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KLAY_H */
