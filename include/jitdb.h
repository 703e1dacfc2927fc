/*
 * jitdb - level-batched Child-Sum Tree-LSTM forward for MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of "Just-in-Time Dynamic-Batching"
 * (arXiv 1904.07421).  The paper collects the computation graphs of a batch of
 * samples, files every node in a look-up table by its depth in the computation
 * graph (section 4.2), and then visits the table in depth order, running all
 * nodes of one slot as a single batched launch: stack, execute, slice
 * (section 4.3).  Here the samples are trees, the node type is one Tree-LSTM
 * cell (section 3), and the two calls are the two halves of that method:
 *
 *   jitdb_schedule           the analysis: depth table, slot order, child lists
 *   jitdb_treelstm_forward   the execution: one batched cell evaluation per depth
 *
 * Around them: jitdb_schedule_append (trees that arrive later join a table), jitdb_forest_fingerprint
 * and jitdb_cache_* (a cache of tables keyed by the parent array), jitdb_schedule_typed and
 * jitdb_treelstm_forward_typed (the table keyed by depth and signature, one cell per signature),
 * jitdb_treelstm_pack and jitdb_treelstm_forward_packed (weights packed once for many calls),
 * jitdb_treelstm_forward_train and jitdb_treelstm_backward (the training step).
 *
 * Conventions
 *   - Every function returns JITDB_OK (0) or a negative jitdb_status.  Nothing
 *     throws, exits or prints (a failed host-side allocation comes back as JITDB_E_NOMEM).
 *   - "dev" pointers are device (HBM) memory of the current HIP device, owned
 *     by the caller; "host" pointers are ordinary host memory.  The library
 *     allocates no device memory (jitdb_cache_create allocates a small host-side table, and the
 *     profiling calls create HIP events): scratch comes from caller-supplied workspaces whose
 *     sizes the *_workspace_bytes queries return.  Workspaces must be 256-byte
 *     aligned.  Nothing is retained after a call returns except what was
 *     written into caller buffers.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - A forest is ONE parent array over global node ids 0..N-1; parent -1 marks
 *     a root.  Ids are arbitrary: parent[v] < v is NOT required and trees need
 *     not be contiguous.
 */
#ifndef JITDB_H
#define JITDB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    JITDB_OK = 0,
    JITDB_E_NULL = -1,         /* a required pointer is NULL */
    JITDB_E_BADARG = -2,       /* size, dimension, dtype or alignment out of range */
    JITDB_E_PARENT_RANGE = -3, /* some parent[v] is < -1, >= N, or == v */
    JITDB_E_CYCLE = -4,        /* some node never reaches a root */
    JITDB_E_WORKSPACE = -5,    /* workspace smaller than the matching *_workspace_bytes */
    JITDB_E_HIP = -6,          /* a HIP runtime call failed */
    JITDB_E_SCHEDULE = -7,     /* forward was handed a schedule that is not complete */
    JITDB_E_SIGNATURE = -8,    /* a signature is outside [0, n_sig) */
    JITDB_E_NOMEM = -9,        /* a host-side allocation failed (launch list, cache table, profiling events) */
    JITDB_E_ARITY = -10        /* a node has more children than its (N-ary) cell has child positions */
} jitdb_status;

typedef enum {
    JITDB_F32 = 0,  /* x, W, U, h in fp32; fp32 MFMA */
    JITDB_BF16 = 1  /* x, W, U, h in bfloat16; bf16 MFMA with fp32 accumulate; b, c in fp32 */
} jitdb_dtype;

/* Largest forest one call accepts (ids and offsets are int32 with headroom). */
#define JITDB_MAX_NODES (1 << 28)
/* Most signatures one table distinguishes; also N * n_sig^2 must stay below 2^31. */
#define JITDB_MAX_SIGNATURES 64

/*
 * The schedule of a forest: the paper's depth-keyed table (section 4.2),
 * specialised to one node type, in flat arrays.
 *
 * "Depth" is the depth in the COMPUTATION graph: a node can run once all its
 * inputs (its children) have run, so depth = height in the tree, 0 for leaves,
 * 1 + max over children otherwise.  Nodes of equal height are independent and
 * form one level batch.  The order inside a slot and among children, which the
 * paper leaves open, is fixed as ascending node id so that the result is unique.
 *
 * The caller fills n_nodes and all pointers before jitdb_schedule; the call
 * fills the arrays, n_levels and n_edges.
 */
typedef struct {
    int64_t n_nodes;         /* in: N, 0 <= N <= JITDB_MAX_NODES */
    int32_t *height;         /* dev [N]   out: height of every node */
    int32_t *level_ptr;      /* dev [N+1] out: entries 0..n_levels valid; level l = positions
                                          [level_ptr[l], level_ptr[l+1]) */
    int32_t *perm;           /* dev [N]   out: position -> node id, sorted by (height, id) */
    int32_t *inv_perm;       /* dev [N]   out: node id -> position */
    int32_t *child_ptr;      /* dev [N+1] out: children of node j are child_idx[child_ptr[j] .. child_ptr[j+1]) */
    int32_t *child_idx;      /* dev [N]   out: entries 0..n_edges valid, child ids ascending per parent */
    int32_t *host_level_ptr; /* host [N+1] out: copy of level_ptr[0..n_levels]; the forward sizes
                                          its per-level launches from it */
    int32_t n_levels;        /* out: L = 1 + max height (0 if N == 0) */
    int64_t n_edges;         /* out: E = N - number of roots */
    int32_t *host_level_kids; /* host [N+1] or NULL, out: entry l < n_levels = number of children of the nodes of
                                          level l (0 for level 0), -1 = not known.  Optional: with it the forward
                                          recognises levels in which every node has exactly one child (chains:
                                          sequences, the thin tail of a forest) and runs each as a single launch */
} jitdb_schedule_t;

/* Bytes of device workspace jitdb_schedule needs for a forest of n_nodes (0 if n_nodes is invalid). */
size_t jitdb_schedule_workspace_bytes(int64_t n_nodes);

/*
 * Analysis step (section 4.2: organise the nodes by depth; section 4.3: nodes
 * that can be batched together share a slot).
 *
 *   parent  dev [N] int32, -1 = root.
 *   s       in/out, see jitdb_schedule_t.
 *
 * Runs on `hip_stream` and synchronises that stream twice (to learn the number
 * of levels, then to hand back level_ptr).  On JITDB_E_PARENT_RANGE or
 * JITDB_E_CYCLE the output arrays hold unspecified values; no kernel reads or
 * writes out of bounds for any input.  N == 0 succeeds with n_levels = 0.
 * The schedule depends only on `parent` and may be reused for any number of
 * forward calls (the paper's cached graph rewrite, section 4.3).
 */
int jitdb_schedule(const int32_t *parent, jitdb_schedule_t *s,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace jitdb_schedule_append needs (0 if an argument is invalid). */
size_t jitdb_schedule_append_workspace_bytes(int64_t n_base, int64_t n_new);

/*
 * Incremental analysis: trees that arrive while earlier work is still executing (the
 * serving case of section 2) are appended to a forest that has a schedule already, at
 * the cost of analysing the new trees only.
 *
 *   base        a complete schedule of a forest of N_a nodes (N_a == 0 allowed; then only
 *               n_nodes and host_level_ptr need to be set).  Read, not changed.
 *   parent_new  dev [n_new] int32, the arriving trees with ids local to them (0 .. n_new-1,
 *               -1 = root); node v becomes node N_a + v of the joint forest.
 *   out         in/out like jitdb_schedule_t in jitdb_schedule, n_nodes == N_a + n_new and
 *               every array sized for it; must not share memory with base.
 *
 * `out` receives exactly what jitdb_schedule returns for the concatenated parent array
 * (the old parents followed by parent_new[v] + N_a): new ids sort after the old ones inside
 * every level, and trees share no nodes, so the old level segments and child lists are
 * kept and shifted (one linear pass) instead of being sorted again.  Errors in
 * parent_new are reported as by jitdb_schedule.  Synchronises the stream as often as
 * jitdb_schedule does for the new part; the merge itself is asynchronous on the stream.
 */
int jitdb_schedule_append(const jitdb_schedule_t *base, const int32_t *parent_new, int64_t n_new,
                          jitdb_schedule_t *out, void *workspace, size_t workspace_bytes,
                          void *hip_stream);

/*
 * Schedule cache (the paper keeps the rewritten graph and reuses it when the same structure
 * returns, section 4.3).  The key is a 128-bit fingerprint of the parent array plus N:
 *
 *     word_i = i * 2^32 + (parent[i] mod 2^32)
 *     fp[0]  = sum_i mix64(word_i + 0x9E3779B97F4A7C15)   mod 2^64
 *     fp[1]  = sum_i mix64(word_i xor 0xD1B54A32D192ED03) mod 2^64
 *
 * with mix64 the output function of SplitMix64.  Two different forests of equal size share a
 * key with probability about 2^-128; a caller that cannot accept that compares the parent
 * arrays on a hit.
 *
 *   parent    dev [n_nodes] int32 (any values: the fingerprint does not validate the forest)
 *   fp_dev    dev [2] uint64, written by the kernels
 *   fp_host   host [2] uint64 or NULL.  If given, the result is copied there and the stream is
 *             synchronised once; if NULL the call is asynchronous.
 */
int jitdb_forest_fingerprint(const int32_t *parent, int64_t n_nodes, uint64_t *fp_dev,
                             uint64_t *fp_host, void *hip_stream);

/*
 * The table of the cache, host side only (no GPU call): it maps a key to one of `capacity`
 * slots; the caller keeps the schedule objects, slot by slot, and owns their memory.
 * Thread-safe.  Replacement: least recently used, a successful lookup counts as a use.
 *
 *   jitdb_cache_lookup   slot of the key, or -1 (also for NULL arguments)
 *   jitdb_cache_insert   slot now assigned to the key: the key's own if present, else the
 *                        lowest unused slot, else the slot of the least recently used key,
 *                        which is dropped (*evicted = 1; evicted may be NULL); -1 for NULL
 *                        arguments or when the host is out of memory (the table is unchanged)
 *   jitdb_cache_stats    counts of lookups that hit / missed and of keys held (NULLs skipped)
 */
typedef struct jitdb_cache jitdb_cache_t;
int jitdb_cache_create(int32_t capacity, jitdb_cache_t **out);   /* capacity in [1, 2^20] */
void jitdb_cache_destroy(jitdb_cache_t *cache);
int32_t jitdb_cache_lookup(jitdb_cache_t *cache, const uint64_t *fp, int64_t n_nodes);
int32_t jitdb_cache_insert(jitdb_cache_t *cache, const uint64_t *fp, int64_t n_nodes, int32_t *evicted);
void jitdb_cache_stats(const jitdb_cache_t *cache, int64_t *hits, int64_t *misses, int32_t *entries);

/*
 * The generic table (sections 4.2 and 4.3): the paper files every node under a key made of its
 * depth and of what must agree for two nodes to run as one batch: operator type, settings,
 * input layouts.  Here the caller folds those into one integer per node, the signature, and
 * each signature names one cell (one weight set).  A node takes part in two batched operations
 * with different partners: its own cell, shared with the nodes of its (height, signature), and
 * the forget projection that its PARENT's cell applies to it, shared with the nodes of its
 * (height, parent's signature).  Nodes are therefore filed by (height, sig, psig), psig being the
 * parent's signature (a root: its own): sub-slot (l, t, p) is the batch of one projection, and
 * slot (l, t), the batch of one cell, is the run of its n_sig sub-slots.
 *
 *   n_sig          in: number of signatures, 1 .. JITDB_MAX_SIGNATURES, N * n_sig^2 < 2^31
 *   slot_capacity  in: entries slot_ptr and host_slot_ptr have room for; n_levels * n_sig^2 + 1
 *                  are needed (N * n_sig^2 + 1 always suffices), else JITDB_E_WORKSPACE
 *   key            dev [N] out: (height * n_sig + sig) * n_sig + psig
 *   slot_ptr       dev out: sub-slot (l, t, p) = positions slot_ptr[q] .. slot_ptr[q + 1] of perm,
 *                  q = (l * n_sig + t) * n_sig + p; empty ones allowed;
 *                  level_ptr[l] == slot_ptr[l * n_sig^2]
 *   host_slot_ptr  host copy of slot_ptr, filled before the call returns
 */
typedef struct jitdb_slots {
    int32_t n_sig;
    int64_t slot_capacity;
    int32_t *key;
    int32_t *slot_ptr;
    int32_t *host_slot_ptr;
} jitdb_slots_t;

/* Bytes of device workspace jitdb_schedule_typed needs (0 if an argument is invalid). */
size_t jitdb_schedule_typed_workspace_bytes(int64_t n_nodes, int32_t n_sig);

/*
 * jitdb_schedule with the second key.  `sig` is dev [N] int32, any value in [0, n_sig) per node.
 * `s` receives what jitdb_schedule returns except that positions are ordered by
 * (height, sig, psig, id), so every level is a run of n_sig slots of n_sig sub-slots each;
 * `slots` receives the boundaries.  Errors as jitdb_schedule, plus JITDB_E_SIGNATURE.
 * Synchronises the stream twice.
 */
int jitdb_schedule_typed(const int32_t *parent, const int32_t *sig, jitdb_schedule_t *s,
                         jitdb_slots_t *slots, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/* Bytes of device workspace jitdb_treelstm_forward_typed needs (0 if an argument is invalid). */
size_t jitdb_treelstm_typed_workspace_bytes(int64_t n_nodes, int64_t n_edges,
                                            int32_t D, int32_t H, jitdb_dtype dtype, int32_t n_sig);

/*
 * jitdb_treelstm_forward over a typed table: W is dev [n_sig, 4H, D], U dev [n_sig, 4H, H],
 * b dev [n_sig, 4H]; node j is evaluated by cell sig[j], including the forget gates it applies
 * to its children.  One batched evaluation per non-empty slot, levels in ascending order; a
 * slot's steps are those of a level in jitdb_treelstm_forward (stack, gate GEMM + cell update
 * with the slot's weights; forget projection per sub-slot with the parent cell's weights); the
 * slots of a large level share one grouped launch per step.
 * `s` and `slots` come from jitdb_schedule_typed (slot_ptr is read on the device).
 */
int jitdb_treelstm_forward_typed(const void *x, const void *W, const void *U, const float *b,
                                 int32_t D, int32_t H, jitdb_dtype dtype,
                                 const jitdb_schedule_t *s, const jitdb_slots_t *slots,
                                 void *h_out, float *c_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * A table whose signatures name cells of different operator TYPE (the paper's key holds the operator
 * type and its settings next to the depth, sections 4.2 and 4.3: nodes of different type never share
 * a slot).  Two types:
 *
 *   JITDB_CELL_CHILDSUM  the cell of jitdb_treelstm_forward: W [4H, D], U [4H, H], b [4H], gate rows
 *                        i, o, u, f; any number of children.
 *   JITDB_CELL_NARY      the N-ary Tree-LSTM cell of the model the paper cites, `arity` = N child positions,
 *                        1 <= N <= JITDB_MAX_NARY.  Children are taken in ascending node id (position 1,
 *                        2, ...); with hc = [h of child 1 ; ... ; h of child N] (zero blocks for missing ones)
 *                            i, o = sigmoid(W x + U hc + b)   u = tanh(W x + U hc + b)
 *                            f_l  = sigmoid(W_{f_l} x + U_{f_l} hc + b_{f_l})      l = 1..N
 *                            c    = i*u + sum over present children l of f_l * c_l   h = o * tanh(c)
 *                        W [(3+N)H, D], U [(3+N)H, N*H] (column block l multiplies the child in position l),
 *                        b [(3+N)H], gate rows i, o, u, f_1, ..., f_N.
 *
 * All cells share D, H and the dtype.  Cells may differ freely along edges (a child-sum parent applies
 * its own forget weights to the h of an N-ary child and vice versa).  `cells` is a HOST array of n_sig
 * entries whose W, U, b are device pointers; `s`, `slots` come from jitdb_schedule_typed with the same
 * n_sig.  Child-sum slots run as in jitdb_treelstm_forward_typed; an N-ary slot is one stack step, one
 * contraction for all its 3 + N gates and one cell update.
 *
 * Asynchronous like jitdb_treelstm_forward_typed unless the table holds an N-ary cell: then the call
 * waits for the stream once at its end and returns JITDB_E_ARITY if some node under an N-ary cell has more
 * than N children (its surplus children were left out; h_out, c_out are then not to be used).
 */
typedef enum { JITDB_CELL_CHILDSUM = 0, JITDB_CELL_NARY = 1 } jitdb_cell_kind;
#define JITDB_MAX_NARY 4
typedef struct jitdb_cell {
    int32_t kind;      /* jitdb_cell_kind */
    int32_t arity;     /* JITDB_CELL_NARY: N; ignored for JITDB_CELL_CHILDSUM */
    const void *W;     /* dev, dtype elements */
    const void *U;     /* dev, dtype elements */
    const float *b;    /* dev, fp32 */
} jitdb_cell_t;
size_t jitdb_treelstm_cells_workspace_bytes(int64_t n_nodes, int64_t n_edges, int32_t D, int32_t H,
                                            jitdb_dtype dtype, const jitdb_cell_t *cells, int32_t n_sig);
int jitdb_treelstm_forward_cells(const void *x, const jitdb_cell_t *cells, int32_t n_sig,
                                 int32_t D, int32_t H, jitdb_dtype dtype,
                                 const jitdb_schedule_t *s, const jitdb_slots_t *slots,
                                 void *h_out, float *c_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace jitdb_treelstm_forward needs (0 if an argument is invalid). */
size_t jitdb_treelstm_workspace_bytes(int64_t n_nodes, int64_t n_edges,
                                      int32_t D, int32_t H, jitdb_dtype dtype);

/*
 * Execution step (section 4.3: per slot, stack the samples on the batch axis,
 * run the common subgraph once, slice the outputs back), for the Child-Sum
 * Tree-LSTM cell the paper analyses in section 3 (33 operators, 4 of which
 * depend on the number of children).  For node j with children C(j):
 *
 *     hs  = sum_{k in C(j)} h_k
 *     i   = sigmoid(W_i x_j + U_i hs + b_i)      o = sigmoid(W_o x_j + U_o hs + b_o)
 *     u   = tanh   (W_u x_j + U_u hs + b_u)
 *     f_k = sigmoid(W_f x_j + U_f h_k + b_f)     (one per child, from that child's h)
 *     c_j = i*u + sum_k f_k*c_k                  h_j = o*tanh(c_j)
 *
 *   x      dev [N, D] row-major, row = node id.          dtype elements
 *   W      dev [4H, D] row-major, gate rows i, o, u, f.  dtype elements
 *   U      dev [4H, H] row-major, same gate order.       dtype elements
 *   b      dev [4H] fp32 (both dtypes).
 *   s      a schedule produced by jitdb_schedule for the same forest.
 *   h_out  dev [N, H] row-major, row = node id.          dtype elements
 *   c_out  dev [N, H] row-major, row = node id.          fp32 (both dtypes)
 *
 * D >= 1, H >= 1 (any values; rows are padded internally; D % 4 == 0 takes the fast
 * row copy); x, h_out and c_out 16-byte aligned.  With
 * JITDB_BF16, h is rounded to bfloat16 (nearest even) when stored and that
 * rounded value feeds the parents; sums, gates and c stay fp32.
 *
 * Fully asynchronous on `hip_stream`: level sizes come from s->host_level_ptr,
 * no device-to-host copy or synchronisation happens.  Levels run in order on
 * that one stream.  N == 0 succeeds and launches nothing.
 *
 * If s->host_level_kids is set, the run of top levels in which every node has
 * exactly one child (kids == nodes of the level; sequences, thin tails) takes
 * one launch per level that reads x and the child's h, c in place; the results
 * agree with the general launches within rounding (the forget gate's two
 * products are then summed in one accumulator).  Without it every level takes
 * the general launches.
 */
int jitdb_treelstm_forward(const void *x, const void *W, const void *U, const float *b,
                           int32_t D, int32_t H, jitdb_dtype dtype,
                           const jitdb_schedule_t *s,
                           void *h_out, float *c_out,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * jitdb_treelstm_forward for callers that cannot allocate device memory and so have no workspace
 * to pass: code recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and errors as jitdb_treelstm_forward, without the workspace: the scratch
 * memory is a fixed array of JITDB_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held
 * from the moment the library's code is loaded on that GPU until the process ends.  The call
 * allocates and frees nothing on the device (no hipMalloc, no hipFree, no library that does).
 *
 *   - Forests whose jitdb_treelstm_workspace_bytes exceeds JITDB_STATIC_SCRATCH_BYTES are refused
 *     with JITDB_E_WORKSPACE and nothing is launched (64 MiB: e.g. 25 000 nodes at D = 300, H = 150
 *     in bf16; use jitdb_treelstm_forward with a workspace of your own beyond that).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 *     (different streams, or different host threads) race.  Calls on one stream are ordered and safe.
 *     The array keeps the previous call's contents; the call needs none of it and none of it zeroed.
 *   - The first call on a GPU looks up the array's device address (hipGetSymbolAddress): make one
 *     call outside graph capture before capturing.
 */
#define JITDB_STATIC_SCRATCH_BYTES (64 * 1024 * 1024)
int jitdb_treelstm_forward_static(const void *x, const void *W, const void *U, const float *b,
                                  int32_t D, int32_t H, jitdb_dtype dtype,
                                  const jitdb_schedule_t *s,
                                  void *h_out, float *c_out, void *hip_stream);

/*
 * Weights packed once for many calls.  jitdb_treelstm_forward re-packs W, U, b into the GEMM's
 * operand layout in every call (two short launches; one more per further signature); a serving
 * loop whose weights do not change packs them once and hands the result to
 * jitdb_treelstm_forward_packed, which is jitdb_treelstm_forward (slots == NULL, one cell) or
 * jitdb_treelstm_forward_typed (slots from jitdb_schedule_typed) without that step.
 *
 *   W, U, b   as in jitdb_treelstm_forward_typed: [n_sig, 4H, D], [n_sig, 4H, H], [n_sig, 4H]
 *   packed    dev, 256-byte aligned, jitdb_treelstm_packed_bytes(D, H, dtype, n_sig) bytes; the
 *             layout is private to the library and depends on (D, H, dtype, n_sig)
 * Workspace of the forward call: jitdb_treelstm_typed_workspace_bytes(..., n_sig).  Results
 * equal those of the unpacked calls bit for bit.
 */
size_t jitdb_treelstm_packed_bytes(int32_t D, int32_t H, jitdb_dtype dtype, int32_t n_sig);
int jitdb_treelstm_pack(const void *W, const void *U, const float *b, int32_t D, int32_t H,
                        jitdb_dtype dtype, int32_t n_sig, void *packed, size_t packed_bytes,
                        void *hip_stream);
int jitdb_treelstm_forward_packed(const void *x, const void *packed, int32_t D, int32_t H,
                                  jitdb_dtype dtype, const jitdb_schedule_t *s,
                                  const jitdb_slots_t *slots, void *h_out, float *c_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Execution step for training (the paper runs its backward pass through the same batched
 * graph, section 5): jitdb_treelstm_forward plus the activations a backward pass needs.
 *
 *   gates_out  dev [N, 3H] in dtype elements (like h), rows by node id: i | o | u after their
 *              non-linearities.
 *   fgate_out  dev [N, H] in dtype elements: row k = the forget gate f_k the parent of node k
 *              applied to it; rows of roots are not written.
 * With JITDB_BF16 the kept activations are bfloat16 (the usual mixed-precision choice: they are
 * values in [-1, 1], the cell state c stays fp32); this halves what the training step moves for them.
 * Everything else as in jitdb_treelstm_forward (same workspace size, same results).
 */
int jitdb_treelstm_forward_train(const void *x, const void *W, const void *U, const float *b,
                                 int32_t D, int32_t H, jitdb_dtype dtype,
                                 const jitdb_schedule_t *s,
                                 void *h_out, float *c_out, void *gates_out, void *fgate_out,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of device workspace jitdb_treelstm_backward needs for this schedule (0 if an argument is invalid). */
size_t jitdb_treelstm_backward_workspace_bytes(const jitdb_schedule_t *s, int32_t D, int32_t H,
                                               jitdb_dtype dtype);

/*
 * Backward pass of the execution step (section 5 reports training beside inference; the
 * backward graph is batched by the same table, visited from the roots down).  For the scalar
 *     L = sum_j <gh_j, h_j> + <gc_j, c_j>
 * it returns dL/dx, dL/dW, dL/dU, dL/db of the forward defined at jitdb_treelstm_forward.
 *
 *   x, W, U, s, dtype   as handed to jitdb_treelstm_forward_train.
 *   h, c, gates, fgate  what that call returned (dev; c fp32, the others in dtype elements).
 *   gh, gc              dev [N, H] fp32 cotangents of h and c for every node; either may be NULL (= zeros).
 *   dx [N, D], dW [4H, D], dU [4H, H], db [4H]   dev, fp32, overwritten.
 *
 * With JITDB_BF16 the GEMM operands (gate derivatives, x, h, weights) are bfloat16 and all
 * sums fp32.  Asynchronous on `hip_stream`; N == 0 zeroes dW, dU, db.  x, h and dx 16-byte aligned.
 */
int jitdb_treelstm_backward(const void *x, const void *W, const void *U,
                            int32_t D, int32_t H, jitdb_dtype dtype, const jitdb_schedule_t *s,
                            const void *h, const float *c, const void *gates, const void *fgate,
                            const float *gh, const float *gc,
                            float *dx, float *dW, float *dU, float *db,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Per-kernel timing, for measuring the execution step against the hardware
 * roofline (the paper reports only wall-clock samples/s, section 5; the
 * kernels here are this implementation's own).  Between jitdb_profile_start
 * and jitdb_profile_stop every kernel launch of jitdb_treelstm_forward is
 * bracketed by a pair of HIP events recorded on the call's stream.  The event records keep
 * consecutive kernels from overlapping, so a recorded call runs a few per cent slower (much
 * slower for forests of many thin levels): time throughput without recording.
 *
 *   jitdb_profile_start(capacity)  creates `capacity` event pairs (host objects)
 *                                  and switches recording on; launches beyond the
 *                                  capacity run unrecorded and are counted in `dropped`.
 *   jitdb_profile_stop(out)        waits for the recorded events, adds up the elapsed
 *                                  time and launch count per kernel class, destroys
 *                                  the events and switches recording off.
 *
 * Process-wide state, not thread safe: use from one thread, one stream at a time.
 */
typedef enum {
    JITDB_K_PACK = 0,       /* once per call: weight re-packing, row records */
    JITDB_K_STACK = 1,      /* stack: row = [x_j | sum_k h_k] per level */
    JITDB_K_LEAF = 2,       /* leaf level: W x + cell (tiled kernel) */
    JITDB_K_INTERNAL = 3,   /* internal levels: [x;hs][W;U] + cell with per-child forget gates (tiled kernel) */
    JITDB_K_PROJ = 4,       /* P_k = U_f h_k (tiled kernel) */
    JITDB_K_THIN_LEAF = 5,      /* the same three jobs done by the kernel for small levels */
    JITDB_K_THIN_INTERNAL = 6,
    JITDB_K_THIN_PROJ = 7,      /* includes the next slot's stack step when the two share a launch */
    JITDB_K_CHAIN = 8,          /* a level whose nodes all have one child: gather, all four gates and the cell
                                   update in one launch (no stack step, no projection) */
    JITDB_K_CLASSES = 9
} jitdb_kernel_class;

typedef struct {
    double ms[JITDB_K_CLASSES];        /* summed event time per class, milliseconds */
    int64_t launches[JITDB_K_CLASSES]; /* recorded launches per class */
    int64_t rows[JITDB_K_CLASSES];     /* level rows (nodes) those launches covered; 0 for PACK */
    int64_t edges[JITDB_K_CLASSES];    /* children whose forget projections those launches computed themselves
                                          (CHAIN); 0 for the classes that read them from the projection step */
    int64_t dropped;                   /* launches that found no free event pair */
} jitdb_profile_t;

int jitdb_profile_start(int32_t capacity);
int jitdb_profile_stop(jitdb_profile_t *out);

/*
 * Machine peaks measured on the spot, for quoting kernel rates against what this device
 * sustains as well as against the data sheet (the paper reports wall-clock throughput only,
 * section 5; these calls exist for the benchmark and are not part of the method).
 *
 *   jitdb_probe_copy   times a plain device copy of `bytes` (multiple of 16; src, dst dev,
 *                      16-byte aligned, not overlapping) and returns (read + written) GB/s.
 *   jitdb_probe_mfma   times a loop of independent 32x32 MFMAs of the dtype's kind on every
 *                      CU and returns TFLOP/s; `sink` is dev memory for one float (never
 *                      written in practice).
 *   jitdb_probe_stream the same for other shapes of stream, to find the best the memory system gives:
 *                      `kind` = JITDB_STREAM_COPY (as jitdb_probe_copy), _READ (src only is read;
 *                      GB/s read), _WRITE (dst only is written; GB/s written), _COPY_NT (four
 *                      non-temporal 16-byte loads and stores in flight per thread), _COPY_CHUNK (one
 *                      contiguous chunk per block); copies return (read + written) GB/s.  dst must
 *                      be valid device memory of `bytes` for every kind.
 * All run on `hip_stream` and wait for it.
 */
enum { JITDB_STREAM_COPY = 0, JITDB_STREAM_READ = 1, JITDB_STREAM_WRITE = 2, JITDB_STREAM_COPY_NT = 3,
       JITDB_STREAM_COPY_CHUNK = 4 };
int jitdb_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream, double *gb_per_s);
int jitdb_probe_stream(int kind, const void *src, void *dst, size_t bytes, void *hip_stream, double *gb_per_s);
int jitdb_probe_mfma(jitdb_dtype dtype, float *sink, void *hip_stream, double *tflop_per_s);

/* Static, NUL-terminated description of a status code. */
const char *jitdb_strerror(int code);

/* Text describing the most recent HIP runtime failure behind a JITDB_E_HIP (which call site,
 * which HIP error).  Process-wide, for diagnostics; static storage, never NULL. */
const char *jitdb_last_hip_error(void);

/* Library version, "major.minor". */
const char *jitdb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* JITDB_H */
