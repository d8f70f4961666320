/*
 * acrobat.h - C ABI of the MI355X batched dataflow-graph executor.
 *
 * The library runs the data-parallel hot path of compile-time-assisted auto-batching
 * (paper sections 2.2, 4.1 and 5): a mini-batch of input structures (binary trees or
 * variable-length sequences) is turned into a depth schedule (one batch per depth) and
 * every batch is executed by one gather-fused cell kernel that reads its operands by
 * index from the state arena, runs the dense cell contraction, applies the gate
 * non-linearities and writes the new states back.
 *
 * General rules
 *  - All sizes and indices are int32.  All floating point data is fp32, row-major.
 *  - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory
 *    on the context's GPU.  The caller owns every buffer passed in; the library keeps
 *    no caller pointer after a call returns.
 *  - Host structure arrays are consumed before the call returns.  Device work is
 *    enqueued on the given HIP stream (a hipStream_t passed as void*, NULL = the null
 *    stream) and the call returns without synchronising, unless profiling is on.
 *  - Every function returns ACROBAT_OK (0) or a negative code; nothing is launched
 *    when validation fails.  acrobat_last_error() gives a human readable reason.
 *  - No C++ exception crosses this boundary.
 *  - A context must not be used from two threads at once.
 *  - Throughput: the last levels of a mini-batch are few nodes wide and leave most of the GPU idle.  Two contexts,
 *    each fed on a stream of its own with mini-batches in turn, overlap those levels of one batch with the wide
 *    first levels of the next (measured on tree batches: 1.2 to 1.6 times the single-stream throughput).  The
 *    calls that run as ONE launch whose workgroups wait for each other (see acrobat_set_persistent) do not
 *    overlap one another that way: the library lets them take turns.
 *  - Stream capture (hipStreamBeginCapture on the given stream): a forward call may be recorded
 *    into a HIP graph once an uncaptured call of at least the same sizes has run on the context
 *    (a captured call allocates nothing and waits for nothing; otherwise it fails with
 *    ACROBAT_EINVAL), with profiling off.  The graph's upload node reads the context's staging
 *    buffer at every replay: no other call may use the context until the graph is no longer
 *    replayed.  Capturing and instantiating costs more than a forward call itself, so this pays
 *    only for a mini-batch that is replayed unchanged; the schedule of a new mini-batch needs a
 *    new graph.
 */
#ifndef ACROBAT_H
#define ACROBAT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
/* The library is built with hidden symbol visibility; what this header declares is its whole ABI. */
#if defined(__GNUC__)
#pragma GCC visibility push(default)
#endif

#define ACROBAT_OK 0
#define ACROBAT_EINVAL (-1)  /* null pointer, negative size, unsupported shape            */
#define ACROBAT_ESTRUCT (-2) /* malformed structure: bad child index, one child only, two  */
                             /* parents, cycle, not exactly one root, token out of range   */
#define ACROBAT_ENOMEM (-3)  /* host or device allocation failed                           */
#define ACROBAT_EHIP (-4)    /* a HIP runtime call failed                                  */
#define ACROBAT_ETIMEOUT (-5) /* a bounded wait inside a persistent kernel ran out (acrobat_device_status) */

typedef struct acrobat_ctx acrobat_ctx;

/* Create a context bound to HIP device `device`.  Owns the index staging buffers and
 * scratch memory, which grow on demand and are freed by acrobat_destroy. */
int acrobat_create(acrobat_ctx** out, int device);
void acrobat_destroy(acrobat_ctx* ctx);
/* Message of the last failing call on this context ("" if none); valid until the next call. */
const char* acrobat_last_error(const acrobat_ctx* ctx);
/* Static description of a return code. */
const char* acrobat_strerror(int code);

/* A mini-batch of binary trees (host memory, read-only).  Nodes of tree t occupy the global
 * ids [tree_off[t], tree_off[t+1]); `left`/`right` hold tree-LOCAL child ids, both -1 for a
 * leaf.  Any numbering of the nodes inside a tree is accepted.  `token` is the id of the
 * table row a leaf reads (ignored for internal nodes). */
typedef struct {
  int32_t n_trees;
  const int32_t* tree_off; /* [n_trees + 1], tree_off[0] == 0, non-decreasing */
  const int32_t* left;     /* [N] */
  const int32_t* right;    /* [N] */
  const int32_t* token;    /* [N] */
} acrobat_trees;

/* ---- host level scheduler (no GPU needed) --------------------------------------------
 * Depth schedule of section 4.1 (footnote: depth = 0 for a node that consumes nothing
 * produced in the graph, else 1 + the largest producer depth; batches run by increasing
 * depth).  One schedule node is one whole cell (grain-size coarsening, appendix "Grain Size Coarsening"), all
 * leaves sit in level 0 (hoisted input transforms, appendix "Operator Hoisting") and the two children of a
 * node are concurrent.  Inside a level nodes are listed by ascending global id.
 *
 * Outputs are caller-allocated host arrays: level_off[N + 1] (only n_levels + 1 entries are
 * written), level_nodes[N], and optionally lrow[N] / rrow[N] = global ids of the children of
 * the node at the same list position (-1 at leaves); either may be NULL.
 * vocab >= 0 additionally checks 0 <= token < vocab at every leaf; vocab < 0 skips that. */
int acrobat_schedule_trees(const acrobat_trees* trees, int32_t vocab, int32_t* n_levels,
                           int32_t* level_off, int32_t* level_nodes, int32_t* lrow, int32_t* rrow);

/* Sequence schedule (listing 2: step t of every sequence has depth t).  Level t lists the
 * rows seq_off[s] + t of all sequences with len[s] > t by ascending s, seq_off being the
 * exclusive prefix sum of len.  level_off[max len + 1], level_rows[sum len] caller-allocated. */
int acrobat_schedule_seqs(int32_t n_seq, const int32_t* len, int32_t* n_levels,
                          int32_t* level_off, int32_t* level_rows);

/* Bidirectional-RNN schedule with program phases (section 4.1, appendix "Combating Eagerness of Depth Scheduling"): operators of a phase
 * are scheduled and executed before any operator of the next phase, so depth counts inside a
 * phase.  Phase 0 holds the two recurrences (listing 2: step k of a direction has depth k), phase 1
 * every per-token output operator - all of them in ONE batch although the sequences differ in
 * length.  Nodes are coded  fwd(row) = row,  bwd(row) = R + row,  out(row) = 2R + row  with
 * R = sum len and row = seq_off[s] + t; a level lists its codes in ascending order.
 * level_off[max len + 2], level_codes[3 R] caller-allocated; n_levels = max len + 1 (0 if R == 0). */
int acrobat_schedule_birnn(int32_t n_seq, const int32_t* len, int32_t* n_levels, int32_t* level_off,
                           int32_t* level_codes);

/* ---- forward calls --------------------------------------------------------------------
 * Binary TreeLSTM (model of table 3).  Gate order of the 5H weight rows: (i, f_l, f_r, o, u).
 *   leaf:      z = W_leaf E[token] + b_leaf ; child states are the shared zero state
 *   internal:  z = U [h_l ; h_r] + b        ; U columns 0..H-1 act on h_l, H..2H-1 on h_r
 *   c = s(z_i) tanh(z_u) + s(z_fl) c_l + s(z_fr) c_r ;  h = s(z_o) tanh(c)
 * Level 0 is one batched kernel over all leaves that gathers embedding rows by token id
 * (hoisting + gather fusion, section 5.2); each later level is one kernel that gathers the
 * children's h and c rows by index, contracts [n_level x 2H] with U^T (all five gates in one
 * pass: horizontal fusion, appendix "Exploiting Data Reuse") and applies the gates (vertical fusion).
 * Requires H, D multiples of 32.  d_h and d_c receive one row per node, row = global node id.
 * Device pointers: d_emb [V,D], d_Wleaf [5H,D], d_bleaf [5H] or NULL (= 0), d_U [5H,2H],
 * d_b [5H] or NULL, d_h / d_c [N,H] (written). */
int acrobat_treelstm_forward(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t H, int32_t D,
                             int32_t V, const float* d_emb, const float* d_Wleaf,
                             const float* d_bleaf, const float* d_U, const float* d_b, float* d_h,
                             float* d_c, void* hip_stream);

/* acrobat_treelstm_forward for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same results (same kernels, same schedule,
 * same choice of kernel variant per level as long as a level's partial tiles fit the fixed workspace; a
 * level whose partial tiles do not fit runs unsplit, which only changes the summation order), but the
 * call allocates and frees nothing on the device or in pinned memory: the index lists are staged in a
 * pinned buffer of fixed size that acrobat_create made, and their device copy and the partial tiles of
 * k-split levels live in one array of ACROBAT_NOALLOC_SCRATCH_MIB MiB that is part of the library's
 * device image.  Each GPU the library is used on holds that array until the process ends.
 *  - At most ACROBAT_NOALLOC_MAX_NODES nodes per call, else ACROBAT_EINVAL (nothing is launched).
 *  - Every call on a GPU, from any context, shares that GPU's array: calls that overlap on one GPU
 *    (two streams, two contexts, two threads) race.  Calls on one stream are safe back to back.
 *    The index lists are uploaded whole and every partial tile is written before it is read; the only
 *    words that must be zero when a call starts are the tile counters of evenly split levels at the end
 *    of the array, which are zero when the library is loaded and which every launch leaves at zero.
 *  - Per-launch profiling and the unfused-gather ablation are not available here (the settings are
 *    ignored); acrobat_last_schedule works as usual.  The host-side schedule still uses the C++ heap. */
#define ACROBAT_NOALLOC_MAX_NODES 65536
#define ACROBAT_NOALLOC_SCRATCH_MIB 32
int acrobat_treelstm_forward_noalloc(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t H, int32_t D,
                                     int32_t V, const float* d_emb, const float* d_Wleaf,
                                     const float* d_bleaf, const float* d_U, const float* d_b, float* d_h,
                                     float* d_c, void* hip_stream);

/* MV-RNN (model of table 3; Evaluation, "Overall Performance": the cell multiplies two activations).  Every node
 * carries a vector and a d x d matrix; with left child (a, A) and right child (b, B):
 *   p = tanh(W [B a ; A b])      P = W_M [A ; B]      W, W_M: [d, 2d]
 * A leaf's (a, A) are rows `token` of the tables and are read in place by the parent's kernel
 * (no copy of leaf embeddings, Evaluation, "Overall Performance").  d_vec [N,d] / d_mat [N,d,d] receive the states of
 * internal nodes at row = global node id; leaf rows are written (copied from the tables) only
 * if copy_leaves != 0.  Requires d == 64 or d == 128.  Tables: d_vec_tab [V,d], d_mat_tab [V,d,d]. */
int acrobat_mvrnn_forward(acrobat_ctx* ctx, const acrobat_trees* trees, int32_t d, int32_t V,
                          const float* d_vec_tab, const float* d_mat_tab, const float* d_W,
                          const float* d_WM, float* d_vec, float* d_mat, int32_t copy_leaves,
                          void* hip_stream);

/* Variable-length LSTM (recurrence of listing 1 with the four-gate cell of appendix "Exploiting Data Reuse").
 * Gate order of the 4H rows: (i, f, o, u);  z = W_x x_t + W_h h_{t-1} + b ;
 * c_t = s(z_f) c_{t-1} + s(z_i) tanh(z_u) ; h_t = s(z_o) tanh(c_t) ; h_{-1} = c_{-1} = 0.
 * len[n_seq] (host, each >= 0).  Rows are packed sequence-major: row(s,t) = seq_off[s] + t.
 * The input transform of all steps of all sequences runs first as one dense batch (hoisted,
 * appendix "Operator Hoisting"); then one kernel per time step over the still-active sequences.
 * Requires H, D multiples of 32.  d_x [sum len, D], d_Wx [4H,D], d_Wh [4H,H], d_b [4H] or
 * NULL, d_h / d_c [sum len, H] (written). */
int acrobat_varlen_lstm_forward(acrobat_ctx* ctx, int32_t n_seq, const int32_t* len, int32_t H,
                                int32_t D, const float* d_x, const float* d_Wx,
                                const float* d_Wh, const float* d_b, float* d_h, float* d_c,
                                void* hip_stream);

/* Level-launch strategy of the recurrence (the paper's activity breakdown, table 6, and its remark on
 * persistence in Evaluation, "Overall Performance": launch overhead is of the order of the kernel time).
 * Enabled (the default), acrobat_varlen_lstm_forward runs all time steps in ONE launch whenever H is 128,
 * 256 or 512, at most 256 sequences have a step to run, and every workgroup of that launch is resident on
 * the GPU at once (an occupancy query; otherwise, or when disabled, one launch per step as described
 * above).  The batches are the same - step t over the sequences with len > t - and so is the schedule
 * that acrobat_last_schedule reports; the workgroups keep W_h on chip for all steps and synchronise
 * among themselves through arrival counters in device memory.  Every wait inside that kernel is bounded
 * by max_polls polls of a counter (max_polls < 0: the default, about a quarter of a million; max_polls == 0 is a
 * test hook: every wait gives up at once, whether or not it would have had to wait, so the error path below runs
 * deterministically): a
 * workgroup whose wait runs out raises a status word (in pinned host memory; nothing touches it otherwise),
 * all workgroups then leave at their next polls and the kernel ends normally with incomplete outputs.
 * acrobat_device_status reports that: call it once the stream has been synchronised; it returns ACROBAT_OK
 * or ACROBAT_ETIMEOUT and clears the condition.  Until it has been called the word stays raised and later
 * persistent launches of the context give up at their first long wait too.
 * The same switch covers acrobat_birnn_forward (H in {128, 256, 512}, at most 256 non-empty sequences, every
 * workgroup resident at once): both recurrences then run in one launch, blocks of 16 sequences per direction,
 * H / 16 workgroups per block exchanging h after every step in the same way.
 * It also covers acrobat_mvrnn_forward (d == 64 up to a widest internal level of 2 048 nodes, d == 128 up to 512):
 * all internal levels then run in ONE launch in which
 * a node waits for its own two children only (flag words per node, polled with the same bound) instead of a
 * whole level waiting for the previous one, provided every workgroup of that launch is resident at once and the
 * call is not being captured into a graph (a captured call keeps one launch per level).
 * Nothing else may occupy the GPU's compute units for long while such a launch runs (another stream's
 * kernels delay the workgroups that are not yet resident; the bound turns a too long delay into
 * ACROBAT_ETIMEOUT instead of a hang).  Two launches of this kind must never share the GPU - each could hold
 * the slots the other's missing workgroups need - so the library orders its own: when one comes from another
 * stream than the one before it on that GPU (from any context of the process), the new stream first waits for
 * an event recorded on the earlier one.  This does not cover launches captured into a graph, nor other
 * processes. */
int acrobat_set_persistent(acrobat_ctx* ctx, int32_t enabled, int32_t max_polls);
int acrobat_device_status(acrobat_ctx* ctx);

/* Diagnostic: what a barrier among workgroups inside one kernel costs on this GPU.  groups x group_size
 * workgroups (groups <= 8, at most 256 workgroups and never more than the GPU has compute units) run
 * `rounds` rounds of: store store_floats floats each, announce that, wait for the whole group (bounded as
 * above), read load_floats floats of what the group stored.  same_xcd != 0: workgroup b belongs to group
 * b % groups, so with groups == 8 a group's members share an XCD and its L2; else to group b / group_size,
 * members spread over all XCDs.  style 0: one arrival counter per group, agent-scope release before the
 * arrival and acquire after the wait (the fences write back / invalidate the XCD's L2), plain loads;
 * write_through != 0 then stores the payload with agent-scope atomic stores.  style 1: the same counter
 * without fences - write-through stores completed before the arrival, agent-scope loads.  style 2: style 1
 * with a flag line per consumer instead of the counter (group_size <= 32).  style 3: style 1 with payload
 * addresses of its own for every round (rounds x workgroups x store_floats x 4 bytes, at most 1 GiB) and PLAIN
 * payload loads: data that is written once per launch, written through, and only read after it has been
 * announced has never been in a cache on the reader's side, so a plain load cannot find a stale copy of it and
 * may be served by the L2 of the reader's XCD (the recurrence kernels' exchanged rows are of that kind; an
 * element that does turn out stale is counted, see below).
 * The persistent recurrence kernel uses style 1.  Outputs (host): *us_per_round = kernel time /
 * rounds; phase_us[6]: [0..4] = mean over workgroups and rounds of the time spent in payload stores + workgroup
 * barrier, announcing, waiting, acquire + workgroup barrier, payload loads (including the completion of the
 * acquire's invalidate); [5] = style 3 only: number of payload elements that were read and did not hold the
 * value stored in that round (0 if the reasoning above holds; store_floats must then be a power of two, and the
 * load time of style 3 includes this check).
 * Allocates its buffers per call and synchronises the stream. */
int acrobat_sync_probe(acrobat_ctx* ctx, int32_t groups, int32_t group_size, int32_t rounds, int32_t same_xcd,
                       int32_t style, int32_t write_through, int32_t store_floats, int32_t load_floats,
                       double* us_per_round, double* phase_us, void* hip_stream);

/* Bidirectional RNN with a per-token output layer (the BiRNN of table 3; cell of listing 1 used
 * in both directions with separate parameters, appendix "Exploiting Data Reuse" (code duplication); output operators batched by program
 * phases, Evaluation, "Benefits of Optimizations").  With p = forward or backward:
 *   hf_t = s(Wf_x x_t + bf + Wf_h hf_{t-1}), hf_{-1} = f.h_init     (steps t = 0 .. len-1)
 *   hb_t = s(Wb_x x_t + bb + Wb_h hb_{t+1}), hb_{len} = b.h_init    (steps t = len-1 .. 0)
 *   y_t  = relu(cb + C [hf_t ; hb_t])                               (C: [n_out, 2H])
 * The input transforms of both directions are hoisted (one dense batch each, sharing a launch);
 * the two recurrences are independent, step k of both directions shares one launch; the output
 * batch follows.  Rows are packed as for the LSTM.
 * Requires H, D multiples of 32, 1 <= n_out.  All pointers in acrobat_rnn_dir are device
 * pointers: Wx [H,D], Wh [H,H], b [H] or NULL, h_init [H].  d_hf / d_hb [sum len, H] and
 * d_y [sum len, n_out] are written. */
typedef struct {
  const float* Wx;
  const float* Wh;
  const float* b;
  const float* h_init;
} acrobat_rnn_dir;

int acrobat_birnn_forward(acrobat_ctx* ctx, int32_t n_seq, const int32_t* len, int32_t H, int32_t D,
                          int32_t n_out, const float* d_x, const acrobat_rnn_dir* fwd,
                          const acrobat_rnn_dir* bwd, const float* d_C, const float* d_cb,
                          float* d_hf, float* d_hb, float* d_y, void* hip_stream);

/* ---- generic runtime: batched execution of an explicit dataflow graph ---------------------
 * The step before the specialised entry points above (section 4.1, listing 2; appendix "Other Details"): the
 * unbatched program of a mini-batch calls acrobat_dfg_invoke once per operator instance, passing
 * the depth it computed inline, and acrobat_dfg_run executes the graph bucket by bucket - a
 * bucket being all nodes of one (phase, depth, op), in ascending node id - with one batched
 * index upload and one gather-fused kernel launch per bucket.  An op is one of the cell kernels
 * of this library bound to its parameters and arenas; a new cell needs an op description, not a
 * scheduler.
 *
 * acrobat_op_desc: the batch-independent arguments of a cell kernel.  For node i of a bucket the
 * kernel computes z[g*H + j] = sum_k in[k] * W[(gate_row(g)*H + j)*ldw + k] with in = row arg0 of
 * src0 (row stride ld0, kseg floats) followed, if nseg == 2, by row arg1 of src1, and then,
 * by epilogue:
 *   TREE_LEAF      (c, h)[out_row] from gates (i, o, u) = weight row blocks 0, 3, 4 of a [5H, kseg] matrix
 *   TREE_INTERNAL  (c, h)[out_row] from gates (i, f_l, f_r, o, u) and rows arg0, arg1 of cprev_src
 *   LSTM_STEP      (c, h)[out_row] from gates (i, f, o, u) + zadd[out_row, 4H] and row arg0 of cprev_src
 *                  (cprev_src NULL: zero previous state)
 *   STORE_Z / STORE_Z1   zout[out_row, 4H] / zout[out_row, H] = z + bias   (four gates / one)
 *   RNN_STEP       h[out_row] = sigmoid(z + bias + zadd[out_row, H])   (zadd NULL: no such term)
 *   RELU_OUT       y[out_row*ldo + j] = relu(z + bias[j]) for j < n_cols (W has n_cols rows; H = n_cols
 *                  rounded up to a multiple of 32)
 *   MVRNN          the matrix-vector cell (Evaluation, "Overall Performance"), no contraction segments (nseg = 0): H = d, 64 or 128;
 *                  arg0 / arg1 name the left / right child - a value >= 0 is a row of the arenas h = vec
 *                  [out_rows, d] and c = mat [out_rows, d, d] (an internal child), a value -(t + 1) is row t of
 *                  the tables src0 = vec_tab [src0_rows, d] and src1 = mat_tab [src0_rows, d, d] (a leaf child,
 *                  read in place); W [d, 2d], W2 = W_M [d, 2d]; writes row out_row of h and c:
 *                  vec = tanh(W [B a ; A b]), mat = W_M [A ; B] for children (a, A), (b, B)
 * All pointers are device pointers and must stay valid until the run has finished on its stream. */
#define ACROBAT_EPI_TREE_LEAF 0
#define ACROBAT_EPI_TREE_INTERNAL 1
#define ACROBAT_EPI_LSTM_STEP 2
#define ACROBAT_EPI_STORE_Z 3
#define ACROBAT_EPI_RNN_STEP 4
#define ACROBAT_EPI_RELU_OUT 5
#define ACROBAT_EPI_STORE_Z1 6
#define ACROBAT_EPI_MVRNN 7

typedef struct {
  int32_t epilogue; /* ACROBAT_EPI_* */
  int32_t H;        /* hidden size, multiple of 32 */
  int32_t nseg;     /* operand segments: 0 (no contraction), 1 or 2 */
  int32_t kseg;     /* floats per segment, multiple of 32 */
  const float* src0; int32_t ld0;
  const float* src1; int32_t ld1;
  const float* W; int32_t ldw;
  const float* bias;
  float* h; float* c;
  const float* cprev_src;
  const float* zadd;
  float* zout;
  int32_t n_cols; float* y; int32_t ldo;
  /* row counts for the range check of acrobat_dfg_invoke's arguments: arg0 < src0_rows (also the
   * rows of cprev_src), arg1 < src1_rows, out_row < out_rows (rows of h, c, zadd, zout, y) */
  int32_t src0_rows, src1_rows, out_rows;
  const float* W2; /* MVRNN only: W_M */
} acrobat_op_desc;

typedef struct acrobat_dfg acrobat_dfg;

/* The graph uses the context's index buffers and workspace: one run at a time per context.
 * ctx may be NULL for a graph that is only built and scheduled (acrobat_dfg_run then fails). */
int acrobat_dfg_create(acrobat_ctx* ctx, acrobat_dfg** out);
void acrobat_dfg_destroy(acrobat_dfg* g);
/* Message of the last failed acrobat_dfg_* call on this graph (owned by the graph). */
const char* acrobat_dfg_last_error(const acrobat_dfg* g);
/* Binds a cell kernel to its parameters; *op_id counts from 0.  ACROBAT_EINVAL on bad shapes. */
int acrobat_dfg_register_op(acrobat_dfg* g, const acrobat_op_desc* desc, int32_t* op_id);
/* Drops all nodes, keeps the ops. */
int acrobat_dfg_clear(acrobat_dfg* g);
/* Adds one operator instance.  out_row / arg0 / arg1: rows as described above (arg1 ignored unless
 * the op has two segments).  prod0 / prod1: node ids of the instances that produce the operands,
 * -1 for graph inputs; they serve the check of the inline depth (section 4.1, goal G.1): a node
 * must be in the same or a later phase than its producers and deeper than those of its own phase,
 * else ACROBAT_ESTRUCT.  Rows are checked against the op's row counts (an MVRNN op also takes the
 * negative leaf codes down to -src0_rows).  *node (may be NULL) receives the new node's id (0, 1, 2, ...). */
int acrobat_dfg_invoke(acrobat_dfg* g, int32_t op, int32_t phase, int32_t depth, int32_t out_row,
                       int32_t arg0, int32_t arg1, int32_t prod0, int32_t prod1, int32_t* node);
/* The unbatched TreeLSTM program (recursive evaluation of every tree, depth computed inline,
 * leaves hoisted to depth 0) written against acrobat_dfg_invoke: node (tree t, j) becomes an
 * instance of op_leaf (arg0 = token) or op_internal (args = children's arena rows) writing arena
 * row tree_off[t] + j.  Same structure checks and error codes as acrobat_schedule_trees. */
int acrobat_dfg_build_treelstm(acrobat_dfg* g, const acrobat_trees* trees, int32_t vocab,
                               int32_t op_leaf, int32_t op_internal);
/* Adds a ghost operation (section 4.1, appendix "Combating Eagerness of Depth Scheduling"): a node that occupies `depth` and is never
 * executed.  A program whose branches reach the same operator after different numbers of steps
 * invokes ghosts on the shorter branch and names the ghost as the operator's producer, so the
 * operator lands at one depth - in one batch - for every instance.  Checked against `prod` (a
 * node id or -1) like any node; *node (may be NULL) receives its id.  Results never change. */
int acrobat_dfg_ghost(acrobat_dfg* g, int32_t phase, int32_t depth, int32_t prod, int32_t* node);
/* Executes all nodes on the stream (asynchronously unless profiling is on).  Buckets of one
 * (phase, depth) are independent of each other (concurrent operators, section 4.1): two of them
 * with the same shapes share a launch. */
int acrobat_dfg_run(acrobat_dfg* g, void* hip_stream);
/* Buckets of the last run or of acrobat_dfg_schedule (host arrays owned by the graph, valid until
 * its next call): bucket_off[n_buckets + 1] into order[], bucket_op[n_buckets]. */
int acrobat_dfg_schedule(acrobat_dfg* g, int32_t* n_buckets, const int32_t** bucket_off,
                         const int32_t** order, const int32_t** bucket_op);

/* ---- tensor-dependent control flow: tree generation with a doubly recurrent network ------
 * Section 4.2: a program whose control flow depends on tensor values cannot be run to its end
 * before anything is evaluated.  Every instance therefore runs on a fiber (a cooperatively
 * scheduled stack), and so does every part of an instance that can proceed on its own; all fibers
 * advance until each waits for a value, then everything invoked so far is executed in batches
 * through the generic runtime above, the values are copied to the host, and the fibers go on.
 *
 * The program shipped here is the doubly recurrent network of table 3 (top-down generation of a
 * tree from one input vector per instance; the paper prints no equations, this is the cited
 * model with listing 1's cell as the recurrent unit).  Node i with parent p, previous sibling q:
 *   a_i = s(Wa [a_p ; emb[l_p]] + ba)   (root: a_p = the instance's row of d_x0, l_p = 0)
 *   f_i = s(Wf [f_q ; emb[l_q]] + bf)   (first child and root: f_q = 0, l_q = 0)
 *   g_i = s(Wp [a_i ; f_i] + bp)        y_i = Wo g_i + bo        s(t) = 1 / (1 + exp(-t))
 * Whether i has children, whether a sibling follows, and its label l_i are decided once y_i is
 * on the host.  As in the paper's evaluation (Evaluation, "Overall Performance", untrained parameters) the decisions
 * are emulated: a counter-based generator (splitmix64 steps) keyed by the node's position -
 * key(root of instance s) = mix(seed ^ mix(s)), key(child k) = mix(key(parent) + k + 1);
 * children iff depth + 1 < max_depth and u(mix(key ^ 1)) < p_child; sibling iff not the root,
 * k + 1 < max_children and u(mix(key ^ 2)) < p_sibling; label = mix(key ^ 3) mod n_labels;
 * u(b) = (b >> 11) / 2^53 - so an instance grows the same tree in every mode.
 *
 * mode: ACROBAT_TDC_SEQUENTIAL - no fibers, instance after instance, one evaluation per node;
 * ACROBAT_TDC_INSTANCE_FIBERS - one fiber per instance (batch parallelism only, each instance
 * generated depth first); ACROBAT_TDC_FORK_JOIN - also one fiber per list of children (subtrees
 * grow concurrently).  use_ghosts: a later sibling's ancestral cell is held back by a ghost
 * operation to the depth of its fraternal cell, so each evaluation has one batch per operator.
 *
 * The fraternal state of a first child depends on the parameters only (no previous sibling: zero
 * state, label 0).  Like other constant tensors (Evaluation, "Overall Performance") it is computed once, with the roots,
 * and reused by its consumers; the first children's own rows of d_f are written by one more batch
 * after the last evaluation.
 *
 * Nodes are numbered in the order of creation; node i's states are row i of d_a, d_f, d_g
 * [max_nodes, H] and d_y [max_nodes, n_out] (device, written).  acrobat_drnn_trees: host arrays
 * of max_nodes int32 each, caller-owned, any may be NULL: instance, parent and previous sibling
 * (node ids, -1: none), index among the siblings, depth (root 0), label, and the evaluation
 * (0, 1, ...) that computed the node.  ACROBAT_ENOMEM if more than max_nodes nodes would be
 * generated (device rows written so far stay written).  The call synchronises the stream at every
 * evaluation and returns when the last one has finished.  From 192 instances on (fiber modes,
 * profiling off) the instances are dealt out to two groups - instance s to group s mod 2 - that are
 * evaluated independently, the second on a stream of the library's own (default priority, ordered
 * behind what the given stream holds at the call): the host runs one group's program while the
 * other's kernels execute; `round` then counts each group's evaluations.  Requires H and n_out
 * multiples of 32. */
#define ACROBAT_TDC_SEQUENTIAL 0
#define ACROBAT_TDC_INSTANCE_FIBERS 1
#define ACROBAT_TDC_FORK_JOIN 2

typedef struct {
  uint64_t seed;
  int32_t max_depth;    /* levels per tree, 1 .. 4096 */
  int32_t max_children; /* children per node, >= 1 */
  float p_child, p_sibling;
  /* 0: emulated decisions as described above.  1: the decisions are read off the scores - children
   * iff depth + 1 < max_depth and y[0] > 0; a sibling follows iff the node is not a root,
   * k + 1 < max_children and y[1] > 0; label = the first l with the largest y[2 + l],
   * l < min(n_labels, n_out - 2) - seed, p_child and p_sibling are then unused, and
   * acrobat_drnn_schedule (which has no scores) refuses the mode.  The scores are fp32 results: a
   * score within rounding error of its threshold (or two label scores that close to each other) may
   * legitimately decide differently than a higher-precision evaluation would, and the tree then grows
   * differently from there on. */
  int32_t from_scores;
} acrobat_drnn_decisions;

typedef struct { /* device pointers */
  int32_t H, n_labels, n_out;
  const float* emb;                  /* [n_labels, H] */
  const float* Wa; const float* ba;  /* [H, 2H], [H] or NULL */
  const float* Wf; const float* bf;
  const float* Wp; const float* bp;
  const float* Wo; const float* bo;  /* [n_out, H], [n_out] or NULL */
} acrobat_drnn_params;

typedef struct {
  int32_t* inst; int32_t* parent; int32_t* prev; int32_t* sib_index; int32_t* depth; int32_t* label;
  int32_t* round;
} acrobat_drnn_trees;

typedef struct {
  int32_t n_nodes;
  int32_t n_rounds;  /* evaluations */
  int32_t n_buckets; /* batches (one per (depth, operator) and evaluation) */
  int32_t n_fibers;  /* fibers started */
  int32_t n_ghosts;  /* ghost operations invoked */
} acrobat_drnn_stats;

int acrobat_drnn_forward(acrobat_ctx* ctx, int32_t n_inst, const float* d_x0,
                         const acrobat_drnn_params* params, const acrobat_drnn_decisions* decisions,
                         int32_t mode, int32_t use_ghosts, int32_t max_nodes, acrobat_drnn_trees* trees,
                         float* d_a, float* d_f, float* d_g, float* d_y, acrobat_drnn_stats* stats,
                         void* hip_stream);
/* The same program, fibers and batching without any tensor work (host only, no context): the
 * structure of the generated trees and the evaluation each node would belong to. */
int acrobat_drnn_schedule(int32_t n_inst, int32_t n_labels, const acrobat_drnn_decisions* decisions,
                          int32_t mode, int32_t use_ghosts, int32_t max_nodes,
                          acrobat_drnn_trees* trees, acrobat_drnn_stats* stats);

/* ---- introspection --------------------------------------------------------------------
 * Schedule built by the last forward call on this context (host arrays owned by the context,
 * valid until the next forward call): level_off[n_levels + 1], level_nodes[level_off[n_levels]]. */
int acrobat_last_schedule(const acrobat_ctx* ctx, int32_t* n_levels, const int32_t** level_off,
                          const int32_t** level_nodes);

/* Per-launch timing.  With profiling on, a forward call gives every kernel launch a start and a
 * stop event of its own (stamped by the runtime with the kernel's begin and end, so `ms` is the
 * kernel's execution time without launch gaps) and synchronises the stream before returning.
 * The reduction kernel of a k-split level has its own record (ACROBAT_K_SPLITK_REDUCE) directly
 * behind the record of its level. */
typedef struct {
  int32_t kind;  /* ACROBAT_K_* */
  int32_t level; /* depth of the batch */
  int32_t n;     /* nodes (rows) in the batch */
  int32_t tile;  /* nodes per workgroup tile of the kernel variant that was launched */
  int32_t ksplit; /* workgroups sharing the contraction range of one tile; 0: the level was cut into equal
                     shares, one per compute unit, whatever tile boundaries they cross */
  float ms;      /* execution time of the kernel */
} acrobat_launch_record;

#define ACROBAT_K_TREE_LEAF 1
#define ACROBAT_K_TREE_INTERNAL 2
#define ACROBAT_K_MVRNN_LEVEL 3
#define ACROBAT_K_MVRNN_LEAFCOPY 4
#define ACROBAT_K_LSTM_INPUT 5
#define ACROBAT_K_LSTM_STEP 6
#define ACROBAT_K_RNN_INPUT 7
#define ACROBAT_K_RNN_STEP 8
#define ACROBAT_K_RNN_OUTPUT 9
#define ACROBAT_K_SPLITK_REDUCE 10
#define ACROBAT_K_GATHER 11
#define ACROBAT_K_DFG_BUCKET 12 /* level = bucket index */
#define ACROBAT_K_LSTM_PERSISTENT 13 /* all time steps of the recurrence in one launch; n = all rows */
#define ACROBAT_K_MVRNN_PERSISTENT 14 /* all internal levels of an MV-RNN batch in one launch; n = internal nodes */
#define ACROBAT_K_RNN_PERSISTENT 15 /* all steps of both directions of a bidirectional RNN in one launch; n = rows of both */

int acrobat_set_profiling(acrobat_ctx* ctx, int32_t enabled);

/* Ablation of gather fusion (section 5.2; measured in the paper's Evaluation, "Benefits of Optimizations").  Enabled (the
 * default), the level kernels read their operand rows in place through the index lists.  Disabled,
 * acrobat_treelstm_forward first copies every level's operand rows (embedding rows; child h and c
 * rows) into contiguous scratch with an explicit gather launch and the level kernel reads the
 * copies - the scheme of frameworks without gather fusion.  Results are bit-identical. */
int acrobat_set_gather_fusion(acrobat_ctx* ctx, int32_t enabled);

/* Tuning and test hook; no result ever depends on it beyond the summation order of the contraction.
 * The launcher normally picks a kernel variant per level from the level's size.  force_tile != 0 makes
 * every cell level of this context use one variant instead: 64 or 32 = nodes per workgroup tile of the
 * tiled kernel, 6 = the stepwise kernel for latency-bound levels, 16 = the kernel for small levels that feeds the
 * matrix cores straight from global memory (16-node tiles), 65 or 33 = 64- or 32-node tiles with the level
 * cut into equal shares, one per compute unit, inside one launch; force_ksplit (a power of two up to 32,
 * 0 = automatic) is then the number of workgroups sharing a tile's contraction range (tile 6: slabs moved
 * per step, 4 or 8; ignored for 65 and 33).  A forced shape that does not apply to a level (k range not divisible, workspace
 * too small) falls back to the automatic choice for that level.  mvrnn_variant: 0 = default MV-RNN
 * level kernels, 1 = the streaming kernel.  All zero restores the defaults.  The library reads no
 * environment variables. */
int acrobat_set_tuning(acrobat_ctx* ctx, int32_t force_tile, int32_t force_ksplit, int32_t mvrnn_variant);
/* Records of the last forward call (context-owned, valid until the next forward call). */
int acrobat_last_profile(const acrobat_ctx* ctx, int32_t* n_records,
                         const acrobat_launch_record** records);

#if defined(__GNUC__)
#pragma GCC visibility pop
#endif
#ifdef __cplusplus
}
#endif
#endif /* ACROBAT_H */
