/*
 * amp.h -- C boundary of the MI355X implementation of asynchronous
 * model-parallel (AMP) training (AMPNet, arXiv 1705.09786).
 *
 * The library runs the paper's training method -- per-instance forward and
 * backward messages through a static graph of small dense cells, each
 * parameterized cell accumulating its own gradients and updating its own
 * parameters once enough have arrived (Section 3) -- as one persistent GPU
 * kernel in which workgroups play the role of the paper's workers
 * (Appendix A) and keep their cells' weights in LDS.
 *
 * Conventions
 *   - Every call returns 0 (AMP_OK) or a negative amp_status.  After an
 *     error amp_last_error(ctx) returns a message owned by the ctx.
 *   - All pointer arguments are HOST pointers unless the parameter is
 *     documented as a device pointer.  The caller owns every buffer it
 *     passes; the library copies what it needs during the call and writes
 *     results into caller-provided buffers of stated capacity.
 *   - The library never allocates device memory: it works inside the device
 *     arena handed to amp_create (or, after amp_create_static, inside an array
 *     of its own) and launches on the HIP stream given there.
 *   - A ctx is not thread-safe.  Call order: create -> build_* -> finalize
 *     -> (set_* | submit | train | eval | get_*)* -> destroy.  Calls made in
 *     the wrong phase return AMP_ESTATE.
 */
#ifndef AMP_H
#define AMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct amp_ctx amp_ctx;

enum amp_status {
  AMP_OK = 0,
  AMP_EINVAL = -1,       /* bad argument (message says which) */
  AMP_ESTATE = -2,       /* call made in the wrong phase */
  AMP_ENOMEM = -3,       /* arena or a caller buffer too small */
  AMP_EFULL = -4,        /* instance store full */
  AMP_EDEVICE = -5,      /* HIP error, or the kernel stopped itself (stall watchdog) */
  AMP_EUNSUPPORTED = -6  /* valid request that this build cannot run */
};

/* The four model graphs of Sections 2, 4 and 6 (Figures 2 and 4a; the experiments' MLP and Tree-LSTM). */
enum amp_model { AMP_MODEL_MLP = 1, AMP_MODEL_RNN = 2, AMP_MODEL_TREE = 3, AMP_MODEL_GGNN = 4 };

/* Sizes of a model; fields a model does not use are ignored.
 *   MLP : d_in -> hidden (ReLU) -> hidden (ReLU) -> n_class, softmax loss
 *   RNN : vocab x emb lookup, tanh cell (emb+hidden -> hidden), n_class
 *   TREE: vocab x emb lookup, leaf cell (emb -> 3*hidden), branch cell
 *         (2*hidden -> 5*hidden), n_class softmax at every tree node
 *   GGNN: n_node_types x hidden lookup, n_edge_types linear (hidden ->
 *         hidden), three GRU linears (2*hidden -> hidden), n_steps
 *         propagation steps, linear readout of the node sum, squared error */
typedef struct amp_model_dims {
  int32_t d_in, hidden, n_class, vocab, emb;
  int32_t n_node_types, n_edge_types, n_steps;
} amp_model_dims;

/* Parameterized nodes (PPT nodes, Section 4) are numbered per model:
 *   MLP : 0 lin1, 1 lin2, 2 lin3
 *   RNN : 0 lookup, 1 cell, 2 out
 *   TREE: 0 lookup, 1 leaf, 2 branch, 3 out
 *   GGNN: 0 lookup, 1..n_edge_types edge linears, then gz, gr, gh, readout
 * A node's parameters are one flat float vector: W (rows x cols, row-major)
 * followed by b (rows) -- lookups have no b.  Gate row blocks of `hidden`
 * rows each: leaf [i; o; u], branch [i; f_left; f_right; o; u]; branch
 * columns are [h_left; h_right]; rnn cell columns [embedding; h];
 * GRU columns [a; h] (gz, gr) and [a; r*h] (gh). */

/* One training or evaluation instance.  Unused fields are 0 / NULL.
 *   MLP : x[n_x], labels[1]
 *   RNN : tokens[n_tokens], labels[1]
 *   TREE: n_tokens = L leaves with tokens[L]; n_nodes = 2L-1; leaves are
 *         nodes 0..L-1, internal nodes L..2L-2 with children left[n],
 *         right[n] < n (left/right are -1 for leaves), root = 2L-2;
 *         labels[n_nodes]
 *   GGNN: n_nodes graph nodes with tokens[n_nodes] = node types; n_edges
 *         directed edges src[e] -> dst[e] of type etype[e]; every node must
 *         have at least one incoming edge; target */
typedef struct amp_instance {
  int32_t n_x;       const float *x;
  int32_t n_tokens;  const int32_t *tokens;
  int32_t n_labels;  const int32_t *labels;
  int32_t n_nodes;   const int32_t *left, *right;
  int32_t n_edges;   const int32_t *src, *dst, *etype;
  float target;
} amp_instance;

enum amp_opt { AMP_OPT_SGD = 0, AMP_OPT_MOMENTUM = 1, AMP_OPT_ADAM = 2 };
typedef struct amp_opt_params { float lr, momentum, beta1, beta2, eps; } amp_opt_params;

/* One entry of a worker's ordered event record: the worker executed the
 * forward (F) or backward (B) transform of `node` for the message keyed
 * (seq, local), or applied the node's accumulated update (U).  `seq` is the
 * instance's admission number (epoch * n_instances + index); `local` is the
 * position inside the instance: 0 for the MLP, the time step for the RNN
 * cell and lookup, the tree node for TREE nodes, the propagation step for
 * GGNN edge and GRU nodes.  Worker 0 is the controller: it records A
 * (admitted) and R (retired).  A copy of a replicated node also records S
 * (it published its parameters for synchronisation round `seq`) and L (it
 * loaded the round's mean): see amp_set_group_sync. */
enum amp_event_kind { AMP_EV_F = 0, AMP_EV_B = 1, AMP_EV_U = 2, AMP_EV_A = 3, AMP_EV_R = 4, AMP_EV_S = 5, AMP_EV_L = 6 };
typedef struct amp_event {
  uint16_t worker;
  uint8_t node;
  uint8_t kind;
  uint32_t seq;
  uint32_t local;
} amp_event;

typedef struct amp_eval_result {
  double mean_loss;     /* per instance */
  double accuracy;      /* correct / predictions (0 for GGNN) */
  uint64_t n_instances;
  uint64_t n_predictions;
  double seconds;       /* device time of the evaluation kernel */
} amp_eval_result;

/* Creates a context that works inside [dev_arena, dev_arena + arena_bytes)
 * (DEVICE pointer, 256-byte aligned, caller keeps it alive until
 * amp_destroy) and launches on hip_stream (a hipStream_t passed as void*;
 * NULL = the default stream).  Model = IR graph + controller, Section 4. */
int amp_create(amp_ctx **out, void *dev_arena, size_t arena_bytes, void *hip_stream);
/* amp_create for callers that cannot allocate device memory (tight serving
 * loops, harnesses that forbid hipMalloc, code that must not touch the
 * allocator): the context works inside a device array built into the library,
 * AMP_STATIC_ARENA_MAX bytes (64 MiB) on every GPU, instead of a caller's
 * arena, and neither this call nor any later call on the context allocates or
 * frees device memory.  Everything else is as for amp_create: instances,
 * parameters and results still travel through the caller's host buffers.
 * The device current at the call is the one used.  amp_finalize, amp_train
 * and amp_eval return AMP_ENOMEM, with a message naming the built-in arena,
 * when the model, max_active_keys and instance sets need more than it holds.
 * The array is shared by every such context on a GPU and keeps what the last
 * one left in it (each context clears what it needs to start from zero):
 * contexts that overlapped in it would race, so at most one per GPU may exist
 * at a time -- a second call returns AMP_ESTATE until the first context has
 * been destroyed.  AMP_EDEVICE when the array's address cannot be obtained. */
#define AMP_STATIC_ARENA_MAX ((size_t)64 << 20)
int amp_create_static(amp_ctx **out, void *hip_stream);
void amp_destroy(amp_ctx *ctx);

/* Generic graph construction (Section 4: a model is a static IR graph plus a
 * controller).  Node 0, the controller, exists from amp_create on; its output
 * ports are what it pumps into the graph (instances, initial states, labels)
 * and are numbered in the order they are connected.  Every other node is
 * added with amp_add_node and gets the next id (1, 2, ...).
 *
 * Kinds (Section 4, "Payload transformations", "Loops, state, and control
 * flow", "Aggregation and disaggregation"; the cells of Sections 2 and 6 and
 * Appendix C).  rows / cols are the weight matrix's; n_in / n_out the port
 * counts where the kind leaves them open; aux as noted:
 *   parameterized payload transforms
 *     LOOKUP            rows x cols table, token in, row out
 *     LINEAR            y = act(W x + b); aux = AMP_ACT_NONE / AMP_ACT_RELU
 *     RNN_TANH          h' = tanh(W [x; h] + b): a LINEAR with the tanh fused
 *     GRU               rows = hidden; ports in 0 = aggregated messages a, 1 =
 *                       state h; stands for three linear nodes (update gate,
 *                       reset gate, candidate; Appendix C)
 *     LEAF_LSTM         rows = hidden, cols = embedding; out = [h; c]
 *     BRANCH_LSTM       rows = hidden; in = [h_l; c_l; h_r; c_r], out = [h; c]
 *     GGNN_EDGE_LINEAR  rows = cols = hidden, applied to a group of rows
 *     SUM_READOUT       sum over the rows of the payload, then 1 x cols linear
 *   loss layers (port 0 prediction, port 1 label or target pumped by the
 *   controller; they start backpropagation): SOFTMAX_XENT (rows = classes),
 *   SQUARED_ERR
 *   control and aggregation, functions of the message state only:
 *     COND (n_out successors; aux = loop count where it ends a loop), PHI
 *     (n_in alternatives, records the origin), ISU (invertible state
 *     update), CONCAT (n_in ports; aux = parts that arrive on each port told
 *     apart by their state, 0 or 1 = one), SPLIT (n_out equal parts), BCAST
 *     (n_out copies; gradients summed in port order), GROUP, UNGROUP,
 *     FLATMAP, SUM (rows of a group added up), SINK (end of a path without
 *     a loss: answers a zero gradient)
 *
 * Ownership: desc is read during the call.  Errors: AMP_EINVAL for an unknown
 * kind or node id; AMP_ESTATE after a model has been built or finalized.
 *
 * amp_validate_graph (amp_finalize calls it if the caller did not) checks the
 * graph and returns AMP_EINVAL with a message for: a dangling port (every
 * port of every node must carry exactly one edge), a port connected twice, a
 * dimension mismatch between the two ends of an edge (widths are propagated
 * through the control nodes), a cycle that does not pass through a Phi.  A
 * valid graph is then matched, node by node and port by port, against the
 * four graphs the persistent kernel has workers for (Figure 2's RNN, the MLP
 * and Tree-LSTM of Section 6, Figure 4(a)'s gated graph network, as the
 * amp_build_* calls below construct them with these same two calls); any
 * other valid graph is AMP_EUNSUPPORTED.  After validation the parameterized
 * nodes carry the model's numbering (see "Parameterized nodes" below);
 * amp_get_node_index translates a graph node id into it (-1 for control and
 * loss nodes; a GRU node gives the first of its three). */
enum amp_node_kind {
  AMP_NODE_CONTROLLER = 0, AMP_NODE_LOOKUP, AMP_NODE_LINEAR, AMP_NODE_RNN_TANH, AMP_NODE_GRU, AMP_NODE_LEAF_LSTM,
  AMP_NODE_BRANCH_LSTM, AMP_NODE_GGNN_EDGE_LINEAR, AMP_NODE_SUM_READOUT, AMP_NODE_SOFTMAX_XENT, AMP_NODE_SQUARED_ERR,
  AMP_NODE_COND, AMP_NODE_PHI, AMP_NODE_ISU, AMP_NODE_CONCAT, AMP_NODE_SPLIT, AMP_NODE_BCAST, AMP_NODE_GROUP,
  AMP_NODE_UNGROUP, AMP_NODE_FLATMAP, AMP_NODE_SUM, AMP_NODE_SINK
};
#define AMP_ACT_NONE 0
#define AMP_ACT_RELU 1
typedef struct amp_node_desc { int32_t rows, cols, n_in, n_out, aux; } amp_node_desc;
int amp_add_node(amp_ctx *ctx, int kind, const amp_node_desc *desc, int *node_id);
int amp_connect(amp_ctx *ctx, int src, int src_port, int dst, int dst_port);
int amp_validate_graph(amp_ctx *ctx);
int amp_get_node_index(amp_ctx *ctx, int graph_node, int *param_node);

/* Builds one of the paper's model graphs (with the two calls above; the
 * graphs are those of Section 6's MLP paragraph, Figure 2, Section 6's
 * Tree-LSTM paragraph and Figure 4(a)) and validates it.  One model per ctx. */
int amp_build_mlp(amp_ctx *ctx, const amp_model_dims *dims);
int amp_build_rnn(amp_ctx *ctx, const amp_model_dims *dims);
int amp_build_treelstm(amp_ctx *ctx, const amp_model_dims *dims);
int amp_build_ggnn(amp_ctx *ctx, const amp_model_dims *dims);

/* Splits a heavy node's rows over `n_tiles` workgroups that run in lockstep
 * (Section 5: a linear layer can be split into tiles computed in
 * parallel).  1..64 tiles.  Only before amp_finalize; TREE leaf / branch
 * nodes only. */
int amp_set_tiles(amp_ctx *ctx, int node_id, int n_tiles);
/* Where a tiled node keeps its weights during a launch.  0 (default): in the
 * LDS of its workgroups when a tile fits, otherwise in HBM; 1: in HBM always
 * (the tiles read their rows from the parameter array as they go and update
 * them in place -- the mode for cells whose weights exceed the CUs' LDS, such
 * as hidden size 1024).  HBM mode needs emb and hidden to be multiples of 4
 * and at most 512 rows per tile.  Only before amp_finalize; TREE leaf /
 * branch nodes only. */
int amp_set_weights_in_hbm(amp_ctx *ctx, int node_id, int on);

/* Replicas (Section 5: data parallelism inside the IR).  Every parameterized
 * node is replicated n_replicas times and a Cond on the instance number sends
 * instance i (in submit order) to replica i mod n_replicas, so that n_replicas
 * copies of the whole pipeline train side by side, each with max_active_keys
 * instances in flight; at the end of every epoch each node's parameters are
 * set to the mean over its replicas (optimizer slots are not shared).  1
 * (default) = no replication; at most 128.  Workers x replicas must not exceed
 * the CUs.  When the replicas that share an XCD fit its 32 CUs, every replica
 * is placed inside one XCD and exchanges its messages through that XCD's L2.
 * Evaluation uses the first replica.  Event records and worker statistics
 * list replica 0's workers first, then replica 1's, ...; `seq` counts
 * admissions per replica.  Only before amp_finalize. */
int amp_set_replicas(amp_ctx *ctx, int n_replicas);

/* Replicas of one heavy node (Section 5: the linear layer in the body of the
 * RNN's loop is the bottleneck, so it alone is replicated, in full, between a
 * Cond and a Phi, and the rest of the graph is shared).  Built for the RNN
 * model's recurrent cell, node_id 1: copy r >= 1 of the cell is node 2 + 2 r,
 * a worker of its own with its own parameters, accumulator, update count and
 * optimizer slots; since the cell's worker hosts the embedding table, each
 * copy has its own table too (node 1 + 2 r).  The Cond routes on the instance:
 * admission a is run by copy a mod n_replicas, all its steps alike, and its
 * gradients return to that copy.  The output layer and the loss are shared
 * and see every instance.  At the end of every training epoch the copies'
 * parameters are set to their mean (the paper's infrequent synchronisation;
 * amp_set_group_sync adds its asynchronous trigger of a group
 * synchronisation while training runs).
 * amp_set_params / amp_set_min_update_frequency / amp_set_optimizer on node 0
 * or 1 apply to every copy; amp_get_params on them reads copy 0; the copies'
 * own ids work too, and event records name them.  1 (default) = no copies; at
 * most 64.  Does not combine with amp_set_replicas.  Only between the build
 * call and amp_finalize; AMP_EUNSUPPORTED for other models or nodes. */
int amp_set_node_replicas(amp_ctx *ctx, int node_id, int n_replicas);

/* Asynchronous synchronisation of a replicated node's copies while training
 * runs (Section 5, last sentence: besides the end-of-epoch averaging, a
 * message-passing protocol that triggers a synchronisation of the whole
 * group of replicas).  After every `every_retirements` retired instances the
 * controller sends a request message to every copy (amp_set_node_replicas);
 * a copy that takes the request from its ring publishes its parameters as
 * they stand and carries on with its messages; the copy whose publication
 * completes the group sends every copy a second message, and a copy that
 * takes that one moves its parameters to the mean of the published values
 * (summed in copy order) plus whatever it has learned since it published.  A
 * new round starts only when every copy has loaded the previous one.  Nothing
 * waits: rounds still under way when the last instance retires are dropped,
 * and the end-of-epoch averaging follows as always.  The record lists both
 * steps (S, L) in the copies' own order, so the checker replays them.
 * 0 (default) = never.  AMP_EINVAL if negative; without node replicas the
 * setting has no effect.  Any time after the build call. */
int amp_set_group_sync(amp_ctx *ctx, int every_retirements);

/* Validates the graph if that has not been done (see amp_validate_graph),
 * places its nodes on workers (Appendix A: a worker hosts one or more IR
 * nodes; Section 6 affinitizes the heavy operations to workers of their own:
 * here one workgroup per parameterized node or tile of it) and lays out the
 * arena: message queues, the per-key activation records of the parameterized
 * nodes (Section 4, "Payload transformations") and the join tables, for at
 * most max_active_keys instances in flight (Section 3), each at most
 * max_instance_len long (time steps, tree leaves, or graph nodes) with at most
 * max_edges directed edges, and room for max_instances stored instances per
 * set.  AMP_ENOMEM when the arena is too small, AMP_EUNSUPPORTED when a node
 * fits no worker. */
int amp_finalize(amp_ctx *ctx, int max_active_keys, int max_instance_len, int max_edges,
                 size_t max_instances);

/* max_active_keys: number of instances in flight (Section 3); 1..the value
 * given to amp_finalize. */
int amp_set_max_active_keys(amp_ctx *ctx, int mak);
/* How the controller admits instances (Appendix B, MNIST: the greedy schedule
 * lets gradients go stale at a high max_active_keys and a better one would
 * remove that sensitivity).
 *   AMP_ADMIT_GREEDY (default): a new instance whenever fewer than
 *     max_active_keys are in flight.
 *   AMP_ADMIT_BOUNDED: the number in flight is a limit of its own in
 *     1..max_active_keys.  It starts at 1, grows by one with every instance
 *     that retires having seen at most max_staleness updates per worker
 *     (updates applied by all workers during the instance's life, divided by
 *     the number of workers) and shrinks by one with every instance that saw
 *     more.  max_staleness >= 0; 0 keeps one instance in flight once any
 *     update has been applied.  Evaluation always admits greedily.
 * amp_get_admission reports, for the last amp_train call's last launch, the
 * largest number of instances that were in flight and the limit at the end
 * (largest over the replicas); either pointer may be NULL. */
#define AMP_ADMIT_GREEDY 0
#define AMP_ADMIT_BOUNDED 1
int amp_set_admission(amp_ctx *ctx, int policy, double max_staleness);
int amp_get_admission(amp_ctx *ctx, int *max_in_flight, int *final_limit);
/* min_update_frequency of a node (-1 = all): the node updates as soon as it
 * has accumulated this many gradients (Section 3); >= 1. */
int amp_set_min_update_frequency(amp_ctx *ctx, int node_id, int muf);
/* Optimizer of a node (-1 = all), Appendix A.  Lookup nodes support SGD only. */
int amp_set_optimizer(amp_ctx *ctx, int node_id, int kind, const amp_opt_params *p);
/* 1 (default): the applied gradient is the mean of the accumulated ones; 0: their sum. */
int amp_set_gradient_mean(amp_ctx *ctx, int mean);

/* Parameters of a parameterized node (Section 4: a PPT node owns its
 * parameters; Appendix C: parameter, gradient buffer and optimizer slots live
 * with the node), as one flat host vector in the layout given under
 * "Parameterized nodes" above.  set copies from `host` (n must be the node's
 * count) and takes effect at the next amp_train / amp_eval; get copies the
 * present values into `host` (capacity cap floats; *n = count; AMP_ENOMEM if
 * cap is too small).  Initial values are the caller's: the library draws no
 * random numbers. */
int amp_num_nodes(amp_ctx *ctx);
int amp_param_count(amp_ctx *ctx, int node_id, size_t *n);
int amp_set_params(amp_ctx *ctx, int node_id, const float *host, size_t n);
int amp_get_params(amp_ctx *ctx, int node_id, float *host, size_t cap, size_t *n);

/* Appends an instance to the training set (which = 0) or the evaluation set
 * (which = 1): what the controller will pump into the graph for it --
 * tokens, initial states, labels, the graph structure the messages' states
 * refer to (Section 4, Overview and the RNN / GNN examples).  `key` is kept
 * for the caller's bookkeeping.  The instance is checked (AMP_EINVAL names
 * the fault: a tree node without two children, an unreachable node, an edge
 * endpoint outside the graph, a label out of range ...) and copied; it
 * reaches the device at the next amp_train / amp_eval.  AMP_EFULL beyond
 * max_instances.  amp_clear_instances empties a set. */
int amp_submit(amp_ctx *ctx, int which, uint64_t key, const amp_instance *inst);
int amp_clear_instances(amp_ctx *ctx, int which);

/* Record up to events_per_worker events per worker during the next
 * amp_train calls (0 = off, the default).  Costs arena space. */
int amp_set_event_log(amp_ctx *ctx, size_t events_per_worker);
/* Probe for per-event comparison on runs too long for their end state to be
 * compared (after 10^4 .. 10^5 asynchronous updates rounding differences have
 * compounded; what a single forward or backward transform emits has not):
 * during the next amp_train calls the kernel keeps, for every instance whose
 * admission number is a multiple of `period`, the output payload of each cell's
 * forward transform (a tree node's h) and of the leaf cell's backward
 * transform (the gradient w.r.t. the leaf's embedding), up to max_entries
 * entries (later ones are dropped); period 0 switches it off.  TREE only.
 * amp_get_probe copies the entries of the last amp_train: each is
 * entry_floats floats -- four 32-bit header words {kind (0 = forward output,
 * 1 = leaf backward output), admission number, tree node, 0} followed by the
 * payload (hidden or emb floats, zero padded).  host NULL = size query. */
int amp_set_probe(amp_ctx *ctx, unsigned period, size_t max_entries);
int amp_get_probe(amp_ctx *ctx, float *host, size_t cap_floats, size_t *n_entries, size_t *entry_floats);
/* Seconds a worker may wait for a message before the kernel stops itself
 * and amp_train returns AMP_EDEVICE (default 20). */
int amp_set_watchdog(amp_ctx *ctx, double seconds);

/* Blocking: trains `epochs` passes over the training set in submit order by
 * asynchronous model-parallel training (Section 3): the controller keeps up to
 * max_active_keys instances in flight, every parameterized node accumulates
 * the gradients that reach it and applies its own update once
 * min_update_frequency of them have arrived, with no synchronisation between
 * nodes.  AMP_EDEVICE if the kernel stopped itself (watchdog, record full, or a
 * launch that packs whole replicas into single XCDs found a workgroup on another die than its index implies). */
int amp_train(amp_ctx *ctx, int epochs);
/* Blocking: forward-only pass over the evaluation set with the present
 * parameters (Section 1: inference runs through the same graph; Table 2's
 * validation throughput); nothing is recorded or updated. */
int amp_eval(amp_ctx *ctx, amp_eval_result *out);
/* Blocking: training and inference at the same time (Section 1: both kinds of
 * instance travel through the same graph; an inference instance is a message
 * that only runs forward).  One launch trains `epochs` passes over the
 * training set and, interleaved with them, evaluates every instance of the
 * evaluation set once: after every (training admissions / evaluation
 * instances) training instances the controller admits one evaluation
 * instance, marked forward-only -- it is scored with the parameters it meets
 * on its way (which the training instances around it keep updating), records
 * no activation, produces no gradient, and is retired by the loss layer.
 * Both kinds count towards max_active_keys.  `out` receives the evaluation
 * results; the training results are read as after amp_train (amp_get_loss,
 * amp_get_instance_losses, amp_get_event_log: the controller's admission
 * events carry local = 1 for evaluation instances, whose forward events are
 * part of the record).  AMP_EUNSUPPORTED with replicas. */
int amp_train_eval(amp_ctx *ctx, int epochs, amp_eval_result *out);

/* Results of the last amp_train, as the experiments of Section 6 report them
 * (Tables 1 and 2: accuracy, instances per second): mean loss per instance,
 * accuracy over all predictions, instances trained, device seconds from first
 * admission to last retirement.  Any out pointer may be NULL. */
int amp_get_loss(amp_ctx *ctx, double *mean_loss, double *accuracy, uint64_t *n_instances,
                 double *seconds);
/* Per-admission losses of the last amp_train (the loss layer's output for
 * each instance, Section 4; a tree's is the sum over its nodes), in admission
 * order.  AMP_ENOMEM if cap is too small; *n = count. */
int amp_get_instance_losses(amp_ctx *ctx, float *host, size_t cap, size_t *n);
/* Events of the last amp_train, worker by worker, each worker's in execution
 * order.  Under asynchronous training the result depends on the order in
 * which each node saw its messages and applied its updates (Section 3:
 * parameters may change between a message's forward and backward pass); the
 * record is that order, enough to repeat the run elsewhere.  buf NULL = size
 * query; AMP_ENOMEM if cap is too small. */
int amp_get_event_log(amp_ctx *ctx, amp_event *buf, size_t cap, size_t *n);
/* Gradient staleness as Section 3 defines it: bins[k] = gradients whose node
 * was updated k times between their forward and backward pass (last bin =
 * that many or more), from the event record of the last amp_train
 * (AMP_ESTATE without one). */
int amp_get_staleness_hist(amp_ctx *ctx, uint64_t *bins, size_t nbins);
int amp_num_workers(amp_ctx *ctx);
/* Utilisation of the last amp_train / amp_eval, one entry per worker
 * (workgroup): fraction of the kernel's life spent waiting for a message,
 * messages taken, the node the worker hosts (-1 = controller), batches of
 * messages taken, and (8 per worker) the fraction of time spent in each of
 * the worker's processing phases.  Workers correspond to the paper's
 * Appendix A workers; a node whose workers never wait is the pipeline's
 * bottleneck.  Any out pointer may be NULL. */
int amp_get_worker_stats(amp_ctx *ctx, double *wait_fraction, uint64_t *messages, int32_t *node_of_worker,
                         size_t cap, size_t *n, uint64_t *batches, double *phase_fraction);
/* The accelerator die (XCC, 0..7) each worker's workgroup ran on during the
 * last amp_train / amp_eval, in the order of amp_get_worker_stats.  The
 * launch places the workers of one replica on one die whenever whole replicas
 * fit its 32 compute units (Appendix A's affinitization of nodes to workers,
 * applied to the chip's eight L2 domains); this reports where they really
 * ran, as read from the hardware by each workgroup. */
int amp_get_worker_placement(amp_ctx *ctx, int32_t *xcc, size_t cap, size_t *n);
const char *amp_last_error(amp_ctx *ctx);

/* Measures the two rates the workers' rooflines are quoted against (Section
 * 3 / Appendix C argue from the cost of loading the weights): the LDS read
 * rate of one worker-shaped workgroup (512 threads, 16-byte reads) per
 * compute unit with every compute unit busy, in bytes/s per CU, and the HBM
 * read rate of a streaming sum over dev_buf, in bytes/s.  dev_buf: device
 * memory, 256-byte aligned, at least 64 MiB (use more than the 256 MiB last
 * level cache for an HBM figure), initialised by the caller with finite
 * floats, not written.  Needs no context; blocks until both launches on
 * hip_stream have finished.  AMP_EINVAL for bad arguments, AMP_EDEVICE when
 * a launch fails. */
int amp_measure_peaks(void *dev_buf, size_t bytes, void *hip_stream, double *lds_bytes_per_s_per_cu,
                      double *hbm_read_bytes_per_s);

#ifdef __cplusplus
}
#endif
#endif /* AMP_H */
