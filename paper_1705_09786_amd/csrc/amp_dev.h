// Device-visible descriptors shared by the host library and the kernels.
// Plain structs only: the host fills one AmpDev, copies it to the arena, and
// passes its device address to the persistent kernel.
#pragma once
#include <stdint.h>

#define AMP_MAX_NODES 144   // the largest model: an RNN whose cell has 64 copies (3 + 2 x 63 nodes)
#define AMP_MAX_WORKERS 128
#define AMP_MAX_BUFS 24
#define AMP_THREADS 512
#define AMP_LDS_BYTES 163840   // 160 KB per workgroup on gfx950
#define AMP_DYN_LDS_BYTES (AMP_LDS_BYTES - 6144)   // dynamic part; the rest is for static __shared__
#define AMP_TREE_LOOKUP_MAX_MUF 16384
#define AMP_DENSE_MAX_MUF 256         // longest pending-gradient list of a dense node (messages)
#define AMP_STATIC_ARENA_BYTES (64u << 20)   // the library's built-in device arena (amp_create_static)

// LDS layout of a weight tile: rows padded to a multiple of 16, row stride a
// multiple of 16 floats plus, if needed, 4 more so that stride/4 is odd: rows
// are then 16-byte aligned and both row-wise 16-byte reads and column-wise
// 4-byte reads spread evenly over the LDS banks.
#if defined(__HIPCC__)
#define AMP_HD __host__ __device__
#else
#define AMP_HD
#endif
AMP_HD static inline int amp_round16(int v) { return (v + 15) & ~15; }
AMP_HD static inline int amp_round4(int v) { return (v + 3) & ~3; }
AMP_HD static inline int amp_ldrow(int cols) {
  int l = amp_round16(cols);
  if (((l >> 2) & 1) == 0) l += 4;
  return l;
}

// Message code carried by a ring entry: [31] direction, [30:20] slot,
// [19:0] position inside the instance.
#define MSG_CTL_SLOT 2047u   // not an instance's slot (those are 0 .. AMP_MAX_MAK - 1): a request to the worker itself
#define MSG_DIR_B 0x80000000u
#define MSG_SLOT(c) (((c) >> 20) & 0x7ffu)
#define MSG_LOCAL(c) ((c) & 0xfffffu)
#define MSG_MAKE(dirb, slot, local) (((dirb) ? MSG_DIR_B : 0u) | ((unsigned)(slot) << 20) | (unsigned)(local))
#define AMP_MAX_MAK 2047

// Values of ctl[0] when the kernel stopped itself.
#define ABORT_WATCHDOG 1u
#define ABORT_LOG_FULL 2u
#define ABORT_BAD_STATE 3u
#define ABORT_PLACEMENT 4u   // a packed launch found a workgroup on another die than its block index implies

enum AmpRole {
  ROLE_CTRL = 0,
  ROLE_MLP_LIN = 1,      // aux = layer index (0..2)
  ROLE_RNN_CELL = 2,     // hosts lookup + cell
  ROLE_RNN_OUT = 3,
  ROLE_TREE_LOOKUP = 4,
  ROLE_TREE_LEAF = 5,
  ROLE_TREE_BRANCH = 6,
  ROLE_TREE_OUT = 7,
  ROLE_G_LOOKUP = 8,
  ROLE_G_EDGE = 9,       // aux = edge type
  ROLE_G_GATE = 10,      // aux = 0 (z) / 1 (r)
  ROLE_G_CAND = 11,
  ROLE_G_READOUT = 12,
};

// Multi-producer ring of 64-bit entries: high word = ticket + 1 (ready tag),
// low word = message code.  Every consumer keeps a private head; capacity is
// sized by the host so that unconsumed entries never wrap.
struct RingDev {
  unsigned long long* ent;
  unsigned* tail;
  unsigned mask;
  unsigned pad;
};

// One parameterized node.  P = [W rows x cols row-major; b rows] is the master
// copy in HBM (loaded into LDS by the owning workgroups at kernel start,
// written back at exit); G, M, V have the same layout.
struct NodeDev {
  float* P;
  float* G;
  float* M;
  float* V;
  float* S;   // a replicated node's published parameters during a group synchronisation (Section 5); else null
  int rows, cols, has_bias, muf;
  int opt, mean, nblocks, block;   // rows = nblocks * block (gate blocks)
  float lr, mom, b1, b2, eps;
  // Column layout of the node's LDS tile and pending inputs: the cols columns
  // form a first segment of seg0 columns and (cols - seg0) / seg more of seg
  // columns, each padded to segp (a multiple of 4) so that a segment can be
  // fetched from its own 16-byte aligned row.
  int seg, segp, seg0;
};

struct WorkerDev {
  int role, node, tile, ntiles;
  int u0, nu;          // units [u0, u0+nu) of every gate block belong to this tile
  int ring, aux;
  unsigned* wstate;    // persistent per-worker words: [0] count, [1] opt step (node), [2] count, [3] step (hosted lookup)
  unsigned long long* log;
  unsigned* log_n;
  unsigned long long* stats;   // [0] ticks waiting, [1] messages, [2] batches, [3] ticks alive (100 MHz), [4..11] phases
  float* pend;                 // pending (delta, input) pairs of the hosted dense node
  unsigned log_cap;
  int kb;                      // largest batch this worker takes at once
  int rep;                     // which replica of its node this worker is (node replicas, Section 5); else 0
};

// One stored instance set (training or evaluation), flattened.
struct DataDev {
  int n_inst, n_x;
  const float* x;          // [n_inst][n_x]
  const float* target;     // [n_inst]
  const int* tok_off;      // [n_inst+1] into tok
  const int* tok;
  const int* lab_off;      // [n_inst+1] into lab
  const int* lab;
  const int* node_off;     // [n_inst+1] into left/right/parent
  const int* left;
  const int* right;
  const int* parent;       // parent*2 + side, -1 for the root
  const int* edge_off;     // [n_inst+1] into src/dst/etype
  const int* src;
  const int* dst;
  const int* etype;
  const int* tcount;       // [n_inst][8] directed edges per edge type
  const int* tnode;        // tree: [nodes][4] = left, right, parent*2+side (-1 root), label; indexed like left
  // graph adjacency, precomputed per instance (N nodes, E directed edges, T edge types):
  const int* inoff;        // [tok_off[i] + i + v], v = 0..N: start of node v's incoming edges in inedge (relative to edge_off[i])
  const int* inedge;       // [edge_off[i] + .]: incoming edges grouped by destination, ascending edge index inside a group
  const int* tstart;       // [i][9]: start of each type's block in tedge / tsk (prefix sums of tcount)
  const int* tedge;        // [edge_off[i] + tstart[c] + k]: k-th edge of type c, ascending edge index
  const int* tsoff;        // [T * (tok_off[i] + i) + c * (N + 1) + v]: start of the type-c edges leaving node v, in tsk
  const int* tsk;          // [edge_off[i] + tstart[c] + .]: positions k (rows of the type-c group) grouped by source node
  const int* tsrc;         // [edge_off[i] + tstart[c] + k]: source node of the k-th edge of type c (= src[tedge[.]])
  const int* tdst;         // the same for its target node
};

struct AmpDev {
  RingDev ring[AMP_MAX_WORKERS];
  NodeDev node[AMP_MAX_NODES];
  WorkerDev worker[AMP_MAX_WORKERS];
  DataDev data;
  int model, n_workers, n_nodes, mak;
  int d_in, hidden, n_class, vocab, emb, n_node_types, n_edge_types, n_steps;
  int max_len, max_edges, train, pad0;
  int tiles_leaf, tiles_branch;
  // graph model: workgroups ("tiles", split by hidden unit) per dense node -- [0..7] edge types, [8] update gate,
  // [9] reset gate, [10] candidate -- and where each edge type's partial results start among the g_PE parts
  int g_tiles[12];
  int g_eoff[9];
  int g_PE, g_PA;             // parts of the gradient w.r.t. h through the edges (sum of the edge tiles) / of the
                              // gradients the three GRU nodes return (candidate tiles, then update, then reset)
  unsigned n_total, first_seq;
  int admit_bounded, n_updaters;  // staleness-bounded admission on / workers that apply updates
  float max_staleness;            // its bound: updates per worker during an instance's life
  unsigned* ctl;              // [0] abort code, [1] done, [2] abort detail, [3] updates applied by all workers,
                              // [4] largest number of instances in flight, [5] admission limit at the end
  unsigned* slot_seq;         // [mak] admission number held by each slot
  int* slot_inst;             // [mak] the slot's instance: index into the launch's instance set; sign bit set = a
                              // forward-only (evaluation) instance, which the loss layer retires instead of turning round
  const int* adm_inst;        // [n_total] the same word for every admission of the launch, in admission order
  int* smeta;                 // [mak][4] written at admission: admission number, length, node offset (RNN: instance), token offset
  float* loss_out;            // [n_total] summed loss of each admission
  int* correct_out;           // [n_total]
  float* yhat_out;            // [n_total] (GGNN prediction)
  unsigned long long* clock;  // [0] first admission, [1] last retirement (wall_clock64 ticks)
  // Probe (tree model): output payloads of sampled events, for a per-event comparison on runs too long for their
  // end state to be compared.  Entry = [kind (0: a cell's forward output h, 1: the leaf cell's backward output
  // dx), admission number, tree node, 0 | payload], probe_w floats; instances with admission number % probe_period
  // == 0 are sampled; probe_n counts the entries asked for (those beyond probe_cap are dropped).
  float* probe;
  unsigned* probe_n;
  unsigned probe_cap, probe_period;
  int probe_w;
  int node_replicas;          // RNN: copies of the cell between Cond and Phi; admission a goes to copy a mod node_replicas
  int sync_every;             // ... and a request to synchronise them after every sync_every retirements (0 = never)
  long long watchdog_ticks;
  void* buf[AMP_MAX_BUFS];    // model-specific per-slot storage
  long long stride[AMP_MAX_BUFS];
};
