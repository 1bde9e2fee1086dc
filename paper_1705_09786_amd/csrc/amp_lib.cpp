// Host side of the C boundary declared in include/amp.h: graph construction
// and validation, arena layout, instance staging, kernel launch, results.
// No step of the training path runs here: every forward, backward and update
// happens in the persistent kernel.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/amp.h"
#include "amp_dev.h"
#include "amp_graph.h"

extern "C" hipError_t amp_launch(const AmpDev* devs, int n_replicas, int workers_per_replica, hipStream_t stream);
extern "C" hipError_t amp_peak_lds_launch(int n_wg, int iters, float* sink, hipStream_t stream, double* seconds,
                                          double* bytes_per_wg);
extern "C" hipError_t amp_peak_hbm_launch(const void* src, size_t bytes, float* sink, hipStream_t stream, double* seconds);
extern "C" hipError_t amp_average(float* p0, size_t stride_floats, int n_replicas, size_t n, hipStream_t stream);
extern "C" hipError_t amp_static_arena(void** ptr, size_t* bytes);

namespace {

constexpr size_t NSTAT = 13;   // words per worker in the statistics block (AMP_NSTAT of the kernels)

struct HostNode {
  std::string name;
  int rows = 0, cols = 0, has_bias = 0, nblocks = 1, block = 0;
  int muf = 1, opt = AMP_OPT_SGD, tiles = 1;
  int in_hbm = 0;           // tiles read the weights from HBM even if they would fit LDS
  int seg = 0, segp = 0, seg0 = 0;   // column segments of the LDS layout (seg 0 = one unpadded segment; seg0 0 = seg)
  int first_seg() const { return seg0 ? seg0 : seg; }
  int cl() const { return seg ? ((cols - first_seg()) / seg + 1) * segp : cols; }
  amp_opt_params op{0.1f, 0.9f, 0.9f, 0.999f, 1e-8f};
  std::vector<float> params;
  bool dirty = true;        // host copy newer than device copy
  size_t off_P = 0, off_G = 0, off_M = 0, off_V = 0;
  int base = -1, rep = 0;   // a replica of node `base` (Section 5); -1 = a node of its own
  size_t off_S = 0;         // a replicated node's published parameters (group synchronisation); 0 = none
  size_t count() const { return (size_t)rows * cols + (has_bias ? rows : 0); }
};

struct HostWorker {
  int role, node, tile, ntiles, u0, nu, ring, aux;
  int kb = 1, rep = 0;
  size_t off_state, off_pend = 0, pend_bytes = 0;
};

struct InstSet {
  std::vector<uint64_t> keys;
  std::vector<float> x, target;
  std::vector<int> tok_off{0}, tok, lab_off{0}, lab, node_off{0}, left, right, parent, edge_off{0}, src, dst, etype, tcount;
  std::vector<int> tnode;   // tree: left, right, parent code, label per node
  std::vector<int> inoff, inedge, tstart, tedge, tsoff, tsk, tsrc, tdst;   // graph adjacency (see DataDev)
  bool dirty = true;   // host copy newer than what the arena holds
  size_t n() const { return keys.size(); }
  void clear() { *this = InstSet(); }
};

// An instance set as it lies in the arena, dealt to R replicas: kept from call to call until the set changes.
struct Resident {
  bool valid = false;
  int R = 0;
  size_t begin = 0, end = 0;
  std::vector<DataDev> dd;   // per replica
  std::vector<size_t> n;     // instances per replica
};

}  // namespace

struct amp_ctx {
  char* arena = nullptr;
  size_t arena_bytes = 0;
  hipStream_t stream = nullptr;
  int static_dev = -1;   // >= 0: the arena is the library's built-in one on this device (amp_create_static)
  int model = 0;
  amp_model_dims dims{};
  ampgraph::Graph graph;       // the IR graph as described through amp_add_node / amp_connect (or by amp_build_*)
  std::vector<int> param_of;   // per graph node: the model's parameterized-node number, -1 for control and loss nodes
  std::vector<HostNode> nodes;
  std::vector<HostWorker> workers;
  bool finalized = false;
  int max_mak = 0, mak = 1, max_len = 0, max_edges = 0, mean = 1;
  size_t max_instances = 0, log_cap = 0;
  double watchdog_s = 20.0;
  unsigned probe_period = 0;     // sample instances whose admission number is a multiple of this (0 = off)
  size_t probe_cap = 0;          // entries the probe buffer holds
  std::vector<float> last_probe; // entries of the last training call
  size_t last_probe_w = 0;
  int admit_bounded = 0;         // staleness-bounded admission
  double max_staleness = 0;
  int last_max_in_flight = 0, last_limit = 0;   // of the last training launch, largest over the replicas
  InstSet sets[2];
  Resident resident[2];
  // arena layout
  size_t static_end = 0;   // everything below is laid out at finalize
  size_t off_dev = 0, off_ctl = 0, off_slot_seq = 0, off_clock = 0, off_smeta = 0, off_slot_inst = 0;
  std::vector<size_t> off_ring_ent, off_ring_tail;
  size_t sync_end = 0;   // [0, sync_end) of a replica's region: stop word, clock, slot tables, rings -- zero at every launch
  unsigned ring_cap = 0;
  size_t off_buf[AMP_MAX_BUFS] = {0};
  size_t buf_bytes[AMP_MAX_BUFS] = {0};
  long long buf_stride[AMP_MAX_BUFS] = {0};
  bool state_zeroed = false;
  int replicas = 1, last_replicas = 1;
  int node_replicas = 1;                              // copies of the recurrent cell between Cond and Phi (Section 5)
  int sync_every = 0;                                 // retirements between two synchronisation requests to them (0 = never)
  size_t rep_stride = 0;                              // bytes from one replica's static region to the next
  std::vector<unsigned> rep_admitted;                 // admissions so far, per replica
  std::vector<std::vector<amp_event>> launch_events;  // per worker, while a training call runs
  // results of the last train
  std::vector<float> last_loss;
  std::vector<int> last_correct;
  std::vector<amp_event> last_events;
  double last_seconds = 0;
  std::vector<unsigned long long> last_stats;   // NSTAT per worker
  uint64_t last_npred = 0;
  std::string err;
};

namespace {

int fail(amp_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf;
  return code;
}

#define HIPCHK(c, call)                                                                      \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess) return fail(c, AMP_EDEVICE, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

static_assert(AMP_STATIC_ARENA_MAX == AMP_STATIC_ARENA_BYTES, "the header states the built-in arena's size");
const char* arena_name(const amp_ctx* c) {
  return c->static_dev >= 0 ? "the library's built-in arena (amp_create_static)" : "the arena";
}

// Everything replica r owns in the static part of the arena lies rep_stride bytes after replica r - 1's.
char* rep_ptr(const amp_ctx* c, int r, size_t off) { return c->arena + (size_t)r * c->rep_stride + off; }

HostNode make_node(const char* name, int rows, int cols, int has_bias, int nblocks = 1) {
  HostNode n;
  n.name = name;
  n.rows = rows;
  n.cols = cols;
  n.has_bias = has_bias;
  n.nblocks = nblocks;
  n.block = rows / nblocks;
  n.params.assign(n.count(), 0.f);
  return n;
}

int check_build(amp_ctx* c, const amp_model_dims* d) {
  if (!c || !d) return fail(c, AMP_EINVAL, "null argument");
  if (c->model) return fail(c, AMP_ESTATE, "a model graph was already built");
  return AMP_OK;
}

bool positive(std::initializer_list<int> v) {
  for (int x : v)
    if (x < 1) return false;
  return true;
}

unsigned next_pow2(size_t v) {
  unsigned p = 1;
  while (p < v) p <<= 1;
  return p;
}

size_t r4(size_t n) { return (n + 3) & ~(size_t)3; }

size_t tile_rows(const amp_ctx* c, const HostWorker& w) { return (size_t)c->nodes[w.node].nblocks * w.nu; }
size_t pend_stride(const amp_ctx* c, const HostWorker& w) {
  return (size_t)amp_round16((int)tile_rows(c, w)) + (size_t)amp_round16(c->nodes[w.node].cl());
}
// Rows one gradient message can carry (grouped rows of the graph model).
size_t rows_per_message(const amp_ctx* c, const HostWorker& w) {
  if (w.role == ROLE_G_EDGE) return (size_t)c->max_edges;
  if (w.role == ROLE_G_GATE || w.role == ROLE_G_CAND) return (size_t)c->max_len;
  return 1;
}

// LDS floats a worker needs (mirrors the carving in the kernels); sets w.kb.
// Returns 0 when the worker cannot fit.
size_t lds_floats(const amp_ctx* c, HostWorker& w) {
  const size_t avail = AMP_DYN_LDS_BYTES / 4;
  w.kb = 1;
  if (w.role == ROLE_CTRL) return r4(2 * c->max_mak);   // free slots, update count at admission
  if (w.role == ROLE_TREE_LOOKUP) {
    w.kb = 64;
    return r4(c->max_mak) + AMP_TREE_LOOKUP_MAX_MUF;
  }
  if (w.role == ROLE_G_LOOKUP) return r4((size_t)c->dims.n_node_types * c->dims.hidden) + r4((size_t)c->max_len * c->dims.hidden);
  const HostNode& n = c->nodes[w.node];
  const size_t R = tile_rows(c, w), C = n.cols, Rp = amp_round16((int)R), ldw = amp_ldrow(n.cl());
  const size_t stride = pend_stride(c, w), wfl = r4(Rp * ldw) + r4(Rp);
  if (R > AMP_THREADS) return 0;
  size_t f = 0;
  switch (w.role) {
    case ROLE_RNN_CELL:
    case ROLE_TREE_LEAF:
    case ROLE_TREE_BRANCH: {
      // the largest batch (a multiple of 16 messages) whose pre-activation rows fit beside the weights
      const size_t ldy = amp_ldrow((int)R);
      // tree cells: aux 1 = the weights stay in HBM, aux 2 = LDS-resident with the deltas in rows of their own
      if (w.role != ROLE_RNN_CELL && w.aux == 2) w.aux = 0;
      if (w.aux == 1 && w.role != ROLE_RNN_CELL) {
        // weights stay in HBM: rows must be 16-byte aligned and unpadded
        if (c->dims.hidden % 4 || c->dims.emb % 4) return 0;
        for (w.kb = 64; w.kb >= 16; w.kb -= 16) {
          f = r4(Rp) + r4((size_t)w.kb * ldy) + 2 * r4(Rp) + 2 * 64 * 68;
          if (f <= avail) break;
        }
        if (w.kb < 16) return 0;
        break;
      }
      // the update's register accumulator holds 8 waves x 4 (16-row, 64-column) units
      if ((Rp / 16) * ((amp_round16(n.cl()) + 63) / 64) > 32) return 0;
      // a sequence has one message in flight, so the recurrent cell never sees more than max_active_keys at once
      const int kb_top = w.role == ROLE_RNN_CELL ? std::min(64, amp_round16(c->max_mak)) : 64;
      for (w.kb = kb_top; w.kb >= 16; w.kb -= 16) {
        f = wfl + r4((size_t)w.kb * ldy) + r4(Rp) + (size_t)(amp_round16(n.cl()) + 63) / 64 * 64;
        if (f <= avail) break;
      }
      if (w.kb < 16) return 0;
      // a tree cell keeps the deltas in rows of their own (waves without a share of the forward product form them
      // meanwhile) where that costs no batch size
      if (w.role != ROLE_RNN_CELL && f + r4((size_t)w.kb * ldy) <= avail) {
        f += r4((size_t)w.kb * ldy);
        w.aux = 2;
      }
      if (w.role == ROLE_RNN_CELL) {
        // the lookup's gradient accumulator beside the cell's weights, if it fits (worker aux = 1)
        const size_t lkg = r4((size_t)c->dims.vocab * c->dims.emb);
        w.aux = f + lkg <= avail ? 1 : 0;
        if (w.aux) f += lkg;
      }
      break;
    }
    case ROLE_TREE_OUT: {
      // the register-resident gradient accumulator holds 12 elements per thread
      if (R * C > 12 * AMP_THREADS) return 0;
      for (w.kb = 64; w.kb >= 16; w.kb -= 16) {
        f = wfl + r4((size_t)w.kb * amp_round4(c->dims.hidden)) + r4((size_t)w.kb * 64) + r4(c->max_mak);
        if (f <= avail) break;
      }
      if (w.kb < 16) return 0;
      break;
    }
    case ROLE_G_EDGE: {
      // stacked rows of a pass (several messages): as many as fit, up to 128; at least one message's
      const size_t H = c->dims.hidden, Ep = amp_round16(c->max_edges), Hs = amp_ldrow((int)H);
      if ((Rp / 16) * ((amp_round16((int)C) + 63) / 64) > 32) return 0;   // the update's register accumulator
      size_t cap = std::max<size_t>(Ep, 128);
      for (;; cap -= 16) {
        f = wfl + r4(Rp) + (size_t)(amp_round16((int)C) + 63) / 64 * 64 + 2 * r4(cap * Hs) + r4(cap);
        if (f <= avail || cap <= Ep) break;
      }
      w.kb = (int)cap;
      break;
    }
    case ROLE_G_GATE:
    case ROLE_G_CAND: {
      const size_t H = c->dims.hidden, Np = amp_round16(c->max_len), Hs = amp_ldrow((int)H), Cs = amp_ldrow((int)(2 * H));
      if ((Rp / 16) * ((amp_round16((int)C) + 63) / 64) > 32) return 0;
      size_t cap = std::max<size_t>(Np, 64);
      for (;; cap -= 16) {
        f = wfl + r4(Rp) + (size_t)(amp_round16((int)C) + 63) / 64 * 64 + r4(cap * Cs) + r4(cap * Hs);
        if (w.role == ROLE_G_CAND) f += r4(cap * H);
        if (f <= avail || cap <= Np) break;
      }
      w.kb = (int)cap;
      break;
    }
    case ROLE_G_READOUT:
      f = wfl + r4(c->dims.hidden) + AMP_THREADS;
      break;
    case ROLE_MLP_LIN:   // weights and a gradient accumulator of the same layout
      f = 2 * wfl + r4(ldw) + r4(R) + r4(R) + r4(C) + r4(8 * std::max(R, C));
      break;
    default:   // RNN output layer
      f = wfl + r4(C) + r4(R) + r4(R) + r4(C) + r4(8 * std::max(R, C));
  }
  return f <= avail ? f : 0;
}

}  // namespace

extern "C" {

int amp_create(amp_ctx** out, void* dev_arena, size_t arena_bytes, void* hip_stream) {
  if (!out) return AMP_EINVAL;
  *out = nullptr;
  if (!dev_arena || arena_bytes < (1u << 20) || ((uintptr_t)dev_arena & 255)) return AMP_EINVAL;
  amp_ctx* c = new amp_ctx();
  c->arena = (char*)dev_arena;
  c->arena_bytes = arena_bytes;
  c->stream = (hipStream_t)hip_stream;
  *out = c;
  return AMP_OK;
}

// One context at a time may use a device's built-in arena.
static std::mutex g_static_mu;
static bool g_static_in_use[64] = {};

int amp_create_static(amp_ctx** out, void* hip_stream) {
  if (!out) return AMP_EINVAL;
  *out = nullptr;
  void* ptr = nullptr;
  size_t bytes = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return AMP_EDEVICE;
  if (amp_static_arena(&ptr, &bytes) != hipSuccess) return AMP_EDEVICE;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (g_static_in_use[dev]) return AMP_ESTATE;
    g_static_in_use[dev] = true;
  }
  amp_ctx* c = new amp_ctx();
  c->arena = (char*)ptr;
  c->arena_bytes = bytes;
  c->stream = (hipStream_t)hip_stream;
  c->static_dev = dev;
  *out = c;
  return AMP_OK;
}

void amp_destroy(amp_ctx* ctx) {
  if (ctx && ctx->static_dev >= 0) {
    std::lock_guard<std::mutex> lock(g_static_mu);
    g_static_in_use[ctx->static_dev] = false;
  }
  delete ctx;
}

const char* amp_last_error(amp_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int amp_measure_peaks(void* dev_buf, size_t bytes, void* hip_stream, double* lds_bytes_per_s_per_cu,
                      double* hbm_read_bytes_per_s) {
  if (!dev_buf || bytes < (64u << 20) || ((uintptr_t)dev_buf & 255) || !lds_bytes_per_s_per_cu || !hbm_read_bytes_per_s)
    return AMP_EINVAL;
  hipStream_t stream = (hipStream_t)hip_stream;
  int dev_id = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev_id) != hipSuccess || hipGetDeviceProperties(&prop, dev_id) != hipSuccess) return AMP_EDEVICE;
  double sec = 0, per_wg = 0;
  // the first float of the buffer doubles as the kernels' (never written) sink
  if (amp_peak_lds_launch(prop.multiProcessorCount, 20000, (float*)dev_buf, stream, &sec, &per_wg) != hipSuccess || sec <= 0)
    return AMP_EDEVICE;
  *lds_bytes_per_s_per_cu = per_wg / sec;
  if (amp_peak_hbm_launch(dev_buf, bytes, (float*)dev_buf, stream, &sec) != hipSuccess || sec <= 0) return AMP_EDEVICE;
  *hbm_read_bytes_per_s = (double)(bytes / 16 * 16) / sec;
  return AMP_OK;
}

}  // extern "C"

namespace {

// A recognised graph becomes the model the kernel has workers for: the parameterized nodes in the model's
// numbering, with the layout facts the workers need.
int lower_model(amp_ctx* c, int model, const amp_model_dims* d) {
  c->node_replicas = 1;
  switch (model) {
    case AMP_MODEL_MLP:
      if (!positive({d->d_in, d->hidden, d->n_class})) return fail(c, AMP_EINVAL, "mlp: sizes must be >= 1");
      if (d->n_class > 64) return fail(c, AMP_EUNSUPPORTED, "mlp: n_class > 64");
      c->nodes = {make_node("lin1", d->hidden, d->d_in, 1), make_node("lin2", d->hidden, d->hidden, 1),
                  make_node("lin3", d->n_class, d->hidden, 1)};
      break;
    case AMP_MODEL_RNN:
      if (!positive({d->vocab, d->emb, d->hidden, d->n_class})) return fail(c, AMP_EINVAL, "rnn: sizes must be >= 1");
      if (d->n_class > 64) return fail(c, AMP_EUNSUPPORTED, "rnn: n_class > 64");
      c->nodes = {make_node("lookup", d->vocab, d->emb, 0), make_node("cell", d->hidden, d->emb + d->hidden, 1),
                  make_node("out", d->n_class, d->hidden, 1)};
      // the cell's input is Concat(embedding, h): two column segments with a common padded width
      c->nodes[1].seg0 = d->emb;
      c->nodes[1].seg = d->hidden;
      c->nodes[1].segp = amp_round4(std::max(d->emb, d->hidden));
      break;
    case AMP_MODEL_TREE:
      if (!positive({d->vocab, d->emb, d->hidden, d->n_class})) return fail(c, AMP_EINVAL, "tree: sizes must be >= 1");
      if (d->n_class > 64) return fail(c, AMP_EUNSUPPORTED, "tree: n_class > 64");
      c->nodes = {make_node("lookup", d->vocab, d->emb, 0), make_node("leaf", 3 * d->hidden, d->emb, 1, 3),
                  make_node("branch", 5 * d->hidden, 2 * d->hidden, 1, 5), make_node("out", d->n_class, d->hidden, 1)};
      c->nodes[1].tiles = 5;
      c->nodes[2].tiles = 8;
      c->nodes[1].seg = d->emb;
      c->nodes[1].segp = amp_round4(d->emb);
      c->nodes[2].seg = d->hidden;
      c->nodes[2].segp = amp_round4(d->hidden);
      break;
    case AMP_MODEL_GGNN:
      if (!positive({d->n_node_types, d->hidden, d->n_edge_types, d->n_steps}))
        return fail(c, AMP_EINVAL, "ggnn: sizes must be >= 1");
      if (d->n_edge_types > 8) return fail(c, AMP_EUNSUPPORTED, "ggnn: more than 8 edge types");
      c->nodes.clear();
      c->nodes.push_back(make_node("lookup", d->n_node_types, d->hidden, 0));
      for (int k = 0; k < d->n_edge_types; ++k) {
        char nm[16];
        snprintf(nm, sizeof nm, "edge%d", k);
        c->nodes.push_back(make_node(nm, d->hidden, d->hidden, 1));
      }
      for (const char* nm : {"gz", "gr", "gh"}) c->nodes.push_back(make_node(nm, d->hidden, 2 * d->hidden, 1));
      c->nodes.push_back(make_node("readout", 1, d->hidden, 1));
      break;
    default: return fail(c, AMP_EINVAL, "unknown model");
  }
  c->model = model;
  c->dims = *d;
  return AMP_OK;
}

// Validates the ctx's graph, recognises it and lowers it.
int lower_graph(amp_ctx* c) {
  std::string err;
  if (int rc = ampgraph::validate(c->graph, err)) return fail(c, rc, "graph: %s", err.c_str());
  int model = 0;
  amp_model_dims dims{};
  if (int rc = ampgraph::recognise(c->graph, model, dims, c->param_of, err)) return fail(c, rc, "graph: %s", err.c_str());
  return lower_model(c, model, &dims);
}

// The canned builders describe their graph with the same two operations a caller has, then validate it.
int build_canned(amp_ctx* c, int model, const amp_model_dims* d, std::initializer_list<int> sizes, const char* what) {
  if (int r = check_build(c, d)) return r;
  if (c->graph.nodes.size() > 1) return fail(c, AMP_ESTATE, "nodes were already added to this context's graph");
  if (!positive(sizes)) return fail(c, AMP_EINVAL, "%s: sizes must be >= 1", what);
  c->graph = ampgraph::template_graph(model, *d);
  const int rc = lower_graph(c);
  if (rc) c->graph = ampgraph::Graph();
  return rc;
}

}  // namespace

extern "C" {

int amp_build_mlp(amp_ctx* c, const amp_model_dims* d) {
  return d ? build_canned(c, AMP_MODEL_MLP, d, {d->d_in, d->hidden, d->n_class}, "mlp") : fail(c, AMP_EINVAL, "null argument");
}
int amp_build_rnn(amp_ctx* c, const amp_model_dims* d) {
  return d ? build_canned(c, AMP_MODEL_RNN, d, {d->vocab, d->emb, d->hidden, d->n_class}, "rnn") : fail(c, AMP_EINVAL, "null argument");
}
int amp_build_treelstm(amp_ctx* c, const amp_model_dims* d) {
  return d ? build_canned(c, AMP_MODEL_TREE, d, {d->vocab, d->emb, d->hidden, d->n_class}, "tree") : fail(c, AMP_EINVAL, "null argument");
}
int amp_build_ggnn(amp_ctx* c, const amp_model_dims* d) {
  if (!d) return fail(c, AMP_EINVAL, "null argument");
  if (d->n_edge_types > 8) return fail(c, AMP_EUNSUPPORTED, "ggnn: more than 8 edge types");
  return build_canned(c, AMP_MODEL_GGNN, d, {d->n_node_types, d->hidden, d->n_edge_types, d->n_steps}, "ggnn");
}

int amp_add_node(amp_ctx* c, int kind, const amp_node_desc* desc, int* node_id) {
  if (!c || !desc || !node_id) return fail(c, AMP_EINVAL, "null argument");
  if (c->model || c->finalized) return fail(c, AMP_ESTATE, "add_node: the model graph is already built");
  if (kind <= AMP_NODE_CONTROLLER || kind > AMP_NODE_SINK) return fail(c, AMP_EINVAL, "add_node: unknown node kind %d", kind);
  if (desc->n_in < 0 || desc->n_out < 0 || desc->n_in > 64 || desc->n_out > 64 || desc->rows < 0 || desc->cols < 0)
    return fail(c, AMP_EINVAL, "add_node: bad description");
  if (c->graph.nodes.size() >= 4096) return fail(c, AMP_EFULL, "add_node: too many nodes");
  ampgraph::Node n;
  n.kind = kind;
  n.d = *desc;
  c->graph.nodes.push_back(n);
  *node_id = (int)c->graph.nodes.size() - 1;
  return AMP_OK;
}

int amp_connect(amp_ctx* c, int src, int src_port, int dst, int dst_port) {
  if (!c) return AMP_EINVAL;
  if (c->model || c->finalized) return fail(c, AMP_ESTATE, "connect: the model graph is already built");
  const int N = (int)c->graph.nodes.size();
  if (src < 0 || src >= N || dst < 1 || dst >= N) return fail(c, AMP_EINVAL, "connect: no such node (%d -> %d)", src, dst);
  if (src_port < 0 || dst_port < 0 || src_port >= 64 || dst_port >= 64) return fail(c, AMP_EINVAL, "connect: bad port");
  if (src == 0) {
    // the controller's ports are numbered in the order they are connected
    if (src_port != c->graph.nodes[0].d.n_out)
      return fail(c, AMP_EINVAL, "connect: the controller's next free port is %d", c->graph.nodes[0].d.n_out);
    c->graph.nodes[0].d.n_out++;
  }
  c->graph.connect(src, src_port, dst, dst_port);
  return AMP_OK;
}

int amp_validate_graph(amp_ctx* c) {
  if (!c) return AMP_EINVAL;
  if (c->model) return AMP_OK;   // validated when it was built
  if (c->graph.nodes.size() < 2) return fail(c, AMP_ESTATE, "validate_graph: no nodes added");
  return lower_graph(c);
}

int amp_get_node_index(amp_ctx* c, int graph_node, int* param_node) {
  if (!c || !param_node) return fail(c, AMP_EINVAL, "null argument");
  if (!c->model) return fail(c, AMP_ESTATE, "get_node_index: validate the graph first");
  if (graph_node < 0 || graph_node >= (int)c->param_of.size()) return fail(c, AMP_EINVAL, "no graph node %d", graph_node);
  *param_node = c->param_of[graph_node];
  return AMP_OK;
}

int amp_set_tiles(amp_ctx* c, int node_id, int n_tiles) {
  if (!c) return AMP_EINVAL;
  if (!c->model || c->finalized) return fail(c, AMP_ESTATE, "set_tiles: only between build and finalize");
  if (node_id < 0 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "set_tiles: no node %d", node_id);
  if (c->model == AMP_MODEL_GGNN) {
    // edge linears and the three GRU nodes, split by hidden unit; the partial results their tiles hand back are
    // summed by the consumers, which hold at most 12 parts of a kind in flight
    const int ne = c->dims.n_edge_types;
    if (node_id < 1 || node_id > 3 + ne)
      return fail(c, AMP_EUNSUPPORTED, "set_tiles: the graph model's lookup and readout cannot be tiled");
    if (n_tiles < 1 || n_tiles > 4 || n_tiles > c->nodes[node_id].block)
      return fail(c, AMP_EINVAL, "set_tiles: a graph node takes 1..min(4, hidden) tiles");
    c->nodes[node_id].tiles = n_tiles;
    return AMP_OK;
  }
  if (c->model != AMP_MODEL_TREE || (node_id != 1 && node_id != 2))
    return fail(c, AMP_EUNSUPPORTED, "set_tiles: only the tree model's leaf and branch nodes and the graph model's dense nodes can be tiled");
  if (n_tiles < 1 || n_tiles > 64 || n_tiles > c->nodes[node_id].block)
    return fail(c, AMP_EINVAL, "set_tiles: n_tiles must be in 1..min(64, hidden)");
  c->nodes[node_id].tiles = n_tiles;
  return AMP_OK;
}

int amp_set_weights_in_hbm(amp_ctx* c, int node_id, int on) {
  if (!c) return AMP_EINVAL;
  if (!c->model || c->finalized) return fail(c, AMP_ESTATE, "set_weights_in_hbm: only between build and finalize");
  if (node_id < 0 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "set_weights_in_hbm: no node %d", node_id);
  if (c->model != AMP_MODEL_TREE || (node_id != 1 && node_id != 2))
    return fail(c, AMP_EUNSUPPORTED, "set_weights_in_hbm: only the tree model's leaf and branch nodes");
  if (on && (c->dims.hidden % 4 || c->dims.emb % 4))
    return fail(c, AMP_EUNSUPPORTED, "set_weights_in_hbm: emb and hidden must be multiples of 4");
  c->nodes[node_id].in_hbm = on ? 1 : 0;
  return AMP_OK;
}

int amp_set_replicas(amp_ctx* c, int n_replicas) {
  if (!c) return AMP_EINVAL;
  if (!c->model || c->finalized) return fail(c, AMP_ESTATE, "set_replicas: only between build and finalize");
  if (n_replicas < 1 || n_replicas > 128) return fail(c, AMP_EINVAL, "set_replicas: 1..128 replicas");
  c->replicas = n_replicas;
  return AMP_OK;
}

int amp_set_node_replicas(amp_ctx* c, int node_id, int n_replicas) {
  if (!c) return AMP_EINVAL;
  if (!c->model || c->finalized) return fail(c, AMP_ESTATE, "set_node_replicas: only between build and finalize");
  if (c->model != AMP_MODEL_RNN || node_id != 1)
    return fail(c, AMP_EUNSUPPORTED, "set_node_replicas: only the RNN's recurrent cell (node 1) can be replicated");
  if (n_replicas < 1 || n_replicas > 64) return fail(c, AMP_EINVAL, "set_node_replicas: 1..64 replicas");
  // nodes 0..2 are the model's own; a replica r >= 1 adds a copy of the cell and of the table its worker hosts
  c->nodes.resize(3);
  for (int r = 1; r < n_replicas; ++r)
    for (int b = 0; b < 2; ++b) {
      HostNode n = c->nodes[b];
      n.name += ".r" + std::to_string(r);
      n.base = b;
      n.rep = r;
      n.dirty = true;
      c->nodes.push_back(n);
    }
  c->node_replicas = n_replicas;
  return AMP_OK;
}

int amp_set_group_sync(amp_ctx* c, int every_retirements) {
  if (!c) return AMP_EINVAL;
  if (!c->model) return fail(c, AMP_ESTATE, "set_group_sync: build a model first");
  if (every_retirements < 0) return fail(c, AMP_EINVAL, "set_group_sync: the interval must be >= 0");
  c->sync_every = every_retirements;
  return AMP_OK;
}

int amp_finalize(amp_ctx* c, int max_active_keys, int max_instance_len, int max_edges, size_t max_instances) {
  if (!c) return AMP_EINVAL;
  if (c->finalized) return fail(c, AMP_ESTATE, "finalize: already finalized");
  if (!c->model) {
    if (c->graph.nodes.size() < 2) return fail(c, AMP_ESTATE, "finalize: no model graph built");
    if (int rc = lower_graph(c)) return rc;   // a graph made with amp_add_node / amp_connect
  }
  if (max_active_keys < 1 || max_active_keys > AMP_MAX_MAK)
    return fail(c, AMP_EINVAL, "finalize: max_active_keys must be in 1..%d", AMP_MAX_MAK);
  if (max_instance_len < 1 || max_instances < 1) return fail(c, AMP_EINVAL, "finalize: sizes must be >= 1");
  if (c->model == AMP_MODEL_GGNN && max_edges < 1) return fail(c, AMP_EINVAL, "finalize: ggnn needs max_edges >= 1");
  const int NN = c->model == AMP_MODEL_TREE ? 2 * max_instance_len - 1 : max_instance_len;
  if (NN >= (1 << 20)) return fail(c, AMP_EINVAL, "finalize: max_instance_len too large");
  c->max_mak = c->mak = max_active_keys;
  c->max_len = max_instance_len;
  c->max_edges = max_edges;
  c->max_instances = max_instances;

  // ---- workers: one workgroup per node tile, worker 0 = controller
  c->workers.clear();
  auto add_worker = [&](int role, int node, int tile, int ntiles, int aux) {
    HostWorker w{};
    w.role = role;
    w.node = node;
    w.tile = tile;
    w.ntiles = ntiles;
    w.aux = aux;
    if (node >= 0) {
      const int blk = c->nodes[node].block;
      // graph nodes move their rows 16 bytes at a time when the hidden size allows: tiles of whole groups of 4 units
      const int grp = (c->model == AMP_MODEL_GGNN && ntiles > 1 && blk % 4 == 0 && blk / 4 >= ntiles) ? 4 : 1;
      const int nb = blk / grp, base = nb / ntiles, rem = nb % ntiles;
      w.u0 = grp * (tile * base + std::min(tile, rem));
      w.nu = grp * (base + (tile < rem ? 1 : 0));
    }
    c->workers.push_back(w);
  };
  add_worker(ROLE_CTRL, -1, 0, 1, 0);
  int nrings = 0;
  if (c->model == AMP_MODEL_MLP) {
    for (int l = 0; l < 3; ++l) add_worker(ROLE_MLP_LIN, l, 0, 1, l);
    for (size_t i = 0; i < c->workers.size(); ++i) c->workers[i].ring = (int)i;
    nrings = 4;
  } else if (c->model == AMP_MODEL_RNN) {
    // rings: 0 controller, 1 cell, 2 output layer, 3.. the cell's further replicas
    add_worker(ROLE_RNN_CELL, 1, 0, 1, 0);
    add_worker(ROLE_RNN_OUT, 2, 0, 1, 0);
    for (int r = 1; r < c->node_replicas; ++r) {
      add_worker(ROLE_RNN_CELL, 2 + 2 * r, 0, 1, 0);
      c->workers.back().rep = r;
    }
    for (size_t i = 0; i < c->workers.size(); ++i) c->workers[i].ring = (int)i;
    nrings = (int)c->workers.size();
  } else if (c->model == AMP_MODEL_TREE) {
    // rings: 0 controller, 1 lookup, 2 leaf (all leaf tiles), 3 branch (all branch tiles), 4 out
    add_worker(ROLE_TREE_LOOKUP, 0, 0, 1, 0);
    c->workers.back().ring = 1;
    for (int t = 0; t < c->nodes[1].tiles; ++t) {
      add_worker(ROLE_TREE_LEAF, 1, t, c->nodes[1].tiles, 0);
      c->workers.back().ring = 2;
    }
    for (int t = 0; t < c->nodes[2].tiles; ++t) {
      add_worker(ROLE_TREE_BRANCH, 2, t, c->nodes[2].tiles, 0);
      c->workers.back().ring = 3;
    }
    add_worker(ROLE_TREE_OUT, 3, 0, 1, 0);
    c->workers.back().ring = 4;
    nrings = 5;
  } else {
    // rings: 0 controller, 1 lookup, 2.. edge types, then gz, gr, gh, readout
    // every tile of a node reads the node's ring (ring = node + 1) with a head of its own
    const int ne = c->dims.n_edge_types;
    add_worker(ROLE_G_LOOKUP, 0, 0, 1, 0);
    for (int k = 0; k < ne; ++k)
      for (int t = 0; t < c->nodes[1 + k].tiles; ++t) add_worker(ROLE_G_EDGE, 1 + k, t, c->nodes[1 + k].tiles, k);
    for (int t = 0; t < c->nodes[1 + ne].tiles; ++t) add_worker(ROLE_G_GATE, 1 + ne, t, c->nodes[1 + ne].tiles, 0);
    for (int t = 0; t < c->nodes[2 + ne].tiles; ++t) add_worker(ROLE_G_GATE, 2 + ne, t, c->nodes[2 + ne].tiles, 1);
    for (int t = 0; t < c->nodes[3 + ne].tiles; ++t) add_worker(ROLE_G_CAND, 3 + ne, t, c->nodes[3 + ne].tiles, 0);
    add_worker(ROLE_G_READOUT, 4 + ne, 0, 1, 0);
    for (size_t i = 1; i < c->workers.size(); ++i) c->workers[i].ring = c->workers[i].node + 1;
    nrings = 6 + ne;
    int pe = 0;
    for (int k = 0; k < ne; ++k) pe += c->nodes[1 + k].tiles;
    const int pa = c->nodes[1 + ne].tiles + c->nodes[2 + ne].tiles + c->nodes[3 + ne].tiles;
    if (pe > 12 || pa > 12)
      return fail(c, AMP_EUNSUPPORTED, "finalize: at most 12 edge tiles and 12 GRU tiles in all (%d and %d asked for)", pe, pa);
  }
  if (c->workers.size() > AMP_MAX_WORKERS) return fail(c, AMP_EUNSUPPORTED, "finalize: too many workers");
  if (c->nodes.size() > AMP_MAX_NODES) return fail(c, AMP_EUNSUPPORTED, "finalize: too many nodes");
  if (c->node_replicas > 1 && c->replicas > 1)
    return fail(c, AMP_EUNSUPPORTED, "finalize: replicas of a node and replicas of the whole model do not combine");
  if (c->workers.size() * (size_t)c->replicas > 256)
    return fail(c, AMP_EUNSUPPORTED, "finalize: %zu workers x %d replicas exceed 256 workgroups", c->workers.size(), c->replicas);
  for (HostWorker& w : c->workers) {
    if ((w.role == ROLE_TREE_LEAF || w.role == ROLE_TREE_BRANCH) && c->nodes[w.node].in_hbm) w.aux = 1;
    size_t need = lds_floats(c, w) * 4;
    if ((need == 0 || need > AMP_DYN_LDS_BYTES) && (w.role == ROLE_TREE_LEAF || w.role == ROLE_TREE_BRANCH)) {
      // a tile that cannot keep its rows in LDS reads them from HBM instead
      w.aux = 1;
      need = lds_floats(c, w) * 4;
    }
    if (need == 0 || need > AMP_DYN_LDS_BYTES)
      return fail(c, AMP_EUNSUPPORTED, "finalize: the worker for node %d tile %d fits neither %d bytes of LDS nor the streamed mode (sizes a multiple of 4, at most 512 rows per tile); use more tiles",
                  w.node, w.tile, AMP_DYN_LDS_BYTES);
  }

  // ---- arena layout
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes);
    return o;
  };
  c->off_ctl = take(64);
  c->off_clock = take(64);
  c->off_slot_seq = take(sizeof(unsigned) * c->max_mak);
  c->off_smeta = take(16 * (size_t)c->max_mak);
  c->off_slot_inst = take(sizeof(int) * c->max_mak);
  const size_t per_inst_msgs = 4 * (size_t)NN + 8;
  c->ring_cap = next_pow2(per_inst_msgs * c->max_mak);
  c->off_ring_ent.assign(nrings, 0);
  c->off_ring_tail.assign(nrings, 0);
  for (int r = 0; r < nrings; ++r) {
    c->off_ring_ent[r] = take(8 * (size_t)c->ring_cap);
    c->off_ring_tail[r] = take(64);
  }
  c->sync_end = off;
  // the parameters of a node's replicas lie behind the node's own at equal distances (one averaging launch)
  for (size_t i = 0; i < c->nodes.size(); ++i)
    if (c->nodes[i].base < 0) {
      c->nodes[i].off_P = take(c->nodes[i].count() * 4);
      for (HostNode& n : c->nodes)
        if (n.base == (int)i) n.off_P = take(n.count() * 4);
    }
  for (HostNode& n : c->nodes) {
    const size_t b = n.count() * 4;
    n.off_G = take(b);
    n.off_M = take(b);
    n.off_V = take(b);
  }
  // what the copies of a replicated node publish for a synchronisation round, laid out like their parameters
  for (size_t i = 0; i < c->nodes.size(); ++i) {
    c->nodes[i].off_S = c->nodes[i].base < 0 ? 0 : c->nodes[i].off_S;
    bool copied = false;
    for (const HostNode& n : c->nodes) copied = copied || n.base == (int)i;
    if (c->nodes[i].base < 0 && copied) {
      c->nodes[i].off_S = take(c->nodes[i].count() * 4);
      for (HostNode& n : c->nodes)
        if (n.base == (int)i) n.off_S = take(n.count() * 4);
    }
  }
  for (HostWorker& w : c->workers) {
    w.off_state = take(64);
    if (w.node >= 0 && c->nodes[w.node].name.compare(0, 6, "lookup") != 0 && w.role != ROLE_TREE_OUT) {
      w.pend_bytes = pend_stride(c, w) * 4 * AMP_DENSE_MAX_MUF * rows_per_message(c, w);
      w.off_pend = take(w.pend_bytes);
    }
  }
  // model-specific per-slot storage
  const size_t mak = c->max_mak, H = c->dims.hidden;
  auto buf = [&](int i, size_t floats_per_slot) {
    c->buf_stride[i] = (long long)floats_per_slot;
    c->buf_bytes[i] = floats_per_slot * 4 * mak;
    c->off_buf[i] = take(c->buf_bytes[i]);
  };
  if (c->model == AMP_MODEL_MLP) {
    for (int i = 0; i < 4; ++i) buf(i, H);
  } else if (c->model == AMP_MODEL_RNN) {
    const size_t SP = c->nodes[1].segp;
    buf(0, ((size_t)c->max_len + 1) * SP);
    buf(1, (size_t)c->max_len * SP);
    buf(2, SP);
    c->buf_stride[3] = 0;
    c->buf_bytes[3] = 4 * 64 * SP * (size_t)c->node_replicas;   // one block per replica of the cell
    c->off_buf[3] = take(c->buf_bytes[3]);
  } else if (c->model == AMP_MODEL_TREE) {
    const size_t L = c->max_len, N2 = 2 * L - 1, E = c->dims.emb, Ep = amp_round4(c->dims.emb), Hp = amp_round4(c->dims.hidden);
    const size_t TL = c->nodes[1].tiles, TB = c->nodes[2].tiles;
    buf(0, L * Ep);
    buf(1, N2 * 2 * Hp);
    buf(2, N2 * 6 * H);
    buf(3, N2 * H);
    buf(4, N2 * TB * Hp);
    buf(5, N2 * H);
    buf(6, L * TL * Ep);
    buf(7, N2 * 4);
    c->buf_stride[10] = 0;
    c->buf_bytes[10] = 4 * (size_t)AMP_TREE_LOOKUP_MAX_MUF;
    c->off_buf[10] = take(c->buf_bytes[10]);
    c->buf_stride[11] = 0;
    c->buf_bytes[11] = 4 * (size_t)AMP_TREE_LOOKUP_MAX_MUF * E;
    c->off_buf[11] = take(c->buf_bytes[11]);
  } else if (c->model == AMP_MODEL_GGNN) {
    const size_t N = c->max_len, E = c->max_edges, S = c->dims.n_steps, T = c->dims.n_edge_types;
    size_t PE = 0;
    for (size_t k = 0; k < T; ++k) PE += c->nodes[1 + k].tiles;
    const size_t TH = c->nodes[3 + T].tiles, PA = c->nodes[1 + T].tiles + c->nodes[2 + T].tiles + TH;
    buf(0, (S + 1) * N * H);
    for (int i = 1; i <= 4; ++i) buf(i, S * N * H);
    buf(5, E * H);
    buf(6, N * H);
    buf(7, N * H);
    buf(8, TH * N * H);
    buf(9, PA * N * H);
    buf(10, 2 * PA * N * H);
    buf(11, PE * N * H);
    buf(12, N * H);
    buf(13, 8);
    buf(14, 16);   // slot descriptor: what the lookup found out about the instance, one 64-byte line
  }
  // every replica owns a copy of all of the above, rep_stride bytes apart
  c->rep_stride = align_up(off, 4096);
  c->static_end = c->rep_stride * (size_t)c->replicas;
  c->rep_admitted.assign(c->replicas, 0);
  if (c->static_end > c->arena_bytes)
    return fail(c, AMP_ENOMEM, "finalize: %s of %zu bytes is too small, %zu needed before instances", arena_name(c),
                c->arena_bytes, c->static_end);
  c->finalized = true;
  c->state_zeroed = false;
  return AMP_OK;
}

int amp_set_max_active_keys(amp_ctx* c, int mak) {
  if (!c) return AMP_EINVAL;
  if (!c->finalized) return fail(c, AMP_ESTATE, "set_max_active_keys: finalize first");
  if (mak < 1 || mak > c->max_mak) return fail(c, AMP_EINVAL, "max_active_keys must be in 1..%d", c->max_mak);
  c->mak = mak;
  return AMP_OK;
}

int amp_set_min_update_frequency(amp_ctx* c, int node_id, int muf) {
  if (!c) return AMP_EINVAL;
  if (!c->model) return fail(c, AMP_ESTATE, "set_min_update_frequency: build a model first");
  if (muf < 1) return fail(c, AMP_EINVAL, "min_update_frequency must be >= 1");
  if (node_id < -1 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "no node %d", node_id);
  if (c->finalized && c->state_zeroed) {
    // Gradients accumulated by earlier training calls stay with their node (Section 3: a node updates when its
    // own count reaches the threshold).  A threshold at or below a carried count would have had to fire already:
    // refuse it rather than let the count run past the threshold (and the pending-gradient list past its end).
    for (int r = 0; r < c->replicas; ++r)
      for (const HostWorker& w : c->workers) {
        if (w.node < 0) continue;
        unsigned st[4] = {0, 0, 0, 0};
        HIPCHK(c, hipMemcpyAsync(st, rep_ptr(c, r, w.off_state), sizeof st, hipMemcpyDeviceToHost, c->stream));
        HIPCHK(c, hipStreamSynchronize(c->stream));
        // word 0: gradients held by the worker's node; word 2: by the lookup the recurrent cell's worker hosts
        const int held[2] = {w.node, w.role == ROLE_RNN_CELL ? 0 : -1};
        const unsigned cnt[2] = {st[0], st[2]};
        for (int k = 0; k < 2; ++k)
          if (held[k] >= 0 && (node_id < 0 || node_id == held[k]) && cnt[k] >= (unsigned)muf)
            return fail(c, AMP_ESTATE,
                        "set_min_update_frequency: node %d (%s) holds %u accumulated gradients; a threshold of %d would "
                        "already have been reached -- choose a larger one, or train until the node has updated",
                        held[k], c->nodes[held[k]].name.c_str(), cnt[k], muf);
      }
  }
  for (int i = 0; i < (int)c->nodes.size(); ++i)
    if (node_id < 0 || node_id == i || c->nodes[i].base == node_id) c->nodes[i].muf = muf;   // a node and its replicas
  return AMP_OK;
}

int amp_set_optimizer(amp_ctx* c, int node_id, int kind, const amp_opt_params* p) {
  if (!c || !p) return fail(c, AMP_EINVAL, "null argument");
  if (!c->model) return fail(c, AMP_ESTATE, "set_optimizer: build a model first");
  if (kind < AMP_OPT_SGD || kind > AMP_OPT_ADAM) return fail(c, AMP_EINVAL, "unknown optimizer %d", kind);
  if (node_id < -1 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "no node %d", node_id);
  for (int i = 0; i < (int)c->nodes.size(); ++i) {
    if (node_id >= 0 && node_id != i && c->nodes[i].base != node_id) continue;   // a node and its replicas
    const bool lookup = c->nodes[i].name.compare(0, 6, "lookup") == 0;
    if (lookup && kind != AMP_OPT_SGD) {
      if (node_id >= 0) return fail(c, AMP_EUNSUPPORTED, "lookup nodes support SGD only");
      c->nodes[i].opt = AMP_OPT_SGD;   // "all nodes": the lookup keeps SGD with the given rate
      c->nodes[i].op = *p;
      continue;
    }
    c->nodes[i].opt = kind;
    c->nodes[i].op = *p;
  }
  return AMP_OK;
}

int amp_set_gradient_mean(amp_ctx* c, int mean) {
  if (!c) return AMP_EINVAL;
  c->mean = mean ? 1 : 0;
  return AMP_OK;
}

int amp_num_nodes(amp_ctx* c) { return c ? (int)c->nodes.size() : AMP_EINVAL; }
int amp_num_workers(amp_ctx* c) { return c ? (int)c->workers.size() * c->replicas : AMP_EINVAL; }

int amp_get_worker_stats(amp_ctx* c, double* wait_fraction, uint64_t* messages, int32_t* node_of_worker, size_t cap,
                         size_t* n, uint64_t* batches, double* phase_fraction) {
  if (!c) return AMP_EINVAL;
  const size_t wpr = c->workers.size(), nw = c->last_stats.size() / NSTAT;   // workers of the last call
  if (n) *n = nw ? nw : wpr * c->replicas;
  if (c->last_stats.empty()) return fail(c, AMP_ESTATE, "get_worker_stats: nothing run yet");
  if (cap < nw) return fail(c, AMP_ENOMEM, "get_worker_stats: %zu entries needed", nw);
  for (size_t w = 0; w < nw; ++w) {
    const unsigned long long* s = &c->last_stats[NSTAT * w];
    if (wait_fraction) wait_fraction[w] = s[3] ? (double)s[0] / (double)s[3] : 0.0;
    if (messages) messages[w] = s[1];
    if (batches) batches[w] = s[2];
    if (phase_fraction)
      for (int i = 0; i < 8; ++i) phase_fraction[8 * w + i] = s[3] ? (double)s[4 + i] / (double)s[3] : 0.0;
    if (node_of_worker) node_of_worker[w] = c->workers[w % wpr].node;
  }
  return AMP_OK;
}

int amp_get_worker_placement(amp_ctx* c, int32_t* xcc, size_t cap, size_t* n) {
  if (!c) return AMP_EINVAL;
  const size_t nw = c->last_stats.size() / NSTAT;
  if (n) *n = nw;
  if (c->last_stats.empty()) return fail(c, AMP_ESTATE, "get_worker_placement: nothing run yet");
  if (!xcc || cap < nw) return fail(c, AMP_ENOMEM, "get_worker_placement: %zu entries needed", nw);
  for (size_t w = 0; w < nw; ++w) xcc[w] = (int32_t)c->last_stats[NSTAT * w + 12];
  return AMP_OK;
}

int amp_param_count(amp_ctx* c, int node_id, size_t* n) {
  if (!c || !n) return fail(c, AMP_EINVAL, "null argument");
  if (node_id < 0 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "no node %d", node_id);
  *n = c->nodes[node_id].count();
  return AMP_OK;
}

int amp_set_params(amp_ctx* c, int node_id, const float* host, size_t n) {
  if (!c || !host) return fail(c, AMP_EINVAL, "null argument");
  if (node_id < 0 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "no node %d", node_id);
  HostNode& nd = c->nodes[node_id];
  if (n != nd.count())
    return fail(c, AMP_EINVAL, "set_params: node %d (%s) has %zu parameters, got %zu", node_id, nd.name.c_str(), nd.count(), n);
  std::memcpy(nd.params.data(), host, n * 4);
  nd.dirty = true;
  for (HostNode& r : c->nodes)   // its replicas start from the same values
    if (r.base == node_id) {
      r.params = nd.params;
      r.dirty = true;
    }
  return AMP_OK;
}

int amp_get_params(amp_ctx* c, int node_id, float* host, size_t cap, size_t* n) {
  if (!c || !host) return fail(c, AMP_EINVAL, "null argument");
  if (node_id < 0 || node_id >= (int)c->nodes.size()) return fail(c, AMP_EINVAL, "no node %d", node_id);
  HostNode& nd = c->nodes[node_id];
  if (n) *n = nd.count();
  if (cap < nd.count()) return fail(c, AMP_ENOMEM, "get_params: buffer holds %zu floats, %zu needed", cap, nd.count());
  if (c->finalized && !nd.dirty) {
    HIPCHK(c, hipMemcpyAsync(nd.params.data(), c->arena + nd.off_P, nd.count() * 4, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  std::memcpy(host, nd.params.data(), nd.count() * 4);
  return AMP_OK;
}

int amp_submit(amp_ctx* c, int which, uint64_t key, const amp_instance* in) {
  if (!c || !in) return fail(c, AMP_EINVAL, "null argument");
  if (!c->finalized) return fail(c, AMP_ESTATE, "submit: finalize first");
  if (which < 0 || which > 1) return fail(c, AMP_EINVAL, "submit: which must be 0 (train) or 1 (eval)");
  InstSet& S = c->sets[which];
  if (S.n() >= c->max_instances) return fail(c, AMP_EFULL, "submit: instance store holds %zu", c->max_instances);
  const amp_model_dims& d = c->dims;
  auto bad_label = [&](int l) { return l < 0 || l >= d.n_class; };
  switch (c->model) {
    case AMP_MODEL_MLP:
      if (in->n_x != d.d_in || !in->x) return fail(c, AMP_EINVAL, "submit: mlp instance needs x[%d]", d.d_in);
      if (in->n_labels != 1 || !in->labels || bad_label(in->labels[0])) return fail(c, AMP_EINVAL, "submit: bad label");
      S.x.insert(S.x.end(), in->x, in->x + d.d_in);
      S.lab.push_back(in->labels[0]);
      break;
    case AMP_MODEL_RNN:
      if (in->n_tokens < 1 || in->n_tokens > c->max_len || !in->tokens)
        return fail(c, AMP_EINVAL, "submit: sequence length must be in 1..%d", c->max_len);
      for (int t = 0; t < in->n_tokens; ++t)
        if (in->tokens[t] < 0 || in->tokens[t] >= d.vocab) return fail(c, AMP_EINVAL, "submit: token %d out of range", t);
      if (in->n_labels != 1 || !in->labels || bad_label(in->labels[0])) return fail(c, AMP_EINVAL, "submit: bad label");
      S.tok.insert(S.tok.end(), in->tokens, in->tokens + in->n_tokens);
      S.lab.push_back(in->labels[0]);
      break;
    case AMP_MODEL_TREE: {
      const int L = in->n_tokens, NN = 2 * L - 1;
      if (L < 1 || L > c->max_len || !in->tokens) return fail(c, AMP_EINVAL, "submit: leaves must be in 1..%d", c->max_len);
      if (in->n_nodes != NN || in->n_labels != NN || !in->labels || (L > 1 && (!in->left || !in->right)))
        return fail(c, AMP_EINVAL, "submit: a tree with %d leaves needs %d nodes and labels", L, NN);
      for (int l = 0; l < L; ++l)
        if (in->tokens[l] < 0 || in->tokens[l] >= d.vocab) return fail(c, AMP_EINVAL, "submit: token %d out of range", l);
      std::vector<int> par(NN, -1);
      for (int n = 0; n < NN; ++n) {
        if (bad_label(in->labels[n])) return fail(c, AMP_EINVAL, "submit: label of node %d out of range", n);
        if (n < L) {
          if (L > 1 && (in->left[n] != -1 || in->right[n] != -1))
            return fail(c, AMP_EINVAL, "submit: leaf %d has children", n);
          continue;
        }
        const int a = in->left[n], b = in->right[n];
        if (a < 0 || b < 0 || a >= n || b >= n || a == b)
          return fail(c, AMP_EINVAL, "submit: node %d needs two distinct children with smaller ids", n);
        if (par[a] != -1 || par[b] != -1) return fail(c, AMP_EINVAL, "submit: a child of node %d has two parents", n);
        par[a] = 2 * n;
        par[b] = 2 * n + 1;
      }
      for (int n = 0; n < NN - 1; ++n)
        if (par[n] == -1) return fail(c, AMP_EINVAL, "submit: node %d is not reachable from the root", n);
      S.tok.insert(S.tok.end(), in->tokens, in->tokens + L);
      S.lab.insert(S.lab.end(), in->labels, in->labels + NN);
      for (int n = 0; n < NN; ++n) {
        S.left.push_back(n < L ? -1 : in->left[n]);
        S.right.push_back(n < L ? -1 : in->right[n]);
        S.parent.push_back(par[n]);
        const int tn[4] = {n < L ? -1 : in->left[n], n < L ? -1 : in->right[n], par[n], in->labels[n]};
        S.tnode.insert(S.tnode.end(), tn, tn + 4);
      }
      break;
    }
    case AMP_MODEL_GGNN: {
      const int N = in->n_nodes, E = in->n_edges;
      if (N < 1 || N > c->max_len || in->n_tokens != N || !in->tokens)
        return fail(c, AMP_EINVAL, "submit: graph nodes must be in 1..%d with one type each", c->max_len);
      if (E < 1 || E > c->max_edges || !in->src || !in->dst || !in->etype)
        return fail(c, AMP_EINVAL, "submit: directed edges must be in 1..%d", c->max_edges);
      std::vector<int> indeg(N, 0);
      for (int v = 0; v < N; ++v)
        if (in->tokens[v] < 0 || in->tokens[v] >= d.n_node_types) return fail(c, AMP_EINVAL, "submit: node type %d out of range", v);
      for (int e = 0; e < E; ++e) {
        if (in->src[e] < 0 || in->src[e] >= N || in->dst[e] < 0 || in->dst[e] >= N)
          return fail(c, AMP_EINVAL, "submit: edge %d has an endpoint outside 0..%d", e, N - 1);
        if (in->etype[e] < 0 || in->etype[e] >= d.n_edge_types) return fail(c, AMP_EINVAL, "submit: edge %d has a bad type", e);
        indeg[in->dst[e]]++;
      }
      for (int v = 0; v < N; ++v)
        if (!indeg[v]) return fail(c, AMP_EINVAL, "submit: node %d has no incoming edge", v);
      if (!std::isfinite(in->target)) return fail(c, AMP_EINVAL, "submit: target is not finite");
      S.tok.insert(S.tok.end(), in->tokens, in->tokens + N);
      S.src.insert(S.src.end(), in->src, in->src + E);
      S.dst.insert(S.dst.end(), in->dst, in->dst + E);
      S.etype.insert(S.etype.end(), in->etype, in->etype + E);
      {
        int tc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int e = 0; e < E; ++e) tc[in->etype[e]]++;
        S.tcount.insert(S.tcount.end(), tc, tc + 8);
        // adjacency tables: incoming edges by destination; per type, the edges in ascending order and
        // their group positions by source node
        const int T = d.n_edge_types;
        int ts[9] = {0};
        for (int k = 0; k < 8; ++k) ts[k + 1] = ts[k] + tc[k];
        S.tstart.insert(S.tstart.end(), ts, ts + 9);
        std::vector<int> io(N + 1, 0), ie(E), te(E), tso((size_t)T * (N + 1), 0), tk(E), pos(E);
        for (int e = 0; e < E; ++e) io[in->dst[e] + 1]++;
        for (int v = 0; v < N; ++v) io[v + 1] += io[v];
        {
          std::vector<int> fill(io.begin(), io.end() - 1);
          for (int e = 0; e < E; ++e) ie[fill[in->dst[e]]++] = e;
        }
        {
          int fill[8];
          for (int k = 0; k < 8; ++k) fill[k] = ts[k];
          for (int e = 0; e < E; ++e) {
            pos[e] = fill[in->etype[e]] - ts[in->etype[e]];
            te[fill[in->etype[e]]++] = e;
          }
        }
        for (int e = 0; e < E; ++e) tso[(size_t)in->etype[e] * (N + 1) + in->src[e] + 1]++;
        for (int k = 0; k < T; ++k)
          for (int v = 0; v < N; ++v) tso[(size_t)k * (N + 1) + v + 1] += tso[(size_t)k * (N + 1) + v];
        {
          std::vector<int> fill(tso);
          for (int e = 0; e < E; ++e) {   // ascending e = ascending position inside its type
            const int k = in->etype[e];
            tk[ts[k] + fill[(size_t)k * (N + 1) + in->src[e]]++] = pos[e];
          }
        }
        S.inoff.insert(S.inoff.end(), io.begin(), io.end());
        S.inedge.insert(S.inedge.end(), ie.begin(), ie.end());
        S.tedge.insert(S.tedge.end(), te.begin(), te.end());
        S.tsoff.insert(S.tsoff.end(), tso.begin(), tso.end());
        S.tsk.insert(S.tsk.end(), tk.begin(), tk.end());
        for (int q = 0; q < E; ++q) {
          S.tsrc.push_back(in->src[te[q]]);
          S.tdst.push_back(in->dst[te[q]]);
        }
      }
      S.target.push_back(in->target);
      break;
    }
    default: return fail(c, AMP_ESTATE, "submit: no model");
  }
  if (c->model != AMP_MODEL_GGNN) S.target.push_back(0.f);
  S.tok_off.push_back((int)S.tok.size());
  S.lab_off.push_back((int)S.lab.size());
  S.node_off.push_back((int)S.left.size());
  S.edge_off.push_back((int)S.src.size());
  S.keys.push_back(key);
  S.dirty = true;
  return AMP_OK;
}

int amp_clear_instances(amp_ctx* c, int which) {
  if (!c || which < 0 || which > 1) return fail(c, AMP_EINVAL, "bad argument");
  c->sets[which].clear();
  return AMP_OK;
}

int amp_set_event_log(amp_ctx* c, size_t events_per_worker) {
  if (!c) return AMP_EINVAL;
  c->log_cap = events_per_worker;
  return AMP_OK;
}

int amp_set_admission(amp_ctx* c, int policy, double max_staleness) {
  if (!c) return AMP_EINVAL;
  if (policy != AMP_ADMIT_GREEDY && policy != AMP_ADMIT_BOUNDED) return fail(c, AMP_EINVAL, "unknown admission policy %d", policy);
  if (policy == AMP_ADMIT_BOUNDED && !(max_staleness >= 0)) return fail(c, AMP_EINVAL, "max_staleness must be >= 0");
  c->admit_bounded = policy == AMP_ADMIT_BOUNDED;
  c->max_staleness = max_staleness;
  return AMP_OK;
}

int amp_get_admission(amp_ctx* c, int* max_in_flight, int* final_limit) {
  if (!c) return AMP_EINVAL;
  if (max_in_flight) *max_in_flight = c->last_max_in_flight;
  if (final_limit) *final_limit = c->last_limit;
  return AMP_OK;
}

int amp_set_probe(amp_ctx* c, unsigned period, size_t max_entries) {
  if (!c) return AMP_EINVAL;
  if (period && c->model && c->model != AMP_MODEL_TREE) return fail(c, AMP_EUNSUPPORTED, "set_probe: the tree model only");
  if (period && c->replicas > 1) return fail(c, AMP_EUNSUPPORTED, "set_probe: not with replicas");
  if (period && max_entries < 1) return fail(c, AMP_EINVAL, "set_probe: max_entries must be >= 1");
  if (max_entries > (1u << 28)) return fail(c, AMP_EINVAL, "set_probe: max_entries too large");
  c->probe_period = period;
  c->probe_cap = max_entries;
  return AMP_OK;
}

int amp_get_probe(amp_ctx* c, float* host, size_t cap_floats, size_t* n_entries, size_t* entry_floats) {
  if (!c) return AMP_EINVAL;
  const size_t w = c->last_probe_w, n = w ? c->last_probe.size() / w : 0;
  if (n_entries) *n_entries = n;
  if (entry_floats) *entry_floats = w;
  if (!host) return AMP_OK;   // size query
  if (cap_floats < c->last_probe.size()) return fail(c, AMP_ENOMEM, "get_probe: %zu floats needed", c->last_probe.size());
  std::memcpy(host, c->last_probe.data(), c->last_probe.size() * 4);
  return AMP_OK;
}

int amp_set_watchdog(amp_ctx* c, double seconds) {
  if (!c) return AMP_EINVAL;
  if (!(seconds > 0) || seconds > 600) return fail(c, AMP_EINVAL, "watchdog must be in (0, 600] seconds");
  c->watchdog_s = seconds;
  return AMP_OK;
}

}  // extern "C"

// ---------------------------------------------------------------- running
namespace {

template <class T>
int upload(amp_ctx* c, size_t& off, const std::vector<T>& v, const void** dst) {
  const size_t bytes = std::max<size_t>(v.size() * sizeof(T), 4);
  if (off + bytes > c->arena_bytes) return fail(c, AMP_ENOMEM, "%s is too small for the instance set (%zu bytes more needed)", arena_name(c), bytes);
  *dst = c->arena + off;
  if (!v.empty()) HIPCHK(c, hipMemcpyAsync(c->arena + off, v.data(), v.size() * sizeof(T), hipMemcpyHostToDevice, c->stream));
  off = align_up(off + bytes);
  return AMP_OK;
}

template <class T>
void copy_range(std::vector<T>& dst, const std::vector<T>& src, size_t lo, size_t hi) {
  if (hi > lo) dst.insert(dst.end(), src.begin() + lo, src.begin() + hi);
}

// Appends instance i of S to D (all flattened arrays, adjacency tables included).
void append_instance(const amp_ctx* c, InstSet& D, const InstSet& S, size_t i) {
  const size_t T = (size_t)c->dims.n_edge_types;
  if (!S.x.empty()) copy_range(D.x, S.x, i * c->dims.d_in, (i + 1) * c->dims.d_in);
  D.target.push_back(S.target[i]);
  const size_t t0 = S.tok_off[i], t1 = S.tok_off[i + 1], l0 = S.lab_off[i], l1 = S.lab_off[i + 1];
  const size_t n0 = S.node_off[i], n1 = S.node_off[i + 1], e0 = S.edge_off[i], e1 = S.edge_off[i + 1];
  copy_range(D.tok, S.tok, t0, t1);
  copy_range(D.lab, S.lab, l0, l1);
  copy_range(D.left, S.left, n0, n1);
  copy_range(D.right, S.right, n0, n1);
  copy_range(D.parent, S.parent, n0, n1);
  if (!S.tnode.empty()) copy_range(D.tnode, S.tnode, 4 * n0, 4 * n1);
  copy_range(D.src, S.src, e0, e1);
  copy_range(D.dst, S.dst, e0, e1);
  copy_range(D.etype, S.etype, e0, e1);
  if (!S.tcount.empty()) {
    const size_t N = t1 - t0;
    copy_range(D.tcount, S.tcount, 8 * i, 8 * i + 8);
    copy_range(D.tstart, S.tstart, 9 * i, 9 * i + 9);
    copy_range(D.inoff, S.inoff, t0 + i, t0 + i + N + 1);
    copy_range(D.inedge, S.inedge, e0, e1);
    copy_range(D.tedge, S.tedge, e0, e1);
    copy_range(D.tsoff, S.tsoff, T * (t0 + i), T * (t0 + i) + T * (N + 1));
    copy_range(D.tsk, S.tsk, e0, e1);
    copy_range(D.tsrc, S.tsrc, e0, e1);
    copy_range(D.tdst, S.tdst, e0, e1);
  }
  D.tok_off.push_back((int)D.tok.size());
  D.lab_off.push_back((int)D.lab.size());
  D.node_off.push_back((int)D.left.size());
  D.edge_off.push_back((int)D.src.size());
  D.keys.push_back(S.keys[i]);
}

int upload_set(amp_ctx* c, size_t& off, const InstSet& S, DataDev& dd) {
  dd.n_inst = (int)S.n();
  dd.n_x = c->dims.d_in;
  int r;
  if ((r = upload(c, off, S.x, (const void**)&dd.x))) return r;
  if ((r = upload(c, off, S.target, (const void**)&dd.target))) return r;
  if ((r = upload(c, off, S.tok_off, (const void**)&dd.tok_off))) return r;
  if ((r = upload(c, off, S.tok, (const void**)&dd.tok))) return r;
  if ((r = upload(c, off, S.lab_off, (const void**)&dd.lab_off))) return r;
  if ((r = upload(c, off, S.lab, (const void**)&dd.lab))) return r;
  if ((r = upload(c, off, S.node_off, (const void**)&dd.node_off))) return r;
  if ((r = upload(c, off, S.left, (const void**)&dd.left))) return r;
  if ((r = upload(c, off, S.right, (const void**)&dd.right))) return r;
  if ((r = upload(c, off, S.parent, (const void**)&dd.parent))) return r;
  if ((r = upload(c, off, S.edge_off, (const void**)&dd.edge_off))) return r;
  if ((r = upload(c, off, S.src, (const void**)&dd.src))) return r;
  if ((r = upload(c, off, S.dst, (const void**)&dd.dst))) return r;
  if ((r = upload(c, off, S.etype, (const void**)&dd.etype))) return r;
  if ((r = upload(c, off, S.tcount, (const void**)&dd.tcount))) return r;
  if ((r = upload(c, off, S.tnode, (const void**)&dd.tnode))) return r;
  if ((r = upload(c, off, S.inoff, (const void**)&dd.inoff))) return r;
  if ((r = upload(c, off, S.inedge, (const void**)&dd.inedge))) return r;
  if ((r = upload(c, off, S.tstart, (const void**)&dd.tstart))) return r;
  if ((r = upload(c, off, S.tedge, (const void**)&dd.tedge))) return r;
  if ((r = upload(c, off, S.tsoff, (const void**)&dd.tsoff))) return r;
  if ((r = upload(c, off, S.tsk, (const void**)&dd.tsk))) return r;
  if ((r = upload(c, off, S.tsrc, (const void**)&dd.tsrc))) return r;
  if ((r = upload(c, off, S.tdst, (const void**)&dd.tdst))) return r;
  return AMP_OK;
}

// Puts set S into the arena at `begin`, dealt to R replicas: replica r gets instances r, r + R, r + 2R, ...
int make_resident(amp_ctx* c, const InstSet& S, int R, size_t begin, Resident& res) {
  res.valid = false;
  res.R = R;
  res.begin = begin;
  res.dd.assign(R, DataDev());
  res.n.assign(R, 0);
  size_t off = begin;
  if (R == 1) {
    if (int rc = upload_set(c, off, S, res.dd[0])) return rc;
    res.n[0] = S.n();
  } else {
    std::vector<InstSet> parts(R);
    for (size_t i = 0; i < S.n(); ++i) append_instance(c, parts[i % R], S, i);
    for (int r = 0; r < R; ++r) {
      if (int rc = upload_set(c, off, parts[r], res.dd[r])) return rc;
      res.n[r] = parts[r].n();
    }
    // the copies above read pageable host memory: they have left `parts` before it goes away
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  res.end = off;
  res.valid = true;
  return AMP_OK;
}

// One launch: every replica trains (or evaluates) `epochs` passes over its own instance set.
// losses / correct: per replica, per admission of this launch.  Launch outputs lie from `out_begin` on.
// adm: per replica, one word per admission of the launch -- the instance's index in the replica's set, sign bit set for
// a forward-only (evaluation) instance; nullptr = `epochs` passes over the set in order, all of the launch's kind.
int launch_once(amp_ctx* c, const Resident& res, size_t out_begin, int epochs, bool train,
                std::vector<std::vector<float>>& losses, std::vector<std::vector<int>>& correct, double& seconds,
                const std::vector<std::vector<int>>* adm = nullptr) {
  const int R = res.R;
  const size_t wpr = c->workers.size();
  size_t off = out_begin;
  auto take = [&](size_t bytes) -> size_t {
    size_t o = off;
    off = align_up(off + bytes);
    return o;
  };
  std::vector<AmpDev> Ds(R);
  std::vector<size_t> off_loss(R), off_correct(R), off_yhat(R), n_total(R), off_stats(R), off_adm(R);
  std::vector<std::vector<size_t>> off_log(R, std::vector<size_t>(wpr)), off_logn(R, std::vector<size_t>(wpr));
  const size_t log_cap = train ? c->log_cap : 0;
  const size_t off_devs = take(sizeof(AmpDev) * R);
  // what the host reads after every launch lies together: one copy brings it back
  const size_t res_begin = off;
  for (int r = 0; r < R; ++r) {
    n_total[r] = adm ? (*adm)[r].size() : res.n[r] * (size_t)epochs;
    off_loss[r] = take(n_total[r] * 4);
    off_correct[r] = take(n_total[r] * 4);
    off_stats[r] = take(8 * NSTAT * wpr);
  }
  const size_t res_end = off;
  for (int r = 0; r < R; ++r) {
    off_yhat[r] = take(n_total[r] * 4);
    for (size_t w = 0; w < wpr; ++w) off_logn[r][w] = take(64);
  }
  const size_t off_probe_n = take(64);
  const size_t zero_end = off;
  for (int r = 0; r < R; ++r)
    for (size_t w = 0; w < wpr; ++w) off_log[r][w] = take(8 * std::max<size_t>(log_cap, 1));
  // the probe buffer (first replica only): entries of 4 header words and the wider of the two payloads
  const bool probing = train && c->probe_period && c->model == AMP_MODEL_TREE;
  const size_t probe_w = 4 + (size_t)std::max(amp_round4(c->dims.hidden), amp_round4(c->dims.emb));
  const size_t off_probe = take(probing ? c->probe_cap * probe_w * 4 : 4);
  for (int r = 0; r < R; ++r) off_adm[r] = take(4 * std::max<size_t>(n_total[r], 1));
  if (off > c->arena_bytes) return fail(c, AMP_ENOMEM, "%s of %zu bytes is too small, %zu needed", arena_name(c), c->arena_bytes, off);
  HIPCHK(c, hipMemsetAsync(c->arena + res_begin, 0, zero_end - res_begin, c->stream));
  // the admission list of every replica
  std::vector<std::vector<int>> plain;
  if (!adm) {
    plain.resize(R);
    for (int r = 0; r < R; ++r) {
      plain[r].resize(n_total[r]);
      for (size_t i = 0; i < n_total[r]; ++i) plain[r][i] = (int)(i % res.n[r]);
    }
    adm = &plain;
  }
  for (int r = 0; r < R; ++r)
    if (n_total[r])
      HIPCHK(c, hipMemcpyAsync(c->arena + off_adm[r], (*adm)[r].data(), 4 * n_total[r], hipMemcpyHostToDevice, c->stream));
  for (int r = 0; r < R; ++r) {
    AmpDev& D = Ds[r];
    std::memset(&D, 0, sizeof D);
    D.data = res.dd[r];
    // stop word, clock, slot tables and every ring of this replica
    HIPCHK(c, hipMemsetAsync(rep_ptr(c, r, 0), 0, c->sync_end, c->stream));
    for (size_t i = 0; i < c->off_ring_ent.size(); ++i) {
      D.ring[i].ent = (unsigned long long*)rep_ptr(c, r, c->off_ring_ent[i]);
      D.ring[i].tail = (unsigned*)rep_ptr(c, r, c->off_ring_tail[i]);
      D.ring[i].mask = c->ring_cap - 1;
    }
    for (size_t i = 0; i < c->nodes.size(); ++i) {
      const HostNode& n = c->nodes[i];
      NodeDev& nd = D.node[i];
      nd.P = (float*)rep_ptr(c, r, n.off_P);
      nd.G = (float*)rep_ptr(c, r, n.off_G);
      nd.M = (float*)rep_ptr(c, r, n.off_M);
      nd.V = (float*)rep_ptr(c, r, n.off_V);
      nd.S = n.off_S ? (float*)rep_ptr(c, r, n.off_S) : nullptr;
      nd.rows = n.rows;
      nd.cols = n.cols;
      nd.has_bias = n.has_bias;
      nd.muf = n.muf;
      nd.opt = n.opt;
      nd.mean = c->mean;
      nd.nblocks = n.nblocks;
      nd.block = n.block;
      nd.lr = n.op.lr;
      nd.mom = n.op.momentum;
      nd.b1 = n.op.beta1;
      nd.b2 = n.op.beta2;
      nd.eps = n.op.eps;
      nd.seg = n.seg ? n.seg : n.cols;
      nd.segp = n.seg ? n.segp : n.cols;
      nd.seg0 = n.seg ? n.first_seg() : n.cols;
    }
    for (size_t i = 0; i < wpr; ++i) {
      const HostWorker& w = c->workers[i];
      WorkerDev& wd = D.worker[i];
      wd.role = w.role;
      wd.node = w.node;
      wd.tile = w.tile;
      wd.ntiles = w.ntiles;
      wd.u0 = w.u0;
      wd.nu = w.nu;
      wd.ring = w.ring;
      wd.aux = w.aux;
      wd.wstate = (unsigned*)rep_ptr(c, r, w.off_state);
      wd.log = (unsigned long long*)(c->arena + off_log[r][i]);
      wd.log_n = (unsigned*)(c->arena + off_logn[r][i]);
      wd.log_cap = (unsigned)log_cap;
      wd.stats = (unsigned long long*)(c->arena + off_stats[r]) + NSTAT * i;
      wd.pend = w.pend_bytes ? (float*)rep_ptr(c, r, w.off_pend) : nullptr;
      wd.kb = w.kb;
      wd.rep = w.rep;
    }
    D.model = c->model;
    D.n_workers = (int)wpr;
    D.n_nodes = (int)c->nodes.size();
    D.mak = c->mak;
    D.d_in = c->dims.d_in;
    D.hidden = c->dims.hidden;
    D.n_class = c->dims.n_class;
    D.vocab = c->dims.vocab;
    D.emb = c->dims.emb;
    D.n_node_types = c->dims.n_node_types;
    D.n_edge_types = c->dims.n_edge_types;
    D.n_steps = c->dims.n_steps;
    D.max_len = c->max_len;
    D.max_edges = c->max_edges;
    D.train = train ? 1 : 0;
    if (c->model == AMP_MODEL_TREE) {
      D.tiles_leaf = c->nodes[1].tiles;
      D.tiles_branch = c->nodes[2].tiles;
    }
    if (c->model == AMP_MODEL_GGNN) {
      const int ne = c->dims.n_edge_types;
      for (int k = 0; k < 8; ++k) {
        D.g_tiles[k] = k < ne ? c->nodes[1 + k].tiles : 0;
        D.g_eoff[k + 1] = D.g_eoff[k] + D.g_tiles[k];
      }
      D.g_PE = D.g_eoff[8];
      for (int k = 0; k < 3; ++k) D.g_tiles[8 + k] = c->nodes[1 + ne + k].tiles;
      D.g_PA = D.g_tiles[8] + D.g_tiles[9] + D.g_tiles[10];
    }
    D.admit_bounded = train ? c->admit_bounded : 0;
    D.node_replicas = c->node_replicas;
    D.sync_every = train && c->node_replicas > 1 ? c->sync_every : 0;
    D.max_staleness = (float)c->max_staleness;
    D.n_updaters = (int)wpr - 1;   // every worker but the controller applies updates
    D.n_total = (unsigned)n_total[r];
    D.first_seq = train ? c->rep_admitted[r] : 0;
    D.ctl = (unsigned*)rep_ptr(c, r, c->off_ctl);
    D.slot_seq = (unsigned*)rep_ptr(c, r, c->off_slot_seq);
    D.smeta = (int*)rep_ptr(c, r, c->off_smeta);
    D.slot_inst = (int*)rep_ptr(c, r, c->off_slot_inst);
    D.adm_inst = (const int*)(c->arena + off_adm[r]);
    D.loss_out = (float*)(c->arena + off_loss[r]);
    D.correct_out = (int*)(c->arena + off_correct[r]);
    D.yhat_out = (float*)(c->arena + off_yhat[r]);
    D.clock = (unsigned long long*)rep_ptr(c, r, c->off_clock);
    D.watchdog_ticks = (long long)(c->watchdog_s * 1.0e8);   // wall_clock64 counts at 100 MHz
    D.probe = (float*)(c->arena + off_probe);
    D.probe_n = (unsigned*)(c->arena + off_probe_n);
    D.probe_period = probing && r == 0 ? c->probe_period : 0;
    D.probe_cap = (unsigned)c->probe_cap;
    D.probe_w = (int)probe_w;
    for (int i = 0; i < AMP_MAX_BUFS; ++i) {
      D.buf[i] = c->buf_bytes[i] ? rep_ptr(c, r, c->off_buf[i]) : nullptr;
      D.stride[i] = c->buf_stride[i];
    }
  }
  HIPCHK(c, hipMemcpyAsync(c->arena + off_devs, Ds.data(), sizeof(AmpDev) * R, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));

  hipEvent_t e0, e1;
  HIPCHK(c, hipEventCreate(&e0));
  HIPCHK(c, hipEventCreate(&e1));
  HIPCHK(c, hipEventRecord(e0, c->stream));
  HIPCHK(c, amp_launch((const AmpDev*)(c->arena + off_devs), R, (int)wpr, c->stream));
  HIPCHK(c, hipEventRecord(e1, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  float ms = 0;
  HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  seconds += ms * 1e-3;

  std::vector<unsigned> ctl(8 * (size_t)R);
  HIPCHK(c, hipMemcpy2D(ctl.data(), 32, rep_ptr(c, 0, c->off_ctl), c->rep_stride, 32, R, hipMemcpyDeviceToHost));
  if (train) c->last_max_in_flight = c->last_limit = 0;
  for (int r = 0; r < R; ++r) {
    if (train) {
      c->last_max_in_flight = std::max(c->last_max_in_flight, (int)ctl[8 * r + 4]);
      c->last_limit = std::max(c->last_limit, (int)ctl[8 * r + 5]);
    }
    if (ctl[8 * r]) {
      const unsigned why_code = ctl[8 * r];
      const char* why = why_code == ABORT_WATCHDOG ? "a worker waited longer than the watchdog allows"
                        : why_code == ABORT_LOG_FULL ? "event record full"
                        : why_code == ABORT_PLACEMENT ? "a workgroup of a packed launch ran on another die than its block index implies"
                                                      : "inconsistent state";
      c->state_zeroed = false;   // device state is unreliable after an aborted run
      for (HostNode& n : c->nodes) n.dirty = true;
      return fail(c, AMP_EDEVICE, "kernel stopped itself: %s (replica %d, worker %u)", why, r, ctl[8 * r + 2]);
    }
  }
  if (probing) {
    unsigned asked = 0;
    HIPCHK(c, hipMemcpy(&asked, c->arena + off_probe_n, 4, hipMemcpyDeviceToHost));
    const size_t got = std::min<size_t>(asked, c->probe_cap), base = c->last_probe.size();
    c->last_probe_w = probe_w;
    c->last_probe.resize(base + got * probe_w);
    if (got) HIPCHK(c, hipMemcpy(c->last_probe.data() + base, c->arena + off_probe, got * probe_w * 4, hipMemcpyDeviceToHost));
  }
  std::vector<char> back(res_end - res_begin);
  HIPCHK(c, hipMemcpy(back.data(), c->arena + res_begin, back.size(), hipMemcpyDeviceToHost));
  c->last_stats.assign(NSTAT * wpr * R, 0);
  for (int r = 0; r < R; ++r) {
    std::memcpy(c->last_stats.data() + NSTAT * wpr * r, back.data() + (off_stats[r] - res_begin), 8 * NSTAT * wpr);
    const size_t base = losses[r].size();
    losses[r].resize(base + n_total[r]);
    correct[r].resize(base + n_total[r]);
    std::memcpy(losses[r].data() + base, back.data() + (off_loss[r] - res_begin), n_total[r] * 4);
    std::memcpy(correct[r].data() + base, back.data() + (off_correct[r] - res_begin), n_total[r] * 4);
    if (train) c->rep_admitted[r] += (unsigned)n_total[r];
    if (log_cap) {
      std::vector<unsigned long long> raw(log_cap);
      for (size_t w = 0; w < wpr; ++w) {
        unsigned n = 0;
        HIPCHK(c, hipMemcpy(&n, c->arena + off_logn[r][w], 4, hipMemcpyDeviceToHost));
        if (n > log_cap) n = (unsigned)log_cap;
        if (n) HIPCHK(c, hipMemcpy(raw.data(), c->arena + off_log[r][w], 8 * (size_t)n, hipMemcpyDeviceToHost));
        for (unsigned i = 0; i < n; ++i) {
          amp_event e;
          e.worker = (uint16_t)(r * wpr + w);
          e.kind = (uint8_t)((raw[i] >> 28) & 0xf);
          e.node = (uint8_t)((raw[i] >> 20) & 0xff);
          e.local = (uint32_t)(raw[i] & 0xfffff);
          e.seq = (uint32_t)(raw[i] >> 32);
          c->launch_events[r * wpr + w].push_back(e);
        }
      }
    }
  }
  return AMP_OK;
}

int prepare_device(amp_ctx* c);
int run_prepared(amp_ctx* c, int which, int epochs, bool train, amp_eval_result* ev);

int run(amp_ctx* c, int which, int epochs, bool train, amp_eval_result* ev) {
  InstSet& S = c->sets[which];
  if (S.n() == 0) return fail(c, AMP_ESTATE, "no instances submitted");
  if (c->model == AMP_MODEL_TREE && c->nodes[0].muf > AMP_TREE_LOOKUP_MAX_MUF)
    return fail(c, AMP_EUNSUPPORTED, "the tree lookup supports min_update_frequency up to %d", AMP_TREE_LOOKUP_MAX_MUF);
  for (const HostNode& n : c->nodes)
    if (n.name.compare(0, 6, "lookup") != 0 && n.muf > AMP_DENSE_MAX_MUF)
      return fail(c, AMP_EUNSUPPORTED, "dense nodes support min_update_frequency up to %d", AMP_DENSE_MAX_MUF);
  if (S.n() * (size_t)epochs >= 0xffffffffull) return fail(c, AMP_EINVAL, "too many admissions for one call");
  // evaluation runs on the first replica alone: after a training call all replicas hold the same parameters
  const int R = train ? c->replicas : 1;
  const size_t wpr = c->workers.size();
  if (S.n() < (size_t)R) return fail(c, AMP_EINVAL, "fewer instances (%zu) than replicas (%d)", S.n(), R);
  if (int rc = prepare_device(c)) return rc;
  return run_prepared(c, which, epochs, train, ev);
}

// Everything a launch needs on the device besides the instances: a device with enough compute units, zeroed
// accumulators and counters at the first use, the parameters the host changed.
int prepare_device(amp_ctx* c) {
  const size_t wpr = c->workers.size();
  int dev_id = 0;
  HIPCHK(c, hipGetDevice(&dev_id));
  hipDeviceProp_t prop;
  HIPCHK(c, hipGetDeviceProperties(&prop, dev_id));
  if ((int)(wpr * c->replicas) > prop.multiProcessorCount)
    return fail(c, AMP_EUNSUPPORTED, "%zu workers do not fit %d compute units", wpr * c->replicas, prop.multiProcessorCount);

  if (!c->state_zeroed) {
    // accumulators, optimizer slots, per-worker counters start at zero
    for (int r = 0; r < c->replicas; ++r) {
      for (HostNode& n : c->nodes) {
        HIPCHK(c, hipMemsetAsync(rep_ptr(c, r, n.off_G), 0, n.count() * 4, c->stream));
        HIPCHK(c, hipMemsetAsync(rep_ptr(c, r, n.off_M), 0, n.count() * 4, c->stream));
        HIPCHK(c, hipMemsetAsync(rep_ptr(c, r, n.off_V), 0, n.count() * 4, c->stream));
      }
      for (HostWorker& w : c->workers) HIPCHK(c, hipMemsetAsync(rep_ptr(c, r, w.off_state), 0, 64, c->stream));
      for (int i = 0; i < AMP_MAX_BUFS; ++i)
        if (c->buf_bytes[i]) HIPCHK(c, hipMemsetAsync(rep_ptr(c, r, c->off_buf[i]), 0, c->buf_bytes[i], c->stream));
    }
    c->state_zeroed = true;
  }
  for (HostNode& n : c->nodes)
    if (n.dirty) {
      for (int r = 0; r < c->replicas; ++r)
        HIPCHK(c, hipMemcpyAsync(rep_ptr(c, r, n.off_P), n.params.data(), n.count() * 4, hipMemcpyHostToDevice, c->stream));
      n.dirty = false;
    }
  return AMP_OK;
}

int run_prepared(amp_ctx* c, int which, int epochs, bool train, amp_eval_result* ev) {
  InstSet& S = c->sets[which];
  const int R = train ? c->replicas : 1;
  const size_t wpr = c->workers.size();
  // The set stays in the arena from call to call: the training set first, the evaluation set behind it.
  Resident& res = c->resident[which];
  const Resident& other = c->resident[1 - which];
  const size_t begin = which == 1 && other.valid ? other.end : c->static_end;
  if (S.dirty || !res.valid || res.R != R || res.begin != begin) {
    if (which == 0) c->resident[1].valid = false;
    if (int rc = make_resident(c, S, R, begin, res)) return rc;
    S.dirty = false;
  }
  const size_t out_begin = std::max(res.end, other.valid ? other.end : (size_t)0);
  std::vector<std::vector<float>> losses(R);
  std::vector<std::vector<int>> correct(R);
  double seconds = 0;
  c->launch_events.assign(wpr * R, std::vector<amp_event>());
  if (train) c->last_probe.clear();
  // with replicas the parameters are averaged at the end of every epoch (Section 5), hence one launch per epoch
  const bool averaged = R > 1 || (train && c->node_replicas > 1);
  const int launches = averaged ? epochs : 1, per_launch = averaged ? 1 : epochs;
  for (int l = 0; l < launches; ++l) {
    if (int rc = launch_once(c, res, out_begin, per_launch, train, losses, correct, seconds)) return rc;
    if (R > 1)
      for (HostNode& n : c->nodes)
        HIPCHK(c, amp_average((float*)rep_ptr(c, 0, n.off_P), c->rep_stride / 4, R, n.count(), c->stream));
    if (train && c->node_replicas > 1)
      // the copies of a node lie at equal distances behind it
      for (size_t i = 0; i < c->nodes.size(); ++i) {
        const HostNode& n = c->nodes[i];
        int copies = 1;
        for (const HostNode& o : c->nodes) copies += o.base == (int)i;
        if (n.base < 0 && copies > 1)
          HIPCHK(c, amp_average((float*)rep_ptr(c, 0, n.off_P), align_up(n.count() * 4) / 4, copies, n.count(), c->stream));
      }
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));

  // results in submit order, epoch by epoch
  const size_t n = S.n(), n_total = n * (size_t)epochs;
  std::vector<float> loss(n_total);
  std::vector<int> corr(n_total);
  for (int e = 0; e < epochs; ++e)
    for (size_t i = 0; i < n; ++i) {
      const size_t r = i % R, j = i / R;
      loss[e * n + i] = losses[r][(size_t)e * res.n[r] + j];
      corr[e * n + i] = correct[r][(size_t)e * res.n[r] + j];
    }
  uint64_t npred = c->model == AMP_MODEL_TREE ? (uint64_t)S.lab.size() * epochs : n_total;
  if (train) {
    c->last_loss.swap(loss);
    c->last_correct.swap(corr);
    c->last_seconds = seconds;
    c->last_npred = npred;
    c->last_events.clear();
    for (auto& v : c->launch_events) c->last_events.insert(c->last_events.end(), v.begin(), v.end());
    c->last_replicas = R;
  } else if (ev) {
    double sl = 0;
    uint64_t sc = 0;
    for (size_t i = 0; i < n_total; ++i) {
      sl += loss[i];
      sc += corr[i];
    }
    ev->mean_loss = sl / (double)n_total;
    ev->accuracy = c->model == AMP_MODEL_GGNN ? 0.0 : (double)sc / (double)npred;
    ev->n_instances = n_total;
    ev->n_predictions = npred;
    ev->seconds = seconds;
  }
  c->launch_events.clear();
  return AMP_OK;
}

// Training and evaluation instances in one launch (Section 1: training and inference run through the same graph at
// the same time): the two sets are laid out as one, the admission list interleaves them -- after every `stride`
// training admissions one evaluation instance, stride = training admissions / evaluation instances -- and the
// evaluation instances are marked forward-only.
int run_mixed(amp_ctx* c, int epochs, amp_eval_result* ev) {
  InstSet &T = c->sets[0], &E = c->sets[1];
  if (T.n() == 0 || E.n() == 0) return fail(c, AMP_ESTATE, "train_eval: both instance sets must hold instances");
  if (c->replicas != 1) return fail(c, AMP_EUNSUPPORTED, "train_eval: not with replicas");
  if (c->model == AMP_MODEL_TREE && c->nodes[0].muf > AMP_TREE_LOOKUP_MAX_MUF)
    return fail(c, AMP_EUNSUPPORTED, "the tree lookup supports min_update_frequency up to %d", AMP_TREE_LOOKUP_MAX_MUF);
  for (const HostNode& n : c->nodes)
    if (n.name.compare(0, 6, "lookup") != 0 && n.muf > AMP_DENSE_MAX_MUF)
      return fail(c, AMP_EUNSUPPORTED, "dense nodes support min_update_frequency up to %d", AMP_DENSE_MAX_MUF);
  const size_t n_tr = T.n() * (size_t)epochs, n_ev = E.n();
  if (n_tr + n_ev >= 0x7fffffffull) return fail(c, AMP_EINVAL, "too many admissions for one call");
  if (int rc = prepare_device(c)) return rc;
  // one set: training instances first, evaluation instances behind them
  InstSet both;
  for (size_t i = 0; i < T.n(); ++i) append_instance(c, both, T, i);
  for (size_t i = 0; i < E.n(); ++i) append_instance(c, both, E, i);
  c->resident[0].valid = c->resident[1].valid = false;   // the combined set takes their place in the arena
  Resident res;
  if (int rc = make_resident(c, both, 1, c->static_end, res)) return rc;
  HIPCHK(c, hipStreamSynchronize(c->stream));   // `both` is pageable host memory
  std::vector<std::vector<int>> adm(1);
  std::vector<int>& a = adm[0];
  const size_t stride = std::max<size_t>(1, n_tr / n_ev);
  size_t it = 0, ie = 0;
  while (it < n_tr || ie < n_ev) {
    for (size_t k = 0; k < stride && it < n_tr; ++k, ++it) a.push_back((int)(it % T.n()));
    if (ie < n_ev) a.push_back((int)(T.n() + ie++) | (int)0x80000000);
  }
  std::vector<std::vector<float>> losses(1);
  std::vector<std::vector<int>> correct(1);
  double seconds = 0;
  c->launch_events.assign(c->workers.size(), std::vector<amp_event>());
  c->last_probe.clear();
  if (int rc = launch_once(c, res, res.end, 1, true, losses, correct, seconds, &adm)) return rc;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  // split the results by kind, each in its own admission order
  c->last_loss.clear();
  c->last_correct.clear();
  double sl = 0;
  uint64_t sc = 0;
  for (size_t i = 0; i < a.size(); ++i) {
    if (a[i] < 0) {
      sl += losses[0][i];
      sc += correct[0][i];
    } else {
      c->last_loss.push_back(losses[0][i]);
      c->last_correct.push_back(correct[0][i]);
    }
  }
  c->last_seconds = seconds;
  c->last_npred = c->model == AMP_MODEL_TREE ? (uint64_t)T.lab.size() * epochs : n_tr;
  c->last_events.clear();
  for (auto& v : c->launch_events) c->last_events.insert(c->last_events.end(), v.begin(), v.end());
  c->launch_events.clear();
  c->last_replicas = 1;
  const uint64_t npred = c->model == AMP_MODEL_TREE ? (uint64_t)E.lab.size() : n_ev;
  ev->mean_loss = sl / (double)n_ev;
  ev->accuracy = c->model == AMP_MODEL_GGNN ? 0.0 : (double)sc / (double)npred;
  ev->n_instances = n_ev;
  ev->n_predictions = npred;
  ev->seconds = seconds;
  return AMP_OK;
}

}  // namespace

extern "C" {

int amp_train_eval(amp_ctx* c, int epochs, amp_eval_result* out) {
  if (!c || !out) return fail(c, AMP_EINVAL, "null argument");
  if (!c->finalized) return fail(c, AMP_ESTATE, "train_eval: finalize first");
  if (epochs < 1) return fail(c, AMP_EINVAL, "train_eval: epochs must be >= 1");
  return run_mixed(c, epochs, out);
}

int amp_train(amp_ctx* c, int epochs) {
  if (!c) return AMP_EINVAL;
  if (!c->finalized) return fail(c, AMP_ESTATE, "train: finalize first");
  if (epochs < 1) return fail(c, AMP_EINVAL, "train: epochs must be >= 1");
  return run(c, 0, epochs, true, nullptr);
}

int amp_eval(amp_ctx* c, amp_eval_result* out) {
  if (!c || !out) return fail(c, AMP_EINVAL, "null argument");
  if (!c->finalized) return fail(c, AMP_ESTATE, "eval: finalize first");
  return run(c, 1, 1, false, out);
}

int amp_get_loss(amp_ctx* c, double* mean_loss, double* accuracy, uint64_t* n_instances, double* seconds) {
  if (!c) return AMP_EINVAL;
  if (c->last_loss.empty()) return fail(c, AMP_ESTATE, "get_loss: nothing trained yet");
  double sl = 0;
  uint64_t sc = 0;
  for (size_t i = 0; i < c->last_loss.size(); ++i) {
    sl += c->last_loss[i];
    sc += c->last_correct[i];
  }
  if (mean_loss) *mean_loss = sl / (double)c->last_loss.size();
  if (accuracy) *accuracy = c->model == AMP_MODEL_GGNN ? 0.0 : (double)sc / (double)c->last_npred;
  if (n_instances) *n_instances = c->last_loss.size();
  if (seconds) *seconds = c->last_seconds;
  return AMP_OK;
}

int amp_get_instance_losses(amp_ctx* c, float* host, size_t cap, size_t* n) {
  if (!c || !host) return fail(c, AMP_EINVAL, "null argument");
  if (n) *n = c->last_loss.size();
  if (cap < c->last_loss.size()) return fail(c, AMP_ENOMEM, "get_instance_losses: %zu floats needed", c->last_loss.size());
  std::memcpy(host, c->last_loss.data(), c->last_loss.size() * 4);
  return AMP_OK;
}

int amp_get_event_log(amp_ctx* c, amp_event* buf, size_t cap, size_t* n) {
  if (!c) return AMP_EINVAL;
  if (n) *n = c->last_events.size();
  if (!buf) return AMP_OK;   // size query
  if (cap < c->last_events.size()) return fail(c, AMP_ENOMEM, "get_event_log: %zu events needed", c->last_events.size());
  std::memcpy(buf, c->last_events.data(), c->last_events.size() * sizeof(amp_event));
  return AMP_OK;
}

int amp_get_staleness_hist(amp_ctx* c, uint64_t* bins, size_t nbins) {
  if (!c || !bins || nbins < 1) return fail(c, AMP_EINVAL, "bad argument");
  if (c->last_events.empty()) return fail(c, AMP_ESTATE, "get_staleness_hist: no event record (amp_set_event_log)");
  std::fill(bins, bins + nbins, 0);
  // per node: updates so far, and the value at each pending forward
  const size_t nn1 = c->nodes.size(), wpr = c->workers.size(), nn = nn1 * (size_t)c->last_replicas;
  std::vector<uint64_t> updates(nn, 0);
  std::vector<std::vector<std::pair<uint64_t, uint64_t>>> pending(nn);   // (key, updates at forward)
  for (const amp_event& e : c->last_events) {
    if (e.worker % wpr == 0 || e.node >= nn1) continue;
    const size_t node = e.node + nn1 * (e.worker / wpr);   // every replica has its own copy of the node
    const uint64_t key = ((uint64_t)e.seq << 20) | e.local;
    if (e.kind == AMP_EV_U) {
      updates[node]++;
    } else if (e.kind == AMP_EV_F) {
      pending[node].push_back({key, updates[node]});
    } else if (e.kind == AMP_EV_B) {
      auto& p = pending[node];
      for (size_t i = 0; i < p.size(); ++i)
        if (p[i].first == key) {
          const uint64_t st = updates[node] - p[i].second;
          bins[std::min<uint64_t>(st, nbins - 1)]++;
          p[i] = p.back();
          p.pop_back();
          break;
        }
    }
  }
  return AMP_OK;
}

}  // extern "C"
