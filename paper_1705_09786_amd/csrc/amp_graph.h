// Host-side description of a model as a static IR graph (Section 4: a model is an IR graph plus a controller),
// its validation, and its recognition as one of the four graphs the persistent kernel has workers for.
// Pure host code, no device types: nodes with numbered in / out ports, edges between ports.
#pragma once
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <map>
#include <string>
#include <vector>

#include "../../include/amp.h"

namespace ampgraph {

struct Node {
  int kind = 0;
  amp_node_desc d{};
};

struct Edge {
  int src, sport, dst, dport;
};

struct Graph {
  std::vector<Node> nodes;   // node 0 is the controller
  std::vector<Edge> edges;
  Graph() {
    Node c;
    c.kind = AMP_NODE_CONTROLLER;
    nodes.push_back(c);
  }
  int add(int kind, int rows = 0, int cols = 0, int n_in = 1, int n_out = 1, int aux = 0) {
    Node n;
    n.kind = kind;
    n.d.rows = rows;
    n.d.cols = cols;
    n.d.n_in = n_in;
    n.d.n_out = n_out;
    n.d.aux = aux;
    nodes.push_back(n);
    return (int)nodes.size() - 1;
  }
  void connect(int s, int sp, int d, int dp) { edges.push_back({s, sp, d, dp}); }
};

inline const char* kind_name(int k) {
  static const char* names[] = {"controller", "lookup", "linear", "rnn_tanh", "gru", "leaf_lstm", "branch_lstm",
                                "ggnn_edge_linear", "sum_readout", "softmax_xent", "squared_err", "cond", "phi", "isu",
                                "concat", "split", "bcast", "group", "ungroup", "flatmap", "sum", "sink"};
  return (k >= 0 && k <= AMP_NODE_SINK) ? names[k] : "?";
}

inline bool parameterized(int k) { return k >= AMP_NODE_LOOKUP && k <= AMP_NODE_SUM_READOUT; }

// Ports a node of this kind has; -1 = as many as the descriptor says.
inline int ports_in(const Node& n) {
  switch (n.kind) {
    case AMP_NODE_CONTROLLER: return 0;   // the backward messages that answer what it pumped return by themselves
    case AMP_NODE_GRU: return 2;          // aggregated messages, previous state
    case AMP_NODE_SOFTMAX_XENT:
    case AMP_NODE_SQUARED_ERR: return 2;  // prediction, label / target pumped by the controller
    case AMP_NODE_PHI:
    case AMP_NODE_CONCAT: return n.d.n_in;
    default: return 1;
  }
}
inline int ports_out(const Node& n) {
  switch (n.kind) {
    case AMP_NODE_CONTROLLER: return n.d.n_out;   // grows with every connection made from it
    case AMP_NODE_SOFTMAX_XENT:
    case AMP_NODE_SQUARED_ERR:
    case AMP_NODE_SINK: return 0;
    case AMP_NODE_COND:
    case AMP_NODE_SPLIT:
    case AMP_NODE_BCAST: return n.d.n_out;
    default: return 1;
  }
}

// Payload width at a port.  0 = an index / label / scalar the controller pumps (not a float vector), -1 = unknown
// until propagated (control nodes pass their input's width on).
struct Widths {
  std::vector<std::vector<int>> in, out;
};

inline std::string fmt(const char* f, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, f);
  vsnprintf(buf, sizeof buf, f, ap);
  va_end(ap);
  return buf;
}

// Fixed widths a node's own description implies (ins, outs); -1 where the node takes what it is given.
inline void own_widths(const Node& n, std::vector<int>& in, std::vector<int>& out) {
  in.assign(ports_in(n), -1);
  out.assign(ports_out(n), -1);
  const int r = n.d.rows, c = n.d.cols;
  switch (n.kind) {
    case AMP_NODE_CONTROLLER: break;
    case AMP_NODE_LOOKUP: in[0] = 0; out[0] = c; break;                 // rows = table rows, cols = embedding width
    case AMP_NODE_LINEAR:
    case AMP_NODE_RNN_TANH:
    case AMP_NODE_GGNN_EDGE_LINEAR: in[0] = c; out[0] = r; break;
    case AMP_NODE_GRU: in[0] = in[1] = r; out[0] = r; break;            // rows = hidden
    case AMP_NODE_LEAF_LSTM: in[0] = c; out[0] = 2 * r; break;          // rows = hidden, cols = embedding; out = [h; c]
    case AMP_NODE_BRANCH_LSTM: in[0] = 4 * r; out[0] = 2 * r; break;    // in = [h_l; c_l; h_r; c_r]
    case AMP_NODE_SUM_READOUT: in[0] = c; out[0] = 1; break;
    case AMP_NODE_SOFTMAX_XENT: in[0] = r; in[1] = 0; break;            // rows = classes
    case AMP_NODE_SQUARED_ERR: in[0] = 1; in[1] = 0; break;
    default: break;
  }
}

// Checks ports and widths and the loop rule.  Returns AMP_OK or AMP_EINVAL with a message.
inline int validate(const Graph& g, std::string& err) {
  const int N = (int)g.nodes.size();
  std::vector<std::vector<int>> in_from(N), out_to(N);   // edge index per port, -1 = open
  for (int i = 0; i < N; ++i) {
    const Node& n = g.nodes[i];
    if (n.kind < AMP_NODE_CONTROLLER || n.kind > AMP_NODE_SINK) {
      err = fmt("node %d has unknown kind %d", i, n.kind);
      return AMP_EINVAL;
    }
    if (ports_in(n) < 0 || ports_out(n) < 0 || ports_in(n) > 64 || ports_out(n) > 64) {
      err = fmt("node %d (%s): bad port count", i, kind_name(n.kind));
      return AMP_EINVAL;
    }
    in_from[i].assign(ports_in(n), -1);
    out_to[i].assign(ports_out(n), -1);
  }
  for (int e = 0; e < (int)g.edges.size(); ++e) {
    const Edge& ed = g.edges[e];
    if (ed.src < 0 || ed.src >= N || ed.dst < 0 || ed.dst >= N) {
      err = fmt("edge %d names a node that does not exist", e);
      return AMP_EINVAL;
    }
    if (ed.sport < 0 || ed.sport >= (int)out_to[ed.src].size()) {
      err = fmt("node %d (%s) has no output port %d", ed.src, kind_name(g.nodes[ed.src].kind), ed.sport);
      return AMP_EINVAL;
    }
    if (ed.dport < 0 || ed.dport >= (int)in_from[ed.dst].size()) {
      err = fmt("node %d (%s) has no input port %d", ed.dst, kind_name(g.nodes[ed.dst].kind), ed.dport);
      return AMP_EINVAL;
    }
    if (out_to[ed.src][ed.sport] >= 0 || in_from[ed.dst][ed.dport] >= 0) {
      err = fmt("port connected twice: node %d port %d -> node %d port %d", ed.src, ed.sport, ed.dst, ed.dport);
      return AMP_EINVAL;
    }
    out_to[ed.src][ed.sport] = e;
    in_from[ed.dst][ed.dport] = e;
  }
  // dangling ports: every port of every node carries exactly one edge (the controller's input port stands for the
  // backward messages that return to it and takes no edge)
  for (int i = 0; i < N; ++i) {
    for (int p = 0; p < (int)out_to[i].size(); ++p)
      if (out_to[i][p] < 0) {
        err = fmt("dangling port: output %d of node %d (%s) is not connected", p, i, kind_name(g.nodes[i].kind));
        return AMP_EINVAL;
      }
    if (i == 0) continue;
    for (int p = 0; p < (int)in_from[i].size(); ++p)
      if (in_from[i][p] < 0) {
        err = fmt("dangling port: input %d of node %d (%s) is not connected", p, i, kind_name(g.nodes[i].kind));
        return AMP_EINVAL;
      }
  }
  if (g.nodes[0].d.n_out < 1) {
    err = "the controller pumps nothing into the graph";
    return AMP_EINVAL;
  }
  // loops must pass through a Phi (the node that joins the loop's entry with its back edge and records the origin):
  // without the Phi nodes the graph has to be acyclic
  {
    std::vector<int> state(N, 0);   // 0 new, 1 on the stack, 2 done
    std::vector<std::pair<int, int>> stack;
    for (int r = 0; r < N; ++r) {
      if (state[r] || g.nodes[r].kind == AMP_NODE_PHI) continue;
      stack.push_back({r, 0});
      state[r] = 1;
      while (!stack.empty()) {
        auto& top = stack.back();
        const int u = top.first;
        if (top.second == (int)out_to[u].size()) {
          state[u] = 2;
          stack.pop_back();
          continue;
        }
        const int v = g.edges[out_to[u][top.second++]].dst;
        if (g.nodes[v].kind == AMP_NODE_PHI) continue;
        if (state[v] == 1) {
          err = fmt("cycle without a Phi: node %d (%s) is reached again from node %d (%s)", v, kind_name(g.nodes[v].kind), u,
                    kind_name(g.nodes[u].kind));
          return AMP_EINVAL;
        }
        if (state[v] == 0) {
          state[v] = 1;
          stack.push_back({v, 0});
        }
      }
    }
  }
  // widths: start from what the nodes' own descriptions fix, pass widths through the control nodes until nothing
  // changes, and compare the two ends of every edge
  Widths w;
  w.in.resize(N);
  w.out.resize(N);
  for (int i = 0; i < N; ++i) own_widths(g.nodes[i], w.in[i], w.out[i]);
  for (bool changed = true; changed;) {
    changed = false;
    auto set = [&](int& slot, int v) {
      if (v >= 0 && slot < 0) {
        slot = v;
        changed = true;
      }
    };
    for (const Edge& ed : g.edges) {
      set(w.in[ed.dst][ed.dport], w.out[ed.src][ed.sport]);
      if (ed.src != 0) set(w.out[ed.src][ed.sport], w.in[ed.dst][ed.dport]);
      if (ed.src == 0) set(w.out[0][ed.sport], w.in[ed.dst][ed.dport]);
    }
    for (int i = 1; i < N; ++i) {
      const Node& n = g.nodes[i];
      std::vector<int>&in = w.in[i], &out = w.out[i];
      switch (n.kind) {
        case AMP_NODE_COND:
        case AMP_NODE_BCAST:
          for (int& o : out) set(o, in[0]);
          for (int o : out) set(in[0], o);
          break;
        case AMP_NODE_PHI:
          for (int x : in) set(out[0], x);
          for (int& x : in) set(x, out[0]);
          break;
        case AMP_NODE_ISU:
        case AMP_NODE_GROUP:
        case AMP_NODE_UNGROUP:
        case AMP_NODE_FLATMAP:
        case AMP_NODE_SUM:
          set(out[0], in[0]);
          set(in[0], out[0]);
          break;
        case AMP_NODE_CONCAT: {
          // aux = parts that arrive on each port, told apart by their state (0 or 1: one part per port)
          const int parts = n.d.aux > 1 ? n.d.aux : 1;
          int sum = 0;
          bool all = true;
          for (int x : in) {
            all = all && x >= 0;
            sum += x;
          }
          if (all) set(out[0], sum * parts);
          break;
        }
        case AMP_NODE_SPLIT: {
          // equal parts
          if (in[0] >= 0 && n.d.n_out > 0 && in[0] % n.d.n_out == 0)
            for (int& o : out) set(o, in[0] / n.d.n_out);
          break;
        }
        default: break;
      }
    }
  }
  for (const Edge& ed : g.edges) {
    const int a = w.out[ed.src][ed.sport], b = w.in[ed.dst][ed.dport];
    if (a >= 0 && b >= 0 && a != b) {
      err = fmt("dimension mismatch: node %d (%s) port %d sends %d values, node %d (%s) port %d takes %d", ed.src,
                kind_name(g.nodes[ed.src].kind), ed.sport, a, ed.dst, kind_name(g.nodes[ed.dst].kind), ed.dport, b);
      return AMP_EINVAL;
    }
  }
  for (int i = 1; i < N; ++i) {
    const Node& n = g.nodes[i];
    if (n.kind == AMP_NODE_SPLIT && w.in[i][0] >= 0 && n.d.n_out > 0 && w.in[i][0] % n.d.n_out) {
      err = fmt("dimension mismatch: split node %d cannot cut %d values into %d equal parts", i, w.in[i][0], n.d.n_out);
      return AMP_EINVAL;
    }
    if (parameterized(n.kind) && (n.d.rows < 1 || (n.kind != AMP_NODE_GRU && n.kind != AMP_NODE_BRANCH_LSTM && n.d.cols < 1))) {
      err = fmt("node %d (%s): rows and cols must be >= 1", i, kind_name(n.kind));
      return AMP_EINVAL;
    }
  }
  return AMP_OK;
}

// ---------------------------------------------------------------- the four graphs the kernel has workers for
// Built with the same calls a user would make; the order of the parameterized nodes is the per-model numbering
// of include/amp.h.
inline Graph template_graph(int model, const amp_model_dims& d) {
  Graph g;
  auto pump = [&](int dst, int dport) {
    g.connect(0, g.nodes[0].d.n_out, dst, dport);
    g.nodes[0].d.n_out++;
  };
  const int H = d.hidden;
  if (model == AMP_MODEL_MLP) {
    // controller -> Linear+ReLU -> Linear+ReLU -> Linear -> loss; the label goes to the loss layer
    const int l1 = g.add(AMP_NODE_LINEAR, H, d.d_in, 1, 1, AMP_ACT_RELU), l2 = g.add(AMP_NODE_LINEAR, H, H, 1, 1, AMP_ACT_RELU),
              l3 = g.add(AMP_NODE_LINEAR, d.n_class, H), loss = g.add(AMP_NODE_SOFTMAX_XENT, d.n_class);
    pump(l1, 0);
    g.connect(l1, 0, l2, 0);
    g.connect(l2, 0, l3, 0);
    g.connect(l3, 0, loss, 0);
    pump(loss, 1);
  } else if (model == AMP_MODEL_RNN) {
    // Figure 2: lookup -> Concat(embedding, h) -> cell -> Isu(t + 1) -> Cond(end?) -> Phi (loop) | Linear -> loss
    const int lk = g.add(AMP_NODE_LOOKUP, d.vocab, d.emb), cell = g.add(AMP_NODE_RNN_TANH, H, d.emb + H),
              out = g.add(AMP_NODE_LINEAR, d.n_class, H), phi = g.add(AMP_NODE_PHI, 0, 0, 2), cat = g.add(AMP_NODE_CONCAT, 0, 0, 2),
              isu = g.add(AMP_NODE_ISU), cond = g.add(AMP_NODE_COND, 0, 0, 1, 2), loss = g.add(AMP_NODE_SOFTMAX_XENT, d.n_class);
    pump(lk, 0);
    pump(phi, 0);
    pump(loss, 1);
    g.connect(lk, 0, cat, 0);
    g.connect(phi, 0, cat, 1);
    g.connect(cat, 0, cell, 0);
    g.connect(cell, 0, isu, 0);
    g.connect(isu, 0, cond, 0);
    g.connect(cond, 0, phi, 1);
    g.connect(cond, 1, out, 0);
    g.connect(out, 0, loss, 0);
  } else if (model == AMP_MODEL_TREE) {
    // lookup -> leaf cell -> Phi <- branch cell; Phi -> Bcast -> (Split -> Linear -> loss, Cond(root?) -> Isu(to
    // parent) -> Concat of the two children, keyed on the parent -> branch cell)
    const int lk = g.add(AMP_NODE_LOOKUP, d.vocab, d.emb), leaf = g.add(AMP_NODE_LEAF_LSTM, H, d.emb),
              br = g.add(AMP_NODE_BRANCH_LSTM, H), out = g.add(AMP_NODE_LINEAR, d.n_class, H), phi = g.add(AMP_NODE_PHI, 0, 0, 2),
              bc = g.add(AMP_NODE_BCAST, 0, 0, 1, 2), sp = g.add(AMP_NODE_SPLIT, 0, 0, 1, 2), csink = g.add(AMP_NODE_SINK),
              loss = g.add(AMP_NODE_SOFTMAX_XENT, d.n_class), cond = g.add(AMP_NODE_COND, 0, 0, 1, 2),
              rsink = g.add(AMP_NODE_SINK), isu = g.add(AMP_NODE_ISU), cat = g.add(AMP_NODE_CONCAT, 0, 0, 1, 1, 2);
    pump(lk, 0);
    pump(loss, 1);
    g.connect(lk, 0, leaf, 0);
    g.connect(leaf, 0, phi, 0);
    g.connect(br, 0, phi, 1);
    g.connect(phi, 0, bc, 0);
    g.connect(bc, 0, sp, 0);
    g.connect(sp, 0, out, 0);
    g.connect(sp, 1, csink, 0);
    g.connect(out, 0, loss, 0);
    g.connect(bc, 1, cond, 0);
    g.connect(cond, 0, rsink, 0);
    g.connect(cond, 1, isu, 0);
    g.connect(isu, 0, cat, 0);
    g.connect(cat, 0, br, 0);
  } else if (model == AMP_MODEL_GGNN) {
    // Figure 4(a): lookup -> Phi -> Bcast -> Ungroup -> Flatmap (outgoing edges) -> Cond (edge type) -> per type
    // Group -> Linear -> Ungroup -> Phi -> Group (target node) -> Sum -> Group (all nodes) -> GRU(a, h) -> Isu ->
    // Cond (steps done?) -> Phi (loop) | sum readout -> loss
    const int ne = d.n_edge_types;
    const int lk = g.add(AMP_NODE_LOOKUP, d.n_node_types, H);
    std::vector<int> lin(ne);
    for (int c = 0; c < ne; ++c) lin[c] = g.add(AMP_NODE_GGNN_EDGE_LINEAR, H, H);
    const int gru = g.add(AMP_NODE_GRU, H), ro = g.add(AMP_NODE_SUM_READOUT, 1, H);
    const int phi_h = g.add(AMP_NODE_PHI, 0, 0, 2), bc = g.add(AMP_NODE_BCAST, 0, 0, 1, 2), ung = g.add(AMP_NODE_UNGROUP),
              fm = g.add(AMP_NODE_FLATMAP), bytype = g.add(AMP_NODE_COND, 0, 0, 1, ne), phi_e = g.add(AMP_NODE_PHI, 0, 0, ne),
              bydst = g.add(AMP_NODE_GROUP), sum = g.add(AMP_NODE_SUM), all = g.add(AMP_NODE_GROUP), isu = g.add(AMP_NODE_ISU),
              done = g.add(AMP_NODE_COND, 0, 0, 1, 2, d.n_steps), loss = g.add(AMP_NODE_SQUARED_ERR);
    pump(lk, 0);
    pump(loss, 1);
    g.connect(lk, 0, phi_h, 0);
    g.connect(phi_h, 0, bc, 0);
    g.connect(bc, 0, ung, 0);
    g.connect(ung, 0, fm, 0);
    g.connect(fm, 0, bytype, 0);
    for (int c = 0; c < ne; ++c) {
      const int grp = g.add(AMP_NODE_GROUP), ungc = g.add(AMP_NODE_UNGROUP);
      g.connect(bytype, c, grp, 0);
      g.connect(grp, 0, lin[c], 0);
      g.connect(lin[c], 0, ungc, 0);
      g.connect(ungc, 0, phi_e, c);
    }
    g.connect(phi_e, 0, bydst, 0);
    g.connect(bydst, 0, sum, 0);
    g.connect(sum, 0, all, 0);
    g.connect(all, 0, gru, 0);
    g.connect(bc, 1, gru, 1);
    g.connect(gru, 0, isu, 0);
    g.connect(isu, 0, done, 0);
    g.connect(done, 0, phi_h, 1);
    g.connect(done, 1, ro, 0);
    g.connect(ro, 0, loss, 0);
  }
  return g;
}

// Canonical numbering of a port-labelled graph: nodes in the order a depth-first walk from the controller first
// reaches them, output ports ascending.  Two graphs are the same graph iff their canonical forms are equal.
struct Canon {
  std::vector<int> order;                       // canonical position -> node id
  std::vector<std::vector<int>> form;           // per canonical node: kind, rows, cols, n_in, n_out, aux, then (dst, dport) per out port
};

inline Canon canonical(const Graph& g) {
  const int N = (int)g.nodes.size();
  std::vector<std::vector<std::pair<int, int>>> out(N);
  for (int i = 0; i < N; ++i) out[i].assign(std::max(0, ports_out(g.nodes[i])), {-1, -1});
  for (const Edge& e : g.edges)
    if (e.src >= 0 && e.src < N && e.sport >= 0 && e.sport < (int)out[e.src].size()) out[e.src][e.sport] = {e.dst, e.dport};
  std::vector<int> pos(N, -1);
  Canon c;
  std::vector<int> stack{0};
  pos[0] = 0;
  c.order.push_back(0);
  // iterative preorder, ports ascending
  std::vector<std::pair<int, int>> st{{0, 0}};
  while (!st.empty()) {
    auto& top = st.back();
    const int u = top.first;
    if (top.second == (int)out[u].size()) {
      st.pop_back();
      continue;
    }
    const int v = out[u][top.second++].first;
    if (v >= 0 && pos[v] < 0) {
      pos[v] = (int)c.order.size();
      c.order.push_back(v);
      st.push_back({v, 0});
    }
  }
  for (int u : c.order) {
    const Node& n = g.nodes[u];
    std::vector<int> f{n.kind, n.d.rows, n.d.cols, ports_in(n), ports_out(n), n.d.aux};
    for (auto& pr : out[u]) {
      f.push_back(pr.first >= 0 ? pos[pr.first] : -1);
      f.push_back(pr.second);
    }
    c.form.push_back(f);
  }
  return c;
}

// Recognises g as one of the four model graphs.  On success fills model, dims and, per node of g, the model's
// parameterized-node number it became (-1 for control and loss nodes; a GRU node stands for three consecutive
// numbers and gets the first).  AMP_EUNSUPPORTED when the graph is valid but none of the four.
inline int recognise(const Graph& g, int& model, amp_model_dims& dims, std::vector<int>& param_of, std::string& err) {
  dims = amp_model_dims{};
  int n_leaf = 0, n_gru = 0, n_rnn = 0, n_edge = 0;
  for (const Node& n : g.nodes) {
    n_leaf += n.kind == AMP_NODE_LEAF_LSTM;
    n_gru += n.kind == AMP_NODE_GRU;
    n_rnn += n.kind == AMP_NODE_RNN_TANH;
    n_edge += n.kind == AMP_NODE_GGNN_EDGE_LINEAR;
  }
  model = n_leaf ? AMP_MODEL_TREE : n_gru ? AMP_MODEL_GGNN : n_rnn ? AMP_MODEL_RNN : AMP_MODEL_MLP;
  // sizes from the first nodes of the kinds that carry them
  std::vector<const Node*> lin;
  for (const Node& n : g.nodes) {
    switch (n.kind) {
      case AMP_NODE_LOOKUP:
        if (model == AMP_MODEL_GGNN) dims.n_node_types = n.d.rows, dims.hidden = n.d.cols;
        else dims.vocab = n.d.rows, dims.emb = n.d.cols;
        break;
      case AMP_NODE_RNN_TANH:
      case AMP_NODE_LEAF_LSTM:
      case AMP_NODE_GRU: dims.hidden = n.d.rows; break;
      case AMP_NODE_SOFTMAX_XENT: dims.n_class = n.d.rows; break;
      case AMP_NODE_LINEAR: lin.push_back(&n); break;
      default: break;
    }
  }
  if (model == AMP_MODEL_MLP && !lin.empty()) {
    dims.d_in = lin[0]->d.cols;
    dims.hidden = lin[0]->d.rows;
  }
  dims.n_edge_types = n_edge;
  if (model == AMP_MODEL_GGNN) {
    // the loop's Cond (the one an Isu feeds) carries the number of propagation steps
    for (const Edge& e : g.edges)
      if (e.src > 0 && e.src < (int)g.nodes.size() && e.dst > 0 && e.dst < (int)g.nodes.size() &&
          g.nodes[e.src].kind == AMP_NODE_ISU && g.nodes[e.dst].kind == AMP_NODE_COND)
        dims.n_steps = g.nodes[e.dst].d.aux;
  }
  const Graph t = template_graph(model, dims);
  const Canon a = canonical(g), b = canonical(t);
  if (a.order.size() != g.nodes.size()) {
    err = "the graph has nodes the controller's messages never reach";
    return AMP_EUNSUPPORTED;
  }
  if (a.form != b.form) {
    err = fmt("a valid graph, but not one the kernel has workers for (closest: the %s graph; it differs at canonical node %d)",
              model == AMP_MODEL_TREE ? "Tree-LSTM" : model == AMP_MODEL_GGNN ? "gated graph network" : model == AMP_MODEL_RNN ? "RNN" : "MLP",
              (int)(std::mismatch(a.form.begin(), a.form.begin() + std::min(a.form.size(), b.form.size()), b.form.begin()).first -
                    a.form.begin()));
    return AMP_EUNSUPPORTED;
  }
  // the template adds its parameterized nodes in the model's numbering
  std::vector<int> tnum(t.nodes.size(), -1);
  int next = 0;
  for (size_t i = 0; i < t.nodes.size(); ++i)
    if (parameterized(t.nodes[i].kind)) {
      tnum[i] = next;
      next += t.nodes[i].kind == AMP_NODE_GRU ? 3 : 1;
    }
  param_of.assign(g.nodes.size(), -1);
  for (size_t k = 0; k < a.order.size(); ++k) param_of[a.order[k]] = tnum[b.order[k]];
  return AMP_OK;
}

}  // namespace ampgraph
