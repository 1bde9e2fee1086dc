// Gated graph network workers (Figure 4a, Appendix C): lookup, one linear
// node per edge type, the GRU's three linear nodes (update gate, reset gate,
// candidate) and the regression layer.
//
// One message carries a whole group of rows: all edges of one type for an
// edge linear (Group by edge type), all graph nodes for the GRU nodes (the
// final Group over nodes), so each node sees one forward and one backward
// message per instance and propagation step and performs a small
// (rows x cols) x (k rows) product on the matrix cores.  Broadcast / Ungroup /
// Flatmap / Group / sum between them are index arithmetic over adjacency
// tables the host prepared per instance (incoming edges by destination, a
// type's edges in ascending order, a type's edges by source), plus arrival
// counters.  Sums over a variable number of parts (messages into a node,
// gradients back to a source node, Bcast backward) are formed by the worker
// that consumes them, always in the same order: ascending edge index; edge
// types ascending, then update gate, reset gate, candidate.
//
// Slot storage (s = slot, it = step, v = graph node, e = directed edge):
//   buf[0]  Hm  [s][S+1][N][H]  node states before each step (Hm[.][0] = lookup output)
//   buf[1]  A   [s][S][N][H]    aggregated messages (GRU input), recorded by the update gate
//   buf[2]  Z   [s][S][N][H]    update gate
//   buf[3]  Rr  [s][S][N][H]    reset gate
//   buf[4]  Ht  [s][S][N][H]    candidate state
//   buf[5]  Msg [s][E][H]       per-edge messages of the running step
//   buf[6]  gH  [s][N][H]       gradient w.r.t. the final states (from the readout)
//   buf[7]  dZ  [s][N][H]       pre-activation gradient for the update-gate node
//   buf[8]  dR  [s][Th][N][H]   pre-activation gradient for the reset-gate node, one part per candidate tile
//   buf[9]  dA  [s][PA][N][H]   gradient w.r.t. A: parts of the candidate tiles, then the update, then the reset gate's
//   buf[10] dHp [s][2][PA][N][H] gradient w.r.t. h from the same, by step parity: the candidate tiles of step it read
//                               what step it + 1 left (for their own units) while other tiles of step it already
//                               write their parts (over all units), so the two steps must not share a buffer
//   buf[11] dHe [s][PE][N][H]   gradient w.r.t. h through the edges, one part per edge-type tile
//   buf[13] cnt [s][8] (int)    arrival counters: 0 edge tiles forward, 1 gate tiles forward, 2 gate tiles backward,
//                               3 edge tiles backward, 4 candidate tiles forward, 5 candidate tiles backward
//   buf[14] sdesc [s][16]       slot descriptor, written by the lookup when the instance enters: 0 admission number,
//                               1 instance, 2 token offset, 3 graph nodes, 4 edge offset, 5 edges, 6 target (bits),
//                               7 edge types present, 8..15 edges per type -- one 64-byte line, so that a worker
//                               learns all it needs about a message's instance in one fetch
//
// An edge linear or GRU node may be split by hidden unit over several workgroups (Section 5: a linear layer can be
// split into tiles computed in parallel): the tiles read the node's ring in the same order, tile t owns output
// units [u0, u0 + nu) -- those rows of W -- writes its slice of the node's output on the way forward and hands back
// a partial W^T delta over all input columns on the way back; consumers add the parts up in a fixed order (edge
// types ascending and tiles ascending inside a type; update gate, reset gate, candidate).
#pragma once

struct GView {
  int inst, N, E;
  const GQ int *type, *src, *dst, *tcount, *inoff, *inedge, *tstart, *tedge, *tsoff, *tsk;
  float target;
  // filled by g_view_msg only: the admission number, the edge types present, and (edge workers) the number of edges
  // of the worker's type and where they start in tedge / tsk
  unsigned seq, present;
  int kc, tsc;
};

// The instance set's arrays, read once per worker into scalar registers.
struct GData {
  const GQ int *tok_off, *edge_off, *tok, *src, *dst, *tcount, *inoff, *inedge, *tstart, *tedge, *tsoff, *tsk, *tsrc, *tdst;
  const GQ float* target;
  const GQ unsigned* slot_seq;
  const GQ int* slot_inst;
  int n_inst, T;
};

__device__ __forceinline__ GData g_data(const GQ AmpDev* D) {
  GData d;
  d.tok_off = uni_gq<int>(D->data.tok_off);
  d.edge_off = uni_gq<int>(D->data.edge_off);
  d.tok = uni_gq<int>(D->data.tok);
  d.src = uni_gq<int>(D->data.src);
  d.dst = uni_gq<int>(D->data.dst);
  d.tcount = uni_gq<int>(D->data.tcount);
  d.inoff = uni_gq<int>(D->data.inoff);
  d.inedge = uni_gq<int>(D->data.inedge);
  d.tstart = uni_gq<int>(D->data.tstart);
  d.tedge = uni_gq<int>(D->data.tedge);
  d.tsoff = uni_gq<int>(D->data.tsoff);
  d.tsk = uni_gq<int>(D->data.tsk);
  d.tsrc = uni_gq<int>(D->data.tsrc);
  d.tdst = uni_gq<int>(D->data.tdst);
  d.target = uni_gq<float>(D->data.target);
  d.slot_seq = uni_gq<unsigned>(D->slot_seq);
  d.slot_inst = uni_gq<int>(D->slot_inst);
  d.n_inst = uni(D->data.n_inst);
  d.T = uni(D->n_edge_types);
  return d;
}

__device__ __forceinline__ GView g_view(const GData& d, int s) {
  GView v;
  v.inst = uni(d.slot_inst[s]) & 0x7fffffff;
  const int to = uni(d.tok_off[v.inst]), eo = uni(d.edge_off[v.inst]);
  v.N = uni(d.tok_off[v.inst + 1]) - to;
  v.E = uni(d.edge_off[v.inst + 1]) - eo;
  v.type = d.tok + to;
  v.src = d.src + eo;
  v.dst = d.dst + eo;
  v.tcount = d.tcount + v.inst * 8;
  v.inoff = d.inoff + to + v.inst;
  v.inedge = d.inedge + eo;
  v.tstart = d.tstart + v.inst * 9;
  v.tedge = d.tedge + eo;
  v.tsoff = d.tsoff + (long long)d.T * (to + v.inst);
  v.tsk = d.tsk + eo;
  v.target = uni(d.target[v.inst]);
  return v;
}

struct GBufs {
  GQ float *Hm, *A, *Z, *Rr, *Ht, *Msg, *gH, *dZ, *dR, *dA, *dHp, *dHe;
  GQ int* cnt;
  GQ unsigned* sdesc;
  int H, N, Em, S, T;
  int Tz, Tr, Th, PA, PE;     // tiles of the update gate, reset gate and candidate; parts of dA / dHp; parts of dHe
  unsigned te_packed, eoff_packed;   // 4 bits per edge type: tiles of the type / first part of the type in dHe
  __device__ __forceinline__ int te(int c) const { return (te_packed >> (4 * c)) & 15; }
  __device__ __forceinline__ int eoff(int c) const { return (eoff_packed >> (4 * c)) & 15; }
  __device__ __forceinline__ long long st(int s, int it) const { return ((long long)s * S + it) * N * H; }
  __device__ __forceinline__ long long hm(int s, int it) const { return ((long long)s * (S + 1) + it) * N * H; }
  __device__ __forceinline__ long long sl(int s) const { return (long long)s * N * H; }
};

__device__ __forceinline__ GBufs g_bufs(const GQ AmpDev* D) {
  GBufs b;
  b.Hm = uni_gq<float>(D->buf[0]);
  b.A = uni_gq<float>(D->buf[1]);
  b.Z = uni_gq<float>(D->buf[2]);
  b.Rr = uni_gq<float>(D->buf[3]);
  b.Ht = uni_gq<float>(D->buf[4]);
  b.Msg = uni_gq<float>(D->buf[5]);
  b.gH = uni_gq<float>(D->buf[6]);
  b.dZ = uni_gq<float>(D->buf[7]);
  b.dR = uni_gq<float>(D->buf[8]);
  b.dA = uni_gq<float>(D->buf[9]);
  b.dHp = uni_gq<float>(D->buf[10]);
  b.dHe = uni_gq<float>(D->buf[11]);
  b.cnt = uni_gq<int>(D->buf[13]);
  b.sdesc = uni_gq<unsigned>(D->buf[14]);
  b.H = uni(D->hidden);
  b.N = uni(D->max_len);
  b.Em = uni(D->max_edges);
  b.S = uni(D->n_steps);
  b.T = uni(D->n_edge_types);
  b.Tz = uni(D->g_tiles[8]);
  b.Tr = uni(D->g_tiles[9]);
  b.Th = uni(D->g_tiles[10]);
  b.PA = uni(D->g_PA);
  b.PE = uni(D->g_PE);
  unsigned tp = 0, ep = 0;
  for (int c = 0; c < 8; ++c) {
    tp |= (unsigned)D->g_tiles[c] << (4 * c);
    ep |= (unsigned)D->g_eoff[c] << (4 * c);
  }
  b.te_packed = uni(tp);
  b.eoff_packed = uni(ep);
  return b;
}

// Tiles of the edge types that occur in a graph: what the joins over "every edge linear" wait for.
__device__ __forceinline__ int g_present_tiles(const GBufs& B, unsigned present) {
  int n = 0;
#pragma unroll
  for (int c = 0; c < 8; ++c) n += ((present >> c) & 1u) ? B.te(c) : 0;
  return n;
}

// The parts of dHe (by offset in units of N * H) that a graph's state gradient adds up, in order: edge types
// present ascending, tiles ascending.  Uniform across the workgroup.
struct GParts {
  int n;
  int off[12];
};
__device__ __forceinline__ GParts g_edge_parts(const GBufs& B, unsigned present) {
  GParts p;
  p.n = 0;
#pragma unroll
  for (int i = 0; i < 12; ++i) p.off[i] = 0;
#pragma unroll
  for (int c = 0; c < 8; ++c)
    if ((present >> c) & 1u)
      for (int t = 0; t < B.te(c); ++t) {
        const int at = p.n < 12 ? p.n : 11;
#pragma unroll
        for (int i = 0; i < 12; ++i)
          if (i == at) p.off[i] = B.eoff(c) + t;
        p.n++;
      }
  return p;
}

#define GR_LOOKUP 1
#define GR_EDGE0 2
#define GR_GZ(D) (2 + (D)->n_edge_types)
#define GR_GR(D) (3 + (D)->n_edge_types)
#define GR_GH(D) (4 + (D)->n_edge_types)
#define GR_RO(D) (5 + (D)->n_edge_types)

// The rings a graph worker posts to, read once.  `edge` is per lane: lane c (mod 8) holds the ring of edge type c.
struct GRings {
  Ring ctl, lookup, gz, gr, gh, ro, edge;
};

__device__ __forceinline__ GRings g_rings(const GQ AmpDev* D) {
  GRings r;
  const int T = uni(D->n_edge_types);
  r.ctl = ring_regs(D, 0);
  r.lookup = ring_regs(D, GR_LOOKUP);
  r.gz = ring_regs(D, 2 + T);
  r.gr = ring_regs(D, 3 + T);
  r.gh = ring_regs(D, 4 + T);
  r.ro = ring_regs(D, 5 + T);
  const int c = (threadIdx.x & 7) < T ? (threadIdx.x & 7) : 0;
  r.edge.ent = (GQ unsigned long long*)D->ring[GR_EDGE0 + c].ent;
  r.edge.tail = (GQ unsigned*)D->ring[GR_EDGE0 + c].tail;
  r.edge.mask = D->ring[GR_EDGE0 + c].mask;
  return r;
}

// ---------------------------------------------------------------- passes
// A dense graph worker takes up to G_MB messages of one direction from its ring at a time -- a pass -- and
// treats their row groups as one stack of rows: one staging, one product, one publication (a barrier, a fence)
// for all of them, where a message alone costs almost the same chain of memory round trips.  The messages of a
// pass belong to different instances; each keeps its own joins, posts and event records, and a backward pass never
// holds more messages than the node may still count before its update, so every message of a pass sees the
// weights it would have seen alone.
//
// The pass is formed by wave 1: lane l looks at ring entry head + l, the lanes whose entry is there decode their
// instance facts together (the slot descriptor the lookup left: one fetch for all the lanes), and the leading run of entries with lane 0's direction whose rows fit is taken.  The result is handed
// to the workgroup through LDS, in one of two buffers: the next pass is formed while the present one is in use.
#define G_MB 4
#define G_HW 8    // header words: 0 messages, 1 stop flag, 2 stacked rows, 3 stacked graph nodes, 4 direction bit
#define G_RW 16   // words per message: 0 code, 1 admission number, 2 slot, 3 step, 4 rows, 5 first stacked row,
                  // 6 graph nodes, 7 first stacked node, 8 edge types present, 9 instance, 10 token offset,
                  // 11 edge offset, 12 start of the worker's edge type in tedge / tsk, 13..14 the parts of dHe the
                  // instance's state gradient adds up (4 bits each, in order), 15 their number
__shared__ unsigned s_gpass[2][G_HW + G_MB * G_RW];

// The parts of dHe a graph uses, packed 4 bits each (at most 12 parts): edge types present ascending, tiles ascending.
__device__ __forceinline__ void g_pack_parts(const GBufs& B, unsigned present, unsigned& lo, unsigned& hi, unsigned& n) {
  unsigned long long pk = 0;
  n = 0;
  for (int c = 0; c < 8; ++c)
    if ((present >> c) & 1u)
      for (int t = 0; t < B.te(c); ++t) {
        if (n < 12) pk |= (unsigned long long)(B.eoff(c) + t) << (4 * n);
        n++;
      }
  lo = (unsigned)pk;
  hi = (unsigned)(pk >> 32);
}

// Wave 1, all 64 lanes.  cap = stacked rows the worker's LDS holds, maxm = most messages per pass, room = most
// backward messages (what the node may still count before its update), edge = rows are the edges of type ctype
// (otherwise the graph's nodes).  block = wait for the first message (otherwise an empty pass is left when it is
// not there yet, so that a worker can look ahead without waiting for a message its own publication must cause).
template <class R>
__device__ __forceinline__ void g_form_pass(const GQ AmpDev* D, const GData& d, const GBufs& B, const R& r, unsigned head, int cap,
                                            int maxm, int room, int ctype, bool edge, bool block, int buf) {
  const int l = threadIdx.x & 63;
  const bool act = l < maxm;
  const unsigned tk = head + (act ? (unsigned)l : 0u);
  GQ unsigned long long* slot = (GQ unsigned long long*)&r.ent[tk & r.mask];
  const long long t0 = wall_clock64();
  unsigned stop = 0, spins = 0;
  unsigned long long e;
  bool rdy;
  for (;;) {
    e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
    rdy = (unsigned)(e >> 32) == tk + 1u;
    if (uni((int)rdy) || !block) break;
    if ((++spins & 7u) == 0u) {
      if (uni(ld_u32(&D->ctl[0]) | ld_u32(&D->ctl[1]))) {
        // done is only raised once nothing is in flight; re-check the entries once
        e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
        rdy = (unsigned)(e >> 32) == tk + 1u;
        if (uni((int)rdy) && uni(ld_u32(&D->ctl[0])) == 0u) break;
        stop = 1;
        break;
      }
      if (uni((int)(wall_clock64() - t0 > (long long)D->watchdog_ticks))) {
        if (l == 0) raise_abort(D, ABORT_WATCHDOG, blockIdx.x);
        stop = 1;
        break;
      }
    }
    __builtin_amdgcn_s_sleep(1);
  }
  LDSQ unsigned* P = (LDSQ unsigned*)s_gpass[buf];
  const bool have = !stop && uni((int)rdy) != 0;
  int nm = 0, rows = 0, nodes = 0;
  unsigned code0 = 0;
  if (have) {
    fence_acquire();
    code0 = uni((unsigned)e);
    const bool got = act && rdy;
    const unsigned code = got ? (unsigned)e : code0;
    const int s = MSG_SLOT(code);
    const GQ unsigned* sd = B.sdesc + s * 16;
    const v4i d0 = *(const GQ v4i*)sd, d1 = *(const GQ v4i*)(sd + 4);
    const v4i c0 = *(const GQ v4i*)(sd + 8), c1 = *(const GQ v4i*)(sd + 12);
    const unsigned seq = (unsigned)d0.x, present = (unsigned)d1.w;
    const int inst = d0.y, to = d0.z, N = d0.w, eo = d1.x;
    const int cnt[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    int kc = 0, tsc = 0;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      kc = c == ctype ? cnt[c] : kc;
      tsc += c < ctype ? cnt[c] : 0;
    }
    const int K = edge ? kc : N;
    const bool ok = got && ((code ^ code0) & MSG_DIR_B) == 0u;
    const bool bwd = (code0 & MSG_DIR_B) != 0u;
    bool open = true, take = false;
    int r0 = 0, n0 = 0;
#pragma unroll
    for (int j = 0; j < G_MB; ++j) {
      const int Kj = __shfl(K, j), Nj = __shfl(N, j);
      const bool tj = open && __shfl((int)ok, j) != 0 && (j == 0 || (rows + Kj <= cap && (!bwd || j < room)));
      if (l == j) {
        r0 = rows;
        n0 = nodes;
        take = tj;
      }
      open = tj;
      if (tj) {
        rows += Kj;
        nodes += Nj;
        nm++;
      }
    }
    if (take) {
      unsigned plo, phi, pn;
      g_pack_parts(B, present, plo, phi, pn);
      LDSQ unsigned* M = P + G_HW + G_RW * l;
      M[0] = code;
      M[1] = seq;
      M[2] = (unsigned)s;
      M[3] = MSG_LOCAL(code);
      M[4] = (unsigned)K;
      M[5] = (unsigned)r0;
      M[6] = (unsigned)N;
      M[7] = (unsigned)n0;
      M[8] = present;
      M[9] = (unsigned)inst;
      M[10] = (unsigned)to;
      M[11] = (unsigned)eo;
      M[12] = (unsigned)tsc;
      M[13] = plo;
      M[14] = phi;
      M[15] = pn;
    }
  }
  if (l == 0) {
    P[0] = (unsigned)nm;
    P[1] = stop;
    P[2] = (unsigned)rows;
    P[3] = (unsigned)nodes;
    P[4] = code0 & MSG_DIR_B;
    if (block) s_stat[0] += (unsigned long long)(wall_clock64() - t0);
    s_stat[1] += (unsigned long long)nm;
    s_stat[2] += nm ? 1ull : 0ull;
  }
}

// What every thread knows of a pass (all of it the same in every lane), read after the barrier that follows
// g_form_pass.  r1..r3 / q1..q3: the first stacked row / graph node of messages 1..3, INT_MAX for a message the
// pass does not have.
struct GPass {
  const LDSQ unsigned* P;
  int nm, Kt, Nt, r1, r2, r3, q1, q2, q3;
  bool stop, bwd;
  __device__ __forceinline__ const LDSQ unsigned* msg(int m) const { return P + G_HW + G_RW * m; }
  __device__ __forceinline__ const LDSQ unsigned* of_row(int k) const { return msg((k >= r1) + (k >= r2) + (k >= r3)); }
  __device__ __forceinline__ const LDSQ unsigned* of_node(int n) const { return msg((n >= q1) + (n >= q2) + (n >= q3)); }
};

__device__ __forceinline__ GPass g_pass(int buf) {
  GPass p;
  p.P = (const LDSQ unsigned*)s_gpass[buf];
  p.nm = (int)uni(p.P[0]);
  p.stop = uni(p.P[1]) != 0u;
  p.Kt = (int)uni(p.P[2]);
  p.Nt = (int)uni(p.P[3]);
  p.bwd = uni(p.P[4]) != 0u;
  const int big = 0x7fffffff;
  p.r1 = p.nm > 1 ? (int)uni(p.msg(1)[5]) : big;
  p.r2 = p.nm > 2 ? (int)uni(p.msg(2)[5]) : big;
  p.r3 = p.nm > 3 ? (int)uni(p.msg(3)[5]) : big;
  p.q1 = p.nm > 1 ? (int)uni(p.msg(1)[7]) : big;
  p.q2 = p.nm > 2 ? (int)uni(p.msg(2)[7]) : big;
  p.q3 = p.nm > 3 ? (int)uni(p.msg(3)[7]) : big;
  return p;
}

// The view of message m's instance (the same in every lane), for the paths that take one message per pass.
__device__ __forceinline__ GView g_view_msg(const GData& d, const GPass& p, int m) {
  const LDSQ unsigned* M = p.msg(m);
  GView v;
  v.seq = uni(M[1]);
  v.N = (int)uni(M[6]);
  v.present = uni(M[8]);
  v.inst = (int)uni(M[9]);
  const int to = (int)uni(M[10]), eo = (int)uni(M[11]);
  v.kc = (int)uni(M[4]);
  v.tsc = (int)uni(M[12]);
  v.E = 0;
  v.target = 0.f;
  v.type = d.tok + to;
  v.src = d.src + eo;
  v.dst = d.dst + eo;
  v.tcount = d.tcount + v.inst * 8;
  v.inoff = d.inoff + to + v.inst;
  v.inedge = d.inedge + eo;
  v.tstart = d.tstart + v.inst * 9;
  v.tedge = d.tedge + eo;
  v.tsoff = d.tsoff + (long long)d.T * (to + v.inst);
  v.tsk = d.tsk + eo;
  return v;
}

// Items tid, tid + nthr, ... of `total`: two at a time, both fetched (ld) before either is used (st), so that a
// thread with several items has their memory round trips in flight together.
template <class Ld, class St>
__device__ __forceinline__ void for_items2(int total, int tid, int nthr, Ld ld, St st) {
  for (int i = tid; i < total; i += 2 * nthr) {
    const int j = i + nthr;
    const bool hj = j < total;
    const auto a = ld(i);
    const auto b = ld(hj ? j : i);
    st(i, a);
    if (hj) st(j, b);
  }
}

// Bit c set when the graph has edges of type c (at most 8 types).
__device__ __forceinline__ unsigned g_present_types(const GView& v, int T) {
  unsigned m = 0;
#pragma unroll
  for (int c = 0; c < 8; ++c) m |= (c < T && v.tcount[c < T ? c : 0] > 0) ? 1u << c : 0u;
  return uni(m);
}

// Sends one message per edge type that occurs in the graph: lane c of the calling wave posts to type c's ring.
// Whole wave, after a release fence.
__device__ __forceinline__ void g_post_edges(const GRings& R, unsigned present, int s, int it, bool backward) {
  const int c = threadIdx.x & 63;
  if (c < 8 && ((present >> c) & 1u)) ring_post(R.edge, MSG_MAKE(backward, s, it));
}

// Gradient w.r.t. element i of the states that entered a step whose backward
// pass has finished: Bcast / Flatmap backward over the edge types present
// (ascending), the update gate, the reset gate and the candidate.
// `present` = g_present_types(): bit c set when the graph has edges of type c.  All loads are unconditional
// (an absent type reads type 0's row and drops it) so that they are in flight together.  `step` = the propagation
// step whose backward pass produced the parts.
__device__ __forceinline__ float g_state_gradient(const GBufs& B, const GParts& ep, int s, int i, int step) {
  const long long NH = (long long)B.N * B.H;
  const GQ float* he = B.dHe + (long long)s * B.PE * NH + i;
  const GQ float* hp = B.dHp + ((long long)s * 2 + (step & 1)) * B.PA * NH + i;
  float e[12], p[12];
#pragma unroll
  for (int k = 0; k < 12; ++k) e[k] = he[(k < ep.n ? ep.off[k] : ep.off[0]) * NH];
#pragma unroll
  for (int k = 0; k < 12; ++k) p[k] = hp[(k < B.PA ? k : 0) * NH];
  float a = 0.f;
#pragma unroll
  for (int k = 0; k < 12; ++k)
    if (k < ep.n) a += e[k];
  // the GRU's parts: update gate, reset gate (parts Th .. PA - 1), then the candidate (parts 0 .. Th - 1)
  float g = 0.f, cnd = 0.f;
#pragma unroll
  for (int k = 0; k < 12; ++k) {
    if (k >= B.Th && k < B.PA) g += p[k];
    if (k < B.Th) cnd += p[k];
  }
  a += g;
  a += cnd;
  return a;
}

// Four consecutive elements (c .. c + 3) of a_k = sum of the messages on node k's incoming edges, ascending edge
// order; the edge numbers of up to four edges are fetched together, then their rows.
__device__ __forceinline__ v4f g_sum_incoming4(const GQ float* msg, const GView& v, int k, int c, int H) {
  const int p0 = v.inoff[k], p1 = v.inoff[k + 1];
  v4f x = {0.f, 0.f, 0.f, 0.f};
  for (int p = p0; p < p1; p += 4) {
    int e[4];
    v4f m[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) e[a] = v.inedge[p + a < p1 ? p + a : p1 - 1];
#pragma unroll
    for (int a = 0; a < 4; ++a) m[a] = *(const GQ v4f*)(msg + (long long)e[a] * H + c);
#pragma unroll
    for (int a = 0; a < 4; ++a)
      if (p + a < p1) x += m[a];
  }
  return x;
}

__device__ __forceinline__ v4f sigmoid4(v4f y) { return (v4f){sigmoidf_(y.x), sigmoidf_(y.y), sigmoidf_(y.z), sigmoidf_(y.w)}; }
__device__ __forceinline__ v4f tanh4(v4f y) { return (v4f){tanhf(y.x), tanhf(y.y), tanhf(y.z), tanhf(y.w)}; }

// Four consecutive elements of the same sum.
__device__ __forceinline__ v4f g_state_gradient4(const GBufs& B, const GParts& ep, int s, int i, int step) {
  const long long NH = (long long)B.N * B.H;
  const GQ float* he = B.dHe + (long long)s * B.PE * NH + i;
  const GQ float* hp = B.dHp + ((long long)s * 2 + (step & 1)) * B.PA * NH + i;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  v4f a = zero, g = zero, cnd = zero;
  if (B.PE <= 8 && B.PA <= 4) {
    // few parts (no node split, or only lightly): eight and four fetches in flight instead of twelve and twelve
    v4f e[8], p[4];
#pragma unroll
    for (int k = 0; k < 8; ++k) e[k] = *(const GQ v4f*)(he + (k < ep.n ? ep.off[k] : ep.off[0]) * NH);
#pragma unroll
    for (int k = 0; k < 4; ++k) p[k] = *(const GQ v4f*)(hp + (k < B.PA ? k : 0) * NH);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k < ep.n) a += e[k];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (k >= B.Th && k < B.PA) g += p[k];
      if (k < B.Th) cnd += p[k];
    }
  } else {
    v4f e[12], p[12];
#pragma unroll
    for (int k = 0; k < 12; ++k) e[k] = *(const GQ v4f*)(he + (k < ep.n ? ep.off[k] : ep.off[0]) * NH);
#pragma unroll
    for (int k = 0; k < 12; ++k) p[k] = *(const GQ v4f*)(hp + (k < B.PA ? k : 0) * NH);
#pragma unroll
    for (int k = 0; k < 12; ++k)
      if (k < ep.n) a += e[k];
#pragma unroll
    for (int k = 0; k < 12; ++k) {
      if (k >= B.Th && k < B.PA) g += p[k];
      if (k < B.Th) cnd += p[k];
    }
  }
  a += g;
  a += cnd;
  return a;
}

// The same, with the instance's parts of dHe given packed (4 bits each, pn of them): the form a pass record holds.
__device__ __forceinline__ v4f g_state_gradient4p(const GBufs& B, unsigned plo, unsigned phi, int pn, int s, int i, int step) {
  const long long NH = (long long)B.N * B.H;
  const GQ float* he = B.dHe + (long long)s * B.PE * NH + i;
  const GQ float* hp = B.dHp + ((long long)s * 2 + (step & 1)) * B.PA * NH + i;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  v4f a = zero, g = zero, cnd = zero;
  const unsigned long long pk = ((unsigned long long)phi << 32) | plo;
  if (B.PE <= 8 && B.PA <= 4) {
    v4f e[8], p[4];
#pragma unroll
    for (int k = 0; k < 8; ++k) e[k] = *(const GQ v4f*)(he + (long long)((pk >> (4 * (k < pn ? k : 0))) & 15u) * NH);
#pragma unroll
    for (int k = 0; k < 4; ++k) p[k] = *(const GQ v4f*)(hp + (k < B.PA ? k : 0) * NH);
#pragma unroll
    for (int k = 0; k < 8; ++k)
      if (k < pn) a += e[k];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (k >= B.Th && k < B.PA) g += p[k];
      if (k < B.Th) cnd += p[k];
    }
  } else {
    v4f e[12], p[12];
#pragma unroll
    for (int k = 0; k < 12; ++k) e[k] = *(const GQ v4f*)(he + (long long)((pk >> (4 * (k < pn ? k : 0))) & 15u) * NH);
#pragma unroll
    for (int k = 0; k < 12; ++k) p[k] = *(const GQ v4f*)(hp + (k < B.PA ? k : 0) * NH);
#pragma unroll
    for (int k = 0; k < 12; ++k)
      if (k < pn) a += e[k];
#pragma unroll
    for (int k = 0; k < 12; ++k) {
      if (k >= B.Th && k < B.PA) g += p[k];
      if (k < B.Th) cnd += p[k];
    }
  }
  a += g;
  a += cnd;
  return a;
}

// Sum of the PA parts of the gradient w.r.t. A at float offset o (four consecutive elements): update gate, reset
// gate, then candidate -- (update + reset) + candidate when no node is tiled.
__device__ __forceinline__ v4f g_sum_dA4(const GBufs& B, const GQ float* dA, long long o) {
  const long long NH = (long long)B.N * B.H;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  v4f g = zero, cnd = zero;
  if (B.PA <= 4) {
    v4f p[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) p[k] = *(const GQ v4f*)(dA + (k < B.PA ? k : 0) * NH + o);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (k >= B.Th && k < B.PA) g += p[k];
      if (k < B.Th) cnd += p[k];
    }
  } else {
    v4f p[12];
#pragma unroll
    for (int k = 0; k < 12; ++k) p[k] = *(const GQ v4f*)(dA + (k < B.PA ? k : 0) * NH + o);
#pragma unroll
    for (int k = 0; k < 12; ++k) {
      if (k >= B.Th && k < B.PA) g += p[k];
      if (k < B.Th) cnd += p[k];
    }
  }
  return g + cnd;
}
__device__ __forceinline__ float g_sum_dA(const GBufs& B, const GQ float* dA, long long o) {
  const long long NH = (long long)B.N * B.H;
  float g = 0.f, cnd = 0.f;
  for (int k = B.Th; k < B.PA; ++k) g += dA[k * NH + o];
  for (int k = 0; k < B.Th; ++k) cnd += dA[k * NH + o];
  return g + cnd;
}

// LDS pieces every dense graph worker carves: weight tile, bias, row / column maps for the update.
struct GTile {
  float *Wg, *bg;
  LDSQ float *Wl, *bl;
  LDSQ int *rowmap, *colmap;
};

__device__ __forceinline__ GTile g_tile_setup(Lds& L, const GQ NodeDev& nd, const Tile& t) {
  GTile g;
  g.Wg = L.take(t.Rp * t.ldw);
  g.bg = L.take(t.Rp);
  g.Wl = (LDSQ float*)g.Wg;
  g.bl = (LDSQ float*)g.bg;
  const int CMW = ((amp_round16(t.Cl) + 63) >> 6) << 6;
  g.rowmap = (LDSQ int*)L.take(t.Rp);
  g.colmap = (LDSQ int*)L.take(CMW);
  tile_load(nd, t, g.Wg, g.bg);
  for (int i = threadIdx.x; i < t.Rp; i += AMP_THREADS) g.rowmap[i] = i < t.R ? t.grow(i) : -1;
  for (int i = threadIdx.x; i < CMW; i += AMP_THREADS) g.colmap[i] = t.ncol(i);
  return g;
}

// Appends K (delta, input) rows held in LDS to the worker's pending list in HBM and adds the delta rows to the
// bias gradient of row threadIdx.x.
__device__ __forceinline__ void g_pend_append(GQ float* pend, int Rp, int stride, unsigned first, const LDSQ float* Dl, int ldd,
                                              int R, const LDSQ float* X, int ldx, int C, int K, float& gb) {
  // 16 bytes at a time: the rows' padding (beyond R in Dl, beyond C in X) is zero, and ldd >= Rp, ldx >= stride - Rp
  const int per = stride >> 2;
  for (int idx = threadIdx.x; idx < K * per; idx += AMP_THREADS) {
    const int k = idx / per, j = (idx - k * per) << 2;
    const v4f v = j < Rp ? *(const LDSQ v4f*)(Dl + k * ldd + j) : *(const LDSQ v4f*)(X + k * ldx + j - Rp);
    *(GQ v4f*)(pend + (long long)(first + k) * stride + j) = v;
  }
  if ((int)threadIdx.x < R) {
    // eight rows' entries are read together; the sum keeps the rows' order
    int k = 0;
    for (; k + 7 < K; k += 8) {
      float d[8];
#pragma unroll
      for (int a = 0; a < 8; ++a) d[a] = Dl[(k + a) * ldd + threadIdx.x];
#pragma unroll
      for (int a = 0; a < 8; ++a) gb += d[a];
    }
    for (; k < K; ++k) gb += Dl[k * ldd + threadIdx.x];
  }
}

// Counts nmsg gradients (grouped messages, K rows in all, already appended to the pending list) and updates when
// min_update_frequency is reached.
template <int NRBT, int NCGT>
__device__ __forceinline__ void g_count_and_update(const GQ AmpDev* D, const GQ WorkerDev* W, const GQ NodeDev& nd, const Tile& t,
                                                   const GTile& g, const GQ float* pend, unsigned& count, unsigned& nrows,
                                                   unsigned& tstep, int nmsg, int K, float& gb) {
  count += nmsg;
  nrows += K;
  if ((int)count >= uni(nd.muf)) {
    tstep++;
    if (threadIdx.x == 0) note_update(D);
    __syncthreads();   // the appended rows of every wave are in HBM
    tree_update_from_pend<NRBT, NCGT>(g.Wl, g.bl, &nd, t, pend, nrows, count, tstep, g.rowmap, g.colmap, gb);
    gb = 0.f;
    count = 0;
    nrows = 0;
    LOG(W->node, 2, 0, 0);
  }
}

// ---------------------------------------------------------------- lookup
__device__ __noinline__ void role_g_lookup(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& lk = D->node[0];
  const GBufs B = g_bufs(D);
  const GData gd = g_data(D);
  const GRings rg = g_rings(D);
  const int H = B.H, V = D->n_node_types;
  LDSQ float* El = (LDSQ float*)lds;
  LDSQ float* gt = El + ((V * H + 3) & ~3);   // [N][H] gradient w.r.t. the lookup's output
  GQ float* lkP = (GQ float*)lk.P;
  GQ float* lkG = (GQ float*)lk.G;
  for (int i = threadIdx.x; i < V * H; i += AMP_THREADS) El[i] = lkP[i];
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code);
    const unsigned seq = uni(gd.slot_seq[s]);
    const GView v = g_view(gd, s);
    const unsigned present = g_present_types(v, B.T);
    if (!(code & MSG_DIR_B)) {
      GQ float* h0 = B.Hm + B.hm(s, 0);
      for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) {
        const int n = i / H, j = i - n * H;
        h0[i] = El[v.type[n] * H + j];
      }
      if (threadIdx.x < 16) {
        const int w = threadIdx.x;
        const unsigned val = w == 0   ? seq
                             : w == 1 ? (unsigned)v.inst
                             : w == 2 ? (unsigned)gd.tok_off[v.inst]
                             : w == 3 ? (unsigned)v.N
                             : w == 4 ? (unsigned)gd.edge_off[v.inst]
                             : w == 5 ? (unsigned)v.E
                             : w == 6 ? __float_as_uint(v.target)
                             : w == 7 ? present
                                      : (unsigned)v.tcount[w - 8];
        B.sdesc[s * 16 + w] = val;
      }
      LOG(0, 0, seq, 0);
      publish_barrier();
      if (threadIdx.x < 64) {
        fence_release();
        g_post_edges(rg, present, s, 0, false);
      }
      continue;
    }
    // backward: scatter-add the rows into the table's accumulator, node by node
    const GParts ep = g_edge_parts(B, present);
    for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) gt[i] = g_state_gradient(B, ep, s, i, 0);
    lds_barrier();
    for (int j = threadIdx.x; j < H; j += AMP_THREADS)
      for (int n = 0; n < v.N; ++n) lkG[v.type[n] * H + j] += gt[n * H + j];
    LOG(0, 1, seq, 0);
    publish_barrier();
    if (threadIdx.x == 0) {
      fence_release();
      ring_post(rg.ctl, MSG_MAKE(1, s, 0));
    }
    count++;
    if ((int)count >= lk.muf) {
      tstep++;
      if (threadIdx.x == 0) note_update(D);
      const float sc = lk.lr * (lk.mean ? 1.f / (float)count : 1.f);
      for (int i = threadIdx.x; i < V * H; i += AMP_THREADS) {
        El[i] -= sc * lkG[i];
        lkG[i] = 0.f;
      }
      __syncthreads();
      count = 0;
      LOG(0, 2, 0, 0);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < V * H; i += AMP_THREADS) lkP[i] = El[i];
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}

// ---------------------------------------------------------------- edge linear of type c
template <int NRBT, int NCGT>
__device__ __noinline__ void role_g_edge(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const GData gd = g_data(D);
  const GRings rg = g_rings(D);
  const Pend pd = make_pend(W, t);
  GQ float* pend = (GQ float*)pd.base;
  const int H = B.H, ctype = uni(W->aux), CAP = uni(W->kb), Hs = amp_ldrow(H);
  const int u0 = t.u0, nu = t.nu, tile = uni(W->tile);   // this tile's output units = rows of W
  const bool vec = (H & 3) == 0 && (u0 & 3) == 0 && (nu & 3) == 0;   // rows can be moved 16 bytes at a time
  const int G1 = H >> 2, GU = nu >> 2;
  const int NRB = t.Rp >> 4, NCG = amp_round16(H) >> 4;
  Lds L{lds};
  const GTile g = g_tile_setup(L, nd, t);
  LDSQ float* X = (LDSQ float*)L.take(CAP * Hs);     // inputs h_src of the stacked rows; later the products W^T delta
  LDSQ float* Y = (LDSQ float*)L.take(CAP * Hs);     // outputs / deltas
  LDSQ int* erow = (LDSQ int*)L.take(CAP);           // the edge a stacked row stands for
  for (int i = threadIdx.x; i < CAP * Hs; i += AMP_THREADS) X[i] = Y[i] = 0.f;
  GQ float* ndG = (GQ float*)nd.G;
  float gb = (int)threadIdx.x < t.R ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  const int maxm = vec ? G_MB : 1;                    // the element-by-element paths take one message at a time
  const long long NH = (long long)B.N * H;
  const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
  // What a pass needs in LDS before its product: row k of a message = its k-th edge of this type, ascending (Group
  // orders its rows by edge index).  Forward and backward: the source node's state.  Backward also delta_e = this
  // tile's units of dA[dst(e)] (Bcast backward on A: (update + reset) + candidate, each the sum of its tiles' parts).
  auto stage = [&](const GPass& p, int tid, int nthr) {
    if (vec) {
      const int GY = Hs >> 2, GZ = GY - GU;
      for (int idx = tid; idx < p.Kt * (GY - G1); idx += nthr)   // padding columns of the used rows
        *(LDSQ v4f*)(X + (idx / (GY - G1)) * Hs + H + ((idx % (GY - G1)) << 2)) = zero4;
      if (!p.bwd) {
        struct It {
          v4f x;
          int e;
        };
        for_items2(p.Kt * G1, tid, nthr,
                   [&](int idx) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], q = (int)M[11] + (int)M[12] + k - (int)M[5];
                     It r;
                     r.e = gd.tedge[q];
                     r.x = *(const GQ v4f*)(B.Hm + B.hm(s, it) + (long long)gd.tsrc[q] * H + c);
                     return r;
                   },
                   [&](int idx, const It& r) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     *(LDSQ v4f*)(X + k * Hs + c) = r.x;
                     if (c == 0) erow[k] = r.e;
                   });
      } else {
        // the tile's units of the delta rows come with the first GU groups of a row, zeros fill the rest
        struct It {
          v4f x, d;
        };
        for_items2(p.Kt * G1, tid, nthr,
                   [&](int idx) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], q = (int)M[11] + (int)M[12] + k - (int)M[5];
                     const int sn = gd.tsrc[q], dn = gd.tdst[q];
                     It r;
                     r.x = *(const GQ v4f*)(B.Hm + B.hm(s, it) + (long long)sn * H + c);
                     r.d = c < nu ? g_sum_dA4(B, B.dA + (long long)s * B.PA * NH + u0, (long long)dn * H + c) : zero4;
                     return r;
                   },
                   [&](int idx, const It& r) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     *(LDSQ v4f*)(X + k * Hs + c) = r.x;
                     if (c < nu) *(LDSQ v4f*)(Y + k * Hs + c) = r.d;
                   });
        for (int idx = tid; idx < p.Kt * GZ; idx += nthr)
          *(LDSQ v4f*)(Y + (idx / GZ) * Hs + nu + ((idx % GZ) << 2)) = zero4;
      }
      return;
    }
    // element by element: one message
    const GView v = g_view_msg(gd, p, 0);
    const int s = (int)uni(p.msg(0)[2]), it = (int)uni(p.msg(0)[3]), K = p.Kt;
    const GQ int* te = v.tedge + v.tsc;
    const GQ float* h = B.Hm + B.hm(s, it);
    for (int i = tid; i < K * Hs; i += nthr) {
      const int k = i / Hs, j = i - k * Hs;
      X[i] = j < H ? h[v.src[te[k]] * H + j] : 0.f;   // padding columns of a used row are zero
    }
    if (p.bwd) {
      const GQ float* dA = B.dA + (long long)s * B.PA * NH + u0;
      for (int i = tid; i < K * Hs; i += nthr) {
        const int k = i / Hs, j = i - k * Hs;
        Y[i] = j < nu ? g_sum_dA(B, dA, (long long)v.dst[te[k]] * H + j) : 0.f;
      }
    }
  };
  auto room = [&](unsigned cnt) {
    const int muf = uni(nd.muf);
    return (int)cnt >= muf || muf < 1 ? (muf < 1 ? 1 : muf) : muf - (int)cnt;
  };
  // Wave 1 looks for the next pass while the present one's stores drain; if it is there, waves 1..7 stage it while
  // wave 0 publishes the present one, otherwise wave 1 waits for it afterwards.
  int pb = 0;
  bool staged = false;
  if ((threadIdx.x >> 6) == 1) g_form_pass(D, gd, B, mine, head, CAP, maxm, room(count), ctype, true, true, pb);
  lds_barrier();
  for (;;) {
    const GPass p = g_pass(pb);
    if (p.stop) break;
    head += (unsigned)p.nm;
    PHASE(0);
    if (!staged) stage(p, threadIdx.x, AMP_THREADS);
    lds_barrier();
    const int NB = (p.Kt + 15) >> 4;
    const unsigned cnt_after = p.bwd ? count + (unsigned)p.nm : count;
    // wave 1 looks for the next pass while the other waves write this one's results out
    const bool scout = (threadIdx.x >> 6) == 1;
    const int wtid = threadIdx.x < 64 ? threadIdx.x : threadIdx.x - 64, wn = AMP_THREADS - 64;
    if (!p.bwd) {
      PHASE(1);
      mfma_rows<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, g.bl, X, Hs, NB, Y, Hs);
      PHASE(2);
      // this tile's units of every message
      if (scout) {
        g_form_pass(D, gd, B, mine, head, CAP, maxm, room(cnt_after), ctype, true, false, pb ^ 1);
      } else if (vec) {
        for (int idx = wtid; idx < p.Kt * GU; idx += wn) {
          const int k = idx / GU, c = (idx - k * GU) << 2;
          const int s = p.of_row(k)[2];
          *(GQ v4f*)(B.Msg + ((long long)s * B.Em + erow[k]) * H + u0 + c) = *(const LDSQ v4f*)(Y + k * Hs + c);
        }
      } else {
        const GView v = g_view_msg(gd, p, 0);
        const GQ int* te = v.tedge + v.tsc;
        GQ float* msg = B.Msg + (long long)(int)uni(p.msg(0)[2]) * B.Em * H + u0;
        for (int i = wtid; i < p.Kt * nu; i += wn) {
          const int k = i / nu, j = i - k * nu;
          msg[te[k] * H + j] = Y[k * Hs + j];
        }
      }
      for (int m = 0; m < p.nm; ++m) LOG(W->node, 0, p.msg(m)[1], p.msg(m)[3]);
    } else {
      PHASE(4);
      for (int m = 0; m < p.nm; ++m) LOG(W->node, 1, p.msg(m)[1], p.msg(m)[3]);
      g_pend_append(pend, pd.Rp, pd.stride, nrows, Y, Hs, nu, X, Hs, H, p.Kt, gb);   // one gradient per group
      lds_barrier();
      PHASE(5);
      mfma_cols<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, Y, Hs, NB, X, Hs);
      PHASE(6);
      // dh_src += W^T delta_e: per source node, its edges of this type in ascending order -> this tile's part
      if (scout) {
        g_form_pass(D, gd, B, mine, head, CAP, maxm, room(cnt_after), ctype, true, false, pb ^ 1);
      } else if (vec) {
        for (int idx = wtid; idx < p.Nt * G1; idx += wn) {
          const int n = idx / G1, c = (idx - n * G1) << 2;
          const LDSQ unsigned* M = p.of_node(n);
          const int s = M[2], r0 = M[5], N = M[6], nn = n - (int)M[7], inst = M[9], to = M[10], eo = M[11], tsc = M[12];
          const GQ int* so = gd.tsoff + (long long)gd.T * (to + inst) + ctype * (N + 1) + nn;
          const GQ int* sk = gd.tsk + eo + tsc;
          const int p0 = so[0], p1 = so[1];
          v4f a = zero4;
          for (int q = p0; q < p1; q += 4) {
            int kk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) kk[u] = sk[q + u < p1 ? q + u : p1 - 1];
#pragma unroll
            for (int u = 0; u < 4; ++u)
              if (q + u < p1) a += *(const LDSQ v4f*)(X + (r0 + kk[u]) * Hs + c);
          }
          *(GQ v4f*)(B.dHe + ((long long)s * B.PE + B.eoff(ctype) + tile) * NH + nn * H + c) = a;
        }
      } else {
        const GView v = g_view_msg(gd, p, 0);
        GQ float* dHe = B.dHe + ((long long)(int)uni(p.msg(0)[2]) * B.PE + B.eoff(ctype) + tile) * NH;
        const GQ int* so = v.tsoff + ctype * (v.N + 1);
        const GQ int* sk = v.tsk + v.tsc;
        for (int i = wtid; i < v.N * H; i += wn) {
          const int n = i / H, j = i - n * H;
          float a = 0.f;
          for (int q = so[n]; q < so[n + 1]; ++q) a += X[sk[q] * Hs + j];
          dHe[i] = a;
        }
      }
    }
    publish_barrier();
    const GPass pn = g_pass(pb ^ 1);
    const bool have = pn.nm > 0;
    if (have && threadIdx.x >= 64) stage(pn, threadIdx.x - 64, AMP_THREADS - 64);
    if (threadIdx.x < 64) {
      fence_release();
      const int m = threadIdx.x;
      if (m < p.nm) {
        const int s = p.msg(m)[2], it = p.msg(m)[3];
        const int nact = g_present_tiles(B, p.msg(m)[8]);   // tiles of every edge type the graph uses
        if (!p.bwd) {
          // the last tile to arrive completes the step's messages; Ungroup, regrouping by target node and the sum
          // are the GRU nodes' part
          if (join_arrive(B.cnt + s * 8 + 0, nact)) {
            ring_post(rg.gz, MSG_MAKE(0, s, it));
            ring_post(rg.gr, MSG_MAKE(0, s, it));
          }
        } else if (join_arrive(B.cnt + s * 8 + 3, nact)) {
          if (it > 0)
            ring_post(rg.gh, MSG_MAKE(1, s, it - 1));
          else
            ring_post(rg.lookup, MSG_MAKE(1, s, 0));
        }
      }
    }
    PHASE(3);
    if (p.bwd) g_count_and_update<NRBT, NCGT>(D, W, nd, t, g, pend, count, nrows, tstep, p.nm, p.Kt, gb);
    PHASE(7);
    if (!have && (threadIdx.x >> 6) == 1) g_form_pass(D, gd, B, mine, head, CAP, maxm, room(count), ctype, true, true, pb ^ 1);
    lds_barrier();
    staged = have;
    pb ^= 1;
  }
  tile_store(nd, t, g.Wg, g.bg);
  if ((int)threadIdx.x < t.R) ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] = gb;
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
    W->wstate[4] = nrows;
  }
}

// ---------------------------------------------------------------- GRU gate nodes (aux 0: update z, aux 1: reset r)
template <int NRBT, int NCGT>
__device__ __noinline__ void role_g_gate(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const GData gd = g_data(D);
  const GRings rg = g_rings(D);
  const Pend pd = make_pend(W, t);
  GQ float* pend = (GQ float*)pd.base;
  const int H = B.H, C = 2 * H, CAP = uni(W->kb), which = uni(W->aux), Hs = amp_ldrow(H), Cs = amp_ldrow(C);
  const int u0 = t.u0, nu = t.nu, tile = uni(W->tile);   // this tile's output units = rows of W
  const bool vec = (H & 3) == 0 && (u0 & 3) == 0 && (nu & 3) == 0;   // rows can be moved 16 bytes at a time
  const int G1 = H >> 2, GU = nu >> 2;
  const int part = B.Th + (which ? B.Tz : 0) + tile;     // this tile's part of dA / dHp
  const int NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  const GTile g = g_tile_setup(L, nd, t);
  LDSQ float* X = (LDSQ float*)L.take(CAP * Cs);     // inputs of the stacked rows; later W^T delta
  LDSQ float* Y = (LDSQ float*)L.take(CAP * Hs);
  for (int i = threadIdx.x; i < CAP * Cs; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < CAP * Hs; i += AMP_THREADS) Y[i] = 0.f;
  GQ float* ndG = (GQ float*)nd.G;
  float gb = (int)threadIdx.x < t.R ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  const int maxm = vec ? G_MB : 1;                    // the element-by-element paths take one message at a time
  const bool rec_a = which == 0 && tile == 0;         // the update gate's first tile records the aggregated messages
  const long long NHp = (long long)B.N * H;
  const int ndp = which == 0 ? 1 : B.Th;
  const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
  // What a pass needs in LDS before its product.  Forward: Ungroup, regroup by target node, sum (a_v = sum over
  // incoming edges in edge order) beside the states.  Backward: the recorded inputs and this tile's units of the
  // pre-activation gradient: the update gate's was written by the candidate tile that owns each unit; the reset
  // gate's is the sum of the candidate tiles' parts (each a full-width W^T delta).
  // `nthr` threads, `tid` = this thread's number among them.
  auto stage = [&](const GPass& p, int tid, int nthr) {
    if (vec) {
      // 16 bytes per thread and step; the padding columns of a used row are written as zeros every time (an
      // unused row may hold anything, and the products leave 0 x anything in its padding)
      const int GP = (Cs - C) >> 2;
      for (int idx = tid; idx < p.Kt * GP; idx += nthr)
        *(LDSQ v4f*)(X + (idx / GP) * Cs + C + ((idx % GP) << 2)) = zero4;
      if (!p.bwd) {
        // one item per (row, 4 units): its part of h travels while the chain inoff -> inedge -> message rows runs
        struct It {
          v4f hv, m0, m1, m2, m3;
          int p0, p1;
        };
        for_items2(p.Kt * G1, tid, nthr,
                   [&](int idx) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], kk = k - (int)M[5], inst = M[9], to = M[10], eo = M[11];
                     const GQ float* msg = B.Msg + (long long)s * B.Em * H + c;
                     const GQ int* inoff = gd.inoff + to + inst + kk;
                     const GQ int* inedge = gd.inedge + eo;
                     It r;
                     r.hv = *(const GQ v4f*)(B.Hm + B.hm(s, it) + kk * H + c);
                     r.p0 = inoff[0];
                     r.p1 = inoff[1];
                     // the first four incoming edges without a branch (a node of a molecule rarely has more)
                     int e[4];
#pragma unroll
                     for (int a = 0; a < 4; ++a) {
                       const int q = r.p0 + a < r.p1 ? r.p0 + a : r.p1 - 1;
                       e[a] = q >= r.p0 ? inedge[q] : 0;   // a node without incoming edges reads row 0 and drops it
                     }
                     r.m0 = *(const GQ v4f*)(msg + (long long)e[0] * H);
                     r.m1 = *(const GQ v4f*)(msg + (long long)e[1] * H);
                     r.m2 = *(const GQ v4f*)(msg + (long long)e[2] * H);
                     r.m3 = *(const GQ v4f*)(msg + (long long)e[3] * H);
                     return r;
                   },
                   [&](int idx, const It& r) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const int deg = r.p1 - r.p0;
                     v4f x = zero4;
                     if (deg > 0) x += r.m0;
                     if (deg > 1) x += r.m1;
                     if (deg > 2) x += r.m2;
                     if (deg > 3) x += r.m3;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], kk = k - (int)M[5];
                     if (deg > 4) {
                       const GQ float* msg = B.Msg + (long long)s * B.Em * H + c;
                       const GQ int* inedge = gd.inedge + (int)M[11];
                       for (int q = r.p0 + 4; q < r.p1; ++q) x += *(const GQ v4f*)(msg + (long long)inedge[q] * H);
                     }
                     if (rec_a) *(GQ v4f*)(B.A + B.st(s, it) + kk * H + c) = x;   // read again by all three GRU nodes
                     *(LDSQ v4f*)(X + k * Cs + c) = x;
                     *(LDSQ v4f*)(X + k * Cs + H + c) = r.hv;
                   });
      } else {
        // the H real columns of every row, the delta's zero padding afterwards
        const int GY = Hs >> 2, GZ = GY - G1;
        struct It {
          v4f a, hv, dp;
        };
        for_items2(p.Kt * G1, tid, nthr,
                   [&](int idx) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], kk = k - (int)M[5];
                     const bool ind = c < nu;
                     const int o = kk * H + c, od = kk * H + (ind ? c : 0);
                     const GQ float* dpre = (which == 0 ? B.dZ + B.sl(s) : B.dR + B.sl(s) * B.Th) + u0;
                     It r;
                     r.a = *(const GQ v4f*)(B.A + B.st(s, it) + o);
                     r.hv = *(const GQ v4f*)(B.Hm + B.hm(s, it) + o);
                     v4f dq[4];
#pragma unroll
                     for (int q = 0; q < 4; ++q) dq[q] = *(const GQ v4f*)(dpre + (q < ndp ? q : 0) * NHp + od);
                     r.dp = dq[0];
#pragma unroll
                     for (int q = 1; q < 4; ++q)
                       if (q < ndp) r.dp += dq[q];
                     if (!ind) r.dp = zero4;
                     return r;
                   },
                   [&](int idx, const It& r) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     *(LDSQ v4f*)(X + k * Cs + c) = r.a;
                     *(LDSQ v4f*)(X + k * Cs + H + c) = r.hv;
                     *(LDSQ v4f*)(Y + k * Hs + c) = r.dp;
                   });
        for (int idx = tid; idx < p.Kt * GZ; idx += nthr)
          *(LDSQ v4f*)(Y + (idx / GZ) * Hs + H + ((idx % GZ) << 2)) = zero4;
      }
      return;
    }
    // element by element: one message
    const GView v = g_view_msg(gd, p, 0);
    const int s = (int)uni(p.msg(0)[2]), it = (int)uni(p.msg(0)[3]), K = p.Kt;
    GQ float* A = B.A + B.st(s, it);
    const GQ float* h = B.Hm + B.hm(s, it);
    if (!p.bwd) {
      const GQ float* msg = B.Msg + (long long)s * B.Em * H;
      for (int i = tid; i < K * Cs; i += nthr) {
        const int k = i / Cs, c = i - k * Cs;
        float x = 0.f;   // padding columns of a used row are zero
        if (c < H) {
          for (int q = v.inoff[k]; q < v.inoff[k + 1]; ++q) x += msg[v.inedge[q] * H + c];
          if (rec_a) A[k * H + c] = x;
        } else if (c < C) {
          x = h[k * H + c - H];
        }
        X[i] = x;
      }
    } else {
      const GQ float* dpre = (which == 0 ? B.dZ + B.sl(s) : B.dR + B.sl(s) * B.Th) + u0;
      for (int i = tid; i < K * Cs; i += nthr) {
        const int k = i / Cs, c = i - k * Cs;
        X[i] = c < H ? A[k * H + c] : c < C ? h[k * H + c - H] : 0.f;
      }
      for (int i = tid; i < K * Hs; i += nthr) {
        const int k = i / Hs, j = i - k * Hs;
        float d = 0.f;
        if (j < nu)
          for (int q = 0; q < ndp; ++q) d += dpre[q * NHp + k * H + j];
        Y[i] = d;
      }
    }
  };
  auto room = [&](unsigned cnt) {
    const int muf = uni(nd.muf);
    return (int)cnt >= muf || muf < 1 ? (muf < 1 ? 1 : muf) : muf - (int)cnt;
  };
  // Wave 1 looks for the next pass while the present one's stores drain; if it is there, waves 1..7 stage it while
  // wave 0 publishes the present one (fence, joins, posts) -- the two do not touch the same memory -- otherwise
  // wave 1 waits for it afterwards.
  int pb = 0;
  bool staged = false;
  if ((threadIdx.x >> 6) == 1) g_form_pass(D, gd, B, mine, head, CAP, maxm, room(count), 0, false, true, pb);
  lds_barrier();
  for (;;) {
    const GPass p = g_pass(pb);
    if (p.stop) break;
    head += (unsigned)p.nm;
    PHASE(0);
    if (!staged) stage(p, threadIdx.x, AMP_THREADS);
    lds_barrier();
    const int NB = (p.Kt + 15) >> 4;
    const unsigned cnt_after = p.bwd ? count + (unsigned)p.nm : count;
    // wave 1 looks for the next pass while the other waves write this one's results out
    const bool scout = (threadIdx.x >> 6) == 1;
    const int wtid = threadIdx.x < 64 ? threadIdx.x : threadIdx.x - 64, wn = AMP_THREADS - 64;
    if (!p.bwd) {
      PHASE(1);
      mfma_rows<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, g.bl, X, Cs, NB, Y, Hs);
      PHASE(2);
      GQ float* out = which == 0 ? B.Z : B.Rr;
      if (scout) {
        g_form_pass(D, gd, B, mine, head, CAP, maxm, room(cnt_after), 0, false, false, pb ^ 1);
      } else if (vec) {
        for (int idx = wtid; idx < p.Kt * GU; idx += wn) {
          const int k = idx / GU, c = (idx - k * GU) << 2;
          const LDSQ unsigned* M = p.of_row(k);
          const int s = M[2], it = M[3], kk = k - (int)M[5];
          *(GQ v4f*)(out + B.st(s, it) + kk * H + u0 + c) = sigmoid4(*(const LDSQ v4f*)(Y + k * Hs + c));
        }
      } else {
        GQ float* outp = out + B.st((int)uni(p.msg(0)[2]), (int)uni(p.msg(0)[3])) + u0;
        for (int i = wtid; i < p.Kt * nu; i += wn) outp[(i / nu) * H + i % nu] = sigmoidf_(Y[(i / nu) * Hs + i % nu]);
      }
      for (int m = 0; m < p.nm; ++m) LOG(W->node, 0, p.msg(m)[1], p.msg(m)[3]);
    } else {
      PHASE(4);
      for (int m = 0; m < p.nm; ++m) LOG(W->node, 1, p.msg(m)[1], p.msg(m)[3]);
      g_pend_append(pend, pd.Rp, pd.stride, nrows, Y, Hs, nu, X, Cs, C, p.Kt, gb);
      lds_barrier();
      PHASE(5);
      mfma_cols<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, Y, Hs, NB, X, Cs);
      PHASE(6);
      if (scout) {
        g_form_pass(D, gd, B, mine, head, CAP, maxm, room(cnt_after), 0, false, false, pb ^ 1);
      } else if (vec) {
        for (int idx = wtid; idx < p.Kt * G1; idx += wn) {
          const int k = idx / G1, c = (idx - k * G1) << 2;
          const LDSQ unsigned* M = p.of_row(k);
          const int s = M[2], it = M[3], kk = k - (int)M[5];
          GQ float* dA = B.dA + ((long long)s * B.PA + part) * B.N * H;
          GQ float* dHp = B.dHp + (((long long)s * 2 + (it & 1)) * B.PA + part) * B.N * H;
          *(GQ v4f*)(dA + kk * H + c) = *(const LDSQ v4f*)(X + k * Cs + c);
          *(GQ v4f*)(dHp + kk * H + c) = *(const LDSQ v4f*)(X + k * Cs + H + c);
        }
      } else {
        const int s = (int)uni(p.msg(0)[2]), it = (int)uni(p.msg(0)[3]);
        GQ float* dA = B.dA + ((long long)s * B.PA + part) * B.N * H;
        GQ float* dHp = B.dHp + (((long long)s * 2 + (it & 1)) * B.PA + part) * B.N * H;
        for (int i = wtid; i < p.Kt * C; i += wn) {
          const int k = i / C, c = i - k * C;
          if (c < H)
            dA[k * H + c] = X[k * Cs + c];
          else
            dHp[k * H + c - H] = X[k * Cs + c];
        }
      }
    }
    publish_barrier();
    const GPass pn = g_pass(pb ^ 1);
    const bool have = pn.nm > 0;
    if (have && threadIdx.x >= 64) stage(pn, threadIdx.x - 64, AMP_THREADS - 64);
    if (threadIdx.x < 64) {
      fence_release();
      const int m = threadIdx.x;
      if (!p.bwd) {
        // every tile of both gates done: the candidate can start
        if (m < p.nm && join_arrive(B.cnt + (int)p.msg(m)[2] * 8 + 1, B.Tz + B.Tr))
          ring_post(rg.gh, MSG_MAKE(0, p.msg(m)[2], p.msg(m)[3]));
      } else {
        // both gates done: back through sum / Group to the edge types
        int go = 0;
        if (m < p.nm) go = join_arrive(B.cnt + (int)p.msg(m)[2] * 8 + 2, B.Tz + B.Tr);
        for (int q = 0; q < p.nm; ++q)
          if (__shfl(go, q)) g_post_edges(rg, uni(p.msg(q)[8]), (int)uni(p.msg(q)[2]), (int)uni(p.msg(q)[3]), true);
      }
    }
    PHASE(3);
    if (p.bwd) g_count_and_update<NRBT, NCGT>(D, W, nd, t, g, pend, count, nrows, tstep, p.nm, p.Kt, gb);
    PHASE(7);
    if (!have && (threadIdx.x >> 6) == 1) g_form_pass(D, gd, B, mine, head, CAP, maxm, room(count), 0, false, true, pb ^ 1);
    lds_barrier();
    staged = have;
    pb ^= 1;
  }
  tile_store(nd, t, g.Wg, g.bg);
  if ((int)threadIdx.x < t.R) ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] = gb;
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
    W->wstate[4] = nrows;
  }
}

// ---------------------------------------------------------------- GRU candidate node + blend + loop control
template <int NRBT, int NCGT>
__device__ __noinline__ void role_g_cand(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const GData gd = g_data(D);
  const GRings rg = g_rings(D);
  const Pend pd = make_pend(W, t);
  GQ float* pend = (GQ float*)pd.base;
  const int H = B.H, C = 2 * H, CAP = uni(W->kb), Hs = amp_ldrow(H), Cs = amp_ldrow(C);
  const int u0 = t.u0, nu = t.nu, tile = uni(W->tile);   // this tile's output units = rows of W
  const bool vec = (H & 3) == 0 && (u0 & 3) == 0 && (nu & 3) == 0;   // rows can be moved 16 bytes at a time
  const int G1 = H >> 2, GU = nu >> 2;
  const int NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  const GTile g = g_tile_setup(L, nd, t);
  LDSQ float* X = (LDSQ float*)L.take(CAP * Cs);     // inputs of the stacked rows; later W^T delta
  LDSQ float* Y = (LDSQ float*)L.take(CAP * Hs);
  LDSQ float* gt = (LDSQ float*)L.take(CAP * H);     // gradient w.r.t. the states leaving the step
  for (int i = threadIdx.x; i < CAP * Cs; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < CAP * Hs; i += AMP_THREADS) Y[i] = 0.f;
  GQ float* ndG = (GQ float*)nd.G;
  float gb = (int)threadIdx.x < t.R ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  const int maxm = vec ? G_MB : 1;                    // the element-by-element paths take one message at a time
  const long long NH = (long long)B.N * H;
  const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
  // What a pass needs in LDS before its product: X = [A; r * h] and, on the way back, the delta rows (with the
  // gradient w.r.t. the step's output states, kept in gt, and the update gate's pre-activation gradient, written
  // to dZ).  `nthr` threads, `tid` = this thread's number among them.
  auto stage = [&](const GPass& p, int tid, int nthr) {
    if (vec) {
      const int GP = (Cs - C) >> 2;   // padding columns of the used rows of X
      for (int idx = tid; idx < p.Kt * GP; idx += nthr)
        *(LDSQ v4f*)(X + (idx / GP) * Cs + C + ((idx % GP) << 2)) = zero4;
      struct It {
        v4f a, rh;
      };
      for_items2(p.Kt * G1, tid, nthr,
                 [&](int idx) {
                   const int k = idx / G1, c = (idx - k * G1) << 2;
                   const LDSQ unsigned* M = p.of_row(k);
                   const int s = M[2], it = M[3], o = (k - (int)M[5]) * H + c;
                   const long long st = B.st(s, it);
                   It r;
                   r.a = *(const GQ v4f*)(B.A + st + o);
                   r.rh = *(const GQ v4f*)(B.Rr + st + o) * *(const GQ v4f*)(B.Hm + B.hm(s, it) + o);
                   return r;
                 },
                 [&](int idx, const It& r) {
                   const int k = idx / G1, c = (idx - k * G1) << 2;
                   *(LDSQ v4f*)(X + k * Cs + c) = r.a;
                   *(LDSQ v4f*)(X + k * Cs + H + c) = r.rh;
                 });
      if (!p.bwd) return;
      // backward through blend and tanh: the gradient w.r.t. the states leaving the step, for this tile's units
      // (from the readout after the last step, otherwise the sum of what the next step's backward pass left);
      // delta rows in tile order, zeros for the rest of each row
      const int GY = Hs >> 2, GZ = GY - GU;
      struct Ib {
        v4f z, ht, hv, gg;
      };
      for_items2(p.Kt * GU, tid, nthr,
                 [&](int idx) {
                   const int k = idx / GU, c = (idx - k * GU) << 2;
                   const LDSQ unsigned* M = p.of_row(k);
                   const int s = M[2], it = M[3], o = (k - (int)M[5]) * H + u0 + c;
                   const long long st = B.st(s, it);
                   Ib r;
                   r.z = *(const GQ v4f*)(B.Z + st + o);
                   r.ht = *(const GQ v4f*)(B.Ht + st + o);
                   r.hv = *(const GQ v4f*)(B.Hm + B.hm(s, it) + o);
                   if (it + 1 == B.S)
                     r.gg = *(const GQ v4f*)(B.gH + B.sl(s) + o);
                   else
                     r.gg = g_state_gradient4p(B, M[13], M[14], (int)M[15], s, o, it + 1);
                   return r;
                 },
                 [&](int idx, const Ib& r) {
                   const int k = idx / GU, c = (idx - k * GU) << 2;
                   const LDSQ unsigned* M = p.of_row(k);
                   const int s = M[2], o = (k - (int)M[5]) * H + u0 + c;
                   *(LDSQ v4f*)(gt + k * H + u0 + c) = r.gg;
                   *(GQ v4f*)(B.dZ + B.sl(s) + o) = r.gg * (r.ht - r.hv) * r.z * (1.f - r.z);
                   *(LDSQ v4f*)(Y + k * Hs + c) = r.gg * r.z * (1.f - r.ht * r.ht);
                 });
      for (int idx = tid; idx < p.Kt * GZ; idx += nthr)
        *(LDSQ v4f*)(Y + (idx / GZ) * Hs + nu + ((idx % GZ) << 2)) = zero4;
      return;
    }
    // element by element: one message
    const int s = (int)uni(p.msg(0)[2]), it = (int)uni(p.msg(0)[3]), K = p.Kt;
    const GQ float* A = B.A + B.st(s, it);
    const GQ float* h = B.Hm + B.hm(s, it);
    const GQ float* Z = B.Z + B.st(s, it);
    const GQ float* Rr = B.Rr + B.st(s, it);
    const GQ float* Ht = B.Ht + B.st(s, it);
    for (int i = tid; i < K * Cs; i += nthr) {
      const int k = i / Cs, c = i - k * Cs;
      X[i] = c < H ? A[k * H + c] : c < C ? Rr[k * H + c - H] * h[k * H + c - H] : 0.f;
    }
    if (!p.bwd) return;
    const GParts ep = g_edge_parts(B, uni(p.msg(0)[8]));
    const GQ float* gH = B.gH + B.sl(s);
    GQ float* dZ = B.dZ + B.sl(s);
    const bool from_readout = it + 1 == B.S;
    for (int i = tid; i < K * nu; i += nthr) {
      const int k = i / nu, j = i - k * nu, o = k * H + u0 + j;
      const float gg = from_readout ? gH[o] : g_state_gradient(B, ep, s, o, it + 1);
      const float z = Z[o], ht = Ht[o];
      gt[o] = gg;
      dZ[o] = gg * (ht - h[o]) * z * (1.f - z);
      Y[k * Hs + j] = gg * z * (1.f - ht * ht);
    }
    for (int i = tid; i < K * (Hs - nu); i += nthr) Y[(i / (Hs - nu)) * Hs + nu + i % (Hs - nu)] = 0.f;
  };
  auto room = [&](unsigned cnt) {
    const int muf = uni(nd.muf);
    return (int)cnt >= muf || muf < 1 ? (muf < 1 ? 1 : muf) : muf - (int)cnt;
  };
  // Wave 1 looks for the next pass while the present one's stores drain; if it is there, waves 1..7 stage it while
  // wave 0 publishes the present one (fence, joins, posts) -- the two do not touch the same memory -- otherwise
  // wave 1 waits for it afterwards.
  int pb = 0;
  bool staged = false;
  if ((threadIdx.x >> 6) == 1) g_form_pass(D, gd, B, mine, head, CAP, maxm, room(count), 0, false, true, pb);
  lds_barrier();
  for (;;) {
    const GPass p = g_pass(pb);
    if (p.stop) break;
    head += (unsigned)p.nm;
    PHASE(0);
    if (!staged) stage(p, threadIdx.x, AMP_THREADS);
    lds_barrier();
    const int NB = (p.Kt + 15) >> 4;
    const unsigned cnt_after = p.bwd ? count + (unsigned)p.nm : count;
    // wave 1 looks for the next pass while the other waves write this one's results out
    const bool scout = (threadIdx.x >> 6) == 1;
    const int wtid = threadIdx.x < 64 ? threadIdx.x : threadIdx.x - 64, wn = AMP_THREADS - 64;
    if (!p.bwd) {
      PHASE(1);
      mfma_rows<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, g.bl, X, Cs, NB, Y, Hs);
      PHASE(2);
      // this tile's units of the candidate and of the next state
      if (scout) {
        g_form_pass(D, gd, B, mine, head, CAP, maxm, room(cnt_after), 0, false, false, pb ^ 1);
      } else if (vec) {
        struct It {
          v4f z, hv;
        };
        for_items2(p.Kt * GU, wtid, wn,
                   [&](int idx) {
                     const int k = idx / GU, c = (idx - k * GU) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], o = (k - (int)M[5]) * H + u0 + c;
                     It r;
                     r.z = *(const GQ v4f*)(B.Z + B.st(s, it) + o);
                     r.hv = *(const GQ v4f*)(B.Hm + B.hm(s, it) + o);
                     return r;
                   },
                   [&](int idx, const It& r) {
                     const int k = idx / GU, c = (idx - k * GU) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], o = (k - (int)M[5]) * H + u0 + c;
                     const v4f ht = tanh4(*(const LDSQ v4f*)(Y + k * Hs + c));
                     *(GQ v4f*)(B.Ht + B.st(s, it) + o) = ht;
                     *(GQ v4f*)(B.Hm + B.hm(s, it + 1) + o) = (1.f - r.z) * r.hv + r.z * ht;
                   });
      } else {
        const int s = (int)uni(p.msg(0)[2]), it = (int)uni(p.msg(0)[3]);
        const GQ float* h = B.Hm + B.hm(s, it);
        const GQ float* Z = B.Z + B.st(s, it);
        GQ float* Ht = B.Ht + B.st(s, it);
        GQ float* hn = B.Hm + B.hm(s, it + 1);
        for (int i = wtid; i < p.Kt * nu; i += wn) {
          const int k = i / nu, j = i - k * nu, o = k * H + u0 + j;
          const float ht = tanhf(Y[k * Hs + j]), z = Z[o];
          Ht[o] = ht;
          hn[o] = (1.f - z) * h[o] + z * ht;
        }
      }
      for (int m = 0; m < p.nm; ++m) LOG(W->node, 0, p.msg(m)[1], p.msg(m)[3]);
    } else {
      // backward through blend, tanh (staged above), the candidate linear and r * h
      PHASE(4);
      for (int m = 0; m < p.nm; ++m) LOG(W->node, 1, p.msg(m)[1], p.msg(m)[3]);
      g_pend_append(pend, pd.Rp, pd.stride, nrows, Y, Hs, nu, X, Cs, C, p.Kt, gb);
      lds_barrier();
      PHASE(5);
      mfma_cols<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, Y, Hs, NB, X, Cs);
      PHASE(6);
      // This tile's parts, over all H columns: W^T delta w.r.t. A; the reset gate's pre-activation gradient, linear
      // in the tile's partial W^T delta w.r.t. r * h; the gradient w.r.t. h, to which the blend's direct term
      // gg (1 - z) belongs for the units this tile owns.
      if (scout) {
        g_form_pass(D, gd, B, mine, head, CAP, maxm, room(cnt_after), 0, false, false, pb ^ 1);
      } else if (vec) {
        struct It {
          v4f r, z, hv;
        };
        for_items2(p.Kt * G1, wtid, wn,
                   [&](int idx) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], o = (k - (int)M[5]) * H + c;
                     const long long st = B.st(s, it);
                     It r;
                     r.r = *(const GQ v4f*)(B.Rr + st + o);
                     r.z = *(const GQ v4f*)(B.Z + st + o);
                     r.hv = *(const GQ v4f*)(B.Hm + B.hm(s, it) + o);
                     return r;
                   },
                   [&](int idx, const It& r) {
                     const int k = idx / G1, c = (idx - k * G1) << 2;
                     const LDSQ unsigned* M = p.of_row(k);
                     const int s = M[2], it = M[3], o = (k - (int)M[5]) * H + c;
                     const bool own = c >= u0 && c < u0 + nu;
                     const v4f drh = *(const LDSQ v4f*)(X + k * Cs + H + c);
                     const v4f gg = own ? *(const LDSQ v4f*)(gt + k * H + c) : zero4;
                     *(GQ v4f*)(B.dA + ((long long)s * B.PA + tile) * NH + o) = *(const LDSQ v4f*)(X + k * Cs + c);
                     *(GQ v4f*)(B.dR + ((long long)s * B.Th + tile) * NH + o) = drh * r.hv * r.r * (1.f - r.r);
                     *(GQ v4f*)(B.dHp + (((long long)s * 2 + (it & 1)) * B.PA + tile) * NH + o) =
                         own ? drh * r.r + gg * (1.f - r.z) : drh * r.r;
                   });
      } else {
        const int s = (int)uni(p.msg(0)[2]), it = (int)uni(p.msg(0)[3]);
        const GQ float* h = B.Hm + B.hm(s, it);
        const GQ float* Z = B.Z + B.st(s, it);
        const GQ float* Rr = B.Rr + B.st(s, it);
        GQ float* dA = B.dA + ((long long)s * B.PA + tile) * NH;
        GQ float* dHp = B.dHp + (((long long)s * 2 + (it & 1)) * B.PA + tile) * NH;
        GQ float* dR = B.dR + ((long long)s * B.Th + tile) * NH;
        for (int i = wtid; i < p.Kt * H; i += wn) {
          const int k = i / H, j = i - k * H;
          const float drh = X[k * Cs + H + j], r = Rr[i], z = Z[i];
          dA[i] = X[k * Cs + j];
          dR[i] = drh * h[i] * r * (1.f - r);
          dHp[i] = (j >= u0 && j < u0 + nu) ? drh * r + gt[i] * (1.f - z) : drh * r;
        }
      }
    }
    publish_barrier();
    const GPass pn = g_pass(pb ^ 1);
    const bool have = pn.nm > 0;
    if (have && threadIdx.x >= 64) stage(pn, threadIdx.x - 64, AMP_THREADS - 64);
    if (threadIdx.x < 64) {
      fence_release();
      const int m = threadIdx.x;
      if (!p.bwd) {
        // the next state is complete when every tile has written its units
        int go = 0;
        if (m < p.nm) go = B.Th == 1 || join_arrive(B.cnt + (int)p.msg(m)[2] * 8 + 4, B.Th);
        for (int q = 0; q < p.nm; ++q) {
          if (!__shfl(go, q)) continue;
          const int s = (int)uni(p.msg(q)[2]), it = (int)uni(p.msg(q)[3]);
          if (it + 1 < B.S)
            g_post_edges(rg, uni(p.msg(q)[8]), s, it + 1, false);
          else if (m == 0)
            ring_post(rg.ro, MSG_MAKE(0, s, 0));
        }
      } else if (m < p.nm) {
        // every candidate tile's parts are there: on to the two gates
        const int s = p.msg(m)[2], it = p.msg(m)[3];
        if (B.Th == 1 || join_arrive(B.cnt + s * 8 + 5, B.Th)) {
          ring_post(rg.gz, MSG_MAKE(1, s, it));
          ring_post(rg.gr, MSG_MAKE(1, s, it));
        }
      }
    }
    PHASE(3);
    if (p.bwd) g_count_and_update<NRBT, NCGT>(D, W, nd, t, g, pend, count, nrows, tstep, p.nm, p.Kt, gb);
    PHASE(7);
    if (!have && (threadIdx.x >> 6) == 1) g_form_pass(D, gd, B, mine, head, CAP, maxm, room(count), 0, false, true, pb ^ 1);
    lds_barrier();
    staged = have;
    pb ^= 1;
  }
  tile_store(nd, t, g.Wg, g.bg);
  if ((int)threadIdx.x < t.R) ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] = gb;
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
    W->wstate[4] = nrows;
  }
}

// ---------------------------------------------------------------- readout: sum over nodes -> linear -> squared error
__device__ __noinline__ void role_g_readout(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const GData gd = g_data(D);
  const GRings rg = g_rings(D);
  const int H = B.H;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  float* pooled = L.take(H);
  float* red = L.take(AMP_THREADS);
  tile_load(nd, t, Wl, bl);
  GQ float* ndG = (GQ float*)nd.G;
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code);
    const unsigned seq = uni(gd.slot_seq[s]);
    const GView v = g_view(gd, s);
    const GQ float* h = B.Hm + B.hm(s, B.S);
    for (int j = threadIdx.x; j < H; j += AMP_THREADS) {
      float a = 0.f;
      for (int n = 0; n < v.N; ++n) a += h[n * H + j];
      pooled[j] = a;
    }
    __syncthreads();
    float p = 0.f;
    for (int j = threadIdx.x; j < H; j += AMP_THREADS) p += Wl[j] * pooled[j];
    red[threadIdx.x] = p;
    __syncthreads();
    for (int o = AMP_THREADS / 2; o; o >>= 1) {
      if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
      __syncthreads();
    }
    const float yhat = red[0] + bl[0];
    const float d = yhat - v.target;
    LOG(W->node, 0, seq, 0);
    if (threadIdx.x == 0) {
      ((GQ float*)D->loss_out)[seq - D->first_seq] = 0.5f * d * d;
      ((GQ float*)D->yhat_out)[seq - D->first_seq] = yhat;
    }
    if (!D->train || uni(gd.slot_inst[s]) < 0) {   // an evaluation instance: retired here, nothing turns round
      publish_barrier();
      if (threadIdx.x == 0) {
        fence_release();
        ring_post(rg.ctl, MSG_MAKE(1, s, 0));
      }
      continue;
    }
    LOG(W->node, 1, seq, 0);
    GQ float* gH = B.gH + B.sl(s);
    for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) gH[i] = d * Wl[i % H];
    for (int j = threadIdx.x; j < H; j += AMP_THREADS) ndG[j] += d * pooled[j];
    if (threadIdx.x == 0) ndG[H] += d;
    publish_barrier();
    if (threadIdx.x == 0) {
      fence_release();
      ring_post(rg.gh, MSG_MAKE(1, s, B.S - 1));
    }
    count_and_update(D, W, nd, t, Wl, bl, count, tstep);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}
