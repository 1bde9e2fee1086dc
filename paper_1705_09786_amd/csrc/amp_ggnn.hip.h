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
  // filled by g_view_rec only: the admission number, the edge types present, and (edge workers) the number of edges
  // of the worker's type and where they start in tedge / tsk
  unsigned seq, present;
  int kc, tsc;
};

// The instance set's arrays, read once per worker into scalar registers.
struct GData {
  const GQ int *tok_off, *edge_off, *tok, *src, *dst, *tcount, *inoff, *inedge, *tstart, *tedge, *tsoff, *tsk;
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

// The instance facts of a message, decoded once by the thread that took the message from the ring and handed to the
// workgroup through LDS: the decode is a chain of two dependent fetches (slot -> instance -> offsets and counts),
// which this way runs beside the publication of the previous message instead of in front of every thread's work.
// Two records, alternating with the ring ticket: the next message's is written while the present one's is in use.
__shared__ unsigned s_grec[2][12];

// ONE thread.  ctype = the edge type whose count and start the record should carry (0 for the GRU workers).
__device__ __forceinline__ void g_decode(const GData& d, unsigned code, int ctype, int b) {
  const int s = MSG_SLOT(code);
  const unsigned seq = d.slot_seq[s];
  const int inst = d.slot_inst[s] & 0x7fffffff;
  const int to = d.tok_off[inst], to1 = d.tok_off[inst + 1], eo = d.edge_off[inst], eo1 = d.edge_off[inst + 1];
  const float tg = d.target[inst];
  const v4i c0 = *(const GQ v4i*)(d.tcount + inst * 8), c1 = *(const GQ v4i*)(d.tcount + inst * 8 + 4);
  const int tsc = d.tstart[inst * 9 + ctype];
  const int cnt[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
  unsigned present = 0;
  int kc = 0;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    present |= (c < d.T && cnt[c] > 0) ? 1u << c : 0u;
    kc = c == ctype ? cnt[c] : kc;
  }
  unsigned* r = s_grec[b];
  r[0] = seq;
  r[1] = (unsigned)inst;
  r[2] = (unsigned)to;
  r[3] = (unsigned)(to1 - to);
  r[4] = (unsigned)eo;
  r[5] = (unsigned)(eo1 - eo);
  r[6] = __float_as_uint(tg);
  r[7] = present;
  r[8] = (unsigned)kc;
  r[9] = (unsigned)tsc;
}

// All threads, after the barrier that follows g_decode.
__device__ __forceinline__ GView g_view_rec(const GData& d, int b) {
  const unsigned* r = s_grec[b];
  GView v;
  v.seq = uni(r[0]);
  v.inst = (int)uni(r[1]);
  const int to = (int)uni(r[2]), eo = (int)uni(r[4]);
  v.N = (int)uni(r[3]);
  v.E = (int)uni(r[5]);
  v.target = __uint_as_float(uni(r[6]));
  v.present = uni(r[7]);
  v.kc = (int)uni(r[8]);
  v.tsc = (int)uni(r[9]);
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
  if ((int)threadIdx.x < R)
    for (int k = 0; k < K; ++k) gb += Dl[k * ldd + threadIdx.x];
}

// Counts one gradient (a grouped message of K rows already appended to the
// pending list) and updates when min_update_frequency is reached.
template <int NRBT, int NCGT>
__device__ __forceinline__ void g_count_and_update(const GQ AmpDev* D, const GQ WorkerDev* W, const GQ NodeDev& nd, const Tile& t,
                                                   const GTile& g, const GQ float* pend, unsigned& count, unsigned& nrows,
                                                   unsigned& tstep, int K, float& gb) {
  count++;
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
  const int H = B.H, ctype = uni(W->aux), Ep = amp_round16(B.Em), Hs = amp_ldrow(H);
  const int u0 = t.u0, nu = t.nu, tile = uni(W->tile);   // this tile's output units = rows of W
  const bool vec = (H & 3) == 0 && (u0 & 3) == 0 && (nu & 3) == 0;   // rows can be moved 16 bytes at a time
  const int G1 = H >> 2, GU = nu >> 2;
  const int NRB = t.Rp >> 4, NCG = amp_round16(H) >> 4;
  Lds L{lds};
  const GTile g = g_tile_setup(L, nd, t);
  LDSQ float* X = (LDSQ float*)L.take(Ep * Hs);     // inputs h_src; later the products W^T delta
  LDSQ float* Y = (LDSQ float*)L.take(Ep * Hs);     // outputs / deltas
  for (int i = threadIdx.x; i < Ep * Hs; i += AMP_THREADS) X[i] = Y[i] = 0.f;
  GQ float* ndG = (GQ float*)nd.G;
  float gb = (int)threadIdx.x < t.R ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  // Thread 64 (wave 1) waits for the next message while wave 0 publishes the present one.
  if (threadIdx.x == 64) {
    poll_msg(D, mine, head, s_ctl);
    if (s_ctl[1] == 0u) g_decode(gd, s_ctl[0], ctype, head & 1);
  }
  lds_barrier();
  for (;;) {
    const unsigned code = uni(s_ctl[0]);
    if (uni(s_ctl[1]) != 0u) break;
    const GView v = g_view_rec(gd, head & 1);
    head++;
    const int s = MSG_SLOT(code), it = MSG_LOCAL(code);
    const unsigned seq = v.seq;
    const int K = v.kc, NB = (K + 15) >> 4;
    const GQ int* te = v.tedge + v.tsc;   // edges of this type, ascending (Group orders its rows by edge index)
    const GQ float* h = B.Hm + B.hm(s, it);
    const int nact = g_present_tiles(B, v.present);   // tiles of every edge type the graph uses
    if (vec) {
      const int GY = Hs >> 2;   // padding columns of a used row are written as zeros every time
      for (int idx = threadIdx.x; idx < K * GY; idx += AMP_THREADS) {
        const int k = idx / GY, c = (idx - k * GY) << 2;
        const bool in = c < H;
        const v4f x = *(const GQ v4f*)(h + (long long)v.src[te[k]] * H + (in ? c : 0));
        *(LDSQ v4f*)(X + k * Hs + c) = in ? x : (v4f){0.f, 0.f, 0.f, 0.f};
      }
    } else
    for (int i = threadIdx.x; i < K * Hs; i += AMP_THREADS) {
      const int k = i / Hs, j = i - k * Hs;
      X[i] = j < H ? h[v.src[te[k]] * H + j] : 0.f;   // padding columns of a used row are zero
    }
    if (!(code & MSG_DIR_B)) {
      lds_barrier();
      mfma_rows<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, g.bl, X, Hs, NB, Y, Hs);
      GQ float* msg = B.Msg + (long long)s * B.Em * H + u0;   // this tile's units of every message
      if (vec) {
        for (int idx = threadIdx.x; idx < K * GU; idx += AMP_THREADS) {
          const int k = idx / GU, c = (idx - k * GU) << 2;
          *(GQ v4f*)(msg + (long long)te[k] * H + c) = *(const LDSQ v4f*)(Y + k * Hs + c);
        }
      } else
      for (int i = threadIdx.x; i < K * nu; i += AMP_THREADS) {
        const int k = i / nu, j = i - k * nu;
        msg[te[k] * H + j] = Y[k * Hs + j];
      }
      LOG(W->node, 0, seq, it);
      publish_barrier();
      if (threadIdx.x == 0) {
        fence_release();
        // the last type to arrive completes the step's messages; Ungroup, regrouping by target node and the sum are the GRU nodes' part
        if (join_arrive(B.cnt + s * 8 + 0, nact)) {
          ring_post(rg.gz, MSG_MAKE(0, s, it));
          ring_post(rg.gr, MSG_MAKE(0, s, it));
        }
      }
    } else {
    // ---- backward: delta_e = this tile's units of dA[dst(e)] (Bcast backward on A: (update + reset) + candidate,
    // each the sum of its tiles' parts); one gradient for the group
    {
      const long long NH = (long long)B.N * H;
      const GQ float* dA = B.dA + (long long)s * B.PA * NH + u0;
      if (vec) {
        // the tile's units first (one group per thread and round trip), then zeros for the rest of each row
        const int GY = Hs >> 2, GZ = GY - GU;
        for (int idx = threadIdx.x; idx < K * GU; idx += AMP_THREADS) {
          const int k = idx / GU, c = (idx - k * GU) << 2;
          *(LDSQ v4f*)(Y + k * Hs + c) = g_sum_dA4(B, dA, (long long)v.dst[te[k]] * H + c);
        }
        for (int idx = threadIdx.x; idx < K * GZ; idx += AMP_THREADS)
          *(LDSQ v4f*)(Y + (idx / GZ) * Hs + nu + ((idx % GZ) << 2)) = (v4f){0.f, 0.f, 0.f, 0.f};
      } else
      for (int i = threadIdx.x; i < K * Hs; i += AMP_THREADS) {
        const int k = i / Hs, j = i - k * Hs;
        Y[i] = j < nu ? g_sum_dA(B, dA, (long long)v.dst[te[k]] * H + j) : 0.f;
      }
    }
    lds_barrier();
    LOG(W->node, 1, seq, it);
    g_pend_append(pend, pd.Rp, pd.stride, nrows, Y, Hs, nu, X, Hs, H, K, gb);
    lds_barrier();
    mfma_cols<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, Y, Hs, NB, X, Hs);
    // dh_src += W^T delta_e: per source node, its edges of this type in ascending order
    {
      GQ float* dHe = B.dHe + ((long long)s * B.PE + B.eoff(ctype) + tile) * B.N * H;   // this tile's part
      const GQ int* so = v.tsoff + ctype * (v.N + 1);
      const GQ int* sk = v.tsk + v.tsc;
      if (vec) {
        for (int idx = threadIdx.x; idx < v.N * G1; idx += AMP_THREADS) {
          const int n = idx / G1, c = (idx - n * G1) << 2;
          const int p0 = so[n], p1 = so[n + 1];
          v4f a = {0.f, 0.f, 0.f, 0.f};
          for (int p = p0; p < p1; p += 4) {
            int kk[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) kk[u] = sk[p + u < p1 ? p + u : p1 - 1];
#pragma unroll
            for (int u = 0; u < 4; ++u)
              if (p + u < p1) a += *(const LDSQ v4f*)(X + kk[u] * Hs + c);
          }
          *(GQ v4f*)(dHe + n * H + c) = a;
        }
      } else
      for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) {
        const int n = i / H, j = i - n * H;
        float a = 0.f;
        for (int p = so[n]; p < so[n + 1]; ++p) a += X[sk[p] * Hs + j];
        dHe[i] = a;
      }
    }
    publish_barrier();
    if (threadIdx.x == 0) {
      fence_release();
      if (join_arrive(B.cnt + s * 8 + 3, nact)) {
        if (it > 0)
          ring_post(rg.gh, MSG_MAKE(1, s, it - 1));
        else
          ring_post(rg.lookup, MSG_MAKE(1, s, 0));
      }
    }
    g_count_and_update<NRBT, NCGT>(D, W, nd, t, g, pend, count, nrows, tstep, K, gb);
    }
    if (threadIdx.x == 64) {
      poll_msg(D, mine, head, s_ctl);
      if (s_ctl[1] == 0u) g_decode(gd, s_ctl[0], ctype, head & 1);
    }
    lds_barrier();
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
  const int H = B.H, C = 2 * H, Np = amp_round16(B.N), which = uni(W->aux), Hs = amp_ldrow(H), Cs = amp_ldrow(C);
  const int u0 = t.u0, nu = t.nu, tile = uni(W->tile);   // this tile's output units = rows of W
  const bool vec = (H & 3) == 0 && (u0 & 3) == 0 && (nu & 3) == 0;   // rows can be moved 16 bytes at a time
  const int G1 = H >> 2, GU = nu >> 2;
  const int part = B.Th + (which ? B.Tz : 0) + tile;     // this tile's part of dA / dHp
  const int NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  const GTile g = g_tile_setup(L, nd, t);
  LDSQ float* X = (LDSQ float*)L.take(Np * Cs);     // inputs; later W^T delta
  LDSQ float* Y = (LDSQ float*)L.take(Np * Hs);
  for (int i = threadIdx.x; i < Np * Cs; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < Np * Hs; i += AMP_THREADS) Y[i] = 0.f;
  GQ float* ndG = (GQ float*)nd.G;
  float gb = (int)threadIdx.x < t.R ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  // Thread 64 (wave 1) waits for the next message while wave 0 publishes the present one.
  if (threadIdx.x == 64) {
    poll_msg(D, mine, head, s_ctl);
    if (s_ctl[1] == 0u) g_decode(gd, s_ctl[0], 0, head & 1);
  }
  lds_barrier();
  for (;;) {
    const unsigned code = uni(s_ctl[0]);
    if (uni(s_ctl[1]) != 0u) break;
    const GView v = g_view_rec(gd, head & 1);
    head++;
    const int s = MSG_SLOT(code), it = MSG_LOCAL(code);
    const unsigned seq = v.seq;
    const int K = v.N, NB = (K + 15) >> 4;
    GQ float* A = B.A + B.st(s, it);
    const GQ float* h = B.Hm + B.hm(s, it);
    GQ float* outp = (which == 0 ? B.Z : B.Rr) + B.st(s, it) + u0;   // this tile's units of every row
    const bool rec_a = which == 0 && tile == 0;   // the update gate's first tile records the aggregated messages
    PHASE(0);
    if (!(code & MSG_DIR_B)) {
      // Ungroup, regroup by target node, sum: a_v = sum over incoming edges in edge order
      const GQ float* msg = B.Msg + (long long)s * B.Em * H;
      if (vec) {
        // 16 bytes per thread and step; the padding columns of a used row are written as zeros every time (an
        // unused row may hold anything, and the products leave 0 x anything in its padding)
        // one thread per (node, 4 units): its part of h travels while the chain inoff -> inedge -> message rows runs,
        // so a graph of up to 20 nodes takes one pass
        for (int idx = threadIdx.x; idx < K * G1; idx += AMP_THREADS) {
          const int k = idx / G1, c = (idx - k * G1) << 2;
          const v4f hv = *(const GQ v4f*)(h + k * H + c);
          const v4f x = g_sum_incoming4(msg, v, k, c, H);
          if (rec_a) *(GQ v4f*)(A + k * H + c) = x;
          *(LDSQ v4f*)(X + k * Cs + c) = x;
          *(LDSQ v4f*)(X + k * Cs + H + c) = hv;
        }
        const int GP = (Cs - C) >> 2;
        for (int idx = threadIdx.x; idx < K * GP; idx += AMP_THREADS)
          *(LDSQ v4f*)(X + (idx / GP) * Cs + C + ((idx % GP) << 2)) = (v4f){0.f, 0.f, 0.f, 0.f};
      } else
      for (int i = threadIdx.x; i < K * Cs; i += AMP_THREADS) {
        const int k = i / Cs, c = i - k * Cs;
        float x = 0.f;   // padding columns of a used row are zero
        if (c < H) {
          for (int p = v.inoff[k]; p < v.inoff[k + 1]; ++p) x += msg[v.inedge[p] * H + c];
          if (rec_a) A[k * H + c] = x;   // the recorded activation, read again by all three GRU nodes
        } else if (c < C) {
          x = h[k * H + c - H];
        }
        X[i] = x;
      }
      lds_barrier();
      PHASE(1);
      mfma_rows<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, g.bl, X, Cs, NB, Y, Hs);
      PHASE(2);
      if (vec) {
        for (int idx = threadIdx.x; idx < K * GU; idx += AMP_THREADS) {
          const int k = idx / GU, c = (idx - k * GU) << 2;
          *(GQ v4f*)(outp + k * H + c) = sigmoid4(*(const LDSQ v4f*)(Y + k * Hs + c));
        }
      } else
      for (int i = threadIdx.x; i < K * nu; i += AMP_THREADS) outp[(i / nu) * H + i % nu] = sigmoidf_(Y[(i / nu) * Hs + i % nu]);
      LOG(W->node, 0, seq, it);
      publish_barrier();
      if (threadIdx.x == 0) {
        fence_release();
        // every tile of both gates done: the candidate can start
        if (join_arrive(B.cnt + s * 8 + 1, B.Tz + B.Tr)) ring_post(rg.gh, MSG_MAKE(0, s, it));
      }
      PHASE(3);
    } else {
    // this tile's units of the pre-activation gradient: the update gate's was written by the candidate tile that
    // owns each unit; the reset gate's is the sum of the candidate tiles' parts (each a full-width W^T delta)
    const GQ float* dpre = (which == 0 ? B.dZ + B.sl(s) : B.dR + B.sl(s) * B.Th) + u0;
    const int ndp = which == 0 ? 1 : B.Th;
    const long long NHp = (long long)B.N * H;
    if (vec) {
      // the H real columns of every row in one pass (one group per thread and round trip for graphs of up to 20
      // nodes), the delta's zero padding afterwards
      const int GY = Hs >> 2, GZ = GY - G1;
      for (int idx = threadIdx.x; idx < K * G1; idx += AMP_THREADS) {
        const int k = idx / G1, c = (idx - k * G1) << 2;
        const bool ind = c < nu;
        const int o = k * H + c, od = k * H + (ind ? c : 0);
        const v4f a = *(const GQ v4f*)(A + o), hv = *(const GQ v4f*)(h + o);
        v4f dq[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) dq[p] = *(const GQ v4f*)(dpre + (p < ndp ? p : 0) * NHp + od);
        v4f dp = dq[0];
#pragma unroll
        for (int p = 1; p < 4; ++p)
          if (p < ndp) dp += dq[p];
        *(LDSQ v4f*)(X + k * Cs + c) = a;
        *(LDSQ v4f*)(X + k * Cs + H + c) = hv;
        *(LDSQ v4f*)(Y + k * Hs + c) = ind ? dp : (v4f){0.f, 0.f, 0.f, 0.f};
      }
      for (int idx = threadIdx.x; idx < K * GZ; idx += AMP_THREADS)
        *(LDSQ v4f*)(Y + (idx / GZ) * Hs + H + ((idx % GZ) << 2)) = (v4f){0.f, 0.f, 0.f, 0.f};
      const int GP = (Cs - C) >> 2;   // padding columns of the used rows of X
      for (int idx = threadIdx.x; idx < K * GP; idx += AMP_THREADS)
        *(LDSQ v4f*)(X + (idx / GP) * Cs + C + ((idx % GP) << 2)) = (v4f){0.f, 0.f, 0.f, 0.f};
    } else {
      for (int i = threadIdx.x; i < K * Cs; i += AMP_THREADS) {
        const int k = i / Cs, c = i - k * Cs;
        X[i] = c < H ? A[k * H + c] : c < C ? h[k * H + c - H] : 0.f;
      }
      for (int i = threadIdx.x; i < K * Hs; i += AMP_THREADS) {
        const int k = i / Hs, j = i - k * Hs;
        float d = 0.f;
        if (j < nu)
          for (int p = 0; p < ndp; ++p) d += dpre[p * NHp + k * H + j];
        Y[i] = d;
      }
    }
    lds_barrier();
    PHASE(4);
    LOG(W->node, 1, seq, it);
    g_pend_append(pend, pd.Rp, pd.stride, nrows, Y, Hs, nu, X, Cs, C, K, gb);
    lds_barrier();
    PHASE(5);
    mfma_cols<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, Y, Hs, NB, X, Cs);
    PHASE(6);
    GQ float* dA = B.dA + ((long long)s * B.PA + part) * B.N * H;
    GQ float* dHp = B.dHp + (((long long)s * 2 + (it & 1)) * B.PA + part) * B.N * H;
    if (vec) {
      for (int idx = threadIdx.x; idx < K * G1; idx += AMP_THREADS) {
        const int k = idx / G1, c = (idx - k * G1) << 2;
        *(GQ v4f*)(dA + k * H + c) = *(const LDSQ v4f*)(X + k * Cs + c);
        *(GQ v4f*)(dHp + k * H + c) = *(const LDSQ v4f*)(X + k * Cs + H + c);
      }
    } else
    for (int i = threadIdx.x; i < K * C; i += AMP_THREADS) {
      const int k = i / C, c = i - k * C;
      if (c < H)
        dA[k * H + c] = X[k * Cs + c];
      else
        dHp[k * H + c - H] = X[k * Cs + c];
    }
    publish_barrier();
    if (threadIdx.x < 64) {
      fence_release();
      // both gates done: back through sum / Group to the edge types
      int go = 0;
      if (threadIdx.x == 0) go = join_arrive(B.cnt + s * 8 + 2, B.Tz + B.Tr);
      if (__shfl(go, 0)) g_post_edges(rg, v.present, s, it, true);
    }
    g_count_and_update<NRBT, NCGT>(D, W, nd, t, g, pend, count, nrows, tstep, K, gb);
    PHASE(7);
    }
    if (threadIdx.x == 64) {
      poll_msg(D, mine, head, s_ctl);
      if (s_ctl[1] == 0u) g_decode(gd, s_ctl[0], 0, head & 1);
    }
    lds_barrier();
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
  const int H = B.H, C = 2 * H, Np = amp_round16(B.N), Hs = amp_ldrow(H), Cs = amp_ldrow(C);
  const int u0 = t.u0, nu = t.nu, tile = uni(W->tile);   // this tile's output units = rows of W
  const bool vec = (H & 3) == 0 && (u0 & 3) == 0 && (nu & 3) == 0;   // rows can be moved 16 bytes at a time
  const int G1 = H >> 2, GU = nu >> 2;
  const int NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  const GTile g = g_tile_setup(L, nd, t);
  LDSQ float* X = (LDSQ float*)L.take(Np * Cs);     // inputs; later W^T delta
  LDSQ float* Y = (LDSQ float*)L.take(Np * Hs);
  LDSQ float* gt = (LDSQ float*)L.take(B.N * H);    // gradient w.r.t. the states leaving the step
  for (int i = threadIdx.x; i < Np * Cs; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < Np * Hs; i += AMP_THREADS) Y[i] = 0.f;
  GQ float* ndG = (GQ float*)nd.G;
  float gb = (int)threadIdx.x < t.R ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  // What a message needs in LDS before its product: X = [A; r * h] and, on the way back, the delta rows (with the
  // gradient w.r.t. the step's output states, kept in gt, and the update gate's pre-activation gradient, written
  // to dZ).  `nthr` threads, `tid` = this thread's number among them: the whole workgroup stages the message it is
  // about to process; waves 1..7 alone stage the next one, if it is already waiting, while wave 0 publishes the
  // present one (fence, join, posts) -- the two do not touch the same memory.
  auto stage = [&](unsigned mcode, int rec, int tid, int nthr) {
    const int s = MSG_SLOT(mcode), it = MSG_LOCAL(mcode);
    const GView v = g_view_rec(gd, rec);
    const int K = v.N;
    const GQ float* A = B.A + B.st(s, it);
    const GQ float* h = B.Hm + B.hm(s, it);
    const GQ float* Z = B.Z + B.st(s, it);
    const GQ float* Rr = B.Rr + B.st(s, it);
    const GQ float* Ht = B.Ht + B.st(s, it);
    if (vec) {
      for (int idx = tid; idx < K * G1; idx += nthr) {
        const int k = idx / G1, c = (idx - k * G1) << 2, o = k * H + c;
        const v4f a = *(const GQ v4f*)(A + o), r = *(const GQ v4f*)(Rr + o), hv = *(const GQ v4f*)(h + o);
        *(LDSQ v4f*)(X + k * Cs + c) = a;
        *(LDSQ v4f*)(X + k * Cs + H + c) = r * hv;
      }
      const int GP = (Cs - C) >> 2;   // padding columns of the used rows of X
      for (int idx = tid; idx < K * GP; idx += nthr)
        *(LDSQ v4f*)(X + (idx / GP) * Cs + C + ((idx % GP) << 2)) = (v4f){0.f, 0.f, 0.f, 0.f};
    } else
    for (int i = tid; i < K * Cs; i += nthr) {
      const int k = i / Cs, c = i - k * Cs;
      X[i] = c < H ? A[k * H + c] : c < C ? Rr[k * H + c - H] * h[k * H + c - H] : 0.f;
    }
    if (!(mcode & MSG_DIR_B)) return;
    // backward through blend and tanh: the gradient w.r.t. the states leaving the step, for this tile's units;
    // delta rows in tile order
    const unsigned present = v.present;
    const GQ float* gH = B.gH + B.sl(s);
    GQ float* dZ = B.dZ + B.sl(s);
    const bool from_readout = it + 1 == B.S;
    const GParts ep = g_edge_parts(B, present);
    if (vec) {
      // the tile's units first (one group per thread and round trip), then zeros for the rest of each row
      const int GY = Hs >> 2, GZ = GY - GU;
      for (int idx = tid; idx < K * GU; idx += nthr) {
        const int k = idx / GU, c = (idx - k * GU) << 2;
        const int o = k * H + u0 + c;
        const v4f z = *(const GQ v4f*)(Z + o), ht = *(const GQ v4f*)(Ht + o), hv = *(const GQ v4f*)(h + o);
        const v4f gg = from_readout ? *(const GQ v4f*)(gH + o) : g_state_gradient4(B, ep, s, o, it + 1);
        *(LDSQ v4f*)(gt + o) = gg;
        *(GQ v4f*)(dZ + o) = gg * (ht - hv) * z * (1.f - z);
        *(LDSQ v4f*)(Y + k * Hs + c) = gg * z * (1.f - ht * ht);
      }
      for (int idx = tid; idx < K * GZ; idx += nthr)
        *(LDSQ v4f*)(Y + (idx / GZ) * Hs + nu + ((idx % GZ) << 2)) = (v4f){0.f, 0.f, 0.f, 0.f};
    } else {
      for (int i = tid; i < K * nu; i += nthr) {
        const int k = i / nu, j = i - k * nu, o = k * H + u0 + j;
        const float gg = from_readout ? gH[o] : g_state_gradient(B, ep, s, o, it + 1);
        const float z = Z[o], ht = Ht[o];
        gt[o] = gg;
        dZ[o] = gg * (ht - h[o]) * z * (1.f - z);
        Y[k * Hs + j] = gg * z * (1.f - ht * ht);
      }
      for (int i = tid; i < K * (Hs - nu); i += nthr) Y[(i / (Hs - nu)) * Hs + nu + i % (Hs - nu)] = 0.f;
    }
  };
  // Thread 64 (wave 1) looks for the next message while the present one's stores drain; if it is there, waves 1..7
  // stage it while wave 0 publishes the present one, otherwise thread 64 waits for it afterwards.
  bool staged = false;
  if (threadIdx.x == 64) {
    poll_msg(D, mine, head, s_ctl);
    if (s_ctl[1] == 0u) g_decode(gd, s_ctl[0], 0, head & 1);
  }
  lds_barrier();
  for (;;) {
    const unsigned code = uni(s_ctl[0]);
    if (uni(s_ctl[1]) != 0u) break;
    const int rec = head & 1;
    const GView v = g_view_rec(gd, rec);
    head++;
    const int s = MSG_SLOT(code), it = MSG_LOCAL(code);
    const unsigned seq = v.seq;
    const unsigned present = v.present;
    const int K = v.N, NB = (K + 15) >> 4;
    const GQ float* h = B.Hm + B.hm(s, it);
    const GQ float* Z = B.Z + B.st(s, it);
    const GQ float* Rr = B.Rr + B.st(s, it);
    GQ float* Ht = B.Ht + B.st(s, it);
    PHASE(0);
    if (!staged) stage(code, rec, threadIdx.x, AMP_THREADS);
    bool have = false;
    unsigned ncode = 0;
    if (!(code & MSG_DIR_B)) {
      lds_barrier();
      PHASE(1);
      mfma_rows<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, g.bl, X, Cs, NB, Y, Hs);
      PHASE(2);
      GQ float* hn = B.Hm + B.hm(s, it + 1);
      // this tile's units of the candidate and of the next state
      if (vec) {
        for (int idx = threadIdx.x; idx < K * GU; idx += AMP_THREADS) {
          const int k = idx / GU, c = (idx - k * GU) << 2, o = k * H + u0 + c;
          const v4f z = *(const GQ v4f*)(Z + o), hv = *(const GQ v4f*)(h + o);
          const v4f ht = tanh4(*(const LDSQ v4f*)(Y + k * Hs + c));
          *(GQ v4f*)(Ht + o) = ht;
          *(GQ v4f*)(hn + o) = (1.f - z) * hv + z * ht;
        }
      } else
      for (int i = threadIdx.x; i < K * nu; i += AMP_THREADS) {
        const int k = i / nu, j = i - k * nu, o = k * H + u0 + j;
        const float ht = tanhf(Y[k * Hs + j]), z = Z[o];
        Ht[o] = ht;
        hn[o] = (1.f - z) * h[o] + z * ht;
      }
      LOG(W->node, 0, seq, it);
      if (threadIdx.x == 64) {
        peek_msg(mine, head, s_ctl);
        if (s_ctl[2] != 0u) g_decode(gd, s_ctl[0], 0, head & 1);
      }
      publish_barrier();
      have = uni(s_ctl[2]) != 0u;
      ncode = uni(s_ctl[0]);
      if (have && threadIdx.x >= 64) stage(ncode, head & 1, threadIdx.x - 64, AMP_THREADS - 64);
      if (threadIdx.x < 64) {
        fence_release();
        // the next state is complete when every tile has written its units
        int go = B.Th == 1;
        if (threadIdx.x == 0 && !go) go = join_arrive(B.cnt + s * 8 + 4, B.Th);
        if (__shfl(go, 0)) {
          if (it + 1 < B.S)
            g_post_edges(rg, present, s, it + 1, false);
          else if (threadIdx.x == 0)
            ring_post(rg.ro, MSG_MAKE(0, s, 0));
        }
      }
      PHASE(3);
    } else {
    // backward through blend, tanh (staged above), the candidate linear and r*h
    lds_barrier();
    PHASE(4);
    LOG(W->node, 1, seq, it);
    g_pend_append(pend, pd.Rp, pd.stride, nrows, Y, Hs, nu, X, Cs, C, K, gb);
    lds_barrier();
    PHASE(5);
    mfma_cols<NRBT, NCGT>(g.Wl, t.ldw, NRB, NCG, Y, Hs, NB, X, Cs);
    PHASE(6);
    {
      // This tile's parts, over all H columns: W^T delta w.r.t. A; the reset gate's pre-activation gradient, linear
      // in the tile's partial W^T delta w.r.t. r * h; the gradient w.r.t. h, to which the blend's direct term
      // gg (1 - z) belongs for the units this tile owns.
      GQ float* dA = B.dA + ((long long)s * B.PA + tile) * B.N * H;
      GQ float* dHp = B.dHp + (((long long)s * 2 + (it & 1)) * B.PA + tile) * B.N * H;
      GQ float* dR = B.dR + ((long long)s * B.Th + tile) * B.N * H;
      if (vec) {
        for (int idx = threadIdx.x; idx < K * G1; idx += AMP_THREADS) {
          const int k = idx / G1, c = (idx - k * G1) << 2, o = k * H + c;
          const bool own = c >= u0 && c < u0 + nu;
          const v4f r = *(const GQ v4f*)(Rr + o), z = *(const GQ v4f*)(Z + o), hv = *(const GQ v4f*)(h + o);
          const v4f drh = *(const LDSQ v4f*)(X + k * Cs + H + c);
          const v4f gg = own ? *(const LDSQ v4f*)(gt + o) : (v4f){0.f, 0.f, 0.f, 0.f};
          *(GQ v4f*)(dA + o) = *(const LDSQ v4f*)(X + k * Cs + c);
          *(GQ v4f*)(dR + o) = drh * hv * r * (1.f - r);
          *(GQ v4f*)(dHp + o) = own ? drh * r + gg * (1.f - z) : drh * r;
        }
      } else
      for (int i = threadIdx.x; i < K * H; i += AMP_THREADS) {
        const int k = i / H, j = i - k * H;
        const float drh = X[k * Cs + H + j], r = Rr[i], z = Z[i];
        dA[i] = X[k * Cs + j];
        dR[i] = drh * h[i] * r * (1.f - r);
        dHp[i] = (j >= u0 && j < u0 + nu) ? drh * r + gt[i] * (1.f - z) : drh * r;
      }
    }
    if (threadIdx.x == 64) {
        peek_msg(mine, head, s_ctl);
        if (s_ctl[2] != 0u) g_decode(gd, s_ctl[0], 0, head & 1);
      }
    publish_barrier();
    have = uni(s_ctl[2]) != 0u;
    ncode = uni(s_ctl[0]);
    if (have && threadIdx.x >= 64) stage(ncode, head & 1, threadIdx.x - 64, AMP_THREADS - 64);
    if (threadIdx.x == 0) {
      fence_release();
      // every candidate tile's parts are there: on to the two gates
      if (B.Th == 1 || join_arrive(B.cnt + s * 8 + 5, B.Th)) {
        ring_post(rg.gz, MSG_MAKE(1, s, it));
        ring_post(rg.gr, MSG_MAKE(1, s, it));
      }
    }
    PHASE(7);
    g_count_and_update<NRBT, NCGT>(D, W, nd, t, g, pend, count, nrows, tstep, K, gb);
    }
    if (!have && threadIdx.x == 64) {
      poll_msg(D, mine, head, s_ctl);
      if (s_ctl[1] == 0u) g_decode(gd, s_ctl[0], 0, head & 1);
    }
    lds_barrier();
    staged = have;
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
