// Tree-LSTM workers (Section 5, Tree-LSTM paragraph): lookup, leaf cell,
// branch cell, output layer with a softmax loss at every tree node.
//
// Leaf and branch cells are split over several workgroups ("tiles", Section
// 5.1); the tiles of a cell read the same ring in the same order, so they act
// as one node with one event order.  Tile t owns hidden units [u0, u0+nu) of
// every gate, computes those units' h and c entirely, and contributes a
// partial W^T delta over all input columns on the way back.
//
// Slot storage (s = slot, n = tree node, l = leaf):
//   buf[0] xin  [s][l][D]        embedding recorded by the lookup's forward
//   buf[1] hc   [s][n][2H]       node output: h then c
//   buf[2] gate [s][n][6H]       gate activations and tanh(c) recorded at forward
//   buf[3] gout [s][n][H]        dh from the output layer
//   buf[4] gpar [s][n][TB][H]    dh partials from the parent's tiles
//   buf[5] gc   [s][n][H]        dc from the parent
//   buf[6] gx   [s][l][TL][D]    dx partials from the leaf tiles
//   buf[7] cnt  [s][n][4] (int)  arrival counters: tiles done / children done /
//                                gradient parts / leaf-tile dx parts
#pragma once

struct TreeView {
  int inst, L, NN, toff, noff, loff;
  const int *left, *right, *parent, *tok, *lab;
};

__device__ __forceinline__ TreeView tree_view(const AmpDev* D, unsigned seq) {
  TreeView v;
  v.inst = seq % D->data.n_inst;
  v.toff = D->data.tok_off[v.inst];
  v.L = D->data.tok_off[v.inst + 1] - v.toff;
  v.NN = 2 * v.L - 1;
  v.noff = D->data.node_off[v.inst];
  v.loff = D->data.lab_off[v.inst];
  v.left = D->data.left + v.noff;
  v.right = D->data.right + v.noff;
  v.parent = D->data.parent + v.noff;
  v.tok = D->data.tok + v.toff;
  v.lab = D->data.lab + v.loff;
  return v;
}

struct TreeBufs {
  float *xin, *hc, *gate, *gout, *gpar, *gc, *gx;
  int* cnt;
  int H, D, NNmax, Lmax, TL, TB;
  __device__ __forceinline__ long long node(int s, int n) const { return (long long)s * NNmax + n; }
  __device__ __forceinline__ long long leaf(int s, int l) const { return (long long)s * Lmax + l; }
};

__device__ __forceinline__ TreeBufs tree_bufs(const AmpDev* D) {
  TreeBufs b;
  b.xin = (float*)D->buf[0];
  b.hc = (float*)D->buf[1];
  b.gate = (float*)D->buf[2];
  b.gout = (float*)D->buf[3];
  b.gpar = (float*)D->buf[4];
  b.gc = (float*)D->buf[5];
  b.gx = (float*)D->buf[6];
  b.cnt = (int*)D->buf[7];
  b.H = D->hidden;
  b.D = D->emb;
  b.Lmax = D->max_len;
  b.NNmax = 2 * D->max_len - 1;
  b.TL = D->tiles_leaf;
  b.TB = D->tiles_branch;
  return b;
}

// Ring numbers of the tree model.
#define TR_LOOKUP 1
#define TR_LEAF 2
#define TR_BRANCH 3
#define TR_OUT 4

// A tile has finished its units of node n: when all tiles have, the node's
// [h; c] goes to the output layer and, through Isu / Concat, to its parent,
// which fires once both children are there.  ONE thread.
__device__ void tree_node_part_done(const AmpDev* D, const TreeBufs& B, const TreeView& v, int s, int n, int ntiles) {
  fence_release();
  int* c = B.cnt + B.node(s, n) * 4;
  if (!join_arrive(c + 0, ntiles)) return;
  ring_post(D->ring[TR_OUT], MSG_MAKE(0, s, n));
  const int pp = v.parent[n];
  if (pp < 0) return;
  const int p = pp >> 1;
  if (join_arrive(B.cnt + B.node(s, p) * 4 + 1, 2)) ring_post(D->ring[TR_BRANCH], MSG_MAKE(0, s, p));
}

// One gradient part for node n has been written: Bcast's backward waits for
// the output layer's part and (unless n is the root) every parent tile's.
__device__ void tree_grad_part_done(const AmpDev* D, const TreeBufs& B, const TreeView& v, int s, int n) {
  const int expect = v.parent[n] < 0 ? 1 : 1 + B.TB;
  if (join_arrive(B.cnt + B.node(s, n) * 4 + 2, expect))
    ring_post(D->ring[n < v.L ? TR_LEAF : TR_BRANCH], MSG_MAKE(1, s, n));
}

// ------------------------------------------------------------ lookup
__device__ void role_tree_lookup(const AmpDev* D, const WorkerDev* W, float* lds) {
  const NodeDev& lk = D->node[0];
  const TreeBufs B = tree_bufs(D);
  const int E = B.D;
  int* left_cnt = (int*)lds;                 // [mak] leaves not yet answered
  int* pend = left_cnt + ((D->mak + 3) & ~3); // tokens touched since the last update
  for (int i = threadIdx.x; i < D->mak; i += AMP_THREADS) left_cnt[i] = 0;
  __syncthreads();
  const RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  // tokens whose gradients were still waiting for an update when the previous call ended
  int* keep = (int*)D->buf[10];
  for (unsigned k = threadIdx.x; k < count; k += AMP_THREADS) pend[k] = keep[k];
  __syncthreads();
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code), l = MSG_LOCAL(code);
    const unsigned seq = D->slot_seq[s];
    const TreeView v = tree_view(D, seq);
    const int tok = v.tok[l];
    if (!(code & MSG_DIR_B)) {
      const float* row = lk.P + (long long)tok * E;
      float* x = B.xin + B.leaf(s, l) * E;
      for (int c = threadIdx.x; c < E; c += AMP_THREADS) x[c] = row[c];
      LOG(0, 0, seq, l);
      __syncthreads();
      if (threadIdx.x == 0) {
        if (l == 0) left_cnt[s] = v.L;
        fence_release();
        ring_post(D->ring[TR_LEAF], MSG_MAKE(0, s, l));
      }
      continue;
    }
    // backward: sum the leaf tiles' partials in tile order, add to the table's accumulator
    const float* gx = B.gx + B.leaf(s, l) * B.TL * E;
    float* g = lk.G + (long long)tok * E;
    for (int c = threadIdx.x; c < E; c += AMP_THREADS) {
      float a = 0.f;
      for (int t = 0; t < B.TL; ++t) a += gx[t * E + c];
      g[c] += a;
    }
    LOG(0, 1, seq, l);
    if (threadIdx.x == 0) pend[count] = tok;
    count++;
    __syncthreads();
    if (threadIdx.x == 0) {
      if (--left_cnt[s] == 0) {
        fence_release();
        ring_post(D->ring[0], MSG_MAKE(1, s, 0));
      }
    }
    if ((int)count >= lk.muf) {
      // SGD on the touched rows only: an untouched row has a zero gradient
      tstep++;
      const float sc = lk.lr * (lk.mean ? 1.f / (float)count : 1.f);
      for (unsigned k = 0; k < count; ++k) {
        float* row = lk.P + (long long)pend[k] * E;
        float* gr = lk.G + (long long)pend[k] * E;
        for (int c = threadIdx.x; c < E; c += AMP_THREADS) {
          row[c] -= sc * gr[c];
          gr[c] = 0.f;
        }
        __syncthreads();   // a token may occur twice: its row must be finished before it is seen again
      }
      count = 0;
      LOG(0, 2, 0, 0);
    }
  }
  // gradients still pending stay in G; remember their tokens for the next call
  __syncthreads();
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
  for (unsigned k = threadIdx.x; k < count; k += AMP_THREADS) keep[k] = pend[k];
}

// ------------------------------------------------------------ leaf / branch cells
// is_branch = false: rows [i; o; u] over the embedding.
// is_branch = true : rows [i; f_l; f_r; o; u] over [h_l; h_r].
template <bool BR>
__device__ void role_tree_cell(const AmpDev* D, const WorkerDev* W, float* lds) {
  const NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const int R = t.R, C = t.C, H = B.H, nu = t.nu, u0 = t.u0;
  constexpr int NG = BR ? 5 : 3;
  Lds L{lds};
  float* Wl = L.take(R * t.ldw);
  float* bl = L.take(R);
  float* xs = L.take(C);
  float* ys = L.take(R);
  float* ds = L.take(R);
  float* dx = L.take(C);
  float* part = L.take(8 * (R > C ? R : C));
  tile_load(nd, t, Wl, bl);
  const RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code), n = MSG_LOCAL(code);
    const unsigned seq = D->slot_seq[s];
    const TreeView v = tree_view(D, seq);
    const int a = BR ? v.left[n] : 0, b = BR ? v.right[n] : 0;
    const float* hca = B.hc + B.node(s, a) * 2 * H;
    const float* hcb = B.hc + B.node(s, b) * 2 * H;
    float* hcn = B.hc + B.node(s, n) * 2 * H;
    float* gt = B.gate + B.node(s, n) * 6 * H;
    // input columns: the embedding, or the children's hidden states
    if (BR) {
      for (int c = threadIdx.x; c < C; c += AMP_THREADS) xs[c] = c < H ? hca[c] : hcb[c - H];
    } else {
      const float* x = B.xin + B.leaf(s, n) * C;
      for (int c = threadIdx.x; c < C; c += AMP_THREADS) xs[c] = x[c];
    }
    __syncthreads();
    if (!(code & MSG_DIR_B)) {
      gemv_rows(Wl, t.ldw, R, C, bl, xs, part, ys);
      for (int j = threadIdx.x; j < nu; j += AMP_THREADS) {
        const int u = u0 + j;
        float c_, o_;
        if (BR) {
          const float i_ = sigmoidf_(ys[j]), fl = sigmoidf_(ys[nu + j]), fr = sigmoidf_(ys[2 * nu + j]);
          o_ = sigmoidf_(ys[3 * nu + j]);
          const float g_ = tanhf(ys[4 * nu + j]);
          c_ = i_ * g_ + fl * hca[H + u] + fr * hcb[H + u];
          gt[u] = i_;
          gt[H + u] = fl;
          gt[2 * H + u] = fr;
          gt[3 * H + u] = o_;
          gt[4 * H + u] = g_;
        } else {
          const float i_ = sigmoidf_(ys[j]);
          o_ = sigmoidf_(ys[nu + j]);
          const float g_ = tanhf(ys[2 * nu + j]);
          c_ = i_ * g_;
          gt[u] = i_;
          gt[3 * H + u] = o_;
          gt[4 * H + u] = g_;
        }
        const float tc = tanhf(c_);
        gt[5 * H + u] = tc;
        hcn[u] = o_ * tc;
        hcn[H + u] = c_;
      }
      LOG(W->node, 0, seq, n);
      __syncthreads();
      if (threadIdx.x == 0) tree_node_part_done(D, B, v, s, n, W->ntiles);
      continue;
    }
    // ---- backward
    const bool root = v.parent[n] < 0;
    const float* gout = B.gout + B.node(s, n) * H;
    const float* gpar = B.gpar + B.node(s, n) * B.TB * H;
    const float* gcn = B.gc + B.node(s, n) * H;
    for (int j = threadIdx.x; j < nu; j += AMP_THREADS) {
      const int u = u0 + j;
      float dh = gout[u], dc = 0.f;
      if (!root) {
        float p = 0.f;
        for (int k = 0; k < B.TB; ++k) p += gpar[k * H + u];
        dh += p;
        dc = gcn[u];
      }
      const float i_ = gt[u], o_ = gt[3 * H + u], g_ = gt[4 * H + u], tc = gt[5 * H + u];
      const float dct = dc + dh * o_ * (1.f - tc * tc);
      const float d_o = dh * tc * o_ * (1.f - o_);
      const float d_i = dct * g_ * i_ * (1.f - i_);
      const float d_g = dct * i_ * (1.f - g_ * g_);
      if (BR) {
        const float fl = gt[H + u], fr = gt[2 * H + u];
        ds[j] = d_i;
        ds[nu + j] = dct * hca[H + u] * fl * (1.f - fl);
        ds[2 * nu + j] = dct * hcb[H + u] * fr * (1.f - fr);
        ds[3 * nu + j] = d_o;
        ds[4 * nu + j] = d_g;
        B.gc[B.node(s, a) * H + u] = dct * fl;
        B.gc[B.node(s, b) * H + u] = dct * fr;
      } else {
        ds[j] = d_i;
        ds[nu + j] = d_o;
        ds[2 * nu + j] = d_g;
      }
    }
    __syncthreads();
    LOG(W->node, 1, seq, n);
    gemv_cols(Wl, t.ldw, R, C, ds, part, dx);
    if (BR) {
      float* pa = B.gpar + (B.node(s, a) * B.TB + W->tile) * H;
      float* pb = B.gpar + (B.node(s, b) * B.TB + W->tile) * H;
      for (int c = threadIdx.x; c < C; c += AMP_THREADS) {
        if (c < H)
          pa[c] = dx[c];
        else
          pb[c - H] = dx[c];
      }
    } else {
      float* px = B.gx + (B.leaf(s, n) * B.TL + W->tile) * C;
      for (int c = threadIdx.x; c < C; c += AMP_THREADS) px[c] = dx[c];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      if (BR) {
        tree_grad_part_done(D, B, v, s, a);
        tree_grad_part_done(D, B, v, s, b);
      } else {
        if (join_arrive(B.cnt + B.node(s, n) * 4 + 3, B.TL)) ring_post(D->ring[TR_LOOKUP], MSG_MAKE(1, s, n));
      }
    }
    tile_accumulate(nd, t, ds, xs);
    count_and_update(D, W, nd, t, Wl, bl, count, tstep);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
  (void)NG;
}

// ------------------------------------------------------------ output layer + loss at every node
__device__ void role_tree_out(const AmpDev* D, const WorkerDev* W, float* lds) {
  const NodeDev& nd = D->node[3];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const int R = t.R, C = t.C, H = B.H;
  Lds L{lds};
  float* Wl = L.take(R * t.ldw);
  float* bl = L.take(R);
  float* xs = L.take(C);
  float* ys = L.take(R);
  float* ds = L.take(R);
  float* dx = L.take(C);
  float* part = L.take(8 * (R > C ? R : C));
  int* done_cnt = (int*)L.take(D->mak);     // eval: nodes scored per slot
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < D->mak; i += AMP_THREADS) done_cnt[i] = 0;
  __syncthreads();
  const RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code), n = MSG_LOCAL(code);
    const unsigned seq = D->slot_seq[s];
    const TreeView v = tree_view(D, seq);
    const float* h = B.hc + B.node(s, n) * 2 * H;
    for (int c = threadIdx.x; c < C; c += AMP_THREADS) xs[c] = h[c];
    __syncthreads();
    gemv_rows(Wl, t.ldw, R, C, bl, xs, part, ys);
    LOG(3, 0, seq, n);
    const int label = v.lab[n];
    softmax_xent_wave0(ys, R, label, ds, &s_loss, &s_pred);
    if (threadIdx.x == 0) {
      D->loss_out[seq - D->first_seq] += s_loss;
      D->correct_out[seq - D->first_seq] += s_pred == label;
    }
    if (!D->train) {
      if (threadIdx.x == 0 && ++done_cnt[s] == v.NN) {
        done_cnt[s] = 0;
        fence_release();
        ring_post(D->ring[0], MSG_MAKE(1, s, 0));
      }
      continue;
    }
    LOG(3, 1, seq, n);
    gemv_cols(Wl, t.ldw, R, C, ds, part, dx);
    float* go = B.gout + B.node(s, n) * H;
    for (int c = threadIdx.x; c < C; c += AMP_THREADS) go[c] = dx[c];
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      tree_grad_part_done(D, B, v, s, n);
    }
    tile_accumulate(nd, t, ds, xs);
    count_and_update(D, W, nd, t, Wl, bl, count, tstep);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}
