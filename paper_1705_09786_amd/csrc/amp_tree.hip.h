// Tree-LSTM workers (Section 5, Tree-LSTM paragraph): lookup, leaf cell,
// branch cell, output layer with a softmax loss at every tree node.
//
// Leaf and branch cells are split over several workgroups ("tiles", Section
// 5.1); the tiles of a cell read the same ring in the same order and cut
// their batches at the same places, so they act as one node with one event
// order.  Tile t owns hidden units [u0, u0+nu) of every gate, computes those
// units' h and c entirely, and contributes a partial W^T delta over all
// input columns on the way back.
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
//   buf[10] lookup: tokens of the gradients waiting for the next update
//   buf[11] lookup: their gradient rows [AMP_TREE_LOOKUP_MAX_MUF][D]
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

__device__ __forceinline__ bool code_is_b(unsigned c) { return (c & MSG_DIR_B) != 0; }

// A tile has finished its units of node n: when all tiles have, the node's
// [h; c] goes to the output layer and, through Isu / Concat, to its parent,
// which fires once both children are there.  One lane, after a release fence.
__device__ __forceinline__ void tree_node_part_done(const AmpDev* D, const TreeBufs& B, int s, int n, int parent_code, int ntiles) {
  int* c = B.cnt + B.node(s, n) * 4;
  if (!join_arrive(c + 0, ntiles)) return;
  ring_post(D->ring[TR_OUT], MSG_MAKE(0, s, n));
  if (parent_code < 0) return;
  const int p = parent_code >> 1;
  if (join_arrive(B.cnt + B.node(s, p) * 4 + 1, 2)) ring_post(D->ring[TR_BRANCH], MSG_MAKE(0, s, p));
}

// One gradient part for node n has been written: Bcast's backward waits for
// the output layer's part and (unless n is the root) every parent tile's.
__device__ __forceinline__ void tree_grad_part_done(const AmpDev* D, const TreeBufs& B, int s, int n, bool is_root, bool is_leaf) {
  const int expect = is_root ? 1 : 1 + B.TB;
  if (join_arrive(B.cnt + B.node(s, n) * 4 + 2, expect))
    ring_post(D->ring[is_leaf ? TR_LEAF : TR_BRANCH], MSG_MAKE(1, s, n));
}

// ------------------------------------------------------------ lookup
// Thread c owns column c of every row it touches, so the messages of a batch
// need no barriers between them.
__device__ __noinline__ void role_tree_lookup(const AmpDev* D, const WorkerDev* W) {
  float* lds = amp_lds;
  const NodeDev& lk = D->node[0];
  const TreeBufs B = tree_bufs(D);
  const int E = B.D, KB = W->kb;
  int* left_cnt = (int*)lds;                  // [mak] leaves not yet answered
  int* pend_tok = left_cnt + ((D->mak + 3) & ~3);
  for (int i = threadIdx.x; i < D->mak; i += AMP_THREADS) left_cnt[i] = 0;
  BatchMsg& M = s_M;
  const RingDev& mine = D->ring[W->ring];
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  int* keep = (int*)D->buf[10];
  float* prow = (float*)D->buf[11];
  for (unsigned k = threadIdx.x; k < count; k += AMP_THREADS) pend_tok[k] = keep[k];
  __syncthreads();
  for (;;) {
    const int n = wait_batch(D, mine, head, KB, lk.muf - (int)count, s_codes, &s_n, code_is_b);
    if (n == 0) break;
    if ((int)threadIdx.x < n) {
      const int k = threadIdx.x;
      const unsigned code = s_codes[k];
      const int s = MSG_SLOT(code), l = MSG_LOCAL(code);
      const unsigned seq = D->slot_seq[s];
      const TreeView v = tree_view(D, seq);
      M.s[k] = s;
      M.n[k] = l;
      M.seq[k] = seq;
      M.a[k] = v.tok[l];
      M.aux[k] = code_is_b(code);
      if (!code_is_b(code) && l == 0) left_cnt[s] = v.L;
    }
    __syncthreads();
    // ordinal of each backward message inside the batch
    if (threadIdx.x == 0) {
      int nb = 0;
      for (int k = 0; k < n; ++k) {
        M.b[k] = nb;
        if (M.aux[k]) pend_tok[count + nb++] = M.a[k];
      }
      M.nB = nb;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < E; c += AMP_THREADS) {
      float v[KB_MAX];
#pragma unroll
      for (int k = 0; k < KB_MAX; ++k) {
        v[k] = 0.f;
        if (k < n) {
          if (!M.aux[k]) {
            v[k] = lk.P[(long long)M.a[k] * E + c];
          } else {
            const float* gx = B.gx + B.leaf(M.s[k], M.n[k]) * B.TL * E + c;
            float a = 0.f;
            for (int t = 0; t < B.TL; ++t) a += gx[t * E];
            v[k] = a;
          }
        }
      }
#pragma unroll
      for (int k = 0; k < KB_MAX; ++k) {
        if (k < n) {
          if (!M.aux[k])
            B.xin[B.leaf(M.s[k], M.n[k]) * E + c] = v[k];
          else
            prow[(long long)(count + M.b[k]) * E + c] = v[k];
        }
      }
    }
    if (threadIdx.x == 0 && W->log_cap)
      for (int k = 0; k < n; ++k) log_event(D, W, &s_logn, 0, M.aux[k], M.seq[k], M.n[k]);
    __syncthreads();
    if (threadIdx.x < 64) {
      fence_release();
      const int k = threadIdx.x;
      if (k < n) {
        if (!M.aux[k]) {
          ring_post(D->ring[TR_LEAF], MSG_MAKE(0, M.s[k], M.n[k]));
        } else if (D->train) {
          if (atomicSub(&left_cnt[M.s[k]], 1) == 1) ring_post(D->ring[0], MSG_MAKE(1, M.s[k], 0));
        }
      }
    }
    count += M.nB;
    if ((int)count >= lk.muf) {
      // SGD on the touched rows: each waiting gradient row is subtracted from its
      // token's row, in arrival order (rows never touched have a zero gradient)
      tstep++;
      const float sc = lk.lr * (lk.mean ? 1.f / (float)count : 1.f);
      __syncthreads();
      for (int c = threadIdx.x; c < E; c += AMP_THREADS) {
        for (unsigned k0 = 0; k0 < count; k0 += 16) {
          const int kc = count - k0 < 16u ? (int)(count - k0) : 16;
          float w[16], g[16];
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (k < kc) {
              w[k] = lk.P[(long long)pend_tok[k0 + k] * E + c];
              g[k] = prow[(long long)(k0 + k) * E + c];
            }
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (k < kc) {
              // a token seen earlier in this chunk: continue from that result
              float base = w[k];
#pragma unroll
              for (int j = 0; j < 16; ++j)
                if (j < k && pend_tok[k0 + j] == pend_tok[k0 + k]) base = w[j];
              w[k] = base - sc * g[k];
            }
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (k < kc) lk.P[(long long)pend_tok[k0 + k] * E + c] = w[k];
        }
      }
      count = 0;
      if (threadIdx.x == 0) log_event(D, W, &s_logn, 0, 2, 0, 0);
    }
    __syncthreads();
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
  for (unsigned k = threadIdx.x; k < count; k += AMP_THREADS) keep[k] = pend_tok[k];
}

// ------------------------------------------------------------ leaf / branch cells
// BR = false: rows [i; o; u] over the embedding.
// BR = true : rows [i; f_l; f_r; o; u] over [h_l; h_r].
template <bool BR>
__device__ __noinline__ void role_tree_cell(const AmpDev* D, const WorkerDev* W) {
  float* lds = amp_lds;
  const NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const Pend pd = make_pend(W, t);
  const int R = t.R, C = t.C, H = B.H, nu = t.nu, u0 = t.u0, KB = W->kb;
  const int ldx = amp_ldrow(C), ldy = amp_ldrow(R), NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  const int xfloats = 16 * ldx > UPD_STAGE * pd.stride ? 16 * ldx : UPD_STAGE * pd.stride;
  float* X = L.take(xfloats);
  float* Y = L.take(16 * ldy);
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < xfloats; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < 16 * ldy; i += AMP_THREADS) Y[i] = 0.f;
  BatchMsg& M = s_M;
  __syncthreads();
  const RingDev& mine = D->ring[W->ring];
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  for (;;) {
    const int n = wait_batch(D, mine, head, KB, nd.muf - (int)count, s_codes, &s_n, code_is_b);
    if (n == 0) break;
    if ((int)threadIdx.x < n) {
      const int k = threadIdx.x;
      const unsigned code = s_codes[k];
      const int s = MSG_SLOT(code), nn = MSG_LOCAL(code);
      const unsigned seq = D->slot_seq[s];
      const TreeView v = tree_view(D, seq);
      M.s[k] = s;
      M.n[k] = nn;
      M.seq[k] = seq;
      M.a[k] = BR ? v.left[nn] : 0;
      M.b[k] = BR ? v.right[nn] : 0;
      M.par[k] = v.parent[nn];
      M.L[k] = v.L;
      M.aux[k] = code_is_b(code);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int nf = 0, nb = 0;
      for (int k = 0; k < n; ++k) {
        if (M.aux[k])
          M.bidx[nb++] = k;
        else
          M.fidx[nf++] = k;
        if (W->tile == 0) log_event(D, W, &s_logn, W->node, M.aux[k], M.seq[k], M.n[k]);
      }
      M.nF = nf;
      M.nB = nb;
    }
    __syncthreads();
    const int nF = M.nF, nB = M.nB;
    PHASE(0);
    // ---------------- forward messages of the batch
    if (nF > 0) {
      for (int i = threadIdx.x; i < nF * ldx; i += AMP_THREADS) {
        const int k = i / ldx, c = i - k * ldx, m = M.fidx[k];
        float v = 0.f;   // padding columns of a used row are zero
        if (c < C) {
          if (BR)
            v = c < H ? B.hc[B.node(M.s[m], M.a[m]) * 2 * H + c] : B.hc[B.node(M.s[m], M.b[m]) * 2 * H + c - H];
          else
            v = B.xin[B.leaf(M.s[m], M.n[m]) * C + c];
        }
        X[i] = v;
      }
      __syncthreads();
      PHASE(1);
      mfma_rows((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)bl, (LDSQ float*)X, ldx, 1, (LDSQ float*)Y, ldy);
      PHASE(2);
      for (int i = threadIdx.x; i < nF * nu; i += AMP_THREADS) {
        const int k = i / nu, j = i - k * nu, m = M.fidx[k], u = u0 + j;
        const float* y = Y + k * ldy;
        float* hcn = B.hc + B.node(M.s[m], M.n[m]) * 2 * H;
        float* gt = B.gate + B.node(M.s[m], M.n[m]) * 6 * H;
        float c_, o_;
        if (BR) {
          const float cl = B.hc[B.node(M.s[m], M.a[m]) * 2 * H + H + u];
          const float cr = B.hc[B.node(M.s[m], M.b[m]) * 2 * H + H + u];
          const float i_ = sigmoidf_(y[j]), fl = sigmoidf_(y[nu + j]), fr = sigmoidf_(y[2 * nu + j]);
          o_ = sigmoidf_(y[3 * nu + j]);
          const float g_ = tanhf(y[4 * nu + j]);
          c_ = i_ * g_ + fl * cl + fr * cr;
          gt[u] = i_;
          gt[H + u] = fl;
          gt[2 * H + u] = fr;
          gt[3 * H + u] = o_;
          gt[4 * H + u] = g_;
        } else {
          const float i_ = sigmoidf_(y[j]);
          o_ = sigmoidf_(y[nu + j]);
          const float g_ = tanhf(y[2 * nu + j]);
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
      __syncthreads();
      PHASE(3);
    }
    // ---------------- backward messages of the batch
    if (nB > 0) {
      for (int i = threadIdx.x; i < nB * ldx; i += AMP_THREADS) {
        const int k = i / ldx, c = i - k * ldx, m = M.bidx[k];
        float v = 0.f;   // padding columns of a used row are zero
        if (c < C) {
          if (BR)
            v = c < H ? B.hc[B.node(M.s[m], M.a[m]) * 2 * H + c] : B.hc[B.node(M.s[m], M.b[m]) * 2 * H + c - H];
          else
            v = B.xin[B.leaf(M.s[m], M.n[m]) * C + c];
        }
        X[i] = v;
      }
      for (int i = threadIdx.x; i < nB * (ldy - R); i += AMP_THREADS) {
        const int k = i / (ldy - R), r = R + i - k * (ldy - R);
        Y[k * ldy + r] = 0.f;
      }
      for (int i = threadIdx.x; i < nB * nu; i += AMP_THREADS) {
        const int k = i / nu, j = i - k * nu, m = M.bidx[k], u = u0 + j;
        const long long nn = B.node(M.s[m], M.n[m]);
        const float* gt = B.gate + nn * 6 * H;
        float dh = B.gout[nn * H + u], dc = 0.f;
        if (M.par[m] >= 0) {
          const float* gp = B.gpar + nn * B.TB * H + u;
          float p = 0.f;
          for (int q = 0; q < B.TB; ++q) p += gp[q * H];
          dh += p;
          dc = B.gc[nn * H + u];
        }
        const float i_ = gt[u], o_ = gt[3 * H + u], g_ = gt[4 * H + u], tc = gt[5 * H + u];
        const float dct = dc + dh * o_ * (1.f - tc * tc);
        const float d_o = dh * tc * o_ * (1.f - o_);
        const float d_i = dct * g_ * i_ * (1.f - i_);
        const float d_g = dct * i_ * (1.f - g_ * g_);
        float* ds = Y + k * ldy;
        if (BR) {
          const long long na = B.node(M.s[m], M.a[m]), nb = B.node(M.s[m], M.b[m]);
          const float fl = gt[H + u], fr = gt[2 * H + u];
          ds[j] = d_i;
          ds[nu + j] = dct * B.hc[na * 2 * H + H + u] * fl * (1.f - fl);
          ds[2 * nu + j] = dct * B.hc[nb * 2 * H + H + u] * fr * (1.f - fr);
          ds[3 * nu + j] = d_o;
          ds[4 * nu + j] = d_g;
          B.gc[na * H + u] = dct * fl;
          B.gc[nb * H + u] = dct * fr;
        } else {
          ds[j] = d_i;
          ds[nu + j] = d_o;
          ds[2 * nu + j] = d_g;
        }
      }
      __syncthreads();
      PHASE(4);
      pend_append(pd, count, Y, ldy, R, X, ldx, C, nB);
      __syncthreads();
      mfma_cols((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)Y, ldy, 1, (LDSQ float*)X, ldx);
      PHASE(5);
      for (int i = threadIdx.x; i < nB * C; i += AMP_THREADS) {
        const int k = i / C, c = i - k * C, m = M.bidx[k];
        const float v = X[k * ldx + c];
        if (BR) {
          if (c < H)
            B.gpar[(B.node(M.s[m], M.a[m]) * B.TB + W->tile) * H + c] = v;
          else
            B.gpar[(B.node(M.s[m], M.b[m]) * B.TB + W->tile) * H + c - H] = v;
        } else {
          B.gx[(B.leaf(M.s[m], M.n[m]) * B.TL + W->tile) * C + c] = v;
        }
      }
      __syncthreads();
    }
    // ---------------- joins and posts, one lane per message
    if (threadIdx.x < 64) {
      fence_release();
      const int k = threadIdx.x;
      if (k < n) {
        const int s = M.s[k], nn = M.n[k];
        if (!M.aux[k]) {
          tree_node_part_done(D, B, s, nn, M.par[k], W->ntiles);
        } else if (BR) {
          tree_grad_part_done(D, B, s, M.a[k], false, M.a[k] < M.L[k]);
          tree_grad_part_done(D, B, s, M.b[k], false, M.b[k] < M.L[k]);
        } else {
          if (join_arrive(B.cnt + B.node(s, nn) * 4 + 3, B.TL)) ring_post(D->ring[TR_LOOKUP], MSG_MAKE(1, s, nn));
        }
      }
    }
    PHASE(6);
    count += nB;
    if ((int)count >= nd.muf) {
      tstep++;
      mfma_update((LDSQ float*)Wl, (LDSQ float*)bl, &nd, t, pd.base, pd.stride, count, count, tstep, (LDSQ float*)X);
      count = 0;
      LOG(W->node, 2, 0, 0);
    }
    __syncthreads();
    PHASE(7);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}

// ------------------------------------------------------------ output layer + loss at every node
// One wave per message: forward, softmax loss and backward in one event.
__device__ __noinline__ void role_tree_out(const AmpDev* D, const WorkerDev* W) {
  float* lds = amp_lds;
  const NodeDev& nd = D->node[3];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const Pend pd = make_pend(W, t);
  const int R = t.R, C = t.C, H = B.H, KB = W->kb;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, NW = AMP_THREADS >> 6;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  float* hbuf = L.take(NW * C);            // per wave: the node's h
  float* zbuf = L.take(NW * 64);           // per wave: logits, then dz
  float* stage = L.take(UPD_STAGE * pd.stride);
  int* done_cnt = (int*)L.take(D->mak);    // eval: nodes scored per slot
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < D->mak; i += AMP_THREADS) done_cnt[i] = 0;
  BatchMsg& M = s_M;
  __syncthreads();
  const RingDev& mine = D->ring[W->ring];
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  for (;;) {
    const int room = D->train ? nd.muf - (int)count : KB_MAX;
    const int n = wait_batch(D, mine, head, KB, room, s_codes, &s_n, [](unsigned) { return true; });
    if (n == 0) break;
    if ((int)threadIdx.x < n) {
      const int k = threadIdx.x;
      const unsigned code = s_codes[k];
      const int s = MSG_SLOT(code), nn = MSG_LOCAL(code);
      const unsigned seq = D->slot_seq[s];
      const TreeView v = tree_view(D, seq);
      M.s[k] = s;
      M.n[k] = nn;
      M.seq[k] = seq;
      M.a[k] = v.lab[nn];
      M.par[k] = v.parent[nn];
      M.L[k] = v.L;
    }
    __syncthreads();
    float* hw = hbuf + wave * C;
    float* zw = zbuf + wave * 64;
    for (int k = wave; k < n; k += NW) {
      const int s = M.s[k], nn = M.n[k], label = M.a[k];
      const float* h = B.hc + B.node(s, nn) * 2 * H;
      for (int c = lane; c < C; c += 64) hw[c] = h[c];
      // logits: lane r keeps z_r
      float zmine = -3.0e38f;
      for (int r = 0; r < R; ++r) {
        float a = 0.f;
        for (int c = lane; c < C; c += 64) a = fmaf(Wl[r * t.ldw + c], hw[c], a);
        for (int off = 32; off; off >>= 1) a += __shfl_xor(a, off);
        if (lane == r) zmine = a + bl[r];
      }
      float m = zmine;
      int am = lane < R ? lane : 0x7fffffff;
      for (int off = 32; off; off >>= 1) {
        const float om = __shfl_xor(m, off);
        const int oa = __shfl_xor(am, off);
        if (om > m || (om == m && oa < am)) {
          m = om;
          am = oa;
        }
      }
      const float e = lane < R ? expf(zmine - m) : 0.f;
      float se = e;
      for (int off = 32; off; off >>= 1) se += __shfl_xor(se, off);
      const float zl = __shfl(zmine, label);
      const float dz = e / se - (lane == label ? 1.f : 0.f);
      if (lane < 64) zw[lane] = lane < R ? dz : 0.f;
      if (lane == 0) {
        const unsigned idx = M.seq[k] - D->first_seq;
        atomicAdd(&D->loss_out[idx], -(zl - m - logf(se)));
        if (am == label) atomicAdd(&D->correct_out[idx], 1);
      }
      if (!D->train) continue;
      // dh = W^T dz, and the (dz, h) pair joins the pending gradients
      float* go = B.gout + B.node(s, nn) * H;
      for (int c = lane; c < C; c += 64) {
        float a = 0.f;
        for (int r = 0; r < R; ++r) a = fmaf(Wl[r * t.ldw + c], zw[r], a);
        go[c] = a;
      }
      float* pe = pd.base + (long long)(count + k) * pd.stride;
      for (int j = lane; j < pd.stride; j += 64) {
        float v = 0.f;
        if (j < pd.Rp) {
          if (j < R) v = zw[j];
        } else if (j - pd.Rp < C) {
          v = hw[j - pd.Rp];
        }
        pe[j] = v;
      }
    }
    if (threadIdx.x == 0 && W->log_cap)
      for (int k = 0; k < n; ++k) {
        log_event(D, W, &s_logn, 3, 0, M.seq[k], M.n[k]);
        if (D->train) log_event(D, W, &s_logn, 3, 1, M.seq[k], M.n[k]);
      }
    __syncthreads();
    if (threadIdx.x < 64) {
      fence_release();
      const int k = threadIdx.x;
      if (k < n) {
        if (!D->train) {
          if (atomicAdd(&done_cnt[M.s[k]], 1) + 1 == 2 * M.L[k] - 1) {
            done_cnt[M.s[k]] = 0;
            ring_post(D->ring[0], MSG_MAKE(1, M.s[k], 0));
          }
        } else {
          tree_grad_part_done(D, B, M.s[k], M.n[k], M.par[k] < 0, M.n[k] < M.L[k]);
        }
      }
    }
    if (D->train) {
      count += n;
      if ((int)count >= nd.muf) {
        tstep++;
        mfma_update((LDSQ float*)Wl, (LDSQ float*)bl, &nd, t, pd.base, pd.stride, count, count, tstep, (LDSQ float*)stage);
        count = 0;
        LOG(3, 2, 0, 0);
      }
    }
    __syncthreads();
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}
