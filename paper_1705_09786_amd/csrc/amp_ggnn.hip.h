// Gated graph network workers (Figure 4a, Appendix C): lookup, one linear
// node per edge type, the GRU's three linear nodes (update gate, reset gate,
// candidate) and the regression layer.
//
// One message carries a whole group of rows: all edges of one type for an
// edge linear (Group by edge type), all graph nodes for the GRU nodes (the
// final Group over nodes), so each node sees one forward and one backward
// message per instance and propagation step and performs a small
// (rows x cols) x (k rows) product.  Broadcast / Ungroup / Flatmap / Group /
// sum between them are index arithmetic over the instance's edge list plus
// arrival counters.
//
// Slot storage (s = slot, it = step, v = graph node, e = directed edge):
//   buf[0]  Hm  [s][S+1][N][H]  node states before each step (Hm[.][0] = lookup output)
//   buf[1]  A   [s][S][N][H]    aggregated messages (GRU input)
//   buf[2]  Z   [s][S][N][H]    update gate
//   buf[3]  Rr  [s][S][N][H]    reset gate
//   buf[4]  Ht  [s][S][N][H]    candidate state
//   buf[5]  Msg [s][E][H]       per-edge messages of the running step
//   buf[6]  gH  [s][N][H]       gradient w.r.t. the states leaving the running step
//   buf[7]  dZ  [s][N][H]       pre-activation gradient for the update-gate node
//   buf[8]  dR  [s][N][H]       pre-activation gradient for the reset-gate node
//   buf[9]  dA  [s][3][N][H]    gradient w.r.t. A from candidate / update / reset nodes
//   buf[10] dHp [s][3][N][H]    gradient w.r.t. h from the same three
//   buf[11] dHe [s][T][N][H]    gradient w.r.t. h through the edges, per edge type
//   buf[12] dAs [s][N][H]       summed gradient w.r.t. A
//   buf[13] cnt [s][8] (int)    arrival counters
#pragma once

struct GView {
  int inst, N, E;
  const int *type, *src, *dst, *et, *tcount;
  float target;
};

__device__ __forceinline__ GView g_view(const GQ AmpDev* D, unsigned seq) {
  GView v;
  v.inst = seq % D->data.n_inst;
  const int to = D->data.tok_off[v.inst], eo = D->data.edge_off[v.inst];
  v.N = D->data.tok_off[v.inst + 1] - to;
  v.E = D->data.edge_off[v.inst + 1] - eo;
  v.type = D->data.tok + to;
  v.src = D->data.src + eo;
  v.dst = D->data.dst + eo;
  v.et = D->data.etype + eo;
  v.tcount = D->data.tcount + v.inst * 8;
  v.target = D->data.target[v.inst];
  return v;
}

struct GBufs {
  float *Hm, *A, *Z, *Rr, *Ht, *Msg, *gH, *dZ, *dR, *dA, *dHp, *dHe, *dAs;
  int* cnt;
  int H, N, Em, S, T;
  __device__ __forceinline__ long long st(int s, int it) const { return ((long long)s * S + it) * N * H; }
  __device__ __forceinline__ long long hm(int s, int it) const { return ((long long)s * (S + 1) + it) * N * H; }
  __device__ __forceinline__ long long sl(int s) const { return (long long)s * N * H; }
};

__device__ __forceinline__ GBufs g_bufs(const GQ AmpDev* D) {
  GBufs b;
  b.Hm = (float*)D->buf[0];
  b.A = (float*)D->buf[1];
  b.Z = (float*)D->buf[2];
  b.Rr = (float*)D->buf[3];
  b.Ht = (float*)D->buf[4];
  b.Msg = (float*)D->buf[5];
  b.gH = (float*)D->buf[6];
  b.dZ = (float*)D->buf[7];
  b.dR = (float*)D->buf[8];
  b.dA = (float*)D->buf[9];
  b.dHp = (float*)D->buf[10];
  b.dHe = (float*)D->buf[11];
  b.dAs = (float*)D->buf[12];
  b.cnt = (int*)D->buf[13];
  b.H = D->hidden;
  b.N = D->max_len;
  b.Em = D->max_edges;
  b.S = D->n_steps;
  b.T = D->n_edge_types;
  return b;
}

#define GR_LOOKUP 1
#define GR_EDGE0 2
#define GR_GZ(D) (2 + (D)->n_edge_types)
#define GR_GR(D) (3 + (D)->n_edge_types)
#define GR_GH(D) (4 + (D)->n_edge_types)
#define GR_RO(D) (5 + (D)->n_edge_types)

__device__ __forceinline__ int g_active_types(const GView& v, int T) {
  int n = 0;
  for (int c = 0; c < T; ++c) n += v.tcount[c] > 0;
  return n;
}

// Sends one message per edge type that occurs in the graph.  ONE thread, after a release fence.
__device__ __forceinline__ void g_post_edges(const GQ AmpDev* D, const GView& v, int s, int it, bool backward) {
  for (int c = 0; c < D->n_edge_types; ++c)
    if (v.tcount[c] > 0) ring_post(D->ring[GR_EDGE0 + c], MSG_MAKE(backward, s, it));
}

// Counts one gradient (a grouped message of K rows already appended to the
// pending list) and updates when min_update_frequency is reached.
__device__ __forceinline__ void g_count_and_update(const GQ AmpDev* D, const GQ WorkerDev* W, const GQ NodeDev& nd, const Tile& t,
                                                   float* Wl, float* bl, const Pend& pd, unsigned& count,
                                                   unsigned& nrows, unsigned& tstep, int K, float* stage) {
  count++;
  nrows += K;
  if ((int)count >= nd.muf) {
    tstep++;
    mfma_update((LDSQ float*)Wl, (LDSQ float*)bl, &nd, t, pd.base, pd.stride, count, nrows, tstep, (LDSQ float*)stage);
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
  const int H = B.H, V = D->n_node_types;
  float* El = lds;
  for (int i = threadIdx.x; i < V * H; i += AMP_THREADS) El[i] = lk.P[i];
  __syncthreads();
  const GQ RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code);
    const unsigned seq = D->slot_seq[s];
    const GView v = g_view(D, seq);
    if (!(code & MSG_DIR_B)) {
      float* h0 = B.Hm + B.hm(s, 0);
      for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) {
        const int n = i / H, j = i - n * H;
        h0[i] = El[v.type[n] * H + j];
      }
      LOG(0, 0, seq, 0);
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        g_post_edges(D, v, s, 0, false);
      }
      continue;
    }
    // backward: scatter-add the rows into the table's accumulator, node by node
    const float* g = B.gH + B.sl(s);
    for (int j = threadIdx.x; j < H; j += AMP_THREADS)
      for (int n = 0; n < v.N; ++n) lk.G[v.type[n] * H + j] += g[n * H + j];
    LOG(0, 1, seq, 0);
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      ring_post(D->ring[0], MSG_MAKE(1, s, 0));
    }
    count++;
    if ((int)count >= lk.muf) {
      tstep++;
      const float sc = lk.lr * (lk.mean ? 1.f / (float)count : 1.f);
      for (int i = threadIdx.x; i < V * H; i += AMP_THREADS) {
        El[i] -= sc * lk.G[i];
        lk.G[i] = 0.f;
      }
      __syncthreads();
      count = 0;
      LOG(0, 2, 0, 0);
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < V * H; i += AMP_THREADS) lk.P[i] = El[i];
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}

// ---------------------------------------------------------------- edge linear of type c
__device__ __noinline__ void role_g_edge(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const Pend pd = make_pend(W, t);
  const int H = B.H, ctype = W->aux, Ep = amp_round16(B.Em), Hs = amp_ldrow(H);
  const int NRB = t.Rp >> 4, NCG = amp_round16(H) >> 4;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  const int xfloats = Ep * Hs > UPD_STAGE * pd.stride ? Ep * Hs : UPD_STAGE * pd.stride;
  float* X = L.take(xfloats);     // inputs h_src; later the products W^T delta; staging at updates
  float* Y = L.take(Ep * Hs);     // outputs / deltas
  float* acc = L.take(B.N * H);
  int* elist = (int*)L.take(B.Em);
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < xfloats; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < Ep * Hs; i += AMP_THREADS) Y[i] = 0.f;
  __syncthreads();
  const GQ RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  __shared__ int s_k, s_last, s_lastb;
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code), it = MSG_LOCAL(code);
    const unsigned seq = D->slot_seq[s];
    const GView v = g_view(D, seq);
    // edges of this type, ascending (Group orders its rows by edge index)
    if (threadIdx.x == 0) {
      int k = 0;
      for (int e = 0; e < v.E; ++e)
        if (v.et[e] == ctype) elist[k++] = e;
      s_k = k;
    }
    __syncthreads();
    const int K = s_k, NB = (K + 15) >> 4;
    const float* h = B.Hm + B.hm(s, it);
    for (int i = threadIdx.x; i < K * Hs; i += AMP_THREADS) {
      const int k = i / Hs, j = i - k * Hs;
      X[i] = j < H ? h[v.src[elist[k]] * H + j] : 0.f;   // padding columns of a used row are zero
    }
    __syncthreads();
    const int nact = g_active_types(v, B.T);
    if (!(code & MSG_DIR_B)) {
      mfma_rows((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)bl, (LDSQ float*)X, Hs, NB, (LDSQ float*)Y, Hs);
      float* msg = B.Msg + (long long)s * B.Em * H;
      for (int i = threadIdx.x; i < K * H; i += AMP_THREADS) {
        const int k = i / H, j = i - k * H;
        msg[elist[k] * H + j] = Y[k * Hs + j];
      }
      LOG(W->node, 0, seq, it);
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        s_last = join_arrive(B.cnt + s * 8 + 0, nact);
      }
      __syncthreads();
      if (s_last) {
        // Ungroup, regroup by target node, sum: a_v = sum over incoming edges in edge order
        float* A = B.A + B.st(s, it);
        for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) {
          const int n = i / H, j = i - n * H;
          float a = 0.f;
          for (int e = 0; e < v.E; ++e)
            if (v.dst[e] == n) a += msg[e * H + j];
          A[i] = a;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
          fence_release();
          ring_post(D->ring[GR_GZ(D)], MSG_MAKE(0, s, it));
          ring_post(D->ring[GR_GR(D)], MSG_MAKE(0, s, it));
        }
      }
      continue;
    }
    // ---- backward: delta_e = dA[dst(e)]; dh_src(e) += W^T delta_e; one gradient for the group
    const float* dAs = B.dAs + B.sl(s);
    for (int i = threadIdx.x; i < K * Hs; i += AMP_THREADS) {
      const int k = i / Hs, j = i - k * Hs;
      Y[i] = j < H ? dAs[v.dst[elist[k]] * H + j] : 0.f;
    }
    for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) acc[i] = 0.f;
    __syncthreads();
    LOG(W->node, 1, seq, it);
    pend_append(pd, nrows, Y, Hs, H, X, Hs, H, K);
    __syncthreads();
    mfma_cols((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)Y, Hs, NB, (LDSQ float*)X, Hs);
    for (int j = threadIdx.x; j < H; j += AMP_THREADS)
      for (int k = 0; k < K; ++k) acc[v.src[elist[k]] * H + j] += X[k * Hs + j];
    __syncthreads();
    float* dHe = B.dHe + ((long long)s * B.T + ctype) * B.N * H;
    for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) dHe[i] = acc[i];
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      s_lastb = join_arrive(B.cnt + s * 8 + 3, nact);
    }
    __syncthreads();
    if (s_lastb) {
      // Flatmap / Bcast backward: total gradient w.r.t. the states entering this step
      float* gH = B.gH + B.sl(s);
      const float* dHp = B.dHp + (long long)s * 3 * B.N * H;
      const float* all = B.dHe + (long long)s * B.T * B.N * H;
      for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) {
        float a = 0.f;
        for (int c = 0; c < B.T; ++c)
          if (v.tcount[c] > 0) a += all[(long long)c * B.N * H + i];
        a += dHp[B.N * H + i] + dHp[2 * B.N * H + i];
        a += dHp[i];
        gH[i] = a;
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        if (it > 0)
          ring_post(D->ring[GR_GH(D)], MSG_MAKE(1, s, it - 1));
        else
          ring_post(D->ring[GR_LOOKUP], MSG_MAKE(1, s, 0));
      }
    }
    g_count_and_update(D, W, nd, t, Wl, bl, pd, count, nrows, tstep, K, X);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
    W->wstate[4] = nrows;
  }
}

// ---------------------------------------------------------------- GRU gate nodes (aux 0: update z, aux 1: reset r)
__device__ __noinline__ void role_g_gate(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const Pend pd = make_pend(W, t);
  const int H = B.H, C = 2 * H, Np = amp_round16(B.N), which = W->aux, Hs = amp_ldrow(H), Cs = amp_ldrow(C);
  const int NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  const int xfloats = Np * Cs > UPD_STAGE * pd.stride ? Np * Cs : UPD_STAGE * pd.stride;
  float* X = L.take(xfloats);     // inputs; later W^T delta; staging at updates
  float* Y = L.take(Np * Hs);
  float* DX = X;
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < xfloats; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < Np * Hs; i += AMP_THREADS) Y[i] = 0.f;
  __syncthreads();
  const GQ RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  __shared__ int s_last;
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code), it = MSG_LOCAL(code);
    const unsigned seq = D->slot_seq[s];
    const GView v = g_view(D, seq);
    const int K = v.N;
    const float* A = B.A + B.st(s, it);
    const float* h = B.Hm + B.hm(s, it);
    for (int i = threadIdx.x; i < K * Cs; i += AMP_THREADS) {
      const int k = i / Cs, c = i - k * Cs;
      X[i] = c < H ? A[k * H + c] : c < C ? h[k * H + c - H] : 0.f;   // padding columns of a used row are zero
    }
    __syncthreads();
    float* outp = (which == 0 ? B.Z : B.Rr) + B.st(s, it);
    if (!(code & MSG_DIR_B)) {
      mfma_rows((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)bl, (LDSQ float*)X, Cs, (K + 15) >> 4, (LDSQ float*)Y, Hs);
      for (int i = threadIdx.x; i < K * H; i += AMP_THREADS) outp[i] = sigmoidf_(Y[(i / H) * Hs + i % H]);
      LOG(W->node, 0, seq, it);
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        if (join_arrive(B.cnt + s * 8 + 1, 2)) ring_post(D->ring[GR_GH(D)], MSG_MAKE(0, s, it));
      }
      continue;
    }
    const float* dpre = (which == 0 ? B.dZ : B.dR) + B.sl(s);
    for (int i = threadIdx.x; i < K * Hs; i += AMP_THREADS) {
      const int k = i / Hs, j = i - k * Hs;
      Y[i] = j < H ? dpre[k * H + j] : 0.f;
    }
    __syncthreads();
    LOG(W->node, 1, seq, it);
    pend_append(pd, nrows, Y, Hs, H, X, Cs, C, K);
    __syncthreads();
    mfma_cols((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)Y, Hs, (K + 15) >> 4, (LDSQ float*)DX, Cs);
    float* dA = B.dA + ((long long)s * 3 + 1 + which) * B.N * H;
    float* dHp = B.dHp + ((long long)s * 3 + 1 + which) * B.N * H;
    for (int i = threadIdx.x; i < K * C; i += AMP_THREADS) {
      const int k = i / C, c = i - k * C;
      if (c < H)
        dA[k * H + c] = DX[k * Cs + c];
      else
        dHp[k * H + c - H] = DX[k * Cs + c];
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      s_last = join_arrive(B.cnt + s * 8 + 2, 2);
    }
    __syncthreads();
    if (s_last) {
      // Bcast backward on A: (update + reset) + candidate, then back through sum / Group to the edges
      const float* all = B.dA + (long long)s * 3 * B.N * H;
      float* dAs = B.dAs + B.sl(s);
      for (int i = threadIdx.x; i < K * H; i += AMP_THREADS)
        dAs[i] = (all[B.N * H + i] + all[2 * B.N * H + i]) + all[i];
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        g_post_edges(D, v, s, it, true);
      }
    }
    g_count_and_update(D, W, nd, t, Wl, bl, pd, count, nrows, tstep, K, X);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
    W->wstate[4] = nrows;
  }
}

// ---------------------------------------------------------------- GRU candidate node + blend + loop control
__device__ __noinline__ void role_g_cand(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const GBufs B = g_bufs(D);
  const Pend pd = make_pend(W, t);
  const int H = B.H, C = 2 * H, Np = amp_round16(B.N), Hs = amp_ldrow(H), Cs = amp_ldrow(C);
  const int NRB = t.Rp >> 4, NCG = amp_round16(C) >> 4;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  const int xfloats = Np * Cs > UPD_STAGE * pd.stride ? Np * Cs : UPD_STAGE * pd.stride;
  float* X = L.take(xfloats);     // inputs; later W^T delta; staging at updates
  float* Y = L.take(Np * Hs);
  float* DX = X;
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < xfloats; i += AMP_THREADS) X[i] = 0.f;
  for (int i = threadIdx.x; i < Np * Hs; i += AMP_THREADS) Y[i] = 0.f;
  __syncthreads();
  const GQ RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1], nrows = W->wstate[4];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code), it = MSG_LOCAL(code);
    const unsigned seq = D->slot_seq[s];
    const GView v = g_view(D, seq);
    const int K = v.N;
    const float* A = B.A + B.st(s, it);
    const float* h = B.Hm + B.hm(s, it);
    const float* Z = B.Z + B.st(s, it);
    const float* Rr = B.Rr + B.st(s, it);
    float* Ht = B.Ht + B.st(s, it);
    for (int i = threadIdx.x; i < K * Cs; i += AMP_THREADS) {
      const int k = i / Cs, c = i - k * Cs;
      X[i] = c < H ? A[k * H + c] : c < C ? Rr[k * H + c - H] * h[k * H + c - H] : 0.f;
    }
    __syncthreads();
    if (!(code & MSG_DIR_B)) {
      mfma_rows((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)bl, (LDSQ float*)X, Cs, (K + 15) >> 4, (LDSQ float*)Y, Hs);
      float* hn = B.Hm + B.hm(s, it + 1);
      for (int i = threadIdx.x; i < K * H; i += AMP_THREADS) {
        const float ht = tanhf(Y[(i / H) * Hs + i % H]), z = Z[i];
        Ht[i] = ht;
        hn[i] = (1.f - z) * h[i] + z * ht;
      }
      LOG(W->node, 0, seq, it);
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        if (it + 1 < B.S)
          g_post_edges(D, v, s, it + 1, false);
        else
          ring_post(D->ring[GR_RO(D)], MSG_MAKE(0, s, 0));
      }
      continue;
    }
    // backward through blend, tanh, the candidate linear and r*h
    const float* gH = B.gH + B.sl(s);
    float* dZ = B.dZ + B.sl(s);
    float* dR = B.dR + B.sl(s);
    for (int i = threadIdx.x; i < K * H; i += AMP_THREADS) {
      const float g = gH[i], z = Z[i], ht = Ht[i];
      dZ[i] = g * (ht - h[i]) * z * (1.f - z);
      Y[(i / H) * Hs + i % H] = g * z * (1.f - ht * ht);
    }
    for (int i = threadIdx.x; i < K * (Hs - H); i += AMP_THREADS) Y[(i / (Hs - H)) * Hs + H + i % (Hs - H)] = 0.f;
    __syncthreads();
    LOG(W->node, 1, seq, it);
    pend_append(pd, nrows, Y, Hs, H, X, Cs, C, K);
    __syncthreads();
    mfma_cols((LDSQ float*)Wl, t.ldw, NRB, NCG, (LDSQ float*)Y, Hs, (K + 15) >> 4, (LDSQ float*)DX, Cs);
    float* dA = B.dA + (long long)s * 3 * B.N * H;
    float* dHp = B.dHp + (long long)s * 3 * B.N * H;
    for (int i = threadIdx.x; i < K * H; i += AMP_THREADS) {
      const int k = i / H, j = i - k * H;
      const float drh = DX[k * Cs + H + j], r = Rr[i], z = Z[i];
      dA[i] = DX[k * Cs + j];
      dR[i] = drh * h[i] * r * (1.f - r);
      dHp[i] = drh * r + gH[i] * (1.f - z);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      ring_post(D->ring[GR_GZ(D)], MSG_MAKE(1, s, it));
      ring_post(D->ring[GR_GR(D)], MSG_MAKE(1, s, it));
    }
    g_count_and_update(D, W, nd, t, Wl, bl, pd, count, nrows, tstep, K, X);
  }
  tile_store(nd, t, Wl, bl);
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
  const int H = B.H;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  float* pooled = L.take(H);
  float* red = L.take(AMP_THREADS);
  tile_load(nd, t, Wl, bl);
  const GQ RingDev& mine = D->ring[W->ring];
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code);
    const unsigned seq = D->slot_seq[s];
    const GView v = g_view(D, seq);
    const float* h = B.Hm + B.hm(s, B.S);
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
      D->loss_out[seq - D->first_seq] = 0.5f * d * d;
      D->yhat_out[seq - D->first_seq] = yhat;
    }
    if (!D->train) {
      __syncthreads();
      if (threadIdx.x == 0) {
        fence_release();
        ring_post(D->ring[0], MSG_MAKE(1, s, 0));
      }
      continue;
    }
    LOG(W->node, 1, seq, 0);
    float* gH = B.gH + B.sl(s);
    for (int i = threadIdx.x; i < v.N * H; i += AMP_THREADS) gH[i] = d * Wl[i % H];
    for (int j = threadIdx.x; j < H; j += AMP_THREADS) nd.G[j] += d * pooled[j];
    if (threadIdx.x == 0) nd.G[H] += d;
    __syncthreads();
    if (threadIdx.x == 0) {
      fence_release();
      ring_post(D->ring[GR_GH(D)], MSG_MAKE(1, s, B.S - 1));
    }
    count_and_update(D, W, nd, t, Wl, bl, count, tstep);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}
