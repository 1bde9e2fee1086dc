// Tree-LSTM workers (Section 5, Tree-LSTM paragraph): lookup, leaf cell,
// branch cell, output layer with a softmax loss at every tree node.
//
// Leaf and branch cells are split over several workgroups ("tiles", Section
// 5.1); the tiles of a cell read the same ring in the same order and cut
// their batches at the same updates, so they act as one node with one event
// order.  Tile t owns hidden units [u0, u0+nu) of every gate, computes those
// units' h and c entirely, and contributes a partial W^T delta over all
// input columns on the way back.
//
// A worker takes up to 64 waiting messages at once.  The inputs of the
// forward product go from the slot storage in HBM straight into the matrix
// cores' operand registers (rows there are padded to multiples of 4 floats so
// that every 16-byte fetch is aligned); the input gradient goes from the
// accumulators straight back to HBM.
//
// Slot storage (s = slot, n = tree node, l = leaf; Hp, Ep = H, E rounded up to 4;
// padding entries stay zero):
//   buf[0] xin  [s][l][Ep]       embedding recorded by the lookup's forward
//   buf[1] hc   [s][n][2][Hp]    node output: h then c
//   buf[2] gate [s][n][6][H]     gate activations and tanh(c) recorded at forward
//   buf[3] gout [s][n][H]        dh from the output layer
//   buf[4] gpar [s][n][TB][Hp]   dh partials from the parent's tiles
//   buf[5] gc   [s][n][H]        dc from the parent
//   buf[6] gx   [s][l][TL][Ep]   dx partials from the leaf tiles
//   buf[7] cnt  [s][n][4] (int)  arrival counters: tiles done / children done /
//                                gradient parts / leaf-tile dx parts
//   buf[10] lookup: tokens of the gradients waiting for the next update
//   buf[11] lookup: their gradient rows [AMP_TREE_LOOKUP_MAX_MUF][E]
#pragma once

struct TreeBufs {
  float *xin, *hc, *gate, *gout, *gpar, *gc, *gx;
  int* cnt;
  int H, Hp, E, Ep, NNmax, Lmax, TL, TB;
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
  b.Hp = amp_round4(D->hidden);
  b.E = D->emb;
  b.Ep = amp_round4(D->emb);
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

typedef int v4i __attribute__((ext_vector_type(4)));

// What the controller wrote for slot s at admission: admission number, leaves, node offset, token offset.
__device__ __forceinline__ v4i tree_slot(const AmpDev* D, int s) { return *(const v4i*)(D->smeta + 4 * s); }
// left, right, parent * 2 + side (-1 for the root), label of node n of the instance whose nodes start at noff
__device__ __forceinline__ v4i tree_node(const AmpDev* D, int noff, int n) {
  return *(const v4i*)(D->data.tnode + 4 * (long long)(noff + n));
}

// Wave 0, all 64 lanes, after lanes k < n have written M.aux[k]: positions of
// the batch's forward and backward messages, and the event record (tile 0 only).
__device__ __forceinline__ void batch_split_and_log(const AmpDev* D, const WorkerDev* W, BatchMsg& M, int n, int node,
                                                    bool both_kinds) {
  const int k = threadIdx.x;   // < 64
  const bool in = k < n, isb = in && M.aux[k] != 0;
  const unsigned long long mb = __ballot(isb), mf = __ballot(in && !isb);
  const unsigned long long lt = (1ull << k) - 1ull;
  if (isb) M.bidx[__popcll(mb & lt)] = k;
  if (in && !isb) M.fidx[__popcll(mf & lt)] = k;
  if (k == 0) {
    M.nF = __popcll(mf);
    M.nB = __popcll(mb);
  }
  if (W->log_cap && W->tile == 0) {
    // both_kinds: every message is a forward event followed by a backward event (output layer in training)
    const unsigned per = both_kinds ? 2u : 1u, base = s_logn;
    if (base + per * (unsigned)n > W->log_cap) {
      if (k == 0) raise_abort(D, ABORT_LOG_FULL, blockIdx.x);
    } else {
      if (in) {
        const unsigned long long tail = ((unsigned long long)M.seq[k] << 32) | ((unsigned)node << 20) | ((unsigned)M.n[k] & 0xfffffu);
        if (both_kinds) {
          W->log[base + 2 * k] = tail;
          W->log[base + 2 * k + 1] = tail | (1ull << 28);
        } else {
          W->log[base + k] = tail | ((unsigned long long)(isb ? 1 : 0) << 28);
        }
      }
      if (k == 0) s_logn = base + per * (unsigned)n;
    }
  }
}

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
__device__ __noinline__ void role_tree_lookup(const AmpDev* D, const WorkerDev* W) {
  float* lds = amp_lds;
  const NodeDev& lk = D->node[0];
  const TreeBufs B = tree_bufs(D);
  const int E = B.E, Ep = B.Ep, KB = W->kb, E4 = E >> 2;
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
    if (threadIdx.x < 64) {
      const int k = threadIdx.x;
      if (k < n) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), l = MSG_LOCAL(code);
        const v4i sm = tree_slot(D, s);
        M.s[k] = s;
        M.n[k] = l;
        M.seq[k] = (unsigned)sm.x;
        M.a[k] = D->data.tok[sm.w + l];
        M.aux[k] = code_is_b(code);
        if (!code_is_b(code) && l == 0) left_cnt[s] = sm.y;
      }
      batch_split_and_log(D, W, M, n, 0, false);
      // backward message k is the b-th gradient of the batch: remember its token
      const bool isb = k < n && M.aux[k] != 0;
      const unsigned long long mb = __ballot(isb);
      if (isb) {
        const int b = __popcll(mb & ((1ull << k) - 1ull));
        M.b[k] = b;
        pend_tok[count + b] = M.a[k];
      }
    }
    __syncthreads();
    if ((E & 3) == 0) {
      // forward: table row -> xin; backward: sum of the leaf tiles' partials -> pending gradient row
      for (int idx = threadIdx.x; idx < n * E4; idx += AMP_THREADS) {
        const int k = idx / E4, c = (idx - k * E4) << 2;
        if (!M.aux[k]) {
          *(v4f*)(B.xin + B.leaf(M.s[k], M.n[k]) * Ep + c) = *(const v4f*)(lk.P + (long long)M.a[k] * E + c);
        } else {
          const float* gx = B.gx + B.leaf(M.s[k], M.n[k]) * B.TL * Ep + c;
          v4f a = {0.f, 0.f, 0.f, 0.f};
          for (int t = 0; t < B.TL; ++t) a += *(const v4f*)(gx + t * Ep);
          *(v4f*)(prow + (long long)(count + M.b[k]) * E + c) = a;
        }
      }
    } else {
      for (int idx = threadIdx.x; idx < n * E; idx += AMP_THREADS) {
        const int k = idx / E, c = idx - k * E;
        if (!M.aux[k]) {
          B.xin[B.leaf(M.s[k], M.n[k]) * Ep + c] = lk.P[(long long)M.a[k] * E + c];
        } else {
          const float* gx = B.gx + B.leaf(M.s[k], M.n[k]) * B.TL * Ep + c;
          float a = 0.f;
          for (int t = 0; t < B.TL; ++t) a += gx[t * Ep];
          prow[(long long)(count + M.b[k]) * E + c] = a;
        }
      }
    }
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

// ------------------------------------------------------------ matrix-core products of a cell tile
// Y[j][r] = b[r] + sum_c W[r][c] x_j[c] for the nF forward messages of the batch.
// Wave item = (16 messages, 16 weight rows); the messages' inputs are fetched
// from HBM (xbase + M.off0 / off1 for the first / second column segment)
// eight 16-column groups ahead of their use.
template <bool BR>
__device__ __forceinline__ void tree_fwd_mfma(const LDSQ float* Wl, const Tile& t, const LDSQ float* bl, const float* xbase,
                                              const BatchMsg& M, int nF, LDSQ float* Y, int ldy) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = t.Rp >> 4, NCG = amp_round16(t.Cl) >> 4, NBF = (nF + 15) >> 4;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  for (int item = wave; item < NBF * NRB; item += AMP_THREADS / 64) {
    const int rb = item % NRB, nb = item / NRB;
    int mi = nb * 16 + i;
    if (mi > nF - 1) mi = nF - 1;   // rows beyond the batch repeat its last message; their results are dropped
    const int m = M.fidx[mi];
    const float* p0 = xbase + M.off0[m] + 4 * q;
    const float* p1 = xbase + M.off1[m] + 4 * q - t.segp;
    const LDSQ float* wp = Wl + (rb * 16 + i) * t.ldw + 4 * q;
    auto fetch = [&](int kg) -> v4f {
      const int lc = kg * 16 + 4 * q;
      if (lc >= t.Cl) return zero;
      return *(const v4f*)((BR && lc >= t.segp ? p1 : p0) + kg * 16);
    };
    v4f acc0 = zero, acc1 = zero, xa[8], xb[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) xa[j] = fetch(j);
    for (int kc = 0; kc < NCG; kc += 16) {
#pragma unroll
      for (int j = 0; j < 8; ++j) xb[j] = fetch(kc + 8 + j);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (kc + j < NCG) {
          const v4f w = *(const LDSQ v4f*)(wp + 16 * (kc + j));
          acc0 = MFMA(w.x, xa[j].x, acc0);
          acc1 = MFMA(w.y, xa[j].y, acc1);
          acc0 = MFMA(w.z, xa[j].z, acc0);
          acc1 = MFMA(w.w, xa[j].w, acc1);
        }
#pragma unroll
      for (int j = 0; j < 8; ++j) xa[j] = fetch(kc + 16 + j);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (kc + 8 + j < NCG) {
          const v4f w = *(const LDSQ v4f*)(wp + 16 * (kc + 8 + j));
          acc0 = MFMA(w.x, xb[j].x, acc0);
          acc1 = MFMA(w.y, xb[j].y, acc1);
          acc0 = MFMA(w.z, xb[j].z, acc0);
          acc1 = MFMA(w.w, xb[j].w, acc1);
        }
    }
    const v4f b4 = *(const LDSQ v4f*)(bl + rb * 16 + 4 * q);
    *(LDSQ v4f*)(Y + (nb * 16 + i) * ldy + rb * 16 + 4 * q) = acc0 + acc1 + b4;
  }
}

// dx_j[c] = sum_r W[r][c] delta_j[r] for the nB backward messages; delta rows
// in LDS (Dl, stride ldd, zero beyond the tile's rows); the result goes from
// the accumulators to HBM at obase + M.dst0 / dst1 (+ column inside the segment).
template <bool BR>
__device__ __forceinline__ void tree_bwd_mfma(const LDSQ float* Wl, const Tile& t, const LDSQ float* Dl, int ldd,
                                              const BatchMsg& M, int nB, float* obase) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = t.Rp >> 4, NCG = amp_round16(t.Cl) >> 4, NBB = (nB + 15) >> 4;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  for (int item = wave; item < NCG * NBB; item += AMP_THREADS / 64) {
    const int cb = item % NCG, nb = item / NCG;
    const LDSQ float* wp = Wl + (4 * q) * t.ldw + cb * 16 + i;
    const LDSQ float* dp = Dl + (nb * 16 + i) * ldd + 4 * q;
    v4f acc0 = zero, acc1 = zero;
    for (int g = 0; g < NRB; ++g) {
      const v4f d0 = *(const LDSQ v4f*)(dp + 16 * g);
      const LDSQ float* w = wp + 16 * g * t.ldw;
      const float w0 = w[0], w1 = w[t.ldw], w2 = w[2 * t.ldw], w3 = w[3 * t.ldw];
      acc0 = MFMA(w0, d0.x, acc0);
      acc1 = MFMA(w1, d0.y, acc1);
      acc0 = MFMA(w2, d0.z, acc0);
      acc1 = MFMA(w3, d0.w, acc1);
    }
    const int mi = nb * 16 + i, lc = cb * 16 + 4 * q;
    if (mi < nB && lc < t.Cl) {
      const int m = M.bidx[mi];
      float* o = (BR && lc >= t.segp) ? obase + M.dst1[m] + (lc - t.segp) : obase + M.dst0[m] + lc;
      *(v4f*)o = acc0 + acc1;
    }
  }
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
  const int R = t.R, H = B.H, Hp = B.Hp, nu = t.nu, u0 = t.u0, KB = W->kb;
  const int ldy = amp_ldrow(R);
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  const int yfloats = KB * ldy > UPD_STAGE * pd.stride ? KB * ldy : UPD_STAGE * pd.stride;
  float* Y = L.take(yfloats);   // forward: pre-activations; backward: deltas; staging at updates
  tile_load(nd, t, Wl, bl);
  for (int i = threadIdx.x; i < yfloats; i += AMP_THREADS) Y[i] = 0.f;
  BatchMsg& M = s_M;
  __syncthreads();
  const RingDev& mine = D->ring[W->ring];
  const float* xbase = BR ? B.hc : B.xin;
  float* obase = BR ? B.gpar : B.gx;
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  for (;;) {
    const int n = wait_batch(D, mine, head, KB, nd.muf - (int)count, s_codes, &s_n, code_is_b);
    if (n == 0) break;
    if (threadIdx.x < 64) {
      const int k = threadIdx.x;
      if (k < n) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), nn = MSG_LOCAL(code);
        const v4i sm = tree_slot(D, s);
        const v4i tn = tree_node(D, sm.z, nn);
        M.s[k] = s;
        M.n[k] = nn;
        M.seq[k] = (unsigned)sm.x;
        M.a[k] = tn.x;
        M.b[k] = tn.y;
        M.par[k] = tn.z;
        M.L[k] = sm.y;
        M.aux[k] = code_is_b(code);
        if (BR) {
          M.off0[k] = (int)(B.node(s, tn.x) * 2 * Hp);
          M.off1[k] = (int)(B.node(s, tn.y) * 2 * Hp);
          M.dst0[k] = (int)((B.node(s, tn.x) * B.TB + W->tile) * Hp);
          M.dst1[k] = (int)((B.node(s, tn.y) * B.TB + W->tile) * Hp);
        } else {
          M.off0[k] = M.off1[k] = (int)(B.leaf(s, nn) * B.Ep);
          M.dst0[k] = M.dst1[k] = (int)((B.leaf(s, nn) * B.TL + W->tile) * B.Ep);
        }
      }
      batch_split_and_log(D, W, M, n, W->node, false);
    }
    __syncthreads();
    const int nF = M.nF, nB = M.nB;
    PHASE(0);
    // ---------------- forward messages of the batch
    if (nF > 0) {
      tree_fwd_mfma<BR>((const LDSQ float*)Wl, t, (const LDSQ float*)bl, xbase, M, nF, (LDSQ float*)Y, ldy);
      __syncthreads();
      PHASE(1);
      for (int i = threadIdx.x; i < nF * nu; i += AMP_THREADS) {
        const int k = i / nu, j = i - k * nu, m = M.fidx[k], u = u0 + j;
        const float* y = Y + k * ldy;
        const long long nn = B.node(M.s[m], M.n[m]);
        float* hcn = B.hc + nn * 2 * Hp;
        float* gt = B.gate + nn * 6 * H;
        float c_, o_;
        if (BR) {
          const float cl = xbase[M.off0[m] + Hp + u];
          const float cr = xbase[M.off1[m] + Hp + u];
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
        hcn[Hp + u] = c_;
      }
      __syncthreads();
      PHASE(2);
    }
    // ---------------- backward messages of the batch
    if (nB > 0) {
      // delta rows (tile order [gate][unit], zero beyond R) into Y
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
          const float* gp = B.gpar + nn * B.TB * Hp + u;
          float p = 0.f;
          for (int q = 0; q < B.TB; ++q) p += gp[q * Hp];
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
          ds[nu + j] = dct * xbase[M.off0[m] + Hp + u] * fl * (1.f - fl);
          ds[2 * nu + j] = dct * xbase[M.off1[m] + Hp + u] * fr * (1.f - fr);
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
      PHASE(3);
      // the (delta, input) pairs join the pending gradients: entry = [delta (Rp) | input in LDS column layout (Cp)]
      for (int i = threadIdx.x; i < nB * (pd.stride >> 2); i += AMP_THREADS) {
        const int k = i / (pd.stride >> 2), j = (i - k * (pd.stride >> 2)) << 2, m = M.bidx[k];
        v4f v = {0.f, 0.f, 0.f, 0.f};
        if (j < pd.Rp) {
          if (j < ldy) v = *(const v4f*)(Y + k * ldy + j);   // ldy >= R, zero beyond R
        } else {
          const int lc = j - pd.Rp;
          if (lc < t.Cl) v = *(const v4f*)(xbase + ((BR && lc >= t.segp) ? M.off1[m] + lc - t.segp : M.off0[m] + lc));
        }
        *(v4f*)(pd.base + (long long)(count + k) * pd.stride + j) = v;
      }
      PHASE(4);
      tree_bwd_mfma<BR>((const LDSQ float*)Wl, t, (const LDSQ float*)Y, ldy, M, nB, obase);
      __syncthreads();
      PHASE(5);
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
      mfma_update((LDSQ float*)Wl, (LDSQ float*)bl, &nd, t, pd.base, pd.stride, count, count, tstep, (LDSQ float*)Y);
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
// The node where a forward message turns round (Section 4: the loss layer
// initiates backpropagation).  The batch's h vectors are fetched into LDS
// together; then one wave per message: logits, loss, d logits, W^T d logits,
// and the (d logits, h) pair joins the node's pending gradients.
__device__ __noinline__ void role_tree_out(const AmpDev* D, const WorkerDev* W) {
  float* lds = amp_lds;
  const NodeDev& nd = D->node[3];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const Pend pd = make_pend(W, t);
  const int R = t.R, C = t.C, H = B.H, Hp = B.Hp, KB = W->kb;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, NW = AMP_THREADS >> 6;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  float* hbuf = L.take(KB * Hp);           // per message: the node's h
  float* zbuf = L.take(NW * 64);           // per wave: d logits
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
    if (threadIdx.x < 64) {
      const int k = threadIdx.x;
      if (k < n) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), nn = MSG_LOCAL(code);
        const v4i sm = tree_slot(D, s);
        const v4i tn = tree_node(D, sm.z, nn);
        M.s[k] = s;
        M.n[k] = nn;
        M.seq[k] = (unsigned)sm.x;
        M.a[k] = tn.w;
        M.par[k] = tn.z;
        M.L[k] = sm.y;
        M.aux[k] = 0;
        M.off0[k] = (int)(B.node(s, nn) * 2 * Hp);
      }
      batch_split_and_log(D, W, M, n, 3, D->train != 0);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < n * (Hp >> 2); idx += AMP_THREADS) {
      const int k = idx / (Hp >> 2), c = (idx - k * (Hp >> 2)) << 2;
      *(v4f*)(hbuf + k * Hp + c) = *(const v4f*)(B.hc + M.off0[k] + c);
    }
    __syncthreads();
    float* zw = zbuf + wave * 64;
    for (int k = wave; k < n; k += NW) {
      const int s = M.s[k], nn = M.n[k], label = M.a[k];
      const float* hw = hbuf + k * Hp;
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
      zw[lane] = lane < R ? dz : 0.f;
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
