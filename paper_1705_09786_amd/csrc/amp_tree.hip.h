// Tree-LSTM workers (Section 6, Tree-LSTM paragraph): lookup, leaf cell,
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
// accumulators straight back to HBM.  Each backward message appends its (delta,
// input) pair to the tile's pending list in HBM; the update forms the
// accumulated gradient from that list on the matrix cores.
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
  GQ float *xin, *hc, *gate, *gout, *gpar, *gc, *gx;
  GQ int* cnt;
  int H, Hp, E, Ep, NNmax, Lmax, TL, TB;
  __device__ __forceinline__ long long node(int s, int n) const { return (long long)s * NNmax + n; }
  __device__ __forceinline__ long long leaf(int s, int l) const { return (long long)s * Lmax + l; }
};

__device__ __forceinline__ TreeBufs tree_bufs(const GQ AmpDev* D) {
  TreeBufs b;
  b.xin = uni_gq<float>(D->buf[0]);
  b.hc = uni_gq<float>(D->buf[1]);
  b.gate = uni_gq<float>(D->buf[2]);
  b.gout = uni_gq<float>(D->buf[3]);
  b.gpar = uni_gq<float>(D->buf[4]);
  b.gc = uni_gq<float>(D->buf[5]);
  b.gx = uni_gq<float>(D->buf[6]);
  b.cnt = uni_gq<int>(D->buf[7]);
  b.H = uni(D->hidden);
  b.Hp = amp_round4(b.H);
  b.E = uni(D->emb);
  b.Ep = amp_round4(b.E);
  b.Lmax = uni(D->max_len);
  b.NNmax = 2 * b.Lmax - 1;
  b.TL = uni(D->tiles_leaf);
  b.TB = uni(D->tiles_branch);
  return b;
}

// Ring numbers of the tree model.
#define TR_LOOKUP 1
#define TR_LEAF 2
#define TR_BRANCH 3
#define TR_OUT 4

__device__ __forceinline__ bool code_is_b(unsigned c) { return (c & MSG_DIR_B) != 0; }

// What a worker keeps of its descriptor and of the rings it posts to, read once (into scalar registers).
struct WorkerRegs {
  int node, tile, ntiles, kb, train;
  unsigned log_cap;
  GQ unsigned long long* log;
  Ring ctl, lookup, leaf, branch, out;   // the tree model's rings
};

__device__ __forceinline__ WorkerRegs worker_regs(const GQ AmpDev* D, const GQ WorkerDev* W) {
  WorkerRegs w;
  w.node = uni(W->node);
  w.tile = uni(W->tile);
  w.ntiles = uni(W->ntiles);
  w.kb = uni(W->kb);
  w.train = uni(D->train);
  w.log_cap = uni(W->log_cap);
  w.log = uni_gq<unsigned long long>(W->log);
  w.ctl = ring_regs(D, 0);
  w.lookup = ring_regs(D, 1);
  w.leaf = ring_regs(D, 2);
  w.branch = ring_regs(D, 3);
  w.out = ring_regs(D, 4);
  return w;
}


// What the controller wrote for slot s at admission: admission number, leaves, node offset, token offset.
__device__ __forceinline__ v4i tree_slot(const GQ int* smeta, int s) { return *(const GQ v4i*)(smeta + 4 * s); }
// left, right, parent * 2 + side (-1 for the root), label of node n of the instance whose nodes start at noff
__device__ __forceinline__ v4i tree_node(const GQ int* tnode, int noff, int n) {
  return *(const GQ v4i*)(tnode + 4 * (long long)(noff + n));
}

// One wave, all 64 lanes (k = lane), after lanes k < n have written M.aux[k]: positions
// of the batch's forward and backward messages, and the event record (tile 0 only).
__device__ __forceinline__ void batch_split_and_log(const GQ AmpDev* D, const WorkerRegs& W, BatchMsg& M, int n, int node,
                                                    bool both_kinds) {
  const int k = threadIdx.x & 63;
  const bool in = k < n, isb = in && M.aux[k] != 0;
  const unsigned long long mb = __ballot(isb), mf = __ballot(in && !isb);
  const unsigned long long lt = (1ull << k) - 1ull;
  if (isb) M.bidx[__popcll(mb & lt)] = k;
  if (in && !isb) M.fidx[__popcll(mf & lt)] = k;
  if (k == 0) {
    M.nF = __popcll(mf);
    M.nB = __popcll(mb);
  }
  if (W.log_cap && W.tile == 0) {
    // both_kinds: every message is a forward event followed by a backward event (output layer in training)
    const unsigned per = both_kinds ? 2u : 1u, base = s_logn;
    if (base + per * (unsigned)n > W.log_cap) {
      if (k == 0) raise_abort(D, ABORT_LOG_FULL, blockIdx.x);
    } else {
      if (in) {
        const unsigned long long tail = ((unsigned long long)M.seq[k] << 32) | ((unsigned)node << 20) | ((unsigned)M.n[k] & 0xfffffu);
        if (both_kinds) {
          W.log[base + 2 * k] = tail;
          W.log[base + 2 * k + 1] = tail | (1ull << 28);
        } else {
          W.log[base + k] = tail | ((unsigned long long)(isb ? 1 : 0) << 28);
        }
      }
      if (k == 0) s_logn = base + per * (unsigned)n;
    }
  }
}

// A tile has finished its units of node n: when all tiles have, the node's
// [h; c] goes to the output layer and, through Isu / Concat, to its parent,
// which fires once both children are there.  One lane, after a release fence.
__device__ __forceinline__ void tree_node_part_done(const WorkerRegs& W, const TreeBufs& B, int s, int n, int parent_code) {
  GQ int* c = B.cnt + B.node(s, n) * 4;
  if (!join_arrive(c + 0, W.ntiles)) return;
  ring_post(W.out, MSG_MAKE(0, s, n));
  if (parent_code < 0) return;
  const int p = parent_code >> 1;
  if (join_arrive(B.cnt + B.node(s, p) * 4 + 1, 2)) ring_post(W.branch, MSG_MAKE(0, s, p));
}

// One gradient part for node n has been written: Bcast's backward waits for
// the output layer's part and (unless n is the root) every parent tile's.
__device__ __forceinline__ void tree_grad_part_done(const WorkerRegs& W, const TreeBufs& B, int s, int n, bool is_root, bool is_leaf) {
  const int expect = is_root ? 1 : 1 + B.TB;
  if (join_arrive(B.cnt + B.node(s, n) * 4 + 2, expect)) {
    if (is_leaf)
      ring_post(W.leaf, MSG_MAKE(1, s, n));
    else
      ring_post(W.branch, MSG_MAKE(1, s, n));
  }
}

// ------------------------------------------------------------ lookup
__device__ __noinline__ void role_tree_lookup(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& lk = D->node[0];
  const TreeBufs B = tree_bufs(D);
  const WorkerRegs wr = worker_regs(D, W);
  const int E = B.E, Ep = B.Ep, KB = wr.kb, E4 = E >> 2, lk_muf = uni(lk.muf);
  const GQ int* smeta = uni_gq<int>(D->smeta);
  int* left_cnt = (int*)lds;                  // [mak] leaves not yet answered
  int* pend_tok = left_cnt + ((D->mak + 3) & ~3);
  for (int i = threadIdx.x; i < D->mak; i += AMP_THREADS) left_cnt[i] = 0;
  BatchMsg& M = s_M;
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  GQ int* keep = (GQ int*)D->buf[10];
  GQ float* prow = (GQ float*)D->buf[11];
  GQ float* lkP = (GQ float*)lk.P;
  const GQ int* tokens = (const GQ int*)D->data.tok;
  GQ float* probe = uni_gq<float>(D->probe);
  GQ unsigned* probe_n = uni_gq<unsigned>(D->probe_n);
  const unsigned probe_period = uni(D->probe_period), probe_cap = uni(D->probe_cap);
  const int probe_w = uni(D->probe_w);
  for (unsigned k = threadIdx.x; k < count; k += AMP_THREADS) pend_tok[k] = keep[k];
  __syncthreads();
  // Wave 1 takes and decodes the next batch while wave 0 is still publishing the present one (wave 0 keeps what its
  // posts need in registers, so the batch's LDS record is free from the publish barrier on).
  const int wave = threadIdx.x >> 6;
  auto take_batch = [&](int room) {
    const int n = poll_batch(D, mine, head, KB, room, s_codes, &s_n, code_is_b);
    if (n > 0) {
      const int k = threadIdx.x & 63;
      if (k < n) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), l = MSG_LOCAL(code);
        const v4i sm = tree_slot(smeta, s);
        M.s[k] = s;
        M.n[k] = l;
        M.seq[k] = (unsigned)sm.x;
        M.a[k] = tokens[sm.w + l];
        M.aux[k] = code_is_b(code);
        if (!code_is_b(code) && l == 0) left_cnt[s] = sm.y;
        // probe: the gradient w.r.t. this leaf's embedding (the leaf cell's backward output) of a sampled instance
        int entry = -1;
        if (probe_period && code_is_b(code) && (unsigned)sm.x % probe_period == 0u) {
          const unsigned e = __hip_atomic_fetch_add(probe_n, 1u, __ATOMIC_RELAXED, AGENT);
          if (e < probe_cap) {
            entry = (int)e;
            GQ int* hdr = (GQ int*)(probe + (long long)e * probe_w);
            hdr[0] = 1;
            hdr[1] = sm.x;
            hdr[2] = l;
            hdr[3] = 0;
          }
        }
        M.par[k] = entry;
      }
      batch_split_and_log(D, wr, M, n, 0, false);
      // backward message k is the b-th gradient of the batch: remember its token
      const bool isb = k < n && M.aux[k] != 0;
      const unsigned long long mb = __ballot(isb);
      if (isb) {
        const int b = __popcll(mb & ((1ull << k) - 1ull));
        M.b[k] = b;
        pend_tok[count + b] = M.a[k];
      }
    }
  };
  if (wave == 1) take_batch(lk_muf - (int)count);
  lds_barrier();
  for (;;) {
    const int n = s_n;
    if (n == 0) break;
    head += n;
    const int nB = M.nB;
    if ((E & 3) == 0) {
      // forward: table row -> xin; backward: sum of the leaf tiles' partials -> pending gradient row
      for (int idx = threadIdx.x; idx < n * E4; idx += AMP_THREADS) {
        const int k = idx / E4, c = (idx - k * E4) << 2;
        if (!M.aux[k]) {
          *(GQ v4f*)(B.xin + B.leaf(M.s[k], M.n[k]) * Ep + c) = *(const GQ v4f*)(lkP + (long long)M.a[k] * E + c);
        } else {
          const GQ float* gx = B.gx + B.leaf(M.s[k], M.n[k]) * B.TL * Ep + c;
          v4f a = {0.f, 0.f, 0.f, 0.f};
          for (int t0 = 0; t0 < B.TL; t0 += 16) {   // sixteen parts in flight at a time, added in tile order
            v4f p[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) p[u] = *(const GQ v4f*)(gx + (t0 + u < B.TL ? t0 + u : B.TL - 1) * Ep);
#pragma unroll
            for (int u = 0; u < 16; ++u)
              if (t0 + u < B.TL) a += p[u];
          }
          *(GQ v4f*)(prow + (long long)(count + M.b[k]) * E + c) = a;
          if (M.par[k] >= 0) *(GQ v4f*)(probe + (long long)M.par[k] * probe_w + 4 + c) = a;
        }
      }
    } else {
      for (int idx = threadIdx.x; idx < n * E; idx += AMP_THREADS) {
        const int k = idx / E, c = idx - k * E;
        if (!M.aux[k]) {
          B.xin[B.leaf(M.s[k], M.n[k]) * Ep + c] = lkP[(long long)M.a[k] * E + c];
        } else {
          const GQ float* gx = B.gx + B.leaf(M.s[k], M.n[k]) * B.TL * Ep + c;
          float a = 0.f;
          for (int t = 0; t < B.TL; ++t) a += gx[t * Ep];
          prow[(long long)(count + M.b[k]) * E + c] = a;
          if (M.par[k] >= 0) probe[(long long)M.par[k] * probe_w + 4 + c] = a;
        }
      }
    }
    // what lane k of wave 0 needs of message k for its post, before the batch's record is given up
    int js = 0, jn = 0, jaux = 0;
    if (threadIdx.x < 64 && (int)threadIdx.x < n) {
      js = M.s[threadIdx.x];
      jn = M.n[threadIdx.x];
      jaux = M.aux[threadIdx.x];
    }
    publish_barrier();
    if (threadIdx.x < 64) {
      fence_release();
      if ((int)threadIdx.x < n) {
        if (!jaux) {
          ring_post(wr.leaf, MSG_MAKE(0, js, jn));
        } else if (wr.train) {
          if (atomicSub(&left_cnt[js], 1) == 1) ring_post(wr.ctl, MSG_MAKE(1, js, 0));
        }
      }
    }
    count += nB;
    if ((int)count >= lk_muf) {
      // SGD on the touched rows: each waiting gradient row is subtracted from its
      // token's row, in arrival order (rows never touched have a zero gradient)
      tstep++;
      if (threadIdx.x == 0) note_update(D);
      const float sc = lk.lr * (lk.mean ? 1.f / (float)count : 1.f);
      __syncthreads();
      for (int c = threadIdx.x; c < E; c += AMP_THREADS) {
        for (unsigned k0 = 0; k0 < count; k0 += 16) {
          const int kc = count - k0 < 16u ? (int)(count - k0) : 16;
          float w[16], g[16];
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (k < kc) {
              w[k] = lkP[(long long)pend_tok[k0 + k] * E + c];
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
            if (k < kc) lkP[(long long)pend_tok[k0 + k] * E + c] = w[k];
        }
      }
      count = 0;
      lds_barrier();   // every wave has finished with the token list before wave 1 starts the next one
      // recorded by the wave that records the next batch's events, so that the update comes first
      if (threadIdx.x == 64) log_event(D, W, &s_logn, 0, 2, 0, 0);
    }
    if (wave == 1) take_batch(lk_muf - (int)count);
    lds_barrier();
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
  for (unsigned k = threadIdx.x; k < count; k += AMP_THREADS) keep[k] = pend_tok[k];
}

// ------------------------------------------------------------ matrix-core products of a cell tile
// The products are templates over the tile's shape -- NRBT 16-row blocks and
// NCGT 16-column groups, 0 = known only at run time -- because fixed trip
// counts and strides let the compiler unroll the loops, fold the LDS
// addresses into instruction offsets and keep every operand in registers.
// One wave issues at most one matrix instruction every ~32 clocks and needs
// four or more independent accumulators to get there, so the loops below are
// shaped to give every wave an equal share and several accumulators.
#define TREE_XG 20        // 16-column groups of the input held in registers at once
#define TREE_GU 4         // (16-row block, 64-column block) gradient units per wave

template <int NRBT, int NCGT>
struct TreeShape {
  int NRB, NCG, ldw, ldy;
  __device__ __forceinline__ TreeShape(const Tile& t) {
    NRB = NRBT ? NRBT : t.Rp >> 4;
    NCG = NCGT ? NCGT : amp_round16(t.Cl) >> 4;
    ldw = NCGT ? amp_ldrow(NCGT * 16) : t.ldw;
    ldy = NRBT ? amp_ldrow(NRBT * 16) : amp_ldrow(t.Rp);
  }
};

// Y[j][r] = b[r] + sum_c W[r][c] x_j[c] for the nF forward messages of the batch.
// A 16-message block is shared by 8 / (number of blocks) waves, each taking
// every wpn-th 16-row block of the weights.  A wave fetches its messages'
// inputs from HBM (xbase + M.off0 / off1 for the first / second column
// segment) once, straight into operand registers, and uses them for NJ (up to
// three) row blocks at a time.  Loads are unconditional so that they overlap:
// a column group beyond the input reads a valid address and is replaced by zero.
template <bool BR, int NJ, int NRBT, int NCGT>
__device__ __forceinline__ void tree_fwd_pass(const LDSQ float* Wl, const Tile& t, const LDSQ float* bl, const GQ float* p0,
                                              const GQ float* p1, int r0, int wpn, LDSQ float* yrow) {
  const TreeShape<NRBT, NCGT> sh(t);
  const int lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  constexpr int NA = NJ == 1 ? 4 : 2;   // accumulators per row block
  v4f acc[NJ][NA];
  const LDSQ float* wr[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
#pragma unroll
    for (int a = 0; a < NA; ++a) acc[j][a] = zero;
    wr[j] = Wl + ((r0 + j * wpn) * 16 + i) * sh.ldw + 4 * q;
  }
  for (int c0 = 0; c0 < sh.NCG; c0 += TREE_XG) {
    v4f x[TREE_XG];
#pragma unroll
    for (int g = 0; g < TREE_XG; ++g) {
      const int lc = (c0 + g) * 16 + 4 * q;
      const bool in = lc < t.Cl;
      const GQ float* p = in ? (BR && lc >= t.segp ? p1 : p0) + (c0 + g) * 16 : p0;
      const v4f v = *(const GQ v4f*)p;
      x[g] = in ? v : zero;
    }
    // all fetches are in flight before the first product waits for one
    asm volatile("" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]),
                      "+v"(x[8]), "+v"(x[9]), "+v"(x[10]), "+v"(x[11]), "+v"(x[12]), "+v"(x[13]), "+v"(x[14]),
                      "+v"(x[15]), "+v"(x[16]), "+v"(x[17]), "+v"(x[18]), "+v"(x[19]));
#pragma unroll
    for (int g = 0; g < TREE_XG; ++g) {
      if (NCGT ? g < NCGT : c0 + g < sh.NCG) {
        v4f w[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) w[j] = *(const LDSQ v4f*)(wr[j] + 16 * (c0 + g));
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          acc[j][0] = MFMA(w[j].x, x[g].x, acc[j][0]);
          acc[j][1] = MFMA(w[j].y, x[g].y, acc[j][1]);
        }
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          acc[j][NA == 4 ? 2 : 0] = MFMA(w[j].z, x[g].z, acc[j][NA == 4 ? 2 : 0]);
          acc[j][NA == 4 ? 3 : 1] = MFMA(w[j].w, x[g].w, acc[j][NA == 4 ? 3 : 1]);
        }
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int rb = r0 + j * wpn;
    v4f r = *(const LDSQ v4f*)(bl + rb * 16 + 4 * q);
#pragma unroll
    for (int a = 0; a < NA; ++a) r += acc[j][a];
    *(LDSQ v4f*)(yrow + rb * 16 + 4 * q) = r;
  }
}

template <bool BR, int NRBT, int NCGT>
__device__ __forceinline__ void tree_fwd_mfma(const LDSQ float* Wl, const Tile& t, const LDSQ float* bl, const GQ float* xbase,
                                              const BatchMsg& M, int nF, LDSQ float* Y) {
  const TreeShape<NRBT, NCGT> sh(t);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NBF = (nF + 15) >> 4;
  const int wpn = NBF == 1 ? 8 : NBF == 2 ? 4 : 2;
  // waves w and w + 4 share a SIMD: rotating the row-block offset with the message block evens out the
  // number of row blocks per SIMD when the blocks do not divide evenly among a block's waves
  const int nb = wave / wpn, sub = (wave - nb * wpn + (wpn >> 1) * (nb & 1)) % wpn;
  if (nb >= NBF) return;
  int mi = nb * 16 + i;
  if (mi > nF - 1) mi = nF - 1;   // rows beyond the batch repeat its last message; their results are dropped
  const int m = M.fidx[mi];
  const GQ float* p0 = xbase + M.off0[m] + 4 * q;
  const GQ float* p1 = xbase + M.off1[m] + 4 * q - t.segp;
  LDSQ float* yrow = Y + (nb * 16 + i) * sh.ldy;
  for (int r0 = sub; r0 < sh.NRB; r0 += 3 * wpn) {
    const int left = (sh.NRB - r0 + wpn - 1) / wpn;   // row blocks r0, r0 + wpn, ... still to do
    if (left >= 3)
      tree_fwd_pass<BR, 3, NRBT, NCGT>(Wl, t, bl, p0, p1, r0, wpn, yrow);
    else if (left == 2)
      tree_fwd_pass<BR, 2, NRBT, NCGT>(Wl, t, bl, p0, p1, r0, wpn, yrow);
    else
      tree_fwd_pass<BR, 1, NRBT, NCGT>(Wl, t, bl, p0, p1, r0, wpn, yrow);
  }
}

// dx_j[c] = sum_r W[r][c] delta_j[r] for the nB backward messages; delta rows
// in LDS (Dl, zero beyond the tile's rows); the result goes from the
// accumulators to HBM at obase + M.dst0 / dst1 (+ column inside the
// segment).  Wave item = 16 weight columns, for all NBB message blocks.
template <bool BR, int NBB, int NRBT, int NCGT>
__device__ __forceinline__ void tree_bwd_blocks(const LDSQ float* Wl, const Tile& t, const LDSQ float* Dl, const BatchMsg& M,
                                                int nB, GQ float* obase) {
  const TreeShape<NRBT, NCGT> sh(t);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  constexpr int NA = NBB == 1 ? 4 : 2;
  for (int cb = wave; cb < sh.NCG; cb += AMP_THREADS / 64) {
    const LDSQ float* wp = Wl + (4 * q) * sh.ldw + cb * 16 + i;
    const LDSQ float* dp = Dl + i * sh.ldy + 4 * q;
    v4f acc[NBB][NA];
#pragma unroll
    for (int nb = 0; nb < NBB; ++nb)
#pragma unroll
      for (int a = 0; a < NA; ++a) acc[nb][a] = zero;
#pragma unroll 6
    for (int g = 0; g < sh.NRB; ++g) {
      v4f d[NBB];
#pragma unroll
      for (int nb = 0; nb < NBB; ++nb) d[nb] = *(const LDSQ v4f*)(dp + nb * 16 * sh.ldy + 16 * g);
      const LDSQ float* w = wp + 16 * g * sh.ldw;
      const float a0 = w[0], a1 = w[sh.ldw], a2 = w[2 * sh.ldw], a3 = w[3 * sh.ldw];
#pragma unroll
      for (int nb = 0; nb < NBB; ++nb) {
        acc[nb][0] = MFMA(a0, d[nb].x, acc[nb][0]);
        acc[nb][1] = MFMA(a1, d[nb].y, acc[nb][1]);
      }
#pragma unroll
      for (int nb = 0; nb < NBB; ++nb) {
        acc[nb][NA == 4 ? 2 : 0] = MFMA(a2, d[nb].z, acc[nb][NA == 4 ? 2 : 0]);
        acc[nb][NA == 4 ? 3 : 1] = MFMA(a3, d[nb].w, acc[nb][NA == 4 ? 3 : 1]);
      }
    }
    const int lc = cb * 16 + 4 * q;
#pragma unroll
    for (int nb = 0; nb < NBB; ++nb) {
      const int mi = nb * 16 + i;
      if (mi < nB && lc < t.Cl) {
        const int m = M.bidx[mi];
        GQ float* o = (BR && lc >= t.segp) ? obase + M.dst1[m] + (lc - t.segp) : obase + M.dst0[m] + lc;
        v4f r = acc[nb][0] + acc[nb][1];
        if (NA == 4) r += acc[nb][2] + acc[nb][3];
        *(GQ v4f*)o = r;
      }
    }
  }
}

template <bool BR, int NRBT, int NCGT>
__device__ __forceinline__ void tree_bwd_mfma(const LDSQ float* Wl, const Tile& t, const LDSQ float* Dl, const BatchMsg& M,
                                              int nB, GQ float* obase) {
  const int NBB = (nB + 15) >> 4;
  if (NBB == 1)
    tree_bwd_blocks<BR, 1, NRBT, NCGT>(Wl, t, Dl, M, nB, obase);
  else if (NBB == 2)
    tree_bwd_blocks<BR, 2, NRBT, NCGT>(Wl, t, Dl, M, nB, obase);
  else if (NBB == 3)
    tree_bwd_blocks<BR, 3, NRBT, NCGT>(Wl, t, Dl, M, nB, obase);
  else
    tree_bwd_blocks<BR, 4, NRBT, NCGT>(Wl, t, Dl, M, nB, obase);
}

// The optimizer step on the LDS weights from the accumulators of tree_update_from_pend (layout described there).
template <int NRBT, int NCGT>
__device__ __forceinline__ void tree_update_apply(LDSQ float* Wl, LDSQ float* bl, const GQ NodeDev& nd, const Tile& t,
                                                  const TreeShape<NRBT, NCGT>& sh, v4f (&g)[TREE_GU][4], unsigned n_grad,
                                                  unsigned tstep, const LDSQ int* rowmap, const LDSQ int* colmap, float gb) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = sh.NRB, Cp = sh.NCG * 16, CM = (Cp + 63) >> 6, NU = NRB * CM;
  const OptCoef o = opt_coef(nd, tstep);
  const float inv = nd.mean ? 1.f / (float)n_grad : 1.f;
  // optimizer step from the accumulators.  Plain SGD needs no per-element slots: padding rows and columns
  // have a zero gradient (their delta / input entries are zero), so whole 16-byte groups are updated.
  if (o.kind == 0) {
    const float sc = o.lr * inv;
#pragma unroll
    for (int u = 0; u < TREE_GU; ++u) {
      const int id = wave + 8 * u, cm = id / NRB, rb = id - cm * NRB, lc = cm * 64 + 4 * i;
      if (id < NU && lc < Cp) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          LDSQ v4f* wp = (LDSQ v4f*)(Wl + (rb * 16 + 4 * q + e) * sh.ldw + lc);
          const v4f gv = {g[u][0][e], g[u][1][e], g[u][2][e], g[u][3][e]};
          *wp = *wp - sc * gv;
        }
      }
    }
  } else {
    // momentum / Adam: the slots are in HBM.  A unit's sixteen elements per lane are fetched together, then stepped,
    // then stored (a fetch behind the previous element's stores would wait for them).
    GQ float* Mq = (GQ float*)nd.M;
    GQ float* Vq = (GQ float*)nd.V;
#pragma unroll
    for (int u = 0; u < TREE_GU; ++u) {
      const int id = wave + 8 * u, cm = id / NRB, rb = id - cm * NRB;
      if (id < NU) {
        long long gi[4][4];
        float mo[4][4], vo[4][4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int nc = colmap[cm * 64 + 4 * i + v];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int nr = rowmap[rb * 16 + 4 * q + e];
            gi[v][e] = (nr >= 0 && nc >= 0) ? (long long)nr * t.C + nc : -1;
            const long long at = gi[v][e] >= 0 ? gi[v][e] : 0;
            mo[v][e] = Mq[at];
            vo[v][e] = o.kind == 2 ? Vq[at] : 0.f;
          }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int lc = cm * 64 + 4 * i + v;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (gi[v][e] >= 0) {
              const int r = rb * 16 + 4 * q + e;
              const float gr = g[u][v][e] * inv, w = Wl[r * sh.ldw + lc];
              if (o.kind == 1) {
                const float m = fmaf(o.mom, mo[v][e], gr);
                Mq[gi[v][e]] = m;
                Wl[r * sh.ldw + lc] = w - o.lr * m;
              } else {
                const float m = fmaf(o.b1, mo[v][e], (1.f - o.b1) * gr);
                const float vv = fmaf(o.b2, vo[v][e], (1.f - o.b2) * gr * gr);
                Mq[gi[v][e]] = m;
                Vq[gi[v][e]] = vv;
                Wl[r * sh.ldw + lc] = w - o.lr * (m * o.c1) / (sqrtf(vv * o.c2) + o.eps);
              }
            }
        }
      }
    }
  }
  if ((int)threadIdx.x < t.R && nd.has_bias) {
    const int r = threadIdx.x;
    bl[r] = opt_apply(o, bl[r], gb * inv, nd.M, nd.V, (long long)nd.rows * t.C + rowmap[r]);
  }
}

// The node's update (Section 3) for one tile, from the `count` pending
// (delta, input) pairs in HBM, entry k at pend + k * stride = [delta (Rp) |
// input in LDS column layout (Cp)]:  G[r][c] = sum_k delta_k[r] x_k[c] in
// arrival order, formed on the matrix cores with the pairs fetched straight
// into operand registers, then the optimizer step on the LDS weights.
// Unit u of a wave is the (16-row block rb, 64-column block cm) with
// rb + NRB * cm = wave + 8 u; its four 16 x 16 tiles take the columns
// cm * 64 + 4 i + v, v = 0..3, so that one 16-byte fetch of an input feeds all
// four.  Lane (i, q) ends up with G[rb*16 + 4q + e][cm*64 + 4i + v] in g[u][v][e].
// gb = the accumulated bias gradient of tile row threadIdx.x; n_grad = the
// number of gradients (messages) behind the count pending rows.
template <int NRBT, int NCGT>
__device__ __noinline__ void tree_update_from_pend(LDSQ float* Wl, LDSQ float* bl, const GQ NodeDev* ndp, Tile t,
                                                   const GQ float* pend, unsigned count, unsigned n_grad, unsigned tstep,
                                                   const LDSQ int* rowmap, const LDSQ int* colmap, float gb) {
  const TreeShape<NRBT, NCGT> sh(t);
  const GQ NodeDev& nd = *ndp;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = sh.NRB, Rp = NRB * 16, Cp = sh.NCG * 16, stride = Rp + Cp, CM = (Cp + 63) >> 6, NU = NRB * CM;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  v4f g[TREE_GU][4];
  int aoff[TREE_GU], xoff[TREE_GU];
  bool xin[TREE_GU];
#pragma unroll
  for (int u = 0; u < TREE_GU; ++u) {
    const int id = wave + 8 * u < NU ? wave + 8 * u : 0, cm = id / NRB, rb = id - cm * NRB, lc = cm * 64 + 4 * i;
    aoff[u] = rb * 16 + i;
    xin[u] = lc < Cp;
    xoff[u] = Rp + (xin[u] ? lc : 0);
#pragma unroll
    for (int v = 0; v < 4; ++v) g[u][v] = zero;
  }
  constexpr int NH = 4;
  for (unsigned k0 = 0; k0 < count; k0 += 4 * NH) {
    // NH groups of four pending pairs per round, all fetches in flight together
    float a[NH][TREE_GU];
    v4f x[NH][TREE_GU];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const unsigned k = k0 + 4 * h + q;
      const bool kin = k < count;
      const GQ float* e = pend + (long long)(kin ? k : count - 1) * stride;
#pragma unroll
      for (int u = 0; u < TREE_GU; ++u) {
        const float av = e[aoff[u]];
        const v4f xv = *(const GQ v4f*)(e + xoff[u]);
        a[h][u] = kin ? av : 0.f;
        x[h][u] = xin[u] ? xv : zero;
      }
    }
    asm volatile("" : "+v"(x[0][0]), "+v"(x[0][1]), "+v"(x[0][2]), "+v"(x[0][3]), "+v"(x[1][0]), "+v"(x[1][1]), "+v"(x[1][2]),
                      "+v"(x[1][3]), "+v"(x[2][0]), "+v"(x[2][1]), "+v"(x[2][2]), "+v"(x[2][3]), "+v"(x[3][0]), "+v"(x[3][1]),
                      "+v"(x[3][2]), "+v"(x[3][3]));
#pragma unroll
    for (int h = 0; h < NH; ++h)
#pragma unroll
      for (int u = 0; u < TREE_GU; ++u)
        if (wave + 8 * u < NU) {
          g[u][0] = MFMA(a[h][u], x[h][u].x, g[u][0]);
          g[u][1] = MFMA(a[h][u], x[h][u].y, g[u][1]);
          g[u][2] = MFMA(a[h][u], x[h][u].z, g[u][2]);
          g[u][3] = MFMA(a[h][u], x[h][u].w, g[u][3]);
        }
  }
  tree_update_apply<NRBT, NCGT>(Wl, bl, nd, t, sh, g, n_grad, tstep, rowmap, colmap, gb);
}

// ------------------------------------------------------------ products of a tile whose weights stay in HBM
// For cells too large for the CUs' LDS (hidden size 1024: 12.6 MB and 41.9 MB
// of weights) a tile keeps no copy of its rows: the products read them from
// the node's parameter array (rows x cols, row-major, cols a multiple of 4) in
// HBM / L2 as they go, and the update writes them back in place.  rowoff[lr] =
// (node row of tile row lr) * cols, row 0 for the padding rows of the last
// 16-row block, whose results are dropped or meet a zero delta.

// Y[j][r] = b[r] + sum_c W[r][c] x_j[c] as a K-chunked product: the batch's inputs go through LDS 64 columns
// at a time (Xs, two buffers of kb rows x 68 floats, fetched once per chunk by the whole workgroup), every wave
// owns up to three 16-row blocks of the weights for all message blocks, and both the next chunk's inputs and the
// next chunk's weight rows are fetched while the matrix cores work on the present chunk.
#define TREE_XC 64        // columns per chunk
#define TREE_XS (TREE_XC + 4)

// NJ = 16-row blocks a wave owns in this pass (blocks r0 + wave, + 8, ...); a wave whose last block lies beyond the
// tile skips that block's fetches and products.
template <bool BR, int NBF, int NJ>
__device__ __forceinline__ void tree_fwd_stream_pass(const GQ float* P, const LDSQ int* rowoff, const Tile& t,
                                                     const LDSQ float* bl, const GQ float* xbase, const BatchMsg& M, int nF,
                                                     LDSQ float* Y, int ldy, LDSQ float* Xs, int r0) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = t.Rp >> 4, NCH = (t.Cl + TREE_XC - 1) / TREE_XC;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  constexpr int NX = NBF > 2 ? 2 : 1;   // staging passes of 32 messages
  // staging role of this thread: message row sm (+ 32 per pass), 16-byte piece sp of the chunk
  const int sm = threadIdx.x >> 4, sp = (threadIdx.x & 15) << 2;
  const GQ float* xp0[NX];
  const GQ float* xp1[NX];
#pragma unroll
  for (int a = 0; a < NX; ++a) {
    int mi = sm + 32 * a;
    if (mi > nF - 1) mi = nF - 1;   // rows beyond the batch repeat its last message; their results are dropped
    const int m = M.fidx[mi];
    xp0[a] = xbase + M.off0[m] + sp;
    xp1[a] = xbase + M.off1[m] + sp - t.segp;
  }
  auto xfetch = [&](int ch, int a) -> v4f {
    const int lc = ch * TREE_XC + sp;
    const bool in = lc < t.Cl;
    const v4f v = *(const GQ v4f*)(in ? (BR && lc >= t.segp ? xp1[a] : xp0[a]) + ch * TREE_XC : xp0[a]);
    return in ? v : zero;
  };
  {
    // this wave's row blocks: r0 + wave, + 8, ...; only the last can lie beyond the tile
    const bool last_in = r0 + wave + 8 * (NJ - 1) < NRB;
    const GQ float* wrow[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int rb = r0 + wave + 8 * j < NRB ? r0 + wave + 8 * j : NRB - 1;
      wrow[j] = P + rowoff[rb * 16 + i] + 4 * q;
    }
    auto wfetch = [&](int ch, int j, int g) -> v4f {
      const int lc = ch * TREE_XC + g * 16 + 4 * q;
      return *(const GQ v4f*)(lc < t.Cl ? wrow[j] + ch * TREE_XC + g * 16 : wrow[j]);   // beyond the input: x is zero
    };
    v4f acc[NJ][NBF];
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int nb = 0; nb < NBF; ++nb) acc[j][nb] = zero;
    v4f wa[NJ][4], wb[NJ][4], xr[NX];
    // prologue: chunk 0
#pragma unroll
    for (int a = 0; a < NX; ++a) xr[a] = xfetch(0, a);
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) wa[j][g] = (j < NJ - 1 || last_in) ? wfetch(0, j, g) : zero;
    lds_barrier();   // the previous pass has finished with Xs
#pragma unroll
    for (int a = 0; a < NX; ++a) *(LDSQ v4f*)(Xs + (sm + 32 * a) * TREE_XS + sp) = xr[a];
    lds_barrier();
    for (int ch = 0; ch < NCH; ch += 2) {
      // ---- even chunk: operands wa, Xs buffer 0; fetch chunk ch + 1 into wb / xr
#pragma unroll
      for (int a = 0; a < NX; ++a) xr[a] = xfetch(ch + 1, a);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) wb[j][g] = (j < NJ - 1 || last_in) ? wfetch(ch + 1, j, g) : zero;
      asm volatile("" ::: "memory");   // the fetches are issued before the products below start
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        v4f x[NBF];
#pragma unroll
        for (int nb = 0; nb < NBF; ++nb) x[nb] = *(const LDSQ v4f*)(Xs + (nb * 16 + i) * TREE_XS + g * 16 + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e)   // component-major: consecutive products go to different accumulators
#pragma unroll
          for (int j = 0; j < NJ - 1; ++j)
#pragma unroll
            for (int nb = 0; nb < NBF; ++nb) acc[j][nb] = MFMA(wa[j][g][e], x[nb][e], acc[j][nb]);
        if (last_in) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int nb = 0; nb < NBF; ++nb) acc[NJ - 1][nb] = MFMA(wa[NJ - 1][g][e], x[nb][e], acc[NJ - 1][nb]);
        }
      }
#pragma unroll
      for (int a = 0; a < NX; ++a) *(LDSQ v4f*)(Xs + 64 * TREE_XS + (sm + 32 * a) * TREE_XS + sp) = xr[a];
      lds_barrier();
      if (ch + 1 >= NCH) break;
      // ---- odd chunk: operands wb, Xs buffer 1; fetch chunk ch + 2 into wa / xr
#pragma unroll
      for (int a = 0; a < NX; ++a) xr[a] = xfetch(ch + 2, a);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) wa[j][g] = (j < NJ - 1 || last_in) ? wfetch(ch + 2, j, g) : zero;
      asm volatile("" ::: "memory");
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        v4f x[NBF];
#pragma unroll
        for (int nb = 0; nb < NBF; ++nb)
          x[nb] = *(const LDSQ v4f*)(Xs + 64 * TREE_XS + (nb * 16 + i) * TREE_XS + g * 16 + 4 * q);
#pragma unroll
        for (int e = 0; e < 4; ++e)   // component-major: consecutive products go to different accumulators
#pragma unroll
          for (int j = 0; j < NJ - 1; ++j)
#pragma unroll
            for (int nb = 0; nb < NBF; ++nb) acc[j][nb] = MFMA(wb[j][g][e], x[nb][e], acc[j][nb]);
        if (last_in) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int nb = 0; nb < NBF; ++nb) acc[NJ - 1][nb] = MFMA(wb[NJ - 1][g][e], x[nb][e], acc[NJ - 1][nb]);
        }
      }
#pragma unroll
      for (int a = 0; a < NX; ++a) *(LDSQ v4f*)(Xs + (sm + 32 * a) * TREE_XS + sp) = xr[a];
      lds_barrier();
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int rb = r0 + wave + 8 * j;
      if (rb < NRB) {
        const v4f b4 = *(const LDSQ v4f*)(bl + rb * 16 + 4 * q);
#pragma unroll
        for (int nb = 0; nb < NBF; ++nb) *(LDSQ v4f*)(Y + (nb * 16 + i) * ldy + rb * 16 + 4 * q) = acc[j][nb] + b4;
      }
    }
  }
}

template <bool BR, int NBF>
__device__ __forceinline__ void tree_fwd_stream_blocks(const GQ float* P, const LDSQ int* rowoff, const Tile& t,
                                                       const LDSQ float* bl, const GQ float* xbase, const BatchMsg& M, int nF,
                                                       LDSQ float* Y, int ldy, LDSQ float* Xs) {
  const int NRB = t.Rp >> 4;
  for (int r0 = 0; r0 < NRB; r0 += 24) {
    const int left = NRB - r0;
    if (left > 16)
      tree_fwd_stream_pass<BR, NBF, 3>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs, r0);
    else if (left > 8)
      tree_fwd_stream_pass<BR, NBF, 2>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs, r0);
    else
      tree_fwd_stream_pass<BR, NBF, 1>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs, r0);
  }
}

template <bool BR>
__device__ __forceinline__ void tree_fwd_stream(const GQ float* P, const LDSQ int* rowoff, const Tile& t, const LDSQ float* bl,
                                                const GQ float* xbase, const BatchMsg& M, int nF, LDSQ float* Y, int ldy,
                                                LDSQ float* Xs) {
  const int NBF = (nF + 15) >> 4;
  if (NBF == 1)
    tree_fwd_stream_blocks<BR, 1>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs);
  else if (NBF == 2)
    tree_fwd_stream_blocks<BR, 2>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs);
  else if (NBF == 3)
    tree_fwd_stream_blocks<BR, 3>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs);
  else
    tree_fwd_stream_blocks<BR, 4>(P, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs);
}

// dx_j[c] = sum_r W[r][c] delta_j[r].  A wave owns every 8th block of 64 weight columns for all NBB message
// blocks.  For a (16-row block, 64-column block) unit lane (i, q) fetches rows 4q .. 4q+3 of the block at columns
// 4i .. 4i+3 -- 16 bytes per fetch, 256 contiguous bytes per row across the 16 lanes -- and component e of those
// fetches is the weight operand of output tile e, whose 16 columns are 4m + e: one fetch feeds four products, and
// a lane ends up with 16 consecutive columns of its message's input gradient.  The rows are walked TREE_SR blocks
// at a time with two register buffers, the next stretch in flight while the matrix cores work on the present one.
#define TREE_SR 4
template <bool BR, int NBB>
__device__ __forceinline__ void tree_bwd_stream_blocks(const GQ float* P, const LDSQ int* rowoff, const Tile& t,
                                                       const LDSQ float* Dl, int ldd, const BatchMsg& M, int nB, GQ float* obase) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = t.Rp >> 4, CM = (amp_round16(t.Cl) + 63) >> 6;
  const int NGC = (NRB + TREE_SR - 1) / TREE_SR;                 // row stretches per column block
  const int ncb = wave < CM ? (CM - wave + 7) >> 3 : 0;           // column blocks of this wave
  const int T = ncb * NGC;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  const LDSQ float* dp = Dl + i * ldd + 4 * q;
  auto afetch = [&](int it, v4f (&a)[TREE_SR][4]) {
    const int cb = wave + 8 * (it / NGC), g0 = (it % NGC) * TREE_SR;
    const int col = cb * 64 + 4 * i < t.Cl ? cb * 64 + 4 * i : 0;
#pragma unroll
    for (int g = 0; g < TREE_SR; ++g) {
      const int gg = g0 + g < NRB ? g0 + g : NRB - 1;
#pragma unroll
      for (int sx = 0; sx < 4; ++sx) a[g][sx] = *(const GQ v4f*)(P + rowoff[gg * 16 + 4 * q + sx] + col);
    }
  };
  v4f acc[NBB][4];
#pragma unroll
  for (int nb = 0; nb < NBB; ++nb)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[nb][e] = zero;
  auto work = [&](int it, v4f (&a)[TREE_SR][4]) {
    const int cb = wave + 8 * (it / NGC), gc = it % NGC, g0 = gc * TREE_SR;
#pragma unroll
    for (int g = 0; g < TREE_SR; ++g)
      if (g0 + g < NRB) {
#pragma unroll
        for (int nb = 0; nb < NBB; ++nb) {
          const v4f d = *(const LDSQ v4f*)(dp + nb * 16 * ldd + 16 * (g0 + g));
#pragma unroll
          for (int sx = 0; sx < 4; ++sx)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[nb][e] = MFMA(a[g][sx][e], d[sx], acc[nb][e]);
        }
      }
    if (gc == NGC - 1) {
#pragma unroll
      for (int nb = 0; nb < NBB; ++nb) {
        const int mi = nb * 16 + i;
        if (mi < nB) {
          const int m = M.bidx[mi];
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int lc = cb * 64 + 16 * q + 4 * v;
            if (lc < t.Cl) {
              GQ float* o = (BR && lc >= t.segp) ? obase + M.dst1[m] + (lc - t.segp) : obase + M.dst0[m] + lc;
              *(GQ v4f*)o = (v4f){acc[nb][0][v], acc[nb][1][v], acc[nb][2][v], acc[nb][3][v]};
            }
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[nb][e] = zero;
      }
    }
  };
  v4f a0[TREE_SR][4], a1[TREE_SR][4];
  if (T > 0) afetch(0, a0);
  for (int it = 0; it < T; it += 2) {
    if (it + 1 < T) afetch(it + 1, a1);
    asm volatile("" ::: "memory");   // the fetches are issued before the products below start
    work(it, a0);
    if (it + 1 >= T) break;
    if (it + 2 < T) afetch(it + 2, a0);
    asm volatile("" ::: "memory");
    work(it + 1, a1);
  }
}

template <bool BR>
__device__ __forceinline__ void tree_bwd_stream(const GQ float* P, const LDSQ int* rowoff, const Tile& t, const LDSQ float* Dl,
                                                int ldd, const BatchMsg& M, int nB, GQ float* obase) {
  const int NBB = (nB + 15) >> 4;
  if (NBB == 1)
    tree_bwd_stream_blocks<BR, 1>(P, rowoff, t, Dl, ldd, M, nB, obase);
  else if (NBB == 2)
    tree_bwd_stream_blocks<BR, 2>(P, rowoff, t, Dl, ldd, M, nB, obase);
  else if (NBB == 3)
    tree_bwd_stream_blocks<BR, 3>(P, rowoff, t, Dl, ldd, M, nB, obase);
  else
    tree_bwd_stream_blocks<BR, 4>(P, rowoff, t, Dl, ldd, M, nB, obase);
}

// The update of a streamed tile: as tree_update_from_pend, in passes of 8 waves
// x TREE_GU (16-row, 64-column) units, each pass re-reading the pending list;
// the optimizer step goes to the parameter array in HBM.
__device__ __noinline__ void tree_update_stream(GQ float* P, LDSQ float* bl, const GQ NodeDev* ndp, Tile t, const GQ float* pend,
                                                unsigned count, unsigned tstep, const LDSQ int* rowmap, float gb) {
  const GQ NodeDev& nd = *ndp;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  const int NRB = t.Rp >> 4, Rp = t.Rp, Cp = amp_round16(t.Cl), stride = Rp + Cp, CM = (Cp + 63) >> 6, NU = NRB * CM;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  const OptCoef o = opt_coef(nd, tstep);
  const float inv = nd.mean ? 1.f / (float)count : 1.f;
  constexpr int NH = 4;
  for (int u0 = 0; u0 < NU; u0 += 8 * TREE_GU) {
    v4f g[TREE_GU][4];
    int aoff[TREE_GU], xoff[TREE_GU];
    bool xin[TREE_GU];
#pragma unroll
    for (int u = 0; u < TREE_GU; ++u) {
      const int id = u0 + wave + 8 * u < NU ? u0 + wave + 8 * u : 0, cm = id / NRB, rb = id - cm * NRB, lc = cm * 64 + 4 * i;
      aoff[u] = rb * 16 + i;
      xin[u] = lc < Cp;
      xoff[u] = Rp + (xin[u] ? lc : 0);
#pragma unroll
      for (int v = 0; v < 4; ++v) g[u][v] = zero;
    }
    for (unsigned k0 = 0; k0 < count; k0 += 4 * NH) {
      float a[NH][TREE_GU];
      v4f x[NH][TREE_GU];
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        const unsigned k = k0 + 4 * h + q;
        const bool kin = k < count;
        const GQ float* e = pend + (long long)(kin ? k : count - 1) * stride;
#pragma unroll
        for (int u = 0; u < TREE_GU; ++u) {
          const float av = e[aoff[u]];
          const v4f xv = *(const GQ v4f*)(e + xoff[u]);
          a[h][u] = kin ? av : 0.f;
          x[h][u] = xin[u] ? xv : zero;
        }
      }
      asm volatile("" : "+v"(x[0][0]), "+v"(x[0][1]), "+v"(x[0][2]), "+v"(x[0][3]), "+v"(x[1][0]), "+v"(x[1][1]), "+v"(x[1][2]),
                        "+v"(x[1][3]), "+v"(x[2][0]), "+v"(x[2][1]), "+v"(x[2][2]), "+v"(x[2][3]), "+v"(x[3][0]), "+v"(x[3][1]),
                        "+v"(x[3][2]), "+v"(x[3][3]));
#pragma unroll
      for (int h = 0; h < NH; ++h)
#pragma unroll
        for (int u = 0; u < TREE_GU; ++u) {
          g[u][0] = MFMA(a[h][u], x[h][u].x, g[u][0]);
          g[u][1] = MFMA(a[h][u], x[h][u].y, g[u][1]);
          g[u][2] = MFMA(a[h][u], x[h][u].z, g[u][2]);
          g[u][3] = MFMA(a[h][u], x[h][u].w, g[u][3]);
        }
    }
#pragma unroll
    for (int u = 0; u < TREE_GU; ++u) {
      const int id = u0 + wave + 8 * u, cm = id / NRB, rb = id - cm * NRB, lc = cm * 64 + 4 * i;
      if (id < NU && lc < t.Cl) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int nr = rowmap[rb * 16 + 4 * q + e];
          if (nr >= 0) {
            const long long gi = (long long)nr * t.C + lc;
            GQ v4f* wp = (GQ v4f*)(P + gi);
            v4f wv = *wp;
#pragma unroll
            for (int v = 0; v < 4; ++v) wv[v] = opt_apply(o, wv[v], g[u][v][e] * inv, nd.M, nd.V, gi + v);
            *wp = wv;
          }
        }
      }
    }
  }
  if ((int)threadIdx.x < t.R && nd.has_bias) {
    const int r = threadIdx.x;
    bl[r] = opt_apply(o, bl[r], gb * inv, nd.M, nd.V, (long long)nd.rows * t.C + rowmap[r]);
  }
}

// ------------------------------------------------------------ leaf / branch cells
// BR = false: rows [i; o; u] over the embedding.
// BR = true : rows [i; f_l; f_r; o; u] over [h_l; h_r].
// NRBT / NCGT: the tile's 16-row blocks / 16-column groups when known at compile time, else 0.
// STREAM: the tile's weights stay in HBM (worker aux = 1) instead of LDS.
template <bool BR, int NRBT, int NCGT, bool STREAM>
__device__ __noinline__ void role_tree_cell(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[W->node];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const Pend pd = make_pend(W, t);
  GQ float* pend = (GQ float*)pd.base;
  const WorkerRegs wr = worker_regs(D, W);
  const int R = t.R, H = B.H, Hp = B.Hp, nu = t.nu, u0 = t.u0, KB = wr.kb, nd_muf = uni(nd.muf);
  const GQ int* smeta = uni_gq<int>(D->smeta);
  const GQ int* tnode = uni_gq<int>(D->data.tnode);
  const int ldy = amp_ldrow(R);
  Lds L{lds};
  float* Wg = L.take(STREAM ? 0 : t.Rp * t.ldw);
  float* bg = L.take(t.Rp);
  LDSQ float* Wl = (LDSQ float*)Wg;
  LDSQ float* bl = (LDSQ float*)bg;
  const int yfloats = KB * ldy;
  LDSQ float* Y = (LDSQ float*)L.take(yfloats);   // forward: pre-activations; backward: deltas
  // LDS-resident weights: the deltas have rows of their own, so that waves without a share of the forward product
  // can form them while the others are at it
  // (worker aux = 2: the host found room for them at the same batch size)
  const bool SIDE = !STREAM && uni(W->aux) == 2;
  LDSQ float* Yd = SIDE ? (LDSQ float*)L.take(yfloats) : Y;
  // node row of a tile row / node column of an LDS column (-1 = padding)
  const int CMW = STREAM ? 0 : ((amp_round16(t.Cl) + 63) >> 6) << 6;
  LDSQ int* rowmap = (LDSQ int*)L.take(t.Rp);
  LDSQ int* colmap = (LDSQ int*)L.take(CMW);
  LDSQ int* rowoff = (LDSQ int*)L.take(STREAM ? t.Rp : 0);   // streamed weights: node row * cols
  LDSQ float* Xs = (LDSQ float*)L.take(STREAM ? 2 * 64 * TREE_XS : 0);   // streamed weights: input chunks
  GQ float* ndP = uni_gq<float>(nd.P);
  if (STREAM) {
    for (int i = threadIdx.x; i < t.Rp; i += AMP_THREADS) {
      rowoff[i] = i < R ? t.grow(i) * t.C : 0;
      bl[i] = (i < R && nd.has_bias) ? ndP[(long long)nd.rows * t.C + t.grow(i)] : 0.f;
    }
  } else {
    tile_load(nd, t, Wg, bg);
  }
  for (int i = threadIdx.x; i < yfloats; i += AMP_THREADS) Y[i] = 0.f;
  if (SIDE)
    for (int i = threadIdx.x; i < yfloats; i += AMP_THREADS) Yd[i] = 0.f;
  for (int i = threadIdx.x; i < t.Rp; i += AMP_THREADS) rowmap[i] = i < R ? t.grow(i) : -1;
  for (int i = threadIdx.x; i < CMW; i += AMP_THREADS) colmap[i] = t.ncol(i);
  __syncthreads();
  // bias gradient of tile row threadIdx.x accumulated since the last update (rests in HBM between launches)
  GQ float* ndG = uni_gq<float>(nd.G);
  float accb = ((int)threadIdx.x < R && nd.has_bias) ? ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] : 0.f;
  BatchMsg& M = s_M;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  const GQ float* xbase = BR ? B.hc : B.xin;
  GQ float* obase = BR ? B.gpar : B.gx;
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  // Wave 1 takes the next batch from the ring and decodes it while wave 0 is still publishing the present one
  // (wave 0 keeps what its joins need in registers, so the batch's LDS record is free from the publish barrier on).
  const int wave = threadIdx.x >> 6;
  auto take_batch = [&](int room) {
    const int n = poll_batch(D, mine, head, KB, room, s_codes, &s_n, code_is_b);
    if (n > 0) {
      const int k = threadIdx.x & 63;
      if (k < n) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), nn = MSG_LOCAL(code);
        const v4i sm = tree_slot(smeta, s);
        const v4i tn = tree_node(tnode, sm.z, nn);
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
          M.dst0[k] = (int)((B.node(s, tn.x) * B.TB + wr.tile) * Hp);
          M.dst1[k] = (int)((B.node(s, tn.y) * B.TB + wr.tile) * Hp);
        } else {
          M.off0[k] = M.off1[k] = (int)(B.leaf(s, nn) * B.Ep);
          M.dst0[k] = M.dst1[k] = (int)((B.leaf(s, nn) * B.TL + wr.tile) * B.Ep);
        }
      }
      batch_split_and_log(D, wr, M, n, wr.node, false);
    }
  };
  if (wave == 1) take_batch(nd_muf - (int)count);
  lds_barrier();
  for (;;) {
    const int n = s_n;
    if (n == 0) break;
    head += n;
    const int nF = M.nF, nB = M.nB;
    // The deltas of the batch's backward messages (tile order [gate][unit], zero beyond R) into Yd, pair i =
    // (message, unit) by thread first + j * stride.
    auto form_deltas = [&](int first, int stride) {
      for (int i = first; i < nB * (ldy - R); i += stride) {
        const int k = i / (ldy - R), r = R + i - k * (ldy - R);
        Yd[k * ldy + r] = 0.f;
      }
      for (int i = first; i < nB * nu; i += stride) {
        const int k = i / nu, j = i - k * nu, m = M.bidx[k], u = u0 + j;
        const long long nn = B.node(M.s[m], M.n[m]);
        const GQ float* gt = B.gate + nn * 6 * H;
        float dh = B.gout[nn * H + u], dc = 0.f;
        if (M.par[m] >= 0) {
          const GQ float* gp = B.gpar + nn * B.TB * Hp + u;
          float p = 0.f;
          int q = 0;
          for (; q + 15 < B.TB; q += 16) {   // sixteen parts in flight at a time, added in tile order
            float pp[16];
#pragma unroll
            for (int a = 0; a < 16; ++a) pp[a] = gp[(q + a) * Hp];
#pragma unroll
            for (int a = 0; a < 16; ++a) p += pp[a];
          }
          for (; q + 3 < B.TB; q += 4) {
            const float p0 = gp[q * Hp], p1 = gp[(q + 1) * Hp], p2 = gp[(q + 2) * Hp], p3 = gp[(q + 3) * Hp];
            p = (((p + p0) + p1) + p2) + p3;
          }
          for (; q < B.TB; ++q) p += gp[q * Hp];
          dh += p;
          dc = B.gc[nn * H + u];
        }
        const float i_ = gt[u], o_ = gt[3 * H + u], g_ = gt[4 * H + u], tc = gt[5 * H + u];
        const float dct = dc + dh * o_ * (1.f - tc * tc);
        const float d_o = dh * tc * o_ * (1.f - o_);
        const float d_i = dct * g_ * i_ * (1.f - i_);
        const float d_g = dct * i_ * (1.f - g_ * g_);
        LDSQ float* ds = Yd + k * ldy;
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
    };
    // Waves without a share of the forward product (tree_fwd_mfma: a 16-message block is shared by 8, 4 or 2 waves,
    // each taking every wpn-th 16-row block) form the deltas meanwhile.
    int n_side = 0, side_rank = -1;
    if (SIDE && nF > 0 && nB > 0) {
      const TreeShape<NRBT, NCGT> sh(t);
      const int NBF = (nF + 15) >> 4, wpn = NBF == 1 ? 8 : NBF == 2 ? 4 : 2, me = uni((int)(threadIdx.x >> 6));
      for (int w = 0; w < AMP_THREADS / 64; ++w) {
        const int nbw = w / wpn, subw = (w - nbw * wpn + (wpn >> 1) * (nbw & 1)) % wpn;
        if (!(nbw < NBF && subw < sh.NRB)) {
          if (w == me) side_rank = n_side;
          ++n_side;
        }
      }
    }
    PHASE(0);
    // ---------------- forward messages of the batch
    if (nF > 0) {
      // the children's c of this thread's first (message, unit) pair travel while the product is formed
      float pcl = 0.f, pcr = 0.f;
      if (BR && (int)threadIdx.x < nF * nu) {
        const int k = threadIdx.x / nu, m = M.fidx[k], u = u0 + (int)threadIdx.x - k * nu;
        pcl = xbase[M.off0[m] + Hp + u];
        pcr = xbase[M.off1[m] + Hp + u];
        asm volatile("" ::: "memory");
      }
      if (side_rank >= 0) form_deltas(side_rank * 64 + (int)(threadIdx.x & 63), n_side * 64);
      if (STREAM)
        tree_fwd_stream<BR>(ndP, rowoff, t, bl, xbase, M, nF, Y, ldy, Xs);
      else
        tree_fwd_mfma<BR, NRBT, NCGT>(Wl, t, bl, xbase, M, nF, Y);
      lds_barrier();
      PHASE(1);
      for (int i = threadIdx.x; i < nF * nu; i += AMP_THREADS) {
        const int k = i / nu, j = i - k * nu, m = M.fidx[k], u = u0 + j;
        const LDSQ float* y = Y + k * ldy;
        const long long nn = B.node(M.s[m], M.n[m]);
        GQ float* hcn = B.hc + nn * 2 * Hp;
        GQ float* gt = B.gate + nn * 6 * H;
        float c_, o_;
        if (BR) {
          const bool first = i == (int)threadIdx.x;
          const float cl = first ? pcl : xbase[M.off0[m] + Hp + u];
          const float cr = first ? pcr : xbase[M.off1[m] + Hp + u];
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
      lds_barrier();
      PHASE(2);
    }
    // ---------------- backward messages of the batch
    if (nB > 0) {
      if (n_side == 0) form_deltas((int)threadIdx.x, AMP_THREADS);
      lds_barrier();
      PHASE(3);
      // The (delta, input) pairs join the pending gradients: entry = [delta (Rp) | input in LDS column layout (Cp)].
      // The input part depends on nothing computed here: its first four 16-byte groups per thread are fetched now,
      // travel while the delta parts are stored and the product is formed, and are stored afterwards.
      const int perx = pd.Cp >> 2, totalx = nB * perx;
      v4f xv[4];
      GQ float* xd[4];
      bool xin[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int idx = threadIdx.x + a * AMP_THREADS;
        const int ii = idx < totalx ? idx : totalx - 1;
        const int k = ii / perx, lc = (ii - k * perx) << 2, m = M.bidx[k];
        xin[a] = lc < t.Cl;
        xd[a] = idx < totalx ? pend + (long long)(count + k) * pd.stride + pd.Rp + lc : nullptr;
        xv[a] = *(const GQ v4f*)(xbase + (xin[a] ? ((BR && lc >= t.segp) ? M.off1[m] + lc - t.segp : M.off0[m] + lc) : M.off0[m]));
      }
      asm volatile("" ::: "memory");   // the fetches are issued before the stores below
      {
        const int perd = pd.Rp >> 2, totald = nB * perd;
        for (int idx = threadIdx.x; idx < totald; idx += AMP_THREADS) {
          const int k = idx / perd, j = (idx - k * perd) << 2;
          *(GQ v4f*)(pend + (long long)(count + k) * pd.stride + j) = *(const LDSQ v4f*)(Yd + k * ldy + j);   // ldy >= Rp, zero beyond R
        }
      }
      if ((int)threadIdx.x < R) {
        // the reads of eight messages' deltas are issued together; the sum keeps the messages' order
        int k = 0;
        for (; k + 7 < nB; k += 8) {
          float y[8];
#pragma unroll
          for (int a = 0; a < 8; ++a) y[a] = Yd[(k + a) * ldy + threadIdx.x];
#pragma unroll
          for (int a = 0; a < 8; ++a) accb += y[a];
        }
        for (; k < nB; ++k) accb += Yd[k * ldy + threadIdx.x];
      }
      PHASE(4);
      if (STREAM)
        tree_bwd_stream<BR>(ndP, rowoff, t, Yd, ldy, M, nB, obase);
      else
        tree_bwd_mfma<BR, NRBT, NCGT>(Wl, t, Yd, M, nB, obase);
#pragma unroll
      for (int a = 0; a < 4; ++a)
        if (xd[a]) *(GQ v4f*)xd[a] = xin[a] ? xv[a] : (v4f){0.f, 0.f, 0.f, 0.f};
      // the rest of the input parts (batches of more than 4 x 512 groups)
      for (int idx = threadIdx.x + 4 * AMP_THREADS; idx < totalx; idx += AMP_THREADS) {
        const int k = idx / perx, lc = (idx - k * perx) << 2, m = M.bidx[k];
        const bool in = lc < t.Cl;
        const v4f xr = *(const GQ v4f*)(xbase + (in ? ((BR && lc >= t.segp) ? M.off1[m] + lc - t.segp : M.off0[m] + lc) : M.off0[m]));
        *(GQ v4f*)(pend + (long long)(count + k) * pd.stride + pd.Rp + lc) = in ? xr : (v4f){0.f, 0.f, 0.f, 0.f};
      }
      PHASE(5);
    }
    // what lane k of wave 0 needs of message k for its joins, before the batch's record is given up
    int js = 0, jn = 0, jaux = 0, jpar = 0, ja = 0, jb = 0, jL = 0;
    if (threadIdx.x < 64 && (int)threadIdx.x < n) {
      const int k = threadIdx.x;
      js = M.s[k];
      jn = M.n[k];
      jaux = M.aux[k];
      jpar = M.par[k];
      ja = M.a[k];
      jb = M.b[k];
      jL = M.L[k];
    }
    // every wave's HBM stores have landed before wave 0 publishes the batch
    publish_barrier();
    // ---------------- joins and posts, one lane per message
    if (threadIdx.x < 64) {
      fence_release();
      if ((int)threadIdx.x < n) {
        if (!jaux) {
          tree_node_part_done(wr, B, js, jn, jpar);
        } else if (BR) {
          tree_grad_part_done(wr, B, js, ja, false, ja < jL);
          tree_grad_part_done(wr, B, js, jb, false, jb < jL);
        } else {
          if (join_arrive(B.cnt + B.node(js, jn) * 4 + 3, B.TL)) ring_post(wr.lookup, MSG_MAKE(1, js, jn));
        }
      }
    }
    PHASE(6);
    count += nB;
    if ((int)count >= nd_muf) {
      // the node's own update (Section 3): optimizer step on the LDS weights with the accumulated gradient
      tstep++;
      if (threadIdx.x == 0) note_update(D);
      if (STREAM)
        tree_update_stream(ndP, bl, &nd, t, pend, count, tstep, rowmap, accb);
      else
        tree_update_from_pend<NRBT, NCGT>(Wl, bl, &nd, t, pend, count, count, tstep, rowmap, colmap, accb);
      accb = 0.f;
      count = 0;
      // recorded by the wave that records the next batch's events, so that the update comes first
      if (threadIdx.x == 64) log_event(D, W, &s_logn, wr.node, 2, 0, 0);
    }
    if (wave == 1) take_batch(nd_muf - (int)count);
    lds_barrier();
    PHASE(7);
  }
  if (STREAM) {
    __syncthreads();
    if ((int)threadIdx.x < R && nd.has_bias) ndP[(long long)nd.rows * t.C + t.grow(threadIdx.x)] = bl[threadIdx.x];
  } else {
    tile_store(nd, t, Wg, bg);
  }
  if ((int)threadIdx.x < R && nd.has_bias) ndG[(long long)nd.rows * t.C + t.grow(threadIdx.x)] = accb;
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}

// ------------------------------------------------------------ output layer + loss at every node
// The node where a forward message turns round (Section 4: the loss layer
// initiates backpropagation).  The batch's h vectors are fetched into LDS
// together; logits, softmax loss, d logits and W^T d logits are then computed
// thread-parallel over (message, class) and (message, column).  The node's
// gradient accumulator (n_class x H, spread over the threads) stays in
// registers from one update to the next; between launches it rests in HBM.
__device__ __noinline__ void role_tree_out(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[3];
  const Tile t = make_tile(nd, W);
  const TreeBufs B = tree_bufs(D);
  const WorkerRegs wr = worker_regs(D, W);
  const int R = t.R, C = t.C, H = B.H, Hp = B.Hp, KB = wr.kb, ldw = t.ldw, nd_muf = uni(nd.muf);
  const GQ int* smeta = uni_gq<int>(D->smeta);
  const GQ int* tnode = uni_gq<int>(D->data.tnode);
  const GQ int* slot_inst = uni_gq<int>(D->slot_inst);
  GQ float* probe = uni_gq<float>(D->probe);
  GQ unsigned* probe_n = uni_gq<unsigned>(D->probe_n);
  const unsigned probe_period = uni(D->probe_period), probe_cap = uni(D->probe_cap);
  const int probe_w = uni(D->probe_w);
  Lds L{lds};
  float* Wg = L.take(t.Rp * t.ldw);
  float* bg = L.take(t.Rp);
  LDSQ float* Wl = (LDSQ float*)Wg;
  LDSQ float* bl = (LDSQ float*)bg;
  LDSQ float* hbuf = (LDSQ float*)L.take(KB * Hp);    // per message: the node's h
  LDSQ float* zbuf = (LDSQ float*)L.take(KB * 64);    // per message: logits, then d logits (R <= 64)
  LDSQ int* done_cnt = (LDSQ int*)L.take(D->mak);     // eval: nodes scored per slot
  tile_load(nd, t, Wg, bg);
  for (int i = threadIdx.x; i < D->mak; i += AMP_THREADS) done_cnt[i] = 0;
  // this thread's accumulator elements e = threadIdx.x + 512 j (row e / C, column e % C), and the bias gradient of row threadIdx.x
  GQ float* ndG = (GQ float*)nd.G;
  constexpr int NE = 12;   // n_class * H <= 12 * 512
  float gacc[NE], gb;
  int er[NE], ec[NE];
#pragma unroll
  for (int j = 0; j < NE; ++j) {
    const int e = threadIdx.x + AMP_THREADS * j;
    er[j] = e < R * C ? e / C : -1;
    ec[j] = e < R * C ? e - (e / C) * C : 0;
    gacc[j] = er[j] >= 0 ? ndG[e] : 0.f;
  }
  gb = (int)threadIdx.x < R ? ndG[R * C + threadIdx.x] : 0.f;
  BatchMsg& M = s_M;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring));
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  for (;;) {
    const int room = wr.train ? nd_muf - (int)count : KB_MAX;
    const int n = wait_batch(D, mine, head, KB, room, s_codes, &s_n, [](unsigned) { return true; });
    if (n == 0) break;
    if (threadIdx.x < 64) {
      const int k = threadIdx.x;
      if (k < n) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), nn = MSG_LOCAL(code);
        const v4i sm = tree_slot(smeta, s);
        const v4i tn = tree_node(tnode, sm.z, nn);
        M.s[k] = s;
        M.n[k] = nn;
        M.seq[k] = (unsigned)sm.x;
        M.a[k] = tn.w;
        M.par[k] = tn.z;
        M.L[k] = sm.y;
        // 1 = a node of an evaluation instance: scored, then counted towards the instance's retirement; no gradient
        M.aux[k] = (!wr.train || slot_inst[s] < 0) ? 1 : 0;
        M.off0[k] = (int)(B.node(s, nn) * 2 * Hp);
        M.dst0[k] = (int)(B.node(s, nn) * H);
        // probe: this node's h (its cell's forward output) if the instance is sampled
        int entry = -1;
        if (probe_period && (unsigned)sm.x % probe_period == 0u) {
          const unsigned e = __hip_atomic_fetch_add(probe_n, 1u, __ATOMIC_RELAXED, AGENT);
          if (e < probe_cap) {
            entry = (int)e;
            GQ int* hdr = (GQ int*)(probe + (long long)e * probe_w);
            hdr[0] = 0;
            hdr[1] = sm.x;
            hdr[2] = nn;
            hdr[3] = 0;
          }
        }
        M.b[k] = entry;
      }
      // the event record: a training node's message is a forward event followed by a backward event (the loss turns
      // it round in place), an evaluation node's a forward event only
      {
        const bool in = k < n, tr = in && M.aux[k] == 0;
        const unsigned long long mt = __ballot(tr);
        if (k == 0) M.nB = __popcll(mt);   // gradients in this batch
        if (wr.log_cap) {
          const unsigned base = s_logn, at = base + (unsigned)k + (unsigned)__popcll(mt & ((1ull << k) - 1ull));
          const unsigned total = (unsigned)n + (unsigned)__popcll(mt);
          if (base + total > wr.log_cap) {
            if (k == 0) raise_abort(D, ABORT_LOG_FULL, blockIdx.x);
          } else {
            if (in) {
              const unsigned long long tail = ((unsigned long long)M.seq[k] << 32) | (3ull << 20) | ((unsigned)M.n[k] & 0xfffffu);
              wr.log[at] = tail;
              if (tr) wr.log[at + 1] = tail | (1ull << 28);
            }
            if (k == 0) s_logn = base + total;
          }
        }
      }
    }
    lds_barrier();
    for (int idx = threadIdx.x; idx < n * (Hp >> 2); idx += AMP_THREADS) {
      const int k = idx / (Hp >> 2), c = (idx - k * (Hp >> 2)) << 2;
      const v4f hv = *(const GQ v4f*)(B.hc + M.off0[k] + c);
      *(LDSQ v4f*)(hbuf + k * Hp + c) = hv;
      if (probe_period && M.b[k] >= 0) *(GQ v4f*)(probe + (long long)M.b[k] * probe_w + 4 + c) = hv;
    }
    lds_barrier();
    // logits z[k][r]
    for (int idx = threadIdx.x; idx < n * R; idx += AMP_THREADS) {
      const int k = idx / R, r = idx - k * R;
      const LDSQ float* w = Wl + r * ldw;
      const LDSQ float* h = hbuf + k * Hp;
      float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
      int c = 0;
      // sixteen columns' operands are read together (rows start 16-byte aligned), then multiplied in column order
      for (; c + 15 < C; c += 16) {
        v4f wv[4], hv[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          wv[g] = *(const LDSQ v4f*)(w + c + 4 * g);
          hv[g] = *(const LDSQ v4f*)(h + c + 4 * g);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          a0 = fmaf(wv[g].x, hv[g].x, a0);
          a1 = fmaf(wv[g].y, hv[g].y, a1);
          a2 = fmaf(wv[g].z, hv[g].z, a2);
          a3 = fmaf(wv[g].w, hv[g].w, a3);
        }
      }
      for (; c + 3 < C; c += 4) {
        a0 = fmaf(w[c], h[c], a0);
        a1 = fmaf(w[c + 1], h[c + 1], a1);
        a2 = fmaf(w[c + 2], h[c + 2], a2);
        a3 = fmaf(w[c + 3], h[c + 3], a3);
      }
      for (; c < C; ++c) a0 = fmaf(w[c], h[c], a0);
      zbuf[k * 64 + r] = ((a0 + a1) + (a2 + a3)) + bl[r];
    }
    lds_barrier();
    // softmax cross-entropy per message; z becomes dz = p - onehot(label)
    if ((int)threadIdx.x < n) {
      const int k = threadIdx.x, label = M.a[k];
      LDSQ float* z = zbuf + k * 64;
      float m = z[0];
      int am = 0;
      for (int r = 1; r < R; ++r)
        if (z[r] > m) {
          m = z[r];
          am = r;
        }
      float se = 0.f;
      for (int r = 0; r < R; ++r) se += expf(z[r] - m);
      const float zl = z[label];
      const float inv = 1.f / se;
      // d logits; zero for an evaluation node, which then adds nothing to the gradient sums below
      const float keep = M.aux[k] ? 0.f : 1.f;
      for (int r = 0; r < R; ++r) z[r] = keep * (expf(z[r] - m) * inv - (r == label ? 1.f : 0.f));
      const unsigned idx = M.seq[k] - D->first_seq;
      __hip_atomic_fetch_add((GQ float*)&D->loss_out[idx], -(zl - m - logf(se)), __ATOMIC_RELAXED, AGENT);
      if (am == label) __hip_atomic_fetch_add((GQ int*)&D->correct_out[idx], 1, __ATOMIC_RELAXED, AGENT);
    }
    if (D->train) {
      lds_barrier();
      // dh[k][c] = sum_r W[r][c] dz[k][r]
      for (int idx = threadIdx.x; idx < n * C; idx += AMP_THREADS) {
        const int k = idx / C, c = idx - k * C;
        const LDSQ float* z = zbuf + k * 64;
        float a = 0.f;
        for (int r = 0; r < R; ++r) a = fmaf(Wl[r * ldw + c], z[r], a);
        B.gout[M.dst0[k] + c] = a;
      }
      // G[r][c] += sum_k dz[k][r] h[k][c], messages in ring order
#pragma unroll
      for (int j = 0; j < NE; ++j)
        if (er[j] >= 0) {
          float a = gacc[j];
          int k = 0;
          for (; k + 7 < n; k += 8) {   // eight messages' operands are read together, then added in ring order
            float zz[8], hh[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              zz[q] = zbuf[(k + q) * 64 + er[j]];
              hh[q] = hbuf[(k + q) * Hp + ec[j]];
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) a = fmaf(zz[q], hh[q], a);
          }
          for (; k < n; ++k) a = fmaf(zbuf[k * 64 + er[j]], hbuf[k * Hp + ec[j]], a);
          gacc[j] = a;
        }
      if ((int)threadIdx.x < R)
        for (int k = 0; k < n; ++k) gb += zbuf[k * 64 + threadIdx.x];
    }
    // every wave's HBM stores have landed before wave 0 publishes the batch
    publish_barrier();
    if (threadIdx.x < 64) {
      fence_release();
      const int k = threadIdx.x;
      if (k < n) {
        if (M.aux[k]) {
          if (atomicAdd((int*)&done_cnt[M.s[k]], 1) + 1 == 2 * M.L[k] - 1) {
            done_cnt[M.s[k]] = 0;
            ring_post(wr.ctl, MSG_MAKE(1, M.s[k], 0));
          }
        } else {
          tree_grad_part_done(wr, B, M.s[k], M.n[k], M.par[k] < 0, M.n[k] < M.L[k]);
        }
      }
    }
    if (D->train) {
      count += M.nB;
      if ((int)count >= nd.muf) {
        // the node's own update (Section 3)
        tstep++;
        if (threadIdx.x == 0) note_update(D);
        const OptCoef o = opt_coef(nd, tstep);
        const float inv = nd.mean ? 1.f / (float)count : 1.f;
#pragma unroll
        for (int j = 0; j < NE; ++j)
          if (er[j] >= 0) {
            const int li = er[j] * ldw + ec[j];
            Wl[li] = opt_apply(o, Wl[li], gacc[j] * inv, nd.M, nd.V, (long long)er[j] * C + ec[j]);
            gacc[j] = 0.f;
          }
        if ((int)threadIdx.x < R) {
          bl[threadIdx.x] = opt_apply(o, bl[threadIdx.x], gb * inv, nd.M, nd.V, (long long)R * C + threadIdx.x);
          gb = 0.f;
        }
        count = 0;
        LOG(3, 2, 0, 0);
      }
    }
    lds_barrier();
  }
  tile_store(nd, t, Wg, bg);
#pragma unroll
  for (int j = 0; j < NE; ++j)
    if (er[j] >= 0) ndG[threadIdx.x + AMP_THREADS * j] = gacc[j];
  if ((int)threadIdx.x < R) ndG[R * C + threadIdx.x] = gb;
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}
