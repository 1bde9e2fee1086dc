// Workers of the variable-length RNN (Figure 2).
//
// The recurrent cell may be replicated (Section 5: copies of the heavy linear layer between a Cond and a Phi): every
// copy is a cell worker of its own with its own parameters (node 2 + 2 r for copy r >= 1, hosting table node
// 1 + 2 r) and its own ring (2 + r); the Cond routes on the instance -- admission a goes to copy a mod
// node_replicas, all its steps alike, and its gradient returns to the copy that holds its activations -- and the
// copies' parameters are averaged at the end of every epoch.  The output layer and the loss are shared.
//
// The cell worker hosts the lookup table and the recurrent cell:
// Concat(embedding, h) -> Linear-1 -> tanh -> Isu(t+1) -> Cond(end?) is one
// forward event, and the loop edge is a message to the worker's own ring.
// With max_active_keys sequences in flight the ring holds up to that many
// step messages of different sequences at a time; they are taken as one batch
// and go through the cell on the matrix cores, 16 messages to a block.
//
// Slot storage, rows of SP = segp floats (the larger of emb and hidden, rounded
// up to 4; padding stays zero):
//   buf[0] hs [s][max_len + 1][SP]  row 0 = the zero initial state, row t + 1 = the cell's output at step t
//   buf[1] es [s][max_len][SP]      embedding recorded at forward time (the backward pass and
//                                   the cell's pending gradients use what the forward pass saw)
//   buf[2] dh [s][SP]               gradient w.r.t. the hidden state travelling down the loop
//   buf[3] de [KB_MAX][SP]          the batch's gradients w.r.t. the embeddings
#pragma once

struct RnnBufs {
  GQ float *hs, *es, *dh, *de;
  int SP, TM;
  __device__ __forceinline__ long long hrow(int s, int row) const { return ((long long)s * (TM + 1) + row) * SP; }
  __device__ __forceinline__ long long erow(int s, int t) const { return ((long long)s * TM + t) * SP; }
};

__device__ __forceinline__ RnnBufs rnn_bufs(const GQ AmpDev* D) {
  RnnBufs b;
  b.hs = uni_gq<float>(D->buf[0]);
  b.es = uni_gq<float>(D->buf[1]);
  b.dh = uni_gq<float>(D->buf[2]);
  b.de = uni_gq<float>(D->buf[3]);   // one block of 64 rows per cell worker
  b.SP = uni(D->node[1].segp);
  b.TM = uni(D->max_len);
  return b;
}

// NRBT / NCGT: the cell's 16-row blocks / 16-column groups when known at compile time (0 = any shape).
template <int NRBT, int NCGT>
__device__ __noinline__ void role_rnn_cell(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const int nc = uni(W->node), nl = nc - 1;   // the cell's node and the table's (1 and 0; a copy's own pair)
  const GQ NodeDev& nd = D->node[nc];
  const GQ NodeDev& lk = D->node[nl];
  const Tile t = make_tile(nd, W);
  RnnBufs B = rnn_bufs(D);
  B.de += (long long)uni(W->rep) * 64 * B.SP;
  const Pend pd = make_pend(W, t);
  GQ float* pend = (GQ float*)pd.base;
  const int R = t.R, H = t.R, E = D->emb, V = D->vocab, KB = W->kb, SP = B.SP;
  const int ldy = amp_ldrow(R);
  Lds L{lds};
  float* Wg = L.take(t.Rp * t.ldw);
  float* bg = L.take(t.Rp);
  LDSQ float* Wl = (LDSQ float*)Wg;
  LDSQ float* bl = (LDSQ float*)bg;
  const int yfloats = KB * ldy;
  LDSQ float* Y = (LDSQ float*)L.take(yfloats);   // forward: pre-activations; backward: deltas
  const int CMW = ((amp_round16(t.Cl) + 63) >> 6) << 6;
  LDSQ int* rowmap = (LDSQ int*)L.take(t.Rp);
  LDSQ int* colmap = (LDSQ int*)L.take(CMW);
  // The lookup's accumulated gradient (vocab x emb) stays in LDS when the host found room for it (worker aux = 1):
  // adding a batch's rows to it in HBM is a fetch and a store behind each other in every batch with backward messages.
  const bool g_lds = uni(W->aux) != 0;
  LDSQ float* Gk = (LDSQ float*)L.take(g_lds ? V * E : 0);
  tile_load(nd, t, Wg, bg);
  for (int i = threadIdx.x; i < yfloats; i += AMP_THREADS) Y[i] = 0.f;
  for (int i = threadIdx.x; i < t.Rp; i += AMP_THREADS) rowmap[i] = i < R ? t.grow(i) : -1;
  for (int i = threadIdx.x; i < CMW; i += AMP_THREADS) colmap[i] = t.ncol(i);
  GQ float* ndG = uni_gq<float>(nd.G);
  GQ float* lkP = uni_gq<float>(lk.P);
  GQ float* lkG = uni_gq<float>(lk.G);
  if (g_lds)
    for (int i = threadIdx.x; i < V * E; i += AMP_THREADS) Gk[i] = lkG[i];
  // bias gradient of row threadIdx.x accumulated since the last update (rests in HBM between launches)
  float accb = ((int)threadIdx.x < R && nd.has_bias) ? ndG[(long long)nd.rows * t.C + threadIdx.x] : 0.f;
  BatchMsg& M = s_M;
  __syncthreads();
  const Ring mine = ring_regs(D, uni(W->ring)), out = ring_regs(D, 2), ctl = ring_regs(D, 0);
  const GQ int* tokens = uni_gq<int>(D->data.tok);
  const GQ int* smeta = uni_gq<int>(D->smeta);
  const int nd_muf = uni(nd.muf), lk_muf = uni(lk.muf);
  // both input segments are addressed from hs, both gradient segments from dh
  const GQ float* xbase = B.hs;
  GQ float* obase = B.dh;
  const int es_off = (int)(B.es - B.hs), de_off = (int)(B.de - B.dh);
  // An embedding as wide as the padded segment is fetched by the forward product straight from the table; a
  // narrower one goes through its zero-padded row of es first.
  const bool direct = E == SP;
  const int tab_off = (int)(lkP - B.hs);
  unsigned head = 0;
  unsigned count = W->wstate[0], tstep = W->wstate[1], lcount = W->wstate[2], lstep = W->wstate[3];
  for (;;) {
    const int room_c = nd_muf - (int)count, room_l = lk_muf - (int)lcount;
    const int n = wait_batch(D, mine, head, KB, room_c < room_l ? room_c : room_l, s_codes, &s_n, code_is_b);
    if (n == 0) break;
    if (MSG_SLOT(uni(s_codes[0])) == MSG_CTL_SLOT) {
      // A request to this copy itself (always alone in its batch): a synchronisation round of the cell's copies
      // (Section 5).  First message of a round: publish the parameters as they stand -- the cell's from LDS, the
      // table's from HBM -- and arrive at the round's counter; the arrival that completes the group sends every copy
      // the second message.  Second message: every copy's publication is there; move to their mean (summed in copy
      // order) and keep what was learned since the own publication; tell the controller.
      const unsigned rl = MSG_LOCAL(uni(s_codes[0])), rnd = rl >> 1;
      const int NR = uni(D->node_replicas), rep = uni(W->rep);
      GQ float* cS0 = uni_gq<float>(D->node[1].S);
      GQ float* lS0 = uni_gq<float>(D->node[0].S);
      const long long cstr = NR > 1 ? uni_gq<float>(D->node[4].S) - cS0 : 0, lstr = NR > 1 ? uni_gq<float>(D->node[3].S) - lS0 : 0;
      GQ float* cS = cS0 + rep * cstr;
      GQ float* lS = lS0 + rep * lstr;
      const int nW = R * t.C;
      if (!(rl & 1u)) {
        for (int i = threadIdx.x; i < nW; i += AMP_THREADS) {
          const int lr = i / t.C, c = i - lr * t.C;
          cS[(long long)t.grow(lr) * t.C + c] = Wl[lr * t.ldw + t.lcol(c)];
        }
        if (nd.has_bias)
          for (int lr = threadIdx.x; lr < R; lr += AMP_THREADS) cS[(long long)nd.rows * t.C + t.grow(lr)] = bl[lr];
        for (int i = threadIdx.x; i < V * E; i += AMP_THREADS) lS[i] = lkP[i];
        LOG(nl, 5, rnd, 0);
        LOG(nc, 5, rnd, 0);
        publish_barrier();
        if (threadIdx.x == 0) {
          fence_release();
          if (join_arrive((GQ int*)&D->ctl[6], NR))
            for (int q = 0; q < NR; ++q) ring_post(D->ring[q == 0 ? 1 : 2 + q], MSG_MAKE(0, MSG_CTL_SLOT, (rnd << 1) | 1u));
        }
      } else {
        const float inv = 1.f / (float)NR;
        for (int i = threadIdx.x; i < nW; i += AMP_THREADS) {
          const int lr = i / t.C, c = i - lr * t.C;
          const long long gi = (long long)t.grow(lr) * t.C + c;
          float m = 0.f;
          for (int q = 0; q < NR; ++q) m += cS0[q * cstr + gi];
          LDSQ float* w = Wl + lr * t.ldw + t.lcol(c);
          *w = m * inv + (*w - cS[gi]);
        }
        if (nd.has_bias)
          for (int lr = threadIdx.x; lr < R; lr += AMP_THREADS) {
            const long long gi = (long long)nd.rows * t.C + t.grow(lr);
            float m = 0.f;
            for (int q = 0; q < NR; ++q) m += cS0[q * cstr + gi];
            bl[lr] = m * inv + (bl[lr] - cS[gi]);
          }
        for (int i = threadIdx.x; i < V * E; i += AMP_THREADS) {
          float m = 0.f;
          for (int q = 0; q < NR; ++q) m += lS0[q * lstr + i];
          lkP[i] = m * inv + (lkP[i] - lS[i]);
        }
        LOG(nl, 6, rnd, 0);
        LOG(nc, 6, rnd, 0);
        if (threadIdx.x == 0) ring_post(ctl, MSG_MAKE(1, MSG_CTL_SLOT, rnd));
      }
      __syncthreads();
      continue;
    }
    if (threadIdx.x < 64) {
      const int k = threadIdx.x;
      const bool in = k < n;
      bool isb = false;
      if (in) {
        const unsigned code = s_codes[k];
        const int s = MSG_SLOT(code), tt = MSG_LOCAL(code);
        const v4i sm = *(const GQ v4i*)(smeta + 4 * s);   // admission number, length, -, token offset
        isb = code_is_b(code);
        M.s[k] = s;
        M.n[k] = tt;
        M.seq[k] = (unsigned)sm.x;
        M.L[k] = sm.y;
        M.a[k] = tokens[sm.w + tt];
        M.aux[k] = isb;
        M.off0[k] = (direct && !isb) ? tab_off + M.a[k] * E : es_off + (int)B.erow(s, tt);
        M.off1[k] = (int)B.hrow(s, tt);   // the previous step's output; row 0 holds zeros
        M.dst1[k] = s * SP;
      }
      // positions of the forward / backward messages; a backward message's embedding gradient goes to row b of de
      const unsigned long long mb = __ballot(isb), mf = __ballot(in && !isb);
      const unsigned long long lt = (1ull << k) - 1ull;
      if (isb) {
        const int b = __popcll(mb & lt);
        M.bidx[b] = k;
        M.dst0[k] = de_off + b * SP;
      }
      if (in && !isb) M.fidx[__popcll(mf & lt)] = k;
      if (k == 0) {
        M.nF = __popcll(mf);
        M.nB = __popcll(mb);
      }
      // every message is an event of both hosted nodes: lookup then cell going forward, cell then lookup going back
      if (s_log_cap) {
        const unsigned base = s_logn;
        GQ unsigned long long* logp = (GQ unsigned long long*)s_log_ptr;
        if (base + 2u * (unsigned)n > s_log_cap) {
          if (k == 0) raise_abort(D, ABORT_LOG_FULL, blockIdx.x);
        } else {
          if (in) {
            const unsigned long long tail = ((unsigned long long)M.seq[k] << 32) | ((unsigned)M.n[k] & 0xfffffu);
            const unsigned long long dirb = (unsigned long long)(isb ? 1 : 0) << 28;
            logp[base + 2 * k] = tail | dirb | ((unsigned long long)(isb ? nc : nl) << 20);
            logp[base + 2 * k + 1] = tail | dirb | ((unsigned long long)(isb ? nl : nc) << 20);
          }
          if (k == 0) s_logn = base + 2u * (unsigned)n;
        }
      }
    }
    lds_barrier();
    const int nF = M.nF, nB = M.nB;
    PHASE(0);
    // ---------------- forward messages of the batch
    if (nF > 0) {
      // lookup: the token's row as the table stands now, recorded for the backward pass
      for (int i = threadIdx.x; i < nF * E; i += AMP_THREADS) {
        const int k = i / E, c = i - k * E, m = M.fidx[k];
        B.es[B.erow(M.s[m], M.n[m]) + c] = lkP[(long long)M.a[m] * E + c];
      }
      if (!direct) __syncthreads();
      tree_fwd_mfma<true, NRBT, NCGT>(Wl, t, bl, xbase, M, nF, Y);
      lds_barrier();
      PHASE(1);
      for (int i = threadIdx.x; i < nF * H; i += AMP_THREADS) {
        const int k = i / H, r = i - k * H, m = M.fidx[k];
        B.hs[B.hrow(M.s[m], M.n[m] + 1) + r] = tanhf(Y[k * ldy + r]);
      }
      lds_barrier();
      PHASE(2);
    }
    // ---------------- backward messages of the batch
    if (nB > 0) {
      for (int i = threadIdx.x; i < nB * (ldy - R); i += AMP_THREADS) {
        const int k = i / (ldy - R), r = R + i - k * (ldy - R);
        Y[k * ldy + r] = 0.f;
      }
      for (int i = threadIdx.x; i < nB * H; i += AMP_THREADS) {
        const int k = i / H, r = i - k * H, m = M.bidx[k];
        const float y = B.hs[B.hrow(M.s[m], M.n[m] + 1) + r];
        Y[k * ldy + r] = B.dh[(long long)M.s[m] * SP + r] * (1.f - y * y);
      }
      lds_barrier();
      PHASE(3);
      // the (delta, input) pairs join the pending gradients: entry = [delta (Rp) | input in LDS column layout (Cp)]
      {
        const int per = pd.stride >> 2, total = nB * per;
        for (int idx = threadIdx.x; idx < total; idx += AMP_THREADS) {
          const int k = idx / per, j = (idx - k * per) << 2, m = M.bidx[k];
          v4f v = {0.f, 0.f, 0.f, 0.f};
          if (j < pd.Rp) {
            v = *(const LDSQ v4f*)(Y + k * ldy + j);   // ldy >= Rp, zero beyond R
          } else {
            const int lc = j - pd.Rp;
            if (lc < t.Cl) v = *(const GQ v4f*)(xbase + (lc >= t.segp ? M.off1[m] + lc - t.segp : M.off0[m] + lc));
          }
          *(GQ v4f*)(pend + (long long)(count + k) * pd.stride + j) = v;
        }
      }
      if ((int)threadIdx.x < R)
        for (int k = 0; k < nB; ++k) accb += Y[k * ldy + threadIdx.x];
      PHASE(4);
      tree_bwd_mfma<true, NRBT, NCGT>(Wl, t, Y, M, nB, obase);
      // the lookup's gradient: rows of de added to their tokens' rows in arrival order
      __syncthreads();
      if (g_lds) {
        // column c of every row belongs to thread c: no other thread touches it
        for (int c = threadIdx.x; c < E; c += AMP_THREADS)
          for (int k0 = 0; k0 < nB; k0 += 16) {
            const int kc = nB - k0 < 16 ? nB - k0 : 16;
            float d[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) d[k] = B.de[(k < kc ? k0 + k : k0) * SP + c];
#pragma unroll
            for (int k = 0; k < 16; ++k)
              if (k < kc) Gk[M.a[M.bidx[k0 + k]] * E + c] += d[k];
          }
      } else
      for (int c = threadIdx.x; c < E; c += AMP_THREADS)
        for (int k0 = 0; k0 < nB; k0 += 16) {
          // sixteen rows at a time, all fetches in flight together; a token seen earlier in the chunk continues
          // from that row's result
          const int kc = nB - k0 < 16 ? nB - k0 : 16;
          float g[16], d[16];
          int tok[16];
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            const int kk = k < kc ? k0 + k : k0;
            tok[k] = M.a[M.bidx[kk]];
            g[k] = lkG[(long long)tok[k] * E + c];
            d[k] = B.de[kk * SP + c];
          }
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            float base = g[k];
#pragma unroll
            for (int j = 0; j < 16; ++j)
              if (j < k && tok[j] == tok[k]) base = g[j];
            g[k] = base + d[k];
          }
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (k < kc) lkG[(long long)tok[k] * E + c] = g[k];
        }
    }
    // every wave's HBM stores have landed before wave 0 publishes the batch
    publish_barrier();
    PHASE(5);
    if (threadIdx.x < 64) {
      fence_release();
      const int k = threadIdx.x;
      if (k < n) {
        const int s = M.s[k], tt = M.n[k];
        if (!M.aux[k]) {
          if (tt + 1 < M.L[k])
            ring_post(mine, MSG_MAKE(0, s, tt + 1));
          else
            ring_post(out, MSG_MAKE(0, s, 0));
        } else {
          if (tt > 0)
            ring_post(mine, MSG_MAKE(1, s, tt - 1));
          else
            ring_post(ctl, MSG_MAKE(1, s, 0));
        }
      }
    }
    PHASE(6);
    count += nB;
    lcount += nB;
    if ((int)count >= nd_muf) {
      // the cell's own update (Section 3)
      tstep++;
      if (threadIdx.x == 0) note_update(D);
      tree_update_from_pend<NRBT, NCGT>(Wl, bl, &nd, t, pend, count, count, tstep, rowmap, colmap, accb);
      accb = 0.f;
      count = 0;
      LOG(nc, 2, 0, 0);
    }
    if ((int)lcount >= lk_muf) {
      // the lookup's update: plain SGD over the whole (small) table
      lstep++;
      if (threadIdx.x == 0) note_update(D);
      const float sc = lk.lr * (lk.mean ? 1.f / (float)lcount : 1.f);
      if (g_lds)
        for (int i = threadIdx.x; i < V * E; i += AMP_THREADS) {
          lkP[i] -= sc * Gk[i];
          Gk[i] = 0.f;
        }
      else
        for (int i = threadIdx.x; i < V * E; i += AMP_THREADS) {
          lkP[i] -= sc * lkG[i];
          lkG[i] = 0.f;
        }
      lcount = 0;
      LOG(nl, 2, 0, 0);
    }
    __syncthreads();
    PHASE(7);
  }
  tile_store(nd, t, Wg, bg);
  if (g_lds)
    for (int i = threadIdx.x; i < V * E; i += AMP_THREADS) lkG[i] = Gk[i];
  if ((int)threadIdx.x < R && nd.has_bias) ndG[(long long)nd.rows * t.C + threadIdx.x] = accb;
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
    W->wstate[2] = lcount;
    W->wstate[3] = lstep;
  }
}

// Output layer + softmax loss of the RNN: forward and backward in one event.
__device__ __noinline__ void role_rnn_out(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[2];
  const Tile t = make_tile(nd, W);
  const RnnBufs B = rnn_bufs(D);
  const int R = t.R, C = t.C;
  Lds L{lds};
  float* Wl = L.take(t.Rp * t.ldw);
  float* bl = L.take(t.Rp);
  float* xs = L.take(C);
  float* ys = L.take(R);
  float* ds = L.take(R);
  float* dx = L.take(C);
  float* part = L.take(8 * (R > C ? R : C));
  tile_load(nd, t, Wl, bl);
  const GQ RingDev& mine = D->ring[W->ring];
  const int NR = D->node_replicas;
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code);
    const v4i sm = *(const GQ v4i*)(D->smeta + 4 * s);
    const unsigned seq = (unsigned)sm.x;
    const int T = sm.y, inst = sm.z;
    const GQ float* x = B.hs + B.hrow(s, T);
    for (int c = threadIdx.x; c < C; c += AMP_THREADS) xs[c] = x[c];
    __syncthreads();
    gemv_rows((LDSQ float*)Wl, t.ldw, R, C, (LDSQ float*)bl, (LDSQ float*)xs, (LDSQ float*)part, (LDSQ float*)ys);
    LOG(2, 0, seq, 0);
    const int label = D->data.lab[D->data.lab_off[inst]];
    softmax_xent_wave0(ys, R, label, ds, &s_loss, &s_pred);
    if (threadIdx.x == 0) {
      D->loss_out[seq - D->first_seq] = s_loss;
      D->correct_out[seq - D->first_seq] = s_pred == label;
    }
    if (!D->train || D->slot_inst[s] < 0) {   // an evaluation instance: retired here, nothing turns round
      publish_barrier();
      if (threadIdx.x == 0) {
        fence_release();
        ring_post(D->ring[0], MSG_MAKE(1, s, 0));
      }
      continue;
    }
    LOG(2, 1, seq, 0);
    gemv_cols((LDSQ float*)Wl, t.ldw, R, C, (LDSQ float*)ds, (LDSQ float*)part, (LDSQ float*)dx);
    for (int c = threadIdx.x; c < C; c += AMP_THREADS) B.dh[(long long)s * B.SP + c] = dx[c];
    tile_accumulate(nd, t, ds, xs);
    publish_barrier();
    if (threadIdx.x == 0) {
      fence_release();
      // back to the copy of the cell that ran this instance forward (ring 1, or 2 + r for copy r >= 1)
      const int rep = (int)(seq % (unsigned)NR);
      ring_post(D->ring[rep == 0 ? 1 : 2 + rep], MSG_MAKE(1, s, T - 1));
    }
    count_and_update(D, W, nd, t, Wl, bl, count, tstep);
  }
  tile_store(nd, t, Wl, bl);
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}
