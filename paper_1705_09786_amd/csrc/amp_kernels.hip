// Persistent AMP training kernel for gfx950.
//
// One launch = one amp_train / amp_eval call.  Workgroup w plays worker w
// (Appendix A of the paper: a worker hosts one or more IR nodes and is fed by
// a multi-producer queue): it keeps its nodes' weights in LDS, takes keyed
// messages from its ring, runs the node's forward or backward transform,
// accumulates the gradient, applies the node's own update once
// min_update_frequency gradients have arrived (Section 3), and posts the
// resulting messages.  Worker 0 is the controller (Section 4): it admits
// instances while fewer than max_active_keys are active and retires them when
// their last backward message has come back.
//
// Control-flow nodes of the IR (Cond, Phi, Isu, Concat, Bcast, Group,
// Ungroup, Flatmap) are pure functions of the message state; here they are
// the index arithmetic a producer performs when it decides where a result
// goes, plus arrival counters where several messages must meet.
#include <hip/hip_runtime.h>
#include <mutex>
#include "amp_common.hip.h"

struct Lds {
  float* p;
  __device__ __forceinline__ float* take(int n) {
    float* r = p;
    p += (n + 3) & ~3;
    return r;
  }
};

__shared__ unsigned s_ctl[4];
__shared__ unsigned s_logn;
__shared__ float s_loss;
__shared__ int s_pred;

#define LOG(node, kind, seq, local)                                         \
  do {                                                                      \
    if (threadIdx.x == 0) log_event(D, W, &s_logn, node, kind, seq, local); \
  } while (0)

// ============================================================ controller
// Single-thread wait on the controller's ring.
__device__ __forceinline__ bool ctrl_wait(const GQ AmpDev* D, const GQ RingDev& r, unsigned& head, unsigned& code) {
  const unsigned want = head + 1u;
  GQ unsigned long long* slot = (GQ unsigned long long*)&r.ent[head & r.mask];
  const long long t0 = wall_clock64();
  unsigned spins = 0;
  for (;;) {
    const unsigned long long e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
    if ((unsigned)(e >> 32) == want) {
      fence_acquire();
      code = (unsigned)e;
      head++;
      return true;
    }
    if ((++spins & 7u) == 0u) {
      if (ld_u32(&D->ctl[0])) return false;
      if (wall_clock64() - t0 > D->watchdog_ticks) {
        raise_abort(D, ABORT_WATCHDOG, 0);
        return false;
      }
    }
    __builtin_amdgcn_s_sleep(1);
  }
}

__device__ __noinline__ void role_ctrl(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  if (threadIdx.x == 0) {
    int* freelist = (int*)lds;
    const int mak = D->mak;
    int nfree = mak;
    for (int i = 0; i < mak; ++i) freelist[i] = mak - 1 - i;
    unsigned next = 0, retired = 0, head = 0;
    int active = 0, max_active = 0;
    // Admission.  Greedy: a new instance whenever fewer than max_active_keys are in flight -- at a high
    // max_active_keys the gradients then go stale and training can become unstable (Appendix B, MNIST, which asks
    // for a better schedule).  Staleness-bounded: the number in flight is a limit of its own, between 1 and
    // max_active_keys, which starts at 1, grows by one with every instance that retires having seen at most
    // max_staleness updates per worker during its life, and shrinks by one with every instance that saw more.
    const bool bounded = D->admit_bounded != 0;
    unsigned* upd_at = (unsigned*)(freelist + mak);   // [slot] updates applied so far when the slot's instance was admitted
    int limit = bounded ? 1 : mak;
    const float per_worker = 1.f / (float)(D->n_updaters > 0 ? D->n_updaters : 1);
    const unsigned n_total = D->n_total;
    // Synchronisation of a replicated node's copies (Section 5): after every sync_every retirements a request goes to
    // every copy's ring; a new round waits until every copy has reported that it loaded the previous one.
    const int NR = D->model == 2 ? D->node_replicas : 1;
    const unsigned sync_every = NR > 1 ? (unsigned)D->sync_every : 0u;
    unsigned sync_round = 0, sync_due = 0;
    int sync_acks = NR;
    const GQ RingDev& mine = D->ring[W->ring];
    D->clock[0] = wall_clock64();
    bool ok = true;
    while (retired < n_total && ok) {
      while (active < limit && next < n_total) {
        const int s = freelist[--nfree];
        const unsigned seq = D->first_seq + next;
        // which instance this admission is, and whether it only runs forward (training and inference instances
        // share a launch: Section 1)
        const int word = D->adm_inst[next], inst = word & 0x7fffffff;
        if (bounded) upd_at[s] = ld_u32(&D->ctl[3]);
        D->slot_seq[s] = seq;
        D->slot_inst[s] = word;
        log_event(D, W, &s_logn, 0, 3, seq, word < 0 ? 1u : 0u);
        if (D->model == 3) {
          // tree: the slot's instance facts for the workers, then one token message per leaf to the lookup (worker 1)
          const int toff = D->data.tok_off[inst], L = D->data.tok_off[inst + 1] - toff;
          int* sm = D->smeta + 4 * s;
          sm[0] = (int)seq;
          sm[1] = L;
          sm[2] = D->data.node_off[inst];
          sm[3] = toff;
          fence_release();
          const unsigned t = ring_reserve(D->ring[1], L);
          for (int l = 0; l < L; ++l) ring_put(D->ring[1], t + l, MSG_MAKE(0, s, l));
        } else {
          if (D->model == 2) {
            // RNN: admission number, length, instance, token offset
            const int toff = D->data.tok_off[inst];
            int* sm = D->smeta + 4 * s;
            sm[0] = (int)seq;
            sm[1] = D->data.tok_off[inst + 1] - toff;
            sm[2] = inst;
            sm[3] = toff;
          }
          fence_release();
          // RNN with a replicated cell: the Cond in front of the copies routes on the admission number
          const int rep = D->model == 2 ? (int)(seq % (unsigned)D->node_replicas) : 0;
          ring_post(D->ring[rep == 0 ? 1 : 2 + rep], MSG_MAKE(0, s, 0));
        }
        next++;
        active++;
        if (active > max_active) max_active = active;
      }
      unsigned code;
      ok = ctrl_wait(D, mine, head, code);
      if (ok && MSG_SLOT(code) == MSG_CTL_SLOT) {
        sync_acks++;   // a copy has loaded the round's mean
      } else if (ok) {
        const int s = MSG_SLOT(code);
        log_event(D, W, &s_logn, 0, 4, D->slot_seq[s], 0);
        freelist[nfree++] = s;
        active--;
        retired++;
        if (bounded) {
          const float seen = (float)(ld_u32(&D->ctl[3]) - upd_at[s]) * per_worker;
          if (seen > D->max_staleness)
            limit = limit > 1 ? limit - 1 : 1;
          else
            limit = limit < mak ? limit + 1 : mak;
        }
        if (sync_every && retired % sync_every == 0u) sync_due++;
      }
      if (sync_due && sync_acks == NR && retired < n_total) {
        sync_due = 0;   // requests that fell due while a round was under way merge into one
        sync_acks = 0;
        sync_round++;
        for (int r = 0; r < NR; ++r) ring_post(D->ring[r == 0 ? 1 : 2 + r], MSG_MAKE(0, MSG_CTL_SLOT, sync_round << 1));
      }
    }
    D->clock[1] = wall_clock64();
    D->ctl[4] = (unsigned)max_active;
    D->ctl[5] = (unsigned)limit;
    fence_release();
    __hip_atomic_store((GQ unsigned*)&D->ctl[1], 1u, __ATOMIC_RELAXED, AGENT);
  }
}

// ============================================================ shared tail of a dense backward
// Counts the gradient, updates when min_update_frequency is reached.
__device__ __forceinline__ void count_and_update(const GQ AmpDev* D, const GQ WorkerDev* W, const GQ NodeDev& nd, const Tile& t,
                                                 float* Wl, float* bl, unsigned& count, unsigned& tstep) {
  count++;
  if ((int)count >= nd.muf) {
    tstep++;
    if (threadIdx.x == 0) note_update(D);
    tile_update(nd, t, Wl, bl, count, tstep);
    count = 0;
    LOG(W->node, 2, 0, 0);
  }
}

// ============================================================ MLP
// Worker for linear layer `aux` (0..2) with its ReLU fused; the last layer
// also hosts the softmax loss, which turns the forward message round.
// Slot storage: buf[0]=act1, buf[1]=act2 (post-ReLU outputs), buf[2]=grad
// w.r.t. act1, buf[3]=grad w.r.t. act2.  Weights, bias and the gradient
// accumulator (same layout) stay in LDS for the life of the launch; the
// accumulator rests in HBM between launches.
__device__ __noinline__ void role_mlp_lin(const GQ AmpDev* D, const GQ WorkerDev* W) {
  float* lds = amp_lds;
  const GQ NodeDev& nd = D->node[uni(W->node)];
  const Tile t = make_tile(nd, W);
  const int R = t.R, C = t.C, li = uni(W->aux), ldw = t.ldw, muf = uni(nd.muf), train = uni(D->train);
  const bool first = li == 0, last = li == 2;
  Lds L{lds};
  float* Wg = L.take(t.Rp * ldw);
  float* bg = L.take(t.Rp);
  LDSQ float* Wl = (LDSQ float*)Wg;
  LDSQ float* bl = (LDSQ float*)bg;
  LDSQ float* Gl = (LDSQ float*)L.take(t.Rp * ldw);
  LDSQ float* gbl = (LDSQ float*)L.take(t.Rp);
  LDSQ float* xs = (LDSQ float*)L.take(ldw);
  LDSQ float* ys = (LDSQ float*)L.take(R);
  LDSQ float* ds = (LDSQ float*)L.take(R);
  LDSQ float* dx = (LDSQ float*)L.take(C);
  LDSQ float* part = (LDSQ float*)L.take(8 * (R > C ? R : C));
  tile_load(nd, t, Wg, bg);
  GQ float* ndG = uni_gq<float>(nd.G);
  GQ float* ndM = uni_gq<float>(nd.M);
  GQ float* ndV = uni_gq<float>(nd.V);
  const long long boff = (long long)uni(nd.rows) * C;
  const int has_bias = uni(nd.has_bias);
  for (int i = threadIdx.x; i < t.Rp * ldw; i += AMP_THREADS) {
    const int lr = i / ldw, c = i - lr * ldw;
    Gl[i] = (lr < R && c < C) ? ndG[(long long)lr * C + c] : 0.f;
  }
  for (int i = threadIdx.x; i < t.Rp; i += AMP_THREADS) gbl[i] = (i < R && has_bias) ? ndG[boff + i] : 0.f;
  for (int i = threadIdx.x; i < ldw; i += AMP_THREADS) xs[i] = 0.f;
  __syncthreads();
  const GQ float* act_in = first ? nullptr : uni_gq<float>(D->buf[li - 1]);
  GQ float* act_out = last ? nullptr : uni_gq<float>(D->buf[li]);
  const GQ float* g_in = last ? nullptr : uni_gq<float>(D->buf[2 + li]);
  GQ float* g_out = first ? nullptr : uni_gq<float>(D->buf[2 + li - 1]);
  const GQ float* datax = uni_gq<float>(D->data.x);
  const GQ int* lab = uni_gq<int>(D->data.lab);
  const GQ int* lab_off = uni_gq<int>(D->data.lab_off);
  const GQ unsigned* slot_seq = uni_gq<unsigned>(D->slot_seq);
  const GQ int* slot_inst = uni_gq<int>(D->slot_inst);
  GQ float* loss_out = uni_gq<float>(D->loss_out);
  GQ int* correct_out = uni_gq<int>(D->correct_out);
  const unsigned first_seq = uni(D->first_seq);
  const int ring = uni(W->ring);
  const Ring mine = ring_regs(D, ring), next = ring_regs(D, last ? ring : ring + 1), prev = ring_regs(D, ring - 1), ctl = ring_regs(D, 0);
  unsigned head = 0, code;
  unsigned count = W->wstate[0], tstep = W->wstate[1];
  while (wait_msg(D, mine, head, s_ctl, code)) {
    const int s = MSG_SLOT(code);
    const unsigned seq = uni(slot_seq[s]);
    const int word = uni(slot_inst[s]), inst = word & 0x7fffffff;
    const bool fwd_only = !train || word < 0;   // an evaluation instance: the loss layer retires it
    const GQ float* x = first ? datax + (long long)inst * C : act_in + (long long)s * C;
    bool backward = (code & MSG_DIR_B) != 0;
    for (int c = threadIdx.x; c < C; c += AMP_THREADS) xs[c] = x[c];
    if (backward)
      for (int r = threadIdx.x; r < R; r += AMP_THREADS)
        ds[r] = act_out[(long long)s * R + r] > 0.f ? g_in[(long long)s * R + r] : 0.f;
    lds_barrier();
    if (!backward) {
      gemv_rows(Wl, ldw, R, C, bl, xs, part, ys);
      LOG(W->node, 0, seq, 0);
      if (!last) {
        for (int r = threadIdx.x; r < R; r += AMP_THREADS) act_out[(long long)s * R + r] = fmaxf(ys[r], 0.f);
        publish_barrier();
        if (threadIdx.x == 0) {
          fence_release();
          ring_post(next, MSG_MAKE(0, s, 0));
        }
        continue;
      }
      const int label = lab[lab_off[inst]];
      softmax_xent_wave0((float*)ys, R, label, (float*)ds, &s_loss, &s_pred);
      if (threadIdx.x == 0) {
        loss_out[seq - first_seq] = s_loss;
        correct_out[seq - first_seq] = s_pred == label;
      }
      if (fwd_only) {
        publish_barrier();
        if (threadIdx.x == 0) {
          fence_release();
          ring_post(ctl, MSG_MAKE(1, s, 0));
        }
        continue;
      }
      backward = true;   // the loss layer starts backpropagation
    }
    LOG(W->node, 1, seq, 0);
    if (!first) {
      gemv_cols(Wl, ldw, R, C, ds, part, dx);
      for (int c = threadIdx.x; c < C; c += AMP_THREADS) g_out[(long long)s * C + c] = dx[c];
    }
    // every wave's HBM stores have landed before thread 0 publishes
    publish_barrier();
    if (threadIdx.x == 0) {
      fence_release();
      ring_post(prev, MSG_MAKE(1, s, 0));
    }
    tile_accumulate_lds(t, Gl, gbl, ds, xs);
    count++;
    if ((int)count >= muf) {
      // the node's own update (Section 3) from the accumulator in LDS
      tstep++;
      if (threadIdx.x == 0) note_update(D);
      lds_barrier();
      const OptCoef o = opt_coef(nd, tstep);
      const float inv = nd.mean ? 1.f / (float)count : 1.f;
      for (int i = threadIdx.x; i < R * ldw; i += AMP_THREADS) {
        const int lr = i / ldw, c = i - lr * ldw;
        if (c < C) {
          Wl[i] = opt_apply(o, Wl[i], Gl[i] * inv, ndM, ndV, (long long)lr * C + c);
          Gl[i] = 0.f;
        }
      }
      if (has_bias)
        for (int lr = threadIdx.x; lr < R; lr += AMP_THREADS) {
          bl[lr] = opt_apply(o, bl[lr], gbl[lr] * inv, ndM, ndV, boff + lr);
          gbl[lr] = 0.f;
        }
      count = 0;
      LOG(W->node, 2, 0, 0);
    }
    lds_barrier();
  }
  tile_store(nd, t, Wg, bg);
  for (int i = threadIdx.x; i < R * ldw; i += AMP_THREADS) {
    const int lr = i / ldw, c = i - lr * ldw;
    if (c < C) ndG[(long long)lr * C + c] = Gl[i];
  }
  if (has_bias)
    for (int lr = threadIdx.x; lr < R; lr += AMP_THREADS) ndG[boff + lr] = gbl[lr];
  if (threadIdx.x == 0) {
    W->wstate[0] = count;
    W->wstate[1] = tstep;
  }
}

#include "amp_batch.hip.h"
#include "amp_tree.hip.h"
#include "amp_rnn.hip.h"
#include "amp_ggnn.hip.h"

// ============================================================ entry
extern "C" __global__ void __launch_bounds__(AMP_THREADS) amp_persistent(const AmpDev* Dp, int workers_per_replica,
                                                                         int n_replicas, int xcd_packed) {
  // Every replica has its own descriptor.  Plain mapping: replica r = blocks [r * workers_per_replica, (r + 1) *
  // workers_per_replica).  Packed mapping: workgroups are dealt to the 8 XCDs round-robin by their index, so block
  // b lands on XCD b % 8; all workers of a replica take blocks of one residue, replicas x, x + 8, ... share XCD x,
  // and a replica's rings, stash and joins stay in one L2.  Blocks without a worker leave at once.
  int replica, wi;
  if (xcd_packed) {
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
    replica = x + 8 * (j / workers_per_replica);
    wi = j % workers_per_replica;
    if (replica >= n_replicas) return;
  } else {
    replica = blockIdx.x / workers_per_replica;
    wi = blockIdx.x - replica * workers_per_replica;
  }
  const GQ AmpDev* D = (const GQ AmpDev*)Dp + replica;
  const GQ WorkerDev* W = &D->worker[wi];
  long long t_begin = 0;
  if (threadIdx.x == 0) {
    s_logn = 0;
    s_log_cap = W->tile == 0 ? W->log_cap : 0u;
    s_log_ptr = W->log;
    for (int i = 0; i < AMP_NSTAT; ++i) s_stat[i] = 0;
    t_begin = wall_clock64();
    // packed: the whole replica shares one L2 if block b really runs on die b % 8 (hardware register XCC_ID, id 20,
    // bits 3:0); releases then skip the L2 write-back.  A workgroup that finds itself elsewhere stops the replica
    // before it has exchanged anything.
    s_nowb = 0;
    if (xcd_packed) {
      const int xcc = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf);
      if (xcc == (int)(blockIdx.x & 7))
        s_nowb = 1;
      else
        s_nowb = -1;
    }
  }
  __syncthreads();
  if (s_nowb < 0) {
    if (threadIdx.x == 0) {
      raise_abort(D, ABORT_PLACEMENT, blockIdx.x);
      W->stats[12] = (unsigned long long)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf);
    }
    return;
  }
  switch (W->role) {
    case ROLE_CTRL: role_ctrl(D, W); break;
    case ROLE_MLP_LIN: role_mlp_lin(D, W); break;
    case ROLE_RNN_CELL:
      // hidden = emb = 128 (8 row blocks, 16 column groups) has products with fixed trip counts
      if (D->node[1].rows == 128 && D->node[1].cols == 256 && D->node[1].seg0 == 128)
        role_rnn_cell<8, 16>(D, W);
      else
        role_rnn_cell<0, 0>(D, W);
      break;
    case ROLE_RNN_OUT: role_rnn_out(D, W); break;
    case ROLE_TREE_LOOKUP: role_tree_lookup(D, W); break;
    case ROLE_TREE_LEAF:
    case ROLE_TREE_BRANCH: {
      // hidden 150 / embedding 300 (nineteen 16-column groups) split into tiles of six, four or three 16-row blocks
      // (5 + 8 tiles, the fewest that fit LDS; 8 leaf tiles; 16 branch tiles) has instantiations with fixed trip counts
      const GQ NodeDev& nd = D->node[W->node];
      const int rp = amp_round16(nd.nblocks * W->nu), cl = (nd.cols / nd.seg) * nd.segp;
      const bool c19 = amp_round16(cl) == 304;
      if (W->role == ROLE_TREE_LEAF) {
        if (W->aux == 1) role_tree_cell<false, 0, 0, true>(D, W);
        else if (c19 && rp == 96) role_tree_cell<false, 6, 19, false>(D, W);
        else if (c19 && rp == 64) role_tree_cell<false, 4, 19, false>(D, W);
        else if (c19 && rp == 48) role_tree_cell<false, 3, 19, false>(D, W);
        else role_tree_cell<false, 0, 0, false>(D, W);
      } else {
        if (W->aux == 1) role_tree_cell<true, 0, 0, true>(D, W);
        else if (c19 && rp == 96) role_tree_cell<true, 6, 19, false>(D, W);
        else if (c19 && rp == 64) role_tree_cell<true, 4, 19, false>(D, W);
        else if (c19 && rp == 48) role_tree_cell<true, 3, 19, false>(D, W);
        else role_tree_cell<true, 0, 0, false>(D, W);
      }
      break;
    }
    case ROLE_TREE_OUT: role_tree_out(D, W); break;
    case ROLE_G_LOOKUP: role_g_lookup(D, W); break;
    // hidden size 97..112 (7 / 13 column groups; 7 row blocks, or 4, 3 and 2 when the node is split over two or three tiles)
    // has products with fixed trip counts
    case ROLE_G_EDGE: {
      const int rb = amp_round16(W->nu) >> 4;
      const bool c7 = amp_round16(D->hidden) == 112;
      if (c7 && rb == 7) role_g_edge<7, 7>(D, W);
      else if (c7 && rb == 4) role_g_edge<4, 7>(D, W);
      else if (c7 && rb == 3) role_g_edge<3, 7>(D, W);
      else if (c7 && rb == 2) role_g_edge<2, 7>(D, W);
      else role_g_edge<0, 0>(D, W);
      break;
    }
    case ROLE_G_GATE: {
      const int rb = amp_round16(W->nu) >> 4;
      const bool c13 = amp_round16(D->hidden) == 112 && amp_round16(2 * D->hidden) == 208;
      if (c13 && rb == 7) role_g_gate<7, 13>(D, W);
      else if (c13 && rb == 4) role_g_gate<4, 13>(D, W);
      else if (c13 && rb == 3) role_g_gate<3, 13>(D, W);
      else if (c13 && rb == 2) role_g_gate<2, 13>(D, W);
      else role_g_gate<0, 0>(D, W);
      break;
    }
    case ROLE_G_CAND: {
      const int rb = amp_round16(W->nu) >> 4;
      const bool c13 = amp_round16(D->hidden) == 112 && amp_round16(2 * D->hidden) == 208;
      if (c13 && rb == 7) role_g_cand<7, 13>(D, W);
      else if (c13 && rb == 4) role_g_cand<4, 13>(D, W);
      else if (c13 && rb == 3) role_g_cand<3, 13>(D, W);
      else if (c13 && rb == 2) role_g_cand<2, 13>(D, W);
      else role_g_cand<0, 0>(D, W);
      break;
    }
    case ROLE_G_READOUT: role_g_readout(D, W); break;
    default: break;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (W->log_cap) *W->log_n = s_logn;
    for (int i = 0; i < AMP_NSTAT; ++i) W->stats[i] = s_stat[i];
    W->stats[3] = (unsigned long long)(wall_clock64() - t_begin);
    // which of the eight dies this workgroup ran on: hardware register XCC_ID (id 20), bits 3:0
    W->stats[12] = (unsigned long long)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf);
  }
}

extern "C" hipError_t amp_launch(const AmpDev* devs, int n_replicas, int workers_per_replica, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)amp_persistent, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       AMP_DYN_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // One XCD has 32 CUs: the packed mapping needs the replicas that share an XCD to fit it.  Measured: replicas
  // gain from staying inside one L2 (15 Tree-LSTM replicas 184k -> 256k trees/s), and again from releases without
  // an L2 write-back, which only a packed replica can do (16 replicas 316k -> 409k trees/s); a single pipeline of
  // many workers is faster spread over all eight L2s (30 tree workers 42.8k against 40.3k packed, 17 graph workers
  // 21.7k against 21.3k, 16 tree workers 29.5k against 28.6k), one of few
  // workers faster packed (the 4-worker MLP 52k -> 55k instances/s; the RNN with eight copies of its cell, 10
  // workers, 105k -> 112k sequences/s; the unsplit 10-worker graph pipeline the same either way): up to 12.
  const int per_xcd = (n_replicas + 7) / 8;
  const bool packed = per_xcd * workers_per_replica <= 32 && (n_replicas > 1 || workers_per_replica <= 12);
  const int grid = packed ? 8 * per_xcd * workers_per_replica : n_replicas * workers_per_replica;
  hipLaunchKernelGGL(amp_persistent, dim3(grid), dim3(AMP_THREADS), AMP_DYN_LDS_BYTES, stream, devs, workers_per_replica,
                     n_replicas, packed ? 1 : 0);
  return hipGetLastError();
}

// End-of-epoch synchronisation of replicas (Section 5): every replica's copy of a node's parameters becomes
// the mean over the replicas, summed in replica order.
__global__ void amp_average_kernel(float* p0, size_t stride_floats, int n_replicas, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int r = 0; r < n_replicas; ++r) s += p0[(size_t)r * stride_floats + i];
  s /= (float)n_replicas;
  for (int r = 0; r < n_replicas; ++r) p0[(size_t)r * stride_floats + i] = s;
}

extern "C" hipError_t amp_average(float* p0, size_t stride_floats, int n_replicas, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(amp_average_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p0, stride_floats, n_replicas, n);
  return hipGetLastError();
}

// ============================================================ built-in arena
// Device memory that exists without any allocation call: amp_create_static hands it to a context in place of a
// caller-provided arena.  Every GPU the library's code object is loaded on holds its own copy, at its own address,
// until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address it
// returns (looked up once per device, with that device current) is what kernels, copies and clears are given.
static __device__ __align__(256) unsigned char scratch[AMP_STATIC_ARENA_BYTES];

extern "C" hipError_t amp_static_arena(void** ptr, size_t* bytes) {
  constexpr int MAX_DEV = 64;
  static std::mutex mu;
  static void* addr[MAX_DEV] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEV) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || ((uintptr_t)p & 255)) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  *bytes = AMP_STATIC_ARENA_BYTES;
  return hipSuccess;
}

// ============================================================ peak micro-benchmarks
// What the roofline fractions are measured against can itself be measured: the
// LDS read rate of one workgroup per CU shaped like a worker (512 threads,
// 16-byte reads, several independent reads in flight), and the HBM read rate
// of a grid-wide streaming sum.
extern "C" __global__ void __launch_bounds__(AMP_THREADS) amp_peak_lds_kernel(int iters, float* sink) {
  LDSQ float* l = (LDSQ float*)amp_lds;
  const int nfl = AMP_DYN_LDS_BYTES / 4;
  for (int i = threadIdx.x; i < nfl; i += AMP_THREADS) l[i] = (float)(i & 7);
  __syncthreads();
  // each thread walks the whole LDS in 16-byte steps, eight reads per round
  const int nv = nfl / 4;   // 16-byte groups
  v4f a[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) a[k] = (v4f){0.f, 0.f, 0.f, 0.f};
  int pos = threadIdx.x;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      a[k] += *(const LDSQ v4f*)(l + 4 * pos);
      pos += AMP_THREADS;
      if (pos >= nv) pos -= nv;
    }
  }
  v4f r = a[0];
#pragma unroll
  for (int k = 1; k < 8; ++k) r += a[k];
  if (r.x + r.y + r.z + r.w == -1.f) sink[0] = r.x;   // never true: keeps the reads alive
}

extern "C" __global__ void __launch_bounds__(256) amp_peak_hbm_kernel(const v4f* src, size_t n16, float* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  v4f a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    a0 += src[i];
    a1 += src[i + stride];
    a2 += src[i + 2 * stride];
    a3 += src[i + 3 * stride];
  }
  for (; i < n16; i += stride) a0 += src[i];
  const v4f r = a0 + a1 + a2 + a3;
  if (r.x + r.y + r.z + r.w == -1.2345f) sink[0] = r.x;
}

// Launches the LDS benchmark on n_wg workgroups (one per CU: the dynamic LDS
// size allows no second one) and returns the seconds the timed launch took
// and the bytes it read per workgroup.
extern "C" hipError_t amp_peak_lds_launch(int n_wg, int iters, float* sink, hipStream_t stream, double* seconds,
                                          double* bytes_per_wg) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)amp_peak_lds_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       AMP_DYN_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipEvent_t t0, t1;
  hipError_t e;
  if ((e = hipEventCreate(&t0)) != hipSuccess) return e;
  if ((e = hipEventCreate(&t1)) != hipSuccess) return e;
  hipLaunchKernelGGL(amp_peak_lds_kernel, dim3(n_wg), dim3(AMP_THREADS), AMP_DYN_LDS_BYTES, stream, iters / 8 + 1, sink);   // warm-up
  (void)hipEventRecord(t0, stream);
  hipLaunchKernelGGL(amp_peak_lds_kernel, dim3(n_wg), dim3(AMP_THREADS), AMP_DYN_LDS_BYTES, stream, iters, sink);
  (void)hipEventRecord(t1, stream);
  if ((e = hipEventSynchronize(t1)) != hipSuccess) return e;
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, t0, t1);
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  *seconds = ms * 1e-3;
  *bytes_per_wg = (double)iters * 8.0 * AMP_THREADS * 16.0;
  return hipGetLastError();
}

extern "C" hipError_t amp_peak_hbm_launch(const void* src, size_t bytes, float* sink, hipStream_t stream, double* seconds) {
  hipEvent_t t0, t1;
  hipError_t e;
  if ((e = hipEventCreate(&t0)) != hipSuccess) return e;
  if ((e = hipEventCreate(&t1)) != hipSuccess) return e;
  const size_t n16 = bytes / 16;
  const int grid = 256 * 16;
  hipLaunchKernelGGL(amp_peak_hbm_kernel, dim3(grid), dim3(256), 0, stream, (const v4f*)src, n16, sink);   // warm-up
  (void)hipEventRecord(t0, stream);
  hipLaunchKernelGGL(amp_peak_hbm_kernel, dim3(grid), dim3(256), 0, stream, (const v4f*)src, n16, sink);
  (void)hipEventRecord(t1, stream);
  if ((e = hipEventSynchronize(t1)) != hipSuccess) return e;
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, t0, t1);
  (void)hipEventDestroy(t0);
  (void)hipEventDestroy(t1);
  *seconds = ms * 1e-3;
  return hipGetLastError();
}
