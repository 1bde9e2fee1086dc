// Device-side building blocks of the persistent AMP kernel: message rings,
// watchdog-bounded waits, LDS-resident matrix-vector products, gradient
// accumulation, local optimizer steps and the event record.
#pragma once
#include <hip/hip_runtime.h>
#include "amp_dev.h"

#define AGENT __HIP_MEMORY_SCOPE_AGENT

// Address-space qualifiers.  Pointers read from the device descriptor are
// generic; a generic access is a FLAT instruction, which occupies both the
// vector-memory and the LDS counters, so that every later wait for an LDS
// read also waits for the outstanding HBM traffic.  Hot paths therefore cast
// HBM pointers to GQ (global) and LDS pointers to LDSQ.
#define GQ __attribute__((address_space(1)))
#define LDSQ __attribute__((address_space(3)))
typedef float v4f __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));

// The workgroup's dynamic LDS; every role carves its buffers out of it.  The alignment matters: the dynamic part
// starts where the static variables end, and a base that is only 8-byte aligned makes every 16-byte LDS access of
// the workers a split one (measured: the grouped-row product then takes 7 us instead of 3.1 us).
extern __shared__ __attribute__((aligned(256))) float amp_lds[];

__device__ __forceinline__ unsigned ld_u32(const unsigned* p) {
  return __hip_atomic_load((const GQ unsigned*)p, __ATOMIC_RELAXED, AGENT);
}
// s_nowb: every workgroup this one exchanges data with runs on the same XCD (a launch that packs a replica into
// one die, checked against the hardware's die number when the kernel starts).  Stores that have been acknowledged
// are then in the L2 all of them read through, so a release needs no L2 write-back, only the wait.  Measured with
// two workgroups handing 4 KB back and forth on one die: 0.93 us per hand-over instead of 1.31 us, every word right.
__shared__ int s_nowb;
__device__ __forceinline__ void fence_release() {
  if (s_nowb)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
}
__device__ __forceinline__ void fence_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }

// The barrier in front of a post.  __syncthreads() does not wait for a wave's outstanding HBM stores (at
// workgroup scope the compiler emits no wait for them: the waves of a workgroup share one L1), and the posting
// wave's release fence writes back the L2 as it stands and waits for its own wave's accesses only -- a store of
// another wave still on its way would miss the write-back and the receiver would read the old value.  So every
// wave first waits until its own stores have reached the L2.
__device__ __forceinline__ void publish_barrier() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
}

// Workgroup barrier that orders LDS accesses only; between phases that hand
// data over through LDS this one is enough.  HBM data written by one wave and
// read by another wave of the workgroup needs __syncthreads(); data published
// to other workgroups needs publish_barrier().
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---------------------------------------------------------------- rings
// A ring's descriptor held in (scalar) registers for the life of a worker: posting through it needs no fetch of
// the descriptor from HBM in front of the atomic.
struct Ring {
  GQ unsigned long long* ent;
  GQ unsigned* tail;
  unsigned mask;
};

// Called by ONE thread, after a release fence that covers the payload.
template <class R>
__device__ __forceinline__ void ring_post(const R& r, unsigned code) {
  unsigned t = __hip_atomic_fetch_add((GQ unsigned*)r.tail, 1u, __ATOMIC_RELAXED, AGENT);
  unsigned long long e = ((unsigned long long)(t + 1u) << 32) | code;
  __hip_atomic_store((GQ unsigned long long*)&r.ent[t & r.mask], e, __ATOMIC_RELAXED, AGENT);
}

// Reserves n consecutive tickets; entry i is published with ring_put.
template <class R>
__device__ __forceinline__ unsigned ring_reserve(const R& r, unsigned n) {
  return __hip_atomic_fetch_add((GQ unsigned*)r.tail, n, __ATOMIC_RELAXED, AGENT);
}
template <class R>
__device__ __forceinline__ void ring_put(const R& r, unsigned ticket, unsigned code) {
  unsigned long long e = ((unsigned long long)(ticket + 1u) << 32) | code;
  __hip_atomic_store((GQ unsigned long long*)&r.ent[ticket & r.mask], e, __ATOMIC_RELAXED, AGENT);
}

__device__ __forceinline__ void raise_abort(const GQ AmpDev* D, unsigned code, unsigned detail) {
  unsigned expected = 0;
  if (__hip_atomic_compare_exchange_strong((GQ unsigned*)&D->ctl[0], &expected, code, __ATOMIC_RELAXED, __ATOMIC_RELAXED, AGENT))
    __hip_atomic_store((GQ unsigned*)&D->ctl[2], detail, __ATOMIC_RELAXED, AGENT);
}

// Per-workgroup utilisation counters: [0] ticks spent waiting for messages, [1] messages taken,
// [2] batches taken, [3] last phase boundary, [4..11] ticks per phase (role-specific), [12] the XCC (accelerator
// die) the workgroup ran on.
#define AMP_NSTAT 13
__shared__ unsigned long long s_stat[AMP_NSTAT];
// Thread 0 charges the time since the previous boundary to phase i.  Compiled in only with -DAMP_PHASE_STATS:
// eight clock reads per batch cost about 3 % of a tile worker's time.
#ifndef AMP_PHASE_STATS
#define PHASE(i) do {} while (0)
#else
#define PHASE(i)                                             \
  do {                                                       \
    if (threadIdx.x == 0) {                                  \
      const unsigned long long now_ = wall_clock64();        \
      if (s_stat[3]) s_stat[4 + (i)] += now_ - s_stat[3];    \
      s_stat[3] = now_;                                      \
    }                                                        \
  } while (0)
#endif

// A value known to be the same in every lane, moved to a scalar register: addresses derived from it need no
// vector registers (a worker's per-message pointers would otherwise be spilled to scratch memory and reloaded,
// at L2 latency, in front of every phase).
__device__ __forceinline__ unsigned uni(unsigned v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uni(float v) { return __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(v))); }
__device__ __forceinline__ long long uni(long long v) {
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)v >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}
// The descriptors in HBM are read with vector loads (the compiler cannot prove them unwritten), which leaves every
// base pointer in a pair of vector registers; these put them back into scalar ones.
template <class T>
__device__ __forceinline__ GQ T* uni_gq(const void* p) {
  return (GQ T*)(unsigned long long)uni((long long)(unsigned long long)p);
}

__device__ __forceinline__ Ring ring_regs(const GQ AmpDev* D, int idx) {
  Ring r;
  r.ent = uni_gq<unsigned long long>(D->ring[idx].ent);
  r.tail = uni_gq<unsigned>(D->ring[idx].tail);
  r.mask = uni(D->ring[idx].mask);
  return r;
}

// ONE thread.  Waits for the entry with ticket `head` of ring r and leaves its code in s_ctl[0] and a stop flag
// in s_ctl[1] (run over: done flag, abort flag, or this wait exceeded the watchdog, which raises the abort flag so
// that every workgroup leaves).  No barrier.
template <class R>
__device__ __forceinline__ void poll_msg(const GQ AmpDev* D, const R& r, unsigned head, unsigned* s_ctl) {
  const unsigned want = head + 1u;
  GQ unsigned long long* slot = (GQ unsigned long long*)&r.ent[head & r.mask];
  const long long t0 = wall_clock64();
  unsigned stop = 0, spins = 0;
  unsigned long long e;
  for (;;) {
    e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
    if ((unsigned)(e >> 32) == want) break;
    if ((++spins & 7u) == 0u) {
      if (ld_u32(&D->ctl[0]) | ld_u32(&D->ctl[1])) {
        // done is only raised once nothing is in flight; re-check the slot once
        e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
        if ((unsigned)(e >> 32) == want && ld_u32(&D->ctl[0]) == 0u) break;
        stop = 1;
        break;
      }
      if (wall_clock64() - t0 > D->watchdog_ticks) {
        raise_abort(D, ABORT_WATCHDOG, blockIdx.x);
        stop = 1;
        break;
      }
    }
    __builtin_amdgcn_s_sleep(1);
  }
  if (!stop) fence_acquire();
  s_stat[0] += (unsigned long long)(wall_clock64() - t0);
  s_stat[1] += 1ull - stop;
  s_ctl[0] = (unsigned)e;
  s_ctl[1] = stop;
}

// Whole workgroup: thread 0 polls, everybody gets the code; returns false when the run is over.
// s_ctl: two words of LDS.
template <class R>
__device__ __forceinline__ bool wait_msg(const GQ AmpDev* D, const R& r, unsigned& head, unsigned* s_ctl, unsigned& code) {
  if (threadIdx.x == 0) poll_msg(D, r, head, s_ctl);
  __syncthreads();
  // the same for every lane: kept in scalar registers, and so is everything derived from it
  code = uni(s_ctl[0]);
  const bool ok = uni(s_ctl[1]) == 0u;
  lds_barrier();
  if (ok) head++;
  return ok;
}

// ---------------------------------------------------------------- event record
// The worker's record buffer and its capacity, copied into LDS when the kernel starts (s_log_cap = 0 when the
// record is off or this worker is not its node's first tile): an event costs no descriptor fetch from HBM.
__shared__ unsigned long long* s_log_ptr;
__shared__ unsigned s_log_cap;

__device__ __forceinline__ void log_event(const GQ AmpDev* D, const GQ WorkerDev* W, unsigned* s_logn, int node, int kind,
                                          unsigned seq, unsigned local) {
  const unsigned cap = s_log_cap;
  if (cap == 0) return;
  unsigned n = *s_logn;
  if (n >= cap) {
    raise_abort(D, ABORT_LOG_FULL, blockIdx.x);
    return;
  }
  ((GQ unsigned long long*)s_log_ptr)[n] = ((unsigned long long)seq << 32) | ((unsigned)kind << 28) | ((unsigned)node << 20) | (local & 0xfffffu);
  *s_logn = n + 1;
}

// ---------------------------------------------------------------- LDS matvec
// Weights of a tile live in LDS as Wl[R][ldw] with ldw odd, so that threads
// walking down a column (stride ldw) and threads walking along a row both hit
// distinct banks.

// y[r] = b[r] + sum_c Wl[r][c] * x[c].  Thread (p, r) sums the p-th column
// chunk of row r; partials meet in `part` (>= P * R floats).  All threads.
__device__ __forceinline__ void gemv_rows(const LDSQ float* Wl, int ldw, int R, int C, const LDSQ float* bl, const LDSQ float* x,
                                          LDSQ float* part, LDSQ float* y) {
  int P = AMP_THREADS / R;
  if (P < 1) P = 1;
  if (P > 8) P = 8;
  const int chunk = (C + P - 1) / P;
  for (int idx = threadIdx.x; idx < R * P; idx += AMP_THREADS) {
    const int p = idx / R, r = idx - p * R;
    const int c0 = p * chunk;
    int c1 = c0 + chunk;
    if (c1 > C) c1 = C;
    const LDSQ float* w = Wl + r * ldw;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int c = c0;
    for (; c + 3 < c1; c += 4) {
      s0 = fmaf(w[c], x[c], s0);
      s1 = fmaf(w[c + 1], x[c + 1], s1);
      s2 = fmaf(w[c + 2], x[c + 2], s2);
      s3 = fmaf(w[c + 3], x[c + 3], s3);
    }
    for (; c < c1; ++c) s0 = fmaf(w[c], x[c], s0);
    part[p * R + r] = (s0 + s1) + (s2 + s3);
  }
  lds_barrier();
  for (int r = threadIdx.x; r < R; r += AMP_THREADS) {
    float s = bl ? bl[r] : 0.f;
    for (int p = 0; p < P; ++p) s += part[p * R + r];
    y[r] = s;
  }
  lds_barrier();
}

// dx[c] = sum_r Wl[r][c] * d[r].  Thread (p, c) sums the p-th row chunk of
// column c.  `part` >= P * C floats.  All threads.
__device__ __forceinline__ void gemv_cols(const LDSQ float* Wl, int ldw, int R, int C, const LDSQ float* d, LDSQ float* part,
                                          LDSQ float* dx) {
  int P = AMP_THREADS / C;
  if (P < 1) P = 1;
  if (P > 8) P = 8;
  const int chunk = (R + P - 1) / P;
  for (int idx = threadIdx.x; idx < C * P; idx += AMP_THREADS) {
    const int p = idx / C, c = idx - p * C;
    const int r0 = p * chunk;
    int r1 = r0 + chunk;
    if (r1 > R) r1 = R;
    const LDSQ float* w = Wl + c;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int r = r0;
    for (; r + 3 < r1; r += 4) {
      s0 = fmaf(w[r * ldw], d[r], s0);
      s1 = fmaf(w[(r + 1) * ldw], d[r + 1], s1);
      s2 = fmaf(w[(r + 2) * ldw], d[r + 2], s2);
      s3 = fmaf(w[(r + 3) * ldw], d[r + 3], s3);
    }
    for (; r < r1; ++r) s0 = fmaf(w[r * ldw], d[r], s0);
    part[p * C + c] = (s0 + s1) + (s2 + s3);
  }
  lds_barrier();
  for (int c = threadIdx.x; c < C; c += AMP_THREADS) {
    float s = 0.f;
    for (int p = 0; p < P; ++p) s += part[p * C + c];
    dx[c] = s;
  }
  lds_barrier();
}

// ---------------------------------------------------------------- tiles
// A tile owns units [u0, u0+nu) of each of the node's gate blocks.  Local row
// lr = g * nu + j  <->  node row g * block + u0 + j.
struct Tile {
  int R, C, ldw, nu, u0, block, nblocks, Rp;
  int seg, segp, seg0, Cl;   // column segments (see NodeDev); Cl = padded column count
  __device__ __forceinline__ int grow(int lr) const {
    const int g = lr / nu;
    return g * block + u0 + (lr - g * nu);
  }
  // LDS column of node column c
  __device__ __forceinline__ int lcol(int c) const {
    if (c < seg0) return c;
    const int sg = (c - seg0) / seg;
    return (sg + 1) * segp + (c - seg0 - sg * seg);
  }
  // node column of LDS column lc, -1 for a padding column
  __device__ __forceinline__ int ncol(int lc) const {
    const int sg = lc / segp, o = lc - sg * segp;
    if (lc >= Cl) return -1;
    if (sg == 0) return o < seg0 ? o : -1;
    return o < seg ? seg0 + (sg - 1) * seg + o : -1;
  }
};

__device__ __forceinline__ Tile make_tile(const GQ NodeDev& nd, const GQ WorkerDev* W) {
  Tile t;
  t.nu = uni(W->nu);
  t.u0 = uni(W->u0);
  t.block = uni(nd.block);
  t.nblocks = uni(nd.nblocks);
  t.R = t.nblocks * t.nu;
  t.C = uni(nd.cols);
  t.seg = uni(nd.seg);
  t.segp = uni(nd.segp);
  t.seg0 = uni(nd.seg0);
  t.Cl = ((t.C - t.seg0) / t.seg + 1) * t.segp;
  t.ldw = amp_ldrow(t.Cl);
  t.Rp = amp_round16(t.R);
  return t;
}

// Wl holds Rp x ldw floats, bl holds Rp; everything outside R x C is zero.
__device__ __forceinline__ void tile_load(const GQ NodeDev& nd, const Tile& t, float* Wl, float* bl) {
  for (int i = threadIdx.x; i < t.Rp * t.ldw; i += AMP_THREADS) Wl[i] = 0.f;
  for (int i = threadIdx.x; i < t.Rp; i += AMP_THREADS) bl[i] = 0.f;
  __syncthreads();
  for (int i = threadIdx.x; i < t.R * t.C; i += AMP_THREADS) {
    const int lr = i / t.C, c = i - lr * t.C;
    Wl[lr * t.ldw + t.lcol(c)] = nd.P[(long long)t.grow(lr) * t.C + c];
  }
  if (nd.has_bias)
    for (int lr = threadIdx.x; lr < t.R; lr += AMP_THREADS) bl[lr] = nd.P[(long long)nd.rows * t.C + t.grow(lr)];
  __syncthreads();
}

__device__ __forceinline__ void tile_store(const GQ NodeDev& nd, const Tile& t, const float* Wl, const float* bl) {
  __syncthreads();
  for (int i = threadIdx.x; i < t.R * t.C; i += AMP_THREADS) {
    const int lr = i / t.C, c = i - lr * t.C;
    nd.P[(long long)t.grow(lr) * t.C + c] = Wl[lr * t.ldw + t.lcol(c)];
  }
  if (nd.has_bias)
    for (int lr = threadIdx.x; lr < t.R; lr += AMP_THREADS) nd.P[(long long)nd.rows * t.C + t.grow(lr)] = bl[lr];
}

// G[row][c] += d[lr] * x[c] over the tile's rows; bias gradient alike.
__device__ __forceinline__ void tile_accumulate(const GQ NodeDev& nd, const Tile& t, const float* d, const float* x) {
  for (int i = threadIdx.x; i < t.R * t.C; i += AMP_THREADS) {
    const int lr = i / t.C, c = i - lr * t.C;
    float* g = nd.G + (long long)t.grow(lr) * t.C + c;
    *g = fmaf(d[lr], x[c], *g);
  }
  if (nd.has_bias)
    for (int lr = threadIdx.x; lr < t.R; lr += AMP_THREADS) nd.G[(long long)nd.rows * t.C + t.grow(lr)] += d[lr];
}

// The same with the accumulator in LDS (Gl laid out like the weight tile, gbl like the bias): x must be padded
// with zeros up to ldw.
__device__ __forceinline__ void tile_accumulate_lds(const Tile& t, LDSQ float* Gl, LDSQ float* gbl, const LDSQ float* d,
                                                    const LDSQ float* x) {
  for (int i = threadIdx.x; i < t.R * t.ldw; i += AMP_THREADS) {
    const int lr = i / t.ldw, c = i - lr * t.ldw;
    Gl[i] = fmaf(d[lr], x[c], Gl[i]);
  }
  for (int lr = threadIdx.x; lr < t.R; lr += AMP_THREADS) gbl[lr] += d[lr];
}

// One optimizer step on a value held in LDS (w) with slots in HBM.
struct OptCoef {
  float lr, mom, b1, b2, eps, c1, c2;  // c1 = 1/(1-b1^t), c2 = 1/(1-b2^t)
  int kind;
};

__device__ __forceinline__ OptCoef opt_coef(const GQ NodeDev& nd, unsigned tstep) {
  OptCoef o;
  o.kind = nd.opt;
  o.lr = nd.lr;
  o.mom = nd.mom;
  o.b1 = nd.b1;
  o.b2 = nd.b2;
  o.eps = nd.eps;
  o.c1 = o.c2 = 1.f;
  if (nd.opt == 2) {
    o.c1 = (float)(1.0 / (1.0 - pow((double)nd.b1, (double)tstep)));
    o.c2 = (float)(1.0 / (1.0 - pow((double)nd.b2, (double)tstep)));
  }
  return o;
}

__device__ __forceinline__ float opt_apply(const OptCoef& o, float w, float g, GQ float* M, GQ float* V, long long gi) {
  if (o.kind == 0) return w - o.lr * g;
  if (o.kind == 1) {
    const float m = fmaf(o.mom, M[gi], g);
    M[gi] = m;
    return w - o.lr * m;
  }
  const float m = fmaf(o.b1, M[gi], (1.f - o.b1) * g);
  const float v = fmaf(o.b2, V[gi], (1.f - o.b2) * g * g);
  M[gi] = m;
  V[gi] = v;
  return w - o.lr * (m * o.c1) / (sqrtf(v * o.c2) + o.eps);
}

__device__ __forceinline__ float opt_apply(const OptCoef& o, float w, float g, float* Mp, float* Vp, long long gi) {
  return opt_apply(o, w, g, (GQ float*)Mp, (GQ float*)Vp, gi);
}

// Applies the node's optimizer to the tile with the accumulated gradient
// (mean over `count` gradients unless the node sums), clears the accumulator.
// tstep is the 1-based number of this update.
__device__ __forceinline__ void tile_update(const GQ NodeDev& nd, const Tile& t, float* Wl, float* bl, unsigned count, unsigned tstep) {
  __syncthreads();
  const OptCoef o = opt_coef(nd, tstep);
  const float inv = nd.mean ? 1.f / (float)count : 1.f;
  for (int i = threadIdx.x; i < t.R * t.C; i += AMP_THREADS) {
    const int lr = i / t.C, c = i - lr * t.C;
    const long long gi = (long long)t.grow(lr) * t.C + c;
    const float g = nd.G[gi] * inv;
    nd.G[gi] = 0.f;
    Wl[lr * t.ldw + t.lcol(c)] = opt_apply(o, Wl[lr * t.ldw + t.lcol(c)], g, nd.M, nd.V, gi);
  }
  if (nd.has_bias)
    for (int lr = threadIdx.x; lr < t.R; lr += AMP_THREADS) {
      const long long gi = (long long)nd.rows * t.C + t.grow(lr);
      const float g = nd.G[gi] * inv;
      nd.G[gi] = 0.f;
      bl[lr] = opt_apply(o, bl[lr], g, nd.M, nd.V, gi);
    }
  __syncthreads();
}

// softmax cross-entropy over n <= 64 logits held in LDS, by wave 0.
// Writes dz[k] = p_k - [k == label]; returns loss and argmax through LDS words.
__device__ __forceinline__ void softmax_xent_wave0(const float* z, int n, int label, float* dz, float* s_loss, int* s_pred) {
  if (threadIdx.x < 64) {
    const int k = threadIdx.x;
    float v = k < n ? z[k] : -3.0e38f;
    float m = v;
    int am = k < n ? k : 0x7fffffff;
    for (int off = 32; off; off >>= 1) {
      const float om = __shfl_xor(m, off);
      const int oa = __shfl_xor(am, off);
      if (om > m || (om == m && oa < am)) {
        m = om;
        am = oa;
      }
    }
    float e = k < n ? expf(v - m) : 0.f;
    float s = e;
    for (int off = 32; off; off >>= 1) s += __shfl_xor(s, off);
    if (k < n) dz[k] = e / s - (k == label ? 1.f : 0.f);
    const float zl = __shfl(v, label);
    if (k == 0) {
      *s_loss = -(zl - m - logf(s));
      *s_pred = am;
    }
  }
  __syncthreads();
}

// ONE thread, at every update a worker applies: the controller's staleness-bounded admission reads this count.
__device__ __forceinline__ void note_update(const GQ AmpDev* D) {
  if (D->admit_bounded) __hip_atomic_fetch_add((GQ unsigned*)&D->ctl[3], 1u, __ATOMIC_RELAXED, AGENT);
}

// Arrival counter of a join: returns true for the arrival that completes
// `expect` parts; that caller resets the counter (the slot is not reused
// before the instance has retired) and may then post.  ONE thread, after a
// release fence covering its own part.  The completing arrival itself needs
// no fence: it reads nothing of the other parts, every writer had its part
// written back to memory before it arrived here, and the receiver of the post
// invalidates its caches before it reads.  (A fence here would be one more
// L2 write-back and invalidation per join, and an XCD's L2 serves those one
// at a time, 55-70 ns each: measured with 32 workgroups on one XCD.)
//
// That shortcut leans on how gfx950 implements agent-scope release (an L2
// write-back that completes before the writer's atomic is issued); the HIP
// memory model itself gives the receiver no happens-before edge to the other
// parts' writes.  Built with -DAMP_STRICT_JOIN the completing arrival makes the
// edge explicit: its read-modify-write acquires (and so synchronises with every
// earlier arrival's release fence through the counter's release sequence) and a
// release fence precedes the post.  The two builds must give the same results;
// a parity test runs both.
__device__ __forceinline__ bool join_arrive(GQ int* counter, int expect) {
#ifdef AMP_STRICT_JOIN
  const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_ACQ_REL, AGENT);
  if (old + 1 != expect) return false;
  __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, AGENT);
  fence_release();
  return true;
#else
  const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, AGENT);
  if (old + 1 != expect) return false;
  __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, AGENT);
  return true;
#endif
}

__device__ __forceinline__ bool join_arrive(int* counter, int expect) { return join_arrive((GQ int*)counter, expect); }

__device__ __forceinline__ float sigmoidf_(float x) { return 1.f / (1.f + expf(-x)); }
