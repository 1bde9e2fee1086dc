// Batched message handling for dense-cell workers.
//
// A worker that finds several messages waiting takes them together: their
// forward products share one pass over the LDS-resident weights, one acquire
// and one release fence cover the whole batch, and the arrival counters and
// ring tickets of the batch are handled by the lanes of one wave in parallel.
// A batch never straddles an update: it is cut at the backward message that
// brings the node's gradient count to min_update_frequency, so processing the
// batch at once is the same as processing its messages one by one in ring
// order.
//
// Gradients are not accumulated element by element per message.  Each
// backward message appends its (delta, input) pair to a per-worker list in
// HBM; when the node updates, the accumulated gradient
//     G = sum_k delta_k (x) input_k      (k in arrival order)
// is formed block by block in registers and goes straight into the optimizer
// step on the LDS-resident weights.
#pragma once

#define KB_MAX 32

__device__ __forceinline__ int round8(int v) { return (v + 7) & ~7; }

// Per-message scratch of the running batch, one per workgroup.
struct BatchMsg {
  int s[KB_MAX], n[KB_MAX], a[KB_MAX], b[KB_MAX], par[KB_MAX], L[KB_MAX], aux[KB_MAX];
  unsigned seq[KB_MAX];
  int fidx[KB_MAX], bidx[KB_MAX];
  int nF, nB;
};
__shared__ BatchMsg s_M;
__shared__ unsigned s_codes[KB_MAX];
__shared__ int s_n;

// Wave 0 looks at up to kmax consecutive ring entries at once and takes the
// leading run that is ready, cut so that at most `room` backward messages
// (those for which is_b(code) holds) are in it.  Returns the batch size, 0
// when the run is over.  s_codes / s_n are LDS.
template <class IsB>
__device__ int wait_batch(const AmpDev* D, const RingDev& r, unsigned& head, int kmax, int room, unsigned* s_codes,
                          int* s_n, IsB is_b) {
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    const unsigned ticket = head + lane;
    unsigned long long* slot = &r.ent[ticket & r.mask];
    const long long t0 = wall_clock64();
    unsigned spins = 0;
    int n = 0;
    unsigned code = 0;
    for (;;) {
      unsigned long long e = 0;
      if (lane < kmax) e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
      const bool ready = lane < kmax && (unsigned)(e >> 32) == ticket + 1u;
      const unsigned long long m = __ballot(ready);
      n = __builtin_ctzll(~m);   // leading run of ready entries (m has at most kmax <= 32 bits set)
      code = (unsigned)e;
      if (n > 0) break;
      int stop = 0;
      if (lane == 0 && (++spins & 7u) == 0u) {
        if (ld_u32(&D->ctl[0]) | ld_u32(&D->ctl[1])) {
          stop = 1;
        } else if (wall_clock64() - t0 > D->watchdog_ticks) {
          raise_abort(D, ABORT_WATCHDOG, blockIdx.x);
          stop = 1;
        }
      }
      stop = __shfl(stop, 0);
      if (stop) {
        // done is raised only when nothing is in flight; a last look avoids losing a message
        e = lane < kmax ? __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT) : 0ull;
        const unsigned long long m2 = __ballot(lane < kmax && (unsigned)(e >> 32) == ticket + 1u);
        n = __builtin_ctzll(~m2);
        code = (unsigned)e;
        if (n == 0 || ld_u32(&D->ctl[0]) != 0u) {
          n = 0;
        }
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    if (n > 0) {
      fence_acquire();
      // cut after the room-th backward message
      const bool b = lane < n && is_b(code);
      const unsigned long long mb = __ballot(b);
      const int before = __popcll(mb & ((1ull << lane) - 1ull));
      const unsigned long long cutm = __ballot(b && before + 1 == room);
      if (cutm) {
        const int cut = __builtin_ctzll(cutm) + 1;
        if (cut < n) n = cut;
      }
      if (lane < n) s_codes[lane] = code;
    }
    if (lane == 0) {
      *s_n = n;
      s_stat[0] += (unsigned long long)(wall_clock64() - t0);
      s_stat[1] += (unsigned long long)n;
    }
  }
  __syncthreads();
  const int n = *s_n;
  head += n;
  return n;
}

// ---------------------------------------------------------------- grouped-row products
// Y[k][r] = b[r] + sum_c Wl[r][c] X[k][c], k < K.  X rows have stride ldx, Y
// rows stride ldy (both multiples of 4, buffers 16-byte aligned, row count
// rounded up to 4; padding rows of X must hold finite values).
// Thread (p, g, r): output row r, k-rows 4g..4g+3, p-th column chunk.
__device__ void gemm_rows(const float* Wl, int ldw, int R, int C, const float* bl, const float* X, int ldx, int K,
                          float* part, float* Y, int ldy) {
  const int nkg = (K + 3) >> 2;
  int P = AMP_THREADS / (R * nkg);
  if (P < 1) P = 1;
  if (P > 8) P = 8;
  const int chunk = (((C + P - 1) / P) + 3) & ~3;
  const int total = R * nkg * P;
  for (int idx = threadIdx.x; idx < total; idx += AMP_THREADS) {
    const int p = idx / (R * nkg);
    const int rem = idx - p * R * nkg;
    const int g = rem / R, r = rem - g * R;
    const int c0 = p * chunk;
    int c1 = c0 + chunk;
    if (c1 > C) c1 = C;
    const float* w = Wl + r * ldw;
    const float* x0 = X + (4 * g) * ldx;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int c = c0;
    for (; c + 3 < c1; c += 4) {
      const float w0 = w[c], w1 = w[c + 1], w2 = w[c + 2], w3 = w[c + 3];
      const float4 xa = *(const float4*)(x0 + c);
      const float4 xb = *(const float4*)(x0 + ldx + c);
      const float4 xc = *(const float4*)(x0 + 2 * ldx + c);
      const float4 xd = *(const float4*)(x0 + 3 * ldx + c);
      a0 = fmaf(w0, xa.x, a0); a0 = fmaf(w1, xa.y, a0); a0 = fmaf(w2, xa.z, a0); a0 = fmaf(w3, xa.w, a0);
      a1 = fmaf(w0, xb.x, a1); a1 = fmaf(w1, xb.y, a1); a1 = fmaf(w2, xb.z, a1); a1 = fmaf(w3, xb.w, a1);
      a2 = fmaf(w0, xc.x, a2); a2 = fmaf(w1, xc.y, a2); a2 = fmaf(w2, xc.z, a2); a2 = fmaf(w3, xc.w, a2);
      a3 = fmaf(w0, xd.x, a3); a3 = fmaf(w1, xd.y, a3); a3 = fmaf(w2, xd.z, a3); a3 = fmaf(w3, xd.w, a3);
    }
    for (; c < c1; ++c) {
      const float wv = w[c];
      a0 = fmaf(wv, x0[c], a0);
      a1 = fmaf(wv, x0[ldx + c], a1);
      a2 = fmaf(wv, x0[2 * ldx + c], a2);
      a3 = fmaf(wv, x0[3 * ldx + c], a3);
    }
    float* o = (P == 1 ? Y : part + p * nkg * 4 * ldy) + (4 * g) * ldy + r;
    o[0] = a0;
    o[ldy] = a1;
    o[2 * ldy] = a2;
    o[3 * ldy] = a3;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < nkg * 4 * R; i += AMP_THREADS) {
    const int k = i / R, r = i - k * R;
    const int at = k * ldy + r;
    float s = P == 1 ? Y[at] : 0.f;
    if (P > 1)
      for (int p = 0; p < P; ++p) s += part[p * nkg * 4 * ldy + at];
    Y[at] = s + (bl ? bl[r] : 0.f);
  }
  __syncthreads();
}

// DX[k][c] = sum_r Wl[r][c] Dl[k][r], k < K.  Dl rows stride ldd, DX rows
// stride ldx (multiples of 4).  Thread (p, g, c): column c, k-rows 4g..4g+3,
// p-th row chunk.
__device__ void gemm_cols(const float* Wl, int ldw, int R, int C, const float* Dl, int ldd, int K, float* part,
                          float* DX, int ldx) {
  const int nkg = (K + 3) >> 2;
  int P = AMP_THREADS / (C * nkg);
  if (P < 1) P = 1;
  if (P > 8) P = 8;
  const int chunk = (((R + P - 1) / P) + 3) & ~3;
  const int total = C * nkg * P;
  for (int idx = threadIdx.x; idx < total; idx += AMP_THREADS) {
    const int p = idx / (C * nkg);
    const int rem = idx - p * C * nkg;
    const int g = rem / C, c = rem - g * C;
    const int r0 = p * chunk;
    int r1 = r0 + chunk;
    if (r1 > R) r1 = R;
    const float* d0 = Dl + (4 * g) * ldd;
    const float* w = Wl + c;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int r = r0;
    for (; r + 3 < r1; r += 4) {
      const float w0 = w[r * ldw], w1 = w[(r + 1) * ldw], w2 = w[(r + 2) * ldw], w3 = w[(r + 3) * ldw];
      const float4 da = *(const float4*)(d0 + r);
      const float4 db = *(const float4*)(d0 + ldd + r);
      const float4 dc = *(const float4*)(d0 + 2 * ldd + r);
      const float4 dd = *(const float4*)(d0 + 3 * ldd + r);
      a0 = fmaf(w0, da.x, a0); a0 = fmaf(w1, da.y, a0); a0 = fmaf(w2, da.z, a0); a0 = fmaf(w3, da.w, a0);
      a1 = fmaf(w0, db.x, a1); a1 = fmaf(w1, db.y, a1); a1 = fmaf(w2, db.z, a1); a1 = fmaf(w3, db.w, a1);
      a2 = fmaf(w0, dc.x, a2); a2 = fmaf(w1, dc.y, a2); a2 = fmaf(w2, dc.z, a2); a2 = fmaf(w3, dc.w, a2);
      a3 = fmaf(w0, dd.x, a3); a3 = fmaf(w1, dd.y, a3); a3 = fmaf(w2, dd.z, a3); a3 = fmaf(w3, dd.w, a3);
    }
    for (; r < r1; ++r) {
      const float wv = w[r * ldw];
      a0 = fmaf(wv, d0[r], a0);
      a1 = fmaf(wv, d0[ldd + r], a1);
      a2 = fmaf(wv, d0[2 * ldd + r], a2);
      a3 = fmaf(wv, d0[3 * ldd + r], a3);
    }
    float* o = (P == 1 ? DX : part + p * nkg * 4 * ldx) + (4 * g) * ldx + c;
    o[0] = a0;
    o[ldx] = a1;
    o[2 * ldx] = a2;
    o[3 * ldx] = a3;
  }
  __syncthreads();
  if (P > 1) {
    for (int i = threadIdx.x; i < nkg * 4 * C; i += AMP_THREADS) {
      const int k = i / C, c = i - k * C;
      const int at = k * ldx + c;
      float s = 0.f;
      for (int p = 0; p < P; ++p) s += part[p * nkg * 4 * ldx + at];
      DX[at] = s;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- pending gradients
// Entry e of a worker's list: pend + e * stride, [delta (R8 floats) | input (C8 floats)],
// R8 / C8 = tile rows / cols rounded up to 8, stride = R8 + C8.
struct Pend {
  float* base;
  int R8, C8, stride;
};

__device__ __forceinline__ Pend make_pend(const WorkerDev* W, const Tile& t) {
  Pend p;
  p.base = W->pend;
  p.R8 = round8(t.R);
  p.C8 = round8(t.C);
  p.stride = p.R8 + p.C8;
  return p;
}

// Appends K pairs held in LDS (delta rows stride ldd, input rows stride ldx) as entries first..first+K-1.
__device__ void pend_append(const Pend& p, unsigned first, const float* Dl, int ldd, int R, const float* X, int ldx,
                            int C, int K) {
  for (int i = threadIdx.x; i < K * p.stride; i += AMP_THREADS) {
    const int k = i / p.stride, j = i - k * p.stride;
    float v = 0.f;
    if (j < p.R8) {
      if (j < R) v = Dl[k * ldd + j];
    } else if (j - p.R8 < C) {
      v = X[k * ldx + j - p.R8];
    }
    p.base[(long long)(first + k) * p.stride + i - k * p.stride] = v;
  }
}

// The node's update from `count` pending pairs.  Thread blocks of 8 rows x 8
// columns (columns 4*bj..4*bj+3 and C8/2 + 4*bj..+3, so that the lanes of a
// wave read consecutive 16-byte pieces of an input row).  `stage` is LDS for
// 8 entries (8 * stride floats, 16-byte aligned).  tstep: 1-based update number.
__device__ void tile_update_deferred(const NodeDev& nd, const Tile& t, float* Wl, float* bl, const Pend& p,
                                     unsigned count, unsigned tstep, float* stage) {
  __syncthreads();
  const OptCoef o = opt_coef(nd, tstep);
  const float inv = nd.mean ? 1.f / (float)count : 1.f;
  const int nbr = p.R8 >> 3, nbc = p.C8 >> 3, nblk = nbr * nbc, half = p.C8 >> 1;
  for (int base = 0; base < nblk; base += AMP_THREADS) {
    const int blk = base + threadIdx.x;
    const bool act = blk < nblk;
    const int bi = act ? blk / nbc : 0, bj = act ? blk - bi * nbc : 0;
    float acc[64];
    float accb[8];
#pragma unroll
    for (int i = 0; i < 64; ++i) acc[i] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) accb[i] = 0.f;
    for (unsigned k0 = 0; k0 < count; k0 += 8) {
      const int kc = count - k0 < 8u ? (int)(count - k0) : 8;
      __syncthreads();
      const float4* src = (const float4*)(p.base + (long long)k0 * p.stride);
      for (int i = threadIdx.x; i < (kc * p.stride) >> 2; i += AMP_THREADS) ((float4*)stage)[i] = src[i];
      __syncthreads();
      if (act) {
        for (int kk = 0; kk < kc; ++kk) {
          const float* e = stage + kk * p.stride;
          const float4 d0 = *(const float4*)(e + 8 * bi), d1 = *(const float4*)(e + 8 * bi + 4);
          const float4 x0 = *(const float4*)(e + p.R8 + 4 * bj), x1 = *(const float4*)(e + p.R8 + half + 4 * bj);
          const float d[8] = {d0.x, d0.y, d0.z, d0.w, d1.x, d1.y, d1.z, d1.w};
          const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
#pragma unroll
          for (int i = 0; i < 8; ++i) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[i * 8 + j] = fmaf(d[i], x[j], acc[i * 8 + j]);
            accb[i] += d[i];
          }
        }
      }
    }
    if (act) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = 8 * bi + i;
        if (r >= t.R) continue;
        const long long grow = t.grow(r);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int c = (j < 4 ? 4 * bj + j : half + 4 * bj + j - 4);
          if (c >= t.C) continue;
          const long long gi = grow * t.C + c;
          Wl[r * t.ldw + c] = opt_apply(o, Wl[r * t.ldw + c], acc[i * 8 + j] * inv, nd.M, nd.V, gi);
        }
        if (bj == 0 && nd.has_bias) {
          const long long gi = (long long)nd.rows * t.C + grow;
          bl[r] = opt_apply(o, bl[r], accb[i] * inv, nd.M, nd.V, gi);
        }
      }
    }
  }
  __syncthreads();
}
