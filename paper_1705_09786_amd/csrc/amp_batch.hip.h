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
// step on the weights (tree_update_from_pend, tree_update_stream).
#pragma once

#define KB_MAX 64

__device__ __forceinline__ int round8(int v) { return (v + 7) & ~7; }

// Per-message scratch of the running batch, one per workgroup.
struct BatchMsg {
  int s[KB_MAX], n[KB_MAX], a[KB_MAX], b[KB_MAX], par[KB_MAX], L[KB_MAX], aux[KB_MAX];
  unsigned seq[KB_MAX];
  int fidx[KB_MAX], bidx[KB_MAX];
  int off0[KB_MAX], off1[KB_MAX];   // float offsets of the input segments
  int dst0[KB_MAX], dst1[KB_MAX];   // float offsets where the input gradient's segments go
  int nF, nB;
};
__shared__ BatchMsg s_M;
__shared__ unsigned s_codes[KB_MAX];
__shared__ int s_n;

// One whole wave (any one) looks at up to kmax consecutive ring entries at once
// and takes the leading run that is ready, cut so that at most `room` backward
// messages (those for which is_b(code) holds) are in it.  Leaves the codes in
// s_codes and the batch size in *s_n (0 when the run is over) and returns it;
// no barrier.  s_codes / s_n are LDS.
template <class R, class IsB>
__device__ __forceinline__ int poll_batch(const GQ AmpDev* D, const R& r, unsigned head, int kmax, int room, unsigned* s_codes,
                                          int* s_n, IsB is_b) {
  {
    // a node whose carried gradient count already reaches its threshold (the host refuses to lower a threshold that
    // far) still cuts at the first backward message, so the pending list never grows past its end
    if (room < 1) room = 1;
    const int lane = threadIdx.x & 63;
    const unsigned ticket = head + lane;
    GQ unsigned long long* slot = (GQ unsigned long long*)&r.ent[ticket & r.mask];
    const long long t0 = wall_clock64();
    unsigned spins = 0;
    int n = 0;
    unsigned code = 0;
    for (;;) {
      unsigned long long e = 0;
      if (lane < kmax) e = __hip_atomic_load(slot, __ATOMIC_RELAXED, AGENT);
      const bool ready = lane < kmax && (unsigned)(e >> 32) == ticket + 1u;
      const unsigned long long m = __ballot(ready);
      n = ~m ? __builtin_ctzll(~m) : 64;   // leading run of ready entries
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
        n = ~m2 ? __builtin_ctzll(~m2) : 64;
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
      // a request to the worker itself (not an instance's message) is taken alone: the run is cut in front of it
      const unsigned long long mc = __ballot(lane < n && MSG_SLOT(code) == MSG_CTL_SLOT);
      if (mc) {
        const int first = __builtin_ctzll(mc);
        n = first == 0 ? 1 : first;
      }
      // cut after the room-th backward message
      const bool b = lane < n && is_b(code);
      const unsigned long long mb = __ballot(b);
      const int before = __popcll(mb & ((1ull << lane) - 1ull));   // lane < 64
      const unsigned long long cutm = __ballot(b && before + 1 == room);
      if (cutm) {
        const int cut = __builtin_ctzll(cutm) + 1;
        if (cut < n) n = cut;
      }
      if (lane < n) s_codes[lane] = code;
    }
    if (lane == 0) {
      *s_n = n;
      const unsigned long long now = wall_clock64();
      s_stat[0] += now - (unsigned long long)t0;
      s_stat[1] += (unsigned long long)n;
      s_stat[2] += 1;
      s_stat[3] = now;
    }
  }
  return *s_n;
}

// The same by wave 0 for the whole workgroup: ends with a barrier and advances head.
template <class R, class IsB>
__device__ __forceinline__ int wait_batch(const GQ AmpDev* D, const R& r, unsigned& head, int kmax, int room, unsigned* s_codes,
                                          int* s_n, IsB is_b) {
  if (threadIdx.x < 64) poll_batch(D, r, head, kmax, room, s_codes, s_n, is_b);
  lds_barrier();
  const int n = *s_n;
  head += n;
  return n;
}

// ---------------------------------------------------------------- grouped-row products on the matrix cores
// All operands live in LDS.  Weight tile Wl: Rp x ldw (Rp = 16 * NRB rows, ldw
// from amp_ldrow, zero outside R x C).  Row blocks X / Y / D hold 16 * NB rows
// each (one row per message or grouped row) with strides from amp_ldrow, so
// every 16-byte read below is aligned and bank-friendly.  Rows are independent
// of each other, so rows that carry no message may hold anything; but in a row
// that carries one, the padding columns (beyond C in X, beyond R in D) must be
// zero: they meet the weight tile's zero padding, and 0 x inf would be NaN.
//
// v_mfma_f32_16x16x4_f32: lane l supplies A[l%16][l/16] and B[l/16][l%16] and
// receives D[4*(l/16)+v][l%16], v = 0..3.  fp32 in, fp32 accumulate.
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x4f32((a), (b), (c), 0, 0, 0)

// Y[j][r] = b[r] + sum_c W[r][c] X[j][c]   (M = weight rows, N = messages, K = columns)
// Generic shape: one (row block, message block) item per wave at a time.
__device__ __noinline__ void mfma_rows_any(const LDSQ float* Wl, int ldw, int NRB, int NCG, const LDSQ float* bl,
                                           const LDSQ float* X, int ldx, int NB, LDSQ float* Y, int ldy) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  for (int item = wave; item < NRB * NB; item += AMP_THREADS / 64) {
    const int rb = item % NRB, nb = item / NRB;
    const LDSQ float* wp = Wl + (rb * 16 + i) * ldw + 4 * q;
    const LDSQ float* xp = X + (nb * 16 + i) * ldx + 4 * q;
    v4f acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g < NCG; ++g) {
      const v4f w0 = *(const LDSQ v4f*)(wp + 16 * g), x0 = *(const LDSQ v4f*)(xp + 16 * g);
      acc0 = MFMA(w0.x, x0.x, acc0);
      acc1 = MFMA(w0.y, x0.y, acc1);
      acc0 = MFMA(w0.z, x0.z, acc0);
      acc1 = MFMA(w0.w, x0.w, acc1);
    }
    const v4f b4 = *(const LDSQ v4f*)(bl + rb * 16 + 4 * q);
    *(LDSQ v4f*)(Y + (nb * 16 + i) * ldy + rb * 16 + 4 * q) = acc0 + acc1 + b4;
  }
}

// Fixed shape (NRB row blocks, NCG column groups, NB message blocks known at compile time): a wave owns row
// block rb for all message blocks, so a weight operand is read once for NB products and the unrolled loop keeps
// 2 NB (4 for NB = 1) independent accumulators going.
template <int NRB, int NCG, int NB>
__device__ __forceinline__ void mfma_rows_fixed(const LDSQ float* Wl, int ldw, const LDSQ float* bl, const LDSQ float* X, int ldx,
                                                LDSQ float* Y, int ldy) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  constexpr int NA = NB == 1 ? 4 : 2;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  for (int rb = wave; rb < NRB; rb += AMP_THREADS / 64) {
    const LDSQ float* wp = Wl + (rb * 16 + i) * ldw + 4 * q;
    const LDSQ float* xp = X + i * ldx + 4 * q;
    v4f acc[NB][NA];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int a = 0; a < NA; ++a) acc[nb][a] = zero;
    // operands of column group g + 1 are fetched from LDS before the products of group g are issued
    v4f w = *(const LDSQ v4f*)wp, x[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) x[nb] = *(const LDSQ v4f*)(xp + nb * 16 * ldx);
#pragma unroll
    for (int g = 0; g < NCG; ++g) {
      v4f wn = w, xn[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) xn[nb] = x[nb];
      if (g + 1 < NCG) {
        wn = *(const LDSQ v4f*)(wp + 16 * (g + 1));
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) xn[nb] = *(const LDSQ v4f*)(xp + nb * 16 * ldx + 16 * (g + 1));
        // the fetches above are issued before this point, the products below (which need acc[0][0]) after it
        asm volatile("" : "+v"(acc[0][0]) : : "memory");
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        acc[nb][0] = MFMA(w.x, x[nb].x, acc[nb][0]);
        acc[nb][1] = MFMA(w.y, x[nb].y, acc[nb][1]);
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        acc[nb][NA == 4 ? 2 : 0] = MFMA(w.z, x[nb].z, acc[nb][NA == 4 ? 2 : 0]);
        acc[nb][NA == 4 ? 3 : 1] = MFMA(w.w, x[nb].w, acc[nb][NA == 4 ? 3 : 1]);
      }
      w = wn;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) x[nb] = xn[nb];
    }
    const v4f b4 = *(const LDSQ v4f*)(bl + rb * 16 + 4 * q);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      v4f r = acc[nb][0] + acc[nb][1] + b4;
      if (NA == 4) r += acc[nb][2] + acc[nb][3];
      *(LDSQ v4f*)(Y + (nb * 16 + i) * ldy + rb * 16 + 4 * q) = r;
    }
  }
}

// Fixed shape with few row blocks (a node split over several tiles): (row block, message block) items dealt out to
// the waves, so that all waves work where the per-row-block mapping above would leave most of them idle.
template <int NRB, int NCG>
__device__ __forceinline__ void mfma_rows_items(const LDSQ float* Wl, int ldw, const LDSQ float* bl, const LDSQ float* X, int ldx,
                                                int NB, LDSQ float* Y, int ldy) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  for (int item = wave; item < NRB * NB; item += AMP_THREADS / 64) {
  const int rb = item % NRB, nb = item / NRB;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  const LDSQ float* wp = Wl + (rb * 16 + i) * ldw + 4 * q;
  const LDSQ float* xp = X + (nb * 16 + i) * ldx + 4 * q;
  v4f acc0 = zero, acc1 = zero, acc2 = zero, acc3 = zero;
  v4f w = *(const LDSQ v4f*)wp, x = *(const LDSQ v4f*)xp;
#pragma unroll
  for (int g = 0; g < NCG; ++g) {
    v4f wn = w, xn = x;
    if (g + 1 < NCG) {
      wn = *(const LDSQ v4f*)(wp + 16 * (g + 1));
      xn = *(const LDSQ v4f*)(xp + 16 * (g + 1));
      asm volatile("" : "+v"(acc0) : : "memory");
    }
    acc0 = MFMA(w.x, x.x, acc0);
    acc1 = MFMA(w.y, x.y, acc1);
    acc2 = MFMA(w.z, x.z, acc2);
    acc3 = MFMA(w.w, x.w, acc3);
    w = wn;
    x = xn;
  }
  const v4f b4 = *(const LDSQ v4f*)(bl + rb * 16 + 4 * q);
  *(LDSQ v4f*)(Y + (nb * 16 + i) * ldy + rb * 16 + 4 * q) = (acc0 + acc1) + (acc2 + acc3) + b4;
  }
}

// NRBT / NCGT = 0: shape known only at run time.  Ends with a barrier.
template <int NRBT, int NCGT>
__device__ __forceinline__ void mfma_rows(const LDSQ float* Wl, int ldw, int NRB, int NCG, const LDSQ float* bl,
                                          const LDSQ float* X, int ldx, int NB, LDSQ float* Y, int ldy) {
  if (NRBT && NRBT <= 4 && NB >= 2)
    mfma_rows_items<NRBT ? NRBT : 1, NCGT ? NCGT : 1>(Wl, ldw, bl, X, ldx, NB, Y, ldy);
  else if (NRBT && NB == 1)
    mfma_rows_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 1>(Wl, ldw, bl, X, ldx, Y, ldy);
  else if (NRBT && NB == 2)
    mfma_rows_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 2>(Wl, ldw, bl, X, ldx, Y, ldy);
  else if (NRBT && NB == 3)
    mfma_rows_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 3>(Wl, ldw, bl, X, ldx, Y, ldy);
  else if (NRBT && NB == 4)
    mfma_rows_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 4>(Wl, ldw, bl, X, ldx, Y, ldy);
  else
    mfma_rows_any(Wl, ldw, NRB, NCG, bl, X, ldx, NB, Y, ldy);
  lds_barrier();
}

// DX[j][c] = sum_r W[r][c] D[j][r]   (M = weight columns, N = messages, K = weight rows)
__device__ __noinline__ void mfma_cols_any(const LDSQ float* Wl, int ldw, int NRB, int NCG, const LDSQ float* Dl, int ldd,
                                           int NB, LDSQ float* DX, int ldx) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  for (int item = wave; item < NCG * NB; item += AMP_THREADS / 64) {
    const int cb = item % NCG, nb = item / NCG;
    const LDSQ float* wp = Wl + (4 * q) * ldw + cb * 16 + i;
    const LDSQ float* dp = Dl + (nb * 16 + i) * ldd + 4 * q;
    v4f acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int g = 0; g < NRB; ++g) {
      const v4f d0 = *(const LDSQ v4f*)(dp + 16 * g);
      const LDSQ float* w = wp + 16 * g * ldw;
      const float w0 = w[0], w1 = w[ldw], w2 = w[2 * ldw], w3 = w[3 * ldw];
      acc0 = MFMA(w0, d0.x, acc0);
      acc1 = MFMA(w1, d0.y, acc1);
      acc0 = MFMA(w2, d0.z, acc0);
      acc1 = MFMA(w3, d0.w, acc1);
    }
    *(LDSQ v4f*)(DX + (nb * 16 + i) * ldx + cb * 16 + 4 * q) = acc0 + acc1;
  }
}

// Fixed shape: a wave owns column group cb for all message blocks.
template <int NRB, int NCG, int NB>
__device__ __forceinline__ void mfma_cols_fixed(const LDSQ float* Wl, int ldw, const LDSQ float* Dl, int ldd, LDSQ float* DX,
                                                int ldx) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, i = lane & 15, q = lane >> 4;
  constexpr int NA = NB == 1 ? 4 : 2;
  const v4f zero = {0.f, 0.f, 0.f, 0.f};
  for (int cb = wave; cb < NCG; cb += AMP_THREADS / 64) {
    const LDSQ float* wp = Wl + (4 * q) * ldw + cb * 16 + i;
    const LDSQ float* dp = Dl + i * ldd + 4 * q;
    v4f acc[NB][NA];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int a = 0; a < NA; ++a) acc[nb][a] = zero;
    // operands of row block g + 1 are fetched from LDS before the products of block g are issued
    v4f d[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) d[nb] = *(const LDSQ v4f*)(dp + nb * 16 * ldd);
    float w0 = wp[0], w1 = wp[ldw], w2 = wp[2 * ldw], w3 = wp[3 * ldw];
#pragma unroll
    for (int g = 0; g < NRB; ++g) {
      v4f dn[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) dn[nb] = d[nb];
      float n0 = w0, n1 = w1, n2 = w2, n3 = w3;
      if (g + 1 < NRB) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) dn[nb] = *(const LDSQ v4f*)(dp + nb * 16 * ldd + 16 * (g + 1));
        const LDSQ float* w = wp + 16 * (g + 1) * ldw;
        n0 = w[0];
        n1 = w[ldw];
        n2 = w[2 * ldw];
        n3 = w[3 * ldw];
        asm volatile("" : "+v"(acc[0][0]) : : "memory");
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        acc[nb][0] = MFMA(w0, d[nb].x, acc[nb][0]);
        acc[nb][1] = MFMA(w1, d[nb].y, acc[nb][1]);
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        acc[nb][NA == 4 ? 2 : 0] = MFMA(w2, d[nb].z, acc[nb][NA == 4 ? 2 : 0]);
        acc[nb][NA == 4 ? 3 : 1] = MFMA(w3, d[nb].w, acc[nb][NA == 4 ? 3 : 1]);
      }
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) d[nb] = dn[nb];
      w0 = n0;
      w1 = n1;
      w2 = n2;
      w3 = n3;
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      v4f r = acc[nb][0] + acc[nb][1];
      if (NA == 4) r += acc[nb][2] + acc[nb][3];
      *(LDSQ v4f*)(DX + (nb * 16 + i) * ldx + cb * 16 + 4 * q) = r;
    }
  }
}

template <int NRBT, int NCGT>
__device__ __forceinline__ void mfma_cols(const LDSQ float* Wl, int ldw, int NRB, int NCG, const LDSQ float* Dl, int ldd,
                                          int NB, LDSQ float* DX, int ldx) {
  if (NRBT && NB == 1)
    mfma_cols_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 1>(Wl, ldw, Dl, ldd, DX, ldx);
  else if (NRBT && NB == 2)
    mfma_cols_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 2>(Wl, ldw, Dl, ldd, DX, ldx);
  else if (NRBT && NB == 3)
    mfma_cols_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 3>(Wl, ldw, Dl, ldd, DX, ldx);
  else if (NRBT && NB == 4)
    mfma_cols_fixed<NRBT ? NRBT : 1, NCGT ? NCGT : 1, 4>(Wl, ldw, Dl, ldd, DX, ldx);
  else
    mfma_cols_any(Wl, ldw, NRB, NCG, Dl, ldd, NB, DX, ldx);
  lds_barrier();
}

// ---------------------------------------------------------------- pending gradients
// Entry e of a worker's list in HBM: pend + e * stride, [delta (Rp floats) |
// input (Cp floats)], Rp / Cp = tile rows / cols rounded up to 16, zero padded.
struct Pend {
  float* base;
  int Rp, Cp, stride;
};

__device__ __forceinline__ Pend make_pend(const GQ WorkerDev* W, const Tile& t) {
  Pend p;
  p.base = (float*)uni_gq<float>(W->pend);
  p.Rp = t.Rp;
  p.Cp = amp_round16(t.Cl);
  p.stride = p.Rp + p.Cp;
  return p;
}
