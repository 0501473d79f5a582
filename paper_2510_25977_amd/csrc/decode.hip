// bf16 decode path in ONE launch (M <= 32): the four products of the factored MLP (paper Alg. 2) as the four
// phases of a single kernel that works through a queue of tiles.
//
//   P1  T^T  = [Ug|Uu]^T X^T          16-column tiles, contraction over d cut into S1 ranges    (16 x 16 x 32 MFMAs)
//   P2  H^T  = SiLU(Vg^T Tg^T) .* (Vu^T Tu^T)     32-column tiles                               (32 x 32 x 16 MFMAs)
//   P4  Td^T = Ud^T H^T               16-column tiles, contraction over ffn cut into S4 ranges
//   P5  Y^T  = Vd^T Td^T              32-column tiles
//
// Four dependent launches cost about 11 us on this machine before any work is done, more than streaming the
// factors takes; one launch pays that once.  It does not pay off, though: handing a phase's result over inside the
// kernel (write-through store, acknowledgement, counter, poll, read) takes as long as a launch does, and a workgroup
// goes through its four or five items one after the other, so this variant measures slower than the four launches
// and is used on request only (SVDMLP_FLAG_STREAM_ONE_KERNEL).  The phases depend on each other through the (tiny)
// activations, so workgroups have to wait for each other inside the kernel.  That is made safe without assuming that the whole
// grid is resident: work items (tiles, in phase order) are handed out by an atomic counter, and an item only ever
// waits for items with smaller numbers.  A smaller number has been claimed earlier, by a workgroup that is running
// and that finishes its claimed items in order, so every wait ends whatever number of workgroups the device can
// hold at once, and whatever else runs beside the kernel.  Every wait is bounded all the same (POLL_LIMIT): on a
// timeout the context's error word is set and the workgroups drain the queue without computing.
//
// A workgroup requests the weight frags of its item before it waits for the item's dependency (weights depend on
// nothing), and claims its next item while it works on the current one, so HBM keeps streaming while the
// counters settle.  Activations and split-K partial tiles cross workgroups (and XCDs, whose L2s are not coherent
// with each other) as device-scope relaxed atomic stores (write-through); readers need no cache invalidate: caches
// are invalidated at kernel start, and nobody reads an activation before the counter that publishes it has been
// seen.  Cross-workgroup sums are added in range order by the last workgroup to take a tile's ticket, so results
// are bit-reproducible.  All counters are back at zero when the kernel ends (the last workgroup to leave resets
// them), so a forward carries no state from the host and can be recorded into a graph.
#include "common.h"

namespace svdmlp {

constexpr int QW = 8;                    // waves per workgroup
constexpr int QCAP = 8;                  // contraction blocks (of the phase's MFMA) a wave may hold per item
constexpr int POLL_LIMIT = 1 << 20;
constexpr int CTR_STRIDE = 32;           // uints: every counter in a cache line of its own
enum { C_QHEAD = 0, C_DONE1 = 1, C_DONE2 = 2, C_DONE4 = 3, C_EXIT = 4, C_ERR = 5 };

struct DqArgs {
  const char *wU, *wVg, *wVu, *wUd, *wVd;
  const uint16_t* X;
  uint16_t* Y;
  char *T, *H, *Td;                      // activation frags (one 32-row tile)
  float* part;                           // split-K partial tiles: P1's, then P4's
  int *tick1, *tick4;                    // tickets per 16-column tile, TICKET_STRIDE ints apart (zero between forwards)
  unsigned* ctr;                         // counters, CTR_STRIDE uints apart (zero between forwards; C_ERR is sticky)
  int M, d, r;
  int KB1, KBr, KBf, KBq;                // contraction blocks of 16: d, r, ffn, rd
  int t1, S1, t2, t4, S4, t5;            // tiles and ranges per phase
  int n1, n2, n4, n5;                    // items per phase
  int poll_limit;                        // polls a wait may take before it gives up (POLL_LIMIT; tests shrink it)
};

__device__ __forceinline__ f32x4 mfma16q(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// 16 bytes as four write-through dword stores
__device__ __forceinline__ void store16_wt(char* dst, const bf16x8& v) {
  const u32x4 u = __builtin_bit_cast(u32x4, v);
  unsigned* p = reinterpret_cast<unsigned*>(dst);
#pragma unroll
  for (int i = 0; i < 4; ++i) __hip_atomic_store(p + i, u[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct DqShared {
  f32x4 red[2][QW][4][64];               // staging of the waves' accumulator tiles (64 KiB)
  int item, ok, last;
};

// Thread 0 polls counter `which` until it shows `target`; everybody learns the outcome.  Two barriers.
__device__ __forceinline__ bool dq_wait(DqShared& sh, const DqArgs& a, int which, unsigned target) {
  if (threadIdx.x == 0) {
    int ok = 0;
    for (int polls = 0; polls < a.poll_limit; ++polls) {
      if (__hip_atomic_load(a.ctr + which * CTR_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) { ok = 1; break; }
      __builtin_amdgcn_s_sleep(1);
    }
    if (!ok) __hip_atomic_store(a.ctr + C_ERR * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sh.ok = ok;
  }
  __syncthreads();
  const bool ok = sh.ok != 0;
  __syncthreads();
  return ok;
}

// The calling wave's output stores have been acknowledged by memory -> count one finished tile.
__device__ __forceinline__ void dq_signal(const DqArgs& a, int which, int lane) {
  asm volatile("" ::: "memory");
  wait_vmcnt<0>();
  if (lane == 0) __hip_atomic_fetch_add(a.ctr + which * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------------------------------------
// P1 / P4: one 16-column tile over one contraction range, MT 16-row tiles of the batch.
// Lane l of a wave: row / column i = l % 16, contraction group g = l / 16 (k = 32 kb2 + 8 g .. + 7); a 16-row weight
// operand of block pair (2 kb2, 2 kb2 + 1) is lanes 16 hn .. and 32 + 16 hn .. of those two 32-row frags.
// ------------------------------------------------------------------------------------------------
template <bool FIRST, int MT>
__device__ __forceinline__ void dq_split_phase(DqShared& sh, const DqArgs& a, int it, bool& failed, unsigned& known) {
  const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
  const int S = FIRST ? a.S1 : a.S4;
  const int tile = it / S, sp = it % S;
  const int KB = FIRST ? a.KB1 : a.KBf, KB2 = KB / 2;
  const int kbs = (KB2 + S - 1) / S, kw = (kbs + QW - 1) / QW;
  int k0 = sp * kbs + w * kw, k1 = k0 + kw;
  const int kend = (sp + 1) * kbs < KB2 ? (sp + 1) * kbs : KB2;
  if (k1 > kend) k1 = kend;
  const int i = lane % 16, g = lane / 16, fsel = g / 2;
  const int tile32 = tile / 2, hn = tile % 2;
  const size_t wl = (size_t)(16 * hn + i + 32 * (g % 2)) * 16;
  // wU: [32-column tile][KB1] frags; wUd: [KBf][32-column tile] frags
  const char* wbase = FIRST ? a.wU + (size_t)tile32 * KB * FRAG_BYTES + wl : a.wUd + (size_t)tile32 * FRAG_BYTES + wl;
  const size_t wstride = FIRST ? (size_t)FRAG_BYTES : (size_t)(a.t4 / 2) * FRAG_BYTES;

  bf16x8 W[QCAP];
#pragma unroll
  for (int j = 0; j < QCAP; ++j)
    if (k0 + j < k1) W[j] = *reinterpret_cast<const bf16x8*>(wbase + (size_t)(2 * (k0 + j) + fsel) * wstride);
  if (!FIRST) {   // the ffn-wide activation must be complete
    if (!failed && !(known & (1u << C_DONE2))) {
      if (dq_wait(sh, a, C_DONE2, (unsigned)a.t2)) known |= 1u << C_DONE2;
      else failed = true;
    }
  }
  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (!failed) {
#pragma unroll
    for (int j = 0; j < QCAP; ++j)
      if (k0 + j < k1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          bf16x8 av;
          if (FIRST) {
            const int row = 16 * mt + i;
            av = *reinterpret_cast<const bf16x8*>(a.X + (size_t)(row < a.M ? row : a.M - 1) * a.d + 32 * (k0 + j) + 8 * g);
          } else {
            av = *reinterpret_cast<const bf16x8*>(a.H + (size_t)(2 * (k0 + j) + fsel) * FRAG_BYTES + (16 * mt + i + 32 * (g % 2)) * 16);
          }
          acc[mt] = mfma16q(W[j], av, acc[mt]);
        }
      }
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) sh.red[0][w][mt][lane] = acc[mt];
  __syncthreads();
  f32x4 v[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) v[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (w == 0) {
#pragma unroll
    for (int ww = 0; ww < QW; ++ww)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) v[mt] += sh.red[0][ww][mt][lane];
  }
  bool finish = w == 0;
  if (S > 1) {
    float* tpart = (FIRST ? a.part : a.part + (size_t)a.n1 * MT * 256) + (size_t)tile * S * (MT * 256);
    int* ticket = (FIRST ? a.tick1 : a.tick4) + tile * TICKET_STRIDE;
    if (w == 0) {
      float* mine = tpart + (size_t)sp * (MT * 256);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          __hip_atomic_store(&mine[(mt * 4 + e) * 64 + lane], v[mt][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("" ::: "memory");
      wait_vmcnt<0>();   // the stores have been acknowledged by memory
      if (lane == 0) sh.last = (__hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == S - 1);
    }
    __syncthreads();
    finish = w == 0 && sh.last != 0;
    if (finish) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) v[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
      constexpr int QB = 8 / MT;   // partial tiles in flight (8 KiB); additions in range order
      for (int q0 = 0; q0 < S; q0 += QB) {
        f32x4 tmp[QB][MT];
#pragma unroll
        for (int qq = 0; qq < QB; ++qq) {
          const int q = q0 + qq < S ? q0 + qq : S - 1;
          const float* src = tpart + (size_t)q * (MT * 256) + lane;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int e = 0; e < 4; ++e)
              tmp[qq][mt][e] = __hip_atomic_load(src + (mt * 4 + e) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int qq = 0; qq < QB; ++qq)
          if (q0 + qq < S) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) v[mt] += tmp[qq][mt];
          }
      }
      if (lane == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next forward
    }
  }
  if (finish) {
    // The tile is contraction block `frag` of the next product's activation, in chain order: element s of frag lane
    // (row, h) is column 8 (s / 4) + 4 h + s % 4: the four values of lane (m, g = h), then those of lane (m, g = 2 + h).
    // Lanes 0..31 write the frag lanes of rows 0..15, lanes 32..63 those of rows 16..31 (zeros if MT = 1).
    const int m = lane % 16, h = (lane / 16) % 2, up = lane / 32;
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float lo = __shfl(v[0][e], m + 16 * h, 64), hi = __shfl(v[0][e], m + 16 * (2 + h), 64);
      if (MT == 2) {
        const float lo1 = __shfl(v[MT - 1][e], m + 16 * h, 64), hi1 = __shfl(v[MT - 1][e], m + 16 * (2 + h), 64);
        lo = up ? lo1 : lo;
        hi = up ? hi1 : hi;
      } else if (up) {
        lo = 0.f;
        hi = 0.f;
      }
      o[e] = (__bf16)lo;
      o[4 + e] = (__bf16)hi;
    }
    size_t frag;
    if (FIRST) {
      const int p0 = 16 * tile;
      const int which = p0 >= a.r ? 1 : 0;
      frag = (size_t)which * (a.r / 16) + (p0 - which * a.r) / 16;
    } else {
      frag = (size_t)tile;
    }
    store16_wt((FIRST ? a.T : a.Td) + (frag * 64 + 16 * up + m + 32 * h) * 16, o);
    dq_signal(a, FIRST ? C_DONE1 : C_DONE4, lane);
  }
}

// ------------------------------------------------------------------------------------------------
// P2 / P5: one 32-column tile over the whole contraction (r resp. rd), 32 x 32 x 16 MFMAs, lane = activation row.
// ------------------------------------------------------------------------------------------------
template <bool GATE>
__device__ __forceinline__ void dq_whole_phase(DqShared& sh, const DqArgs& a, int tile, bool& failed, unsigned& known) {
  constexpr int NACC = GATE ? 2 : 1;
  const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
  const int KB = GATE ? a.KBr : a.KBq;
  const int kw = (KB + QW - 1) / QW;
  const int k0 = w * kw;
  const int k1 = k0 + kw < KB ? k0 + kw : KB;
  const size_t lane16 = (size_t)lane * 16;
  const char* w0 = (GATE ? a.wVg : a.wVd) + (size_t)tile * KB * FRAG_BYTES + lane16;
  const char* w1 = GATE ? a.wVu + (size_t)tile * KB * FRAG_BYTES + lane16 : nullptr;
  bf16x8 W0[QCAP], W1[GATE ? QCAP : 1];
#pragma unroll
  for (int j = 0; j < QCAP; ++j)
    if (k0 + j < k1) {
      W0[j] = *reinterpret_cast<const bf16x8*>(w0 + (size_t)(k0 + j) * FRAG_BYTES);
      if (GATE) W1[j] = *reinterpret_cast<const bf16x8*>(w1 + (size_t)(k0 + j) * FRAG_BYTES);
    }
  constexpr int DEP = GATE ? C_DONE1 : C_DONE4;
  if (!failed && !(known & (1u << DEP))) {
    if (dq_wait(sh, a, DEP, (unsigned)(GATE ? a.t1 : a.t4))) known |= 1u << DEP;
    else failed = true;
  }
  if (!GATE) {
    // the last phase also looks at the error word: a wait that ran out anywhere makes this forward's output NaN
    if (threadIdx.x == 0) sh.last = (int)__hip_atomic_load(a.ctr + C_ERR * CTR_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (sh.last) failed = true;
    __syncthreads();
  }
  f32x16 acc[NACC];
#pragma unroll
  for (int n = 0; n < NACC; ++n)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[n][e] = 0.f;
  if (!failed) {
    const char* act = (GATE ? a.T : a.Td) + lane16;
#pragma unroll
    for (int j = 0; j < QCAP; ++j)
      if (k0 + j < k1) {
        const bf16x8 av = *reinterpret_cast<const bf16x8*>(act + (size_t)(k0 + j) * FRAG_BYTES);
        acc[0] = mfma32(W0[j], av, acc[0]);
        if (GATE) {
          const bf16x8 au = *reinterpret_cast<const bf16x8*>(act + (size_t)(KB + k0 + j) * FRAG_BYTES);
          acc[NACC - 1] = mfma32(W1[j], au, acc[NACC - 1]);
        }
      }
  }
#pragma unroll
  for (int n = 0; n < NACC; ++n)
#pragma unroll
    for (int pl = 0; pl < 4; ++pl)
      sh.red[n][w][pl][lane] = f32x4{acc[n][4 * pl], acc[n][4 * pl + 1], acc[n][4 * pl + 2], acc[n][4 * pl + 3]};
  __syncthreads();
  // wave t < 2 finishes registers 8 t .. 8 t + 7 of the tile (= one chain-order frag)
  if (w < 2) {
    float v[NACC][8];
#pragma unroll
    for (int n = 0; n < NACC; ++n) {
#pragma unroll
      for (int s = 0; s < 8; ++s) v[n][s] = 0.f;
#pragma unroll
      for (int ww = 0; ww < QW; ++ww) {
        const f32x4 x0 = sh.red[n][ww][2 * w][lane], x1 = sh.red[n][ww][2 * w + 1][lane];
#pragma unroll
        for (int s = 0; s < 4; ++s) { v[n][s] += x0[s]; v[n][4 + s] += x1[s]; }
      }
    }
    if (GATE) {
      bf16x8 o;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const float gq = v[0][s];
        o[s] = (__bf16)(gq * __builtin_amdgcn_rcpf(1.0f + __expf(-gq)) * v[NACC - 1][s]);
      }
      store16_wt(a.H + (((size_t)2 * tile + w) * 64 + lane) * 16, o);
      asm volatile("" ::: "memory");
      wait_vmcnt<0>();
    } else {
      // lane = row m; slots s <-> columns 32 tile + 16 w + 8 (s / 4) + 4 h + s % 4
      const int il = lane % 32, h = lane / 32;
      if (il < a.M) {
        uint16_t* y = a.Y + (size_t)il * a.d + 32 * tile + 16 * w + 4 * h;
#pragma unroll
        for (int gq = 0; gq < 2; ++gq) {
          bf16x4 o;
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = failed ? (__bf16)__builtin_nanf("") : (__bf16)v[0][4 * gq + q];   // a forward whose wait ran out is visibly wrong
          *reinterpret_cast<bf16x4*>(y + 8 * gq) = o;
        }
      }
    }
  }
  if (GATE) {
    __syncthreads();   // both frags of the tile have been acknowledged
    if (threadIdx.x == 0) __hip_atomic_fetch_add(a.ctr + C_DONE2 * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <int MT>
__global__ __launch_bounds__(QW * 64) void k_decode(DqArgs a) {
  __shared__ DqShared sh;
  const int total = a.n1 + a.n2 + a.n4 + a.n5;
  if (threadIdx.x == 0)
    sh.item = (int)__hip_atomic_fetch_add(a.ctr + C_QHEAD * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  bool failed = false;
  unsigned known = 0;   // phases this workgroup has already seen complete (bit = counter index)
  while (true) {
    const int it = sh.item;
    __syncthreads();   // everybody has read the item before the slot is written again
    if (it >= total) break;
    // The next item is claimed now; its number is looked at when this item is done.  Not during the first phase:
    // the workgroups that start first would take a second item of it each, and the phase would take two rounds.
    unsigned nxt = 0;
    const bool ahead = it >= a.n1;
    if (ahead && threadIdx.x == 0)
      nxt = __hip_atomic_fetch_add(a.ctr + C_QHEAD * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (it < a.n1) dq_split_phase<true, MT>(sh, a, it, failed, known);
    else if (it < a.n1 + a.n2) dq_whole_phase<true>(sh, a, it - a.n1, failed, known);
    else if (it < a.n1 + a.n2 + a.n4) dq_split_phase<false, MT>(sh, a, it - a.n1 - a.n2, failed, known);
    else dq_whole_phase<false>(sh, a, it - a.n1 - a.n2 - a.n4, failed, known);
    __syncthreads();   // the staging buffer and the flags are free again
    if (!ahead && threadIdx.x == 0)
      nxt = __hip_atomic_fetch_add(a.ctr + C_QHEAD * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (threadIdx.x == 0) sh.item = (int)nxt;
    __syncthreads();
  }
  // the last workgroup to leave puts the counters back to zero for the next forward
  if (threadIdx.x == 0) {
    const unsigned old = __hip_atomic_fetch_add(a.ctr + C_EXIT * CTR_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == gridDim.x - 1) {
      for (int c = C_QHEAD; c <= C_EXIT; ++c)
        __hip_atomic_store(a.ctr + c * CTR_STRIDE, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

static int ceil_div(int x, int y) { return (x + y - 1) / y; }

// Decomposition of the four phases; false if the shape does not fit the kernel's per-wave register caps.
static bool plan_decode(const Plan& p, int64_t M, DqArgs* a) {
  if (M > 32 || p.d % 32 || p.ffn % 32) return false;
  const int mt = M <= 16 ? 1 : 2;
  a->KB1 = (int)(p.d / 16); a->KBr = (int)(p.r / 16); a->KBf = (int)(p.ffn / 16); a->KBq = (int)(p.rd / 16);
  a->t1 = (int)(2 * p.r / 16); a->t2 = (int)(p.ffn / 32); a->t4 = (int)(p.rd / 16); a->t5 = (int)(p.d / 32);
  if (a->t1 > 2048 || a->t4 > 2048) return false;
  a->S1 = stream_splits16(a->t1, a->KB1 / 2, mt);
  a->S4 = stream_splits16(a->t4, a->KBf / 2, mt);
  // more ranges if a wave would otherwise hold more than QCAP blocks
  while (ceil_div(ceil_div(a->KB1 / 2, a->S1), QW) > QCAP && a->S1 < 64) ++a->S1;
  while (ceil_div(ceil_div(a->KBf / 2, a->S4), QW) > QCAP && a->S4 < 64) ++a->S4;
  if (ceil_div(ceil_div(a->KB1 / 2, a->S1), QW) > QCAP || ceil_div(ceil_div(a->KBf / 2, a->S4), QW) > QCAP) return false;
  if (ceil_div(a->KBr, QW) > QCAP || ceil_div(a->KBq, QW) > QCAP) return false;
  a->n1 = a->t1 * a->S1; a->n2 = a->t2; a->n4 = a->t4 * a->S4; a->n5 = a->t5;
  const size_t part_floats = ((size_t)8 << 20) / 4;
  if (((size_t)a->n1 + (size_t)a->n4) * mt * 256 > part_floats) return false;
  return true;
}

char* decode_error_word(const Ctx* c) { return c->ws + c->plan.off_cnt + (size_t)C_ERR * CTR_STRIDE * sizeof(unsigned); }

bool bf16_decode_supported(const Ctx* c, int64_t M) {
  DqArgs a;
  return c->n_cus >= 8 && plan_decode(c->plan, M, &a);
}

int bf16_decode_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  DqArgs a;
  if (!plan_decode(p, M, &a)) return (int)hipErrorInvalidValue;
  a.wU = ws + p.off_wU; a.wVg = ws + p.off_wVg; a.wVu = ws + p.off_wVu; a.wUd = ws + p.off_wUd; a.wVd = ws + p.off_wVd;
  a.X = static_cast<const uint16_t*>(X); a.Y = static_cast<uint16_t*>(Y);
  a.T = ws + p.off_T; a.H = ws + p.off_H; a.Td = ws + p.off_Td;
  a.part = reinterpret_cast<float*>(ws + p.off_part);
  a.ctr = reinterpret_cast<unsigned*>(ws + p.off_cnt);                       // six counter lines
  a.tick1 = reinterpret_cast<int*>(ws + p.off_cnt + CNT_ONE_KERNEL_BYTES);   // the ticket lines of the four-launch path
  a.tick4 = a.tick1 + 2048 * TICKET_STRIDE;
  a.M = (int)M; a.d = (int)p.d; a.r = (int)p.r;
  a.poll_limit = c->poll_limit >= 0 ? c->poll_limit : POLL_LIMIT;
  static const char* const names[1] = {"k_decode"};
  const int ps = prof_open_forward(c, 1, names);
  const int G = c->n_cus > 0 ? (c->n_cus < 256 ? c->n_cus : 256) : 256;     // one workgroup per CU; any number works
  prof_mark(c, ps, 0, 0, st);
  if (M <= 16) hipLaunchKernelGGL(k_decode<1>, dim3(G), dim3(QW * 64), 0, st, a);
  else hipLaunchKernelGGL(k_decode<2>, dim3(G), dim3(QW * 64), 0, st, a);
  prof_mark(c, ps, 0, 1, st);
  return (int)hipGetLastError();
}

}  // namespace svdmlp
