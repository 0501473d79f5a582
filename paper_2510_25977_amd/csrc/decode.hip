// bf16 decode path in ONE persistent launch (M <= 32): the four products of the factored MLP
// (paper Alg. 2) as four phases of a single kernel, one workgroup per CU.
//
//   D1  T^T  = [Ug|Uu]^T X^T          split-K over d, over workgroups
//   D2  H^T  = SiLU(Vg^T Tg^T) .* (Vu^T Tu^T)
//   D4  Td^T = Ud^T H^T               split-K over ffn, over workgroups
//   D5  Y^T  = Vd^T Td^T
//
// The forward is weight-bandwidth bound (every factor element is read exactly once) and the phases depend on
// each other only through tiny activations, so the kernel keeps HBM busy while it synchronises: every wave
// knows from its block id which weight frags it will need in every phase; the frags of the first two phases
// are requested at kernel start and those of each later phase as soon as the previous phase's MFMAs are
// issued, i.e. always one phase ahead of the dependency they wait for.
//
// Wave 0 of a workgroup is the *reducer*: it never loads weights, so its memory counter is never blocked behind
// a prefetch (loads, stores and atomics of a wave complete in order).  It sums the streamers' partial tiles
// from LDS, exchanges partials with other workgroups, takes tickets, signals and polls.  Waves 1..11 are
// *streamers*: they only load frags and issue MFMAs, and meet the reducer at workgroup barriers that do not
// drain outstanding loads.
//
// Phases are separated by completion counters in device memory (monotonic across forwards, compared with a
// generation number: no reset, no second kernel).  Activations and partial tiles cross workgroups (and XCDs,
// whose L2s are not coherent with each other) as device-scope relaxed atomic stores (write-through).  Readers
// need no cache invalidate: caches are invalidated at kernel start, and within the kernel nobody reads an
// activation buffer before the counter that publishes it has been seen, so no stale line can exist; nobody pays
// an L2 write-back or invalidate.  Cross-workgroup sums are
// added in a fixed order by the last workgroup to take a ticket, so results are bit-reproducible.
//
// Every wait is bounded: a reducer that polls longer than POLL_LIMIT gives up, raises the context's error word
// and its workgroup skips the remaining phases, so every wave of the grid exits even if the grid could not
// become co-resident.
#include "common.h"

namespace svdmlp {

constexpr int DW = 12;                   // waves per workgroup: 1 reducer + 11 streamers
constexpr int NS = DW - 1;               // streamer waves
constexpr int CAP1 = 4, CAP2 = 4, CAP4 = 6, CAP5 = 4;   // weight frags a streamer may hold per phase (per work item)
constexpr int VB2 = 2;                   // D2 work items per workgroup
constexpr int POLL_LIMIT = 1 << 21;

struct DecodeArgs {
  const char *wU, *wVg, *wVu, *wUd, *wVd;
  const uint16_t* X;
  uint16_t* Y;
  char *T, *H, *Td;                      // activation frags
  float* part;                           // split-K partial tiles
  unsigned long long* done;              // [0] D1 tiles done, [1] D2 items done, [2] D4 tiles done (monotonic)
  unsigned long long* flags;             // [phase][workgroup], one 128-byte line each: generation whose phase is complete
  int* tickets;                          // [0, t1) D1 tiles, [2048, 2048 + t4) D4 tiles (zero between forwards)
  int* err;
  unsigned long long gen;                // 1-based forward number of this context
  int M, d, r, G;
  int KB1, t1, S1, kbs1, kw1;            // contraction blocks, tiles, splits, blocks per split / per streamer
  int KB2, t2, kw2;
  int KB4, t4, S4, kbs4, kw4;
  int KB5, t5, kw5;
};

// workgroup barrier for LDS hand-offs: waits for this wave's LDS traffic only, never for its global loads
__device__ __forceinline__ void bar_lds() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ void store_frag_wt(char* dst, const bf16x8& v) {
  const u32x4 u = __builtin_bit_cast(u32x4, v);  // 16 bytes as four write-through dword stores
  unsigned* p = reinterpret_cast<unsigned*>(dst);
#pragma unroll
  for (int i = 0; i < 4; ++i) __hip_atomic_store(p + i, u[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS staging of accumulator tiles: red[acc][streamer][lane][16]
typedef float RedBuf[2][NS][64][16];

__device__ __forceinline__ void red_write(RedBuf& red, int n, int ws, int lane, const f32x16& acc) {
  f32x4* dst = reinterpret_cast<f32x4*>(&red[n][ws][lane][0]);
#pragma unroll
  for (int q = 0; q < 4; ++q) dst[q] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
}
// sum over the first nw streamers, in order
__device__ __forceinline__ void red_sum(const RedBuf& red, int n, int nw, int lane, float (&v)[16]) {
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] = 0.f;
  for (int ww = 0; ww < nw; ++ww) {
    const f32x4* src = reinterpret_cast<const f32x4*>(&red[n][ww][lane][0]);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 x = src[q];
      v[4 * q] += x[0]; v[4 * q + 1] += x[1]; v[4 * q + 2] += x[2]; v[4 * q + 3] += x[3];
    }
  }
}

// Reducer only.  Cross-workgroup part of a split-K tile: publish this workgroup's partial, take a ticket, and
// if it was the last one add all S partials in split order into v.  Returns whether this workgroup finishes the tile.
__device__ __forceinline__ bool exchange_partials(float* part_tile, int S, int sp, int* ticket, int lane, float (&v)[16]) {
  if (S == 1) return true;
  float* mine = part_tile + (size_t)sp * 1024;
#pragma unroll
  for (int e = 0; e < 16; ++e) __hip_atomic_store(&mine[e * 64 + lane], v[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("" ::: "memory");
  wait_vmcnt<0>();   // the stores have been acknowledged by memory
  int old = 0;
  if (lane == 0) old = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  old = __builtin_amdgcn_readfirstlane(old);
  if (old != S - 1) return false;
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] = 0.f;
  for (int q0 = 0; q0 < S; q0 += 2) {   // two partial tiles of loads in flight; additions stay in split order
    float tmp[2][16];
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
      const int q = q0 + qq < S ? q0 + qq : S - 1;
      const float* src = part_tile + (size_t)q * 1024 + lane;
#pragma unroll
      for (int e = 0; e < 16; ++e) tmp[qq][e] = __hip_atomic_load(src + e * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll
    for (int qq = 0; qq < 2; ++qq)
      if (q0 + qq < S) {
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] += tmp[qq][e];
      }
  }
  if (lane == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next forward
  return true;
}

constexpr int FLAG_STRIDE = 16;   // in 8-byte words: every workgroup polls a cache line of its own

// Reducer only: the stores above are in memory -> bump a completion counter.  Whoever brings it to `target`
// tells every workgroup by writing the generation into that workgroup's own flag line, so that the waiting
// reducers do not all poll (and delay the atomics on) one address.
__device__ __forceinline__ void signal_done(unsigned long long* ctr, unsigned long long n, unsigned long long target,
                                            unsigned long long* flags, unsigned long long gen, int G, int lane) {
  asm volatile("" ::: "memory");
  wait_vmcnt<0>();
  if (n == 0) return;
  unsigned long long old = 0;
  if (lane == 0) old = __hip_atomic_fetch_add(ctr, n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)old), hi = __builtin_amdgcn_readfirstlane((unsigned)(old >> 32));
  old = ((unsigned long long)hi << 32) | lo;
  if (old + n == target)
    for (int g = lane; g < G; g += 64)
      __hip_atomic_store(&flags[(size_t)g * FLAG_STRIDE], gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Reducer only: poll this workgroup's flag until it shows generation `gen`; false on timeout.
__device__ __forceinline__ bool poll_flag(const unsigned long long* flag, unsigned long long gen) {
  int polls = 0;
  while (true) {
    unsigned long long c = __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)c), hi = __builtin_amdgcn_readfirstlane((unsigned)(c >> 32));
    c = ((unsigned long long)hi << 32) | lo;
    if (c >= gen) return true;
    if (++polls >= POLL_LIMIT) return false;
    __builtin_amdgcn_s_sleep(2);
  }
}

__global__ __launch_bounds__(DW * 64) void k_decode(DecodeArgs a) {
  __shared__ __attribute__((aligned(16))) RedBuf red;
  __shared__ int s_ok;
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const bool reducer = w == 0;
  const int ws = w - 1;                                   // streamer index
  const int il = lane % 32, h = lane / 32;
  const int b = blockIdx.x;
  const size_t lane16 = (size_t)lane * 16;

  // ---------------- work items ----------------
  const bool has1 = b < a.t1 * a.S1;                       // D1: tile b / S1, split b % S1
  const int tile1 = b / a.S1, sp1 = b % a.S1;
  const int k1b = sp1 * a.kbs1 + ws * a.kw1;
  int k1e = k1b + a.kw1;
  { const int e = (sp1 + 1) * a.kbs1 < a.KB1 ? (sp1 + 1) * a.kbs1 : a.KB1; k1e = k1e < e ? k1e : e; }
  const int k2b = ws * a.kw2;                              // D2: tiles b and b + G, whole contraction
  const int k2e = (k2b + a.kw2 < a.KB2) ? k2b + a.kw2 : a.KB2;
  const bool has4 = b < a.t4 * a.S4;                       // D4: tile b / S4, split b % S4
  const int tile4 = b / a.S4, sp4 = b % a.S4;
  const int k4b = sp4 * a.kbs4 + ws * a.kw4;
  int k4e = k4b + a.kw4;
  { const int e = (sp4 + 1) * a.kbs4 < a.KB4 ? (sp4 + 1) * a.kbs4 : a.KB4; k4e = k4e < e ? k4e : e; }
  const bool has5 = b < a.t5;                              // D5: tile b, whole contraction
  const int k5b = ws * a.kw5;
  const int k5e = (k5b + a.kw5 < a.KB5) ? k5b + a.kw5 : a.KB5;
  const int n1 = (a.kbs1 + a.kw1 - 1) / a.kw1, n2 = (a.KB2 + a.kw2 - 1) / a.kw2;   // streamers that hold data
  const int n4 = (a.kbs4 + a.kw4 - 1) / a.kw4, n5 = (a.KB5 + a.kw5 - 1) / a.kw5;

  bf16x8 W1[CAP1], X1[CAP1], W2g[VB2][CAP2], W2u[VB2][CAP2];
  if (!reducer) {
    // ---- requests at kernel start: D1 weights and X ----
    const uint16_t* xrow = a.X + (size_t)(il < a.M ? il : a.M - 1) * a.d + 8 * h;   // natural order: X[il][16 kb + 8 h ..]
#pragma unroll
    for (int j = 0; j < CAP1; ++j)
      if (has1 && k1b + j < k1e) {
        W1[j] = *reinterpret_cast<const bf16x8*>(a.wU + ((size_t)tile1 * a.KB1 + k1b + j) * FRAG_BYTES + lane16);
        X1[j] = *reinterpret_cast<const bf16x8*>(xrow + 16 * (k1b + j));
      }
    // ---- D1 ----
    if (has1) {
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int j = 0; j < CAP1; ++j)
        if (k1b + j < k1e) acc = mfma32(W1[j], X1[j], acc);
      if (ws < n1) red_write(red, 0, ws, lane, acc);
    }
    // ---- D2 weights: requested only now, so that they do not queue in front of the (small) D1 weights; they
    // stream while the reducers exchange the D1 partials ----
#pragma unroll
    for (int v = 0; v < VB2; ++v) {
      const int tile = b + v * a.G;
#pragma unroll
      for (int j = 0; j < CAP2; ++j)
        if (tile < a.t2 && k2b + j < k2e) {
          const size_t off = ((size_t)tile * a.KB2 + k2b + j) * FRAG_BYTES + lane16;
          W2g[v][j] = *reinterpret_cast<const bf16x8*>(a.wVg + off);
          W2u[v][j] = *reinterpret_cast<const bf16x8*>(a.wVu + off);
        }
    }
  }
  bar_lds();
  if (reducer) {
    bool ok = true;
    if (has1) {
      float v[16];
      red_sum(red, 0, n1, lane, v);
      if (exchange_partials(a.part + (size_t)tile1 * a.S1 * 1024, a.S1, sp1, &a.tickets[tile1], lane, v)) {
        const int p0 = 32 * tile1;
        const int which = p0 >= a.r ? 1 : 0;
        const size_t frag = (size_t)which * (a.r / 16) + (p0 - which * a.r) / 16;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          bf16x8 o;
#pragma unroll
          for (int s = 0; s < 8; ++s) o[s] = (__bf16)v[8 * t + s];
          store_frag_wt(a.T + ((frag + t) * 64 + lane) * 16, o);
        }
        signal_done(&a.done[0], 1, a.gen * (unsigned long long)a.t1, a.flags, a.gen, a.G, lane);
      }
    }
    ok = poll_flag(&a.flags[(size_t)b * FLAG_STRIDE], a.gen);
    if (lane == 0) s_ok = ok;
  }
  bar_lds();
  bool ok = s_ok != 0;

  // ---------------- D2 ----------------
  bf16x8 W4[CAP4];
  if (!reducer && ok) {
    bf16x8 A2g[CAP2], A2u[CAP2];
#pragma unroll
    for (int j = 0; j < CAP2; ++j)
      if (k2b + j < k2e) {
        A2g[j] = *reinterpret_cast<const bf16x8*>(a.T + (size_t)(k2b + j) * FRAG_BYTES + lane16);
        A2u[j] = *reinterpret_cast<const bf16x8*>(a.T + (size_t)(a.KB2 + k2b + j) * FRAG_BYTES + lane16);
      }
    // items are processed one after the other so that only one (G, P) accumulator pair is live
    static_assert(VB2 == 2, "barrier sequence below is written for two items");
#pragma unroll
    for (int v = 0; v < VB2; ++v) {
      f32x16 g, p;
#pragma unroll
      for (int e = 0; e < 16; ++e) { g[e] = 0.f; p[e] = 0.f; }
      if (b + v * a.G < a.t2) {
#pragma unroll
        for (int j = 0; j < CAP2; ++j)
          if (k2b + j < k2e) {
            g = mfma32(W2g[v][j], A2g[j], g);
            p = mfma32(W2u[v][j], A2u[j], p);
          }
      }
      if (v == 1) {
        // D4 weights: one phase ahead (Ud frags are contraction-block major: [kb][q tile])
#pragma unroll
        for (int j = 0; j < CAP4; ++j)
          if (has4 && k4b + j < k4e)
            W4[j] = *reinterpret_cast<const bf16x8*>(a.wUd + ((size_t)(k4b + j) * a.t4 + tile4) * FRAG_BYTES + lane16);
        bar_lds();                   // B0: reducer has read item 0
      }
      if (ws < n2) { red_write(red, 0, ws, lane, g); red_write(red, 1, ws, lane, p); }
      bar_lds();                     // A_v: item v staged
    }
  } else if (!reducer) {
    bar_lds(); bar_lds(); bar_lds();
  } else {
    unsigned long long items = 0;
#pragma unroll
    for (int v = 0; v < VB2; ++v) {
      bar_lds();                     // A_v
      const int tile = b + v * a.G;
      float gs[16], ps[16];
      const bool live = ok && tile < a.t2;
      if (live) { red_sum(red, 0, n2, lane, gs); red_sum(red, 1, n2, lane, ps); }
      if (v + 1 < VB2) bar_lds();    // B_v
      if (live) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          bf16x8 o;
#pragma unroll
          for (int s = 0; s < 8; ++s) {
            const float x = gs[8 * t + s];
            o[s] = (__bf16)(x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)) * ps[8 * t + s]);
          }
          store_frag_wt(a.H + (((size_t)2 * tile + t) * 64 + lane) * 16, o);
        }
        ++items;
      }
    }
    signal_done(&a.done[1], items, a.gen * (unsigned long long)a.t2, a.flags + (size_t)a.G * FLAG_STRIDE, a.gen, a.G, lane);
    if (ok) ok = poll_flag(&a.flags[((size_t)a.G + b) * FLAG_STRIDE], a.gen);
    if (lane == 0) s_ok = ok;
  }
  bar_lds();
  ok = s_ok != 0;

  // ---------------- D4 ----------------
  bf16x8 W5[CAP5];
  if (!reducer) {
    if (ok && has4) {
      bf16x8 A4[CAP4];
#pragma unroll
      for (int j = 0; j < CAP4; ++j)
        if (k4b + j < k4e) A4[j] = *reinterpret_cast<const bf16x8*>(a.H + (size_t)(k4b + j) * FRAG_BYTES + lane16);
      f32x16 acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int j = 0; j < CAP4; ++j)
        if (k4b + j < k4e) acc = mfma32(W4[j], A4[j], acc);
      if (ws < n4) red_write(red, 0, ws, lane, acc);
    }
    // D5 weights: one phase ahead
#pragma unroll
    for (int j = 0; j < CAP5; ++j)
      if (ok && has5 && k5b + j < k5e) W5[j] = *reinterpret_cast<const bf16x8*>(a.wVd + ((size_t)b * a.KB5 + k5b + j) * FRAG_BYTES + lane16);
  }
  bar_lds();
  if (reducer) {
    if (ok && has4) {
      float v[16];
      red_sum(red, 0, n4, lane, v);
      float* part4 = a.part + (size_t)a.t1 * a.S1 * 1024;   // D4's partials follow D1's
      if (exchange_partials(part4 + (size_t)tile4 * a.S4 * 1024, a.S4, sp4, &a.tickets[2048 + tile4], lane, v)) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          bf16x8 o;
#pragma unroll
          for (int s = 0; s < 8; ++s) o[s] = (__bf16)v[8 * t + s];
          store_frag_wt(a.Td + (((size_t)2 * tile4 + t) * 64 + lane) * 16, o);
        }
        signal_done(&a.done[2], 1, a.gen * (unsigned long long)a.t4, a.flags + (size_t)2 * a.G * FLAG_STRIDE, a.gen, a.G, lane);
      }
    }
    if (ok) ok = poll_flag(&a.flags[((size_t)2 * a.G + b) * FLAG_STRIDE], a.gen);
    if (lane == 0) s_ok = ok;
  }
  bar_lds();
  ok = s_ok != 0;

  // ---------------- D5 ----------------
  if (!reducer && ok && has5) {
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int j = 0; j < CAP5; ++j)
      if (k5b + j < k5e) {
        const bf16x8 av = *reinterpret_cast<const bf16x8*>(a.Td + (size_t)(k5b + j) * FRAG_BYTES + lane16);
        acc = mfma32(W5[j], av, acc);
      }
    if (ws < n5) red_write(red, 0, ws, lane, acc);
  }
  bar_lds();
  if (reducer) {
    if (ok && has5 && il < a.M) {
      // lane = row m; register 8 t + s <-> column 32 tile + 16 t + 8 (s / 4) + 4 h + s % 4
      float v[16];
      red_sum(red, 0, n5, lane, v);
      uint16_t* y = a.Y + (size_t)il * a.d + 32 * b + 4 * h;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          bf16x4 o;
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = (__bf16)v[8 * t + 4 * g + i];
          *reinterpret_cast<bf16x4*>(y + 16 * t + 8 * g) = o;
        }
    }
    if (!ok && lane == 0) __hip_atomic_store(a.err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

static int ceil_div(int x, int y) { return (x + y - 1) / y; }

// Decomposition of the four phases over G workgroups; false if the shape does not fit the kernel's register caps.
static bool plan_decode(const Plan& p, int G, DecodeArgs* a) {
  a->G = G;
  a->KB1 = (int)(p.d / 16); a->t1 = (int)(2 * p.r / 32);
  a->KB2 = (int)(p.r / 16); a->t2 = (int)(p.ffn / 32);
  a->KB4 = (int)(p.ffn / 16); a->t4 = (int)(p.rd / 32);
  a->KB5 = (int)(p.rd / 16); a->t5 = (int)(p.d / 32);
  if (a->t1 > G || a->t4 > G || a->t5 > G || a->t2 > VB2 * G || a->t1 > 2048 || a->t4 > 2048) return false;
  a->S1 = G / a->t1; a->kbs1 = ceil_div(a->KB1, a->S1); a->kw1 = ceil_div(a->kbs1, NS);
  a->kw2 = ceil_div(a->KB2, NS);
  a->S4 = G / a->t4; a->kbs4 = ceil_div(a->KB4, a->S4); a->kw4 = ceil_div(a->kbs4, NS);
  a->kw5 = ceil_div(a->KB5, NS);
  if (a->kw1 > CAP1 || a->kw2 > CAP2 || a->kw4 > CAP4 || a->kw5 > CAP5) return false;
  const size_t part_floats = ((size_t)8 << 20) / 4;
  if (((size_t)a->t1 * a->S1 + (size_t)a->t4 * a->S4) * 1024 > part_floats) return false;
  return true;
}

bool bf16_decode_supported(const Ctx* c) {
  DecodeArgs a;
  return c->n_cus >= 64 && plan_decode(c->plan, c->n_cus < 256 ? c->n_cus : 256, &a);
}

int bf16_decode_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  DecodeArgs a;
  if (!plan_decode(p, c->n_cus < 256 ? c->n_cus : 256, &a)) return (int)hipErrorInvalidValue;
  a.wU = ws + p.off_wU; a.wVg = ws + p.off_wVg; a.wVu = ws + p.off_wVu; a.wUd = ws + p.off_wUd; a.wVd = ws + p.off_wVd;
  a.X = static_cast<const uint16_t*>(X); a.Y = static_cast<uint16_t*>(Y);
  a.T = ws + p.off_T; a.H = ws + p.off_H; a.Td = ws + p.off_Td;
  a.part = reinterpret_cast<float*>(ws + p.off_part);
  a.tickets = reinterpret_cast<int*>(ws + p.off_cnt);                       // ints [0, 4096)
  a.done = reinterpret_cast<unsigned long long*>(ws + p.off_cnt + 16384);   // three 64-bit counters
  a.err = reinterpret_cast<int*>(ws + p.off_cnt + 16384 + 64);
  a.flags = reinterpret_cast<unsigned long long*>(ws + p.off_cnt + 32768);       // 3 phases x 256 workgroups x 128 B
  a.gen = ++c->decode_gen;
  a.M = (int)M; a.d = (int)p.d; a.r = (int)p.r;
  static const char* const names[1] = {"k_decode"};
  const int ps = prof_open_forward(c, 1, names);
  prof_mark(c, ps, 0, 0, st);
  hipLaunchKernelGGL(k_decode, dim3(a.G), dim3(DW * 64), 0, st, a);
  prof_mark(c, ps, 0, 1, st);
  const int e = (int)hipGetLastError();
  if (e) --c->decode_gen;
  return e;
}

}  // namespace svdmlp
