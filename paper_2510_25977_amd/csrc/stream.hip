// bf16 weight-streaming (decode) path: M <= 128 rows, weight-bandwidth bound.
//
// Each of the four products of the factored MLP (paper Alg. 2) is one launch of k_stream (up to 32 rows D1, D4 and,
// while it has fewer than 256 tiles of 32 columns, D5: k_stream16, 16-column tiles; from 33 rows on the row tiles of
// D1, D4 and D5 may get workgroups of their own):
//   D1  T^T  = [Ug|Uu]^T X^T          split-K over d
//   D2  H^T  = SiLU(Vg^T Tg^T) .* (Vu^T Tu^T)
//   D4  Td^T = Ud^T H^T               split-K over ffn
//   D5  Y^T  = Vd^T Td^T
// Every weight frag (common.h) is read exactly once, straight from HBM into registers with one
// coalesced 16-byte-per-lane load, and multiplied on the matrix cores against the (tiny, L2-resident)
// activation frags of the RT = 1, 2 or 4 tiles of 32 rows that the batch is padded to.  The contraction range
// of a workgroup is split over its 8 waves; their partial tiles are summed through LDS, and, when the
// contraction is also split over workgroups, through a partial buffer in which the last workgroup to
// arrive (an atomic ticket, no spinning) adds the partials in a fixed order, so results are
// bit-reproducible.  Products are computed transposed (lane = activation row), so each output tile is
// already the chain-order frag the next product consumes.
#include "common.h"
#include <mutex>
#include <type_traits>

namespace svdmlp {

enum { PH_D1 = 0, PH_D2 = 1, PH_D4 = 2, PH_D5 = 3 };
constexpr int SW = 8;  // waves per workgroup

struct StreamArgs {
  const char* W0;       // weight frags (D2: gate)
  const char* W1;       // D2: up frags
  const void* act;      // D1: X row-major bf16; otherwise activation frags [row tile][kb] (D2: Tg at 0, Tu at KB frags)
  void* out;            // D1: T frags; D2: H frags; D4: Td frags; D5: Y row-major
  float* part;          // split-K partial tiles [tile][split][accumulator][row tile][16][64]
  int* cnt;             // arrival counters [tile], TICKET_STRIDE ints apart
  int M, KB, tiles, S;  // contraction blocks, output tiles, workgroup-level splits
  int ldx;              // D1: row length of X (= d); D5: row length of Y (= d)
  int r;                // D1: rank (separates gate tiles from up tiles)
  int kb_major;         // weight frag order (1 for Ud)
  int act_rt, out_rt;   // frags between consecutive 32-row tiles of the activation / of the output
  int rtw;              // k_stream: groups of RT row tiles, each group with workgroups of its own (the batch has rtw RT row tiles)
};

template <int PH, int RT>
__global__ __launch_bounds__(SW * 64) void k_stream(StreamArgs a) {
  constexpr int NACC = (PH == PH_D2) ? 2 : 1;
  // D2 with four row tiles: the gate product, then the up product (half the accumulator registers, so that two
  // workgroups still share a CU); otherwise both at once, which keeps more weight loads in flight
  constexpr bool SEQ = PH == PH_D2 && RT == 4;
  constexpr int NPASS = SEQ ? 2 : 1;
  constexpr int NA = NACC / NPASS;            // accumulators (per row tile) live at a time
  constexpr int NT = NACC * RT;               // accumulator tiles of a wave in all: tile n RT + rt
  constexpr int NTP = NA * RT;                // ... per pass
  // ... staged in LDS per round (32 KiB each).  D2 has more workgroups than CUs: 64 KiB lets two of them share a CU
  // (the other phases have at most one workgroup per CU and stage up to four tiles, 128 KiB, in one round)
  constexpr int NB = (PH == PH_D2) ? 2 : (NTP < 4 ? NTP : 4);
  constexpr int ROUNDS = NTP / NB;
  // staging of accumulator tiles: [tile][wave][registers 4 p .. 4 p + 3][lane], 16 bytes per lane
  __shared__ f32x4 red[NB][SW][4][64];
  __shared__ int s_last;
  // the wave index as a scalar: the contraction loop below then has wave-uniform bounds
  const int lane = threadIdx.x % 64, w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  // Workgroups b, b + 8, .. b + 8 (rtw - 1) run on the same XCD and take the rtw row-tile groups of one (tile, range):
  // the first of them brings the weight frags into that XCD's L2, the others find them there.
  // (Not for D2, which has more tiles than there are CUs at any batch size: rtw = 1 there, at compile time.)
  constexpr bool GROUPS = PH != PH_D2;
  const int idx = GROUPS ? (blockIdx.x / (8 * a.rtw)) * 8 + blockIdx.x % 8 : blockIdx.x;
  if (GROUPS && idx >= a.tiles * a.S) return;
  const int rt0 = GROUPS ? (blockIdx.x / 8) % a.rtw * RT : 0;   // first row tile of this workgroup
  const int tile = idx / a.S, sp = idx % a.S;
  const int unit = tile * a.rtw + rt0 / RT;               // output tile x row-tile group: owner of partials and ticket
  const int kbs = (a.KB + a.S - 1) / a.S;                 // contraction blocks of this workgroup
  const int kw = (kbs + SW - 1) / SW;                     // ... of each wave
  int k0 = sp * kbs + w * kw;
  int k1 = k0 + kw;
  const int kend = (sp + 1) * kbs < a.KB ? (sp + 1) * kbs : a.KB;
  if (k1 > kend) k1 = kend;

  const int il = lane % 32, h = lane / 32;
  const size_t wstride = a.kb_major ? (size_t)a.tiles * FRAG_BYTES : (size_t)FRAG_BYTES;
  const char* wp0 = a.W0 + (a.kb_major ? (size_t)tile : (size_t)tile * a.KB) * FRAG_BYTES + lane * 16;
  const char* wp1 = (PH == PH_D2) ? a.W1 + (size_t)tile * a.KB * FRAG_BYTES + lane * 16 : nullptr;
  const uint16_t* xrow[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int row = 32 * (rt0 + rt) + il;
    xrow[rt] = (PH == PH_D1) ? static_cast<const uint16_t*>(a.act) + (size_t)(row < a.M ? row : a.M - 1) * a.ldx + 8 * h : nullptr;
  }
  const char* af = static_cast<const char*>(a.act) + lane * 16;
  // wave t < 2 RT finishes registers 8 (t % 2) .. + 7 (= one chain-order frag) of row tile t / 2
  const int t = w;
  const int rtf = t / 2, hf = t % 2;
  float v[NACC][8];

#pragma unroll
  for (int pass = 0; pass < NPASS; ++pass) {
    f32x16 acc[NA][RT];
#pragma unroll
    for (int n = 0; n < NA; ++n)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][rt][e] = 0.f;
    const char* wa = (SEQ && pass == 1) ? wp1 : wp0;
    const int aoff = SEQ ? pass * a.KB : 0;
    // U contraction blocks at a time: every load of the group (weights first: they come from HBM) is issued before
    // the first MFMA, so a wave has U (2 U for D2) weight frags in flight instead of one.  The whole range of a wave
    // is a handful of blocks; with one load in flight it was that many memory round trips long.
    auto step = [&](auto uc, int kb) __attribute__((always_inline)) {
      constexpr int U = decltype(uc)::value;
      constexpr bool BOTH = PH == PH_D2 && !SEQ;
      bf16x8 wv[U], wu[BOTH ? U : 1], av[U][RT], au[BOTH ? U : 1][RT];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        wv[u] = *reinterpret_cast<const bf16x8*>(wa + (size_t)(kb + u) * wstride);
        if (BOTH) wu[u] = *reinterpret_cast<const bf16x8*>(wp1 + (size_t)(kb + u) * FRAG_BYTES);
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          if (PH == PH_D1) av[u][rt] = *reinterpret_cast<const bf16x8*>(xrow[rt] + 16 * (kb + u));
          else av[u][rt] = *reinterpret_cast<const bf16x8*>(af + ((size_t)(rt0 + rt) * a.act_rt + aoff + kb + u) * FRAG_BYTES);
          if (BOTH) au[u][rt] = *reinterpret_cast<const bf16x8*>(af + ((size_t)(rt0 + rt) * a.act_rt + a.KB + kb + u) * FRAG_BYTES);
        }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          acc[0][rt] = mfma32(wv[u], av[u][rt], acc[0][rt]);
          if (BOTH) acc[NA - 1][rt] = mfma32(wu[u], au[u][rt], acc[NA - 1][rt]);
        }
    };
    constexpr int UMAX = (RT * NA <= 2) ? 4 : 2;   // weight frags in flight per wave that the register budget allows
    int kb = k0;
    if (UMAX >= 4)
      for (; kb + 4 <= k1; kb += 4) step(std::integral_constant<int, UMAX >= 4 ? 4 : 1>{}, kb);
    for (; kb + 2 <= k1; kb += 2) step(std::integral_constant<int, 2>{}, kb);
    if (kb < k1) step(std::integral_constant<int, 1>{}, kb);

    // ---- sum the 8 waves' partial tiles through LDS (fixed order) ----
#pragma unroll
    for (int q = 0; q < ROUNDS; ++q) {
      if (pass > 0 || q > 0) __syncthreads();   // the previous round has been read
#pragma unroll
      for (int jj = 0; jj < NB; ++jj) {
        const int j = q * NB + jj;
#pragma unroll
        for (int pl = 0; pl < 4; ++pl) {
          const f32x16& c = acc[j / RT][j % RT];
          red[jj][w][pl][lane] = f32x4{c[4 * pl], c[4 * pl + 1], c[4 * pl + 2], c[4 * pl + 3]};
        }
      }
      __syncthreads();
      if (t < 2 * RT) {
#pragma unroll
        for (int n = 0; n < NA; ++n) {
          const int j = n * RT + rtf;
          if (j / NB == q) {
            const int jj = j % NB;
#pragma unroll
            for (int s = 0; s < 8; ++s) v[pass * NA + n][s] = 0.f;
#pragma unroll
            for (int ww = 0; ww < SW; ++ww) {
              const f32x4 x0 = red[jj][ww][2 * hf][lane], x1 = red[jj][ww][2 * hf + 1][lane];
#pragma unroll
              for (int s = 0; s < 4; ++s) { v[pass * NA + n][s] += x0[s]; v[pass * NA + n][4 + s] += x1[s]; }
            }
          }
        }
      }
    }
  }
  if (a.S > 1) {
    // Partials cross workgroups (possibly on different XCDs, whose L2s are not coherent with each other) as
    // device-scope relaxed atomics: such stores write through to memory and such loads bypass the local L2,
    // so no cache write-back / invalidate (which a device-scope fence would cost every workgroup) is needed.
    // Ordering: each thread waits for its own stores to be acknowledged, the workgroup barrier collects
    // them, then one thread takes the ticket.
    float* mine = a.part + ((size_t)unit * a.S + sp) * NT * 1024;
    const int eo = (8 * hf) * 64 + lane;
    if (t < 2 * RT) {
#pragma unroll
      for (int n = 0; n < NACC; ++n)
#pragma unroll
        for (int s = 0; s < 8; ++s)
          __hip_atomic_store(&mine[(n * RT + rtf) * 1024 + eo + s * 64], v[n][s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("" ::: "memory");
    wait_vmcnt<0>();
    __syncthreads();
    if (threadIdx.x == 0)
      s_last = (__hip_atomic_fetch_add(&a.cnt[unit * TICKET_STRIDE], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.S - 1);
    __syncthreads();
    if (!s_last) return;
    if (t < 2 * RT) {
#pragma unroll
      for (int n = 0; n < NACC; ++n) {
#pragma unroll
        for (int s = 0; s < 8; ++s) v[n][s] = 0.f;
        // four partial tiles' worth of loads in flight at a time; the additions stay in split order
        for (int q0 = 0; q0 < a.S; q0 += 4) {
          float tmp[4][8];
#pragma unroll
          for (int qq = 0; qq < 4; ++qq) {
            const int q = q0 + qq < a.S ? q0 + qq : a.S - 1;
            const float* src = a.part + (((size_t)unit * a.S + q) * NT + n * RT + rtf) * 1024 + eo;
#pragma unroll
            for (int s = 0; s < 8; ++s) tmp[qq][s] = __hip_atomic_load(src + s * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
          for (int qq = 0; qq < 4; ++qq)
            if (q0 + qq < a.S) {
#pragma unroll
              for (int s = 0; s < 8; ++s) v[n][s] += tmp[qq][s];
            }
        }
      }
    }
    if (threadIdx.x == 0) __hip_atomic_store(&a.cnt[unit * TICKET_STRIDE], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next forward
  }
  if (t >= 2 * RT) return;

  // ---- epilogue ----
  if (PH == PH_D5) {
    // lane = row m; slots s <-> columns 32 tile + 16 hf + 8 (s / 4) + 4 h + s % 4
    const int row = 32 * (rt0 + rtf) + il;
    if (row < a.M) {
      uint16_t* y = static_cast<uint16_t*>(a.out) + (size_t)row * a.ldx + 32 * tile + 16 * hf + 4 * h;
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        bf16x4 o;
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = (__bf16)v[0][4 * g + i];
        *reinterpret_cast<bf16x4*>(y + 8 * g) = o;
      }
    }
    return;
  }
  bf16x8 o;
  if (PH == PH_D2) {
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const float g = v[0][s];
      o[s] = (__bf16)(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * v[NACC - 1][s]);
    }
  } else {
#pragma unroll
    for (int s = 0; s < 8; ++s) o[s] = (__bf16)v[0][s];
  }
  size_t frag = (size_t)(rt0 + rtf) * a.out_rt;
  if (PH == PH_D1) {
    const int p0 = 32 * tile;
    const int which = p0 >= a.r ? 1 : 0;
    frag += (size_t)which * (a.r / 16) + (p0 - which * a.r) / 16 + hf;
  } else {
    frag += (size_t)2 * tile + hf;
  }
  *reinterpret_cast<bf16x8*>(static_cast<char*>(a.out) + (frag * 64 + lane) * 16) = o;
}

// ------------------------------------------------------------------------------------------------
// D1, D4 (and D5 while it has fewer than 256 tiles of 32 columns): the same products on 16 x 16 x 32 MFMAs, one
// 16-column output tile per workgroup group.
// D1 and D4 split their contraction over workgroups, and what the split costs (the partial tile written
// through, and above all the read-back of all S partial tiles by one workgroup, past its L2 and through one CU's
// bounded fetch rate) goes with the tile size: a 16 x 16 fp32 tile is 1 KiB instead of 4 KiB, and twice as many
// tiles need half as many ranges.  The weight frags are the same ones (32 rows x 16 k, lane-major): a 16-row
// operand of contraction block pair (2 kb2, 2 kb2 + 1) is lanes 16 hn .. + 15 and 32 + 16 hn .. + 15 of those two
// frags, i.e. four 256-byte runs per load; every cache line of a frag is still read by exactly one workgroup.
// Lane l of a wave: row / column i = l % 16, contraction group g = l / 16 (k = 32 kb2 + 8 g .. + 7).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

template <int PH, int MT>   // MT = 16-row tiles of the batch (M <= 16 MT <= 32)
__global__ __launch_bounds__(SW * 64) void k_stream16(StreamArgs a) {
  static_assert(PH == PH_D1 || PH == PH_D4 || PH == PH_D5, "the phases with a short row of output tiles");
  static_assert(MT == 1 || MT == 2, "one 32-row activation tile");
  __shared__ f32x4 red[SW][MT][64];
  __shared__ int s_last;
  const int lane = threadIdx.x % 64, w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int tile = blockIdx.x / a.S, sp = blockIdx.x % a.S;   // 16-column tile, contraction range
  const int KB2 = a.KB / 2;                                // contraction blocks of 32
  const int kbs = (KB2 + a.S - 1) / a.S;
  const int kw = (kbs + SW - 1) / SW;
  int k0 = sp * kbs + w * kw;
  int k1 = k0 + kw;
  const int kend = (sp + 1) * kbs < KB2 ? (sp + 1) * kbs : KB2;
  if (k1 > kend) k1 = kend;

  const int i = lane % 16, g = lane / 16;
  const int tile32 = tile / 2, hn = tile % 2, tiles32 = a.tiles / 2;
  // this lane's 16 bytes within a weight frag / an activation frag, and which frag of the pair
  const int fsel = g / 2;
  const size_t wl = (size_t)(16 * hn + i + 32 * (g % 2)) * 16, al = (size_t)(i + 32 * (g % 2)) * 16;
  const char* wbase = a.W0 + (a.kb_major ? (size_t)tile32 : (size_t)tile32 * a.KB) * FRAG_BYTES + wl;
  const size_t wstride = a.kb_major ? (size_t)tiles32 * FRAG_BYTES : (size_t)FRAG_BYTES;   // per 16-k frag
  const uint16_t* xrow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int row = 16 * mt + i;
    xrow[mt] = (PH == PH_D1) ? static_cast<const uint16_t*>(a.act) + (size_t)(row < a.M ? row : a.M - 1) * a.ldx + 8 * g : nullptr;
  }
  const char* abase = static_cast<const char*>(a.act) + al;

  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  // U contraction blocks at a time, every load of the group issued before the first MFMA (see k_stream)
  auto step = [&](auto uc, int kb) __attribute__((always_inline)) {
    constexpr int U = decltype(uc)::value;
    bf16x8 wv[U], av[U][MT];
#pragma unroll
    for (int u = 0; u < U; ++u) wv[u] = *reinterpret_cast<const bf16x8*>(wbase + (size_t)(2 * (kb + u) + fsel) * wstride);
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        if (PH == PH_D1) av[u][mt] = *reinterpret_cast<const bf16x8*>(xrow[mt] + 32 * (kb + u));
        else  // row tile mt / 2, rows 16 (mt % 2) .. of it
          av[u][mt] = *reinterpret_cast<const bf16x8*>(abase + ((size_t)(mt / 2) * a.act_rt + 2 * (kb + u) + fsel) * FRAG_BYTES + (mt % 2) * 256);
      }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt] = mfma16(wv[u], av[u][mt], acc[mt]);
  };
  constexpr int UMAX = MT <= 2 ? 8 : MT == 4 ? 4 : 2;
  int kb = k0;
  if (UMAX >= 8)
    for (; kb + 8 <= k1; kb += 8) step(std::integral_constant<int, UMAX >= 8 ? 8 : 1>{}, kb);
  if (UMAX >= 4)
    for (; kb + 4 <= k1; kb += 4) step(std::integral_constant<int, UMAX >= 4 ? 4 : 1>{}, kb);
  for (; kb + 2 <= k1; kb += 2) step(std::integral_constant<int, 2>{}, kb);
  if (kb < k1) step(std::integral_constant<int, 1>{}, kb);
  // lane (m = l % 16, g): acc[mt][e] = element (output column 4 g + e of the tile, row 16 mt + m)
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) red[w][mt][lane] = acc[mt];
  __syncthreads();
  f32x4 v[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) v[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  if (w == 0) {
#pragma unroll
    for (int ww = 0; ww < SW; ++ww)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) v[mt] += red[ww][mt][lane];
  }
  if (a.S > 1) {
    // same exchange as in k_stream: write-through partial, ticket, the last workgroup adds in range order
    float* mine = a.part + ((size_t)tile * a.S + sp) * (MT * 256);
    if (w == 0) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          __hip_atomic_store(&mine[(mt * 4 + e) * 64 + lane], v[mt][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("" ::: "memory");
    wait_vmcnt<0>();
    __syncthreads();
    if (threadIdx.x == 0)
      s_last = (__hip_atomic_fetch_add(&a.cnt[tile * TICKET_STRIDE], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.S - 1);
    __syncthreads();
    if (!s_last || w != 0) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) v[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int QB = MT >= 8 ? 1 : 8 / MT;   // partial tiles in flight (8 KiB); additions in range order
    for (int q0 = 0; q0 < a.S; q0 += QB) {
      f32x4 tmp[QB][MT];
#pragma unroll
      for (int qq = 0; qq < QB; ++qq) {
        const int q = q0 + qq < a.S ? q0 + qq : a.S - 1;
        const float* src = a.part + ((size_t)tile * a.S + q) * (MT * 256) + lane;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            tmp[qq][mt][e] = __hip_atomic_load(src + (mt * 4 + e) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
#pragma unroll
      for (int qq = 0; qq < QB; ++qq)
        if (q0 + qq < a.S) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) v[mt] += tmp[qq][mt];
        }
    }
    if (lane == 0) __hip_atomic_store(&a.cnt[tile * TICKET_STRIDE], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // for the next forward
  } else if (w != 0) {
    return;
  }
  if (PH == PH_D5) {
    // lane (m, g) holds columns 16 tile + 4 g .. + 3 of row 16 mt + m: eight bytes of Y
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = 16 * mt + i;
      if (row < a.M) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[mt][e];
        *reinterpret_cast<bf16x4*>(static_cast<uint16_t*>(a.out) + (size_t)row * a.ldx + 16 * tile + 4 * g) = o;
      }
    }
    return;
  }
  // The tile is contraction block `frag` of the next product's activation, in chain order: element s of frag lane
  // (row, h) is column 8 (s / 4) + 4 h + s % 4, i.e. the four values of lane (m, g = h), then those of lane (m, g = 2 + h).
  // Per 32-row tile: lanes 0..31 of this wave write the frag lanes of its rows 0..15, lanes 32..63 those of its rows
  // 16..31 (zeros if MT = 1).
  const int m = lane % 16, h = (lane / 16) % 2, up = lane / 32;
  size_t frag;
  if (PH == PH_D1) {
    const int p0 = 16 * tile;
    const int which = p0 >= a.r ? 1 : 0;
    frag = (size_t)which * (a.r / 16) + (p0 - which * a.r) / 16;
  } else {
    frag = (size_t)tile;
  }
  const int dl = 16 * up + m + 32 * h;
#pragma unroll
  for (int rt = 0; rt < (MT + 1) / 2; ++rt) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float lo = __shfl(v[2 * rt][e], m + 16 * h, 64), hi = __shfl(v[2 * rt][e], m + 16 * (2 + h), 64);
      if (MT >= 2) {
        const float lo1 = __shfl(v[MT >= 2 ? 2 * rt + 1 : 0][e], m + 16 * h, 64), hi1 = __shfl(v[MT >= 2 ? 2 * rt + 1 : 0][e], m + 16 * (2 + h), 64);
        lo = up ? lo1 : lo;
        hi = up ? hi1 : hi;
      } else if (up) {
        lo = 0.f;
        hi = 0.f;
      }
      o[e] = (__bf16)lo;
      o[4 + e] = (__bf16)hi;
    }
    *reinterpret_cast<bf16x8*>(static_cast<char*>(a.out) + (((size_t)rt * a.out_rt + frag) * 64 + dl) * 16) = o;
  }
}

// ranges for k_stream16: `tiles` 16-column tiles, KB2 contraction blocks of 32, mt 16-row tiles
int stream_splits16(int tiles, int KB2, int mt) {
  int s = (256 + tiles - 1) / tiles;
  int smax = KB2 / SW;
  if (s > smax) s = smax;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  const size_t part_floats = ((size_t)8 << 20) / 4;   // the partial-tile buffer of the workspace
  while (s > 1 && (size_t)tiles * s * mt * 256 > part_floats) --s;
  return s;
}
// 16-row tiles k_stream16 pads a batch to
int stream_tiles16(int64_t M) { return M <= 16 ? 1 : 2; }
// whether the two split phases of a forward of M rows run on 16-column tiles
bool stream_uses_tile16(int64_t M, int64_t d, int64_t ffn, int64_t r, int64_t rd) {
  // beyond 32 rows the activation frags, re-read for every 16-column weight tile, cost more than the smaller partials
  // save (the 32-column tiles with row-tile groups of their own measure faster there)
  return M <= 32 && d % 32 == 0 && ffn % 32 == 0 && 2 * r / 16 <= 2048 && rd / 16 <= 2048;
}

// The last product on 16-column tiles too: while the 32-column tiles would leave CUs without a workgroup (a phase
// streams its weights at the chip's rate only if every CU pulls: 128 of 256 CUs reach 3.6 of 7.1 TB/s).  Measured at
// the decode shape (128 -> 256 workgroups for 4 MB of Vd): the forward 0.9 us shorter at 1..16 rows, 0.55 us at 32.
bool stream_last_uses_tile16(bool tile16, int tiles32) { return tile16 && tiles32 < 256; }

// Row-tile groups of the two split phases (k_stream; `rt` row tiles in the batch, `tiles` 32-column tiles, KB
// contraction blocks).  With all row tiles in one workgroup the weights are fetched once, but the workgroup that adds
// the partial tiles reads ranges x rt of them through one CU's bounded fetch rate (mlp_small, 128 rows: 512 KiB
// in the down projection).  Groups with workgroups of their own need fewer ranges to fill the chip and spread that
// read-back; in exchange rtw workgroups (of one XCD) fetch the same weight frags, which occupies rtw times the
// requests in flight chip-wide while they stream from HBM.  Measured: at 128 rows phases with 2 and 4 MB of weights
// take 35-40 % less time with four groups, 8 MB 25 % less with four groups, 15 MB 10 % less with two (and no less with
// four when the weights come from HBM); at 64 rows two groups on these 32-column tiles beat the 16-column tiles of
// k_stream16 (whose workgroups re-read twice the activation bytes) by 2.3 us (D1, 8 MB) and 2.5 us (D4, 15 MB).
int stream_row_groups(int rt, int tiles, int KB, bool first) {
  const double weight_mb = (double)tiles * KB * FRAG_BYTES / 1.0e6;
  int rtw = rt;
  // the first phase (activation = the rows of X) takes more copies of a fetch than the down projection, whose
  // workgroups also stream the ffn-wide activation: cold, every row tile on its own still pays with 17 MB of [Ug|Uu]
  // (r = 1024, 128 rows: the forward 67.8 -> 65.4 us), two groups lose a little with 34 MB (r = 2048), and the down
  // projection loses with four groups at 15 MB and 29 MB
  const double lim = first && weight_mb <= 20.0 ? 1.0e9 : 30.0;
  while (rtw > 1 && (weight_mb * (rtw - 1) > lim || tiles * rtw > 2048)) rtw /= 2;
  return rtw;
}

// ... of the last product, whose contraction is not split: groups only while there are fewer workgroups than CUs
int stream_row_groups_whole(int rt, int tiles) {
  int rtw = 1;
  while (2 * rtw <= rt && 2 * rtw * tiles <= 256) rtw *= 2;
  return rtw;
}

int stream_splits(int tiles, int KB, int rt) {
  int s = (256 + tiles - 1) / tiles;      // aim at one workgroup per CU
  int smax = KB / SW;                     // at least one contraction block per wave
  if (s > smax) s = smax;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  const size_t part_floats = ((size_t)8 << 20) / 4;   // the partial-tile buffer of the workspace
  while (s > 1 && (size_t)tiles * s * rt * 1024 > part_floats) --s;
  return s;
}

template <int PH>
static void launch_stream(int rt, const StreamArgs& a, hipStream_t st) {   // rt: row tiles per workgroup
  const dim3 grid(PH == PH_D2 ? a.tiles * a.S : (a.tiles * a.S + 7) / 8 * 8 * a.rtw), block(SW * 64);
  if (rt == 1) hipLaunchKernelGGL((k_stream<PH, 1>), grid, block, 0, st, a);
  else if (rt == 2) hipLaunchKernelGGL((k_stream<PH, 2>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((k_stream<PH, 4>), grid, block, 0, st, a);
}

template <int PH>
static void launch_stream16(int mt, const StreamArgs& a, hipStream_t st) {
  const dim3 grid(a.tiles * a.S), block(SW * 64);
  if (mt == 1) hipLaunchKernelGGL((k_stream16<PH, 1>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((k_stream16<PH, 2>), grid, block, 0, st, a);
}

// The per-forward buffers of the path: the rank-r strips T, the ffn-wide activation H of its (at most 128) rows, the
// down strip Td, the partial tiles of the two phases that split their contraction over workgroups, and their tickets.
struct StreamBufs {
  char* T;
  char* H;
  char* Td;
  float* part;
  int* cnt;
};

static int stream_forward_on(const Ctx* c, const StreamBufs& b, const void* X, int64_t M, void* Y, hipStream_t st);

int bf16_stream_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const StreamBufs b = {ws + p.off_T, ws + p.off_H, ws + p.off_Td, reinterpret_cast<float*>(ws + p.off_part),
                        reinterpret_cast<int*>(ws + p.off_cnt + CNT_ONE_KERNEL_BYTES)};
  return stream_forward_on(c, b, X, M, Y, st);
}

// Whether the weight-streaming path takes a forward of M rows of this plan: up to 128 rows, and no more units (output
// tile x row-tile group) in either split phase than there are ticket lines (2048 per phase: ranks beyond 32768).
bool stream_supported(const Plan& p, int64_t M) {
  if (M < 1 || M > STREAM_MAX_M) return false;
  const int rt = M <= 32 ? 1 : M <= 64 ? 2 : 4;
  if (p.kind == SVDMLP_LINEAR) {
    if (M <= 32 && p.d % 32 == 0 && p.r / 16 <= 2048) return true;   // 16-column tiles
    const int t1 = (int)(p.r / 32);
    return t1 * stream_row_groups(rt, t1, (int)(p.d / 16), true) <= 2048;
  }
  if (stream_uses_tile16(M, p.d, p.ffn, p.r, p.rd)) return true;     // its own limits are part of that predicate
  const int t1 = (int)(2 * p.r / 32), t4 = (int)(p.rd / 32);
  return t1 * stream_row_groups(rt, t1, (int)(p.d / 16), true) <= 2048 &&
         t4 * stream_row_groups(rt, t4, (int)(p.ffn / 16), false) <= 2048;
}

static int stream_forward_on(const Ctx* c, const StreamBufs& b, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  int* cnt = b.cnt;
  float* part = b.part;
  if (M > STREAM_MAX_M) return (int)hipErrorInvalidValue;
  const int rt = M <= 32 ? 1 : M <= 64 ? 2 : 4;   // 32-row tiles the batch is padded to
  const bool t16 = stream_uses_tile16(M, p.d, p.ffn, p.r, p.rd);
  const int mt16 = stream_tiles16(M);
  int e;
  static const char* const names[4] = {"k_stream_d1", "k_stream_d2", "k_stream_d4", "k_stream_d5"};
  const int ps = prof_open_forward(c, 4, names);
  const int fT = (int)(2 * p.r / 16), fH = (int)(p.ffn / 16), fTd = (int)(p.rd / 16);   // frags per 32-row tile

  StreamArgs a;
  // D1
  a = StreamArgs{ws + p.off_wU, nullptr, X, b.T, part, cnt, (int)M, (int)(p.d / 16), (int)(2 * p.r / 32), 1,
                 (int)p.d, (int)p.r, 0, 0, fT, 1};
  a.rtw = stream_row_groups(rt, a.tiles, a.KB, true);
  a.S = stream_splits(a.tiles * a.rtw, a.KB, rt / a.rtw);
  if (a.tiles * a.rtw > 2048) return (int)hipErrorInvalidValue;
  prof_mark(c, ps, 0, 0, st);
  if (t16) {
    a.tiles *= 2;
    a.S = stream_splits16(a.tiles, a.KB / 2, mt16);
    launch_stream16<PH_D1>(mt16, a, st);
  } else {
    launch_stream<PH_D1>(rt / a.rtw, a, st);
  }
  prof_mark(c, ps, 0, 1, st);
  if ((e = (int)hipGetLastError())) return e;
  // D2 (never split over workgroups: its contraction is only r long)
  a = StreamArgs{ws + p.off_wVg, ws + p.off_wVu, b.T, b.H, part, cnt, (int)M, (int)(p.r / 16),
                 (int)(p.ffn / 32), 1, 0, (int)p.r, 0, fT, fH, 1};
  prof_mark(c, ps, 1, 0, st);
  launch_stream<PH_D2>(rt, a, st);
  prof_mark(c, ps, 1, 1, st);
  if ((e = (int)hipGetLastError())) return e;
  // D4
  a = StreamArgs{ws + p.off_wUd, nullptr, b.H, b.Td, part, cnt + 2048 * TICKET_STRIDE, (int)M, (int)(p.ffn / 16),
                 (int)(p.rd / 32), 1, 0, (int)p.r, 1, fH, fTd, 1};
  a.rtw = stream_row_groups(rt, a.tiles, a.KB, false);
  a.S = stream_splits(a.tiles * a.rtw, a.KB, rt / a.rtw);
  if (a.tiles * a.rtw > 2048) return (int)hipErrorInvalidValue;
  prof_mark(c, ps, 2, 0, st);
  if (t16) {
    a.tiles *= 2;
    a.S = stream_splits16(a.tiles, a.KB / 2, mt16);
    launch_stream16<PH_D4>(mt16, a, st);
  } else {
    launch_stream<PH_D4>(rt / a.rtw, a, st);
  }
  prof_mark(c, ps, 2, 1, st);
  if ((e = (int)hipGetLastError())) return e;
  // D5
  a = StreamArgs{ws + p.off_wVd, nullptr, b.Td, Y, part, cnt, (int)M, (int)(p.rd / 16), (int)(p.d / 32), 1,
                 (int)p.d, (int)p.r, 0, fTd, 0, 1};
  a.rtw = stream_row_groups_whole(rt, a.tiles);
  prof_mark(c, ps, 3, 0, st);
  if (stream_last_uses_tile16(t16, a.tiles)) {
    a.tiles *= 2;
    launch_stream16<PH_D5>(mt16, a, st);
  } else {
    launch_stream<PH_D5>(rt / a.rtw, a, st);
  }
  prof_mark(c, ps, 3, 1, st);
  return (int)hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// The same forward with its per-forward buffers in a static device array instead of the caller's workspace, for
// callers that may not allocate device memory and hold no workspace of their own for intermediates (code under graph
// capture, tight serving loops).  Layout of the array: partial tiles (8 MiB, the capacity stream_splits assumes), the
// ticket lines of D1 and D4, then T, H and Td of the call, each 256-byte aligned.  Every GPU the library's code is
// loaded on holds its own copy of the array until the process ends; all calls on one GPU share it, so calls that
// overlap on one GPU race (as forwards on one context do).
// ------------------------------------------------------------------------------------------------
constexpr size_t SCRATCH_PART_BYTES = (size_t)8 << 20;
constexpr size_t SCRATCH_TICKET_BYTES = (size_t)2 * 2048 * TICKET_STRIDE * 4;
constexpr size_t SCRATCH_ACT_OFF = SCRATCH_PART_BYTES + SCRATCH_TICKET_BYTES;
static_assert(STATIC_SCRATCH_BYTES > SCRATCH_ACT_OFF, "room for the activations");
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

// Device address of this GPU's copy of the array.  The array's name is only a host-side handle; the address comes
// from the runtime, once per device, with that device current (svdmlp_create calls this, so the lookup, which may load
// the code object, never happens inside a forward).
constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch_resolve(int device, char** out) {
  if (device < 0 || device >= MAX_DEVICES) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    char* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!ptr) return (int)hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return 0;
}

__global__ __launch_bounds__(256) void k_clear_tickets(int* cnt, int lines) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < lines) cnt[(size_t)i * TICKET_STRIDE] = 0;
}

size_t stream_static_scratch_need(const Plan& p, int64_t M) {
  const size_t rows = M <= 32 ? 32 : M <= 64 ? 64 : 128;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  return SCRATCH_ACT_OFF + up(rows * 2 * p.r * 2) + up(rows * p.ffn * 2) + up(rows * p.rd * 2);
}

int bf16_stream_forward_static(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* base = c->static_scratch;   // resolved at create for this context's device
  if (!base || stream_static_scratch_need(p, M) > STATIC_SCRATCH_BYTES) return (int)hipErrorInvalidValue;
  const size_t rows = M <= 32 ? 32 : M <= 64 ? 64 : 128;
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  StreamBufs b;
  b.part = reinterpret_cast<float*>(base);
  b.cnt = reinterpret_cast<int*>(base + SCRATCH_PART_BYTES);
  b.T = base + SCRATCH_ACT_OFF;
  b.H = b.T + up(rows * 2 * p.r * 2);
  b.Td = b.H + up(rows * p.ffn * 2);
  // The tickets must start at zero.  Every forward leaves them at zero, but the array is shared by every caller on
  // this GPU and outlives them, so they are cleared here, with a kernel (a memset node does not belong in a graph
  // that a caller may be capturing).  The other buffers are written before they are read.
  const int lines = 2 * 2048;
  hipLaunchKernelGGL(k_clear_tickets, dim3((lines + 255) / 256), dim3(256), 0, st, b.cnt, lines);
  const int e = (int)hipGetLastError();
  if (e) return e;
  return stream_forward_on(c, b, X, M, Y, st);
}

// Whether the single factored layer of M <= 128 rows streams: every workgroup of a phase re-reads the activation of
// its rows from L2, (r / 32) d + (n / 32) r elements per row over the two phases; beyond about 0.5 GB of that the
// MFMA-tiled kernels are faster (measured: d = 8192, r = 4096, n = 16384 at 96 / 128 rows 85 / 91 us against 79 us
// tiled, at 64 rows 57 against 78 us; every smaller layer tried streams 1.3 - 3x faster up to 128 rows).
bool linear_stream_pays(int64_t M, int64_t d, int64_t r, int64_t n) {
  const int64_t rows = M <= 32 ? 32 : M <= 64 ? 64 : 128;
  return M <= STREAM_MAX_M && (double)((r / 32) * d + (n / 32) * r) * (double)rows * 2.0 <= 512.0e6;
}

// Single factored layer O = (X U) V for up to 128 rows (paper Sec. 4.2.1 at decode sizes): the first and the last
// phase of the path above back to back.  T = X U is phase D1 with one strip of r columns, O = T V is phase D5 with
// the row length of O; U and V frags are the ones the tiled kernels of this kind read.
int bf16_linear_stream_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  int* cnt = reinterpret_cast<int*>(ws + p.off_cnt + CNT_ONE_KERNEL_BYTES);
  float* part = reinterpret_cast<float*>(ws + p.off_part);
  if (M > STREAM_MAX_M) return (int)hipErrorInvalidValue;
  const int rt = M <= 32 ? 1 : M <= 64 ? 2 : 4;
  const bool t16 = M <= 32 && p.d % 32 == 0 && p.r / 16 <= 2048;
  const int mt16 = stream_tiles16(M);
  static const char* const names[2] = {"k_stream_d1", "k_stream_d5"};
  const int ps = prof_open_forward(c, 2, names);
  const int fT = (int)(p.r / 16);   // frags of T per 32-row tile
  int e;
  StreamArgs a;
  a = StreamArgs{ws + p.off_wU, nullptr, X, ws + p.off_T, part, cnt, (int)M, (int)(p.d / 16), (int)(p.r / 32), 1,
                 (int)p.d, (int)p.r, 0, 0, fT, 1};
  a.rtw = stream_row_groups(rt, a.tiles, a.KB, true);
  a.S = stream_splits(a.tiles * a.rtw, a.KB, rt / a.rtw);
  if (a.tiles * a.rtw > 2048) return (int)hipErrorInvalidValue;
  prof_mark(c, ps, 0, 0, st);
  if (t16) {
    a.tiles *= 2;
    a.S = stream_splits16(a.tiles, a.KB / 2, mt16);
    launch_stream16<PH_D1>(mt16, a, st);
  } else {
    launch_stream<PH_D1>(rt / a.rtw, a, st);
  }
  prof_mark(c, ps, 0, 1, st);
  if ((e = (int)hipGetLastError())) return e;
  a = StreamArgs{ws + p.off_wVd, nullptr, ws + p.off_T, Y, part, cnt, (int)M, (int)(p.r / 16), (int)(p.ffn / 32), 1,
                 (int)p.ffn, (int)p.r, 0, fT, 0, 1};
  a.rtw = stream_row_groups_whole(rt, a.tiles);
  prof_mark(c, ps, 1, 0, st);
  if (stream_last_uses_tile16(t16, a.tiles)) {
    a.tiles *= 2;
    launch_stream16<PH_D5>(mt16, a, st);
  } else {
    launch_stream<PH_D5>(rt / a.rtw, a, st);
  }
  prof_mark(c, ps, 1, 1, st);
  return (int)hipGetLastError();
}

}  // namespace svdmlp
