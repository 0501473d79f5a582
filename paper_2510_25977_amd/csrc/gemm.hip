// bf16 MFMA path for large M with the ffn-wide activation staged through HBM (paper Alg. 3 writes the
// gated activation out and Alg. 2 reads it back for the down projection), gfx950.
//
//   k_gate_up   H    = SiLU(Tg Vg) .* (Tu Vu)     256 rows x 128 ffn columns per workgroup; the gate tile is
//                                                 accumulated first, squashed to SiLU(G) in bf16 pairs, then the up
//                                                 tile is accumulated on top and multiplied in; H leaves as frags
//   k_down1     Tdp  = H Ud over one ffn range     256 rows x 128 rank columns per workgroup, fp32 partials
//
// Why not keep H in registers: a workgroup that owns every rank column of its rows (so that H never has to be
// stored) has room for only 128 rows, and then each byte brought into the CU feeds too few MFMAs: the
// global->LDS copy rate (about 55 B/clk/CU measured) becomes the bound.  A 256 x 128 tile needs 12 KiB of
// operands per 32 MFMAs, two thirds of what that bound allows at full matrix-core rate, and its 128 accumulator
// registers per lane leave room for two workgroups per CU, so one's LDS/barrier/epilogue time is covered by the
// other's MFMAs.  The price is one write and one read of H (2 bytes per element each way).
//
// Both kernels are one machine.  Operands arrive as 1 KiB frags (common.h).  A "unit" is one contraction block
// (16) of the tile: 8 activation frags (256 rows) + 4 weight frags (128 columns) = 12 KiB; LDS is a ring of six
// units (72 KiB).  Wave (wm, wn) owns rows 128 wm.. and columns 64 wn.. of the tile: per unit it reads 4
// activation and 2 weight frags and issues 8 MFMAs.  The pipeline never drains: while the MFMAs of unit k are
// issued the frags of unit k+1 are read into the registers the MFMAs have just released, and the copies of unit
// k+5 are in flight.  Iteration k:
//   wait until this wave's copies of unit k+1 have landed (units k+2..k+4 may stay in flight)
//   barrier           -> everyone's part of unit k+1 has landed; everyone is done with unit k-1
//   issue unit k+5    -> into the slot of unit k-1
//   read the weight frags of unit k+1 (second register set)
//   4 x { wait for activation tile j of unit k; 2 MFMAs; read tile j of unit k+1 into the same registers }
#include "common.h"

namespace svdmlp {

constexpr int G_UNIT = 12 * FRAG_BYTES;
constexpr int G_SLOTS = 6;
constexpr int G_AHEAD = 5;  // units issued before the first one is consumed
constexpr int G_LDS = G_SLOTS * G_UNIT;

// 16 bytes per lane, global -> LDS, with a wave-uniform 64-bit base in SGPRs and a 32-bit per-lane offset:
// no vector ALU work per copy.  M0 carries the (wave-uniform) LDS destination; lane l lands at M0 + 16 l.
__device__ __forceinline__ void dma16_sv(const char* sbase, unsigned voff, unsigned lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(sbase), "v"(voff), "s"(lds_dst) : "memory", "m0");
}

// LDS unit layout: frags 0..7 activation (32-row tiles of the 256 rows), frags 8..11 weights (32-column tiles).
// Producer of the unit stream; all state is wave-uniform.  Wave w copies activation frags 2w, 2w+1 and weight frag w.
struct GProd {
  const char* pa;      // this wave's first activation frag of the next unit
  const char* pw;      // this wave's weight frag of the next unit
  long long a_tile;    // byte distance between the frags of consecutive 32-row tiles
  long long a_kb, w_kb;  // byte distance between consecutive contraction blocks
  unsigned lane16;
  unsigned dst;        // LDS address of this wave's activation frags in slot 0
  unsigned dstw;       // ... and of its weight frag
  int slot;            // slot the next unit goes to
  int issued, total;   // units issued so far / units in the stream
  int switch_at;       // unit at which the sources change to (pa2, pw2); -1 = never
  const char* pa2;
  const char* pw2;

  __device__ __forceinline__ void unit() {
    if (issued < total) {
      const unsigned b = dst + slot * G_UNIT, bw = dstw + slot * G_UNIT;
      dma16_sv(pa, lane16, b);
      dma16_sv(pa + a_tile, lane16, b + FRAG_BYTES);
      dma16_sv(pw, lane16, bw);
      pa += a_kb;
      pw += w_kb;
      slot = slot == G_SLOTS - 1 ? 0 : slot + 1;
      ++issued;
      if (issued == switch_at) {
        pa = pa2;
        pw = pw2;
      }
    }
  }
};

// Operand registers of a wave: four activation frags (single set, refilled tile by tile) and two sets of two
// weight frags.
struct GRegs {
  u32x4 A0, A1, A2, A3, Wa0, Wa1, Wb0, Wb1;
};

// MFMAs of one unit with weight set (Wc0, Wc1), reading the next unit (at aA / aW) behind them; the next unit's
// weight frags go to (Wn0, Wn1).  acc[i][j]: weight tile i (rows of the transposed product), activation tile j (lanes).
__device__ __forceinline__ void g_unit(u32x4& A0, u32x4& A1, u32x4& A2, u32x4& A3, u32x4& Wc0, u32x4& Wc1, u32x4& Wn0,
                                       u32x4& Wn1, unsigned aA, unsigned aW, f32x16 (&acc)[2][4]) {
  Wn0 = lds_read<0 * FRAG_BYTES>(aW);
  Wn1 = lds_read<1 * FRAG_BYTES>(aW);
  lgkm_wait<5>(Wc0, Wc1, A0);
  acc[0][0] = mfma32(as_bf16x8(Wc0), as_bf16x8(A0), acc[0][0]);
  acc[1][0] = mfma32(as_bf16x8(Wc1), as_bf16x8(A0), acc[1][0]);
  __builtin_amdgcn_sched_barrier(0);
  A0 = lds_read<0 * FRAG_BYTES>(aA);
  lgkm_wait<5>(A1);
  acc[0][1] = mfma32(as_bf16x8(Wc0), as_bf16x8(A1), acc[0][1]);
  acc[1][1] = mfma32(as_bf16x8(Wc1), as_bf16x8(A1), acc[1][1]);
  __builtin_amdgcn_sched_barrier(0);
  A1 = lds_read<1 * FRAG_BYTES>(aA);
  lgkm_wait<5>(A2);
  acc[0][2] = mfma32(as_bf16x8(Wc0), as_bf16x8(A2), acc[0][2]);
  acc[1][2] = mfma32(as_bf16x8(Wc1), as_bf16x8(A2), acc[1][2]);
  __builtin_amdgcn_sched_barrier(0);
  A2 = lds_read<2 * FRAG_BYTES>(aA);
  lgkm_wait<5>(A3);
  acc[0][3] = mfma32(as_bf16x8(Wc0), as_bf16x8(A3), acc[0][3]);
  acc[1][3] = mfma32(as_bf16x8(Wc1), as_bf16x8(A3), acc[1][3]);
  __builtin_amdgcn_sched_barrier(0);
  A3 = lds_read<3 * FRAG_BYTES>(aA);
}

struct GPipe {
  GProd prod;
  GRegs R;
  unsigned rdA, rdW;  // per-lane LDS read addresses in slot 0
  int rslot;          // slot of the unit that is read next
  int done;           // units consumed

  // certify the next unit, release the previous one, keep the copies flowing
  __device__ __forceinline__ void gate() {
    const int k = done;
    if (k + 4 < prod.total) wait_vmcnt<9>();
    else if (k + 3 < prod.total) wait_vmcnt<6>();
    else if (k + 2 < prod.total) wait_vmcnt<3>();
    else wait_vmcnt<0>();
    lds_barrier();
    prod.unit();
    ++done;
  }
  __device__ __forceinline__ void next_addr(unsigned& aA, unsigned& aW) {
    aA = rdA + rslot * G_UNIT;
    aW = rdW + rslot * G_UNIT;
    rslot = rslot == G_SLOTS - 1 ? 0 : rslot + 1;
  }
  // requires total >= G_AHEAD
  __device__ __forceinline__ void start() {
#pragma unroll
    for (int i = 0; i < G_AHEAD; ++i) prod.unit();
    wait_vmcnt<3 * (G_AHEAD - 1)>();
    lds_barrier();
    unsigned aA, aW;
    next_addr(aA, aW);
    R.Wa0 = lds_read<0 * FRAG_BYTES>(aW);
    R.Wa1 = lds_read<1 * FRAG_BYTES>(aW);
    R.A0 = lds_read<0 * FRAG_BYTES>(aA);
    R.A1 = lds_read<1 * FRAG_BYTES>(aA);
    R.A2 = lds_read<2 * FRAG_BYTES>(aA);
    R.A3 = lds_read<3 * FRAG_BYTES>(aA);
  }
  // consume n units (n even) into acc
  __device__ __forceinline__ void run(f32x16 (&acc)[2][4], int n) {
    for (int u = 0; u < n; u += 2) {
      unsigned aA, aW;
      gate();
      next_addr(aA, aW);
      __builtin_amdgcn_sched_barrier(0);
      g_unit(R.A0, R.A1, R.A2, R.A3, R.Wa0, R.Wa1, R.Wb0, R.Wb1, aA, aW, acc);
      gate();
      next_addr(aA, aW);
      __builtin_amdgcn_sched_barrier(0);
      g_unit(R.A0, R.A1, R.A2, R.A3, R.Wb0, R.Wb1, R.Wa0, R.Wa1, aA, aW, acc);
    }
  }
  // the reads issued behind the last unit (of a slot that holds nothing new) still have to land before the
  // registers are reused
  __device__ __forceinline__ void finish() {
    lgkm_wait<0>(R.A0, R.A1, R.A2, R.A3);
    lgkm_wait<0>(R.Wa0, R.Wa1, R.Wb0, R.Wb1);
  }
};

__device__ __forceinline__ void g_zero(f32x16 (&acc)[2][4]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
}

// Workgroup -> tile of k_gate_up.  Hardware workgroup ids go round-robin over the 8 XCDs.  With mx > 0 the XCDs
// form a grid of ngm row groups x 8 / ngm column groups; an XCD owns mx row tiles (their rank-r strips stay in its
// L2) and NT / (8 / ngm) column tiles, walked row tile fastest so that the mx workgroups that need the same weight
// tile run together.  mx = 0: plain order.
__device__ __forceinline__ void g_tile_of(int hw, int MT, int NT, int mx, int ngm, int& mt, int& nt) {
  if (mx > 0) {
    const int x = hw % 8, i = hw / 8;
    mt = (x % ngm) * mx + i % mx;
    nt = (x / ngm) * (NT / (8 / ngm)) + i / mx;
  } else {
    mt = hw % MT;
    nt = hw / MT;
  }
}

// ------------------------------------------------------------------------------------------------
// H = SiLU(Tg Vg) .* (Tu Vu)   (paper Alg. 3, second loop nest and gating epilogue)
// T: per 32-row tile the gate strip's KB frags then the up strip's (as written by k_s1).
// wVg, wVu: [ffn tile][KB] frags.  H: [32-row tile][ffn / 16] chain-order frags.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void k_gate_up(const char* __restrict__ T, const char* __restrict__ wVg,
                                                    const char* __restrict__ wVu, char* __restrict__ H, int KB, int KBf,
                                                    int MT, int NT, int mx, int ngm) {
  __shared__ __attribute__((aligned(1024))) char lds[G_LDS];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 2, wn = w % 2;
  int mt, nt;
  g_tile_of(blockIdx.x, MT, NT, mx, ngm, mt, nt);
  const unsigned lds_off = lds_offset_of(lds);

  GPipe pipe;
  GProd& p = pipe.prod;
  const long long strip = (long long)KB * FRAG_BYTES;
  p.a_tile = 2 * strip;
  p.a_kb = FRAG_BYTES;
  p.w_kb = FRAG_BYTES;
  p.pa = T + (long long)(8 * mt + 2 * w) * 2 * strip;
  p.pa2 = p.pa + strip;
  p.pw = wVg + (long long)(4 * nt + w) * strip;
  p.pw2 = wVu + (long long)(4 * nt + w) * strip;
  p.lane16 = lane * 16;
  p.dst = lds_off + 2 * w * FRAG_BYTES;
  p.dstw = lds_off + (8 + w) * FRAG_BYTES;
  p.slot = 0;
  p.issued = 0;
  p.total = 2 * KB;        // gate units, then up units
  p.switch_at = KB;
  pipe.rdA = lds_off + lane * 16 + 4 * wm * FRAG_BYTES;
  pipe.rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  pipe.rslot = 0;
  pipe.done = 0;
  pipe.start();

  f32x16 acc[2][4];
  g_zero(acc);
  pipe.run(acc, KB);
  // SiLU(G), rounded to bf16 and kept as pairs while the up tile is accumulated
  unsigned S[2][4][8];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float g0 = acc[i][j][2 * e], g1 = acc[i][j][2 * e + 1];
        const float s0 = g0 * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g0 * -1.44269504088896f));
        const float s1 = g1 * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g1 * -1.44269504088896f));
        bf16x2 b;
        b[0] = (__bf16)s0;
        b[1] = (__bf16)s1;
        S[i][j][e] = __builtin_bit_cast(unsigned, b);
        asm volatile("" : "+v"(S[i][j][e]));  // computed here, not sunk below the second phase next to its use
      }
  g_zero(acc);
  pipe.run(acc, KB);
  pipe.finish();

  // H frags: registers 8t..8t+7 of tile (i, j) are the frag of ffn contraction block 2 (ffn tile) + t, row tile j
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const long long mtile = 8 * mt + 4 * wm + j;
      const int kb0 = 2 * (4 * nt + 2 * wn + i);
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const unsigned sp = S[i][j][4 * t + e];
          const float s0 = __builtin_bit_cast(float, sp << 16), s1 = __builtin_bit_cast(float, sp & 0xffff0000u);
          o[2 * e] = (__bf16)(s0 * acc[i][j][8 * t + 2 * e]);
          o[2 * e + 1] = (__bf16)(s1 * acc[i][j][8 * t + 2 * e + 1]);
        }
        *reinterpret_cast<bf16x8*>(H + ((mtile * KBf + kb0 + t) * 64 + lane) * 16) = o;
      }
    }
}

// ------------------------------------------------------------------------------------------------
// Tdp[split] = H Ud over the split's ffn range   (first phase of the down-projection XUV kernel, Alg. 2)
// wUd: [ffn / 16][rank tile] frags.  Tdp: [split][32-row tile][rank tile][4 register groups][lane][4] fp32.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void k_down1(const char* __restrict__ H, const char* __restrict__ wUd,
                                                  float* __restrict__ Tdp, int KBf, int nq_total, int MT, int QT, int splits) {
  __shared__ __attribute__((aligned(1024))) char lds[G_LDS];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 2, wn = w % 2;
  // ffn range major: an XCD works on one range (or a few), whose slice of Ud stays in its L2 for every row tile
  const int L = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int qt = L % QT, mt = (L / QT) % MT, sp = L / (QT * MT);
  const int npairs = KBf / 2;
  const int u0 = 2 * (npairs * sp / splits), u1 = 2 * (npairs * (sp + 1) / splits);  // npairs * splits < 2^31 (host)
  const unsigned lds_off = lds_offset_of(lds);

  GPipe pipe;
  GProd& p = pipe.prod;
  p.a_tile = (long long)KBf * FRAG_BYTES;
  p.a_kb = FRAG_BYTES;
  p.w_kb = (long long)nq_total * FRAG_BYTES;
  p.pa = H + ((long long)(8 * mt + 2 * w) * KBf + u0) * FRAG_BYTES;
  p.pw = wUd + ((long long)u0 * nq_total + 4 * qt + w) * FRAG_BYTES;
  p.pa2 = p.pa;
  p.pw2 = p.pw;
  p.lane16 = lane * 16;
  p.dst = lds_off + 2 * w * FRAG_BYTES;
  p.dstw = lds_off + (8 + w) * FRAG_BYTES;
  p.slot = 0;
  p.issued = 0;
  p.total = u1 - u0;
  p.switch_at = -1;
  pipe.rdA = lds_off + lane * 16 + 4 * wm * FRAG_BYTES;
  pipe.rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  pipe.rslot = 0;
  pipe.done = 0;
  pipe.start();

  f32x16 acc[2][4];
  g_zero(acc);
  pipe.run(acc, u1 - u0);
  pipe.finish();

  const long long MT32 = 8LL * MT;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const long long mtile = 8 * mt + 4 * wm + j;
      const int q = 4 * qt + 2 * wn + i;
      f32x4* dst = reinterpret_cast<f32x4*>(Tdp + (((long long)sp * MT32 + mtile) * nq_total + q) * 1024) + lane;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        dst[g * 64] = v;
      }
    }
}

int gemm_splits(int64_t mt256, int64_t qt, int64_t nsteps) {
  // two workgroups per CU on 256 CUs; every split keeps at least four pairs of units
  int64_t s = (512 + mt256 * qt - 1) / (mt256 * qt);
  if (s > nsteps / 4) s = nsteps / 4;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  return (int)s;
}

int launch_gate_up(const Ctx* c, int MT256, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int NT = (int)(p.ffn / 128);
  // the most row tiles per XCD whose strips (256 x 2r bf16 each) fit in half of its 4 MiB L2
  int mx = 0, ngm = 0;
  const long long strip = 256LL * 2 * p.r * 2;
  for (int m = 8; m >= 1; m /= 2) {
    if (MT256 % m || m * strip > (2LL << 20)) continue;
    const int g = MT256 / m;
    if (g > 8 || 8 % g || NT % (8 / g)) continue;
    mx = m;
    ngm = g;
    break;
  }
  hipLaunchKernelGGL(k_gate_up, dim3(MT256 * NT), dim3(256), 0, st, ws + p.off_T, ws + p.off_wVg, ws + p.off_wVu,
                     ws + p.off_Hfull, (int)(p.r / 16), (int)(p.ffn / 16), MT256, NT, mx, ngm);
  return (int)hipGetLastError();
}

int launch_down1(const Ctx* c, int MT256, int splits, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int QT = (int)(p.rd / 128);
  hipLaunchKernelGGL(k_down1, dim3(MT256 * QT * splits), dim3(256), 0, st, ws + p.off_Hfull, ws + p.off_wUd,
                     reinterpret_cast<float*>(ws + p.off_Tdp), (int)(p.ffn / 16), (int)(p.rd / 32), MT256, QT, splits);
  return (int)hipGetLastError();
}

}  // namespace svdmlp
