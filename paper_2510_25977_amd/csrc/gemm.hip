// bf16 MFMA path for large M with the ffn-wide activation staged through HBM (paper Alg. 3 writes the
// gated activation out and Alg. 2 reads it back for the down projection), gfx950.
//
//   k_gate_up   H    = SiLU(Tg Vg) .* (Tu Vu)     256 rows x 256 ffn columns per tile; the gate tile is accumulated
//                                                 first, squashed to SiLU(G) in bf16 pairs, then the up tile is
//                                                 accumulated on top and multiplied in; H leaves as frags
//   k_down1     Tdp  = H Ud over one ffn range     256 rows x 256 rank columns per workgroup, fp32 partials
//   k_out       Y    = Td Vd                       256 rows x 256 columns per workgroup
//
// Why not keep H in registers: a workgroup that owns every rank column of its rows (so that H never has to be
// stored) has room for only 128 rows, and then each byte brought into the CU feeds too few MFMAs.  A CU pulls
// operands in at a bounded rate (measured: 44 B/clk from L2 at best, 20 - 25 B/clk at these kernels' L2 miss rates),
// and the matrix cores, whose clock is power-limited, take 256 x 256 tiles of real data at about 22 B/clk (they would
// take 32 B/clk on all-zero operands): with 16 KiB of operands per 64 MFMAs the 256 x 256 tile is just fed, the
// 128-row fused tile, which needs two to four times the bytes per MFMA, is not.  The price is one write and one read
// of H.
//
// Both kernels are one machine: eight waves, two per SIMD, 128 accumulator registers per lane; wave w owns rows
// 128 (w / 4).. and columns 64 (w % 4).. of the tile.  Operands arrive as 1 KiB frags (common.h).  A "unit" is one
// contraction block (16) of the tile: 8 activation frags (256 rows) + 8 weight frags (256 columns) = 16 KiB.  A
// step is two units; LDS holds four steps (128 KiB).
//
// The two waves of a SIMD (w and w + 4) alternate between a memory phase and a compute phase, half a period
// apart, so that the SIMD's matrix core always has exactly one wave feeding it while the other one fetches:
//   memory phase of step s:  issue the copies of step s+2 (into the slot of step s-2), read the twelve frags of
//                            step s from LDS, do any vector-ALU work that is due (SiLU, output conversion), wait
//                            for this wave's copies of step s+1, barrier
//   compute phase of step s: 16 MFMAs and nothing else; barrier
// Every barrier is a workgroup barrier; waves 4..7 pass one extra barrier at the start, which puts them one phase
// behind waves 0..3 for the rest of the kernel.  Step s is read by waves 0..3 in phase 2s and by waves 4..7 in
// phase 2s+1; its copies were waited for before the barrier that opens phase 2s, and its slot is
// written again by copies issued in phase 2s+4 or later.
#include "common.h"
#include <type_traits>

namespace svdmlp {

constexpr int G_UNIT = 16 * FRAG_BYTES;
constexpr int G_STEP = 2 * G_UNIT;
constexpr int G_SLOTS = 4;  // steps
constexpr int G_LDS = G_SLOTS * G_STEP;
constexpr int G_THREADS = 512;

// 16 bytes per lane, global -> LDS, with a wave-uniform 64-bit base in SGPRs and a 32-bit per-lane offset:
// no vector ALU work per copy.  M0 carries the (wave-uniform) LDS destination; lane l lands at M0 + 16 l.
// The compiler does not look into the asm, so it does not know that the instruction reads the base SGPRs as a memory
// address: a base that a vector instruction has just written (v_readfirstlane, or v_readlane when the compiler
// restores a spilled SGPR) must be five wait states old by then, and nothing here waits (a leading s_nop was
// measured: +2 % on k_gate_up, whose memory phases start with these copies).  An experimental build whose register
// pressure put such a restore right before a store took a memory fault, so the build step checks the generated
// assembly of this file for that pattern (build.py, check_sgpr_hazards) and fails if it finds one; the same holds
// for the stores below.
__device__ __forceinline__ void dma16_sv(const char* sbase, unsigned voff, unsigned lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0" ::"s"(sbase), "v"(voff), "s"(lds_dst) : "memory", "m0");
}

// The same copy with the non-temporal hint, for the gated activation that k_down1 reads once and nobody reads again
// (measured: the forward 1 % shorter, most of it in the next forward's first kernel, whose operands stay in L2; the
// same hint on the weight tiles of k_gate_up, which four workgroups of an XCD read at about the same time, made
// that kernel 7 % longer).
__device__ __forceinline__ void dma16_sv_nt(const char* sbase, unsigned voff, unsigned lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0 nt" ::"s"(sbase), "v"(voff), "s"(lds_dst) : "memory", "m0");
}

// LDS unit layout: frags 0..7 activation (32-row tiles of the 256 rows), frags 8..15 weights (32-column tiles).
// Producer of the step stream; all state is wave-uniform.  Wave w copies activation frag w and weight frag w of
// both units of a step.
struct GProd {
  const char* pa;        // this wave's activation frag of the next unit
  const char* pw;        // this wave's weight frag of the next unit
  long long a_kb, w_kb;  // byte distance between consecutive contraction blocks
  unsigned lane16;
  unsigned dst;          // LDS address of this wave's activation frag in slot 0, unit 0
  unsigned dstw;         // ... and of its weight frag
  int slot;              // slot the next step goes to
  int issued;            // steps issued so far

  template <int NTA = 0, int NTW = 0>
  __device__ __forceinline__ void step() {
    const unsigned b = dst + slot * G_STEP, bw = dstw + slot * G_STEP;
    if (NTA) dma16_sv_nt(pa, lane16, b); else dma16_sv(pa, lane16, b);
    if (NTW) dma16_sv_nt(pw, lane16, bw); else dma16_sv(pw, lane16, bw);
    if (NTA) dma16_sv_nt(pa + a_kb, lane16, b + G_UNIT); else dma16_sv(pa + a_kb, lane16, b + G_UNIT);
    if (NTW) dma16_sv_nt(pw + w_kb, lane16, bw + G_UNIT); else dma16_sv(pw + w_kb, lane16, bw + G_UNIT);
    pa += 2 * a_kb;
    pw += 2 * w_kb;
    slot = (slot + 1) & (G_SLOTS - 1);
    ++issued;
  }
};

// Operand registers of a wave: four activation and two weight frags for each of the two units of a step.  All of
// them are read in the memory phase, so the compute phase issues nothing but MFMAs.
struct GRegs {
  u32x4 A0, A1, A2, A3, Wa0, Wa1, B0, B1, B2, B3, Wb0, Wb1;
};

struct GCons {
  GRegs R;
  unsigned rdA, rdW;  // per-lane LDS read addresses in slot 0
  unsigned rdAh;      // ... of the activation frags when the tile has 128 rows (k_gate_up's half tiles)
  unsigned rdX0, rdX1;  // ... of this lane's 16-byte pieces of row-major activation rows (k_in), first / second unit
  int slot;           // slot of the step that is read next
  int done;           // steps consumed

  // memory phase, LDS part
  __device__ __forceinline__ void fetch() {
    const unsigned aA = rdA + slot * G_STEP, aW = rdW + slot * G_STEP;
    slot = (slot + 1) & (G_SLOTS - 1);
    R.Wa0 = lds_read<0 * FRAG_BYTES>(aW);
    R.Wa1 = lds_read<1 * FRAG_BYTES>(aW);
    R.A0 = lds_read<0 * FRAG_BYTES>(aA);
    R.A1 = lds_read<1 * FRAG_BYTES>(aA);
    R.A2 = lds_read<2 * FRAG_BYTES>(aA);
    R.A3 = lds_read<3 * FRAG_BYTES>(aA);
    R.Wb0 = lds_read<G_UNIT + 0 * FRAG_BYTES>(aW);
    R.Wb1 = lds_read<G_UNIT + 1 * FRAG_BYTES>(aW);
    R.B0 = lds_read<G_UNIT + 0 * FRAG_BYTES>(aA);
    R.B1 = lds_read<G_UNIT + 1 * FRAG_BYTES>(aA);
    R.B2 = lds_read<G_UNIT + 2 * FRAG_BYTES>(aA);
    R.B3 = lds_read<G_UNIT + 3 * FRAG_BYTES>(aA);
  }
  // compute phase.  acc[i][j]: weight tile i (rows of the transposed product), activation tile j (lanes).
  // FIRST: the accumulators start from zero with this step (the zero is the MFMA's C operand).
  template <bool FIRST>
  __device__ __forceinline__ void compute(f32x16 (&acc)[2][4]) {
    ++done;
    f32x16 z;
#pragma unroll
    for (int e = 0; e < 16; ++e) z[e] = 0.f;
    lgkm_wait<6>(R.A0, R.A1, R.A2, R.A3, R.Wa0, R.Wa1);
    acc[0][0] = mfma32(as_bf16x8(R.Wa0), as_bf16x8(R.A0), FIRST ? z : acc[0][0]);
    acc[1][0] = mfma32(as_bf16x8(R.Wa1), as_bf16x8(R.A0), FIRST ? z : acc[1][0]);
    acc[0][1] = mfma32(as_bf16x8(R.Wa0), as_bf16x8(R.A1), FIRST ? z : acc[0][1]);
    acc[1][1] = mfma32(as_bf16x8(R.Wa1), as_bf16x8(R.A1), FIRST ? z : acc[1][1]);
    acc[0][2] = mfma32(as_bf16x8(R.Wa0), as_bf16x8(R.A2), FIRST ? z : acc[0][2]);
    acc[1][2] = mfma32(as_bf16x8(R.Wa1), as_bf16x8(R.A2), FIRST ? z : acc[1][2]);
    acc[0][3] = mfma32(as_bf16x8(R.Wa0), as_bf16x8(R.A3), FIRST ? z : acc[0][3]);
    acc[1][3] = mfma32(as_bf16x8(R.Wa1), as_bf16x8(R.A3), FIRST ? z : acc[1][3]);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<0>(R.B0, R.B1, R.B2, R.B3, R.Wb0, R.Wb1);
    acc[0][0] = mfma32(as_bf16x8(R.Wb0), as_bf16x8(R.B0), acc[0][0]);
    acc[1][0] = mfma32(as_bf16x8(R.Wb1), as_bf16x8(R.B0), acc[1][0]);
    acc[0][1] = mfma32(as_bf16x8(R.Wb0), as_bf16x8(R.B1), acc[0][1]);
    acc[1][1] = mfma32(as_bf16x8(R.Wb1), as_bf16x8(R.B1), acc[1][1]);
    acc[0][2] = mfma32(as_bf16x8(R.Wb0), as_bf16x8(R.B2), acc[0][2]);
    acc[1][2] = mfma32(as_bf16x8(R.Wb1), as_bf16x8(R.B2), acc[1][2]);
    acc[0][3] = mfma32(as_bf16x8(R.Wb0), as_bf16x8(R.B3), acc[0][3]);
    acc[1][3] = mfma32(as_bf16x8(R.Wb1), as_bf16x8(R.B3), acc[1][3]);
    __builtin_amdgcn_sched_barrier(0);
  }
  // Memory phase when the activation comes straight from row-major memory (k_in): a step's activation part is
  // 256 rows x 64 bytes, sixteen rows per KiB, the 16-byte pieces of a row XOR-swizzled by bits 2..3 of the row
  // (so that a quarter wave's reads fall into distinct banks); rows 0..127 sit where the first unit's activation
  // frags would, rows 128..255 in the second unit's place.  Piece 2 u + h of a row is natural-order half h of
  // contraction block u.
  __device__ __forceinline__ void fetch_x() {
    const unsigned a0 = rdX0 + slot * G_STEP, a1 = rdX1 + slot * G_STEP, aW = rdW + slot * G_STEP;
    slot = (slot + 1) & (G_SLOTS - 1);
    R.Wa0 = lds_read<0 * FRAG_BYTES>(aW);
    R.Wa1 = lds_read<1 * FRAG_BYTES>(aW);
    R.A0 = lds_read<0 * FRAG_BYTES>(a0);
    R.A1 = lds_read<2 * FRAG_BYTES>(a0);
    R.A2 = lds_read<4 * FRAG_BYTES>(a0);
    R.A3 = lds_read<6 * FRAG_BYTES>(a0);
    R.Wb0 = lds_read<G_UNIT + 0 * FRAG_BYTES>(aW);
    R.Wb1 = lds_read<G_UNIT + 1 * FRAG_BYTES>(aW);
    R.B0 = lds_read<0 * FRAG_BYTES>(a1);
    R.B1 = lds_read<2 * FRAG_BYTES>(a1);
    R.B2 = lds_read<4 * FRAG_BYTES>(a1);
    R.B3 = lds_read<6 * FRAG_BYTES>(a1);
  }
  // The same two phases for a tile of 128 rows: two activation frags per unit, accumulators acc[i][0..1].
  __device__ __forceinline__ void fetch_half() {
    const unsigned aA = rdAh + slot * G_STEP, aW = rdW + slot * G_STEP;
    slot = (slot + 1) & (G_SLOTS - 1);
    R.Wa0 = lds_read<0 * FRAG_BYTES>(aW);
    R.Wa1 = lds_read<1 * FRAG_BYTES>(aW);
    R.A0 = lds_read<0 * FRAG_BYTES>(aA);
    R.A1 = lds_read<1 * FRAG_BYTES>(aA);
    R.Wb0 = lds_read<G_UNIT + 0 * FRAG_BYTES>(aW);
    R.Wb1 = lds_read<G_UNIT + 1 * FRAG_BYTES>(aW);
    R.B0 = lds_read<G_UNIT + 0 * FRAG_BYTES>(aA);
    R.B1 = lds_read<G_UNIT + 1 * FRAG_BYTES>(aA);
  }
  template <bool FIRST>
  __device__ __forceinline__ void compute_half(f32x16 (&acc)[2][4]) {
    ++done;
    f32x16 z;
#pragma unroll
    for (int e = 0; e < 16; ++e) z[e] = 0.f;
    lgkm_wait<4>(R.A0, R.A1, R.Wa0, R.Wa1);
    acc[0][0] = mfma32(as_bf16x8(R.Wa0), as_bf16x8(R.A0), FIRST ? z : acc[0][0]);
    acc[1][0] = mfma32(as_bf16x8(R.Wa1), as_bf16x8(R.A0), FIRST ? z : acc[1][0]);
    acc[0][1] = mfma32(as_bf16x8(R.Wa0), as_bf16x8(R.A1), FIRST ? z : acc[0][1]);
    acc[1][1] = mfma32(as_bf16x8(R.Wa1), as_bf16x8(R.A1), FIRST ? z : acc[1][1]);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<0>(R.B0, R.B1, R.Wb0, R.Wb1);
    acc[0][0] = mfma32(as_bf16x8(R.Wb0), as_bf16x8(R.B0), acc[0][0]);
    acc[1][0] = mfma32(as_bf16x8(R.Wb1), as_bf16x8(R.B0), acc[1][0]);
    acc[0][1] = mfma32(as_bf16x8(R.Wb0), as_bf16x8(R.B1), acc[0][1]);
    acc[1][1] = mfma32(as_bf16x8(R.Wb1), as_bf16x8(R.B1), acc[1][1]);
    __builtin_amdgcn_sched_barrier(0);
  }
};

// End of a memory phase: this wave's copies of the next step have landed (those of the step after it, if it has
// been issued, may stay in flight: four copies), then the phase barrier.
__device__ __forceinline__ void g_certify(const GProd& prod, const GCons& cons) {
  if (prod.issued >= cons.done + 3) wait_vmcnt<4>();
  else wait_vmcnt<0>();
  lds_barrier();
}

// Workgroup -> tile of k_gate_up.  Tile ids that are congruent mod 8 run on the same XCD (workgroup ids go
// round-robin over the XCDs and a workgroup's tiles are 256 k apart).  With mx > 0 the XCDs form a grid of ngm row
// groups x 8 / ngm column groups; an XCD owns mx row tiles (their rank-r strips stay in its L2) and
// NT / (8 / ngm) column tiles, walked row tile fastest so that the workgroups that need the same weight tile run
// together.  mx = 0: plain order.
__device__ __forceinline__ void g_tile_of(int id, int MT, int NT, int mx, int ngm, int& mt, int& nt) {
  if (mx > 0) {
    const int x = id % 8, i = id / 8;
    mt = (x % ngm) * mx + i % mx;
    nt = (x / ngm) * (NT / (8 / ngm)) + i / mx;
  } else {
    mt = id % MT;
    nt = id / MT;
  }
}

// 16 bytes per lane to a wave-uniform base plus a 32-bit per-lane offset (no 64-bit vector address arithmetic).
// The data registers of a store wider than 8 bytes must not be rewritten by the vector ALU in the next two issue
// slots; the compiler cannot see into the asm, so the wait states are part of it.
__device__ __forceinline__ void store16_sv(char* sbase, unsigned voff, const u32x4& v) {
  asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(voff), "v"(v), "s"(sbase) : "memory");
}

// The same with the non-temporal hint, for data that is written once and read by a later kernel (the gated
// activation): the lines do not stay dirty in the writer's L2, which measurably shortens both this kernel and its
// consumer.
__device__ __forceinline__ void store16_sv_nt(char* sbase, unsigned voff, const u32x4& v) {
  asm volatile("global_store_dwordx4 %0, %1, %2 nt\n\ts_nop 1" ::"v"(voff), "v"(v), "s"(sbase) : "memory");
}

__device__ __forceinline__ unsigned silu_pair(float g0, float g1) {
  const float s0 = g0 * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g0 * -1.44269504088896f));
  const float s1 = g1 * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g1 * -1.44269504088896f));
  bf16x2 b;
  b[0] = (__bf16)s0;
  b[1] = (__bf16)s1;
  return __builtin_bit_cast(unsigned, b);
}
__device__ __forceinline__ unsigned mul_pair(unsigned sp, float p0, float p1) {
  const float s0 = __builtin_bit_cast(float, sp << 16), s1 = __builtin_bit_cast(float, sp & 0xffff0000u);
  bf16x2 b;
  b[0] = (__bf16)(s0 * p0);
  b[1] = (__bf16)(s1 * p1);
  return __builtin_bit_cast(unsigned, b);
}

// ------------------------------------------------------------------------------------------------
// H = SiLU(Tg Vg) .* (Tu Vu)   (paper Alg. 3, second loop nest and gating epilogue)
// T: per 32-row tile the gate strip's KB frags then the up strip's (as written by k_s1).
// wVg, wVu: [ffn tile][KB] frags.  H: [256-row tile][ffn / 16][8 row tiles of 32] chain-order frags (the eight
// activation frags of a unit of k_down1 are contiguous).
// Persistent: a workgroup works through its tiles (GuSched); the copy stream runs on into the next tile and a
// finished tile's stores are not waited for.
// ------------------------------------------------------------------------------------------------
// Tiles of one workgroup of k_gate_up.  ntiles = G q + rem tiles go to G workgroups.  If at most half of the
// workgroups would get a tile in the last round, the rem leftover tiles are cut into upper and lower halves
// (128 rows each) and given to 2 rem workgroups: the last round then costs about half a tile's time instead of a
// whole one.  MODE 0 (full tiles only): workgroup b takes tiles b, b + G, ... below `ntiles`.  MODE 1 (halves only):
// workgroup b takes one half of one of the tiles first .. first + rem - 1.  MODE 2 (both in one launch, so that the
// copy stream runs on from the last full tile into the half and no second launch ramps up): the full tiles below
// `first`, then, for the first 2 rem workgroups, a half as in MODE 1.
enum { GU_FULL = 0, GU_HALF = 1, GU_MIXED = 2 };
template <int MODE>
struct GuSched {
  int b, G, ntiles, first, rem;
  __device__ __forceinline__ void init(int b_, int G_, int ntiles_, int first_, int rem_) {
    b = b_; G = G_; ntiles = ntiles_; first = first_; rem = rem_;
  }
  // full tiles of this workgroup (MODE 2: those below `first`)
  __device__ __forceinline__ int nfull() const {
    const int n = MODE == GU_MIXED ? first : ntiles;
    return MODE == GU_HALF ? 0 : (b < n ? (n - 1 - b) / G + 1 : 0);
  }
  __device__ __forceinline__ int count() const {
    return MODE == GU_HALF ? 1 : MODE == GU_FULL ? nfull() : nfull() + (b < 2 * rem ? 1 : 0);
  }
  // k-th tile of this workgroup: id, and hh = -1 for a full tile, 0 / 1 for the upper / lower half
  __device__ __forceinline__ void tile(int k, int& id, int& hh) const {
    if (MODE == GU_FULL || (MODE == GU_MIXED && k < nfull())) {
      id = b + k * G;
      hh = -1;
    } else if (rem % 8 == 0) {  // both halves of a tile on one XCD, the one its id maps to
      id = first + 8 * (b / 16) + b % 8;
      hh = (b / 8) % 2;
    } else {
      id = first + b / 2;
      hh = b % 2;
    }
  }
};

struct GuTile {
  const char* pa_g;  // this wave's copy sources: gate strip / up strip of its row tile, gate / up frags of its column tile
  const char* pa_u;
  const char* pw_g;
  const char* pw_u;
};
// hh < 0: full tile, wave w copies activation frag w.  Half tile: the four activation frags are copied twice
// (waves w and w + 4 copy the same one), which keeps every wave at two copies per unit.
__device__ __forceinline__ GuTile gu_tile(int id, int hh, int w, const char* T, const char* wVg, const char* wVu, long long strip,
                                          int MT, int NT, int mx, int ngm) {
  int mt, nt;
  g_tile_of(id, MT, NT, mx, ngm, mt, nt);
  const int af = hh < 0 ? w : 4 * hh + w % 4;
  GuTile t;
  t.pa_g = T + (long long)(8 * mt + af) * 2 * strip;
  t.pa_u = t.pa_g + strip;
  t.pw_g = wVg + (long long)(8 * nt + w) * strip;
  t.pw_u = wVu + (long long)(8 * nt + w) * strip;
  return t;
}

// producer of k_gate_up: walks gate units, up units, then the next tile of this workgroup
template <int MODE>
struct GuProd {
  GProd prod;
  GuTile pt;
  GuSched<MODE> sched;
  const char* T;
  const char* wVg;
  const char* wVu;
  long long strip;
  int w, MT, NT, mx, ngm, KB, half, total_steps;
  int p_k, p_step;
  __device__ __forceinline__ void load_tile() {
    int id, hh;
    sched.tile(p_k, id, hh);
    pt = gu_tile(id, hh, w, T, wVg, wVu, strip, MT, NT, mx, ngm);
    prod.pa = pt.pa_g;
    prod.pw = pt.pw_g;
  }
  __device__ __forceinline__ void produce() {
    if (prod.issued < total_steps) {
      prod.step();
      ++p_step;
      if (p_step == half) {
        prod.pa = pt.pa_u;
        prod.pw = pt.pw_u;
      } else if (p_step == KB) {
        p_step = 0;
        ++p_k;
        if (p_k < sched.count()) load_tile();
      }
    }
  }
};

template <int MODE>
__global__ __launch_bounds__(G_THREADS) void k_gate_up(const char* __restrict__ T, const char* __restrict__ wVg,
                                                       const char* __restrict__ wVu, char* __restrict__ H, int KB, int KBf,
                                                       int MT, int NT, int mx, int ngm, int ntiles, int first, int rem) {
  __shared__ __attribute__((aligned(1024))) char lds[G_LDS];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 4, wn = w % 4;
  const unsigned lds_off = lds_offset_of(lds);
  const long long strip = (long long)KB * FRAG_BYTES;

  // producer: position in the stream
  GuProd<MODE> gp;
  GProd& prod = gp.prod;
  gp.sched.init(blockIdx.x, gridDim.x, ntiles, first, rem);
  const int my_tiles = gp.sched.count();
  prod.a_kb = FRAG_BYTES;
  prod.w_kb = FRAG_BYTES;
  prod.lane16 = lane * 16;
  prod.dst = lds_off + w * FRAG_BYTES;
  prod.dstw = lds_off + (8 + w) * FRAG_BYTES;
  prod.slot = 0;
  prod.issued = 0;
  gp.T = T; gp.wVg = wVg; gp.wVu = wVu;
  gp.strip = strip;
  gp.w = w; gp.MT = MT; gp.NT = NT; gp.mx = mx; gp.ngm = ngm;
  const int half = KB / 2;
  gp.KB = KB; gp.half = half;            // steps per tile (two phases), steps per phase
  gp.total_steps = my_tiles * KB;
  gp.p_k = 0;
  gp.p_step = 0;
  if (my_tiles > 0) gp.load_tile();

  GCons cons;
  cons.rdA = lds_off + lane * 16 + 4 * wm * FRAG_BYTES;
  cons.rdAh = lds_off + lane * 16 + 2 * wm * FRAG_BYTES;
  cons.rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  cons.slot = 0;
  cons.done = 0;

  gp.produce();
  gp.produce();
  if (prod.issued >= 2) wait_vmcnt<4>();
  else wait_vmcnt<0>();
  if (w >= 4) lds_barrier();  // second wave of each SIMD: one phase behind from here on
  lds_barrier();

  f32x16 acc[2][4];
  u32x4 S[16];  // SiLU(G) as bf16 pairs, frag by frag, while the up tile is accumulated
  // One tile: gate phase, SiLU, up phase, H out.  HALF: 128 rows; wave (wm, wn) then owns rows 64 wm.. of the half.
  auto one_tile = [&](auto half_c, int mt, int nt, int hh) __attribute__((always_inline)) {
    constexpr bool HALF = decltype(half_c)::value;
    char* hbase = H + ((((long long)mt * KBf + 2 * (8 * nt + 2 * wn)) * 8) + (HALF ? 4 * hh + 2 * wm : 4 * wm)) * FRAG_BYTES;
    constexpr int NB = HALF ? 2 : 4;
    // One step: memory phase (copies of a later step, LDS reads, the SiLU when it is due), compute phase.  FIRST: the
    // accumulators start from zero with this step.  The first step of each phase is written out apart from the loop
    // over the others (no run-time choice between the two kinds of compute phase inside a loop).
    auto step = [&](auto first_c, auto silu_c) __attribute__((always_inline)) {
      constexpr bool FIRST = decltype(first_c)::value, SILU = decltype(silu_c)::value;
      gp.produce();
      if (HALF) cons.fetch_half();
      else cons.fetch();
      if (SILU) {  // SiLU(G), rounded to bf16 pairs; runs under the other wave's compute phase
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
              u32x4 v;
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = silu_pair(acc[a][b][8 * t2 + 2 * e], acc[a][b][8 * t2 + 2 * e + 1]);
              asm volatile("" : "+v"(v));  // computed here, not sunk next to its use
              S[(a * 4 + b) * 2 + t2] = v;
            }
      }
      g_certify(gp.prod, cons);
      if (HALF) cons.template compute_half<FIRST>(acc);
      else cons.template compute<FIRST>(acc);
      lds_barrier();
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    // ---- gate phase ----
    step(T_{}, F_{});
    for (int i = 1; i < half; ++i) step(F_{}, F_{});
    // ---- up phase ----
    step(T_{}, T_{});
    for (int i = 1; i < half; ++i) step(F_{}, F_{});
    // H = SiLU(G) .* P rounded to bf16: registers 8t..8t+7 of tile (a, b) are the frag of ffn contraction block
    // 2 (ffn tile) + t, row tile b.  The stores are left in flight; the next tile's first phases run under them.
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          u32x4 v = S[(a * 4 + b) * 2 + t2];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = mul_pair(v[e], acc[a][b][8 * t2 + 2 * e], acc[a][b][8 * t2 + 2 * e + 1]);
          store16_sv_nt(hbase + ((long long)(2 * a + t2) * 8 + b) * FRAG_BYTES, gp.prod.lane16, v);
        }
  };
  for (int k = 0; k < my_tiles; ++k) {
    int id, hh, mt, nt;
    gp.sched.tile(k, id, hh);
    g_tile_of(id, MT, NT, mx, ngm, mt, nt);
    if constexpr (MODE == GU_FULL) {
      one_tile(std::false_type{}, mt, nt, hh);
    } else if constexpr (MODE == GU_HALF) {
      one_tile(std::true_type{}, mt, nt, hh);
    } else {
      if (hh < 0) one_tile(std::false_type{}, mt, nt, hh);
      else one_tile(std::true_type{}, mt, nt, hh);
    }
  }
  if (w < 4) lds_barrier();  // matches the extra barrier of waves 4..7
}

// ------------------------------------------------------------------------------------------------
// Tdp[split] = H Ud over the split's ffn range   (first phase of the down-projection XUV kernel, Alg. 2)
// wUd: [ffn / 16][rank tile] frags (rank a multiple of 256).
// Tdp: [split][32-row tile][rank tile][4 register groups][lane][4] fp32.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(G_THREADS) void k_down1(const char* __restrict__ H, const char* __restrict__ wUd,
                                                     float* __restrict__ Tdp, int KBf, int nq_total, int MT, int QT, int splits) {
  __shared__ __attribute__((aligned(1024))) char lds[G_LDS];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 4, wn = w % 4;
  // ffn range major: an XCD works on one range (or a few), whose slice of Ud stays in its L2 for every row tile
  const int L = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int qt = L % QT, mt = (L / QT) % MT, sp = L / (QT * MT);
  const int npairs = KBf / 2;
  const int s0 = npairs * sp / splits, s1 = npairs * (sp + 1) / splits;  // steps; npairs * splits < 2^31 (host)
  const int total_steps = s1 - s0;
  const unsigned lds_off = lds_offset_of(lds);

  GProd prod;
  prod.a_kb = 8 * FRAG_BYTES;
  prod.w_kb = (long long)nq_total * FRAG_BYTES;
  prod.pa = H + (((long long)mt * KBf + 2 * s0) * 8 + w) * FRAG_BYTES;
  prod.pw = wUd + ((long long)(2 * s0) * nq_total + 8 * qt + w) * FRAG_BYTES;
  prod.lane16 = lane * 16;
  prod.dst = lds_off + w * FRAG_BYTES;
  prod.dstw = lds_off + (8 + w) * FRAG_BYTES;
  prod.slot = 0;
  prod.issued = 0;
  GCons cons;
  cons.rdA = lds_off + lane * 16 + 4 * wm * FRAG_BYTES;
  cons.rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  cons.slot = 0;
  cons.done = 0;

  if (prod.issued < total_steps) prod.step<1, 0>();
  if (prod.issued < total_steps) prod.step<1, 0>();
  if (prod.issued >= 2) wait_vmcnt<4>();
  else wait_vmcnt<0>();
  if (w >= 4) lds_barrier();
  lds_barrier();

  f32x16 acc[2][4];
  for (int i = 0; i < total_steps; ++i) {
    if (prod.issued < total_steps) prod.step<1, 0>();
    cons.fetch();
    g_certify(prod, cons);
    if (i == 0) cons.compute<true>(acc);
    else cons.compute<false>(acc);
    lds_barrier();
  }
  if (w < 4) lds_barrier();

  const long long MT32 = 8LL * MT;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const long long mtile = 8 * mt + 4 * wm + j;
      const int q = 8 * qt + 2 * wn + i;
      f32x4* dst = reinterpret_cast<f32x4*>(Tdp + (((long long)sp * MT32 + mtile) * nq_total + q) * 1024) + lane;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
        dst[g * 64] = v;
      }
    }
}

// ------------------------------------------------------------------------------------------------
// T = X [Ug | Uu]   (paper Alg. 3, first loop nest; for kind LINEAR: T = X U), 256 rows x 256 rank columns per
// workgroup, contraction over d.  X row-major [M, d] bf16; wU: [rank tile][d / 16] natural-order frags.
// T: per 32-row tile two strips of r_strip / 16 chain-order frags each (rank columns below / from r_strip).
// Used when there are enough 256 x 256 tiles to fill the chip; k_s1 (128 x 128 tiles) otherwise.  With S > 1 the
// contraction is cut into S ranges (few tiles, long contraction): workgroup (tile, range) writes its fp32 tile to
// Tpart in k_reduce's layout ([range][32-row tile][32-column tile][4 register groups][lane][4]) and k_reduce adds
// the ranges and writes T.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(G_THREADS) void k_in(const uint16_t* __restrict__ X, int M, int d, const char* __restrict__ wU,
                                                  int r_strip, char* __restrict__ T, int MT, int PT, int S,
                                                  float* __restrict__ Tpart) {
  __shared__ __attribute__((aligned(1024))) char lds[G_LDS];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 4, wn = w % 4;
  const int L = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int sp = L % S, pt = (L / S) % PT, mt = L / (S * PT);
  const int KBd = d / 16, KBr = r_strip / 16;
  const int s0 = (d / 32) * sp / S, s1 = (d / 32) * (sp + 1) / S;   // steps of this range
  const int total_steps = s1 - s0;
  const unsigned lds_off = lds_offset_of(lds);

  // producer: rows 16 w + lane / 4 of each half of the tile, one 16-byte piece per lane (rows beyond M re-read row
  // M - 1; they only feed output rows that nobody uses)
  const int rl = lane / 4, piece = (lane % 4) ^ ((lane >> 4) & 3);
  int rowA = 256 * mt + 16 * w + rl, rowB = rowA + 128;
  rowA = rowA < M ? rowA : M - 1;
  rowB = rowB < M ? rowB : M - 1;
  const unsigned voffA = (unsigned)rowA * (unsigned)d * 2u + piece * 16, voffB = (unsigned)rowB * (unsigned)d * 2u + piece * 16;
  const char* bx = reinterpret_cast<const char*>(X) + (long long)s0 * 64;
  const char* pw = wU + ((long long)(8 * pt + w) * KBd + 2 * s0) * FRAG_BYTES;
  const unsigned lane16 = lane * 16;
  const unsigned dst = lds_off + w * FRAG_BYTES, dstw = lds_off + (8 + w) * FRAG_BYTES;
  int pslot = 0, issued = 0;
  auto produce = [&]() __attribute__((always_inline)) {
    if (issued < total_steps) {
      const unsigned b = dst + pslot * G_STEP, bw = dstw + pslot * G_STEP;
      dma16_sv(bx, voffA, b);
      dma16_sv(pw, lane16, bw);
      dma16_sv(bx, voffB, b + G_UNIT);
      dma16_sv(pw + FRAG_BYTES, lane16, bw + G_UNIT);
      bx += 64;
      pw += 2 * FRAG_BYTES;
      pslot = (pslot + 1) & (G_SLOTS - 1);
      ++issued;
    }
  };

  GCons cons;
  const int il = lane % 32, h = lane / 32, sw = (il >> 2) & 3;
  const unsigned c0 = (il / 16) * FRAG_BYTES + (il % 16) * 64;
  cons.rdX0 = lds_off + wm * G_UNIT + c0 + ((0 + h) ^ sw) * 16;
  cons.rdX1 = lds_off + wm * G_UNIT + c0 + ((2 + h) ^ sw) * 16;
  cons.rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  cons.slot = 0;
  cons.done = 0;

  produce();
  produce();
  if (issued >= 2) wait_vmcnt<4>();
  else wait_vmcnt<0>();
  if (w >= 4) lds_barrier();
  lds_barrier();

  f32x16 acc[2][4];
  for (int i = 0; i < total_steps; ++i) {
    produce();
    cons.fetch_x();
    if (issued >= cons.done + 3) wait_vmcnt<4>();
    else wait_vmcnt<0>();
    lds_barrier();
    if (i == 0) cons.compute<true>(acc);
    else cons.compute<false>(acc);
    lds_barrier();
  }
  if (w < 4) lds_barrier();

  if (S > 1) {
    const long long MT32 = 8LL * MT;
    const int nq = 8 * PT;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const long long mtile = 8 * mt + 4 * wm + j;
        const int q = 8 * pt + 2 * wn + i;
        f32x4* dstp = reinterpret_cast<f32x4*>(Tpart + (((long long)sp * MT32 + mtile) * nq + q) * 1024) + lane;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          dstp[g * 64] = v;
        }
      }
    return;
  }
  // registers 8t..8t+7 of tile (i, j) are the chain-order frag of rank contraction block 2 (rank tile) + t, row tile j
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int p0 = 32 * (8 * pt + 2 * wn + i);
    const int which = p0 >= r_strip ? 1 : 0;
    const int kb0 = (p0 - which * r_strip) / 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const long long mtile = 8 * mt + 4 * wm + j;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const u32x4 v = __builtin_bit_cast(u32x4, pack_chain(acc[i][j], t));
        store16_sv(T + ((mtile * 2 + which) * KBr + kb0 + t) * FRAG_BYTES, lane16, v);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Y = Td Vd   (second phase of the down-projection XUV kernel, Alg. 2), 256 rows x 256 columns per workgroup.
// Td: [32-row tile][rd / 16] chain-order frags; wVd: [column tile][rd / 16] frags; Y row-major [M, d] bf16.
// The accumulators hold the tile transposed (lane = row, registers = columns); each wave turns its 128 x 64 part
// around through a private piece of LDS (rows padded to 144 bytes so that a half wave's writes fall into
// different banks) and stores whole 128-byte row segments.
// ------------------------------------------------------------------------------------------------
constexpr int OUT_ROW = 144;                      // bytes per staged row: 64 bf16 + 16 bytes of padding
constexpr int OUT_WAVE = 128 * OUT_ROW;           // 18 KiB per wave
constexpr int OUT_LDS = 8 * OUT_WAVE > G_LDS ? 8 * OUT_WAVE : G_LDS;

__global__ __launch_bounds__(G_THREADS) void k_out(const char* __restrict__ Td, const char* __restrict__ wVd,
                                                   uint16_t* __restrict__ Y, int M, int d, int KBq, int MT, int CT) {
  __shared__ __attribute__((aligned(1024))) char lds[OUT_LDS];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 4, wn = w % 4;
  const int L = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int ct = L % CT, mt = L / CT;
  const int total_steps = KBq / 2;
  const unsigned lds_off = lds_offset_of(lds);

  GProd prod;
  prod.a_kb = FRAG_BYTES;
  prod.w_kb = FRAG_BYTES;
  prod.pa = Td + (long long)(8 * mt + w) * KBq * FRAG_BYTES;
  prod.pw = wVd + (long long)(8 * ct + w) * KBq * FRAG_BYTES;
  prod.lane16 = lane * 16;
  prod.dst = lds_off + w * FRAG_BYTES;
  prod.dstw = lds_off + (8 + w) * FRAG_BYTES;
  prod.slot = 0;
  prod.issued = 0;
  GCons cons;
  cons.rdA = lds_off + lane * 16 + 4 * wm * FRAG_BYTES;
  cons.rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  cons.slot = 0;
  cons.done = 0;

  if (prod.issued < total_steps) prod.step();
  if (prod.issued < total_steps) prod.step();
  if (prod.issued >= 2) wait_vmcnt<4>();
  else wait_vmcnt<0>();
  if (w >= 4) lds_barrier();
  lds_barrier();

  f32x16 acc[2][4];
  for (int i = 0; i < total_steps; ++i) {
    if (prod.issued < total_steps) prod.step();
    cons.fetch();
    g_certify(prod, cons);
    if (i == 0) cons.compute<true>(acc);
    else cons.compute<false>(acc);
    lds_barrier();
  }
  if (w < 4) lds_barrier();
  // every wave has read its last operands and no copy is in flight: LDS is free

  char* stage = lds + w * OUT_WAVE;
  const int il = lane % 32, h = lane / 32;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {  // registers 4g..4g+3: columns 32 i + 8 g + 4 h + (0..3) of row 32 j + il
        bf16x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = (__bf16)acc[i][j][4 * g + e];
        *reinterpret_cast<bf16x4*>(stage + (32 * j + il) * OUT_ROW + (32 * i + 8 * g + 4 * h) * 2) = v;
      }
  // rows come back eight per instruction, 16 bytes per lane
  const int rsub = lane / 8, piece = lane % 8;
  const long long m0 = 256LL * mt + 128 * wm;
  const int c0 = 256 * ct + 64 * wn;
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const int row = 8 * k + rsub;
    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * OUT_ROW + piece * 16);
    if (m0 + row < M) *reinterpret_cast<u32x4*>(Y + (m0 + row) * d + c0 + piece * 8) = v;
  }
}

GuPlan gate_up_plan(int MT256, int64_t ffn, int64_t r, int ncu) {
  GuPlan g;
  const int NT = (int)(ffn / 256);
  // XCD grid: ngm row groups x 8 / ngm column groups, mx = MT256 / ngm row tiles per XCD.  The 32 workgroups of an XCD
  // work on mx row tiles x 32 / mx column tiles at a time and march through the contraction together, so per
  // contraction block the XCD's L2 fetches mx strips' and 32 / mx weight tiles' worth of operands for 64 operands'
  // worth of copies: the grid with the smallest mx + 32 / mx has the fewest L2 misses (4 x 8 or 8 x 4: 19 %).  A round
  // touches more than an L2 holds at any rank from 512 on, so nothing is kept from one round to the next and the size
  // of the strips does not enter (measured at r = 1024: 8 x 1 grid, whose strips fit L2, reads 537 MB, 4 x 2 reads
  // less and is faster).  Ties go to more row groups (smaller strips per XCD).  Plain order if nothing divides.
  g.mx = 0;
  g.ngm = 0;
  double best = 1e30;
  for (int gr = 8; gr >= 1; gr /= 2) {
    if (MT256 % gr || NT % (8 / gr)) continue;
    const int mx = MT256 / gr;
    const double a = mx < 32 ? mx : 32, cost = a + 32.0 / a;
    if (cost < best) { best = cost; g.mx = mx; g.ngm = gr; }
  }
  (void)r;
  if (ncu <= 0) ncu = 256;
  g.ntiles = MT256 * NT;
  g.G = g.ntiles < ncu ? g.ntiles : ncu;  // persistent: one workgroup per CU
  const int q = g.ntiles / g.G;
  g.rem = g.ntiles % g.G;
  g.halves = g.rem > 0 && 2 * g.rem <= g.G && q > 0;  // see GuSched
  g.nfull = g.halves ? q * g.G : g.ntiles;
  if (2 * g.ntiles <= ncu) {   // fewer tiles than half the CUs: every tile as two halves, twice the workgroups
    g.halves = true;
    g.nfull = 0;
    g.rem = g.ntiles;
  }
  return g;
}

int launch_gate_up(const Ctx* c, int MT256, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int NT = (int)(p.ffn / 256);
  const GuPlan g = gate_up_plan(MT256, p.ffn, p.r, c->n_cus);
  if (!g.halves)
    hipLaunchKernelGGL(k_gate_up<GU_FULL>, dim3(g.G), dim3(G_THREADS), 0, st, ws + p.off_T, ws + p.off_wVg, ws + p.off_wVu,
                       ws + p.off_Hfull, (int)(p.r / 16), (int)(p.ffn / 16), MT256, NT, g.mx, g.ngm, g.nfull, 0, 0);
  else if (g.nfull == 0)
    hipLaunchKernelGGL(k_gate_up<GU_HALF>, dim3(2 * g.rem), dim3(G_THREADS), 0, st, ws + p.off_T, ws + p.off_wVg, ws + p.off_wVu,
                       ws + p.off_Hfull, (int)(p.r / 16), (int)(p.ffn / 16), MT256, NT, g.mx, g.ngm, g.ntiles, g.nfull, g.rem);
  else   // whole rounds of full tiles, then the leftover tiles as halves, in one launch (2 rem <= G)
    hipLaunchKernelGGL(k_gate_up<GU_MIXED>, dim3(g.G), dim3(G_THREADS), 0, st, ws + p.off_T, ws + p.off_wVg, ws + p.off_wVu,
                       ws + p.off_Hfull, (int)(p.r / 16), (int)(p.ffn / 16), MT256, NT, g.mx, g.ngm, g.ntiles, g.nfull, g.rem);
  return (int)hipGetLastError();
}

int launch_down1(const Ctx* c, int MT256, int splits, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int QT = (int)(p.rd / 256);
  hipLaunchKernelGGL(k_down1, dim3(MT256 * QT * splits), dim3(G_THREADS), 0, st, ws + p.off_Hfull, ws + p.off_wUd,
                     reinterpret_cast<float*>(ws + p.off_Tdp), (int)(p.ffn / 16), (int)(p.rd / 32), MT256, QT, splits);
  return (int)hipGetLastError();
}

// act: [32-row tile][k / 16] chain-order frags; w: [32-column tile][k / 16] frags; Y row-major [M, n], n % 256 == 0
int launch_out_generic(const Ctx* c, const char* act, const char* w, int64_t M, void* Y, int MT256, int64_t n, int64_t k,
                       hipStream_t st) {
  (void)c;
  const int CT = (int)(n / 256);
  hipLaunchKernelGGL(k_out, dim3(MT256 * CT), dim3(G_THREADS), 0, st, act, w, (uint16_t*)Y, (int)M, (int)n, (int)(k / 16),
                     MT256, CT);
  return (int)hipGetLastError();
}

int launch_out(const Ctx* c, int64_t M, void* Y, int MT256, hipStream_t st) {
  const Plan& p = c->plan;
  return launch_out_generic(c, c->ws + p.off_Td, c->ws + p.off_wVd, M, Y, MT256, p.d, p.rd, st);
}

// ncols = rank columns of the product (2 r gated, r linear); r_strip = columns per strip of T; S = ranges of d
// (S > 1: fp32 tiles per range, added by k_reduce).
int launch_in(const Ctx* c, const void* X, int64_t M, int64_t ncols, int64_t r_strip, int S, hipStream_t st) {
  const Plan& p = c->plan;
  const int MT = (int)((M + 255) / 256), PT = (int)(ncols / 256);
  if (!first_valid(FIRST_IN, S, M, p.d, ncols)) return (int)hipErrorInvalidValue;
  if (S > 1 && (size_t)S * MT * 256 * ncols * 4 > p.part_bytes) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(k_in, dim3(MT * PT * S), dim3(G_THREADS), 0, st, (const uint16_t*)X, (int)M, (int)p.d, c->ws + p.off_wU,
                     (int)r_strip, c->ws + p.off_T, MT, PT, S, reinterpret_cast<float*>(c->ws + p.off_Tdp));
  int e = (int)hipGetLastError();
  if (e || S == 1) return e;
  return launch_reduce(c, reinterpret_cast<const float*>(c->ws + p.off_Tdp), c->ws + p.off_T, S, 8 * MT, (int)(ncols / 32), st);
}

}  // namespace svdmlp
