// bf16 MFMA-tiled (prefill) path of the factored gated MLP (paper Alg. 2 / Alg. 3), gfx950: the kernels with
// 128-row tiles and the host code that strings a forward together.
//
//   k_s1      T^T  = [Ug|Uu]^T X^T            rank-r strips of gate and up, written as chain-order frags
//   k_fused   H^T  = SiLU(Vg^T Tg^T) .* (Vu^T Tu^T)   per ffn chunk, kept in registers, immediately
//             Td^T += Ud^T H^T                 contracted with the down factor; fp32 partial per ffn range
//   k_reduce  Td   = sum of the partials, rounded to bf16 frags (fixed order: deterministic)
//   k_s5      Y    = Td Vd
//
// These four are the same machine: operands arrive as 1 KiB frags (common.h) through a ring of 16 KiB
// LDS slots filled by asynchronous global->LDS copies, waves read frags back with ds_read_b128 and feed
// v_mfma_f32_32x32x16_bf16.  The paper's "caching" of the rank-r strip (Sec. 4.2.1) becomes: the strip
// T is produced once by the first stage and re-read from L2 by the tiles that own its rows.  With k_fused the
// ffn-wide activation H (which the paper writes to HBM in Alg. 3) never leaves the register file; the default
// forward stages H through the workspace with the 256-row kernels of gemm.hip, which measure faster, and uses
// k_fused and k_s5 only on request or for extents those kernels do not take (staged_tail / bf16_tiled_forward below).
#include "common.h"

namespace svdmlp {

constexpr int NU = 9;  // ring slots (9 x 16 KiB = 144 KiB of the 160 KiB LDS)
constexpr int PD = 6;  // units kept in flight beyond the ones the current step consumes
constexpr int LDS_BYTES = NU * UNIT_BYTES;

// Ring protocol.  The unit stream is consumed in order; a step that consumes n units does
//   wait_vmcnt<4*(PD-n)>  -> the n units are in LDS (each wave issues 4 loads per unit, in order)
//   lds_barrier           -> every wave's part has landed, and every wave has left the previous step
//   issue n more units    -> into the slots the previous step has just released
//   compute
// so exactly PD units beyond the current step stay in flight.  Issuing never stops (sources are clamped
// at the end of the stream), which keeps the outstanding-load count the constant the wait relies on.

__device__ __forceinline__ const bf16x8* lds_frag(const char* lds, int slot, int frag, int lane) {
  return reinterpret_cast<const bf16x8*>(lds + slot * UNIT_BYTES + frag * FRAG_BYTES + lane * 16);
}

// ------------------------------------------------------------------------------------------------
// 2 x 2 register tile step shared by k_s1 and k_s5: one contraction block (16) of a 64 x 64 wave tile.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void mfma_2x2(const u32x4 (&R)[4], f32x16 (&acc)[2][2]) {
  acc[0][0] = mfma32(as_bf16x8(R[0]), as_bf16x8(R[2]), acc[0][0]);
  acc[0][1] = mfma32(as_bf16x8(R[0]), as_bf16x8(R[3]), acc[0][1]);
  acc[1][0] = mfma32(as_bf16x8(R[1]), as_bf16x8(R[2]), acc[1][0]);
  acc[1][1] = mfma32(as_bf16x8(R[1]), as_bf16x8(R[3]), acc[1][1]);
}

// ------------------------------------------------------------------------------------------------
// S1: T^T[p, m] = sum_k U^T[p, k] X^T[k, m]   (paper Alg. 3, first inner loop nest)
// workgroup tile 128 (p) x 128 (m); wave (wp, wq) owns 64 x 64.
// Unit stream: per 64-wide contraction step a unit of U^T frags (4 p tiles x 4 blocks) and a unit of X
// (128 rows x 64 columns, copied as 16 rows x 64 B per wave-load with the 16 B pieces XOR-swizzled by bits
// 2..3 of the row, so that the 16 lanes of a quarter wave hit 64 distinct banks when they read it back).
// ------------------------------------------------------------------------------------------------
template <int J>
__device__ __forceinline__ void s1_read(u32x4 (&R)[4], unsigned aP, unsigned aX0e, unsigned aX0o, unsigned aX1e, unsigned aX1o) {
  R[0] = lds_read<(0 * 4 + J) * FRAG_BYTES>(aP);
  R[1] = lds_read<(1 * 4 + J) * FRAG_BYTES>(aP);
  R[2] = lds_read<(J / 2) * FRAG_BYTES>((J & 1) ? aX0o : aX0e);
  R[3] = lds_read<(J / 2) * FRAG_BYTES>((J & 1) ? aX1o : aX1e);
}

// S > 1: the contraction over d is cut into S ranges (when the tiles alone would leave most CUs idle); every
// workgroup then writes its fp32 tile to Tpart in k_reduce's layout and k_reduce adds the ranges and writes T.
__global__ __launch_bounds__(256) void k_s1(const uint16_t* __restrict__ X, int M, int d, const char* __restrict__ wU,
                                            int r, char* __restrict__ T, int PT, int S, float* __restrict__ Tpart, int MT128) {
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);  // wave index, kept scalar
  const int wp = w / 2, wq = w % 2;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int sp = id % S, mt = (id / S) / PT, pt = (id / S) % PT;
  const int KBd = d / 16, KBr = r / 16;
  const int nks_all = d / 64;
  const int ks0 = nks_all * sp / S, nks = nks_all * (sp + 1) / S;   // this workgroup's contraction steps [ks0, nks)
  const unsigned lds_off = lds_offset_of(lds);

  // per-wave sources
  const char* srcP = wU + (size_t)(4 * pt + w) * KBd * FRAG_BYTES;  // + ks * 4 KiB + i * 1 KiB (+ lane * 16)
  const unsigned lane16 = lane * 16;
  const uint16_t* srcX[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rg = 2 * w + i / 2, kh = i % 2;
    int row = mt * 128 + 16 * rg + lane / 4;
    row = row < M ? row : M - 1;  // rows beyond M only feed output rows that are never used
    const int piece = (lane % 4) ^ ((lane >> 4) & 3);
    srcX[i] = X + (size_t)row * d + 32 * kh + 8 * piece;  // + ks * 64
  }
  const unsigned m0base = lds_off + (4 * w) * FRAG_BYTES;
  int pslot = 0, pks = ks0;   // producer: ring slot and contraction step of the next unit pair
  auto put_pair = [&]() __attribute__((always_inline)) {
    const int ks = pks < nks ? pks : nks - 1;   // past the end: re-read the last step (never consumed)
    const unsigned dP = m0base + pslot * UNIT_BYTES;
    const unsigned dX = m0base + (pslot + 1 == NU ? 0 : pslot + 1) * UNIT_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcP + (size_t)ks * 4096 + i * 1024 + lane16),
                                       (__attribute__((address_space(3))) void*)(uintptr_t)(dP + i * FRAG_BYTES), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcX[i] + ks * 64),
                                       (__attribute__((address_space(3))) void*)(uintptr_t)(dX + i * FRAG_BYTES), 16, 0, 0);
    pslot += 2;
    pslot = pslot >= NU ? pslot - NU : pslot;
    ++pks;
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // X frag addressing inside an X unit: row group rg (16 rows) and contraction half kh sit at (rg * 2 + kh) KiB;
  // within it row rho at rho * 64 B, piece p at slot p ^ bits 2..3 of rho.  Blocks j = 0, 1 are half kh = 0
  // (pieces h and 2 + h), blocks 2, 3 half kh = 1.
  const int il = lane % 32, h = lane / 32, rho = il % 16;
  unsigned xoff[2][2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int o = 0; o < 2; ++o) {
      const int rg = 2 * (2 * wq + b) + il / 16, piece = 2 * o + h;
      xoff[b][o] = (rg * 2) * FRAG_BYTES + rho * 64 + ((piece ^ ((rho >> 2) & 3)) * 16);
    }
  const unsigned pbase = lds_off + lane16 + (2 * wp) * 4 * FRAG_BYTES;

  put_pair(); put_pair(); put_pair();   // PD = 6 units
  int cslot = 0;
  for (int ks = ks0; ks < nks; ++ks) {
    wait_vmcnt<4 * (PD - 2)>();
    lds_barrier();
    const unsigned aP = pbase + cslot * UNIT_BYTES;
    const unsigned xs = lds_off + (cslot + 1 == NU ? 0 : cslot + 1) * UNIT_BYTES;
    cslot += 2;
    cslot = cslot >= NU ? cslot - NU : cslot;
    const unsigned x0e = xs + xoff[0][0], x0o = xs + xoff[0][1], x1e = xs + xoff[1][0], x1o = xs + xoff[1][1];
    u32x4 R0[4], R1[4], R2[4], R3[4];
    s1_read<0>(R0, aP, x0e, x0o, x1e, x1o);
    s1_read<1>(R1, aP, x0e, x0o, x1e, x1o);
    lgkm_wait<4>(R0[0], R0[1], R0[2], R0[3]);
    s1_read<2>(R2, aP, x0e, x0o, x1e, x1o);
    mfma_2x2(R0, acc);
    put_pair();
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<4>(R1[0], R1[1], R1[2], R1[3]);
    s1_read<3>(R3, aP, x0e, x0o, x1e, x1o);
    mfma_2x2(R1, acc);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<4>(R2[0], R2[1], R2[2], R2[3]);
    mfma_2x2(R2, acc);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<0>(R3[0], R3[1], R3[2], R3[3]);
    mfma_2x2(R3, acc);
    __builtin_amdgcn_sched_barrier(0);
  }
  wait_vmcnt<0>();
  if (S > 1) {
    // fp32 tile of this contraction range: [range][32-row tile][rank tile][4 register groups][lane][4]
    const int nq = 2 * r / 32;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const size_t tile = (size_t)(4 * mt + 2 * wq + b) * nq + 4 * pt + 2 * wp + a;
        f32x4* dst = reinterpret_cast<f32x4*>(Tpart + ((size_t)sp * 4 * MT128 * nq + tile) * 1024) + lane;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 v = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
          dst[g * 64] = v;
        }
      }
    return;
  }
  // epilogue: lane = activation row m; registers 8t..8t+7 are the chain-order frag of contraction block t
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int p0 = 32 * (4 * pt + 2 * wp + a);
    const int which = p0 >= r ? 1 : 0;
    const int kb0 = (p0 - which * r) / 16;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int mtile = 4 * mt + 2 * wq + b;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 v = pack_chain(acc[a][b], t);
        *reinterpret_cast<bf16x8*>(T + (((size_t)(mtile * 2 + which) * KBr + kb0 + t) * 64 + lane) * 16) = v;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Fused gate/up second stage + SiLU gate + down first stage (paper Alg. 3 second loop nest and
// epilogue, then the first phase of the down-projection XUV kernel of Alg. 2), for one 128-row tile
// and one range of ffn chunks.  Wave w owns rows 32w..32w+31 of the tile.
//   per chunk of 64 ffn columns:
//     A-steps (r / 64 of them): G^T, P^T += V^T frags (LDS, shared) x T frags (LDS, wave-private)
//     H = SiLU(G) .* P  -> bf16 chain frags in registers
//     B-steps: Td^T[q, m] += Ud^T frags (LDS, shared) x H frags (registers)
//
// Unit stream of a chunk: for each A-step the units V (gate/up frags of the chunk's two ffn tiles, 4
// contraction blocks), Tg, Tu (each wave's own row tile, 4 contraction blocks); then NB units of Ud frags.
// The producer runs exactly PD = 6 units (= two A-steps) ahead of the consumer, so which unit has to be issued
// at any consumer position is known at compile time relative to the end of the chunk; no cursor state machine.
// ------------------------------------------------------------------------------------------------

// Contraction block J (0..3) of an A-step: this wave's Tg and Tu frags and the four V frags (gate even / odd
// ffn tile, up even / odd).
template <int J>
__device__ __forceinline__ void fused_read_a(u32x4 (&R)[6], unsigned aTg, unsigned aTu, unsigned aV) {
  R[0] = lds_read<J * FRAG_BYTES>(aTg);
  R[1] = lds_read<J * FRAG_BYTES>(aTu);
  R[2] = lds_read<(0 * 4 + J) * FRAG_BYTES>(aV);
  R[3] = lds_read<(1 * 4 + J) * FRAG_BYTES>(aV);
  R[4] = lds_read<(2 * 4 + J) * FRAG_BYTES>(aV);
  R[5] = lds_read<(3 * 4 + J) * FRAG_BYTES>(aV);
}
__device__ __forceinline__ void fused_mfma_a(const u32x4 (&R)[6], f32x16* G, f32x16* P) {
  G[0] = mfma32(as_bf16x8(R[2]), as_bf16x8(R[0]), G[0]);
  G[1] = mfma32(as_bf16x8(R[3]), as_bf16x8(R[0]), G[1]);
  P[0] = mfma32(as_bf16x8(R[4]), as_bf16x8(R[1]), P[0]);
  P[1] = mfma32(as_bf16x8(R[5]), as_bf16x8(R[1]), P[1]);
}
// Frags 4 G4 .. 4 G4 + 3 of a B unit.
template <int G4>
__device__ __forceinline__ void fused_read_b(u32x4 (&U)[4], unsigned aU) {
  U[0] = lds_read<(4 * G4 + 0) * FRAG_BYTES>(aU);
  U[1] = lds_read<(4 * G4 + 1) * FRAG_BYTES>(aU);
  U[2] = lds_read<(4 * G4 + 2) * FRAG_BYTES>(aU);
  U[3] = lds_read<(4 * G4 + 3) * FRAG_BYTES>(aU);
}
// F0 = index of the first of the four frags within the chunk's Ud stream: frag f is (contraction block f / NQ, q tile f % NQ)
template <int NQ>
__device__ __forceinline__ void fused_mfma_b(const u32x4 (&U)[4], const bf16x8* Hf, f32x16* acc, const int F0) {
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[(F0 + i) % NQ] = mfma32(as_bf16x8(U[i]), Hf[(F0 + i) / NQ], acc[(F0 + i) % NQ]);
}
// SiLU(g) * p for elements [E0, E0 + N) of an accumulator tile
template <int E0, int N>
__device__ __forceinline__ void silu_mul(const f32x16& g, const f32x16& p, f32x16& h) {
#pragma unroll
  for (int e = E0; e < E0 + N; ++e)
    h[e] = g[e] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g[e] * -1.44269504088896f)) * p[e];  // exp(-g) = 2^(-g log2 e)
}

template <int NQ>
struct FusedProducer {
  static constexpr int KBC = 4, NB = KBC * NQ / 16;
  const char *vcur, *vnext;   // this wave's V frags (gate | up, even | odd ffn tile) of A-step 0 of the current / next chunk
  const char* tbase;          // this wave's Tg frags of A-step 0 (the same for every chunk); Tu lies tu_off further
  const char *ucur;           // Ud frags of the current chunk, offset to this wave's quarter of unit 0
  size_t tu_off, v_chunk, u_chunk;
  unsigned lane16, u_unit;    // u_unit: distance between consecutive Ud units of a chunk
  unsigned m0base;            // LDS byte address of this wave's quarter of ring slot 0
  int pslot, chunks_left;

  __device__ __forceinline__ void init(const char* T, const char* wVg, const char* wVu, const char* wUd, unsigned lds_off,
                                       int r, int nq_total, int qs, int mtile, int c_begin, int c_end, int w, int lane) {
    const size_t KBr = r / 16;
    lane16 = lane * 16;
    v_chunk = 2 * KBr * FRAG_BYTES;                     // a chunk is two ffn tile panels
    vcur = ((w < 2) ? wVg : wVu) + ((size_t)(c_begin * 2 + (w & 1)) * KBr) * FRAG_BYTES;
    chunks_left = c_end - c_begin;
    vnext = chunks_left > 1 ? vcur + v_chunk : vcur;    // past the end the last chunk is re-read (never consumed)
    tbase = T + ((size_t)(mtile * 2) * KBr) * FRAG_BYTES;
    tu_off = KBr * FRAG_BYTES;
    // Ud unit b of a chunk = frags 16 b .. 16 b + 15 of [contraction block][q tile]; this wave copies frags 4w .. 4w+3
    const int f = 4 * w;
    u_chunk = (size_t)KBC * nq_total * FRAG_BYTES;
    ucur = wUd + ((size_t)c_begin * KBC * nq_total + qs * NQ + (f / NQ) * nq_total + (f % NQ)) * FRAG_BYTES;
    u_unit = (unsigned)((16 / NQ) * nq_total * FRAG_BYTES);
    m0base = lds_off + (4 * w) * FRAG_BYTES;
    pslot = 0;
  }
  __device__ __forceinline__ void put(const char* src) {
    const unsigned dst = m0base + pslot * UNIT_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + i * FRAG_BYTES + lane16),
                                       (__attribute__((address_space(3))) void*)(uintptr_t)(dst + i * FRAG_BYTES), 16, 0, 0);
    pslot = (pslot + 1 == NU) ? 0 : pslot + 1;
  }
  // unit K (0: V, 1: Tg, 2: Tu) of A-step a of the current chunk
  template <int K>
  __device__ __forceinline__ void put_a(int a) {
    if (K == 0) put(vcur + (size_t)a * (4 * FRAG_BYTES));
    else put(tbase + (size_t)a * (4 * FRAG_BYTES) + (K == 2 ? tu_off : 0));
  }
  // unit at position E past the end of the current chunk's A-steps: E < NB is Ud unit E of this chunk, otherwise
  // unit (E - NB) % 3 of A-step (E - NB) / 3 of the next chunk
  template <int E>
  __device__ __forceinline__ void put_rel() {
    if (E < NB) put(ucur + (size_t)E * u_unit);
    else {
      constexpr int a = (E - NB) / 3, k = (E - NB) % 3;
      if (k == 0) put(vnext + a * (4 * FRAG_BYTES));
      else put(tbase + a * (4 * FRAG_BYTES) + (k == 2 ? tu_off : 0));
    }
  }
  __device__ __forceinline__ void next_chunk() {
    vcur = vnext;
    if (chunks_left > 1) { --chunks_left; ucur += u_chunk; }
    if (chunks_left > 1) vnext += v_chunk;
  }
};

template <int NQ, int BN>
__global__ __launch_bounds__(256) void k_fused(const char* __restrict__ T, const char* __restrict__ wVg,
                                               const char* __restrict__ wVu, const char* __restrict__ wUd,
                                               float* __restrict__ Tdp, int r, int nq_total, int MT128, int splits,
                                               int QS, int chunks_total, int mx, int sx) {
  static_assert(BN == 64, "a chunk is 64 ffn columns");
  constexpr int NT = 2;                     // ffn tiles per chunk
  constexpr int KBC = 4;                    // contraction blocks of the chunk in the down product
  constexpr int NB = KBC * NQ / 16;         // B-steps (units) per chunk
  static_assert(NB >= 1 && (NQ % 4) == 0, "a B unit is 16 frags = (16 / NQ) contraction blocks x NQ tiles");
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);  // wave index, kept scalar
  // Workgroup -> (row tile, ffn range, q half).  With mx > 0 the 8 XCDs form a (MT128 / mx) x (splits / sx) grid:
  // an XCD owns mx row tiles (their rank-r strips stay resident in its L2) and sx ffn ranges (each factor byte is
  // then fetched by MT128 / mx XCDs instead of all 8).  Otherwise contiguous logical ids per XCD.
  int mt, s, qs;
  if (mx > 0) {
    const int x = blockIdx.x % 8, i = blockIdx.x / 8, ngm = MT128 / mx;
    mt = (x % ngm) * mx + i / (sx * QS);
    s = (x / ngm) * sx + (i / QS) % sx;
    qs = i % QS;
  } else {
    const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
    mt = id / (splits * QS);
    s = (id / QS) % splits;
    qs = id % QS;
  }
  const int NA = r / 64;
  const int c_begin = (int)((long long)chunks_total * s / splits);
  const int c_end = (int)((long long)chunks_total * (s + 1) / splits);
  const int mtile = 4 * mt + w;
  const unsigned lds_off = lds_offset_of(lds);

  FusedProducer<NQ> prod;
  prod.init(T, wVg, wVu, wUd, lds_off, r, nq_total, qs, mtile, c_begin, c_end, w, lane);

  f32x16 acc[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;

  // prologue: A-steps 0 and 1 of the first chunk (PD = 6 units)
  prod.template put_a<0>(0); prod.template put_a<1>(0); prod.template put_a<2>(0);
  prod.template put_a<0>(1); prod.template put_a<1>(1); prod.template put_a<2>(1);
  int cslot = 0;  // ring slot of the next unit to consume
  auto adv = [&](int sl, int n) __attribute__((always_inline)) { sl += n; return sl >= NU ? sl - NU : sl; };
  const unsigned lbase = lds_off + lane * 16;

  for (int c = c_begin; c < c_end; ++c) {
    f32x16 G[NT], P[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) { G[t][e] = 0.f; P[t][e] = 0.f; }

    for (int g = 0; g < NA; ++g) {
      wait_vmcnt<4 * (PD - 3)>();
      lds_barrier();
      const unsigned aV = lbase + cslot * UNIT_BYTES;
      const unsigned aTg = lbase + adv(cslot, 1) * UNIT_BYTES + (4 * w) * FRAG_BYTES;
      const unsigned aTu = lbase + adv(cslot, 2) * UNIT_BYTES + (4 * w) * FRAG_BYTES;
      cslot = adv(cslot, 3);
      // LDS reads run two contraction blocks ahead of the MFMAs that consume them; the three units this step
      // has to issue (two A-steps ahead in the stream) are slipped in between the MFMA groups.
      u32x4 R0[6], R1[6], R2[6], R3[6];
      fused_read_a<0>(R0, aTg, aTu, aV);
      fused_read_a<1>(R1, aTg, aTu, aV);
      lgkm_wait<6>(R0[0], R0[1], R0[2], R0[3], R0[4], R0[5]);
      fused_read_a<2>(R2, aTg, aTu, aV);
      fused_mfma_a(R0, G, P);
      if (g + 2 < NA) prod.template put_a<0>(g + 2);
      else if (g + 2 == NA) prod.template put_rel<0>();
      else prod.template put_rel<3>();
      __builtin_amdgcn_sched_barrier(0);
      lgkm_wait<6>(R1[0], R1[1], R1[2], R1[3], R1[4], R1[5]);
      fused_read_a<3>(R3, aTg, aTu, aV);
      fused_mfma_a(R1, G, P);
      if (g + 2 < NA) prod.template put_a<1>(g + 2);
      else if (g + 2 == NA) prod.template put_rel<1>();
      else prod.template put_rel<4>();
      __builtin_amdgcn_sched_barrier(0);
      lgkm_wait<6>(R2[0], R2[1], R2[2], R2[3], R2[4], R2[5]);
      fused_mfma_a(R2, G, P);
      if (g + 2 < NA) prod.template put_a<2>(g + 2);
      else if (g + 2 == NA) prod.template put_rel<2>();
      else prod.template put_rel<5>();
      __builtin_amdgcn_sched_barrier(0);
      lgkm_wait<0>(R3[0], R3[1], R3[2], R3[3], R3[4], R3[5]);
      fused_mfma_a(R3, G, P);
      __builtin_amdgcn_sched_barrier(0);
    }

    // SiLU(gate) .* up on the accumulators, rounded to bf16: Hf[2 t + u] is the frag of contraction block 2t+u.
    // Tile 0 is needed by the first B-step; tile 1 (when the chunk has more than one B-step) is computed
    // between the MFMA groups of the first B-step.
    bf16x8 Hf[KBC];
    f32x16 h0, h1;
    silu_mul<0, 16>(G[0], P[0], h0);
    Hf[0] = pack_chain(h0, 0);
    Hf[1] = pack_chain(h0, 1);
    if (NB == 1) {
      silu_mul<0, 16>(G[1], P[1], h1);
      Hf[2] = pack_chain(h1, 0);
      Hf[3] = pack_chain(h1, 1);
    }

#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
      wait_vmcnt<4 * (PD - 1)>();
      lds_barrier();
      const unsigned aU = lbase + cslot * UNIT_BYTES;
      cslot = adv(cslot, 1);
      u32x4 U0[4], U1[4], U2[4], U3[4];
      fused_read_b<0>(U0, aU);
      fused_read_b<1>(U1, aU);
      lgkm_wait<4>(U0[0], U0[1], U0[2], U0[3]);
      fused_read_b<2>(U2, aU);
      fused_mfma_b<NQ>(U0, Hf, acc, 16 * blk + 0);
      if (blk == 0) prod.template put_rel<6>();
      if (blk == 1) prod.template put_rel<7>();
      if (blk == 2) prod.template put_rel<8>();
      if (blk == 3) prod.template put_rel<9>();
      if (NB > 1 && blk == 0) silu_mul<0, 4>(G[1], P[1], h1);
      __builtin_amdgcn_sched_barrier(0);
      lgkm_wait<4>(U1[0], U1[1], U1[2], U1[3]);
      fused_read_b<3>(U3, aU);
      fused_mfma_b<NQ>(U1, Hf, acc, 16 * blk + 4);
      if (NB > 1 && blk == 0) silu_mul<4, 4>(G[1], P[1], h1);
      __builtin_amdgcn_sched_barrier(0);
      lgkm_wait<4>(U2[0], U2[1], U2[2], U2[3]);
      fused_mfma_b<NQ>(U2, Hf, acc, 16 * blk + 8);
      if (NB > 1 && blk == 0) silu_mul<8, 4>(G[1], P[1], h1);
      __builtin_amdgcn_sched_barrier(0);
      lgkm_wait<0>(U3[0], U3[1], U3[2], U3[3]);
      fused_mfma_b<NQ>(U3, Hf, acc, 16 * blk + 12);
      if (NB > 1 && blk == 0) {
        silu_mul<12, 4>(G[1], P[1], h1);
        Hf[2] = pack_chain(h1, 0);
        Hf[3] = pack_chain(h1, 1);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    prod.next_chunk();
  }
  wait_vmcnt<0>();

  // partial Td^T of this ffn range: [split][row tile][q tile][register group of 4][lane][4], fp32
  const int MT32 = 4 * MT128;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    f32x4* dst = reinterpret_cast<f32x4*>(Tdp + (((size_t)s * MT32 + mtile) * nq_total + qs * NQ + q) * 1024) + lane;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 v = {acc[q][4 * g], acc[q][4 * g + 1], acc[q][4 * g + 2], acc[q][4 * g + 3]};
      dst[g * 64] = v;
    }
  }
}

// Td frags = fixed-order sum of the ffn-range partials, rounded to bf16.  One thread per (row tile, q tile,
// contraction block t, lane): registers 8t..8t+7 of the accumulator tile are the chain-order frag.
// BATCH: eight ranges' worth of loads in flight at a time, for many ranges over few rows (few threads, where one load
// per addition makes the kernel a chain of memory round trips); otherwise the plain loop, which is what a grid that is
// bound by HBM wants.  The additions are in range order either way.
template <bool BATCH>
__global__ __launch_bounds__(256) void k_reduce(const float* __restrict__ Tdp, char* __restrict__ Td, int splits, int MT32,
                                                int nq_total) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long total = (long long)MT32 * nq_total * 2 * 64;
  if (idx >= total) return;
  const int lane = (int)(idx % 64);
  const int t = (int)((idx / 64) % 2);
  const long long tile = idx / 128;  // mtile * nq_total + qt
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const size_t split_stride = (size_t)MT32 * nq_total * 1024;
  if (BATCH) {
    for (int sp0 = 0; sp0 < splits; sp0 += 8) {
      f32x4 a[8], b[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int sp = sp0 + j < splits ? sp0 + j : splits - 1;
        const f32x4* src = reinterpret_cast<const f32x4*>(Tdp + sp * split_stride + (size_t)tile * 1024) + 2 * t * 64 + lane;
        a[j] = src[0];
        b[j] = src[64];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (sp0 + j < splits) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] += a[j][e];
            v[4 + e] += b[j][e];
          }
        }
    }
  } else {
    for (int sp = 0; sp < splits; ++sp) {
      const f32x4* src = reinterpret_cast<const f32x4*>(Tdp + sp * split_stride + (size_t)tile * 1024) + 2 * t * 64 + lane;
      const f32x4 a = src[0], b = src[64];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[e] += a[e];
        v[4 + e] += b[e];
      }
    }
  }
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
  const long long mtile = tile / nq_total, qt = tile % nq_total;
  const int KBq = nq_total * 2;
  *reinterpret_cast<bf16x8*>(Td + (((size_t)mtile * KBq + 2 * qt + t) * 64 + lane) * 16) = o;
}

// ------------------------------------------------------------------------------------------------
// S5: Y[m, c] = sum_q Td[m, q] Vd[q, c]   (second phase of the down-projection XUV kernel, Alg. 2)
// workgroup tile 128 (m) x 128 (c); output in the standard row-major layout.  The contraction is only
// r_down long, so a workgroup lives for a few steps: the ring is kept small (4 slots, 64 KiB) so that two
// workgroups share a CU and one's pipeline fill overlaps the other's MFMAs.
// ------------------------------------------------------------------------------------------------
constexpr int NU5 = 4, PD5 = 2;
template <int J>
__device__ __forceinline__ void s5_read(u32x4 (&R)[4], unsigned aP, unsigned aQ) {
  R[0] = lds_read<(0 * 4 + J) * FRAG_BYTES>(aP);
  R[1] = lds_read<(1 * 4 + J) * FRAG_BYTES>(aP);
  R[2] = lds_read<(0 * 4 + J) * FRAG_BYTES>(aQ);
  R[3] = lds_read<(1 * 4 + J) * FRAG_BYTES>(aQ);
}

__global__ __launch_bounds__(256) void k_s5(const char* __restrict__ Td, const char* __restrict__ wVd, uint16_t* __restrict__ Y,
                                            int M, int d, int rd, int CT) {
  __shared__ __attribute__((aligned(1024))) char lds[NU5 * UNIT_BYTES];
  const int lane = threadIdx.x % 64;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);  // wave index, kept scalar
  const int wp = w / 2, wq = w % 2;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int mt = id / CT, ct = id % CT;
  const int KBq = rd / 16, nks = rd / 64;
  const unsigned lds_off = lds_offset_of(lds);
  const unsigned lane16 = lane * 16;
  const char* srcP = Td + (size_t)(4 * mt + w) * KBq * FRAG_BYTES;
  const char* srcQ = wVd + (size_t)(4 * ct + w) * KBq * FRAG_BYTES;
  const unsigned m0base = lds_off + (4 * w) * FRAG_BYTES;
  int pslot = 0, pks = 0;
  auto put_pair = [&]() __attribute__((always_inline)) {
    const int ks = pks < nks ? pks : nks - 1;
    const unsigned dP = m0base + pslot * UNIT_BYTES, dQ = dP + UNIT_BYTES;   // NU5 is even: a pair never wraps
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcP + (size_t)ks * 4096 + i * 1024 + lane16),
                                       (__attribute__((address_space(3))) void*)(uintptr_t)(dP + i * FRAG_BYTES), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(srcQ + (size_t)ks * 4096 + i * 1024 + lane16),
                                       (__attribute__((address_space(3))) void*)(uintptr_t)(dQ + i * FRAG_BYTES), 16, 0, 0);
    pslot = (pslot + 2 == NU5) ? 0 : pslot + 2;
    ++pks;
  };
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
  const unsigned pbase = lds_off + lane16 + (2 * wp) * 4 * FRAG_BYTES;
  const unsigned qbase = lds_off + lane16 + (2 * wq) * 4 * FRAG_BYTES + UNIT_BYTES;
  put_pair();   // PD5 = 2 units
  int cslot = 0;
  for (int ks = 0; ks < nks; ++ks) {
    wait_vmcnt<4 * (PD5 - 2)>();
    lds_barrier();
    const unsigned aP = pbase + cslot * UNIT_BYTES, aQ = qbase + cslot * UNIT_BYTES;
    cslot = (cslot + 2 == NU5) ? 0 : cslot + 2;
    u32x4 R0[4], R1[4], R2[4], R3[4];
    s5_read<0>(R0, aP, aQ);
    s5_read<1>(R1, aP, aQ);
    lgkm_wait<4>(R0[0], R0[1], R0[2], R0[3]);
    s5_read<2>(R2, aP, aQ);
    mfma_2x2(R0, acc);
    put_pair();
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<4>(R1[0], R1[1], R1[2], R1[3]);
    s5_read<3>(R3, aP, aQ);
    mfma_2x2(R1, acc);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<4>(R2[0], R2[1], R2[2], R2[3]);
    mfma_2x2(R2, acc);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<0>(R3[0], R3[1], R3[2], R3[3]);
    mfma_2x2(R3, acc);
    __builtin_amdgcn_sched_barrier(0);
  }
  wait_vmcnt<0>();
  // Epilogue through LDS (the ring is free now): a lane holds one column of sixteen rows, which as direct stores is
  // two bytes per lane and 64 store instructions per wave.  The tile is laid out row-major in LDS as bf16 (rows 272
  // bytes apart: the 16 bytes of padding spread the rows over the banks), then every lane moves 16 bytes at a time:
  // sixteen lanes cover the 256 contiguous bytes of a row of Y.
  constexpr int YS = 128 * 2 + 16;
  static_assert(128 * YS <= NU5 * UNIT_BYTES, "the tile fits the ring");
  __syncthreads();   // every wave has read its last frags
  const int il = lane % 32, h = lane / 32;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int cl = 64 * wq + 32 * b + il;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int ml = 64 * wp + 32 * a + 8 * (e / 4) + 4 * h + (e % 4);
        *reinterpret_cast<__bf16*>(lds + ml * YS + 2 * cl) = (__bf16)acc[a][b][e];
      }
    }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int chunk = i * 256 + (int)threadIdx.x, row = chunk / 16, cc = chunk % 16;
    const int m = 128 * mt + row;
    if (m < M)
      *reinterpret_cast<u32x4*>(Y + (size_t)m * d + 128 * ct + 8 * cc) = *reinterpret_cast<const u32x4*>(lds + row * YS + 16 * cc);
  }
}

// ------------------------------------------------------------------------------------------------
template <int NQ, int BN>
static int launch_fused(const Ctx* c, int MT128, int splits, int QS, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int chunks = (int)(p.ffn / BN);
  // XCD grid: the most row tiles per XCD whose strips (128 x 2r bf16 each) fit in half of its 4 MiB L2
  int mx = 0, sx = 0;
  const long long strip = 128LL * 2 * p.r * 2;
  for (int m = 8; m >= 1; m /= 2) {
    if (MT128 % m || m * strip > (2LL << 20)) continue;
    const int ngm = MT128 / m;
    if (ngm > 8 || 8 % ngm) continue;
    const int ngs = 8 / ngm;
    if (splits % ngs) continue;
    mx = m; sx = splits / ngs;
    break;
  }
  hipLaunchKernelGGL((k_fused<NQ, BN>), dim3(MT128 * splits * QS), dim3(256), 0, st, ws + p.off_T, ws + p.off_wVg,
                     ws + p.off_wVu, ws + p.off_wUd, reinterpret_cast<float*>(ws + p.off_Tdp), (int)p.r, (int)(p.rd / 32),
                     MT128, splits, QS, chunks, mx, sx);
  return (int)hipGetLastError();
}

int launch_reduce(const Ctx* c, const float* part, char* out, int splits, int MT32, int nq, hipStream_t st) {
  (void)c;
  const long long threads = (long long)MT32 * nq * 2 * 64;
  const dim3 grid((unsigned)((threads + 255) / 256));
  if (splits > 8) hipLaunchKernelGGL(k_reduce<true>, grid, dim3(256), 0, st, part, out, splits, MT32, nq);
  else hipLaunchKernelGGL(k_reduce<false>, grid, dim3(256), 0, st, part, out, splits, MT32, nq);
  return (int)hipGetLastError();
}

// First stage T = X [Ug|Uu] (ncols = 2 r_strip rank columns in two strips): the planner's choice between k_in
// (256 x 256 tiles) and k_s1 (128 x 128), either with its contraction cut into ranges (+ k_reduce) when there are few
// tiles.
static int first_stage(const Ctx* c, const void* X, int64_t M, int64_t r_strip, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const StageChoice ch = choose_first(M, p.d, 2 * r_strip, linear_on_small_tiles(p), &c->force);
  if (ch.kernel == FIRST_IN) return launch_in(c, X, M, 2 * r_strip, r_strip, ch.ranges, st);
  const int MT128 = (int)((M + 127) / 128), PT = (int)(2 * r_strip / 128);
  const int S = ch.ranges;
  if (S > 1 && (size_t)S * MT128 * 128 * 2 * r_strip * 4 > p.part_bytes) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(k_s1, dim3(MT128 * PT * S), dim3(256), 0, st, (const uint16_t*)X, (int)M, (int)p.d, ws + p.off_wU,
                     (int)r_strip, ws + p.off_T, PT, S, reinterpret_cast<float*>(ws + p.off_Tdp), MT128);
  int e = (int)hipGetLastError();
  if (e || S == 1) return e;
  const int MT32 = 4 * MT128, nq = (int)(2 * r_strip / 32);
  return launch_reduce(c, reinterpret_cast<const float*>(ws + p.off_Tdp), ws + p.off_T, S, MT32, nq, st);
}

// Everything after k_s1 when the gated activation is staged through HBM (gemm.hip).
static int staged_tail(const Ctx* c, int64_t M, void* Y, int ps, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int MT128 = (int)((M + 127) / 128), MT256 = (int)((M + 255) / 256);
  const int nq_total = (int)(p.rd / 32);
  int e;
  prof_mark(c, ps, 1, 0, st);
  e = launch_gate_up(c, MT256, st);
  prof_mark(c, ps, 1, 1, st);
  if (e) return e;
  const int splits = choose_down(M, p.rd, p.ffn, &c->force).ranges;
  if ((size_t)splits * MT256 * 256 * p.rd * 4 > p.part_bytes) return (int)hipErrorInvalidValue;
  prof_mark(c, ps, 2, 0, st);
  e = launch_down1(c, MT256, splits, st);
  prof_mark(c, ps, 2, 1, st);
  if (e) return e;
  const int MT32 = 8 * MT256;
  prof_mark(c, ps, 3, 0, st);
  e = launch_reduce(c, reinterpret_cast<const float*>(ws + p.off_Tdp), ws + p.off_Td, splits, MT32, nq_total, st);
  prof_mark(c, ps, 3, 1, st);
  if (e) return e;
  prof_mark(c, ps, 4, 0, st);
  if (choose_out(M, p.d, p.rd, false, &c->force).kernel == OUT_256) {
    e = launch_out(c, M, Y, MT256, st);
  } else {
    const int CT = (int)(p.d / 128);
    hipLaunchKernelGGL(k_s5, dim3(MT128 * CT), dim3(256), 0, st, ws + p.off_Td, ws + p.off_wVd, (uint16_t*)Y, (int)M,
                       (int)p.d, (int)p.rd, CT);
    e = (int)hipGetLastError();
  }
  prof_mark(c, ps, 4, 1, st);
  return e;
}

// Single factored layer O = (X U) V  (paper Sec. 4.2.1, the XUV product): k_s1 with the rank split in two equal
// "strips" lays T out as [32-row tile][r / 16] chain-order frags, which is what the output kernels read.
int bf16_linear_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int MT128 = (int)((M + 127) / 128), MT256 = (int)((M + 255) / 256);
  const bool small = linear_on_small_tiles(p);
  const bool out256 = choose_out(M, p.ffn, p.r, small, &c->force).kernel == OUT_256;
  const char* const names[2] = {choose_first(M, p.d, p.r, small, &c->force).kernel == FIRST_IN ? "k_in" : "k_s1",
                                out256 ? "k_out" : "k_s5"};
  const int ps = prof_open_forward(c, 2, names);
  int e;
  prof_mark(c, ps, 0, 0, st);
  e = first_stage(c, X, M, p.r / 2, st);
  prof_mark(c, ps, 0, 1, st);
  if (e) return e;
  prof_mark(c, ps, 1, 0, st);
  if (out256) {
    e = launch_out_generic(c, ws + p.off_T, ws + p.off_wVd, M, Y, MT256, p.ffn, p.r, st);
  } else {
    const int CT = (int)(p.ffn / 128);
    hipLaunchKernelGGL(k_s5, dim3(MT128 * CT), dim3(256), 0, st, ws + p.off_T, ws + p.off_wVd, (uint16_t*)Y, (int)M,
                       (int)p.ffn, (int)p.r, CT);
    e = (int)hipGetLastError();
  }
  prof_mark(c, ps, 1, 1, st);
  return e;
}

int bf16_tiled_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int MT128 = (int)((M + 127) / 128);
  int e;
  const char* const s1name = choose_first(M, p.d, 2 * p.r, false, &c->force).kernel == FIRST_IN ? "k_in" : "k_s1";
  const char* const names_fused[4] = {s1name, "k_fused", "k_reduce", "k_s5"};
  const char* const names_staged[5] = {s1name, "k_gate_up", "k_down1", "k_reduce", choose_out(M, p.d, p.rd, false, &c->force).kernel == OUT_256 ? "k_out" : "k_s5"};
  const bool staged = staged_supported(p.rd, p.ffn) && !(p.flags & SVDMLP_FLAG_TILED_FUSED);
  const int ps = staged ? prof_open_forward(c, 5, names_staged) : prof_open_forward(c, 4, names_fused);
  prof_mark(c, ps, 0, 0, st);
  e = first_stage(c, X, M, p.r, st);
  prof_mark(c, ps, 0, 1, st);
  if (e) return e;

  const int nq_total = (int)(p.rd / 32);
  if (staged) return staged_tail(c, M, Y, ps, st);
  const int NQ = nq_total > 16 ? 16 : nq_total;
  const int QS = nq_total / NQ;
  const int splits = tiled_splits(MT128, p.ffn / 64);
  prof_mark(c, ps, 1, 0, st);
  switch (NQ) {
    case 16: e = launch_fused<16, 64>(c, MT128, splits, QS, st); break;
    case 8: e = launch_fused<8, 64>(c, MT128, splits, QS, st); break;
    case 4: e = launch_fused<4, 64>(c, MT128, splits, QS, st); break;
    default: return (int)hipErrorInvalidValue;
  }
  prof_mark(c, ps, 1, 1, st);
  if (e) return e;

  const int MT32 = 4 * MT128;
  prof_mark(c, ps, 2, 0, st);
  e = launch_reduce(c, reinterpret_cast<const float*>(ws + p.off_Tdp), ws + p.off_Td, splits, MT32, nq_total, st);
  prof_mark(c, ps, 2, 1, st);
  if (e) return e;

  const int CT = (int)(p.d / 128);
  prof_mark(c, ps, 3, 0, st);
  hipLaunchKernelGGL(k_s5, dim3(MT128 * CT), dim3(256), 0, st, ws + p.off_Td, ws + p.off_wVd, (uint16_t*)Y, (int)M, (int)p.d,
                     (int)p.rd, CT);
  prof_mark(c, ps, 3, 1, st);
  return (int)hipGetLastError();
}

}  // namespace svdmlp
