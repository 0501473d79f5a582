// bf16 MFMA-tiled (prefill) path of the factored gated MLP (paper Alg. 2 / Alg. 3), gfx950.
//
//   k_s1      T^T  = [Ug|Uu]^T X^T            rank-r strips of gate and up, written as chain-order frags
//   k_fused   H^T  = SiLU(Vg^T Tg^T) .* (Vu^T Tu^T)   per ffn chunk, kept in registers, immediately
//             Td^T += Ud^T H^T                 contracted with the down factor; fp32 partial per ffn range
//   k_reduce  Td   = sum of the partials, rounded to bf16 frags (fixed order: deterministic)
//   k_s5      Y    = Td Vd
//
// All four are the same machine: operands arrive as 1 KiB frags (common.h) through a ring of 16 KiB
// LDS slots filled by asynchronous global->LDS copies, waves read frags back with ds_read_b128 and feed
// v_mfma_f32_32x32x16_bf16.  The paper's "caching" of the rank-r strip (Sec. 4.2.1) becomes: the strip
// T is produced once by k_s1 and re-read from L2 by the 128-row tile that owns it; the ffn-wide
// activation H (which the paper writes to HBM in Alg. 3) never leaves the register file.
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
// S1: T^T[p, m] = sum_k U^T[p, k] X^T[k, m]   (paper Alg. 3, first inner loop nest)
// workgroup tile 128 (p) x 128 (m); wave (wp, wq) owns 64 x 64.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_s1(const uint16_t* __restrict__ X, int M, int d, const char* __restrict__ wU,
                                            int r, char* __restrict__ T, int PT) {
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
  const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
  const int wp = w / 2, wq = w % 2;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int mt = id / PT, pt = id % PT;
  const int KBd = d / 16, KBr = r / 16;
  const int nks = d / 64;

  // per-wave sources
  const char* srcP = wU + ((size_t)(4 * pt + w) * KBd * 64 + lane) * 16;  // + ks * 4 KiB + i * 1 KiB
  const uint16_t* srcX[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rg = 2 * w + i / 2, kh = i % 2;
    int row = mt * 128 + 16 * rg + lane / 4;
    row = row < M ? row : M - 1;  // rows beyond M only feed output rows that are never used
    const int piece = (lane % 4) ^ ((lane >> 4) & 3);
    srcX[i] = X + (size_t)row * d + 32 * kh + 8 * piece;  // + ks * 64
  }
  auto issue = [&](int u) __attribute__((always_inline)) {
    int ks = u >> 1;
    ks = ks < nks ? ks : nks - 1;
    char* dst = lds + (u % NU) * UNIT_BYTES + (4 * w) * FRAG_BYTES;
    if ((u & 1) == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) dma16(srcP + (size_t)ks * 4096 + i * 1024, dst + i * FRAG_BYTES);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) dma16(srcX[i] + ks * 64, dst + i * FRAG_BYTES);
    }
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // X frag addressing inside an X unit (see issue(): 16 rows x 64 B per wave-load, 16 B pieces XOR-swizzled
  // with bits 2..3 of the row so the 16 lanes of a quarter-wave hit 64 distinct banks)
  const int il = lane % 32, h = lane / 32, rho = il % 16;
  int xoff[2][4];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int rg = 2 * (2 * wq + b) + il / 16, kh = j / 2, piece = 2 * (j % 2) + h;
      xoff[b][j] = (rg * 2 + kh) * FRAG_BYTES + rho * 64 + ((piece ^ ((rho >> 2) & 3)) * 16);
    }

#pragma unroll
  for (int u = 0; u < PD; ++u) issue(u);
  for (int ks = 0; ks < nks; ++ks) {
    wait_vmcnt<4 * (PD - 2)>();
    lds_barrier();
    issue(2 * ks + PD);
    issue(2 * ks + PD + 1);
    const int sP = (2 * ks) % NU, sX = (2 * ks + 1) % NU;
    const char* xs = lds + sX * UNIT_BYTES;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x8 a0 = *lds_frag(lds, sP, (2 * wp + 0) * 4 + j, lane);
      bf16x8 a1 = *lds_frag(lds, sP, (2 * wp + 1) * 4 + j, lane);
      bf16x8 b0 = *reinterpret_cast<const bf16x8*>(xs + xoff[0][j]);
      bf16x8 b1 = *reinterpret_cast<const bf16x8*>(xs + xoff[1][j]);
      acc[0][0] = mfma32(a0, b0, acc[0][0]);
      acc[0][1] = mfma32(a0, b1, acc[0][1]);
      acc[1][0] = mfma32(a1, b0, acc[1][0]);
      acc[1][1] = mfma32(a1, b1, acc[1][1]);
    }
  }
  wait_vmcnt<0>();
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
//   per chunk of BN ffn columns:
//     A-steps (r / 64 of them): G^T, P^T += V^T frags (LDS, shared) x T frags (LDS, wave-private)
//     H = SiLU(G) .* P  -> bf16 chain frags in registers
//     B-steps: Td^T[q, m] += Ud^T frags (LDS, shared) x H frags (registers)
// ------------------------------------------------------------------------------------------------
// Producer side of the fused kernel's unit stream: per chunk, r/64 A-steps of (BN/64 V units, the Tg unit,
// the Tu unit) followed by the chunk's Ud units.  All state is wave-uniform.
template <int NQ, int BN>
struct FusedProducer {
  static constexpr int NV = BN / 64, NT = BN / 32, KBC = BN / 16, NB = KBC * NQ / 16;
  const char *T, *wVg, *wVu, *wUd;
  char* lds;
  int KBr, NA, nq_total, qs, mtile, c_end, w;
  size_t lane16;
  int pc, pg, pk, pslot;
  __device__ __forceinline__ void init(const char* T_, const char* wVg_, const char* wVu_, const char* wUd_, char* lds_,
                                       int r, int nq_total_, int qs_, int mtile_, int c_begin, int c_end_, int w_, int lane) {
    T = T_; wVg = wVg_; wVu = wVu_; wUd = wUd_; lds = lds_;
    KBr = r / 16; NA = r / 64; nq_total = nq_total_; qs = qs_; mtile = mtile_; c_end = c_end_; w = w_;
    lane16 = (size_t)lane * 16;
    pc = c_begin; pg = 0; pk = 0; pslot = 0;
  }
  __device__ __forceinline__ void issue_next() {
    const int c = pc < c_end ? pc : c_end - 1;  // past the end: keep re-reading the last chunk (never consumed)
    const char* src;
    if (pg < NA) {
      if (pk < NV) {
        const char* mat = (w < 2) ? wVg : wVu;
        const int nt = c * NT + 2 * pk + (w & 1);
        src = mat + ((size_t)nt * KBr + 4 * pg) * FRAG_BYTES;
      } else {
        src = T + ((size_t)(mtile * 2 + (pk - NV)) * KBr + 4 * pg) * FRAG_BYTES;
      }
      if (++pk == NV + 2) { pk = 0; ++pg; }
    } else {
      const int f = 16 * pk + 4 * w;
      const int kbl = f / NQ, qtl = f % NQ;
      src = wUd + ((size_t)(c * KBC + kbl) * nq_total + qs * NQ + qtl) * FRAG_BYTES;
      if (++pk == NB) { pk = 0; pg = 0; ++pc; }
    }
    char* dst = lds + pslot * UNIT_BYTES + (4 * w) * FRAG_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(src + i * FRAG_BYTES + lane16, dst + i * FRAG_BYTES);
    pslot = (pslot + 1 == NU) ? 0 : pslot + 1;
  }
};

template <int NQ, int BN>
__global__ __launch_bounds__(256) void k_fused(const char* __restrict__ T, const char* __restrict__ wVg,
                                               const char* __restrict__ wVu, const char* __restrict__ wUd,
                                               float* __restrict__ Tdp, int r, int nq_total, int MT128, int splits,
                                               int QS, int chunks_total) {
  constexpr int NV = BN / 64;               // V units per A-step
  constexpr int NT = BN / 32;               // ffn tiles per chunk
  constexpr int KBC = BN / 16;              // contraction blocks of the chunk in the down product
  constexpr int NB = KBC * NQ / 16;         // B-steps (units) per chunk
  static_assert(NB >= 1 && (NQ % 4) == 0, "a B unit is 16 frags = (16 / NQ) contraction blocks x NQ tiles");
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
  const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int mt = id / (splits * QS);
  const int s = (id / QS) % splits, qs = id % QS;
  const int KBr = r / 16, NA = r / 64;
  const int c_begin = (int)((long long)chunks_total * s / splits);
  const int c_end = (int)((long long)chunks_total * (s + 1) / splits);
  const int mtile = 4 * mt + w;

  // ---- producer cursor over the unit stream (wave-uniform) ----
  FusedProducer<NQ, BN> prod;
  prod.init(T, wVg, wVu, wUd, lds, r, nq_total, qs, mtile, c_begin, c_end, w, lane);

  f32x16 acc[NQ];
#pragma unroll
  for (int q = 0; q < NQ; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;

#pragma unroll
  for (int u = 0; u < PD; ++u) prod.issue_next();
  int cslot = 0;  // ring slot of the next unit to consume
  auto adv = [&](int sl, int n) __attribute__((always_inline)) { sl += n; return sl >= NU ? sl - NU : sl; };

  for (int c = c_begin; c < c_end; ++c) {
    f32x16 G[NT], P[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) { G[t][e] = 0.f; P[t][e] = 0.f; }

    for (int g = 0; g < NA; ++g) {
      wait_vmcnt<4 * (PD - (NV + 2))>();
      lds_barrier();
#pragma unroll
      for (int u = 0; u < NV + 2; ++u) prod.issue_next();
      const int sTg = adv(cslot, NV), sTu = adv(cslot, NV + 1);
      // All LDS reads of the step are written before its MFMAs and the scheduler is then told to interleave
      // them (one contraction block of reads ahead), so that ds_read latency hides under the matrix cores.
      bf16x8 tg[4], tu[4], vf[NV][4][4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        tg[j] = *lds_frag(lds, sTg, 4 * w + j, lane);
        tu[j] = *lds_frag(lds, sTu, 4 * w + j, lane);
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
          for (int k = 0; k < 4; ++k) vf[v][k][j] = *lds_frag(lds, adv(cslot, v), k * 4 + j, lane);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          G[2 * v] = mfma32(vf[v][0][j], tg[j], G[2 * v]);
          G[2 * v + 1] = mfma32(vf[v][1][j], tg[j], G[2 * v + 1]);
          P[2 * v] = mfma32(vf[v][2][j], tu[j], P[2 * v]);
          P[2 * v + 1] = mfma32(vf[v][3][j], tu[j], P[2 * v + 1]);
        }
      // schedule: reads of block 0; then per MFMA of blocks 0..2 one or two reads of the next block; block 3 bare
      __builtin_amdgcn_sched_group_barrier(0x100, 2 + 4 * NV, 0);
#pragma unroll
      for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int m = 0; m < 4 * NV; ++m) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (m < 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      __builtin_amdgcn_sched_group_barrier(0x008, 4 * NV, 0);
      cslot = adv(cslot, NV + 2);
    }

    // SiLU(gate) .* up on the accumulators, rounded to bf16: Hf[2 t + u] is the frag of contraction block 2t+u
    bf16x8 Hf[KBC];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      f32x16 hv;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float gv = G[t][e];
        hv[e] = gv * __builtin_amdgcn_rcpf(1.0f + __expf(-gv)) * P[t][e];
      }
      Hf[2 * t] = pack_chain(hv, 0);
      Hf[2 * t + 1] = pack_chain(hv, 1);
    }

#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
      wait_vmcnt<4 * (PD - 1)>();
      lds_barrier();
      prod.issue_next();
      bf16x8 uf[16];
#pragma unroll
      for (int f = 0; f < 16; ++f) uf[f] = *lds_frag(lds, cslot, f, lane);
#pragma unroll
      for (int f = 0; f < 16; ++f) {
        const int kbl = (16 * blk + f) / NQ, qtl = (16 * blk + f) % NQ;
        acc[qtl] = mfma32(uf[f], Hf[kbl], acc[qtl]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int f = 0; f < 12; ++f) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      cslot = adv(cslot, 1);
    }
  }
  wait_vmcnt<0>();

  // partial Td^T of this ffn range: [split][row tile][q tile][register][lane], fp32
  const int MT32 = 4 * MT128;
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    float* dst = Tdp + ((((size_t)s * MT32 + mtile) * nq_total + qs * NQ + q) * 16) * 64 + lane;
#pragma unroll
    for (int e = 0; e < 16; ++e) dst[e * 64] = acc[q][e];
  }
}

// Td frags = fixed-order sum of the ffn-range partials, rounded to bf16.  One thread per (row tile, q tile,
// contraction block t, lane): registers 8t..8t+7 of the accumulator tile are the chain-order frag.
__global__ __launch_bounds__(256) void k_reduce(const float* __restrict__ Tdp, char* __restrict__ Td, int splits, int MT32,
                                                int nq_total) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long total = (long long)MT32 * nq_total * 2 * 64;
  if (idx >= total) return;
  const int lane = (int)(idx % 64);
  const int t = (int)((idx / 64) % 2);
  const long long tile = idx / 128;  // mtile * nq_total + qt
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const size_t split_stride = (size_t)MT32 * nq_total * 16 * 64;
  for (int sp = 0; sp < splits; ++sp) {
    const float* src = Tdp + sp * split_stride + ((size_t)tile * 16 + 8 * t) * 64 + lane;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] += src[e * 64];
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
// workgroup tile 128 (m) x 128 (c); output in the standard row-major layout.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_s5(const char* __restrict__ Td, const char* __restrict__ wVd, uint16_t* __restrict__ Y,
                                            int M, int d, int rd, int CT) {
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
  const int lane = threadIdx.x % 64, w = threadIdx.x / 64;
  const int wp = w / 2, wq = w % 2;
  const int id = xcd_contiguous_id(blockIdx.x, gridDim.x);
  const int mt = id / CT, ct = id % CT;
  const int KBq = rd / 16, nks = rd / 64;
  const char* srcP = Td + ((size_t)(4 * mt + w) * KBq * 64 + lane) * 16;
  const char* srcQ = wVd + ((size_t)(4 * ct + w) * KBq * 64 + lane) * 16;
  auto issue = [&](int u) __attribute__((always_inline)) {
    int ks = u >> 1;
    ks = ks < nks ? ks : nks - 1;
    char* dst = lds + (u % NU) * UNIT_BYTES + (4 * w) * FRAG_BYTES;
    const char* src = ((u & 1) == 0 ? srcP : srcQ) + (size_t)ks * 4096;
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(src + i * 1024, dst + i * FRAG_BYTES);
  };
  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;
#pragma unroll
  for (int u = 0; u < PD; ++u) issue(u);
  for (int ks = 0; ks < nks; ++ks) {
    wait_vmcnt<4 * (PD - 2)>();
    lds_barrier();
    issue(2 * ks + PD);
    issue(2 * ks + PD + 1);
    const int sP = (2 * ks) % NU, sQ = (2 * ks + 1) % NU;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x8 a0 = *lds_frag(lds, sP, (2 * wp + 0) * 4 + j, lane);
      bf16x8 a1 = *lds_frag(lds, sP, (2 * wp + 1) * 4 + j, lane);
      bf16x8 b0 = *lds_frag(lds, sQ, (2 * wq + 0) * 4 + j, lane);
      bf16x8 b1 = *lds_frag(lds, sQ, (2 * wq + 1) * 4 + j, lane);
      acc[0][0] = mfma32(a0, b0, acc[0][0]);
      acc[0][1] = mfma32(a0, b1, acc[0][1]);
      acc[1][0] = mfma32(a1, b0, acc[1][0]);
      acc[1][1] = mfma32(a1, b1, acc[1][1]);
    }
  }
  wait_vmcnt<0>();
  const int il = lane % 32, h = lane / 32;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int c = 128 * ct + 64 * wq + 32 * b + il;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = 128 * mt + 64 * wp + 32 * a + 8 * (e / 4) + 4 * h + (e % 4);
        if (m < M) {
          __bf16 v = (__bf16)acc[a][b][e];
          Y[(size_t)m * d + c] = *reinterpret_cast<uint16_t*>(&v);
        }
      }
    }
}

// ------------------------------------------------------------------------------------------------
template <int NQ, int BN>
static int launch_fused(const Ctx* c, int MT128, int splits, int QS, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int chunks = (int)(p.ffn / BN);
  hipLaunchKernelGGL((k_fused<NQ, BN>), dim3(MT128 * splits * QS), dim3(256), 0, st, ws + p.off_T, ws + p.off_wVg,
                     ws + p.off_wVu, ws + p.off_wUd, reinterpret_cast<float*>(ws + p.off_Tdp), (int)p.r, (int)(p.rd / 32),
                     MT128, splits, QS, chunks);
  return (int)hipGetLastError();
}

int bf16_tiled_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st) {
  const Plan& p = c->plan;
  char* ws = c->ws;
  const int MT128 = (int)((M + 127) / 128);
  const int PT = (int)(2 * p.r / 128);
  int e;
  static const char* const names[4] = {"k_s1", "k_fused", "k_reduce", "k_s5"};
  const int ps = prof_open_forward(c, 4, names);
  prof_mark(c, ps, 0, 0, st);
  hipLaunchKernelGGL(k_s1, dim3(MT128 * PT), dim3(256), 0, st, (const uint16_t*)X, (int)M, (int)p.d, ws + p.off_wU, (int)p.r,
                     ws + p.off_T, PT);
  prof_mark(c, ps, 0, 1, st);
  if ((e = (int)hipGetLastError())) return e;

  const int nq_total = (int)(p.rd / 32);
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
  const long long threads = (long long)MT32 * nq_total * 2 * 64;
  prof_mark(c, ps, 2, 0, st);
  hipLaunchKernelGGL(k_reduce, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<const float*>(ws + p.off_Tdp), ws + p.off_Td, splits, MT32, nq_total);
  prof_mark(c, ps, 2, 1, st);
  if ((e = (int)hipGetLastError())) return e;

  const int CT = (int)(p.d / 128);
  prof_mark(c, ps, 3, 0, st);
  hipLaunchKernelGGL(k_s5, dim3(MT128 * CT), dim3(256), 0, st, ws + p.off_Td, ws + p.off_wVd, (uint16_t*)Y, (int)M, (int)p.d,
                     (int)p.rd, CT);
  prof_mark(c, ps, 3, 1, st);
  return (int)hipGetLastError();
}

}  // namespace svdmlp
