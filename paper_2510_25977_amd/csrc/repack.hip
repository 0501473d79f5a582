// One-time re-tiling of the factor matrices into matrix-core fragments (see common.h).
// The factors are invariant at inference time (paper Sec. 2.1: SVD is done offline), so the cost of
// this pass is paid once per context, not per forward.
#include "common.h"

namespace svdmlp {

// W is row-major [K, N]; the product it takes part in is act[M,K] * W, so n indexes frag rows and k
// is the contraction index.  The frags cover [Kp, Np] >= [K, N] (ranks rounded up to the tiles): elements beyond
// W are zeros.  One thread writes one lane's 16 bytes of one frag.
__global__ __launch_bounds__(256) void k_repack(const uint16_t* __restrict__ W, int K, int N, int Kp, int Np,
                                                uint4* __restrict__ dst, int order, int tile_order, int tile_offset,
                                                int total_tiles) {
  const int KB = Kp / 16;
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long nfrag = (long long)(Np / 32) * KB;
  if (idx >= nfrag * 64) return;
  const int lane = (int)(idx % 64);
  const long long f = idx / 64;
  const int tile = (int)(f / KB), kb = (int)(f % KB);
  const int il = lane % 32, h = lane / 32;
  const int n = tile * 32 + il;
  uint16_t v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const int kl = (order == ORDER_NATURAL) ? 8 * h + s : 8 * (s / 4) + 4 * h + (s % 4);
    const int k = 16 * kb + kl;
    v[s] = (k < K && n < N) ? W[(size_t)k * N + n] : (uint16_t)0;
  }
  const long long frag = (tile_order == TILE_MAJOR) ? (long long)(tile_offset + tile) * KB + kb
                                                    : (long long)kb * total_tiles + tile_offset + tile;
  uint4 o;
  o.x = v[0] | ((uint32_t)v[1] << 16);
  o.y = v[2] | ((uint32_t)v[3] << 16);
  o.z = v[4] | ((uint32_t)v[5] << 16);
  o.w = v[6] | ((uint32_t)v[7] << 16);
  dst[frag * 64 + lane] = o;
}

static int repack(const void* W, int64_t K, int64_t N, int64_t Kp, int64_t Np, void* dst, int order, int tile_order,
                  int tile_offset, int total_tiles, hipStream_t st) {
  const long long threads = (Np / 32) * (Kp / 16) * 64;
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  hipLaunchKernelGGL(k_repack, dim3(blocks), dim3(256), 0, st, (const uint16_t*)W, (int)K, (int)N, (int)Kp, (int)Np, (uint4*)dst,
                     order, tile_order, tile_offset, total_tiles);
  return (int)hipGetLastError();
}

int bf16_repack_all(const Ctx* c, hipStream_t st) {
  const Plan& p = c->plan;
  const svdmlp_desc& de = c->desc;
  char* ws = c->ws;
  int e;
  if (p.kind == SVDMLP_LINEAR) {
    // U^T: rows p in [0, r), contraction over d, meets row-major X -> natural order; V^T: rows n in [0, ffn),
    // contraction over r, meets T produced by an MFMA -> chain order
    if ((e = repack(de.Ug, p.d, p.r_in, p.d, p.r, ws + p.off_wU, ORDER_NATURAL, TILE_MAJOR, 0, (int)(p.r / 32), st))) return e;
    if ((e = repack(de.Vg, p.r_in, p.ffn, p.r, p.ffn, ws + p.off_wVd, ORDER_CHAIN, TILE_MAJOR, 0, (int)(p.ffn / 32), st))) return e;
    return (int)hipMemsetAsync(ws + p.off_cnt, 0, CNT_BYTES, st);   // tickets of the streaming path start at zero
  }
  // [Ug | Uu]^T: rows p in [0, 2r), contraction over d, meets X read from row-major memory -> natural order
  const int pt = (int)(2 * p.r / 32);
  if ((e = repack(de.Ug, p.d, p.r_in, p.d, p.r, ws + p.off_wU, ORDER_NATURAL, TILE_MAJOR, 0, pt, st))) return e;
  if ((e = repack(de.Uu, p.d, p.r_in, p.d, p.r, ws + p.off_wU, ORDER_NATURAL, TILE_MAJOR, (int)(p.r / 32), pt, st))) return e;
  // Vg^T, Vu^T: rows n in [0, ffn), contraction over r, meet T produced by an MFMA -> chain order
  const int nt = (int)(p.ffn / 32);
  if ((e = repack(de.Vg, p.r_in, p.ffn_in, p.r, p.ffn, ws + p.off_wVg, ORDER_CHAIN, TILE_MAJOR, 0, nt, st))) return e;
  if ((e = repack(de.Vu, p.r_in, p.ffn_in, p.r, p.ffn, ws + p.off_wVu, ORDER_CHAIN, TILE_MAJOR, 0, nt, st))) return e;
  // Ud^T: rows q in [0, rd), contraction over ffn, meets H from registers -> chain order; contraction-block major
  // so that the frags one ffn chunk needs are contiguous
  const int qt = (int)(p.rd / 32);
  if ((e = repack(de.Ud, p.ffn_in, p.rd_in, p.ffn, p.rd, ws + p.off_wUd, ORDER_CHAIN, KB_MAJOR, 0, qt, st))) return e;
  // Vd^T: rows c in [0, d), contraction over rd, meets Td produced by an MFMA -> chain order
  if ((e = repack(de.Vd, p.rd_in, p.d, p.rd, p.d, ws + p.off_wVd, ORDER_CHAIN, TILE_MAJOR, 0, (int)(p.d / 32), st))) return e;
  // tickets of the streaming paths start at zero and are left at zero by every forward; the completion counters
  // of the single-kernel decode path start at zero and only grow
  return (int)hipMemsetAsync(ws + p.off_cnt, 0, CNT_BYTES, st);
}

}  // namespace svdmlp
