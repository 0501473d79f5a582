// C ABI of the svdmlp library: argument checking, workspace planning, path dispatch.
// Host code only; every arithmetic step of the forward runs in the kernels of the other files.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.h"

namespace svdmlp {

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int tiled_splits(int64_t mtiles128, int64_t nchunks) {
  // Enough (row tile, ffn range) pairs to give each of the 256 CUs one workgroup, never more
  // ranges than there are ffn chunks.
  int64_t s = (256 + mtiles128 - 1) / mtiles128;
  if (s > nchunks) s = nchunks;
  if (s < 1) s = 1;
  return (int)s;
}

bool staged_supported(int64_t rd, int64_t ffn) { return rd % 256 == 0 && ffn % 256 == 0; }

// 32-column tiles of the down rank that one workgroup of the fused tiled kernel can own
static bool fused_rank_tiles(int64_t x) { return x == 4 || x == 8 || x == 16; }

int make_plan(const svdmlp_desc* de, Plan* p) {
  if (!de || !p) return SVDMLP_INVALID_ARGUMENT;
  std::memset(p, 0, sizeof(*p));
  if (de->kind != SVDMLP_GATED && de->kind != SVDMLP_LINEAR) return SVDMLP_INVALID_ARGUMENT;
  if (de->dtype != SVDMLP_BF16 && de->dtype != SVDMLP_F32) return SVDMLP_INVALID_ARGUMENT;
  const bool gated = de->kind == SVDMLP_GATED;
  if (de->max_M <= 0 || de->d <= 0 || de->ffn <= 0 || de->r <= 0) return SVDMLP_INVALID_ARGUMENT;
  if (gated && de->r_down <= 0) return SVDMLP_INVALID_ARGUMENT;
  const int64_t lim = de->d < de->ffn ? de->d : de->ffn;
  if (de->r > lim || (gated && de->r_down > lim)) return SVDMLP_INVALID_ARGUMENT;
  if (de->max_M > (int64_t(1) << 24) || de->d > (int64_t(1) << 20) || de->ffn > (int64_t(1) << 20))
    return SVDMLP_UNSUPPORTED;
  if ((de->flags & SVDMLP_FLAG_FORCE_TILED) && (de->flags & SVDMLP_FLAG_FORCE_STREAM)) return SVDMLP_INVALID_ARGUMENT;

  p->max_M = de->max_M; p->d = de->d; p->ffn = de->ffn; p->r = de->r;
  p->rd = gated ? de->r_down : 0;
  p->r_in = p->r;
  p->rd_in = p->rd;
  p->ffn_in = p->ffn;
  p->kind = de->kind; p->dtype = de->dtype; p->flags = de->flags;
  const bool room = (de->flags & SVDMLP_FLAG_PLAN_ROOM) != 0;

  if (de->dtype == SVDMLP_F32) {
    // fp32 intermediates: T [M, 2r] (LINEAR: [M, r]), H [M, ffn], Td [M, rd]
    size_t off = 0;
    p->f32_T = off;  off += (size_t)de->max_M * (gated ? 2 : 1) * de->r;
    if (gated) {
      p->f32_H = off;  off += (size_t)de->max_M * de->ffn;
      p->f32_Td = off; off += (size_t)de->max_M * p->rd;
    }
    p->total_bytes = align_up(off * sizeof(float), 256);
    return SVDMLP_OK;
  }

  // ---- bf16 ----
  if (!gated) {
    // single factored layer O = (X U) V: the first and the last kernel of the tiled path back to back
    const int64_t d = de->d, n = de->ffn;
    if (d % 128 || n % 128) return SVDMLP_UNSUPPORTED;
    const int64_t r = (de->r + 127) / 128 * 128;   // zero-padded rank
    p->r = r;
    p->Mpad = (de->max_M + 255) / 256 * 256;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    p->off_wU = take((size_t)r * d * 2);
    p->off_wVd = take((size_t)n * r * 2);
    p->off_T = take((size_t)p->Mpad * r * 2);
    // fp32 tiles of T per range of d when the first stage cuts its contraction (few tiles): the largest the planner
    // picks for any row count up to max_M (with SVDMLP_FLAG_PLAN_ROOM: room for every candidate)
    size_t pbytes = 0;
    for (int64_t mt = 1; mt <= p->Mpad / 256; ++mt) {
      const StageChoice ch = choose_first(mt * 256, d, r, linear_on_small_tiles(*p), nullptr);
      const int S = room ? MAX_FIRST_RANGES : ch.ranges;
      if (S > 1 && (size_t)S * mt * 256 * r * 4 > pbytes) pbytes = (size_t)S * mt * 256 * r * 4;
    }
    p->part_bytes = pbytes;
    p->off_Tdp = take(pbytes);
    p->off_part = take((size_t)8 << 20);              // streaming path: split-K partial tiles
    p->off_cnt = take(CNT_BYTES);                     // ... and its tickets
    p->total_bytes = off;
    return SVDMLP_OK;
  }
  const int64_t d = de->d;
  if (d % 128) return SVDMLP_UNSUPPORTED;
  // The ffn-wide activation is internal, so ffn is rounded up to the 256-wide tiles of the staged variant: zero
  // columns of Vg and Vu give H = SiLU(0) * 0 = 0 there, and the matching rows of Ud are zeros as well.
  const int64_t ffn = (de->ffn + 255) / 256 * 256;
  p->ffn = ffn;
  // Ranks are rounded up to what the tiles take (zero columns of U, zero rows of V change nothing): r to a multiple
  // of 64, at least 128; the down rank to a multiple of 256 for the staged variant (256-wide rank tiles), else to
  // what the fused one takes (a workgroup owns 4, 8 or 16 32-wide rank tiles, or groups of 16).
  const int64_t r = de->r <= 128 ? 128 : (de->r + 63) / 64 * 64;
  // The fused variant is also the automatic choice when both ranks fit one 128-wide tile: the staged variant would run
  // the down rank padded to 256, and with so little arithmetic per element of H its round trip through HBM is what
  // bounds it (measured at d = 4096, ffn = 14336, r = r_down = 128: fused 9-16 % faster from 512 rows on, 3 % slower
  // at 256 rows; from r = 192 on the staged variant is level or faster).
  const bool want_fused = (de->flags & SVDMLP_FLAG_TILED_FUSED) != 0 || (de->r <= 128 && p->rd <= 128);
  int64_t rd = p->rd;
  if (want_fused) rd = rd <= 128 ? 128 : rd <= 256 ? 256 : (rd + 511) / 512 * 512;
  else rd = (rd + 255) / 256 * 256;
  p->r = r;
  p->rd = rd;

  p->Mpad = (de->max_M + 255) / 256 * 256;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  p->off_wU = take((size_t)2 * r * d * 2);
  p->off_wVg = take((size_t)ffn * r * 2);
  p->off_wVu = take((size_t)ffn * r * 2);
  p->off_wUd = take((size_t)rd * ffn * 2);
  p->off_wVd = take((size_t)d * rd * 2);
  p->off_T = take((size_t)p->Mpad * 2 * r * 2);
  // split-K partial sums of Td: ranges(M) * padded M rows, maximised over M <= max_M (with SVDMLP_FLAG_PLAN_ROOM:
  // room for every candidate of the planner, so that a caller can force and time each of them)
  int64_t rows = 0;
  const int64_t nchunks = ffn / 64;
  for (int64_t mt = 1; mt <= p->Mpad / 128; ++mt) {
    int64_t rws = (int64_t)tiled_splits(mt, nchunks) * mt * 128;
    if (rws > rows) rows = rws;
  }
  if (staged_supported(rd, ffn))
    for (int64_t mt = 1; mt <= p->Mpad / 256; ++mt) {
      const int sp = room ? MAX_DOWN_RANGES : choose_down(mt * 256, rd, ffn, nullptr).ranges;
      int64_t rws = (int64_t)sp * mt * 256;
      if (rws > rows) rows = rws;
    }
  p->part_rows = rows;
  // the same buffer first holds the fp32 tiles of T per range of d when the first stage cuts its contraction (few tiles)
  size_t part_bytes = (size_t)rows * rd * 4;
  for (int64_t mt = 1; mt <= p->Mpad / 256; ++mt) {
    const int S = room ? MAX_FIRST_RANGES : choose_first(mt * 256, d, 2 * r, false, nullptr).ranges;
    if (S > 1 && (size_t)S * mt * 256 * 2 * r * 4 > part_bytes) part_bytes = (size_t)S * mt * 256 * 2 * r * 4;
  }
  p->part_bytes = part_bytes;
  p->off_Tdp = take(part_bytes);
  p->off_Td = take((size_t)p->Mpad * rd * 2);
  p->off_H = take((size_t)STREAM_MAX_M * ffn * 2);  // streaming path: the ffn-wide activation of its rows
  // staged tiled path: the whole gated activation as frags
  p->off_Hfull = take(staged_supported(rd, ffn) ? (size_t)p->Mpad * ffn * 2 : 0);
  p->off_part = take((size_t)8 << 20);              // streaming path: split-K partial tiles
  p->off_cnt = take(CNT_BYTES);                     // streaming paths: tickets, completion counters, per-workgroup flags
  p->total_bytes = off;
  return SVDMLP_OK;
}

static bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace svdmlp

using namespace svdmlp;

extern "C" {

int svdmlp_abi_version(void) { return 1; }

// Paper Eq. 5 (Sec. 4.1): block-aligned rank for a target compression ratio.
int64_t svdmlp_rank_for_ratio(int64_t k, int64_t n, double ratio, int64_t block, double alpha) {
  if (k <= 0 || n <= 0 || block <= 0 || !(ratio >= 0.0 && ratio < 1.0) || !(alpha >= 0.0 && alpha <= 1.0)) return -1;
  const double blocks = std::floor((double)k * (double)n * (1.0 - ratio) / ((double)(k + n) * (double)block) + alpha);
  const int64_t nb = blocks < 1.0 ? 1 : (int64_t)blocks;
  return nb * block;
}

const char* svdmlp_status_string(int status) {
  switch (status) {
    case SVDMLP_OK: return "ok";
    case SVDMLP_INVALID_ARGUMENT: return "invalid argument";
    case SVDMLP_UNSUPPORTED: return "unsupported dtype / kind / extents";
    case SVDMLP_WORKSPACE_TOO_SMALL: return "workspace too small";
    case SVDMLP_HIP_ERROR: return "HIP runtime error";
    case SVDMLP_NO_DEVICE: return "no gfx950 device";
    case SVDMLP_SCRATCH_TOO_SMALL: return "extents beyond the library's static scratch array";
    case SVDMLP_OUT_OF_HOST_MEMORY: return "out of host memory";
    case SVDMLP_TIMED_OUT: return "a bounded wait inside a kernel timed out";
    default: return "unknown status";
  }
}

size_t svdmlp_workspace_bytes(const svdmlp_desc* desc) {
  Plan p;
  if (make_plan(desc, &p) != SVDMLP_OK) return 0;
  return p.total_bytes;
}

// Which kernels a forward of M rows launches and how each one is cut over the chip: the same decision functions
// the launchers call, evaluated for a 256-CU device.  Host only.
int svdmlp_describe(const svdmlp_desc* desc, int64_t M, char* buf, size_t buf_bytes) {
  if (!desc || !buf || buf_bytes == 0) return SVDMLP_INVALID_ARGUMENT;
  buf[0] = 0;
  Plan p;
  const int st = make_plan(desc, &p);
  if (st != SVDMLP_OK) return st;
  if (M <= 0 || M > p.max_M) return SVDMLP_INVALID_ARGUMENT;
  size_t n = 0;
  auto put = [&](const char* fmt, auto... a) {
    if (n < buf_bytes) {
      const int k = std::snprintf(buf + n, buf_bytes - n, fmt, a...);
      if (k > 0) n += (size_t)k;
    }
  };
  const int MT128 = (int)((M + 127) / 128), MT256 = (int)((M + 255) / 256);
  // every candidate of a stage with the time the planner's cost model gives it (microseconds), the chosen one first
  auto put_scores = [&](const StageCandidate* c, int n, const StageChoice& ch, const char* const* kname) {
    put(" est_us=%.1f alternatives:", ch.est_us);
    // the five cheapest of the others, cheapest first
    bool used[64] = {};
    for (int shown = 0; shown < 5; ++shown) {
      int b = -1;
      for (int i = 0; i < n && i < 64; ++i) {
        if (used[i] || (c[i].kernel == ch.kernel && c[i].ranges == ch.ranges)) continue;
        if (b < 0 || c[i].est_us < c[b].est_us) b = i;
      }
      if (b < 0) break;
      used[b] = true;
      put(" %s/%d=%.1f", kname[c[b].kernel], c[b].ranges, c[b].est_us);
    }
    put("]");
  };
  static const char* const first_names[3] = {"", "s1", "in"};
  static const char* const down_names[1] = {"ranges"};
  static const char* const out_names[3] = {"", "out256", "out128"};
  auto first_stage = [&](int64_t ncols) {
    const StageChoice ch = choose_first(M, p.d, ncols, linear_on_small_tiles(p), nullptr);
    StageCandidate c[2 * MAX_FIRST_RANGES];
    const int n = linear_on_small_tiles(p) ? 0 : first_candidates((M + 255) / 256 * 256, p.d, ncols, c, 2 * MAX_FIRST_RANGES);
    if (ch.kernel == FIRST_IN) put(" k_in[tile=256x256 tiles=%d ranges=%d", MT256 * (int)(ncols / 256), ch.ranges);
    else put(" k_s1[tile=128x128 tiles=%d ranges=%d", MT128 * (int)(ncols / 128), ch.ranges);
    put_scores(c, n, ch, first_names);
    if (ch.ranges > 1) put(" k_reduce");
  };
  auto last_stage = [&](int64_t n_out, int64_t k) {
    const StageChoice ch = choose_out(M, n_out, k, linear_on_small_tiles(p), nullptr);
    StageCandidate c[2];
    const int n = linear_on_small_tiles(p) ? 0 : out_candidates(M, n_out, k, c, 2);
    if (ch.kernel == OUT_256) put(" k_out[tile=256x256 tiles=%d", MT256 * (int)(n_out / 256));
    else put(" k_s5[tile=128x128 tiles=%d", MT128 * (int)(n_out / 128));
    put_scores(c, n, ch, out_names);
  };
  if (p.dtype == SVDMLP_F32) {
    put("path=1 fp32-debug:%s", p.kind == SVDMLP_GATED ? " k_f32_gemm x5 (SiLU-gate epilogue in the third)" : " k_f32_gemm x2");
  } else if (p.kind == SVDMLP_LINEAR && ((linear_stream_pays(M, p.d, p.r, p.ffn) && stream_supported(p, M) && !(p.flags & (SVDMLP_FLAG_FORCE_TILED | SVDMLP_FLAG_TILE_128))) ||
                                         (p.flags & SVDMLP_FLAG_FORCE_STREAM))) {
    if (!stream_supported(p, M)) return SVDMLP_UNSUPPORTED;
    const int rt = M <= 32 ? 1 : M <= 64 ? 2 : 4;
    const int t1 = (int)(p.r / 32), t5 = (int)(p.ffn / 32);
    if (M <= 32 && p.d % 32 == 0 && p.r / 16 <= 2048) {
      put("path=7 bf16-linear-streaming: row_tiles=%d k_stream_d1[tile=16 tiles=%d ranges=%d]", rt,
          2 * t1, stream_splits16(2 * t1, (int)(p.d / 32), stream_tiles16(M)));
      if (stream_last_uses_tile16(true, t5)) put(" k_stream_d5[tile=16 tiles=%d]", 2 * t5);
      else put(" k_stream_d5[tiles=%d row_groups=%d]", t5, stream_row_groups_whole(rt, t5));
    } else {
      const int g1 = stream_row_groups(rt, t1, (int)(p.d / 16), true);
      put("path=7 bf16-linear-streaming: row_tiles=%d k_stream_d1[tiles=%d row_groups=%d ranges=%d] k_stream_d5[tiles=%d row_groups=%d]", rt,
          t1, g1, stream_splits(t1 * g1, (int)(p.d / 16), rt / g1), t5, stream_row_groups_whole(rt, t5));
    }
  } else if (p.kind == SVDMLP_LINEAR) {
    put("path=6 bf16-linear:");
    first_stage(p.r);
    last_stage(p.ffn, p.r);
  } else {
    bool stream_path = stream_supported(p, M);
    if (p.flags & SVDMLP_FLAG_FORCE_TILED) stream_path = false;
    if (p.flags & SVDMLP_FLAG_FORCE_STREAM) {
      if (!stream_supported(p, M)) return SVDMLP_UNSUPPORTED;
      stream_path = true;
    }
    if (stream_path) {
      const int rt = M <= 32 ? 1 : M <= 64 ? 2 : 4;
      const int t1 = (int)(2 * p.r / 32), t2 = (int)(p.ffn / 32), t4 = (int)(p.rd / 32), t5 = (int)(p.d / 32);
      if (stream_uses_tile16(M, p.d, p.ffn, p.r, p.rd)) {   // the two split phases (and a short last one) on 16-column tiles
        put("path=3 bf16-streaming: row_tiles=%d k_stream_d1[tile=16 tiles=%d ranges=%d] k_stream_d2[tiles=%d]"
            " k_stream_d4[tile=16 tiles=%d ranges=%d]", rt, 2 * t1, stream_splits16(2 * t1, (int)(p.d / 32), stream_tiles16(M)), t2,
            2 * t4, stream_splits16(2 * t4, (int)(p.ffn / 32), stream_tiles16(M)));
        if (stream_last_uses_tile16(true, t5)) put(" k_stream_d5[tile=16 tiles=%d]", 2 * t5);
        else put(" k_stream_d5[tiles=%d row_groups=%d]", t5, stream_row_groups_whole(rt, t5));
      } else {
        const int g1 = stream_row_groups(rt, t1, (int)(p.d / 16), true), g4 = stream_row_groups(rt, t4, (int)(p.ffn / 16), false);
        put("path=3 bf16-streaming: row_tiles=%d k_stream_d1[tiles=%d row_groups=%d ranges=%d] k_stream_d2[tiles=%d]"
            " k_stream_d4[tiles=%d row_groups=%d ranges=%d] k_stream_d5[tiles=%d row_groups=%d]", rt, t1, g1,
            stream_splits(t1 * g1, (int)(p.d / 16), rt / g1), t2, t4, g4, stream_splits(t4 * g4, (int)(p.ffn / 16), rt / g4), t5,
            stream_row_groups_whole(rt, t5));
      }
      if ((p.flags & SVDMLP_FLAG_STREAM_ONE_KERNEL) && M <= 32) put(" (one persistent kernel, path=4, if the device and the extents allow)");
    } else if (staged_supported(p.rd, p.ffn) && !(p.flags & SVDMLP_FLAG_TILED_FUSED)) {
      put("path=5 bf16-tiled-staged:");
      first_stage(2 * p.r);
      const GuPlan g = gate_up_plan(MT256, p.ffn, p.r, 256);
      put(" k_gate_up[tile=256x256 tiles=%d workgroups=%d full=%d halves=%d xcd_grid=%dx%d]", g.ntiles, g.G, g.nfull,
          g.halves ? 2 * g.rem : 0, g.ngm, g.ngm ? 8 / g.ngm : 0);
      const StageChoice dn = choose_down(M, p.rd, p.ffn, nullptr);
      StageCandidate dc[MAX_DOWN_RANGES];
      const int dn_n = down_candidates(M, p.rd, p.ffn, dc, MAX_DOWN_RANGES);
      put(" k_down1[tile=256x256 tiles=%d ranges=%d", MT256 * (int)(p.rd / 256), dn.ranges);
      put_scores(dc, dn_n, dn, down_names);
      put(" k_reduce");
      last_stage(p.d, p.rd);
    } else {
      put("path=2 bf16-tiled-fused:");
      first_stage(2 * p.r);
      put(" k_fused[rows=128 row_tiles=%d ffn_ranges=%d] k_reduce k_s5[tile=128x128 tiles=%d]", MT128,
          tiled_splits(MT128, p.ffn / 64), MT128 * (int)(p.d / 128));
    }
  }
  return n < buf_bytes ? SVDMLP_OK : SVDMLP_INVALID_ARGUMENT;
}

int svdmlp_create(const svdmlp_desc* desc, svdmlp_ctx** out) {
  if (!desc || !out) return SVDMLP_INVALID_ARGUMENT;
  Plan p;
  int st = make_plan(desc, &p);
  if (st != SVDMLP_OK) return st;
  const bool gated = desc->kind == SVDMLP_GATED;
  if (!desc->Ug || !desc->Vg) return SVDMLP_INVALID_ARGUMENT;
  if (gated && (!desc->Uu || !desc->Vu || !desc->Ud || !desc->Vd)) return SVDMLP_INVALID_ARGUMENT;
  const void* ptrs[6] = {desc->Ug, desc->Vg, desc->Uu, desc->Vu, desc->Ud, desc->Vd};
  for (int i = 0; i < (gated ? 6 : 2); ++i)
    if (!aligned16(ptrs[i])) return SVDMLP_INVALID_ARGUMENT;
  if (p.total_bytes > 0) {
    if (!desc->workspace) return SVDMLP_INVALID_ARGUMENT;
    if (reinterpret_cast<uintptr_t>(desc->workspace) & 255u) return SVDMLP_INVALID_ARGUMENT;
    if (desc->workspace_bytes < p.total_bytes) return SVDMLP_WORKSPACE_TOO_SMALL;
  }
  int n_cus = 0;
  int dev = -1;
  if (!(desc->flags & SVDMLP_FLAG_SKIP_ARCH_CHECK)) {
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return SVDMLP_NO_DEVICE; }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return SVDMLP_NO_DEVICE; }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return SVDMLP_NO_DEVICE;
    n_cus = prop.multiProcessorCount;
  }
  Ctx* c = new (std::nothrow) Ctx;
  if (!c) return SVDMLP_OUT_OF_HOST_MEMORY;
  c->desc = *desc;
  c->plan = p;
  c->ws = static_cast<char*>(desc->workspace);
  c->last_hip_error = 0;
  c->last_path = 0;
  c->n_cus = n_cus;
  c->device = dev;
  if (desc->dtype == SVDMLP_BF16 && gated && !(desc->flags & SVDMLP_FLAG_SKIP_ARCH_CHECK)) {
    // this device's copy of the static scratch array, looked up here so that no forward ever has to
    const int e = static_scratch_resolve(dev, &c->static_scratch);
    if (e != 0) { (void)hipGetLastError(); delete c; return SVDMLP_HIP_ERROR; }
  }
  if (desc->dtype == SVDMLP_BF16 && !(desc->flags & SVDMLP_FLAG_SKIP_ARCH_CHECK)) {
    // One-time re-tiling of the invariant factors into matrix-core fragments.
    int e = (int)hipDeviceSynchronize();
    if (e == 0) e = bf16_repack_all(c, nullptr);
    if (e == 0) e = (int)hipStreamSynchronize(nullptr);
    if (e != 0) { (void)hipGetLastError(); delete c; return SVDMLP_HIP_ERROR; }
  }
  *out = reinterpret_cast<svdmlp_ctx*>(c);
  return SVDMLP_OK;
}

int svdmlp_forward(svdmlp_ctx* ctx, const void* X, int64_t M, void* Y, void* hip_stream) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c || M < 0) return SVDMLP_INVALID_ARGUMENT;
  if (M == 0) return SVDMLP_OK;
  if (!X || !Y || X == Y || M > c->plan.max_M) return SVDMLP_INVALID_ARGUMENT;
  if (!aligned16(X) || !aligned16(Y)) return SVDMLP_INVALID_ARGUMENT;
  if (c->desc.flags & SVDMLP_FLAG_SKIP_ARCH_CHECK) return SVDMLP_NO_DEVICE;  // host-only context: nothing to run on
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int e;
  if (c->plan.dtype == SVDMLP_F32) {
    c->last_path = 1;
    e = f32_forward(c, X, M, Y, st);
  } else if (c->plan.kind == SVDMLP_LINEAR) {
    bool stream_path = linear_stream_pays(M, c->plan.d, c->plan.r, c->plan.ffn) && stream_supported(c->plan, M) &&
                       !(c->plan.flags & (SVDMLP_FLAG_FORCE_TILED | SVDMLP_FLAG_TILE_128));
    if (c->plan.flags & SVDMLP_FLAG_FORCE_STREAM) {
      if (!stream_supported(c->plan, M)) return SVDMLP_UNSUPPORTED;
      stream_path = true;
    }
    c->last_path = stream_path ? 7 : 6;
    e = stream_path ? bf16_linear_stream_forward(c, X, M, Y, st) : bf16_linear_forward(c, X, M, Y, st);
  } else {
    bool stream_path = stream_supported(c->plan, M);   // else the tiled path, which takes any row count
    if (c->plan.flags & SVDMLP_FLAG_FORCE_TILED) stream_path = false;
    if (c->plan.flags & SVDMLP_FLAG_FORCE_STREAM) {
      if (!stream_supported(c->plan, M)) return SVDMLP_UNSUPPORTED;
      stream_path = true;
    }
    const bool one_kernel = stream_path && M <= 32 && (c->plan.flags & SVDMLP_FLAG_STREAM_ONE_KERNEL) && bf16_decode_supported(c, M);
    const bool staged = staged_supported(c->plan.rd, c->plan.ffn) && !(c->plan.flags & SVDMLP_FLAG_TILED_FUSED);
    c->last_path = stream_path ? (one_kernel ? 4 : 3) : (staged ? 5 : 2);
    if (one_kernel) c->ran_one_kernel = true;
    e = !stream_path ? bf16_tiled_forward(c, X, M, Y, st)
                     : one_kernel ? bf16_decode_forward(c, X, M, Y, st) : bf16_stream_forward(c, X, M, Y, st);
  }
  if (e != 0) {
    c->last_hip_error = e;
    (void)hipGetLastError();
    return SVDMLP_HIP_ERROR;
  }
  return SVDMLP_OK;
}

int svdmlp_forward_static_scratch(svdmlp_ctx* ctx, const void* X, int64_t M, void* Y, void* hip_stream) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c || M < 0) return SVDMLP_INVALID_ARGUMENT;
  if (M == 0) return SVDMLP_OK;
  if (!X || !Y || X == Y || M > c->plan.max_M) return SVDMLP_INVALID_ARGUMENT;
  if (!aligned16(X) || !aligned16(Y)) return SVDMLP_INVALID_ARGUMENT;
  if (c->plan.dtype != SVDMLP_BF16 || c->plan.kind != SVDMLP_GATED || !stream_supported(c->plan, M)) return SVDMLP_UNSUPPORTED;
  if (stream_static_scratch_need(c->plan, M) > STATIC_SCRATCH_BYTES) return SVDMLP_SCRATCH_TOO_SMALL;
  if (c->desc.flags & SVDMLP_FLAG_SKIP_ARCH_CHECK) return SVDMLP_NO_DEVICE;  // host-only context: nothing to run on
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != c->device) { (void)hipGetLastError(); return SVDMLP_INVALID_ARGUMENT; }
  c->last_path = 3;
  const int e = bf16_stream_forward_static(c, X, M, Y, static_cast<hipStream_t>(hip_stream));
  if (e != 0) {
    c->last_hip_error = e;
    (void)hipGetLastError();
    return SVDMLP_HIP_ERROR;
  }
  return SVDMLP_OK;
}

size_t svdmlp_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int svdmlp_debug_set_poll_limit(svdmlp_ctx* ctx, int32_t polls) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c || polls < -1) return SVDMLP_INVALID_ARGUMENT;
  c->poll_limit = polls;
  return SVDMLP_OK;
}

int svdmlp_check(svdmlp_ctx* ctx) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return SVDMLP_INVALID_ARGUMENT;
  if (!c->ran_one_kernel) return SVDMLP_OK;
  unsigned word = 0;
  char* err = decode_error_word(c);
  if (hipMemcpy(&word, err, sizeof(word), hipMemcpyDeviceToHost) != hipSuccess) { (void)hipGetLastError(); return SVDMLP_HIP_ERROR; }
  if (!word) return SVDMLP_OK;
  word = 0;
  if (hipMemcpy(err, &word, sizeof(word), hipMemcpyHostToDevice) != hipSuccess) { (void)hipGetLastError(); return SVDMLP_HIP_ERROR; }
  return SVDMLP_TIMED_OUT;
}

int svdmlp_force_plan(svdmlp_ctx* ctx, int32_t first_kernel, int32_t first_ranges, int32_t down_ranges, int32_t out_kernel) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c) return SVDMLP_INVALID_ARGUMENT;
  if (first_kernel < 0 || first_kernel > FIRST_IN || out_kernel < 0 || out_kernel > OUT_128) return SVDMLP_INVALID_ARGUMENT;
  if (first_ranges < 0 || first_ranges > MAX_FIRST_RANGES || down_ranges < 0 || down_ranges > MAX_DOWN_RANGES)
    return SVDMLP_INVALID_ARGUMENT;
  if (first_ranges && !first_kernel) return SVDMLP_INVALID_ARGUMENT;   // ranges belong to a kernel
  if (c->plan.dtype != SVDMLP_BF16) return SVDMLP_UNSUPPORTED;
  c->force = PlanForce{first_kernel, first_ranges, down_ranges, out_kernel};
  return SVDMLP_OK;
}

static void prof_release(Ctx* c) {
  Prof& p = c->prof;
  if (p.ev) {
    for (int i = 0; i < p.cap * PROF_MAXK * 2; ++i) (void)hipEventDestroy(p.ev[i]);
    delete[] p.ev;
  }
  p.ev = nullptr;
  p.cap = p.nfwd = 0;
}

int svdmlp_destroy(svdmlp_ctx* ctx) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (c) prof_release(c);
  delete c;
  return SVDMLP_OK;
}

int svdmlp_profile_begin(svdmlp_ctx* ctx, int max_forwards) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c || max_forwards <= 0 || max_forwards > 4096) return SVDMLP_INVALID_ARGUMENT;
  prof_release(c);
  Prof& p = c->prof;
  const int n = max_forwards * PROF_MAXK * 2;
  p.ev = new (std::nothrow) hipEvent_t[n];
  if (!p.ev) return SVDMLP_OUT_OF_HOST_MEMORY;
  for (int i = 0; i < n; ++i) {
    if (hipEventCreate(&p.ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(p.ev[j]);
      delete[] p.ev;
      p.ev = nullptr;
      (void)hipGetLastError();
      return SVDMLP_HIP_ERROR;
    }
  }
  p.cap = max_forwards;
  p.nfwd = 0;
  p.nk = 0;
  return SVDMLP_OK;
}

int svdmlp_profile_end(svdmlp_ctx* ctx, float* avg_ms, int* n_kernels, int* n_forwards) {
  Ctx* c = reinterpret_cast<Ctx*>(ctx);
  if (!c || !avg_ms || !n_kernels || !n_forwards) return SVDMLP_INVALID_ARGUMENT;
  Prof& p = c->prof;
  if (!p.ev) return SVDMLP_INVALID_ARGUMENT;
  int st = SVDMLP_OK;
  double sum[PROF_MAXK] = {};
  for (int f = 0; f < p.nfwd && st == SVDMLP_OK; ++f)
    for (int k = 0; k < p.nk; ++k) {
      hipEvent_t e0 = p.ev[(f * PROF_MAXK + k) * 2], e1 = p.ev[(f * PROF_MAXK + k) * 2 + 1];
      float ms = 0.f;
      if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
        (void)hipGetLastError();
        st = SVDMLP_HIP_ERROR;
        break;
      }
      sum[k] += ms;
    }
  *n_kernels = p.nk;
  *n_forwards = p.nfwd;
  for (int k = 0; k < p.nk; ++k) avg_ms[k] = p.nfwd ? (float)(sum[k] / p.nfwd) : 0.f;
  prof_release(c);
  return st;
}

const char* svdmlp_profile_kernel_name(const svdmlp_ctx* ctx, int k) {
  const Ctx* c = reinterpret_cast<const Ctx*>(ctx);
  if (!c || k < 0 || k >= c->prof.nk) return nullptr;
  return c->prof.names[k];
}

int svdmlp_last_hip_error(const svdmlp_ctx* ctx) { return ctx ? reinterpret_cast<const Ctx*>(ctx)->last_hip_error : 0; }
int svdmlp_last_path(const svdmlp_ctx* ctx) { return ctx ? reinterpret_cast<const Ctx*>(ctx)->last_path : 0; }

}  // extern "C"
