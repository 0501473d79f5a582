// The planner of the MFMA-tiled path: for each stage whose shape leaves a choice (first product, first phase of the
// down projection, last product) it lists the candidates the kernels can run, gives each a time from a cost model of
// the compute unit, and takes the cheapest.  Host code only.
//
// This is the counterpart of the paper's block-size selection (Sec. 4.2.2, Eq. 10 - 11: arithmetic intensity against
// HBM on one side, the SBUF footprint on the other).  On a CDNA4 compute unit the two sides are different ones:
//   * what a tile costs per contraction block is max(MFMA time, operand bytes / the rate at which the CU pulls
//     operands into LDS).  The MFMA time of a 256 x 256 tile is 512 clocks per block of 16 (64 MFMAs on four matrix
//     cores, 32 clocks each), its operands are 16 KiB; a 128 x 128 tile has a quarter of the MFMAs for half the bytes.
//     The copy rate is what the kernels were measured to sustain while they compute (profiles/: requests x 128 B over
//     the active cycles), 16 - 23 B/clk per CU depending on where the operands come from, so every tile shape here is
//     bound by its operand bytes and the larger tile wins whenever it fills the chip;
//   * what caps the tile is the register file (256 x 256 fp32 accumulators are half of it), so the only way to give
//     every CU a large tile when the output is small is to cut the contraction into ranges, which costs the fp32
//     partial tiles: written by the kernel, read back and added by k_reduce at HBM speed, plus that launch.
// The figures below are measurements on one MI355X at the clock it sustains under this load; they rank candidates,
// they are not a simulator (the GPU test that times every candidate asserts the choice is within a few percent of the
// best one at the benchmark shapes).
#include <cmath>

#include "common.h"

namespace svdmlp {

namespace {

constexpr double CLK_MHZ = 2000.0;        // sustained under MFMA load (GRBM_GUI_ACTIVE over the kernel time)
constexpr int N_CU = 256;
constexpr double MFMA_CLK = 32.0;         // one v_mfma_f32_32x32x16_bf16 occupies a SIMD's matrix core this long
constexpr double PHASE_OVERHEAD = 1.05;   // barriers and issue gaps around the MFMAs of a phase
// Operand copy rates into LDS, bytes per clock per CU, while the kernel computes.  Fitted to the per-kernel times of
// every candidate at eleven shapes (prefill ranks 256 / 512 / 1024, the wide layer, 300 .. 8192 rows).
constexpr double FETCH_S1 = 23.0;         // k_s1: X rows from HBM, U from L2
constexpr double FETCH_IN = 24.0;         // k_in
constexpr double FETCH_OUT = 18.0;        // k_out
constexpr double FETCH_S5 = 20.0;         // k_s5, one workgroup on the CU; two share the rate
// k_down1 streams the ffn-wide activation from HBM; what one CU gets falls with the number of CUs pulling at once:
// 31 B/clk with 64 workgroups, 27 with 128, 21 with 256
double fetch_down(double active_cus) { return 1.0 / (0.02646 + 8.27e-5 * active_cus); }
constexpr double LAUNCH_US = 3.0;         // a dependent launch, as the per-kernel events see it
constexpr double RAMP_US = 2.0;           // filling the pipeline of a kernel's first tile, draining its last stores
constexpr double OUT_EPILOGUE_US = 4.0;   // k_out: turning the tile around through LDS and storing it
constexpr double REDUCE_LAUNCH_US = 1.5;  // k_reduce behind its producer
// fp32 partial tiles: every workgroup writes its own at the end of the kernel, all at about the same time, so the
// write is not hidden; k_reduce then streams them in and the sums out
constexpr double PARTIAL_WRITE_BYTES_PER_US = 5.0e6;
constexpr double REDUCE_BYTES_PER_US = 5.0e6;
constexpr double HBM_STREAM_BYTES_PER_US = 5.0e6;   // what a kernel that also computes pulls from HBM at best

double tile_us(double rows, double cols, double k, double fetch) {
  const double blocks = k / 16.0;
  const double mfma = (rows / 32.0) * (cols / 32.0) / 4.0 * MFMA_CLK * PHASE_OVERHEAD;
  const double copy = (rows + cols) * 32.0 / fetch;
  return blocks * (mfma > copy ? mfma : copy) / CLK_MHZ;
}

double rounds(double workgroups, double per_round) { return std::ceil(workgroups / per_round); }

// fp32 partial tiles of S ranges: written by the producer, read and added by k_reduce, which writes the bf16 result
double partials_us(int S, double rows, double cols) {
  const double part = (double)S * rows * cols * 4.0;
  return part / PARTIAL_WRITE_BYTES_PER_US + REDUCE_LAUNCH_US + (part + rows * cols * 2.0) / REDUCE_BYTES_PER_US;
}
double cut_us(int S, double rows, double cols) { return S <= 1 ? 0.0 : partials_us(S, rows, cols); }

}  // namespace

// ---- first product T = X [Ug | Uu] ---------------------------------------------------------------------------
bool first_valid(int kernel, int S, int64_t M, int64_t d, int64_t ncols) {
  if (S < 1 || S > MAX_FIRST_RANGES || ncols % 128) return false;
  if (S > 1 && d / S < 512) return false;          // at least eight steps of 64 per range
  if (kernel == FIRST_S1) return true;
  if (kernel != FIRST_IN) return false;
  const int64_t Mp = (M + 255) / 256 * 256;
  return ncols % 256 == 0 && d % 64 == 0 && Mp * d * 2 < (int64_t(1) << 32);   // k_in: 32-bit byte offsets into X
}

static double first_us(int kernel, int S, int64_t M, int64_t d, int64_t ncols) {
  if (kernel == FIRST_S1) {
    const double mt = (double)((M + 127) / 128), wgs = mt * (double)(ncols / 128) * S;
    return LAUNCH_US + rounds(wgs, N_CU) * tile_us(128, 128, (double)d / S, FETCH_S1) + RAMP_US + cut_us(S, mt * 128, (double)ncols);
  }
  const double mt = (double)((M + 255) / 256), wgs = mt * (double)(ncols / 256) * S;
  return LAUNCH_US + rounds(wgs, N_CU) * tile_us(256, 256, (double)d / S, FETCH_IN) + RAMP_US + cut_us(S, mt * 256, (double)ncols);
}

int first_candidates(int64_t M, int64_t d, int64_t ncols, StageCandidate* out, int cap) {
  int n = 0;
  for (int kernel = FIRST_S1; kernel <= FIRST_IN; ++kernel)
    for (int S = 1; S <= MAX_FIRST_RANGES && n < cap; ++S) {
      if (!first_valid(kernel, S, M, d, ncols)) continue;
      out[n++] = StageCandidate{kernel, S, first_us(kernel, S, M, d, ncols), true};
    }
  return n;
}

StageChoice choose_first(int64_t M, int64_t d, int64_t ncols, bool small_only, const PlanForce* f) {
  // the answer depends on the number of 256-row tiles only (the workspace is sized per tile count)
  const int64_t Mp = (M + 255) / 256 * 256;
  if (f && f->first_kernel && first_valid(f->first_kernel, f->first_ranges ? f->first_ranges : 1, Mp, d, ncols)) {
    const int S = f->first_ranges ? f->first_ranges : 1;
    return StageChoice{f->first_kernel, S, first_us(f->first_kernel, S, Mp, d, ncols)};
  }
  StageCandidate c[2 * MAX_FIRST_RANGES];
  const int n = first_candidates(Mp, d, ncols, c, 2 * MAX_FIRST_RANGES);
  StageChoice best{FIRST_S1, 1, 1e30};
  for (int i = 0; i < n; ++i) {
    if (small_only && c[i].kernel != FIRST_S1) continue;
    if (c[i].est_us < best.est_us) best = StageChoice{c[i].kernel, c[i].ranges, c[i].est_us};
  }
  return best;
}

// ---- first phase of the down projection Tdp = H Ud, per ffn range ---------------------------------------------
bool down_valid(int splits, int64_t mt256, int64_t qt, int64_t nsteps) {
  if (splits < 1 || splits > MAX_DOWN_RANGES) return false;
  if (splits > 1 && nsteps / splits < 4) return false;                 // every range keeps at least four steps of 32
  return mt256 * qt * splits < (int64_t(1) << 20);
}

static double down_us(int s, int64_t M, int64_t rd, int64_t ffn) {
  const double mt = (double)((M + 255) / 256), qt = (double)(rd / 256), wgs = mt * qt * s;
  const double active = wgs < N_CU ? wgs : N_CU;
  double main_us = rounds(wgs, N_CU) * tile_us(256, 256, (double)ffn / s, fetch_down(active));
  // the activation and the factor come from HBM once, whatever the cut
  const double floor_us = (mt * 256 * (double)ffn * 2.0 + (double)rd * (double)ffn * 2.0) / HBM_STREAM_BYTES_PER_US;
  if (main_us < floor_us) main_us = floor_us;
  // partial tiles are written even with one range (k_reduce turns them into the bf16 strip)
  return LAUNCH_US + main_us + RAMP_US + partials_us(s, mt * 256, (double)rd);
}

int down_candidates(int64_t M, int64_t rd, int64_t ffn, StageCandidate* out, int cap) {
  const int64_t mt = (M + 255) / 256, qt = rd / 256, nsteps = ffn / 32;
  int n = 0;
  for (int s = 1; s <= MAX_DOWN_RANGES && n < cap; ++s) {
    if (!down_valid(s, mt, qt, nsteps)) continue;
    out[n++] = StageCandidate{0, s, down_us(s, M, rd, ffn), true};
  }
  return n;
}

StageChoice choose_down(int64_t M, int64_t rd, int64_t ffn, const PlanForce* f) {
  const int64_t mt = (M + 255) / 256, qt = rd / 256, nsteps = ffn / 32;
  if (f && f->down_ranges && down_valid(f->down_ranges, mt, qt, nsteps))
    return StageChoice{0, f->down_ranges, down_us(f->down_ranges, M, rd, ffn)};
  StageCandidate c[MAX_DOWN_RANGES];
  const int n = down_candidates(M, rd, ffn, c, MAX_DOWN_RANGES);
  StageChoice best{0, 1, 1e30};
  for (int i = 0; i < n; ++i)
    if (c[i].est_us < best.est_us) best = StageChoice{0, c[i].ranges, c[i].est_us};
  return best;
}

// ---- last product Y = Td Vd (O = T V of the single layer) -----------------------------------------------------
static double out_us(int kernel, int64_t M, int64_t n, int64_t k) {
  if (kernel == OUT_256) {
    const double wgs = (double)((M + 255) / 256) * (double)(n / 256);
    return LAUNCH_US + rounds(wgs, N_CU) * (tile_us(256, 256, (double)k, FETCH_OUT) + OUT_EPILOGUE_US) + RAMP_US;
  }
  // 128 x 128 tiles: two workgroups share a CU (and its copy rate) once there are more workgroups than CUs
  const double wgs = (double)((M + 127) / 128) * (double)(n / 128);
  const double share = wgs > N_CU ? 2.0 : 1.0;
  return LAUNCH_US + rounds(wgs, N_CU * share) * (tile_us(128, 128, (double)k, FETCH_S5 / share) + 1.0) + RAMP_US;
}

int out_candidates(int64_t M, int64_t n, int64_t k, StageCandidate* out, int cap) {
  int c = 0;
  if (cap > 0 && n % 256 == 0) out[c++] = StageCandidate{OUT_256, 1, out_us(OUT_256, M, n, k), true};
  if (c < cap) out[c++] = StageCandidate{OUT_128, 1, out_us(OUT_128, M, n, k), true};
  return c;
}

StageChoice choose_out(int64_t M, int64_t n, int64_t k, bool small_only, const PlanForce* f) {
  if (f && f->out_kernel == OUT_128) return StageChoice{OUT_128, 1, out_us(OUT_128, M, n, k)};
  if (f && f->out_kernel == OUT_256 && n % 256 == 0) return StageChoice{OUT_256, 1, out_us(OUT_256, M, n, k)};
  StageCandidate c[2];
  const int nc = out_candidates(M, n, k, c, 2);
  StageChoice best{OUT_128, 1, 1e30};
  for (int i = 0; i < nc; ++i) {
    if (small_only && c[i].kernel != OUT_128) continue;
    if (c[i].est_us < best.est_us) best = StageChoice{c[i].kernel, 1, c[i].est_us};
  }
  return best;
}

}  // namespace svdmlp
