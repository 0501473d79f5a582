// Shared declarations of the svdmlp HIP library (gfx950 only).
//
// Fragment layout ("frag") used for every matrix-core operand that lives in HBM
// ----------------------------------------------------------------------------
// v_mfma_f32_32x32x16_bf16 takes, per lane, eight bf16 of one operand row:
// lane l supplies row (l % 32) and the eight contraction indices of half h = l / 32.
// A frag is the 1 KiB image of one such operand (32 rows x 16 contraction indices)
// exactly as the 64 lanes hold it: lane-major, 16 bytes per lane.  A wave loads a
// frag with one perfectly coalesced 16-byte-per-lane access and LDS copies of it are
// read back conflict-free with ds_read_b128 at lane * 16.
//
// Which eight contraction indices (out of the 16 of a frag) a lane holds:
//   natural order: k = 8 h + s            (s = slot 0..7)   -- data that comes from row-major memory
//   chain order  : k = 8 (s / 4) + 4 h + s % 4               -- data that comes out of a previous MFMA
// The chain order is what a lane of the 32x32 accumulator tile already owns when the
// product was computed transposed (lane = activation row m, registers = output index):
// registers 8t .. 8t+7 of the accumulator, rounded to bf16, ARE the frag for contraction
// block t of the next product.  This is the matrix-core form of the paper's "implicit
// transposition" (Sec. 4.2.1): the intermediate is born in the layout its consumer needs.
// Both operands of an MFMA use the same order, so any order is valid as long as the
// weight frags were built with the order of the activation they meet.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/svdmlp.h"

namespace svdmlp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int FRAG_ELEMS = 512;  // 32 rows x 16 k, bf16
constexpr int FRAG_BYTES = 1024;
constexpr int UNIT_BYTES = 16384;  // one LDS ring slot: 16 frags, filled by 4 waves x 4 loads x 64 lanes x 16 B

enum FragOrder { ORDER_NATURAL = 0, ORDER_CHAIN = 1 };
enum TileOrder { TILE_MAJOR = 0 /* [tile][kb] */, KB_MAJOR = 1 /* [kb][tile] */ };

// ---- device helpers -----------------------------------------------------------------------
#ifdef __HIPCC__
// 16-byte asynchronous copy global -> LDS: lane l's 16 bytes land at lds_wave_base + 16 l.
// (Measured on gfx950: placement is lane-linear; the instruction's immediate offset is not used.)
__device__ __forceinline__ void dma16(const void* gsrc_lane, void* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc_lane,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt left at their maxima).  gfx9 encoding:
// vmcnt[3:0] in bits 3:0, vmcnt[5:4] in bits 15:14, expcnt bits 6:4, lgkmcnt bits 11:8.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 0xF) | ((N >> 4) << 14));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() would also drain every outstanding
// global load (s_waitcnt vmcnt(0)), which would serialise the asynchronous global->LDS copies the ring
// keeps in flight; the copies a step needs are waited for explicitly with wait_vmcnt before this barrier.
// (A workgroup fence, even one restricted to LDS, makes the compiler drain vmcnt because the copies
// write LDS; so the barrier is bare, fenced for the compiler only.  Every wave has consumed its LDS
// reads in MFMAs before it reaches the barrier, so no LDS access is in flight across it.)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// ---- hand-scheduled LDS reads ---------------------------------------------------------------------
// With asynchronous global->LDS copies in a loop the compiler waits for ALL outstanding LDS reads
// (lgkmcnt(0)) before every use and reads only a little ahead, which leaves the matrix cores idle for an
// LDS round trip every few MFMAs.  The kernels therefore issue their ds_read_b128 themselves and wait with
// exact counts (LDS reads return in order): lds_read<OFF>(addr) starts a read, lgkm_wait<N>(regs...)
// blocks until at most N later reads are outstanding and ties the named registers to that point so no use
// of them can be moved above it.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ unsigned lds_offset_of(const void* p) {
  return (unsigned)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}
template <int OFF>
__device__ __forceinline__ u32x4 lds_read(unsigned addr) {
  static_assert(OFF >= 0 && OFF < 65536, "ds_read offset is 16 bits");
  u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x4& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x4& a, u32x4& b, u32x4& c) {
  asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(N));
}
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N>
__device__ __forceinline__ void lgkm_wait(u32x4& a, u32x4& b, u32x4& c, u32x4& d, u32x4& e, u32x4& f) {
  asm volatile("s_waitcnt lgkmcnt(%6)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e), "+v"(f) : "n"(N));
}
__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Registers 8t..8t+7 of a 32x32 accumulator tile, rounded RNE to bf16: a chain-order frag.
__device__ __forceinline__ bf16x8 pack_chain(const f32x16& c, int t) {
  bf16x8 r;
#pragma unroll
  for (int s = 0; s < 8; ++s) r[s] = (__bf16)c[8 * t + s];
  return r;
}

__device__ __forceinline__ float silu_f32(float x) { return x / (1.0f + __expf(-x)); }

// XCD-aware block numbering: consecutive hardware block ids go round-robin over the 8 XCDs, so XCD x runs blocks
// x, x + 8, ...: n / 8 of them, one more if x < n % 8.  The logical id numbers an XCD's blocks consecutively, after
// those of the XCDs before it, which puts a contiguous range of logical ids on one XCD (and its private L2).
__device__ __forceinline__ int xcd_contiguous_id(int hw, int n) {
  const int q = n / 8, rem = n % 8, x = hw % 8;
  return x * q + (x < rem ? x : rem) + hw / 8;
}
#endif

// ---- host-side plan -------------------------------------------------------------------------
struct Plan {
  // extents.  bf16: r and rd are the ranks the kernels run with: the given ranks (r_in, rd_in) rounded up to what the
  // tiles take, the added factor columns / rows being zeros in the re-tiled copies
  int64_t max_M, d, ffn, r, rd;
  int64_t r_in, rd_in;
  int64_t ffn_in;   // gated bf16: ffn likewise runs rounded up to a multiple of 256 (zero columns of Vg, Vu, zero rows of Ud)
  int kind, dtype;
  uint32_t flags;
  // bf16: byte offsets into the workspace (all 256-byte aligned)
  size_t off_wU, off_wVg, off_wVu, off_wUd, off_wVd;  // re-tiled factors
  size_t off_T, off_Tdp, off_Td, off_H, off_Hfull, off_part, off_cnt;
  size_t total_bytes;
  int64_t Mpad;       // max_M rounded up to 256
  int64_t part_rows;  // rows reserved for split-K partial sums of Td
  size_t part_bytes;  // bytes of the partial-sum buffer at off_Tdp
  // f32: element offsets
  size_t f32_T, f32_H, f32_Td;
};

int make_plan(const svdmlp_desc* desc, Plan* plan);  // returns a status code

// number of ffn splits the tiled path uses for a given number of 128-row tiles
int tiled_splits(int64_t mtiles128, int64_t nchunks);
// extents the staged tiled path (gemm.hip) handles
bool staged_supported(int64_t rd, int64_t ffn);

// ---- the planner's choices per stage of the tiled path (planner.hip) -----------------------------
enum { FIRST_S1 = 1, FIRST_IN = 2 };   // first product on 128 x 128 tiles (k_s1) or 256 x 256 tiles (k_in)
enum { OUT_256 = 1, OUT_128 = 2 };     // last product on 256 x 256 tiles (k_out) or 128 x 128 tiles (k_s5)
// A caller's override of the choices (svdmlp_force_plan); 0 = leave it to the planner.
struct PlanForce { int first_kernel, first_ranges, down_ranges, out_kernel; };
struct StageChoice { int kernel, ranges; double est_us; };
// One candidate of a stage with the time the cost model gives it; valid = the kernels take it at these extents.
struct StageCandidate { int kernel, ranges; double est_us; bool valid; };
bool first_valid(int kernel, int S, int64_t M, int64_t d, int64_t ncols);
bool down_valid(int splits, int64_t mt256, int64_t qt, int64_t nsteps);
// ncols = rank columns of the first product (2 r gated, r linear); small_only: kind LINEAR with SVDMLP_FLAG_TILE_128
int first_candidates(int64_t M, int64_t d, int64_t ncols, StageCandidate* out, int cap);
StageChoice choose_first(int64_t M, int64_t d, int64_t ncols, bool small_only, const PlanForce* f);
int down_candidates(int64_t M, int64_t rd, int64_t ffn, StageCandidate* out, int cap);
StageChoice choose_down(int64_t M, int64_t rd, int64_t ffn, const PlanForce* f);
// n = row length of the output, k = its contraction length
int out_candidates(int64_t M, int64_t n, int64_t k, StageCandidate* out, int cap);
StageChoice choose_out(int64_t M, int64_t n, int64_t k, bool small_only, const PlanForce* f);
constexpr int MAX_FIRST_RANGES = 8, MAX_DOWN_RANGES = 32;

// ---- launchers (each returns hipError_t as int; 0 = success) ---------------------------------
struct Ctx;
int f32_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
int bf16_repack_all(const Ctx* c, hipStream_t st);
// schedule of k_gate_up: XCD grid (mx row tiles per XCD, ngm row groups; 0 = plain order), persistent workgroups G,
// tiles run as full 256-row tiles (nfull) and leftover tiles run as two 128-row halves each (rem, if halves)
struct GuPlan { int mx, ngm, ntiles, G, nfull, rem; bool halves; };
GuPlan gate_up_plan(int MT256, int64_t ffn, int64_t r, int ncu);
int launch_gate_up(const Ctx* c, int MT256, hipStream_t st);
int launch_down1(const Ctx* c, int MT256, int splits, hipStream_t st);
int launch_out(const Ctx* c, int64_t M, void* Y, int MT256, hipStream_t st);
// kind LINEAR with SVDMLP_FLAG_TILE_128: k_s1 and k_s5 whatever the row count
inline bool linear_on_small_tiles(const Plan& p) { return p.kind == SVDMLP_LINEAR && (p.flags & SVDMLP_FLAG_TILE_128) != 0; }
int bf16_tiled_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
int launch_reduce(const Ctx* c, const float* part, char* out, int splits, int MT32, int nq, hipStream_t st);
int launch_in(const Ctx* c, const void* X, int64_t M, int64_t ncols, int64_t r_strip, int S, hipStream_t st);
int bf16_linear_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
int launch_out_generic(const Ctx* c, const char* act, const char* w, int64_t M, void* Y, int MT256, int64_t n, int64_t k,
                       hipStream_t st);
// Counter area of the streaming paths: [0, 32 KiB) tickets, completion counters and the error word of the one-kernel
// variant, then its 3 x 256 flag lines, then the tickets of the four-launch variant, one 128-byte line each (tickets
// that share a line are served one after the other): 2048 for D1, 2048 for D4.
constexpr size_t CNT_ONE_KERNEL_BYTES = 32768 + 3 * 256 * 128;
constexpr int TICKET_STRIDE = 32;   // ints
constexpr size_t CNT_BYTES = CNT_ONE_KERNEL_BYTES + 2 * 2048 * TICKET_STRIDE * 4;
constexpr int STREAM_MAX_M = 128;
// workgroup-level contraction ranges of a streaming-path phase with `tiles` output tiles, KB contraction blocks, rt row tiles
int stream_splits(int tiles, int KB, int rt);
int stream_row_groups(int rt, int tiles, int KB, bool first);   // first: phase D1 (else D4)
int stream_row_groups_whole(int rt, int tiles);
bool stream_last_uses_tile16(bool tile16, int tiles32);   // the last product on 16-column tiles as well
int stream_splits16(int tiles, int KB2, int mt);
int stream_tiles16(int64_t M);
bool stream_uses_tile16(int64_t M, int64_t d, int64_t ffn, int64_t r, int64_t rd);   // rows the weight-streaming path takes (four 32-row tiles)
bool stream_supported(const Plan& p, int64_t M);   // rows and ticket capacity the weight-streaming path takes
int bf16_stream_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
// ... with T, H, Td, the partial tiles and the tickets in the library's static device array (stream.hip)
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)16 << 20;
int static_scratch_resolve(int device, char** out);            // hipError_t as int; once per device, at create
size_t stream_static_scratch_need(const Plan& p, int64_t M);  // bytes of the array a forward of M rows takes
int bf16_stream_forward_static(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
int bf16_linear_stream_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
bool linear_stream_pays(int64_t M, int64_t d, int64_t r, int64_t n);
int bf16_decode_forward(const Ctx* c, const void* X, int64_t M, void* Y, hipStream_t st);
bool bf16_decode_supported(const Ctx* c, int64_t M);
char* decode_error_word(const Ctx* c);   // device address of the sticky error word of the one-kernel variant

// Optional per-kernel timing: HIP events recorded on the caller's stream around every kernel launch of
// a forward (only while a profile is open; see svdmlp_profile_begin in svdmlp.h).
constexpr int PROF_MAXK = 8;
struct Prof {
  int cap = 0;                 // forwards the event pool can hold
  int nfwd = 0;                // forwards recorded so far
  int nk = 0;                  // kernels per forward (set by the path that runs)
  hipEvent_t* ev = nullptr;    // [cap][PROF_MAXK][2]
  const char* names[PROF_MAXK] = {};
};

struct Ctx {
  svdmlp_desc desc;
  Plan plan;
  char* ws;
  int last_hip_error;
  int last_path;
  int n_cus = 0;                                 // compute units of the device the context was created on
  int device = -1;                               // ... and its ordinal
  char* static_scratch = nullptr;                // that device's copy of the library's static scratch array
  PlanForce force = {0, 0, 0, 0};                // svdmlp_force_plan
  int poll_limit = -1;                           // svdmlp_debug_set_poll_limit (-1: the kernel's own bound)
  bool ran_one_kernel = false;                   // a forward took the one-kernel streaming variant (svdmlp_check)
  mutable Prof prof;
};

// Bracket one kernel launch with events when a profile is open.  `slot` is the forward's index in the
// pool (or -1); k is the kernel's position in the forward.
inline int prof_open_forward(const Ctx* c, int nk, const char* const* names) {
  Prof& p = c->prof;
  if (!p.ev || p.nfwd >= p.cap) return -1;
  p.nk = nk;
  for (int i = 0; i < nk; ++i) p.names[i] = names[i];
  return p.nfwd++;
}
inline void prof_mark(const Ctx* c, int slot, int k, int end, hipStream_t st) {
  if (slot >= 0) (void)hipEventRecord(c->prof.ev[(slot * PROF_MAXK + k) * 2 + end], st);
}

}  // namespace svdmlp
