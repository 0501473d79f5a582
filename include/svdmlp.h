/*
 * svdmlp.h — C ABI of the fused SVD-factored MLP forward for AMD MI355X (gfx950).
 *
 * The library evaluates, for a gated MLP block whose gate / up / down weights
 * are rank-r factor pairs (paper Alg. 2 "SVD-compressed MLP layer", with the
 * on-chip SiLU-gate epilogue of Alg. 3):
 *
 *     Y = ( ( SiLU( (X Ug) Vg )  .*  ( (X Uu) Vu ) ) Ud ) Vd
 *
 * and, as kind LINEAR, the single fused low-rank linear layer the MLP kernels
 * are derived from (paper Sec. 4.2.1, "XUV NKI kernel"; block form Eq. 1):
 *
 *     O = (X U) V
 *
 * Shapes follow the "Require" line of Alg. 2 (paper names K = d, N = ffn,
 * r2 = r_down):  X[M,d]  Ug,Uu[d,r]  Vg,Vu[r,ffn]  Ud[ffn,r_down]
 * Vd[r_down,d]  Y[M,d].  LINEAR uses Ug as U[d,r] and Vg as V[r,ffn] and
 * produces O[M,ffn]; the other four factor pointers are ignored.
 *
 * Everything is dense row-major (leading dimension = number of columns).
 * All data pointers are DEVICE pointers on the current HIP device, 16-byte
 * aligned; they are borrowed, never owned or freed by the library.
 *
 * Plain C: no C++ types and no exceptions cross this boundary.
 */
#ifndef SVDMLP_H
#define SVDMLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct svdmlp_ctx svdmlp_ctx; /* opaque; host memory only */

/* Storage type of X, the six factors and Y.
 *   BF16: bf16 in HBM, fp32 accumulation on the matrix cores, intermediates
 *         (the rank-r strips T and Td, the ffn-wide activation H) and Y rounded to
 *         bf16 round-to-nearest-even, mirroring the paper's 16-bit cached strip
 *         with 4-byte accumulation (Sec. 2.2 "Matmul tiling", Sec. 4.2.1 "Caching").
 *         The MFMA-tiled path in its default (staged) variant rounds once more:
 *         SiLU(G) to bf16 before it is multiplied by the up product (the squashed
 *         gate tile waits in 16-bit pairs while the up tile takes its registers);
 *         the fused tiled variant and the weight-streaming path form SiLU(G) * P
 *         in fp32.  So one context's results for M <= 128 and M > 128 differ by
 *         up to that rounding (about 2^-9 relative per element of H).
 *   F32 : debug path, fp32 storage and fp32 arithmetic everywhere, no matrix cores. */
enum { SVDMLP_BF16 = 0, SVDMLP_F32 = 1 };

/* GATED: Alg. 2.  LINEAR: the single factored layer O = (X U) V of Sec. 4.2.1.
 * bf16 extents: d a multiple of 128, for LINEAR ffn as well (else SVDMLP_UNSUPPORTED from svdmlp_create; F32 takes any);
 * for GATED ffn is free (it is internal: the re-tiled factors carry it rounded up to a multiple of 256).  Ranks are free
 * (1 <= r, r_down <= min(d, ffn)): the library's re-tiled copies of the factors carry the rank rounded up to what its
 * tiles take (r: a multiple of 64, at least 128, LINEAR: a multiple of 128; r_down: a multiple of 256, or 128 / 256 /
 * 512 / a multiple of 512 where the fused tiled variant runs) with zero columns and rows, which changes no result but
 * costs the time and the workspace of the rounded-up rank: block-aligned ranks (the rank rule of Sec. 4.1) lose nothing. */
enum { SVDMLP_GATED = 0, SVDMLP_LINEAR = 1 };

/* Status codes (0 = success, negative = failure). */
enum {
  SVDMLP_OK = 0,
  SVDMLP_INVALID_ARGUMENT = -1,   /* null pointer, non-positive extent, M > max_M, misaligned pointer, r > min(d,ffn) */
  SVDMLP_UNSUPPORTED = -2,        /* dtype / kind / extent combination the kernels do not cover */
  SVDMLP_WORKSPACE_TOO_SMALL = -3,
  SVDMLP_HIP_ERROR = -4,          /* a HIP runtime call failed; see svdmlp_last_hip_error */
  SVDMLP_NO_DEVICE = -5,          /* no HIP device, or the current device is not gfx950 */
  SVDMLP_SCRATCH_TOO_SMALL = -6,  /* svdmlp_forward_static_scratch: the extents need more than the static array holds */
  SVDMLP_OUT_OF_HOST_MEMORY = -7, /* a host allocation failed (context, event pool) */
  SVDMLP_TIMED_OUT = -8           /* svdmlp_check: a bounded wait inside the one-kernel streaming variant ran out */
};

/* Bits of svdmlp_desc.flags (testing and benchmarking aids; 0 = automatic choice). */
enum {
  SVDMLP_FLAG_FORCE_TILED = 1u << 0,    /* bf16: always take the MFMA-tiled (prefill) path (both kinds) */
  SVDMLP_FLAG_FORCE_STREAM = 1u << 1,   /* bf16: always take the weight-streaming (decode) path; needs M <= 128 */
  SVDMLP_FLAG_SKIP_ARCH_CHECK = 1u << 2,/* do not require gfx950 (host-only unit tests of argument handling) */
  SVDMLP_FLAG_STREAM_ONE_KERNEL = 1u << 3,/* weight-streaming path as one kernel that works through a queue of tiles
                                           instead of four launches (used when M <= 32 and the extents fit its
                                           per-wave register budget); slower than the four launches as measured */
  SVDMLP_FLAG_TILED_FUSED = 1u << 4,    /* MFMA-tiled path: keep the gated activation in registers (one fused kernel)
                                           instead of staging it through the workspace */
  SVDMLP_FLAG_TILE_128 = 1u << 5,       /* kind LINEAR: both products on 128 x 128 tiles whatever the planner would pick
                                           (the small-block point of a block-size comparison, paper Table 3) */
  SVDMLP_FLAG_PLAN_ROOM = 1u << 6       /* size the workspace for every candidate of the planner, not only its choices,
                                           so that svdmlp_force_plan can run any of them (tuning and tests; the
                                           split-K partial buffers grow to 8 / 32 ranges) */
};

typedef struct {
  int32_t kind;             /* SVDMLP_GATED or SVDMLP_LINEAR */
  int32_t dtype;            /* SVDMLP_BF16 or SVDMLP_F32 */
  int64_t max_M;            /* largest row count svdmlp_forward will be called with (sizes the workspace) */
  int64_t d, ffn, r, r_down;/* extents; r_down is the rank of the down projection (ignored for LINEAR) */
  const void *Ug, *Vg;      /* gate factors [d,r], [r,ffn]   (LINEAR: U and V) */
  const void *Uu, *Vu;      /* up factors   [d,r], [r,ffn] */
  const void *Ud, *Vd;      /* down factors [ffn,r_down], [r_down,d] */
  void *workspace;          /* device memory, caller-owned, 256-byte aligned, >= svdmlp_workspace_bytes() */
  size_t workspace_bytes;
  uint32_t flags;
} svdmlp_desc;

/* Bytes of device workspace a context for this description needs.  Pure host function (touches no
 * device).  Returns 0 if the description is invalid or unsupported (svdmlp_create reports why).
 * For BF16 the workspace holds a one-time re-tiled copy of the six factors (the weights are
 * invariant at inference time, paper Sec. 2.1, so they are laid out once for the matrix cores),
 * the rank-r intermediates, split-K partial sums and a few counters.  For F32 it holds the fp32
 * intermediates including the ffn-wide activation. */
size_t svdmlp_workspace_bytes(const svdmlp_desc *desc);

/* Validate the description, lay the factors out in the workspace (BF16: device work on the NULL
 * stream, completed before returning) and return a context in *out.  *out is written only on
 * success.  The factor buffers must stay valid and unchanged until svdmlp_destroy for F32; for
 * BF16 they are not read again after create returns.  The workspace belongs to the context until
 * svdmlp_destroy. */
int svdmlp_create(const svdmlp_desc *desc, svdmlp_ctx **out);

/* Enqueue Y = MLP(X) (or O = (X U) V) for the first M rows on hip_stream (a hipStream_t passed as
 * void*; NULL = the default stream).  X is [M,d]; Y is [M,d] (LINEAR: [M,ffn]); both of the context's
 * dtype, row-major, 16-byte aligned device pointers; Y must not alias X.  Never synchronises with
 * the host and allocates nothing.  1 <= M <= max_M; M == 0 is accepted and does nothing.  At most one
 * forward per context may be in flight at a time (the workspace holds its intermediates), so
 * successive calls must be ordered on one stream or by events.  The call only launches kernels (no memset, no
 * copy), so it may be recorded into a HIP graph by stream capture (not while a per-kernel profile is open). */
int svdmlp_forward(svdmlp_ctx *ctx, const void *X, int64_t M, void *Y, void *hip_stream);

/* svdmlp_forward for callers that cannot allocate device memory for intermediates and cannot hand the library a
 * buffer for them per call: code recorded under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation once they run.  Same arguments, result and rules as svdmlp_forward, restricted to BF16 GATED contexts and
 * 1 <= M <= 128 (the weight-streaming path; anything else returns SVDMLP_UNSUPPORTED), but every per-forward buffer
 * (rank-r strips, the ffn-wide activation of the call's rows, split-K partial tiles, arrival tickets) lives in a
 * static device array inside the library, svdmlp_static_scratch_bytes() = 16 MiB per GPU, instead of the context's
 * workspace; the workspace is only read (the re-tiled factors).  The call allocates nothing, makes no memset and no
 * copy, and only launches kernels (one more than svdmlp_forward: it clears the tickets).  The array's device address
 * was looked up by svdmlp_create; the current device must be the one the context was created on
 * (SVDMLP_INVALID_ARGUMENT otherwise).  Extents whose buffers do not fit, 8.5 MiB + 128-row-padded T, H and Td, i.e.
 * roughly rows * (2 r + ffn + r_down) * 2 bytes > 7.5 MiB with rows = 32, 64 or 128, return SVDMLP_SCRATCH_TOO_SMALL
 * and launch nothing.  Every GPU holds one such array until the process ends, shared by all contexts and callers on
 * it: two of these calls that overlap in time on one GPU (different streams, different contexts) race; order them. */
int svdmlp_forward_static_scratch(svdmlp_ctx *ctx, const void *X, int64_t M, void *Y, void *hip_stream);

/* Size in bytes of that static array (host only). */
size_t svdmlp_static_scratch_bytes(void);

/* The one-kernel streaming variant (SVDMLP_FLAG_STREAM_ONE_KERNEL) waits inside the kernel, with a bound; if a wait
 * runs out, the workgroups stop computing, the output rows of that forward are filled with NaN, and an error word in the
 * workspace is set.  svdmlp_check reads that word (a synchronous 4-byte copy from the device: call it after the
 * forward's stream has been synchronised, never under graph capture) and clears it: SVDMLP_OK, SVDMLP_TIMED_OUT, or
 * SVDMLP_HIP_ERROR if the copy fails.  Contexts that never ran that variant return SVDMLP_OK without touching the
 * device. */
int svdmlp_check(svdmlp_ctx *ctx);

/* Testing aid for that error path: the number of polls a wait inside the one-kernel variant may take before it gives
 * up (-1 = the kernel's own bound, about a million).  With 0 every wait that is not already satisfied gives up at
 * once, so the kernel still ends normally, on its error path, without anything having to hang. */
int svdmlp_debug_set_poll_limit(svdmlp_ctx *ctx, int32_t polls);

/* Release the context's host memory.  Does not free or touch device memory; the caller must make
 * sure no forward is still running.  svdmlp_destroy(NULL) returns SVDMLP_OK. */
int svdmlp_destroy(svdmlp_ctx *ctx);

/* Static, never-NULL description of a status code. */
const char *svdmlp_status_string(int status);

/* Host only, no device needed: writes into buf (NUL-terminated, at most buf_bytes) one line that names the path a
 * forward of M rows on a context of this description takes, its kernels in launch order and how each is cut over
 * the chip (tile shape, number of tiles, contraction ranges, persistent workgroups), and for every stage that leaves a
 * choice the time the planner's cost model gives the chosen candidate (est_us) and the closest alternatives
 * (kernel/ranges=microseconds): the planner's counterpart of the block-size choice of the paper's Sec. 4.2.2,
 * evaluated for a 256-CU device.  Returns SVDMLP_OK, the status
 * svdmlp_create would return for desc (the workspace fields are not looked at), or SVDMLP_INVALID_ARGUMENT if M is not
 * in 1..max_M or the line does not fit. */
int svdmlp_describe(const svdmlp_desc *desc, int64_t M, char *buf, size_t buf_bytes);

/* Override the planner for later forwards of this context on the MFMA-tiled path (bf16 only): the counterpart of
 * trying another block size in the paper's Table 3.  0 leaves a choice to the planner.
 *   first_kernel : 1 = first product on 128 x 128 tiles (k_s1), 2 = on 256 x 256 tiles (k_in)
 *   first_ranges : ranges its contraction over d is cut into, 1 .. 8 (needs first_kernel)
 *   down_ranges  : ffn ranges of the first phase of the down projection (k_down1), 1 .. 32
 *   out_kernel   : 1 = last product on 256 x 256 tiles (k_out), 2 = on 128 x 128 tiles (k_s5)
 * A candidate the kernels cannot run at a forward's extents (svdmlp_describe lists the valid ones) falls back to the
 * planner's choice; one whose partial sums do not fit the workspace makes svdmlp_forward return SVDMLP_HIP_ERROR
 * (create the context with SVDMLP_FLAG_PLAN_ROOM to have room for all).  Returns SVDMLP_OK, SVDMLP_INVALID_ARGUMENT
 * (values out of range) or SVDMLP_UNSUPPORTED (fp32 context). */
int svdmlp_force_plan(svdmlp_ctx *ctx, int32_t first_kernel, int32_t first_ranges, int32_t down_ranges, int32_t out_kernel);

/* The hipError_t (as int) of the last failing HIP call made for this context (0 if none). */
int svdmlp_last_hip_error(const svdmlp_ctx *ctx);

/* Which path the last svdmlp_forward on this context took: 0 none yet, 1 fp32 debug,
 * 2 bf16 MFMA-tiled (prefill) with the gated activation kept in registers (SVDMLP_FLAG_TILED_FUSED, or chosen by the
 * library when r and r_down are both at most 128),
 * 3 bf16 weight-streaming (decode; the default for M <= 128) as four launches, 4 bf16 weight-streaming as one persistent kernel (SVDMLP_FLAG_STREAM_ONE_KERNEL), 5 bf16
 * MFMA-tiled with the gated activation staged through the workspace (the default for M > 128), 6 bf16 single
 * factored layer (SVDMLP_LINEAR) MFMA-tiled, 7 bf16 single factored layer weight-streaming (the default for M <= 128). */
int svdmlp_last_path(const svdmlp_ctx *ctx);

/* Per-kernel timing for benchmarks.  svdmlp_profile_begin creates a pool of HIP events for up to
 * max_forwards forwards (host allocation; not to be called under graph capture); while the profile is
 * open every svdmlp_forward on this context records an event before and after each of its kernels on
 * the stream it launches on (forwards beyond max_forwards are not recorded).  svdmlp_profile_end waits
 * for the recorded events, writes the average duration in milliseconds of each kernel position into
 * avg_ms[0 .. *n_kernels) (capacity 8) and the number of forwards averaged into *n_forwards, then
 * releases the pool.  svdmlp_profile_kernel_name returns the name of kernel position k of the last
 * recorded forward (NULL if out of range); valid until the context is destroyed. */
int svdmlp_profile_begin(svdmlp_ctx *ctx, int max_forwards);
int svdmlp_profile_end(svdmlp_ctx *ctx, float *avg_ms, int *n_kernels, int *n_forwards);
const char *svdmlp_profile_kernel_name(const svdmlp_ctx *ctx, int k);

/* Host only: the rank that the paper's rule (Sec. 4.1, Eq. 5) gives a k x n weight matrix for a target compression
 * ratio (the fraction of the k n parameters removed, 0 <= ratio < 1), snapped to a multiple of `block`:
 *     r = floor( k n (1 - ratio) / ((k + n) block) + alpha ) * block,   at least one block
 * (alpha = 0.5 rounds to the nearest block; the paper uses blocks that are a multiple of its tile size, here a
 * multiple of 128 costs nothing, see the rank rounding above).  Returns -1 for non-positive extents or block, a ratio
 * outside [0, 1) or alpha outside [0, 1]. */
int64_t svdmlp_rank_for_ratio(int64_t k, int64_t n, double ratio, int64_t block, double alpha);

/* Roof microbenchmarks: kernels that do one thing only, so that a benchmark can print what this machine delivers
 * beside the published peaks.  Each call only enqueues one kernel on hip_stream (NULL = default stream); the caller
 * times it (events on that stream) and owns all buffers (device pointers).  They return SVDMLP_OK,
 * SVDMLP_INVALID_ARGUMENT or SVDMLP_HIP_ERROR.
 *   svdmlp_roof_read : `workgroups` workgroups of 256 lanes stream the first bytes / 32768 * 32768 bytes of buf
 *                      (16-byte aligned, at least 32 KiB; use more than the 256 MB memory-side cache) with 16-byte
 *                      loads, eight per lane in flight; sink is 4 bytes that are never written for a buffer filled
 *                      with one repeated byte.  HBM GB/s = bytes read / time.
 *   svdmlp_roof_mfma : `workgroups` workgroups of eight waves, each wave issuing 4 * iters
 *                      v_mfma_f32_32x32x16_bf16 on register operands (four independent accumulators).
 *                      FLOP = workgroups * 8 * 4 * iters * 32768; sink is 4 bytes, never written.
 *   svdmlp_roof_mfma_operands: the same kernel with a choice of operand VALUES, because the sustained clock of the
 *                      matrix cores depends on how many operand bits toggle: operands = 0 all zero, 1 a few small
 *                      values repeating over the lanes (what svdmlp_roof_mfma uses), 2 pseudo-random values uniform
 *                      in (-1, 1), different in every lane.  The last one is the roof for a product of real data.
 *   svdmlp_roof_pingpong: the phase skeleton of the 256 x 256 tile kernels with nothing to copy: `workgroups`
 *                      workgroups of eight waves, the two waves of a SIMD alternating between reading twelve operand
 *                      frags from LDS and sixteen MFMAs, two barriers per step, `steps` steps; LDS filled once with
 *                      operands as above (0 zeros, 1 few values, 2 random).  FLOP = workgroups * 8 * 16 * steps * 32768;
 *                      sink is 4 bytes, never written.
 *   svdmlp_roof_coexec: eight waves per workgroup; waves 0..3 issue 2 * mfma_iters MFMAs each, their SIMD partners
 *                      4..7 evaluate SiLU on 32 registers per lane valu_iters times.  With either count 0 that half
 *                      idles: three launches show whether vector-ALU work hides under the partner's MFMAs.
 *                      sink is 8 bytes, never written.
 *   svdmlp_roof_empty: a kernel of `workgroups` x `threads` that does nothing (chains of dependent launches).
 *   svdmlp_roof_empty_chain: `launches` such kernels enqueued back to back from one call (no caller overhead between
 *                      them): what a dependent launch costs on the device. */
int svdmlp_roof_read(const void *buf, size_t bytes, void *sink, int workgroups, void *hip_stream);
int svdmlp_roof_mfma(int iters, void *sink, int workgroups, void *hip_stream);
int svdmlp_roof_mfma_operands(int iters, int operands, void *sink, int workgroups, void *hip_stream);
int svdmlp_roof_pingpong(int steps, int operands, void *sink, int workgroups, void *hip_stream);
int svdmlp_roof_coexec(int mfma_iters, int valu_iters, void *sink, int workgroups, void *hip_stream);
int svdmlp_roof_empty(int workgroups, int threads, void *hip_stream);
int svdmlp_roof_empty_chain(int launches, int workgroups, int threads, void *hip_stream);

/* ABI version of this header (bumped on any incompatible change). */
int svdmlp_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SVDMLP_H */
