// Roof microbenchmarks (gfx950): what this machine actually delivers for the three things the forward is bounded by,
// measured with kernels that do nothing else.  The benchmark prints them beside the published peaks, so that every
// "fraction of the roof" can be read against a measured roof as well.
//   read   : every lane streams 16-byte loads over a buffer (larger than the 256 MB memory-side cache) -> HBM GB/s
//   mfma   : every wave issues v_mfma_f32_32x32x16_bf16 on register-resident operands, four independent accumulators
//            -> matrix-core TFLOP/s at the clock the chip sustains under that load.  The clock is power-limited and
//            the power of the matrix cores depends on how many operand bits toggle, so the rate depends on the
//            VALUES: all-zero operands run at the full clock, operands drawn like activations and weights (uniform
//            in (-1, 1), every mantissa bit alive) about 30 % slower.  The second figure is the roof a GEMM on real
//            data can reach on this machine.
//   pingpong: the phase skeleton of the 256 x 256 tile kernels (gemm.hip) with nothing to copy: eight waves, the two
//            of a SIMD alternating between a phase that reads twelve operand frags from LDS and a phase of sixteen
//            MFMAs, two workgroup barriers per step, LDS filled once at the start (zeros, a few values, or random).
//            What this reaches is what barriers, LDS reads and the matrix cores' power leave of the peak before a
//            single byte is fetched.
//   empty  : a kernel that does nothing, for timing chains of dependent launches (the floor of a forward that is a
//            sequence of short kernels, as the weight-streaming path is)
#include "common.h"

namespace svdmlp {

constexpr int ROOF_READ_UNROLL = 8;

__global__ __launch_bounds__(256) void k_roof_read(const u32x4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
  // workgroup b reads blocks b, b + gridDim.x, ... of 256 x ROOF_READ_UNROLL x 16 bytes, each lane 16 bytes per load,
  // a wave 1 KiB contiguous per load, all loads of a block in flight before the first use
  const size_t per_block = (size_t)256 * ROOF_READ_UNROLL;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t base = (size_t)blockIdx.x * per_block; base + per_block <= n16; base += (size_t)gridDim.x * per_block) {
    u32x4 v[ROOF_READ_UNROLL];
#pragma unroll
    for (int u = 0; u < ROOF_READ_UNROLL; ++u) v[u] = __builtin_nontemporal_load(src + base + (size_t)u * 256 + threadIdx.x);
#pragma unroll
    for (int u = 0; u < ROOF_READ_UNROLL; ++u) acc ^= v[u];
  }
  // never true for the buffers the benchmark passes (filled with a constant pattern); keeps the loads alive
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) sink[0] = acc[0];
}

// operands: 0 all zero, 1 a few small values that repeat over the lanes (few bits toggle), 2 pseudo-random values
// uniform in (-1, 1), different in every lane, wave and workgroup
template <int operands>   // a template parameter so that a kernel trace names the operand set
__global__ __launch_bounds__(512) void k_roof_mfma(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x % 64;
  bf16x8 a0, a1, b0, b1;
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    float x0 = 0.f, x1 = 0.f, y0 = 0.f, y1 = 0.f;
    if (operands == 1) {
      x0 = x1 = 0.001f * (float)((lane + s) % 7);
      y0 = y1 = 0.002f * (float)((lane * 3 + s) % 5);
    } else if (operands == 2) {
      unsigned h = ((unsigned)blockIdx.x * 512u + threadIdx.x) * 8u + (unsigned)s + 1u;
      float u[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {  // four rounds of an integer hash, one value each
        h *= 2654435761u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        u[q] = (float)(int)h * (1.0f / 2147483648.0f);
      }
      x0 = u[0]; x1 = u[1]; y0 = u[2]; y1 = u[3];
    }
    a0[s] = (__bf16)x0; a1[s] = (__bf16)x1; b0[s] = (__bf16)y0; b1[s] = (__bf16)y1;
  }
  f32x16 c0, c1, c2, c3;
#pragma unroll
  for (int e = 0; e < 16; ++e) { c0[e] = 0.f; c1[e] = 0.f; c2[e] = 0.f; c3[e] = 0.f; }
  for (int i = 0; i < iters; ++i) {
    c0 = mfma32(a0, b0, c0);
    c1 = mfma32(a1, b0, c1);
    c2 = mfma32(a0, b1, c2);
    c3 = mfma32(a1, b1, c3);
  }
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
  if (s == -1.0f) sink[0] = s;   // keeps the accumulators alive; the sums are not -1 for any of the three operand sets
}

// Waves 0..3 of a workgroup (one per SIMD) issue MFMAs as in k_roof_mfma; waves 4..7, their SIMD partners, evaluate
// SiLU (multiply, exp2, add, reciprocal, multiply: two of the five on the transcendental unit) on 32 registers per
// lane, round after round.  Either half can be switched off, so three launches tell whether vector-ALU work of one
// wave runs under the MFMAs of the other wave of its SIMD.
__global__ __launch_bounds__(512) void k_roof_coexec(int mfma_iters, int valu_iters, float* __restrict__ sink) {
  const int lane = threadIdx.x % 64, w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  if (w < 4) {
    bf16x8 a, b;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      a[s] = (__bf16)(0.001f * (float)((lane + s) % 7));
      b[s] = (__bf16)(0.002f * (float)((lane * 3 + s) % 5));
    }
    f32x16 c0, c1;
#pragma unroll
    for (int e = 0; e < 16; ++e) { c0[e] = 0.f; c1[e] = 0.f; }
    for (int i = 0; i < mfma_iters; ++i) {
      c0 = mfma32(a, b, c0);
      c1 = mfma32(a, b, c1);
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c0[e] + c1[e];
    if (s == -1.0f) sink[0] = s;
  } else {
    float g[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) g[e] = 0.01f * (float)(lane + e);
    for (int i = 0; i < valu_iters; ++i) {
#pragma unroll
      for (int e = 0; e < 32; ++e)
        g[e] = g[e] * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g[e] * -1.44269504088896f)) + 0.25f;
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 32; ++e) s += g[e];
    if (s == -1.0f) sink[1] = s;
  }
}

// The phase skeleton of gemm.hip on LDS-resident operands (see the list at the top).  Wave w owns rows 128 (w / 4)..
// and columns 64 (w % 4).. of a 256 x 256 tile; a step is two contraction blocks; four 32 KiB slots are read in turn.
template <int operands>
__global__ __launch_bounds__(512) void k_roof_pingpong(int steps, float* __restrict__ sink) {
  __shared__ __attribute__((aligned(1024))) char lds[4 * 32 * FRAG_BYTES];
  const int lane = threadIdx.x % 64, w = __builtin_amdgcn_readfirstlane(threadIdx.x / 64);
  const int wm = w / 4, wn = w % 4;
  for (int i = threadIdx.x; i < 4 * 32 * FRAG_BYTES / 4; i += 512) {
    unsigned v = 0u;
    if (operands == 1) v = 0x3c003c00u + (i & 0xff);
    if (operands == 2) {  // two bf16 values uniform in (-1, 1) (fp32 truncated to its upper half)
      unsigned h = (i + 1 + blockIdx.x * 32768u) * 2654435761u; h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      unsigned h2 = h * 3266489917u; h2 ^= h2 >> 16;
      const float a = (float)(int)h * (1.0f / 2147483648.0f), b = (float)(int)h2 * (1.0f / 2147483648.0f);
      v = (__builtin_bit_cast(unsigned, a) >> 16) | (__builtin_bit_cast(unsigned, b) & 0xffff0000u);
    }
    reinterpret_cast<unsigned*>(lds)[i] = v;
  }
  __syncthreads();
  const unsigned lds_off = lds_offset_of(lds);
  const unsigned rdA = lds_off + lane * 16 + 4 * wm * FRAG_BYTES, rdW = lds_off + lane * 16 + (8 + 2 * wn) * FRAG_BYTES;
  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  u32x4 A0, A1, A2, A3, Wa0, Wa1, B0, B1, B2, B3, Wb0, Wb1;
  int slot = 0;
  if (w >= 4) lds_barrier();  // second wave of each SIMD: one phase behind
  lds_barrier();
  for (int s = 0; s < steps; ++s) {
    // memory phase: the twelve frags of the step
    const unsigned aA = rdA + slot * 32 * FRAG_BYTES, aW = rdW + slot * 32 * FRAG_BYTES;
    slot = (slot + 1) & 3;
    Wa0 = lds_read<0 * FRAG_BYTES>(aW);
    Wa1 = lds_read<1 * FRAG_BYTES>(aW);
    A0 = lds_read<0 * FRAG_BYTES>(aA);
    A1 = lds_read<1 * FRAG_BYTES>(aA);
    A2 = lds_read<2 * FRAG_BYTES>(aA);
    A3 = lds_read<3 * FRAG_BYTES>(aA);
    Wb0 = lds_read<16 * FRAG_BYTES + 0 * FRAG_BYTES>(aW);
    Wb1 = lds_read<16 * FRAG_BYTES + 1 * FRAG_BYTES>(aW);
    B0 = lds_read<16 * FRAG_BYTES + 0 * FRAG_BYTES>(aA);
    B1 = lds_read<16 * FRAG_BYTES + 1 * FRAG_BYTES>(aA);
    B2 = lds_read<16 * FRAG_BYTES + 2 * FRAG_BYTES>(aA);
    B3 = lds_read<16 * FRAG_BYTES + 3 * FRAG_BYTES>(aA);
    lds_barrier();
    // compute phase
    lgkm_wait<6>(A0, A1, A2, A3, Wa0, Wa1);
    acc[0][0] = mfma32(as_bf16x8(Wa0), as_bf16x8(A0), acc[0][0]);
    acc[1][0] = mfma32(as_bf16x8(Wa1), as_bf16x8(A0), acc[1][0]);
    acc[0][1] = mfma32(as_bf16x8(Wa0), as_bf16x8(A1), acc[0][1]);
    acc[1][1] = mfma32(as_bf16x8(Wa1), as_bf16x8(A1), acc[1][1]);
    acc[0][2] = mfma32(as_bf16x8(Wa0), as_bf16x8(A2), acc[0][2]);
    acc[1][2] = mfma32(as_bf16x8(Wa1), as_bf16x8(A2), acc[1][2]);
    acc[0][3] = mfma32(as_bf16x8(Wa0), as_bf16x8(A3), acc[0][3]);
    acc[1][3] = mfma32(as_bf16x8(Wa1), as_bf16x8(A3), acc[1][3]);
    __builtin_amdgcn_sched_barrier(0);
    lgkm_wait<0>(B0, B1, B2, B3, Wb0, Wb1);
    acc[0][0] = mfma32(as_bf16x8(Wb0), as_bf16x8(B0), acc[0][0]);
    acc[1][0] = mfma32(as_bf16x8(Wb1), as_bf16x8(B0), acc[1][0]);
    acc[0][1] = mfma32(as_bf16x8(Wb0), as_bf16x8(B1), acc[0][1]);
    acc[1][1] = mfma32(as_bf16x8(Wb1), as_bf16x8(B1), acc[1][1]);
    acc[0][2] = mfma32(as_bf16x8(Wb0), as_bf16x8(B2), acc[0][2]);
    acc[1][2] = mfma32(as_bf16x8(Wb1), as_bf16x8(B2), acc[1][2]);
    acc[0][3] = mfma32(as_bf16x8(Wb0), as_bf16x8(B3), acc[0][3]);
    acc[1][3] = mfma32(as_bf16x8(Wb1), as_bf16x8(B3), acc[1][3]);
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();
  }
  if (w < 4) lds_barrier();  // matches the extra barrier of waves 4..7
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) t += acc[i][j][e];
  if (t == -1.0f) sink[0] = t;   // keeps the accumulators alive
}

__global__ void k_roof_empty(int* unused) { (void)unused; }

}  // namespace svdmlp

using namespace svdmlp;

extern "C" {

int svdmlp_roof_read(const void* buf, size_t bytes, void* sink, int workgroups, void* hip_stream) {
  if (!buf || !sink || bytes < 256 * ROOF_READ_UNROLL * 16 || workgroups <= 0 || (reinterpret_cast<uintptr_t>(buf) & 15u))
    return SVDMLP_INVALID_ARGUMENT;
  hipLaunchKernelGGL(k_roof_read, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const u32x4*>(buf), bytes / 16, static_cast<unsigned*>(sink));
  if (hipGetLastError() != hipSuccess) return SVDMLP_HIP_ERROR;
  return SVDMLP_OK;
}

int svdmlp_roof_mfma_operands(int iters, int operands, void* sink, int workgroups, void* hip_stream) {
  if (!sink || iters <= 0 || workgroups <= 0 || operands < 0 || operands > 2) return SVDMLP_INVALID_ARGUMENT;
  const dim3 grid(workgroups), block(512);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* out = static_cast<float*>(sink);
  if (operands == 0) hipLaunchKernelGGL(k_roof_mfma<0>, grid, block, 0, st, iters, out);
  else if (operands == 1) hipLaunchKernelGGL(k_roof_mfma<1>, grid, block, 0, st, iters, out);
  else hipLaunchKernelGGL(k_roof_mfma<2>, grid, block, 0, st, iters, out);
  if (hipGetLastError() != hipSuccess) return SVDMLP_HIP_ERROR;
  return SVDMLP_OK;
}

int svdmlp_roof_mfma(int iters, void* sink, int workgroups, void* hip_stream) {
  return svdmlp_roof_mfma_operands(iters, 1, sink, workgroups, hip_stream);
}

int svdmlp_roof_pingpong(int steps, int operands, void* sink, int workgroups, void* hip_stream) {
  if (!sink || steps <= 0 || workgroups <= 0 || operands < 0 || operands > 2) return SVDMLP_INVALID_ARGUMENT;
  const dim3 grid(workgroups), block(512);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  float* out = static_cast<float*>(sink);
  if (operands == 0) hipLaunchKernelGGL(k_roof_pingpong<0>, grid, block, 0, st, steps, out);
  else if (operands == 1) hipLaunchKernelGGL(k_roof_pingpong<1>, grid, block, 0, st, steps, out);
  else hipLaunchKernelGGL(k_roof_pingpong<2>, grid, block, 0, st, steps, out);
  if (hipGetLastError() != hipSuccess) return SVDMLP_HIP_ERROR;
  return SVDMLP_OK;
}

int svdmlp_roof_coexec(int mfma_iters, int valu_iters, void* sink, int workgroups, void* hip_stream) {
  if (!sink || mfma_iters < 0 || valu_iters < 0 || workgroups <= 0) return SVDMLP_INVALID_ARGUMENT;
  hipLaunchKernelGGL(k_roof_coexec, dim3(workgroups), dim3(512), 0, static_cast<hipStream_t>(hip_stream), mfma_iters,
                     valu_iters, static_cast<float*>(sink));
  if (hipGetLastError() != hipSuccess) return SVDMLP_HIP_ERROR;
  return SVDMLP_OK;
}

int svdmlp_roof_empty(int workgroups, int threads, void* hip_stream) {
  if (workgroups <= 0 || threads <= 0 || threads > 1024) return SVDMLP_INVALID_ARGUMENT;
  hipLaunchKernelGGL(k_roof_empty, dim3(workgroups), dim3(threads), 0, static_cast<hipStream_t>(hip_stream), (int*)nullptr);
  if (hipGetLastError() != hipSuccess) return SVDMLP_HIP_ERROR;
  return SVDMLP_OK;
}

int svdmlp_roof_empty_chain(int launches, int workgroups, int threads, void* hip_stream) {
  if (launches <= 0 || workgroups <= 0 || threads <= 0 || threads > 1024) return SVDMLP_INVALID_ARGUMENT;
  for (int i = 0; i < launches; ++i)
    hipLaunchKernelGGL(k_roof_empty, dim3(workgroups), dim3(threads), 0, static_cast<hipStream_t>(hip_stream), (int*)nullptr);
  if (hipGetLastError() != hipSuccess) return SVDMLP_HIP_ERROR;
  return SVDMLP_OK;
}

}  // extern "C"
