// Measurement aids: what this GPU actually sustains, measured by the same process that times the
// hot path, so that a roofline fraction can be quoted against the published peak and against the
// achievable one side by side.  Three small kernels, none on the hot path:
//   * a streaming read (16 bytes per lane, every byte consumed),
//   * a plain copy (16 bytes per lane read and written),
//   * a register-resident loop of v_mfma_f32_32x32x16_bf16, the instruction the grouped FFN is
//     built on: two A and four B operand fragments feed eight accumulators per wave, the
//     tile shape of the FFN kernel, with no memory access inside the loop.  Operands are either
//     constant or pseudo-random bf16 values (the power the matrix cores draw, and with it the
//     clock the chip sustains, depends on the data); the shader clock during the loop is read
//     from the shader clock counter against the constant 100 MHz reference counter.
#include "ew_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void k_probe_read(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;  // keeps the loads alive; practically never taken
}

__global__ __launch_bounds__(256) void k_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// One pseudo-random bf16 pair in (-2, 2) per 32-bit word: sign and mantissa random, exponent in
// {126, 127} so products and sums stay finite.
__device__ __forceinline__ uint32_t rand_bf16_pair(uint32_t seed) {
  const uint32_t r = mix(seed);
  const uint32_t lo = (r & 0x80FFu) | ((126u + ((r >> 8) & 1u)) << 7);
  const uint32_t hi = ((r >> 16) & 0x80FFu) | ((126u + ((r >> 24) & 1u)) << 7);
  return (lo & 0xFFFFu) | (hi << 16);
}

// out[4*block + {0,1}] = shader-clock ticks and reference ticks (100 MHz) of wave 0's loop;
// out[4*block + 2] = a value derived from the accumulators (keeps the loop alive).
__global__ __launch_bounds__(512) void k_probe_mfma(int iters, int random_operands, unsigned long long* __restrict__ out) {
  const uint32_t tid = blockIdx.x * 512u + threadIdx.x;
  u32x4 a[2], b[4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w) a[i][w] = random_operands ? rand_bf16_pair(tid * 64u + i * 4u + w) : 0x3F803F80u;
#pragma unroll
  for (int f = 0; f < 4; ++f)
#pragma unroll
    for (int w = 0; w < 4; ++w) b[f][w] = random_operands ? rand_bf16_pair(tid * 64u + 32u + f * 4u + w) : 0x3F803F80u;
  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][f][e] = 0.f;
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int i = 0; i < 2; ++i)
        acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[f]),
                                                            acc[i][f], 0, 0, 0);
    // Operands change a little every iteration (alternating sign of one element) so that the loop
    // cannot be folded, at one scalar-free vector instruction per eight MFMAs.
    a[0][0] ^= 0x80000000u;
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int f = 0; f < 4; ++f) s += acc[i][f][0] + acc[i][f][15];
  if (threadIdx.x == 0) {
    out[4 * (size_t)blockIdx.x + 0] = c1 - c0;
    out[4 * (size_t)blockIdx.x + 1] = r1 - r0;
    out[4 * (size_t)blockIdx.x + 2] = (unsigned long long)__float_as_uint(s);
  }
}

}  // namespace

extern "C" int ew_probe_stream(const void* src, void* dst, size_t bytes, int read_only, void* stream) {
  using ew::fail;
  if (!src || !dst || bytes == 0 || bytes % 16) return fail(EW_ERR_INVALID_ARG, "ew_probe_stream: need src, dst and a multiple of 16 bytes");
  if (((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return fail(EW_ERR_INVALID_ARG, "ew_probe_stream: buffers must be 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  const size_t n16 = bytes / 16;
  const int blocks = 256 * 16;  // 16 blocks of 4 waves per CU
  if (!read_only)
    hipLaunchKernelGGL(k_probe_copy, dim3(blocks), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n16);
  else
    hipLaunchKernelGGL(k_probe_read, dim3(blocks), dim3(256), 0, st, (const u32x4*)src, n16, (uint32_t*)dst);
  EW_LAUNCH_CHECK("k_probe_stream");
  return EW_OK;
}

extern "C" int ew_probe_mfma_bf16(int workgroups, int iters, int random_operands, unsigned long long* out, void* stream) {
  using ew::fail;
  if (workgroups < 1 || workgroups > 65536 || iters < 1 || !out) return fail(EW_ERR_INVALID_ARG, "ew_probe_mfma_bf16: bad argument");
  hipLaunchKernelGGL(k_probe_mfma, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, iters, random_operands, out);
  EW_LAUNCH_CHECK("k_probe_mfma");
  return EW_OK;
}
