// Weighted un-permute (+ shared experts) and router scores.
//
// Paper Sec. 2.1: expert outputs are weighted with the router's weights and put back into the
// original token order; the router computes g(x) over all experts.
// Both kernels are bandwidth bound: 16-byte accesses, fp32 accumulation, one pass.
#include "ew_internal.h"

namespace {

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest even (finite inputs)
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct alignas(16) U16x8 { uint16_t v[8]; };

// Sum over a block of 256 threads, in the order k_rmsnorm uses (lanes by butterfly, then the four waves in order).
__device__ __forceinline__ float block_sum_256(float v, float* s_part) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = v;
  __syncthreads();
  return s_part[0] + s_part[1] + s_part[2] + s_part[3];
}

// out[t][h] = sum_j w[t][j] * y[rop[t*k+j]][h] + sum_s shared[s][t][h] (+ residual[t][h]); one block per token.
// normed != nullptr: also normed[t] = out[t] / sqrt(mean_h out[t][h]^2 + eps), from the rounded out[t] and in
// k_rmsnorm's order of operations, so the pair equals moe_unpermute followed by moe_rmsnorm bit for bit.
__global__ __launch_bounds__(256) void k_unpermute_bf16(const uint16_t* __restrict__ y, const int32_t* __restrict__ rop,
                                                        const float* __restrict__ w, const uint16_t* __restrict__ shared,
                                                        const uint16_t* __restrict__ residual, int S, int T, int k, int H,
                                                        uint16_t* __restrict__ out, float eps, uint16_t* __restrict__ normed) {
  const int t = blockIdx.x;
  __shared__ int32_t s_row[64];
  __shared__ float s_w[64];
  __shared__ float s_part[4];
  float ss = 0.f;
  if (threadIdx.x < k) {
    s_row[threadIdx.x] = rop[(size_t)t * k + threadIdx.x];
    s_w[threadIdx.x] = w[(size_t)t * k + threadIdx.x];
  }
  __syncthreads();
  for (int h = threadIdx.x * 8; h < H; h += blockDim.x * 8) {
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j = 0; j < k; ++j) {
      const U16x8 v = *reinterpret_cast<const U16x8*>(y + (size_t)s_row[j] * H + h);
      const float wj = s_w[j];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += wj * bf16_to_f32(v.v[i]);
    }
    for (int sh = 0; sh < S; ++sh) {
      const U16x8 v = *reinterpret_cast<const U16x8*>(shared + ((size_t)sh * T + t) * H + h);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += bf16_to_f32(v.v[i]);
    }
    if (residual) {
      const U16x8 v = *reinterpret_cast<const U16x8*>(residual + (size_t)t * H + h);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += bf16_to_f32(v.v[i]);
    }
    U16x8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      o.v[i] = f32_to_bf16(acc[i]);
      const float f = bf16_to_f32(o.v[i]);
      ss = fmaf(f, f, ss);
    }
    *reinterpret_cast<U16x8*>(out + (size_t)t * H + h) = o;
  }
  if (normed) {
    const float scale = 1.f / sqrtf(block_sum_256(ss, s_part) / (float)H + eps);
    for (int h = threadIdx.x * 8; h < H; h += blockDim.x * 8) {
      const U16x8 v = *reinterpret_cast<const U16x8*>(out + (size_t)t * H + h);  // this thread's own stores
      U16x8 o;
#pragma unroll
      for (int i = 0; i < 8; ++i) o.v[i] = f32_to_bf16(bf16_to_f32(v.v[i]) * scale);
      *reinterpret_cast<U16x8*>(normed + (size_t)t * H + h) = o;
    }
  }
}

__global__ __launch_bounds__(256) void k_unpermute_f32(const float* __restrict__ y, const int32_t* __restrict__ rop,
                                                       const float* __restrict__ w, const float* __restrict__ shared,
                                                       const float* __restrict__ residual, int S, int T, int k, int H,
                                                       float* __restrict__ out, float eps, float* __restrict__ normed) {
  const int t = blockIdx.x;
  __shared__ int32_t s_row[64];
  __shared__ float s_w[64];
  __shared__ float s_part[4];
  float ss = 0.f;
  if (threadIdx.x < k) {
    s_row[threadIdx.x] = rop[(size_t)t * k + threadIdx.x];
    s_w[threadIdx.x] = w[(size_t)t * k + threadIdx.x];
  }
  __syncthreads();
  for (int h = threadIdx.x * 4; h < H; h += blockDim.x * 4) {
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int j = 0; j < k; ++j) {
      const float4 v = *reinterpret_cast<const float4*>(y + (size_t)s_row[j] * H + h);
      const float wj = s_w[j];
      acc.x += wj * v.x; acc.y += wj * v.y; acc.z += wj * v.z; acc.w += wj * v.w;
    }
    for (int sh = 0; sh < S; ++sh) {
      const float4 v = *reinterpret_cast<const float4*>(shared + ((size_t)sh * T + t) * H + h);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (residual) {
      const float4 v = *reinterpret_cast<const float4*>(residual + (size_t)t * H + h);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    *reinterpret_cast<float4*>(out + (size_t)t * H + h) = acc;
    ss = fmaf(acc.x, acc.x, fmaf(acc.y, acc.y, fmaf(acc.z, acc.z, fmaf(acc.w, acc.w, ss))));
  }
  if (normed) {
    const float scale = 1.f / sqrtf(block_sum_256(ss, s_part) / (float)H + eps);
    for (int h = threadIdx.x * 4; h < H; h += blockDim.x * 4) {
      float4 v = *reinterpret_cast<const float4*>(out + (size_t)t * H + h);  // this thread's own stores
      v.x *= scale; v.y *= scale; v.z *= scale; v.w *= scale;
      *reinterpret_cast<float4*>(normed + (size_t)t * H + h) = v;
    }
  }
}

// out[t] = x[t] / sqrt(mean_h x[t][h]^2 + eps): unit-gain RMS normalisation, one block per token.
// A stacking aid (pre-norm residual chains), not a step of the paper's method.
template <bool BF16>
__global__ __launch_bounds__(256) void k_rmsnorm(const void* __restrict__ x_, int H, float eps, void* __restrict__ out_) {
  __shared__ float s_part[4];
  const int t = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float ss = 0.f;
  if constexpr (BF16) {
    const uint16_t* x = reinterpret_cast<const uint16_t*>(x_) + (size_t)t * H;
    for (int h = threadIdx.x * 8; h < H; h += 256 * 8) {
      const U16x8 v = *reinterpret_cast<const U16x8*>(x + h);
#pragma unroll
      for (int i = 0; i < 8; ++i) { const float f = bf16_to_f32(v.v[i]); ss = fmaf(f, f, ss); }
    }
  } else {
    const float* x = reinterpret_cast<const float*>(x_) + (size_t)t * H;
    for (int h = threadIdx.x * 4; h < H; h += 256 * 4) {
      const float4 v = *reinterpret_cast<const float4*>(x + h);
      ss = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss))));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if (lane == 0) s_part[wave] = ss;
  __syncthreads();
  const float scale = 1.f / sqrtf((s_part[0] + s_part[1] + s_part[2] + s_part[3]) / (float)H + eps);
  if constexpr (BF16) {
    const uint16_t* x = reinterpret_cast<const uint16_t*>(x_) + (size_t)t * H;
    uint16_t* out = reinterpret_cast<uint16_t*>(out_) + (size_t)t * H;
    for (int h = threadIdx.x * 8; h < H; h += 256 * 8) {
      const U16x8 v = *reinterpret_cast<const U16x8*>(x + h);
      U16x8 o;
#pragma unroll
      for (int i = 0; i < 8; ++i) o.v[i] = f32_to_bf16(bf16_to_f32(v.v[i]) * scale);
      *reinterpret_cast<U16x8*>(out + h) = o;
    }
  } else {
    const float* x = reinterpret_cast<const float*>(x_) + (size_t)t * H;
    float* out = reinterpret_cast<float*>(out_) + (size_t)t * H;
    for (int h = threadIdx.x * 4; h < H; h += 256 * 4) {
      float4 v = *reinterpret_cast<const float4*>(x + h);
      v.x *= scale; v.y *= scale; v.z *= scale; v.w *= scale;
      *reinterpret_cast<float4*>(out + h) = v;
    }
  }
}

// Router scores: one wave per token; the token's hidden vector lives in registers (strided over
// lanes), each expert's gate row is read coalesced and reduced across the wave.
template <bool BF16>
__global__ __launch_bounds__(256) void k_gate_logits(const void* __restrict__ x_, const float* __restrict__ Wg, int T, int H,
                                                     int E, const int32_t* __restrict__ aid, const float* __restrict__ bias,
                                                     float* __restrict__ logits) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + wave;
  if (t >= T) return;
  const float* brow = bias ? bias + (size_t)aid[t] * E : nullptr;
  for (int e = 0; e < E; ++e) {
    float acc = 0.f;
    const float* wrow = Wg + (size_t)e * H;
    if constexpr (BF16) {
      const uint16_t* x = reinterpret_cast<const uint16_t*>(x_) + (size_t)t * H;
      for (int h = lane * 4; h < H; h += 256) {
        const float4 wv = *reinterpret_cast<const float4*>(wrow + h);
        const ushort4 xv = *reinterpret_cast<const ushort4*>(x + h);
        acc += bf16_to_f32(xv.x) * wv.x + bf16_to_f32(xv.y) * wv.y + bf16_to_f32(xv.z) * wv.z + bf16_to_f32(xv.w) * wv.w;
      }
    } else {
      const float* x = reinterpret_cast<const float*>(x_) + (size_t)t * H;
      for (int h = lane * 4; h < H; h += 256) {
        const float4 wv = *reinterpret_cast<const float4*>(wrow + h);
        const float4 xv = *reinterpret_cast<const float4*>(x + h);
        acc += xv.x * wv.x + xv.y * wv.y + xv.z * wv.z + xv.w * wv.w;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) logits[(size_t)t * E + e] = acc + (brow ? brow[e] : 0.f);
  }
}

// Router scores on the matrix cores (bf16 tokens): A operand = token rows straight from global
// memory (16 bytes per lane), B operand = gate rows
// read as fp32 and split in registers into a bf16 head and a bf16 tail (w = hi + lo to 2^-17),
// so two bf16 MFMAs per tile reproduce the fp32 product to fp32-accumulation accuracy.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void split_bf16(const float4& lo4, const float4& hi4, bf16x8_t* head, bf16x8_t* tail) {
  const float f[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
  bf16x8_t h, t;
  // float -> bf16 casts: the hardware's packed round-to-nearest-even conversion (a fifth of the integer sequence; the
  // split is what bounds this kernel at prefill sizes, every workgroup splits its experts' whole gate rows)
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    h[i] = (__bf16)f[i];
    t[i] = (__bf16)(f[i] - (float)h[i]);
  }
  *head = h;
  *tail = t;
}

// A workgroup owns 16*TT tokens and 16*J experts (blockIdx.y picks the expert block); its NW waves
// split the contraction (K/NW each) and their partial sums meet in LDS, added in wave order.  NW = 16
// for decode-sized batches: few workgroups, so the time is the length of a wave's chain of loads.  A
// workgroup streams its experts' fp32 gate rows once, which one CU does at a few tens of GB/s:
// small batches therefore take J = 1 (four times the workgroups, a quarter of the bytes each),
// large ones 32 tokens x 32 experts with 16 waves (each wave then has one batch of loads in flight instead of a
// chain of them, and the gate rows are split into head and tail once per 32 tokens).  For a given NW the sums do
// not depend on J or TT.
template <int J, int NW, int TT>
__global__ __launch_bounds__(64 * NW) void k_gate_logits_mfma(const uint16_t* __restrict__ x, const float* __restrict__ Wg, int T,
                                                          int H, int E, const int32_t* __restrict__ aid,
                                                          const float* __restrict__ bias, float* __restrict__ logits) {
  constexpr int EB = 16 * J;
  __shared__ float s_red[NW][16][EB + 1];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int m = lane & 15, q = lane >> 4;
  const int t0 = blockIdx.x * 16 * TT;
  const int Kw = H / NW, k_lo = wave * Kw;  // H % (32 NW) == 0
  const uint16_t* xr[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) xr[tt] = x + (size_t)min(t0 + tt * 16 + m, T - 1) * H + k_lo + q * 8;
  for (int e0 = blockIdx.y * EB; e0 < E; e0 += gridDim.y * EB) {
    f32x4_t acc[TT][J];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int j = 0; j < J; ++j) acc[tt][j] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    const float* wr[J];
#pragma unroll
    for (int j = 0; j < J; ++j) wr[j] = Wg + (size_t)min(e0 + j * 16 + m, E - 1) * H + k_lo + q * 8;
#pragma unroll 4
    for (int k0 = 0; k0 < Kw; k0 += 32) {
      bf16x8_t a[TT];
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) a[tt] = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const u32x4_t*>(xr[tt] + k0));
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const float4 w0 = *reinterpret_cast<const float4*>(wr[j] + k0);
        const float4 w1 = *reinterpret_cast<const float4*>(wr[j] + k0 + 4);
        bf16x8_t head, tail;
        split_bf16(w0, w1, &head, &tail);
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          acc[tt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tt], head, acc[tt][j], 0, 0, 0);
          acc[tt][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[tt], tail, acc[tt][j], 0, 0, 0);
        }
      }
    }
    // lane holds expert e0 + 16j + m of tokens t0 + 16tt + 4q + r; one token tile at a time goes through LDS
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
#pragma unroll
      for (int j = 0; j < J; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) s_red[wave][q * 4 + r][j * 16 + m] = acc[tt][j][r];
      __syncthreads();
      for (int idx = threadIdx.x; idx < 16 * EB; idx += 64 * NW) {
        const int tr = idx / EB, ee = idx % EB;
        const int t = t0 + tt * 16 + tr, e = e0 + ee;
        if (t < T && e < E) {
          float sum = s_red[0][tr][ee];
#pragma unroll
          for (int wv = 1; wv < NW; ++wv) sum += s_red[wv][tr][ee];
          logits[(size_t)t * E + e] = sum + (bias ? bias[(size_t)aid[t] * E + e] : 0.f);
        }
      }
      __syncthreads();
    }
  }
}

}  // namespace

namespace {

int unpermute(const char* who, const void* y_sorted, const int32_t* row_of_pair, const float* topk_w, const void* shared_out,
              int num_shared, const void* residual, int T, int k, int H, int dtype, void* out, float eps, void* normed,
              void* stream) {
  using ew::fail;
  if (T < 0 || k < 1 || H < 1 || num_shared < 0) return fail(EW_ERR_INVALID_ARG, "%s: need T>=0, k>=1, H>=1, num_shared>=0", who);
  if (num_shared > 0 && !shared_out) return fail(EW_ERR_INVALID_ARG, "%s: shared_out is NULL but num_shared=%d", who, num_shared);
  const int S = shared_out ? num_shared : 0;
  if (dtype != EW_F32 && dtype != EW_BF16) return fail(EW_ERR_INVALID_ARG, "%s: unknown dtype %d", who, dtype);
  if (k > 64) return fail(EW_ERR_UNSUPPORTED, "%s: k=%d above the supported 64", who, k);
  if (H % (dtype == EW_BF16 ? 8 : 4)) return fail(EW_ERR_UNSUPPORTED, "%s: H=%d must be a multiple of %d", who, H, dtype == EW_BF16 ? 8 : 4);
  if (T == 0) return EW_OK;
  if (!y_sorted || !row_of_pair || !topk_w || !out) return fail(EW_ERR_INVALID_ARG, "%s: NULL device pointer", who);
  hipStream_t st = (hipStream_t)stream;
  if (dtype == EW_BF16)
    hipLaunchKernelGGL(k_unpermute_bf16, dim3(T), dim3(256), 0, st, (const uint16_t*)y_sorted, row_of_pair, topk_w,
                       (const uint16_t*)shared_out, (const uint16_t*)residual, S, T, k, H, (uint16_t*)out, eps, (uint16_t*)normed);
  else
    hipLaunchKernelGGL(k_unpermute_f32, dim3(T), dim3(256), 0, st, (const float*)y_sorted, row_of_pair, topk_w,
                       (const float*)shared_out, (const float*)residual, S, T, k, H, (float*)out, eps, (float*)normed);
  EW_LAUNCH_CHECK("k_unpermute");
  return EW_OK;
}

}  // namespace

extern "C" int moe_unpermute(const void* y_sorted, const int32_t* row_of_pair, const float* topk_w, const void* shared_out,
                             int num_shared, const void* residual, int T, int k, int H, int dtype, void* out, void* stream) {
  return unpermute("moe_unpermute", y_sorted, row_of_pair, topk_w, shared_out, num_shared, residual, T, k, H, dtype, out, 0.f,
                   nullptr, stream);
}

extern "C" int moe_unpermute_rmsnorm(const void* y_sorted, const int32_t* row_of_pair, const float* topk_w, const void* shared_out,
                                     int num_shared, const void* residual, int T, int k, int H, int dtype, void* out, float eps,
                                     void* normed_out, void* stream) {
  if (!(eps >= 0.f)) return ew::fail(EW_ERR_INVALID_ARG, "moe_unpermute_rmsnorm: need eps>=0");
  if (T > 0 && !normed_out) return ew::fail(EW_ERR_INVALID_ARG, "moe_unpermute_rmsnorm: normed_out is NULL");
  if (T > 0 && normed_out == out) return ew::fail(EW_ERR_INVALID_ARG, "moe_unpermute_rmsnorm: normed_out must not be out");
  return unpermute("moe_unpermute_rmsnorm", y_sorted, row_of_pair, topk_w, shared_out, num_shared, residual, T, k, H, dtype, out,
                   eps, normed_out, stream);
}

extern "C" int moe_gate_logits(const void* x, int dtype, const float* Wg, int T, int H, int E, const int32_t* adapter_id,
                               const float* bias, float* logits, void* stream) {
  using ew::fail;
  if (T < 0 || H < 1 || E < 1) return fail(EW_ERR_INVALID_ARG, "moe_gate_logits: need T>=0, H>=1, E>=1");
  if (dtype != EW_F32 && dtype != EW_BF16) return fail(EW_ERR_INVALID_ARG, "moe_gate_logits: unknown dtype %d", dtype);
  if ((adapter_id == nullptr) != (bias == nullptr)) return fail(EW_ERR_INVALID_ARG, "moe_gate_logits: adapter_id and bias go together");
  if (H % 4) return fail(EW_ERR_UNSUPPORTED, "moe_gate_logits: H=%d must be a multiple of 4", H);
  if (T == 0) return EW_OK;
  if (!x || !Wg || !logits) return fail(EW_ERR_INVALID_ARG, "moe_gate_logits: NULL device pointer");
  hipStream_t st = (hipStream_t)stream;
  if (dtype == EW_BF16 && H % 128 == 0) {
    const int tiles = ew::ceil_div(T, 16);
    if (tiles <= 16 && H % 512 == 0)
      hipLaunchKernelGGL((k_gate_logits_mfma<1, 16, 1>), dim3(tiles, ew::ceil_div(E, 16)), dim3(1024), 0, st, (const uint16_t*)x, Wg,
                         T, H, E, adapter_id, bias, logits);
    else if (tiles < 512)
      hipLaunchKernelGGL((k_gate_logits_mfma<1, 4, 1>), dim3(tiles, ew::ceil_div(E, 16)), dim3(256), 0, st, (const uint16_t*)x, Wg, T,
                         H, E, adapter_id, bias, logits);
    else if (H % 512 == 0)
      hipLaunchKernelGGL((k_gate_logits_mfma<2, 16, 4>), dim3(ew::ceil_div(tiles, 4), ew::ceil_div(E, 32)), dim3(1024), 0, st,
                         (const uint16_t*)x, Wg, T, H, E, adapter_id, bias, logits);
    else
      hipLaunchKernelGGL((k_gate_logits_mfma<4, 4, 2>), dim3(ew::ceil_div(tiles, 2), 1), dim3(256), 0, st, (const uint16_t*)x, Wg, T, H,
                         E, adapter_id, bias, logits);
  } else if (dtype == EW_BF16)
    hipLaunchKernelGGL((k_gate_logits<true>), dim3(ew::ceil_div(T, 4)), dim3(256), 0, st, x, Wg, T, H, E, adapter_id, bias, logits);
  else
    hipLaunchKernelGGL((k_gate_logits<false>), dim3(ew::ceil_div(T, 4)), dim3(256), 0, st, x, Wg, T, H, E, adapter_id, bias, logits);
  EW_LAUNCH_CHECK("k_gate_logits");
  return EW_OK;
}

extern "C" int moe_rmsnorm(const void* x, int dtype, int T, int H, float eps, void* out, void* stream) {
  using ew::fail;
  if (T < 0 || H < 1 || !(eps >= 0.f)) return fail(EW_ERR_INVALID_ARG, "moe_rmsnorm: need T>=0, H>=1, eps>=0");
  if (dtype != EW_F32 && dtype != EW_BF16) return fail(EW_ERR_INVALID_ARG, "moe_rmsnorm: unknown dtype %d", dtype);
  if (H % (dtype == EW_BF16 ? 8 : 4)) return fail(EW_ERR_UNSUPPORTED, "moe_rmsnorm: H=%d must be a multiple of %d", H, dtype == EW_BF16 ? 8 : 4);
  if (T == 0) return EW_OK;
  if (!x || !out) return fail(EW_ERR_INVALID_ARG, "moe_rmsnorm: NULL device pointer");
  hipStream_t st = (hipStream_t)stream;
  if (dtype == EW_BF16) hipLaunchKernelGGL((k_rmsnorm<true>), dim3(T), dim3(256), 0, st, x, H, eps, out);
  else hipLaunchKernelGGL((k_rmsnorm<false>), dim3(T), dim3(256), 0, st, x, H, eps, out);
  EW_LAUNCH_CHECK("k_rmsnorm");
  return EW_OK;
}
