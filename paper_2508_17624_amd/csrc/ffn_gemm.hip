// Grouped expert GEMM for prefill-sized batches (many rows per slot): LDS-tiled bf16 MFMA.
//
// Paper Sec. 2.1: the GMM operator multiplies each contiguous chunk of permuted tokens with its
// expert's stacked weights.  Here one workgroup computes a BM x BN tile of one slot's product:
//   MODE 0: act[rows, I] = silu(X . Wg^T) * (X . Wu^T)   (X gathered through pair_of_row)
//   MODE 1: y[rows, H]   = act . W2^T
// Both operands are K-contiguous, so tiles are staged global -> registers -> LDS with 16-byte
// accesses, double buffered (the next K slab is in flight while the current one multiplies).
// LDS rows are 128 bytes (BK = 64 bf16); the 16-byte chunk index is XOR-swizzled with the row so
// that the 16 lanes the LDS serves per clock hit 16 different bank groups both on the
// ds_write_b128 (8 chunks x 2 rows) and on the MFMA-operand ds_read_b128 (16 rows x 1 chunk).
// Four waves form a 2 x 2 grid; each owns a 64 x 64 sub-tile = 2 x 2 v_mfma_f32_32x32x16_bf16
// accumulators.  In MODE 0 a wave's two N sub-tiles are the gate and the up projection of the
// same 32 activation columns, so SwiGLU is a lane-local epilogue.
//
// Tiles are enumerated on the device (k_plan_gemm): the host never learns the counts.  Rows
// past a slot's end are clamped loads and masked stores.  Weight tiles lie wholly inside the
// slot (I % 64 == 0, H % 128 == 0), so no access ever leaves a mapped slot.
#include "ew_internal.h"

namespace ew {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // plain vector: stays in registers (HIP uint4 is a struct)

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kThreads = 256;

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float silu_f32(float g) { return g / (1.f + __expf(-g)); }

// plan[0] = number of m-tiles; plan[1 + 2i] = slot, plan[2 + 2i] = first row (within the slot).
__global__ __launch_bounds__(256) void k_plan_gemm(const int32_t* __restrict__ counts, int P, int32_t* __restrict__ plan) {
  __shared__ int s_w[4];
  const int tid = threadIdx.x, wave = tid / 64, lane = tid & 63;
  int base = 0;
  for (int start = 0; start < P; start += 256) {
    const int s = start + tid;
    const int c = s < P ? counts[s] : 0;
    const int nt = (c + BM - 1) / BM;
    int incl = nt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    int wbase = 0, total = 0;
    for (int w = 0; w < 4; ++w) {
      if (w < wave) wbase += s_w[w];
      total += s_w[w];
    }
    int at = base + wbase + incl - nt;
    for (int i = 0; i < nt; ++i) {
      plan[1 + 2 * (at + i)] = s;
      plan[2 + 2 * (at + i)] = i * BM;
    }
    base += total;
    __syncthreads();
  }
  if (tid == 0) plan[0] = base;
}

struct GemmArgs {
  const uint16_t* x;      // MODE 0: tokens [*, K]; MODE 1: activations [rows, K]
  const int32_t* counts;
  const int32_t* offsets;
  const int32_t* por;     // MODE 0 only; may be NULL
  const uint16_t* w;
  uint16_t* out;          // [rows, NOUT]
  const int32_t* plan;
  size_t slot_stride;
  int k, K, NOUT, ntn;    // ntn = n-tiles per slot
};

// byte offset of 16-byte chunk `chunk` (0..7) of row `row` inside a [rows][64] bf16 LDS tile
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); }

template <int MODE>
__global__ __launch_bounds__(kThreads, 2) void k_ffn_gemm(GemmArgs a) {
  __shared__ __align__(16) unsigned char s_a[2][BM * BK * 2];
  __shared__ __align__(16) unsigned char s_b[2][BN * BK * 2];
  const int nmt = a.plan[0];
  const int mt = blockIdx.x / a.ntn, nt = blockIdx.x - mt * a.ntn;
  if (mt >= nmt) return;
  const int s = a.plan[1 + 2 * mt], m0 = a.plan[2 + 2 * mt];
  const int c = a.counts[s], off = a.offsets[s];
  const int K = a.K, NOUT = a.NOUT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // global -> LDS staging: thread owns chunk (tid % 8) of rows tid/8 + 32*i, i < 4, of both tiles
  const int ld_chunk = tid & 7, ld_row = tid >> 3;
  const uint16_t* a_ptr[4];
  const uint16_t* b_ptr[4];
  const uint16_t* wslot = a.w + (size_t)s * a.slot_stride;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = ld_row + 32 * i;
    int row = m0 + r;
    if (row >= c) row = c - 1;  // clamped duplicate; its outputs are masked
    size_t src;
    if (MODE == 0) src = (size_t)((a.por ? a.por[off + row] : off + row) / a.k);
    else src = (size_t)(off + row);
    a_ptr[i] = a.x + src * K + ld_chunk * 8;
    int wrow;
    if (MODE == 0) wrow = r < 64 ? nt * 64 + r : NOUT + nt * 64 + (r - 64);
    else wrow = nt * BN + r;
    b_ptr[i] = wslot + (size_t)wrow * K + ld_chunk * 8;
  }
  int st_off[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) st_off[i] = lds_off(ld_row + 32 * i, ld_chunk);

  // MFMA operand reads: lane supplies row (lane % 32) of a 32-row sub-tile, K chunk 2*ks + lane/32
  const int fr = lane & 31, fh = lane >> 5;
  int a_row[2], b_row[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    a_row[t] = wm * 64 + t * 32 + fr;
    b_row[t] = (MODE == 0 ? t * 64 + wn * 32 : wn * 64 + t * 32) + fr;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 ra[4], rb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ra[i] = *reinterpret_cast<const u32x4*>(a_ptr[i]);
    rb[i] = *reinterpret_cast<const u32x4*>(b_ptr[i]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    *reinterpret_cast<u32x4*>(&s_a[0][st_off[i]]) = ra[i];
    *reinterpret_cast<u32x4*>(&s_b[0][st_off[i]]) = rb[i];
  }
  __syncthreads();

  const int nk = K / BK;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ra[i] = *reinterpret_cast<const u32x4*>(a_ptr[i] + (size_t)(kt + 1) * BK);
        rb[i] = *reinterpret_cast<const u32x4*>(b_ptr[i] + (size_t)(kt + 1) * BK);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        fa[t] = *reinterpret_cast<const bf16x8*>(&s_a[cur][lds_off(a_row[t], 2 * ks + fh)]);
        fb[t] = *reinterpret_cast<const bf16x8*>(&s_b[cur][lds_off(b_row[t], 2 * ks + fh)]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<u32x4*>(&s_a[cur ^ 1][st_off[i]]) = ra[i];
        *reinterpret_cast<u32x4*>(&s_b[cur ^ 1][st_off[i]]) = rb[i];
      }
    }
    __syncthreads();
  }

  // epilogue.  Accumulator element e of lane l: row 8*(e/4) + 4*(l/32) + e%4, column l%32.
  const int col = lane & 31;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int r = m0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * fh + (e & 3);
      if (r < c) {
        uint16_t* orow = a.out + (size_t)(off + r) * NOUT;
        if (MODE == 0) {
          orow[nt * 64 + wn * 32 + col] = f32_to_bf16(silu_f32(acc[i][0][e]) * acc[i][1][e]);
        } else {
          orow[nt * BN + wn * 64 + col] = f32_to_bf16(acc[i][0][e]);
          orow[nt * BN + wn * 64 + 32 + col] = f32_to_bf16(acc[i][1][e]);
        }
      }
    }
  }
}

}  // namespace

size_t ffn_gemm_plan_ints(int rows, int P) {
  const int max_active = P < rows ? P : rows;
  return 1 + 2 * ((size_t)rows / BM + max_active);
}

// Enqueues plan + both products.  `plan` holds ffn_gemm_plan_ints(rows, P) ints.
int launch_ffn_gemm(const void* x, int rows, int k, int H, int I, int P, const int32_t* counts, const int32_t* offsets,
                    const int32_t* por, const void* w13, const void* w2, void* act, void* y, int32_t* plan, hipStream_t st) {
  hipLaunchKernelGGL(k_plan_gemm, dim3(1), dim3(256), 0, st, counts, P, plan);
  EW_LAUNCH_CHECK("k_plan_gemm");
  const int max_active = P < rows ? P : rows;
  const int max_mt = rows / BM + max_active;
  GemmArgs a{};
  a.counts = counts; a.offsets = offsets; a.plan = plan; a.k = k;
  a.x = (const uint16_t*)x; a.por = por; a.w = (const uint16_t*)w13; a.out = (uint16_t*)act;
  a.slot_stride = (size_t)2 * I * H; a.K = H; a.NOUT = I; a.ntn = I / 64;
  hipLaunchKernelGGL((k_ffn_gemm<0>), dim3(max_mt * a.ntn), dim3(kThreads), 0, st, a);
  EW_LAUNCH_CHECK("k_ffn_gemm<0>");
  a.x = (const uint16_t*)act; a.por = nullptr; a.w = (const uint16_t*)w2; a.out = (uint16_t*)y;
  a.slot_stride = (size_t)H * I; a.K = I; a.NOUT = H; a.ntn = H / BN;
  hipLaunchKernelGGL((k_ffn_gemm<1>), dim3(max_mt * a.ntn), dim3(kThreads), 0, st, a);
  EW_LAUNCH_CHECK("k_ffn_gemm<1>");
  return EW_OK;
}

}  // namespace ew
