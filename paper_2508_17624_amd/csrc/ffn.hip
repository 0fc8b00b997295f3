// Grouped SwiGLU expert FFN over the virtual weight tensors, gfx950.
//
// Paper Sec. 2.1: the experts are computed in one batch by a grouped matrix multiplication over
// the permuted tokens and the stacked expert weights; Sec. 4.1: that operator runs on the virtual
// weight tensor [M + N*E_max, H_out, H_in] and never learns that adapters exist.  Here the operator is ours: two grouped products with the SwiGLU
// activation fused into the first one's epilogue.
//
// Weight-streaming kernel (k_ffn_stream), the decode regime: a slot holds a handful of rows and
// its 16.5 MiB of weights are read once, so the kernel is HBM bound.  Tokens of the slot sit in
// LDS (B operand, <= 16*NT rows); every wave owns 16 output features at a time and streams the
// matching weight rows straight from HBM into MFMA A operands (v_mfma_f32_16x16x32_bf16,
// weights on the M side, tokens on the N side), 64 contiguous bytes per lane and row per
// 128-element K step, next step prefetched into registers while the current one multiplies.
// The contraction index is permuted identically on both operands (lane quarter q covers
// K elements [32q, 32q+32) of each 128 step) so that a lane's global loads are contiguous.
//
// Slots with count 0 are never touched: only slots listed by k_plan are visited, and weight
// addresses stay inside the slot's own [2I,H] / [H,I] block (the padding of the virtual tensor
// is unmapped address space).
#include "ew_internal.h"

#include <atomic>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float silu_f32(float g) { return g / (1.f + __expf(-g)); }

// ------------------------------------------------------------------------------------------
// plan[0] = number of slots with count > 0, plan[1..] = those slots in ascending order.
__global__ __launch_bounds__(256) void k_plan(const int32_t* __restrict__ counts, int P, int32_t* __restrict__ plan) {
  __shared__ int s_w[4];
  const int tid = threadIdx.x, wave = tid / 64, lane = tid & 63;
  int base = 0;
  for (int start = 0; start < P; start += 256) {
    const int s = start + tid;
    const bool flag = s < P && counts[s] > 0;
    const unsigned long long vote = __ballot(flag);
    const int before = __popcll(vote & (lane == 0 ? 0ull : (~0ull >> (64 - lane))));
    if (lane == 0) s_w[wave] = __popcll(vote);
    __syncthreads();
    int wbase = 0, total = 0;
    for (int w = 0; w < 4; ++w) {
      if (w < wave) wbase += s_w[w];
      total += s_w[w];
    }
    if (flag) plan[1 + base + wbase + before] = s;
    base += total;
    __syncthreads();
  }
  if (tid == 0) plan[0] = base;
}

// ------------------------------------------------------------------------------------------
struct StreamArgs {
  const uint16_t* x;        // MODE 0: tokens [T, K]; MODE 1: activations [rows, K]
  const int32_t* counts;
  const int32_t* offsets;
  const int32_t* por;       // pair_of_row or NULL (MODE 0 only)
  const uint16_t* w;        // virtual weight tensor base
  uint16_t* out;            // MODE 0: activations [rows, NOUT]; MODE 1: y [rows, NOUT]
  const int32_t* plan;
  size_t slot_stride;       // elements per slot
  int k, K, NOUT, groups, tiles_per_block;
};

// MODE 0: out = silu(x.Wg^T) * (x.Wu^T), Wg rows [0,NOUT), Wu rows [NOUT,2NOUT) of the slot.
// MODE 1: out = x.W^T, W rows [0,NOUT) of the slot.
template <int MODE, int NT>
__global__ __launch_bounds__(512) void k_ffn_stream(StreamArgs a) {
  extern __shared__ __align__(16) uint16_t s_x[];  // [16*NT][K+8]
  __shared__ int32_t s_src[16 * NT];
  const int nact = a.plan[0];
  const int ai = blockIdx.x / a.groups, g = blockIdx.x - ai * a.groups;
  if (ai >= nact) return;
  const int s = a.plan[1 + ai];
  const int c = a.counts[s], off = a.offsets[s];
  const int K = a.K, ldx = K + 8, NOUT = a.NOUT;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int m = lane & 15, q = lane >> 4;
  const uint16_t* wslot = a.w + (size_t)s * a.slot_stride;
  const int ntiles = NOUT / 16;
  const int tile_lo = g * a.tiles_per_block, tile_hi = min(ntiles, tile_lo + a.tiles_per_block);
  const int nks = K / 128, k8 = K / 8;

  for (int r0 = 0; r0 < c; r0 += 16 * NT) {
    const int nrows = min(16 * NT, c - r0);
    __syncthreads();  // readers of the previous chunk are done
    if (tid < 16 * NT) {
      int src = -1;
      if (tid < nrows) {
        const int row = off + r0 + tid;
        src = MODE == 0 ? (a.por ? a.por[row] : row) / a.k : row;
      }
      s_src[tid] = src;
    }
    __syncthreads();
    for (int idx = tid; idx < 16 * NT * k8; idx += blockDim.x) {
      const int r = idx / k8, c8 = idx - r * k8;
      uint4 v = make_uint4(0, 0, 0, 0);
      const int src = s_src[r];
      if (src >= 0) v = *reinterpret_cast<const uint4*>(a.x + (size_t)src * K + c8 * 8);
      *reinterpret_cast<uint4*>(s_x + (size_t)r * ldx + c8 * 8) = v;
    }
    __syncthreads();

    for (int tile = tile_lo + wave; tile < tile_hi; tile += nwaves) {
      const int f0 = tile * 16;
      const uint16_t* w0 = wslot + (size_t)(f0 + m) * K + q * 32;
      const uint16_t* w1 = w0 + (size_t)NOUT * K;  // MODE 0: the up projection's row
      f32x4 acc0[NT], acc1[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        acc0[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
        acc1[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
      }
      bf16x8 a0[4], a1[4], n0[4], n1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a0[i] = *reinterpret_cast<const bf16x8*>(w0 + i * 8);
        if (MODE == 0) a1[i] = *reinterpret_cast<const bf16x8*>(w1 + i * 8);
      }
      const uint16_t* xs = s_x + (size_t)m * ldx + q * 32;
      for (int ks = 0; ks < nks; ++ks) {
        if (ks + 1 < nks) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            n0[i] = *reinterpret_cast<const bf16x8*>(w0 + (ks + 1) * 128 + i * 8);
            if (MODE == 0) n1[i] = *reinterpret_cast<const bf16x8*>(w1 + (ks + 1) * 128 + i * 8);
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            const bf16x8 b = *reinterpret_cast<const bf16x8*>(xs + (size_t)nt * 16 * ldx + ks * 128 + i * 8);
            acc0[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0[i], b, acc0[nt], 0, 0, 0);
            if (MODE == 0) acc1[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[i], b, acc1[nt], 0, 0, 0);
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a0[i] = n0[i];
          if (MODE == 0) a1[i] = n1[i];
        }
      }
      // epilogue: lane holds features f0 + 4q + r (r < 4) of token nt*16 + m
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int tok = nt * 16 + m;
        if (tok < nrows) {
          ushort4 o;
          if (MODE == 0) {
            o.x = f32_to_bf16(silu_f32(acc0[nt][0]) * acc1[nt][0]);
            o.y = f32_to_bf16(silu_f32(acc0[nt][1]) * acc1[nt][1]);
            o.z = f32_to_bf16(silu_f32(acc0[nt][2]) * acc1[nt][2]);
            o.w = f32_to_bf16(silu_f32(acc0[nt][3]) * acc1[nt][3]);
          } else {
            o.x = f32_to_bf16(acc0[nt][0]);
            o.y = f32_to_bf16(acc0[nt][1]);
            o.z = f32_to_bf16(acc0[nt][2]);
            o.w = f32_to_bf16(acc0[nt][3]);
          }
          *reinterpret_cast<ushort4*>(a.out + (size_t)(off + r0 + tok) * NOUT + f0 + q * 4) = o;
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// fp32 reference-precision path (tiny configurations): one thread per output element.
__device__ __forceinline__ int slot_of_row(const int32_t* __restrict__ offsets, int P, int row) {
  int lo = 0, hi = P;  // largest s with offsets[s] <= row and offsets[s+1] > row
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (offsets[mid] <= row) lo = mid; else hi = mid;
  }
  return lo;
}

__global__ __launch_bounds__(256) void k_ffn_f32_gateup(const float* __restrict__ x, const int32_t* __restrict__ offsets,
                                                        const int32_t* __restrict__ por, const float* __restrict__ w13,
                                                        int rows, int k, int H, int I, int P, float* __restrict__ act) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)rows * I) return;
  const int row = (int)(idx / I), i = (int)(idx - (long long)row * I);
  const int s = slot_of_row(offsets, P, row);
  const int t = (por ? por[row] : row) / k;
  const float* xr = x + (size_t)t * H;
  const float* wg = w13 + ((size_t)s * 2 * I + i) * H;
  const float* wu = wg + (size_t)I * H;
  float g = 0.f, u = 0.f;
  for (int h = 0; h < H; ++h) {
    g = fmaf(xr[h], wg[h], g);
    u = fmaf(xr[h], wu[h], u);
  }
  act[idx] = g / (1.f + expf(-g)) * u;
}

__global__ __launch_bounds__(256) void k_ffn_f32_down(const float* __restrict__ act, const int32_t* __restrict__ offsets,
                                                      const float* __restrict__ w2, int rows, int H, int I, int P,
                                                      float* __restrict__ y) {
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)rows * H) return;
  const int row = (int)(idx / H), h = (int)(idx - (long long)row * H);
  const int s = slot_of_row(offsets, P, row);
  const float* ar = act + (size_t)row * I;
  const float* wr = w2 + ((size_t)s * H + h) * I;
  float acc = 0.f;
  for (int i = 0; i < I; ++i) acc = fmaf(ar[i], wr[i], acc);
  y[idx] = acc;
}

// ------------------------------------------------------------------------------------------
// Tuning state (ew_tune_ffn); 0 = automatic everywhere except the wait, where negative = automatic.
int g_path_override = 0;       // 1 = register-streaming kernel, 2 = tiled GEMM kernel, 3 = LDS-direct streaming kernel
int g_nt_override = 0;         // register-streaming kernel: 16-token tiles per slot chunk (1 or 2)
int g_threads_override = 0;    // register-streaming kernel: threads per block
int g_ws_frags = 0;            // LDS-direct kernel: 32-token fragments of the kernel shape (1, 2, 4, 8)
int g_ws_chunk_frags = 0;      // LDS-direct kernel: 32-token fragments per row chunk at most (<= shape)
int g_ws_wait_ticks = -1;      // LDS-direct kernel: rendezvous wait in 10 ns ticks (0 = never wait)
int g_ws_merge = 0;            // LDS-direct kernel, decode shapes: 1 = the two products always as two launches
// Automatic = never: since the next item is claimed behind the current one's last K slab, the workgroups that finish
// together already start together; waiting for the rest of the cohort measured the same or slower (0 / 1 / 2 / 4 us).
constexpr int kWsWaitDefault = 0;

size_t plan_bytes(int rows, int P) {
  size_t ints = (size_t)P + 1;
  const size_t g = ew::ffn_gemm_plan_ints(rows, P);
  if (g > ints) ints = g;
  const size_t w = ew::ffn_ws_plan_ints(rows, P, 1);
  if (w > ints) ints = w;
  return ew::align_up(ints * sizeof(int32_t), 256);
}

template <int MODE, int NT>
int launch_stream(const StreamArgs& a, int grid, int threads, hipStream_t st) {
  const size_t lds = (size_t)16 * NT * (a.K + 8) * sizeof(uint16_t);
  // per instantiation and per device (the attribute belongs to the device's copy of the function);
  // setting it twice from two racing threads is harmless
  static std::atomic<unsigned long long> attr_set{0};
  int dev = 0;
  EW_HIP(hipGetDevice(&dev));
  const unsigned long long bit = 1ull << (dev & 63);
  if (!(attr_set.load(std::memory_order_relaxed) & bit)) {
    EW_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_ffn_stream<MODE, NT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512));
    attr_set.fetch_or(bit, std::memory_order_relaxed);
  }
  hipLaunchKernelGGL((k_ffn_stream<MODE, NT>), dim3(grid), dim3(threads), lds, st, a);
  EW_LAUNCH_CHECK("k_ffn_stream");
  return EW_OK;
}

}  // namespace

extern "C" void ew_tune_ffn(int path, int stream_token_tiles, int stream_threads, int ws_frags, int ws_chunk_frags,
                            int ws_wait_ticks, int ws_two_launches) {
  g_ws_merge = ws_two_launches ? 1 : 0;
  g_path_override = path;
  g_nt_override = stream_token_tiles;
  g_threads_override = stream_threads;
  g_ws_frags = ws_frags;
  g_ws_chunk_frags = ws_chunk_frags;
  g_ws_wait_ticks = ws_wait_ticks;
}

extern "C" size_t moe_grouped_ffn_workspace_bytes(int T, int k, int H, int I, int P, int dtype) {
  if (T <= 0 || k < 1 || H < 1 || I < 1 || P < 1) return 0;
  const size_t el = dtype == EW_BF16 ? 2 : 4;
  return plan_bytes(T * k, P) + ew::align_up((size_t)T * k * I * el, 256);
}

namespace ew {

bool ffn_ws_shape_of_call(int dtype, int T, int k, int H, int I, int P, int S, WsPlanShape* sh) {
  if (dtype != EW_BF16 || T < 1 || k < 1 || S < 0 || P < 1 || H % 128 || I % 128) return false;
  if (g_path_override == 1 || g_path_override == 2) return false;
  const long long rows = (long long)T * (k + S);
  const int slots = P + S, Kmax = H > I ? H : I;
  if (rows >= (1ll << 31) || slots > 2048 || (unsigned long long)rows * (unsigned long long)Kmax * 2ull >= (1ull << 32)) return false;
  const int nf = ffn_ws_frags(T, (int)rows, slots < rows ? slots : (int)rows, g_ws_frags);
  *sh = ffn_ws_plan_shape((int)rows, slots, nf, g_ws_chunk_frags, g_ws_merge != 1);
  return true;
}

}  // namespace ew

namespace {

// moe_grouped_ffn (S = 0), moe_grouped_ffn_with_shared (S > 0) and moe_grouped_ffn_planned (plan_ready)
int grouped_ffn(const char* who, bool plan_ready, const void* x, int dtype, int T, int k, int H, int I, int P, int S,
                const int32_t* counts,
                const int32_t* offsets, const int32_t* pair_of_row, const void* w13_base, const void* w2_base,
                const void* w13_shared, const void* w2_shared, void* y_sorted, void* ws, size_t ws_bytes, void* stream) {
  using ew::fail;
  if (T < 0 || k < 1 || H < 1 || I < 1 || P < 1 || S < 0) return fail(EW_ERR_INVALID_ARG, "%s: need T>=0, k>=1, H>=1, I>=1, P>=1, S>=0", who);
  if (dtype != EW_F32 && dtype != EW_BF16) return fail(EW_ERR_INVALID_ARG, "%s: unknown dtype %d", who, dtype);
  if ((long long)T * (k + S) >= (1ll << 31)) return fail(EW_ERR_UNSUPPORTED, "%s: the row count must be below 2^31", who);
  if (T == 0) return EW_OK;
  if (!x || !counts || !offsets || !w13_base || !w2_base || !y_sorted || (S > 0 && (!w13_shared || !w2_shared)))
    return fail(EW_ERR_INVALID_ARG, "%s: NULL device pointer", who);
  const size_t need = moe_grouped_ffn_workspace_bytes(T, k + S, H, I, P + S, dtype);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(EW_ERR_WORKSPACE, "%s: workspace needs %zu bytes aligned to 256 (got %zu at %p)", who, need, ws_bytes, ws);
  hipStream_t st = (hipStream_t)stream;
  const int rows = T * k;
  int32_t* plan = (int32_t*)ws;
  char* act = (char*)ws + plan_bytes(T * (k + S), P + S);
  ew::WsPlanShape shape;
  const bool ws_path = ew::ffn_ws_shape_of_call(dtype, T, k, H, I, P, S, &shape);
  if (S > 0 || plan_ready) {
    // only the LDS-direct streaming kernel knows the shared experts' slots and takes a plan built elsewhere
    if (!ws_path)
      return fail(EW_ERR_UNSUPPORTED, "%s: needs bf16, H and I multiples of 128, P+S <= 2048 and T*(k+S)*max(H,I)*2 < 2^32", who);
    const int wait_ticks = g_ws_wait_ticks < 0 ? kWsWaitDefault : g_ws_wait_ticks;
    return ew::launch_ffn_ws(x, rows, k, H, I, P, S, shape, plan_ready, counts, offsets, pair_of_row, w13_base, w2_base, w13_shared,
                             w2_shared, act, y_sorted, plan, wait_ticks, st);
  }

  if (dtype == EW_F32) {
    const long long n1 = (long long)rows * I, n2 = (long long)rows * H;
    hipLaunchKernelGGL(k_ffn_f32_gateup, dim3((unsigned)((n1 + 255) / 256)), dim3(256), 0, st, (const float*)x, offsets,
                       pair_of_row, (const float*)w13_base, rows, k, H, I, P, (float*)act);
    EW_LAUNCH_CHECK("k_ffn_f32_gateup");
    hipLaunchKernelGGL(k_ffn_f32_down, dim3((unsigned)((n2 + 255) / 256)), dim3(256), 0, st, (const float*)act, offsets,
                       (const float*)w2_base, rows, H, I, P, (float*)y_sorted);
    EW_LAUNCH_CHECK("k_ffn_f32_down");
    return EW_OK;
  }

  if (H % 128 || I % 128) return fail(EW_ERR_UNSUPPORTED, "%s(bf16): H and I must be multiples of 128 (H=%d I=%d)", who, H, I);
  const int Kmax = H > I ? H : I;
  int nt = g_nt_override ? g_nt_override : (T <= 16 ? 1 : 2);
  if ((size_t)16 * nt * (Kmax + 8) * 2 > 160 * 1024 - 1024) nt = 1;
  if ((size_t)16 * nt * (Kmax + 8) * 2 > 160 * 1024 - 1024)
    return fail(EW_ERR_UNSUPPORTED, "%s(bf16): max(H,I)=%d above the supported 5000", who, Kmax);
  const int threads = g_threads_override ? g_threads_override : 512;
  const int nwaves = threads / 64;

  // Many rows per slot: compute bound, LDS-tiled GEMM.  Few rows per slot: HBM bound, stream weights.
  // The host knows only the totals, so the average rows per possible slot decides.
  const int max_slots = P < rows ? P : rows;
  // Default: the LDS-direct streaming kernel.  Its byte offsets into x / the activations are 32 bit.
  // and its work plan sorts at most 2048 slots (the limit of the permutation kernels as well).
  if (ws_path) {
    const int wait_ticks = g_ws_wait_ticks < 0 ? kWsWaitDefault : g_ws_wait_ticks;
    return ew::launch_ffn_ws(x, rows, k, H, I, P, 0, shape, false, counts, offsets, pair_of_row, w13_base, w2_base, nullptr, nullptr,
                             act, y_sorted, plan, wait_ticks, st);
  }
  if (g_path_override == 3)
    return fail(EW_ERR_UNSUPPORTED, "%s(bf16): the streaming path needs rows*max(H,I)*2 < 2^32 and P <= 2048", who);
  const bool gemm = g_path_override ? g_path_override == 2 : (rows / max_slots >= 32 && I % 64 == 0);
  if (gemm)
    return ew::launch_ffn_gemm(x, rows, k, H, I, P, counts, offsets, pair_of_row, w13_base, w2_base, act, y_sorted, plan, st);

  hipLaunchKernelGGL(k_plan, dim3(1), dim3(256), 0, st, counts, P, plan);
  EW_LAUNCH_CHECK("k_plan");
  const int max_active = P < rows ? P : rows;

  StreamArgs a{};
  a.counts = counts; a.offsets = offsets; a.plan = plan; a.k = k;
  // gate/up projection + SwiGLU
  a.x = (const uint16_t*)x; a.por = pair_of_row; a.w = (const uint16_t*)w13_base; a.out = (uint16_t*)act;
  a.slot_stride = (size_t)2 * I * H; a.K = H; a.NOUT = I;
  a.tiles_per_block = nwaves; a.groups = ew::ceil_div(I / 16, a.tiles_per_block);
  int rc = nt == 1 ? launch_stream<0, 1>(a, max_active * a.groups, threads, st) : launch_stream<0, 2>(a, max_active * a.groups, threads, st);
  if (rc != EW_OK) return rc;
  // down projection
  a.x = (const uint16_t*)act; a.por = nullptr; a.w = (const uint16_t*)w2_base; a.out = (uint16_t*)y_sorted;
  a.slot_stride = (size_t)H * I; a.K = I; a.NOUT = H;
  a.tiles_per_block = 2 * nwaves; a.groups = ew::ceil_div(H / 16, a.tiles_per_block);
  rc = nt == 1 ? launch_stream<1, 1>(a, max_active * a.groups, threads, st) : launch_stream<1, 2>(a, max_active * a.groups, threads, st);
  return rc;
}

}  // namespace

extern "C" int moe_grouped_ffn(const void* x, int dtype, int T, int k, int H, int I, int P, const int32_t* counts,
                               const int32_t* offsets, const int32_t* pair_of_row, const void* w13_base,
                               const void* w2_base, void* y_sorted, void* ws, size_t ws_bytes, void* stream) {
  return grouped_ffn("moe_grouped_ffn", false, x, dtype, T, k, H, I, P, 0, counts, offsets, pair_of_row, w13_base, w2_base, nullptr,
                     nullptr, y_sorted, ws, ws_bytes, stream);
}

extern "C" int moe_grouped_ffn_with_shared(const void* x, int dtype, int T, int k, int H, int I, int P, int S,
                                           const int32_t* counts, const int32_t* offsets, const int32_t* pair_of_row,
                                           const void* w13_base, const void* w2_base, const void* w13_shared,
                                           const void* w2_shared, void* y_sorted, void* ws, size_t ws_bytes, void* stream) {
  if (S < 1) return ew::fail(EW_ERR_INVALID_ARG, "moe_grouped_ffn_with_shared: S must be at least 1 (S=%d)", S);
  return grouped_ffn("moe_grouped_ffn_with_shared", false, x, dtype, T, k, H, I, P, S, counts, offsets, pair_of_row, w13_base, w2_base,
                     w13_shared, w2_shared, y_sorted, ws, ws_bytes, stream);
}

extern "C" int moe_grouped_ffn_planned(const void* x, int dtype, int T, int k, int H, int I, int P, int S, const int32_t* counts,
                                       const int32_t* offsets, const int32_t* pair_of_row, const void* w13_base,
                                       const void* w2_base, const void* w13_shared, const void* w2_shared, void* y_sorted,
                                       void* ws, size_t ws_bytes, void* stream) {
  return grouped_ffn("moe_grouped_ffn_planned", true, x, dtype, T, k, H, I, P, S, counts, offsets, pair_of_row, w13_base, w2_base,
                     w13_shared, w2_shared, y_sorted, ws, ws_bytes, stream);
}
