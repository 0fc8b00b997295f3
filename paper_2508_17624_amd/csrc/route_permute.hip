// Router top-k, batched rerouting and stable token permutation for gfx950 (wave64).
//
// Paper Sec. 2.1 (router top-k; dispatch = replicate, permute, group by expert id), Sec. 4.1
// (TopK'(x) = {Pi[A(x), j] : j in TopK(x)}) and Sec. 4.3 (rerouting fused into one kernel).
//
// Design for CDNA4:
//  * top-k: one wavefront per token, experts strided over the 64 lanes.  Each logit becomes an
//    order-preserving 32-bit key; a radix select over its bits, driven by wave ballots, finds
//    the k winners with scalar-unit mask arithmetic only (ties go to the lower index).
//  * rerouting is a lookup in the expert map (staged in LDS), fused into whichever kernel first
//    touches the ids: it never costs a launch or a pass over memory of its own.
//  * permutation is a stable counting sort by slot.  Order inside a slot must be ascending
//    pair index, so no atomic cursors: every wave ranks a contiguous run of pairs 64 at a time
//    with a ballot-built peer mask (rank = popcount of lower peers) and a wave-private LDS
//    counter; runs are stitched by exclusive scans over waves (LDS) and over blocks (global).
//  * small batches (decode): with ids given, ONE single-block kernel does lookup, histogram, scan
//    and scatter without leaving the CU; with the router fused, a multi-block top-k + lookup
//    kernel (one wave per token) runs first and that block receives slots.  Large batches use
//    three kernels: per-block histogram (fused with top-k and lookup), column scan, ranked scatter.
#include "ew_internal.h"

#include <atomic>

namespace {

constexpr int kWave = 64;
constexpr int kMaxP = 2048;          // slots supported by the permutation kernels
constexpr int kMaxE = 1024;          // experts supported by the top-k kernels
constexpr int kSmallPairs = 4096;    // single-block path: capacity of its LDS arrays (T*k at most this)
int g_small_pairs = 2048;            // single-block path is used up to this many pairs (tunable, <= kSmallPairs)
constexpr int kSmallCnt = 12288;     // single-block path: waves * P at most this (uint16 counters)
constexpr int kBigThreads = 512;     // multi-block path: threads per block
constexpr int kBigWaves = kBigThreads / kWave;
constexpr int kHistThreads = 1024;   // the histogram kernel is a plain stream: more waves per block hide its latency
constexpr int kBigPairs = 12288;     // multi-block path: pairs per block at most this
constexpr int kBigSteps = kBigPairs / kBigWaves / kWave;  // 64-pair steps per wave = 24
constexpr int kMapLds = 8192;        // expert-map entries staged in LDS at most

// ------------------------------------------------------------------------------------------
// wave primitives
// Wave-wide fp32 sum, result broadcast to every lane.  Row-local Hillis-Steele steps with DPP
// row_shr 1/2/4/8 leave each 16-lane row's total in its last lane; row_bcast15 / row_bcast31
// carry the totals across rows into lane 63.  Fixed order, so the sum is deterministic.
__device__ __forceinline__ float wave_sum_f32(float v) {
#define EW_DPP_ADD(ctrl, rmask)                                                                          \
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), ctrl, rmask, 0xf, false))
  EW_DPP_ADD(0x111, 0xf);  // row_shr:1
  EW_DPP_ADD(0x112, 0xf);  // row_shr:2
  EW_DPP_ADD(0x114, 0xf);  // row_shr:4
  EW_DPP_ADD(0x118, 0xf);  // row_shr:8
  EW_DPP_ADD(0x142, 0xa);  // row_bcast:15 into rows 1 and 3
  EW_DPP_ADD(0x143, 0xc);  // row_bcast:31 into rows 2 and 3
#undef EW_DPP_ADD
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ int wave_incl_scan_i32(int v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int u = __shfl_up(v, o, kWave);
    if (lane >= o) v += u;
  }
  return v;
}

// Monotone map float -> uint32 (larger float, larger key); -0.0 and +0.0 share one key.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Lanes in `active` whose `key` (low `bits` bits significant) equals this lane's.
__device__ __forceinline__ unsigned long long match_any(uint32_t key, int bits, unsigned long long active) {
  unsigned long long m = active;
  for (int b = 0; b < bits; ++b) {
    const bool bit = (key >> b) & 1u;
    const unsigned long long vote = __ballot(bit);
    m &= bit ? vote : ~vote;
  }
  return m;
}

__device__ __forceinline__ unsigned long long lanemask_lt() {
  const unsigned lane = threadIdx.x & (kWave - 1);
  return lane == 0 ? 0ull : (~0ull >> (kWave - lane));
}

// The `n` lowest set bits of m (n <= popcount(m)).
__device__ __forceinline__ unsigned long long lowest_bits(unsigned long long m, int n) {
  unsigned long long t = 0;
  for (int i = 0; i < n; ++i) {
    t |= m & (0ull - m);
    m &= m - 1;
  }
  return t;
}

// One wave selects the top-k of one token's E logits and calls emit(rank, expert, weight) once
// per selected expert, from the lane that holds it (rank 0 = largest logit; equal logits rank by
// lower expert index).  Lane l holds experts l, l+64, ... (VPL per lane, E <= 64*VPL).
//
// Selection is a radix select over the 32 bits of the order-preserving key, most significant
// first: a ballot splits the still-tied candidates by the current bit; if the ones alone fill
// what is still needed they become the candidates, otherwise they are all taken.  What is left
// at the end ties exactly with the k-th value and is filled up from the lowest index.  All of
// that is wave-uniform mask arithmetic on the scalar unit: no cross-lane data movement.
template <int VPL, typename Emit>
__device__ __forceinline__ void wave_topk(const float* __restrict__ row, int E, int k, int renorm, Emit emit) {
  const int lane = threadIdx.x & (kWave - 1);
  float val[VPL];
  uint32_t key[VPL];
  unsigned long long cand[VPL], sel[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int e = lane + v * kWave;
    const bool ok = e < E;
    val[v] = ok ? row[e] : 0.f;
    key[v] = ok ? order_key(val[v]) : 0u;
    cand[v] = __ballot(ok);
    sel[v] = 0ull;
  }
  int need = k;
  for (int b = 31; b >= 0; --b) {
    unsigned long long ones[VPL];
    int c = 0;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      ones[v] = __ballot((key[v] >> b) & 1u) & cand[v];
      c += __popcll(ones[v]);
    }
    if (c >= need) {
#pragma unroll
      for (int v = 0; v < VPL; ++v) cand[v] = ones[v];
    } else {
      need -= c;
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        sel[v] |= ones[v];
        cand[v] &= ~ones[v];
      }
    }
  }
#pragma unroll
  for (int v = 0; v < VPL; ++v) {  // ties with the k-th value: lowest expert index first
    const int have = __popcll(cand[v]);
    const int take = have < need ? have : need;
    sel[v] |= lowest_bits(cand[v], take);
    need -= take;
  }
  // rank of every selected value among the selected ones
  int rank[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) rank[v] = 0;
#pragma unroll
  for (int u = 0; u < VPL; ++u) {
    unsigned long long m = sel[u];
    while (m) {
      const int src = __ffsll((long long)m) - 1;
      m &= m - 1;
      const uint32_t okey = (uint32_t)__builtin_amdgcn_readlane((int)key[u], src);
      const int oe = src + u * kWave;
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const int e = lane + v * kWave;
        rank[v] += (okey > key[v] || (okey == key[v] && oe < e)) ? 1 : 0;
      }
    }
  }
  // softmax over all E logits: max = the rank-0 value
  float vmax = 0.f;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const unsigned long long top = __ballot(((sel[v] >> lane) & 1ull) && rank[v] == 0);
    if (top) vmax = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(val[v]), __ffsll((long long)top) - 1));
  }
  float ex[VPL], part = 0.f, spart = 0.f;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    ex[v] = (lane + v * kWave < E) ? expf(val[v] - vmax) : 0.f;
    part += ex[v];
    if ((sel[v] >> lane) & 1ull) spart += ex[v];
  }
  const float denom = wave_sum_f32(part);
  float scale = 1.f;
  if (renorm) scale = 1.f / wave_sum_f32(spart / denom);
#pragma unroll
  for (int v = 0; v < VPL; ++v)
    if ((sel[v] >> lane) & 1ull) emit(rank[v], lane + v * kWave, ex[v] / denom * scale);
}

// Stages the expert map in LDS when it fits; returns the pointer lookups should use.
__device__ __forceinline__ const int32_t* stage_map(const int32_t* __restrict__ emap, int32_t* s_map, int entries) {
  if (entries > kMapLds) return emap;
  for (int i = threadIdx.x; i < entries; i += blockDim.x) s_map[i] = emap[i];
  return s_map;
}

// Exclusive scans of two values per thread over the block's kBigThreads threads at once (thread order); ta, tb = the
// totals.  s_w: 2 * kBigWaves ints of LDS.  Contains one barrier; s_w may be reused after the next one.
__device__ __forceinline__ void block_exscan2(int a, int b, int& ea, int& eb, int& ta, int& tb, int32_t* s_w) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  const int ia = wave_incl_scan_i32(a), ib = wave_incl_scan_i32(b);
  if (lane == kWave - 1) {
    s_w[2 * wave] = ia;
    s_w[2 * wave + 1] = ib;
  }
  __syncthreads();
  int pa = 0, pb = 0;
  ta = 0;
  tb = 0;
#pragma unroll
  for (int w = 0; w < kBigWaves; ++w) {
    const int xa = s_w[2 * w], xb = s_w[2 * w + 1];
    if (w < wave) { pa += xa; pb += xb; }
    ta += xa;
    tb += xb;
  }
  ea = pa + ia - a;
  eb = pb + ib - b;
}

// Exclusive scan of v[0..P) in place by wave 0 (P <= kMaxP); v[P] = total.  Needs barriers around.
__device__ __forceinline__ void wave0_exscan(int32_t* v, int P) {
  if (threadIdx.x >= kWave) return;
  const int lane = threadIdx.x;
  const int per = (P + kWave - 1) / kWave;
  const int lo = lane * per, hi = min(P, lo + per);
  int sum = 0;
  for (int i = lo; i < hi; ++i) sum += v[i];
  int run = wave_incl_scan_i32(sum) - sum;
  for (int i = lo; i < hi; ++i) {
    const int c = v[i];
    v[i] = run;
    run += c;
  }
  const int total = __shfl(run, kWave - 1, kWave);
  if (lane == 0) v[P] = total;
}

// ------------------------------------------------------------------------------------------
// stand-alone router top-k: one wave per token, 4 waves per block
template <int VPL>
__global__ __launch_bounds__(256) void k_route_topk(const float* __restrict__ logits, int T, int E, int k, int renorm,
                                                    int32_t* __restrict__ ids, float* __restrict__ w) {
  const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
  const int waves_total = gridDim.x * (blockDim.x / kWave);
  for (int t = blockIdx.x * (blockDim.x / kWave) + wave; t < T; t += waves_total) {
    wave_topk<VPL>(logits + (size_t)t * E, E, k, renorm, [&](int rank, int e, float wt) {
      ids[(size_t)t * k + rank] = e;
      w[(size_t)t * k + rank] = wt;
    });
  }
}

// Router top-k with the rerouting fused in (Sec. 4.3: the lookup rides on the kernel that produces
// the ids), one wave per token over as many blocks as the batch needs: the first half of the
// decode-sized path, whose second half (k_small with slots given) is a single block.
template <int VPL>
__global__ __launch_bounds__(256) void k_route_reroute(const float* __restrict__ logits, const int32_t* __restrict__ aid,
                                                       const int32_t* __restrict__ emap, int T, int E, int k, int renorm,
                                                       int32_t* __restrict__ ids, float* __restrict__ w,
                                                       int32_t* __restrict__ slot_ids) {
  const int wave = threadIdx.x / kWave;
  const int t = blockIdx.x * (blockDim.x / kWave) + wave;
  if (t >= T) return;
  const int32_t* maprow = emap + (size_t)aid[t] * E;
  wave_topk<VPL>(logits + (size_t)t * E, E, k, renorm, [&](int rank, int e, float wt) {
    const size_t p = (size_t)t * k + rank;
    ids[p] = e;
    w[p] = wt;
    slot_ids[p] = maprow[e];
  });
}

// Plan request of a permutation call: the grouped FFN's work plan is written too (plan == nullptr: not asked for).
struct SmallPlan {
  int32_t* plan;
  int S;
  ew::WsPlanShape shape;
};

// ------------------------------------------------------------------------------------------
// Single-block path (decode-sized batches).  With given ids everything happens in this one launch;
// with the router fused, k_route_reroute runs first (a single block would walk the tokens' top-k
// selections 16 at a time) and this kernel receives slots (emap == nullptr).
// run = pairs per wave, a multiple of 64.  VPL = 0: ids are given (no top-k).
template <int VPL>
__global__ __launch_bounds__(1024) void k_small(const float* __restrict__ logits, const int32_t* __restrict__ ids_in,
                                                const int32_t* __restrict__ aid, const int32_t* __restrict__ emap,
                                                int T, int E, int k, int P, int map_entries, int renorm, int bits, int run,
                                                int32_t* __restrict__ ids_out, float* __restrict__ w_out,
                                                int32_t* __restrict__ slot_ids, int32_t* __restrict__ counts,
                                                int32_t* __restrict__ offsets, int32_t* __restrict__ pair_of_row,
                                                int32_t* __restrict__ row_of_pair, SmallPlan fp) {
  struct Perm {
    uint16_t slot[kSmallPairs];
    uint16_t rank[kSmallPairs];
    uint16_t cnt[kSmallCnt];
    int32_t off[kMaxP + 1];
  };
  __shared__ union Lds {
    Perm perm;
    ew::WsPlanLds plan;  // after the scatter
  } lds;
  uint16_t (&s_slot)[kSmallPairs] = lds.perm.slot;
  uint16_t (&s_rank)[kSmallPairs] = lds.perm.rank;
  uint16_t (&s_cnt)[kSmallCnt] = lds.perm.cnt;
  int32_t (&s_off)[kMaxP + 1] = lds.perm.off;
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int wave = tid / kWave, lane = tid & (kWave - 1), nwaves = nthreads / kWave;
  const int n = T * k;

  for (int i = tid; i < nwaves * P; i += nthreads) s_cnt[i] = 0;

  // A: ids (top-k or given) -> slot through the expert map
  if constexpr (VPL > 0) {
    for (int t = wave; t < T; t += nwaves) {
      const int32_t* maprow = emap + (size_t)aid[t] * E;
      wave_topk<VPL>(logits + (size_t)t * E, E, k, renorm, [&](int rank, int e, float wt) {
        const int s = maprow[e];
        const int p = t * k + rank;
        ids_out[p] = e;
        w_out[p] = wt;
        slot_ids[p] = s;
        s_slot[p] = (uint16_t)s;
      });
    }
  } else {
    for (int p = tid; p < n; p += nthreads) {
      int s;
      if (emap) {
        s = emap[(size_t)aid[p / k] * E + ids_in[p]];
        slot_ids[p] = s;
      } else {
        s = ids_in[p];  // already slots (written by k_route_reroute)
      }
      s_slot[p] = (uint16_t)s;
    }
  }
  __syncthreads();

  // B: wave w ranks its run [w*run, (w+1)*run) 64 pairs at a time
  {
    uint16_t* cnt = s_cnt + (size_t)wave * P;
    const int lo = wave * run, hi = min(n, lo + run);
    const unsigned long long lt = lanemask_lt();
    for (int base = lo; base < hi; base += kWave) {
      const int i = base + lane;
      const bool valid = i < hi;
      const uint32_t s = valid ? s_slot[i] : 0u;
      const unsigned long long peers = match_any(s, bits, __ballot(valid));
      const int before = __popcll(peers & lt);
      uint16_t old = 0;
      if (valid) old = cnt[s];
      __builtin_amdgcn_wave_barrier();
      if (valid) {
        s_rank[i] = (uint16_t)(old + before);
        if (before == 0) cnt[s] = (uint16_t)(old + __popcll(peers));
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  __syncthreads();

  // C: per slot, exclusive scan over waves (in place); slot totals -> s_off
  for (int s = tid; s < P; s += nthreads) {
    int tot = 0;
    for (int w = 0; w < nwaves; ++w) {
      const int c = s_cnt[(size_t)w * P + s];
      s_cnt[(size_t)w * P + s] = (uint16_t)tot;
      tot += c;
    }
    s_off[s] = tot;
  }
  __syncthreads();
  wave0_exscan(s_off, P);
  __syncthreads();
  for (int s = tid; s < P; s += nthreads) {
    offsets[s] = s_off[s];
    counts[s] = s_off[s + 1] - s_off[s];
  }
  if (tid == 0) offsets[P] = n;

  // D: scatter
  for (int p = tid; p < n; p += nthreads) {
    const int s = s_slot[p];
    const int dest = s_off[s] + s_cnt[(size_t)(p / run) * P + s] + s_rank[p];
    pair_of_row[dest] = p;
    if (row_of_pair) row_of_pair[p] = dest;
  }

  // E: the work plan of the grouped FFN call that consumes counts / offsets, if asked for (block of >= 512 threads)
  if (fp.plan) {
    int32_t have[8] = {0, 0, 0, 0, 0, 0, 0, 0};   // this thread's four slots, taken from LDS before the plan reuses it
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int sl = 4 * tid + i;
      if (tid < 512 && sl < P) {
        have[4 + i] = s_off[sl];
        have[i] = s_off[sl + 1] - s_off[sl];
      }
    }
    __syncthreads();  // the permutation's LDS arrays are dead
    ew::ws_plan_build(counts, offsets, P, fp.S, T, n, fp.shape, fp.plan, lds.plan, have);
  }
}

// ------------------------------------------------------------------------------------------
// Multi-block path, kernel 1: block b owns tokens [b*cht, (b+1)*cht).  ids (top-k or given) ->
// slots (written out) -> LDS histogram -> hist[b][0..P).
template <int VPL>
__global__ __launch_bounds__(kHistThreads) void k_hist(const float* __restrict__ logits, const int32_t* __restrict__ ids_in,
                                                      const int32_t* __restrict__ aid, const int32_t* __restrict__ emap,
                                                      int T, int E, int k, int P, int map_entries, int renorm, int cht,
                                                      int32_t* __restrict__ ids_out, float* __restrict__ w_out,
                                                      int32_t* __restrict__ slot_ids, int32_t* __restrict__ hist) {
  __shared__ int32_t s_hist[kMaxP];
  __shared__ int32_t s_map[kMapLds];
  const int tid = threadIdx.x;
  const int wave = tid / kWave;
  const int t0 = blockIdx.x * cht, t1 = min(T, t0 + cht);
  for (int i = tid; i < P; i += kHistThreads) s_hist[i] = 0;
  const int32_t* map = stage_map(emap, s_map, map_entries);
  __syncthreads();
  if constexpr (VPL > 0) {
    for (int t = t0 + wave; t < t1; t += kHistThreads / kWave) {
      const int32_t* maprow = map + aid[t] * E;
      wave_topk<VPL>(logits + (size_t)t * E, E, k, renorm, [&](int rank, int e, float wt) {
        const int s = maprow[e];
        const size_t p = (size_t)t * k + rank;
        ids_out[p] = e;
        w_out[p] = wt;
        slot_ids[p] = s;
        atomicAdd(&s_hist[s], 1);
      });
    }
  } else {
    // four pairs per thread and pass, all loads of a pass issued before their first use; the
    // token of local pair q is floor((q + 0.5) / k), exact in fp32 for q < 2^14 and k <= 64
    const size_t p0 = (size_t)t0 * k;
    const int n = (t1 - t0) * k;
    const float inv_k = 1.0f / (float)k;
    for (int q0 = tid; q0 < n; q0 += 4 * kHistThreads) {
      int idv[4], av[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int q = q0 + j * kHistThreads;
        const bool ok = q < n;
        idv[j] = ok ? ids_in[p0 + q] : 0;
        av[j] = ok ? aid[t0 + (int)(((float)q + 0.5f) * inv_k)] : 0;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int q = q0 + j * kHistThreads;
        if (q < n) {
          const int s = map[av[j] * E + idv[j]];
          slot_ids[p0 + q] = s;
          atomicAdd(&s_hist[s], 1);
        }
      }
    }
  }
  __syncthreads();
  int32_t* out = hist + (size_t)blockIdx.x * P;
  for (int i = tid; i < P; i += kHistThreads) out[i] = s_hist[i];
}

// Kernel 2: exclusive scan down the columns of hist[nb][P] in place; counts[s] = column total.
// Block bx owns 16 columns; thread (c = tid%16, g = tid/16) owns rows [g*rpg, (g+1)*rpg) and keeps them in registers
// when there are at most kScanRows of them (nb <= 512), so that the matrix is read once; wave w then scans the 64 group
// sums of column w with lane shuffles.
constexpr int kScanCols = 16;
constexpr int kScanGroups = 64;
constexpr int kScanRows = 8;
static_assert(kScanGroups == kWave && kScanCols * kScanGroups / kWave == kScanCols, "one wave per column in the middle step");
__global__ __launch_bounds__(kScanCols * kScanGroups) void k_colscan(int32_t* __restrict__ hist, int nb, int P,
                                                                     int32_t* __restrict__ counts) {
  __shared__ int32_t s_part[kScanCols][kScanGroups + 1];
  const int c = threadIdx.x % kScanCols, g = threadIdx.x / kScanCols;
  const int col = blockIdx.x * kScanCols + c;
  const int rpg = (nb + kScanGroups - 1) / kScanGroups;
  const int r0 = g * rpg, r1 = min(nb, r0 + rpg);
  const bool in_regs = rpg <= kScanRows;  // block-uniform
  int v[kScanRows];
  int sum = 0;
  if (in_regs) {
#pragma unroll
    for (int j = 0; j < kScanRows; ++j) {
      v[j] = (col < P && r0 + j < r1) ? hist[(size_t)(r0 + j) * P + col] : 0;
      sum += v[j];
    }
  } else if (col < P) {
    for (int r = r0; r < r1; ++r) sum += hist[(size_t)r * P + col];
  }
  s_part[c][g] = sum;
  __syncthreads();
  {
    const int w = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    const int x = s_part[w][lane];
    const int inc = wave_incl_scan_i32(x);
    s_part[w][lane] = inc - x;
    if (lane == kWave - 1 && blockIdx.x * kScanCols + w < P) counts[blockIdx.x * kScanCols + w] = inc;
  }
  __syncthreads();
  int run = s_part[c][g];
  if (in_regs) {
#pragma unroll
    for (int j = 0; j < kScanRows; ++j) {
      if (col < P && r0 + j < r1) hist[(size_t)(r0 + j) * P + col] = run;
      run += v[j];
    }
  } else if (col < P) {
    for (int r = r0; r < r1; ++r) {
      const int x = hist[(size_t)r * P + col];
      hist[(size_t)r * P + col] = run;
      run += x;
    }
  }
}

// The wave's slot ids, one pair per lane and step (pair lo + 64 i + lane), all loads issued before any is used:
// one memory round trip instead of one per step.
__device__ __forceinline__ void load_pairs(const int32_t* __restrict__ slot_ids, size_t p0, int lo, int hi, int steps,
                                           uint32_t (&packed)[kBigSteps]) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int i = 0; i < kBigSteps; ++i) {
    const int idx = lo + i * kWave + lane;
    packed[i] = (i < steps && idx < hi) ? (uint32_t)slot_ids[p0 + idx] : 0u;
  }
}

// Ranks the wave's pairs [lo, hi), 64 consecutive pairs per step: packed[i] = slot on entry and
// slot | rank among the wave's earlier pairs of that slot << 12 | valid << 31 on return.  cnt: the wave's counter per
// slot (zeroed).  MASKS: lanes of a step that hold the same slot find each other through a 64-bit lane mask per slot in
// LDS (`mask`, zeroed): every lane ORs its bit in (commutative, so the result does not depend on the order the
// hardware resolves the conflicts in), reads the mask back, and the first lane of each group clears it again.
// Otherwise the lanes compare keys bit by bit with ballots (about six times the vector instructions).
template <bool MASKS>
__device__ __forceinline__ void rank_pairs(int lo, int hi, int steps, int bits, uint16_t* cnt, unsigned long long* mask,
                                           uint32_t (&packed)[kBigSteps]) {
  const int lane = threadIdx.x & (kWave - 1);
  const unsigned long long lt = lanemask_lt();
#pragma unroll
  for (int i = 0; i < kBigSteps; ++i) {
    if (i >= steps) { packed[i] = 0u; continue; }
    const int idx = lo + i * kWave + lane;
    const bool valid = idx < hi;
    const uint32_t s = packed[i];
    unsigned long long peers;
    if constexpr (MASKS) {
      if (valid) __hip_atomic_fetch_or(&mask[s], 1ull << lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      __builtin_amdgcn_wave_barrier();
      peers = valid ? __hip_atomic_load(&mask[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : 0ull;
    } else {
      peers = match_any(s, bits, __ballot(valid));
    }
    const int before = __popcll(peers & lt);
    uint32_t old = 0;
    if (valid) old = cnt[s];
    __builtin_amdgcn_wave_barrier();
    if (valid && before == 0) {
      cnt[s] = (uint16_t)(old + __popcll(peers));
      if constexpr (MASKS) mask[s] = 0ull;
    }
    __builtin_amdgcn_wave_barrier();
    packed[i] = s | ((old + before) << 12) | (valid ? 0x80000000u : 0u);
  }
}

// Kernel 3: block b ranks its pairs and scatters them.  base[b][s] (scanned hist) + offsets[s]
// is where block b's first pair of slot s goes.  row_of_pair is written in pair order straight
// from the ranking.  pair_of_row would be a 4-byte store per lane to 64 different cache lines that
// way, so the block first sorts its pairs by slot in LDS and then writes each slot's run with
// consecutive lanes on consecutive addresses.  MAXP sizes the LDS tables (P <= MAXP).
template <int MAXP>
__global__ __launch_bounds__(kBigThreads) void k_scatter(const int32_t* __restrict__ slot_ids, const int32_t* __restrict__ counts,
                                                         const int32_t* __restrict__ base, int T, int k, int P, int bits, int cht,
                                                         int run, int32_t* __restrict__ offsets, int32_t* __restrict__ pair_of_row,
                                                         int32_t* __restrict__ row_of_pair) {
  __shared__ uint16_t s_cnt[kBigWaves * MAXP];
  __shared__ int32_t s_off[MAXP + 1];    // first row of the block's pairs of slot s
  __shared__ int32_t s_loc[MAXP + 1];    // first position of slot s in the block's sorted order
  __shared__ uint32_t s_sorted[kBigPairs];  // slot << 16 | pair index inside the block, sorted by slot
  const int tid = threadIdx.x;
  const int wave = tid / kWave, lane = tid & (kWave - 1);
  const int t0 = blockIdx.x * cht, t1 = min(T, t0 + cht);
  const size_t p0 = (size_t)t0 * k;
  const int n = (t1 - t0) * k;                                    // pairs of this block, <= kBigPairs
  const int lo = wave * run, hi = min(n, lo + run);               // run: pairs per wave, a multiple of 64
  const int steps = run / kWave;                                  // <= kBigSteps
  uint32_t packed[kBigSteps];                                     // slot | rank << 12 | valid << 31
  load_pairs(slot_ids, p0, lo, hi, steps, packed);
  const int32_t* mybase = base + (size_t)blockIdx.x * P;
  int32_t base_v[MAXP / kBigThreads];                             // this block's row of the scanned histogram
#pragma unroll
  for (int j = 0; j < MAXP / kBigThreads; ++j) {
    const int sl = tid + j * kBigThreads;
    base_v[j] = sl < P ? mybase[sl] : 0;
  }
  // Lanes of a step that hold the same slot find each other through a 64-bit lane mask per (wave,
  // slot) in LDS: every lane ORs its bit in (commutative, so the result does not depend on the
  // order the hardware resolves the conflicts in), reads the mask back, and the first lane of
  // each group clears it again.  It needs waves * P * 8 bytes, which the sorted-pairs array lends
  // while the ranking runs; the table for P > 512 would not fit, there the lanes compare keys bit
  // by bit with ballots instead (about six times the vector instructions).
  constexpr bool kMasks = (size_t)kBigWaves * MAXP * 8 <= sizeof(s_sorted);
  unsigned long long* s_mask = reinterpret_cast<unsigned long long*>(s_sorted);
  for (int i = tid; i < kBigWaves * P; i += kBigThreads) {
    s_cnt[i] = 0;
    if (kMasks) s_mask[i] = 0ull;
  }
  for (int i = tid; i < P; i += kBigThreads) s_off[i] = counts[i];
  __syncthreads();
  wave0_exscan(s_off, P);
  __syncthreads();
  if (blockIdx.x == 0)
    for (int i = tid; i <= P; i += kBigThreads) offsets[i] = s_off[i];

  rank_pairs<kMasks>(lo, hi, steps, bits, s_cnt + (size_t)wave * P, s_mask + (size_t)wave * P, packed);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < MAXP / kBigThreads; ++j) {
    const int s = tid + j * kBigThreads;
    if (s < P) {
      int tot = 0;
#pragma unroll
      for (int w = 0; w < kBigWaves; ++w) {
        const int c = s_cnt[(size_t)w * P + s];
        s_cnt[(size_t)w * P + s] = (uint16_t)tot;
        tot += c;
      }
      s_off[s] += base_v[j];
      s_loc[s] = tot;
    }
  }
  __syncthreads();
  wave0_exscan(s_loc, P);
  __syncthreads();
  const uint16_t* cntx = s_cnt + (size_t)wave * P;
#pragma unroll
  for (int i = 0; i < kBigSteps; ++i) {
    if (packed[i] & 0x80000000u) {
      const uint32_t s = packed[i] & 0xFFFu;
      const int r = (int)cntx[s] + (int)((packed[i] >> 12) & 0x7FFFFu);   // rank among the block's pairs of slot s
      const int idx = lo + i * kWave + lane;
      s_sorted[s_loc[s] + r] = (s << 16) | (uint32_t)idx;
      if (row_of_pair) row_of_pair[p0 + idx] = s_off[s] + r;
    }
  }
  __syncthreads();
  for (int j = tid; j < n; j += kBigThreads) {
    const uint32_t v = s_sorted[j];
    const uint32_t s = v >> 16;
    pair_of_row[s_off[s] + (j - s_loc[s])] = (int32_t)(p0 + (v & 0xFFFFu));
  }
}

// Kernel 3 for 2 <= k <= 8 and P <= 512: the same stable scatter with the ranking done one TOKEN per lane.  A wave
// step then covers 64 tokens = 64 k pairs; a token's k slots are distinct (the ids of a top-k are, and a row of the
// expert map is injective), so a lane's k pairs never meet each other in a slot's lane mask and one mask round ranks
// all of them: the chain of dependent LDS round trips per wave shrinks from one per 64 pairs to one per 64 k pairs
// (the ranking, not memory, bounded the pair-per-lane kernel).  A block that does find a token with a repeated slot
// (ids that no top-k would produce) ranks pair per lane as k_scatter does, so the result is exact for any input.
//   tpw = tokens per wave, a multiple of 64.
template <int K>
__global__ __launch_bounds__(kBigThreads) void k_scatter_tok(const int32_t* __restrict__ slot_ids, const int32_t* __restrict__ counts,
                                                             const int32_t* __restrict__ base, int T, int P, int bits, int cht,
                                                             int tpw, int run, int32_t* __restrict__ offsets,
                                                             int32_t* __restrict__ pair_of_row, int32_t* __restrict__ row_of_pair) {
  constexpr int MAXP = 512;
  constexpr int STEPS = ((kBigPairs / K + kBigWaves - 1) / kBigWaves + kWave - 1) / kWave;  // 64-token steps per wave at most
  constexpr int NV = STEPS * K > kBigSteps ? STEPS * K : kBigSteps;                        // values per lane
  __shared__ uint16_t s_cnt[kBigWaves * MAXP];
  __shared__ int32_t s_off[MAXP + 1];    // first row of the block's pairs of slot s
  __shared__ int32_t s_loc[MAXP + 1];    // first position of slot s in the block's sorted order
  __shared__ uint32_t s_sorted[kBigPairs];  // slot << 16 | pair index inside the block, sorted by slot
  __shared__ int32_t s_w[2 * kBigWaves];
  __shared__ int s_dup;
  static_assert((size_t)kBigWaves * MAXP * 8 <= sizeof(s_sorted), "the lane masks borrow the sorted-pairs array");
  const int tid = threadIdx.x;
  const int wave = tid / kWave, lane = tid & (kWave - 1);
  const int t0 = blockIdx.x * cht, t1 = min(T, t0 + cht);
  const size_t p0 = (size_t)t0 * K;
  const int ntok = t1 - t0, n = ntok * K;                          // pairs of this block, <= kBigPairs
  const int wt0 = wave * tpw, wt1 = min(ntok, wt0 + tpw);          // this wave's tokens
  const int steps = tpw / kWave;                                   // <= STEPS
  uint32_t packed[NV];                                             // slot | rank << 12 | valid << 31; value st*K + j = choice j of token wt0 + 64 st + lane
  bool dup = false;
#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    const int tok = wt0 + st * kWave + lane;
    const bool valid = st < steps && tok < wt1;
    const int32_t* src = slot_ids + p0 + (size_t)tok * K;
#pragma unroll
    for (int j = 0; j < K; ++j) packed[st * K + j] = valid ? (uint32_t)src[j] : 0u;
  }
#pragma unroll
  for (int i = STEPS * K; i < NV; ++i) packed[i] = 0u;
  const int32_t* mybase = base + (size_t)blockIdx.x * P;
  const int32_t base_v = tid < P ? mybase[tid] : 0;                // this block's row of the scanned histogram
  const int32_t count_v = tid < P ? counts[tid] : 0;
  unsigned long long* s_mask = reinterpret_cast<unsigned long long*>(s_sorted);
  for (int i = tid; i < kBigWaves * P; i += kBigThreads) {
    s_cnt[i] = 0;
    s_mask[i] = 0ull;
  }
  if (tid == 0) s_dup = 0;
#pragma unroll
  for (int st = 0; st < STEPS; ++st) {
    if (st < steps && wt0 + st * kWave + lane < wt1) {
#pragma unroll
      for (int j = 1; j < K; ++j)
#pragma unroll
        for (int j2 = 0; j2 < j; ++j2) dup = dup || packed[st * K + j] == packed[st * K + j2];
    }
  }
  __syncthreads();
  if (dup) s_dup = 1;
  __syncthreads();
  const bool generic = s_dup != 0;                                 // block-uniform

  uint16_t* cnt = s_cnt + (size_t)wave * P;
  unsigned long long* mask = s_mask + (size_t)wave * P;
  if (!generic) {
    const unsigned long long lt = lanemask_lt();
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      if (st >= steps) break;
      const bool valid = wt0 + st * kWave + lane < wt1;
      uint32_t sl[K], old[K];
      unsigned long long peers[K];
#pragma unroll
      for (int j = 0; j < K; ++j) {
        sl[j] = packed[st * K + j];
        if (valid) __hip_atomic_fetch_or(&mask[sl[j]], 1ull << lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < K; ++j) {
        peers[j] = valid ? __hip_atomic_load(&mask[sl[j]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) : 0ull;
        old[j] = valid ? cnt[sl[j]] : 0u;
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < K; ++j) {
        const int before = __popcll(peers[j] & lt);
        if (valid && before == 0) {
          cnt[sl[j]] = (uint16_t)(old[j] + __popcll(peers[j]));
          mask[sl[j]] = 0ull;
        }
        packed[st * K + j] = sl[j] | ((old[j] + before) << 12) | (valid ? 0x80000000u : 0u);
      }
      __builtin_amdgcn_wave_barrier();
    }
  } else {
    // pair per lane, on the wave's run of `run` consecutive pairs (re-read: the values above are laid out per token)
    const int lo = wave * run, hi = min(n, lo + run);
    uint32_t pk[kBigSteps];
    load_pairs(slot_ids, p0, lo, hi, run / kWave, pk);
    rank_pairs<true>(lo, hi, run / kWave, bits, cnt, mask, pk);
#pragma unroll
    for (int i = 0; i < kBigSteps; ++i) packed[i] = pk[i];
  }
  __syncthreads();
  {
    // thread s: the waves' counts of slot s become running sums; then the block scans the slots' totals (positions in
    // the block's sorted order) and the call's counts (first rows) together
    int tot = 0;
    if (tid < P) {
#pragma unroll
      for (int w = 0; w < kBigWaves; ++w) {
        const int c = s_cnt[(size_t)w * P + tid];
        s_cnt[(size_t)w * P + tid] = (uint16_t)tot;
        tot += c;
      }
    }
    int first_row, first_pos, rows_total, pos_total;
    block_exscan2(count_v, tot, first_row, first_pos, rows_total, pos_total, s_w);
    if (tid < P) {
      s_off[tid] = first_row + base_v;
      s_loc[tid] = first_pos;
      if (blockIdx.x == 0) offsets[tid] = first_row;
    }
    if (tid == 0) {
      s_loc[P] = pos_total;
      if (blockIdx.x == 0) offsets[P] = rows_total;
    }
  }
  __syncthreads();
  if (!generic) {
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      if (st >= steps) break;
      const int tok = wt0 + st * kWave + lane;
      if (tok < wt1) {
        int32_t rows[K];
#pragma unroll
        for (int j = 0; j < K; ++j) {
          const uint32_t v = packed[st * K + j], s = v & 0xFFFu;
          const int r = (int)cnt[s] + (int)((v >> 12) & 0x7FFFFu);   // rank among the block's pairs of slot s
          s_sorted[s_loc[s] + r] = (s << 16) | (uint32_t)(tok * K + j);
          rows[j] = s_off[s] + r;
        }
        if (row_of_pair) {
          int32_t* dst = row_of_pair + p0 + (size_t)tok * K;        // K consecutive ints per lane
          if constexpr (K % 2 == 0) {
#pragma unroll
            for (int j = 0; j < K; j += 2) *reinterpret_cast<int2*>(dst + j) = make_int2(rows[j], rows[j + 1]);
          } else {
#pragma unroll
            for (int j = 0; j < K; ++j) dst[j] = rows[j];
          }
        }
      }
    }
  } else {
    const int lo = wave * run;
#pragma unroll
    for (int i = 0; i < kBigSteps; ++i) {
      if (packed[i] & 0x80000000u) {
        const uint32_t s = packed[i] & 0xFFFu;
        const int r = (int)cnt[s] + (int)((packed[i] >> 12) & 0x7FFFFu);
        const int idx = lo + i * kWave + lane;
        s_sorted[s_loc[s] + r] = (s << 16) | (uint32_t)idx;
        if (row_of_pair) row_of_pair[p0 + idx] = s_off[s] + r;
      }
    }
  }
  __syncthreads();
  for (int j = tid; j < n; j += kBigThreads) {
    const uint32_t v = s_sorted[j];
    const uint32_t s = v >> 16;
    pair_of_row[s_off[s] + (j - s_loc[s])] = (int32_t)(p0 + (v & 0xFFFFu));
  }
}

__global__ void k_zero_counts(int32_t* counts, int32_t* offsets, int P) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i <= P; i += gridDim.x * blockDim.x) {
    if (i < P) counts[i] = 0;
    offsets[i] = 0;
  }
}

// ------------------------------------------------------------------------------------------
// Tokens per block of the multi-block path: at most kBigPairs pairs, and small enough that a
// batch spreads over about 512 blocks: two 512-thread blocks fit a CU (LDS of k_scatter), so up to
// 2^20 tokens at k = 6 the whole grid is resident at once, and longer chunks mean longer runs per
// slot in the scatter's coalesced writes.
inline int chunk_tokens(int T, int k) {
  const int cap = kBigPairs / k;  // >= 192 for k <= 64
  int want = ew::ceil_div(T, 512);
  if (want < 16) want = 16;
  return want < cap ? want : cap;
}

template <int VPL>
int launch_permute(const float* logits, const int32_t* ids_in, const int32_t* aid, const int32_t* emap, int T, int E,
                   int k, int N, int P, int renorm, int32_t* ids_out, float* w_out, int32_t* slot_ids, int32_t* counts,
                   int32_t* offsets, int32_t* por, int32_t* rop, void* ws, hipStream_t st, const ew::WsPlanShape* shape = nullptr,
                   int S = 0, int32_t* plan = nullptr) {
  const long long n = (long long)T * k;
  const int bits = ew::ilog2_ceil(P);
  const int map_entries = (N + 1) * E;
  if (n <= g_small_pairs) {
    int nwaves = kSmallCnt / P;
    if (nwaves > 16) nwaves = 16;
    int run = ((int)n + nwaves - 1) / nwaves;
    run = (run + kWave - 1) / kWave * kWave;
    // the FFN plan rides on the single-block kernel when that has the 512 threads the plan needs
    SmallPlan fp{nullptr, 0, ew::WsPlanShape{}};
    const bool fused_plan = plan && nwaves * kWave >= 512;
    if (fused_plan) fp = SmallPlan{plan, S, *shape};
    if constexpr (VPL > 0) {
      hipLaunchKernelGGL((k_route_reroute<VPL>), dim3(ew::ceil_div(T, 4)), dim3(256), 0, st, logits, aid, emap, T, E, k, renorm,
                         ids_out, w_out, slot_ids);
      EW_LAUNCH_CHECK("k_route_reroute");
      hipLaunchKernelGGL((k_small<0>), dim3(1), dim3(nwaves * kWave), 0, st, logits, (const int32_t*)slot_ids, aid,
                         (const int32_t*)nullptr, T, E, k, P, map_entries, renorm, bits, run, ids_out, w_out, slot_ids, counts,
                         offsets, por, rop, fp);
    } else {
      hipLaunchKernelGGL((k_small<0>), dim3(1), dim3(nwaves * kWave), 0, st, logits, ids_in, aid, emap, T, E, k, P,
                         map_entries, renorm, bits, run, ids_out, w_out, slot_ids, counts, offsets, por, rop, fp);
    }
    EW_LAUNCH_CHECK("k_small");
    if (plan && !fused_plan) return ew::launch_ffn_ws_plan(counts, offsets, P, S, T, (int)n, *shape, plan, st);
    return EW_OK;
  }
  const int cht = chunk_tokens(T, k);
  const int nb = ew::ceil_div(T, cht);
  const int run = (int)ew::align_up((size_t)ew::ceil_div(cht * k, kBigWaves), kWave);
  int32_t* hist = (int32_t*)ws;
  hipLaunchKernelGGL((k_hist<VPL>), dim3(nb), dim3(kHistThreads), 0, st, logits, ids_in, aid, emap, T, E, k, P,
                     map_entries, renorm, cht, ids_out, w_out, slot_ids, hist);
  EW_LAUNCH_CHECK("k_hist");
  hipLaunchKernelGGL(k_colscan, dim3(ew::ceil_div(P, kScanCols)), dim3(kScanCols * kScanGroups), 0, st, hist, nb, P, counts);
  EW_LAUNCH_CHECK("k_colscan");
  const int tpw = (int)ew::align_up((size_t)ew::ceil_div(cht, kBigWaves), kWave);  // tokens per wave of the token-per-lane kernel
#define EW_SCATTER_TOK(KK)                                                                                                  \
  hipLaunchKernelGGL(k_scatter_tok<KK>, dim3(nb), dim3(kBigThreads), 0, st, slot_ids, counts, hist, T, P, bits, cht, tpw, run, \
                     offsets, por, rop)
  if (P <= 512 && k >= 2 && k <= 8) {
    switch (k) {
      case 2: EW_SCATTER_TOK(2); break;
      case 3: EW_SCATTER_TOK(3); break;
      case 4: EW_SCATTER_TOK(4); break;
      case 5: EW_SCATTER_TOK(5); break;
      case 6: EW_SCATTER_TOK(6); break;
      case 7: EW_SCATTER_TOK(7); break;
      default: EW_SCATTER_TOK(8); break;
    }
  } else if (P <= 512)
    hipLaunchKernelGGL(k_scatter<512>, dim3(nb), dim3(kBigThreads), 0, st, slot_ids, counts, hist, T, k, P, bits, cht, run,
                       offsets, por, rop);
  else
    hipLaunchKernelGGL(k_scatter<kMaxP>, dim3(nb), dim3(kBigThreads), 0, st, slot_ids, counts, hist, T, k, P, bits, cht, run,
                       offsets, por, rop);
#undef EW_SCATTER_TOK
  EW_LAUNCH_CHECK("k_scatter");
  if (plan) return ew::launch_ffn_ws_plan(counts, offsets, P, S, T, (int)n, *shape, plan, st);
  return EW_OK;
}

int check_permute_args(const char* who, const int32_t* aid, const int32_t* emap, int T, int k, int E, int N, int P,
                       int32_t* slot_ids, int32_t* counts, int32_t* offsets, int32_t* por, void* ws, size_t ws_bytes) {
  using ew::fail;
  if (T < 0 || k < 1 || E < 1 || N < 0 || P < 1) return fail(EW_ERR_INVALID_ARG, "%s: need T>=0, k>=1, E>=1, N>=0, P>=1", who);
  if (k > 64) return fail(EW_ERR_UNSUPPORTED, "%s: k=%d above the supported 64", who, k);
  if (P > kMaxP) return fail(EW_ERR_UNSUPPORTED, "%s: P=%d above the supported %d", who, P, kMaxP);
  if ((long long)T * k >= (1ll << 31)) return fail(EW_ERR_UNSUPPORTED, "%s: T*k must be below 2^31", who);
  if (!counts || !offsets) return fail(EW_ERR_INVALID_ARG, "%s: counts/offsets is NULL", who);
  if (T == 0) return EW_OK;
  if (!aid || !emap || !slot_ids || !por) return fail(EW_ERR_INVALID_ARG, "%s: NULL device pointer", who);
  const size_t need = moe_reroute_permute_workspace_bytes(T, k, P);
  if (need && (!ws || ((uintptr_t)ws & 255) || ws_bytes < need))
    return fail(EW_ERR_WORKSPACE, "%s: workspace needs %zu bytes aligned to 256 (got %zu at %p)", who, need, ws_bytes, ws);
  return EW_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Rerouting as separate canonical operators, each a launch and a pass over memory of its own:
// the unfused baseline the paper's fused kernel is compared with (Sec. 5.3, ExpertWeave-SingleOp).
namespace {
__global__ __launch_bounds__(256) void k_so_broadcast(const int32_t* __restrict__ aid, long long n, int k, int32_t* __restrict__ aid_b) {
  for (long long p = (long long)blockIdx.x * 256 + threadIdx.x; p < n; p += (long long)gridDim.x * 256) aid_b[p] = aid[(uint32_t)p / (uint32_t)k];
}
__global__ __launch_bounds__(256) void k_so_offsets(const int32_t* __restrict__ aid_b, const int32_t* __restrict__ ids, long long n,
                                                   int E, int32_t* __restrict__ off) {
  for (long long p = (long long)blockIdx.x * 256 + threadIdx.x; p < n; p += (long long)gridDim.x * 256) off[p] = aid_b[p] * E + ids[p];
}
__global__ __launch_bounds__(256) void k_so_gather(const int32_t* __restrict__ emap, const int32_t* __restrict__ off, long long n,
                                                  int32_t* __restrict__ slot) {
  for (long long p = (long long)blockIdx.x * 256 + threadIdx.x; p < n; p += (long long)gridDim.x * 256) slot[p] = emap[off[p]];
}
}  // namespace

extern "C" size_t moe_reroute_singleop_workspace_bytes(int T, int k) {
  if (T <= 0 || k < 1) return 0;
  return 2 * ew::align_up((size_t)T * k * sizeof(int32_t), 256);
}

extern "C" int moe_reroute_singleop(const int32_t* topk_ids, const int32_t* adapter_id, const int32_t* expert_map, int T, int k,
                                    int E, int N, int32_t* slot_ids, void* ws, size_t ws_bytes, void* stream) {
  using ew::fail;
  if (T < 0 || k < 1 || E < 1 || N < 0) return fail(EW_ERR_INVALID_ARG, "moe_reroute_singleop: need T>=0, k>=1, E>=1, N>=0");
  if ((long long)T * k >= (1ll << 31)) return fail(EW_ERR_UNSUPPORTED, "moe_reroute_singleop: T*k must be below 2^31");
  if (T == 0) return EW_OK;
  if (!topk_ids || !adapter_id || !expert_map || !slot_ids) return fail(EW_ERR_INVALID_ARG, "moe_reroute_singleop: NULL device pointer");
  const size_t need = moe_reroute_singleop_workspace_bytes(T, k);
  if (!ws || ((uintptr_t)ws & 255) || ws_bytes < need)
    return fail(EW_ERR_WORKSPACE, "moe_reroute_singleop: workspace needs %zu bytes aligned to 256 (got %zu at %p)", need, ws_bytes, ws);
  hipStream_t st = (hipStream_t)stream;
  const long long n = (long long)T * k;
  int32_t* aid_b = (int32_t*)ws;
  int32_t* off = (int32_t*)((char*)ws + need / 2);
  const int blocks = (int)((n + 255) / 256 < 16384 ? (n + 255) / 256 : 16384);
  hipLaunchKernelGGL(k_so_broadcast, dim3(blocks), dim3(256), 0, st, adapter_id, n, k, aid_b);
  EW_LAUNCH_CHECK("k_so_broadcast");
  hipLaunchKernelGGL(k_so_offsets, dim3(blocks), dim3(256), 0, st, aid_b, topk_ids, n, E, off);
  EW_LAUNCH_CHECK("k_so_offsets");
  hipLaunchKernelGGL(k_so_gather, dim3(blocks), dim3(256), 0, st, expert_map, off, n, slot_ids);
  EW_LAUNCH_CHECK("k_so_gather");
  return EW_OK;
}

// ------------------------------------------------------------------------------------------
// moe_reroute_permute for callers that cannot allocate: the block-histogram table lives in a
// file-scope device array instead of a caller workspace.  Each GPU holds its own copy of the array
// at its own address; the address is looked up once per device, with that device current, and only
// that pointer (never the array's name, which is a host-side stand-in) is handed to kernels.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kScratchMaxDev = 64;
std::atomic<void*> g_scratch_ptr[kScratchMaxDev];

int static_scratch(void** out) {
  int dev = 0;
  EW_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kScratchMaxDev) return ew::fail(EW_ERR_UNSUPPORTED, "moe_reroute_permute_static: device index %d above %d", dev, kScratchMaxDev - 1);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    EW_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return ew::fail(EW_ERR_HIP, "moe_reroute_permute_static: the scratch array has no device address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // racing first calls store the same address
  }
  *out = p;
  return EW_OK;
}
}  // namespace

extern "C" size_t moe_reroute_permute_static_max_bytes(void) { return kStaticScratchBytes; }

extern "C" int moe_reroute_permute_static(const int32_t* topk_ids, const int32_t* adapter_id, const int32_t* expert_map, int T,
                                          int k, int E, int N, int P, int32_t* slot_ids, int32_t* counts, int32_t* offsets,
                                          int32_t* pair_of_row, int32_t* row_of_pair, void* stream) {
  const size_t need = moe_reroute_permute_workspace_bytes(T, k, P);
  if (need > kStaticScratchBytes)
    return ew::fail(EW_ERR_UNSUPPORTED,
                    "moe_reroute_permute_static: T=%d k=%d P=%d needs %zu bytes of scratch, the built-in buffer holds %zu; "
                    "use moe_reroute_permute with a workspace",
                    T, k, P, need, kStaticScratchBytes);
  void* ws = nullptr;
  if (need) {
    int rc = static_scratch(&ws);
    if (rc != EW_OK) return rc;
  }
  // Every block of the histogram kernel writes its whole row of the table before anything reads it,
  // so nothing has to be cleared between calls; the table keeps the last call's contents.
  return moe_reroute_permute(topk_ids, adapter_id, expert_map, T, k, E, N, P, slot_ids, counts, offsets, pair_of_row,
                             row_of_pair, ws, need, stream);
}

extern "C" void ew_tune_route(int small_pairs) {
  g_small_pairs = small_pairs < 0 ? 0 : (small_pairs > kSmallPairs ? kSmallPairs : small_pairs);
}

// ==========================================================================================
extern "C" size_t moe_reroute_permute_workspace_bytes(int T, int k, int P) {
  if (T <= 0 || k < 1 || k > 64 || P < 1) return 0;
  // sized for the multi-block path even where the single-block one will run: the switch-over is a tuning knob
  const int nb = ew::ceil_div(T, chunk_tokens(T, k));
  return ew::align_up((size_t)nb * P * sizeof(int32_t), 256);
}

extern "C" int moe_route_topk(const float* logits, int T, int E, int k, int renormalize, int32_t* topk_ids,
                              float* topk_w, void* stream) {
  using ew::fail;
  if (T < 0 || E < 1 || k < 1 || k > E) return fail(EW_ERR_INVALID_ARG, "moe_route_topk: need T>=0 and 1<=k<=E (T=%d E=%d k=%d)", T, E, k);
  if (E > kMaxE || k > 64) return fail(EW_ERR_UNSUPPORTED, "moe_route_topk: supports E<=%d and k<=64 (E=%d k=%d)", kMaxE, E, k);
  if (T == 0) return EW_OK;
  if (!logits || !topk_ids || !topk_w) return fail(EW_ERR_INVALID_ARG, "moe_route_topk: NULL device pointer");
  hipStream_t st = (hipStream_t)stream;
  const int blocks = ew::ceil_div(T, 4) < 65536 ? ew::ceil_div(T, 4) : 65536;
#define EW_TOPK(V) hipLaunchKernelGGL((k_route_topk<V>), dim3(blocks), dim3(256), 0, st, logits, T, E, k, renormalize, topk_ids, topk_w)
  if (E <= 64) EW_TOPK(1);
  else if (E <= 128) EW_TOPK(2);
  else if (E <= 256) EW_TOPK(4);
  else if (E <= 512) EW_TOPK(8);
  else EW_TOPK(16);
#undef EW_TOPK
  EW_LAUNCH_CHECK("k_route_topk");
  return EW_OK;
}

extern "C" int moe_reroute_permute(const int32_t* topk_ids, const int32_t* adapter_id, const int32_t* expert_map, int T,
                                   int k, int E, int N, int P, int32_t* slot_ids, int32_t* counts, int32_t* offsets,
                                   int32_t* pair_of_row, int32_t* row_of_pair, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_permute_args("moe_reroute_permute", adapter_id, expert_map, T, k, E, N, P, slot_ids, counts, offsets,
                              pair_of_row, ws, ws_bytes);
  if (rc != EW_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (T == 0) {
    hipLaunchKernelGGL(k_zero_counts, dim3(1), dim3(256), 0, st, counts, offsets, P);
    EW_LAUNCH_CHECK("k_zero_counts");
    return EW_OK;
  }
  if (!topk_ids) return ew::fail(EW_ERR_INVALID_ARG, "moe_reroute_permute: topk_ids is NULL");
  return launch_permute<0>(nullptr, topk_ids, adapter_id, expert_map, T, E, k, N, P, 0, nullptr, nullptr, slot_ids, counts,
                           offsets, pair_of_row, row_of_pair, ws, st);
}

namespace {

int route_reroute_permute(const char* who, const float* logits, const int32_t* adapter_id, const int32_t* expert_map, int T, int E,
                          int k, int N, int P, int renormalize, int32_t* topk_ids, float* topk_w, int32_t* slot_ids,
                          int32_t* counts, int32_t* offsets, int32_t* pair_of_row, int32_t* row_of_pair, void* ws, size_t ws_bytes,
                          const ew::WsPlanShape* shape, int S, int32_t* plan, hipStream_t st) {
  using ew::fail;
  if (k > E) return fail(EW_ERR_INVALID_ARG, "%s: k=%d exceeds E=%d", who, k, E);
  int rc = check_permute_args(who, adapter_id, expert_map, T, k, E, N, P, slot_ids, counts, offsets, pair_of_row, ws, ws_bytes);
  if (rc != EW_OK) return rc;
  if (E > kMaxE) return fail(EW_ERR_UNSUPPORTED, "%s: supports E<=%d (E=%d)", who, kMaxE, E);
  if (T == 0) {
    hipLaunchKernelGGL(k_zero_counts, dim3(1), dim3(256), 0, st, counts, offsets, P);
    EW_LAUNCH_CHECK("k_zero_counts");
    return EW_OK;
  }
  if (!logits || !topk_ids || !topk_w) return fail(EW_ERR_INVALID_ARG, "%s: NULL device pointer", who);
#define EW_FUSED(V)                                                                                                      \
  return launch_permute<V>(logits, nullptr, adapter_id, expert_map, T, E, k, N, P, renormalize, topk_ids, topk_w, slot_ids, \
                           counts, offsets, pair_of_row, row_of_pair, ws, st, shape, S, plan)
  if (E <= 64) EW_FUSED(1);
  else if (E <= 128) EW_FUSED(2);
  else if (E <= 256) EW_FUSED(4);
  else if (E <= 512) EW_FUSED(8);
  else EW_FUSED(16);
#undef EW_FUSED
}

}  // namespace

extern "C" int moe_route_reroute_permute(const float* logits, const int32_t* adapter_id, const int32_t* expert_map, int T,
                                         int E, int k, int N, int P, int renormalize, int32_t* topk_ids, float* topk_w,
                                         int32_t* slot_ids, int32_t* counts, int32_t* offsets, int32_t* pair_of_row,
                                         int32_t* row_of_pair, void* ws, size_t ws_bytes, void* stream) {
  return route_reroute_permute("moe_route_reroute_permute", logits, adapter_id, expert_map, T, E, k, N, P, renormalize, topk_ids,
                               topk_w, slot_ids, counts, offsets, pair_of_row, row_of_pair, ws, ws_bytes, nullptr, 0, nullptr,
                               (hipStream_t)stream);
}

extern "C" int moe_route_reroute_permute_plan(const float* logits, const int32_t* adapter_id, const int32_t* expert_map, int T,
                                              int E, int k, int N, int P, int renormalize, int32_t* topk_ids, float* topk_w,
                                              int32_t* slot_ids, int32_t* counts, int32_t* offsets, int32_t* pair_of_row,
                                              int32_t* row_of_pair, void* ws, size_t ws_bytes, int H, int I, int S, int dtype,
                                              void* ffn_ws, size_t ffn_ws_bytes, void* stream) {
  using ew::fail;
  const char* who = "moe_route_reroute_permute_plan";
  if (T < 0 || k < 1 || P < 1 || H < 1 || I < 1 || S < 0) return fail(EW_ERR_INVALID_ARG, "%s: need T>=0, k>=1, P>=1, H>=1, I>=1, S>=0", who);
  ew::WsPlanShape shape{};
  int32_t* plan = nullptr;
  if (T > 0) {
    if (!ew::ffn_ws_shape_of_call(dtype, T, k, H, I, P, S, &shape))
      return fail(EW_ERR_UNSUPPORTED, "%s: the grouped FFN of these dimensions takes no plan (needs bf16, H and I multiples of 128, "
                  "P+S <= 2048, T*(k+S)*max(H,I)*2 < 2^32)", who);
    const size_t need = moe_grouped_ffn_workspace_bytes(T, k + S, H, I, P + S, dtype);
    if (!ffn_ws || ((uintptr_t)ffn_ws & 255) || ffn_ws_bytes < need)
      return fail(EW_ERR_WORKSPACE, "%s: the FFN workspace needs %zu bytes aligned to 256 (got %zu at %p)", who, need, ffn_ws_bytes, ffn_ws);
    plan = (int32_t*)ffn_ws;
  }
  return route_reroute_permute(who, logits, adapter_id, expert_map, T, E, k, N, P, renormalize, topk_ids, topk_w, slot_ids, counts,
                               offsets, pair_of_row, row_of_pair, ws, ws_bytes, &shape, S, plan, (hipStream_t)stream);
}
