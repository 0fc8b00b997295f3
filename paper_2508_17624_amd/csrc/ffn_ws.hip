// Grouped SwiGLU expert FFN, weight-stationary streaming kernel for gfx950 (bf16 MFMA).
//
// Paper Sec. 2.1: the GMM operator multiplies each contiguous chunk of permuted tokens with its
// expert's stacked weights; Sec. 4.1: it runs over the virtual weight tensor and never learns that
// adapters exist.  Sec. 5.2 names the cost this kernel is built around: with many adapters in a
// batch many more distinct experts are active, so every active slot's 16.5 MiB of weights has to
// be read although it serves only a few dozen to a few hundred rows.  The two products are
// therefore bound by (or close to) HBM bandwidth, and the kernel is organised around streaming:
//   * a workgroup (8 waves) owns one (slot, chunk of up to 32*NF rows, group of 256 weight rows)
//     and walks K in 64-element slabs; every weight element is read once per chunk;
//   * both operands reach LDS by LDS-direct global loads (no registers, no ds_write): 8 lanes
//     fetch one row's 128 bytes, so an instruction touches 8 whole cache lines instead of the 64
//     half-used lines a lane-per-row register load would (the L1 tag rate bound that variant);
//   * waves 0-3 issue only weight loads, waves 4-7 only token loads, each into a ring of its own:
//     the vector-memory counter retires in order, so keeping the two streams in different waves
//     lets each ring be awaited at its own depth.  The loads of the slab being prefetched are
//     issued between the MFMA groups of the slab being multiplied: a load instruction stalls its
//     wave while the memory pipeline is backed up, and the MFMAs in flight cover that stall;
//   * all 8 waves multiply: wave (wr, p) owns 64 weight rows (two 32-row A fragments) and the
//     32-token fragments p, p+2, ... of the chunk (v_mfma_f32_32x32x16_bf16, weights = A/rows,
//     tokens = B/columns), so 6 LDS reads feed 8 MFMAs;
//   * the workgroups are persistent (one per CU) and pull their items from per-XCD work lists that
//     a plan builds on the device from the counts (ffn_ws_plan.h; run by k_plan_ws here or by the
//     permutation's single-block kernel), see k_ffn_ws below;
//   * the model's shared experts are further slots of the same launch (slots P .. P+S-1, every token
//     each, weights from a second base pointer);
//   * decode shapes (chunks of at most 128 rows) run both products in one launch, second-product
//     items waiting for the activation rows they read (k_ffn_ws2), and start every item's walk over K
//     at a slab of its own so that workgroups streaming different slots in step do not meet on the
//     same memory channels.
// MODE 0 packs 16 gate rows and the 16 matching up rows into one A fragment, which makes SwiGLU a
// lane-local epilogue.  Inside a slab lane half h = lane/32 holds K elements [32h, 32h+32) on both
// operands (the contraction index may be permuted as long as both sides agree).
//
// LDS slab layout: [row][8 chunks of 16 B], chunk index XOR-ed with a function of the row so that
// the operand reads (32 rows x one logical chunk per half wave) spread over all banks (measured:
// zero bank-conflict cycles).  An LDS-direct load writes lane i's 16 bytes to base + 16*i, so the
// swizzle is applied on the global side: lane i fetches the logical chunk that belongs at
// physical position i.
//
// Slots with count 0 never appear in the plan and are never dereferenced; weight addresses stay
// inside the slot's own block, so the unmapped padding of the virtual tensor is never touched.
#include "ew_internal.h"
#include "ffn_ws_plan.h"

#include <atomic>
#include <type_traits>

namespace ew {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWsThreads = 512;

// round to nearest even: the hardware's conversion instruction
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }
// g / (1 + e^-g) with the hardware reciprocal (1 ulp, far below the bf16 rounding of the result): the
// epilogue applies it to 64 values per lane and item, and an exact division costs ten times as much
__device__ __forceinline__ float silu_f32(float g) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)); }

// swizzle term of LDS row r (depends on r mod 16): distinct over any 8 consecutive rows and over
// any 8 same-parity rows of 16, i.e. conflict-free for 128- and 256-byte-wide bank groups
__device__ __forceinline__ int swz(int r) { return ((r >> 1) ^ ((r & 1) << 2)) & 7; }

__global__ __launch_bounds__(512) void k_plan_ws(const int32_t* __restrict__ counts, const int32_t* __restrict__ offsets, int P,
                                                 int S, int sh_rows, int sh_first, WsPlanShape sh, int32_t* __restrict__ plan) {
  __shared__ WsPlanLds lds;
  ws_plan_build(counts, offsets, P, S, sh_rows, sh_first, sh, plan, lds);
}

struct WsArgs {
  const uint16_t* x;      // MODE 0: tokens [*, K]; MODE 1: activations [rows, K]
  const int32_t* counts;
  const int32_t* offsets;
  const int32_t* por;     // MODE 0 only; may be NULL
  const uint16_t* w;      // virtual weight tensor base
  const uint16_t* w_sh;   // weights of slots P .. P+S-1 (the shared experts), if the call has any
  int P;                  // routed slots
  int rows_routed;        // sorted rows of the routed slots; the shared experts' rows follow, sh_rows per slot
  int sh_rows;            // tokens of the call (rows of each shared expert); 1 if there is none
  uint16_t* out;          // [rows, NOUT]
  int32_t* plan;          // work plan (k_plan_ws); the kernel advances its counters
  size_t slot_stride;     // elements per slot
  int k, K, NOUT, groups, cap;
  int wait_ticks;         // longest rendezvous wait at the start of an item, in 10 ns ticks (0: never wait)
};

// Both products of a call in one launch (decode shapes): m[0] = gate/up + SwiGLU, m[1] = down.  A list's items are
// then numbered product-0 items first; done[r] counts the waves that have stored their part of the activation rows
// of the chunk starting at sorted row r (8 per product-0 item), and a product-1 item starts reading them once all
// have (done_target = 8 * feature groups of product 0).
struct WsArgs2 {
  WsArgs m[2];
  int32_t* done;
  int done_target;
  unsigned int spin_ticks;  // longest wait for done[], in 10 ns ticks: a safety net, never reached (see k_ffn_ws2)
};

template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));  // vmcnt(N), other counters untouched
}

// LDS operand reads, hidden from the compiler on purpose: it cannot tell which LDS-direct load
// an LDS read depends on and would wait for all of them; the waits are placed by hand instead.
// Issue and wait sit in one statement, so the outputs are valid when it ends.
// Two A fragments (4096 bytes apart) and NB (0..2) B fragments (8192 bytes apart).
template <int NB>
__device__ __forceinline__ void lds_read_a2_b(uint32_t wa, uint32_t tb, u32x4* a, u32x4* b) {
  if constexpr (NB == 0) {
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:4096\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a[0]), "=&v"(a[1]) : "v"(wa));
  } else if constexpr (NB == 1) {
    asm volatile("ds_read_b128 %0, %3\n\tds_read_b128 %1, %3 offset:4096\n\tds_read_b128 %2, %4\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a[0]), "=&v"(a[1]), "=&v"(b[0]) : "v"(wa), "v"(tb));
  } else {
    asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:4096\n\tds_read_b128 %2, %5\n\t"
                 "ds_read_b128 %3, %5 offset:8192\n\ts_waitcnt lgkmcnt(0)"
                 : "=&v"(a[0]), "=&v"(a[1]), "=&v"(b[0]), "=&v"(b[1]) : "v"(wa), "v"(tb));
  }
}
// Operand reads of one k-step for NB = 3 or 4 fragments, issued without waiting ...
template <int NB>
__device__ __forceinline__ void lds_issue_all(uint32_t wa, uint32_t tb, u32x4* a, u32x4* b) {
  if constexpr (NB == 3) {
    asm volatile("ds_read_b128 %0, %5\n\tds_read_b128 %1, %5 offset:4096\n\tds_read_b128 %2, %6\n\t"
                 "ds_read_b128 %3, %6 offset:8192\n\tds_read_b128 %4, %6 offset:16384"
                 : "=&v"(a[0]), "=&v"(a[1]), "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]) : "v"(wa), "v"(tb));
  } else {
    asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:4096\n\tds_read_b128 %2, %7\n\t"
                 "ds_read_b128 %3, %7 offset:8192\n\tds_read_b128 %4, %7 offset:16384\n\tds_read_b128 %5, %7 offset:24576"
                 : "=&v"(a[0]), "=&v"(a[1]), "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]), "=&v"(b[3]) : "v"(wa), "v"(tb));
  }
}
// ... and the point from which their results may be used.
template <int NB>
__device__ __forceinline__ void lds_landed(u32x4* a, u32x4* b) {
  if constexpr (NB == 3)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]));
  else
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a[0]), "+v"(a[1]), "+v"(b[0]), "+v"(b[1]), "+v"(b[2]), "+v"(b[3]));
}

constexpr int kPipeMinNB = 3;  // token fragments per wave from which the operand reads run a k-step ahead

// The eight (NB = 4) or six MFMAs of one k-step, with this wave's global loads number [lo, lo + 2) of the slab being
// prefetched issued after the first four and after the rest: a load instruction stalls the wave while the memory
// pipeline is backed up, and the MFMAs in flight cover that stall.
template <int NB, typename Issue>
__device__ __forceinline__ void ws_mfma_step(const u32x4* a, const u32x4* b, f32x16 (&acc)[2][4], Issue issue, int lo) {
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int i = 0; i < 2; ++i)
      acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[f]), acc[i][f], 0, 0, 0);
  issue(lo, lo + 1);
#pragma unroll
  for (int f = 2; f < NB; ++f)
#pragma unroll
    for (int i = 0; i < 2; ++i)
      acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[f]), acc[i][f], 0, 0, 0);
  issue(lo + 1, lo + 2);
}

// Large tiles (NB = 3 or 4 token fragments per wave): one K slab, software-pipelined across the slab boundary.
// The operand reads always run one k-step ahead of the MFMAs (two operand register sets), and that includes the
// boundary: the slab's first reads are issued right after the barrier that publishes it, and while they are in flight
// the MFMAs of the previous slab's last k-step execute (`carry`: its operands are still in set 1).  So no MFMA group
// ever waits for LDS behind a barrier.  On return set 1 holds the operands of this slab's last k-step, not yet
// multiplied: the caller passes carry = true for the next slab and calls ws_compute_tail after the last one.
template <int NB, typename Issue>
__device__ __forceinline__ void ws_compute_piped(uint32_t wa, uint32_t tb, f32x16 (&acc)[2][4], u32x4 (&a)[2][2], u32x4 (&b)[2][4],
                                                 bool carry, Issue issue) {
  lds_issue_all<NB>(wa, tb, a[0], b[0]);
  if (carry) ws_mfma_step<NB>(a[1], b[1], acc, issue, 0);
  else { issue(0, 1); issue(1, 2); }
  lds_landed<NB>(a[0], b[0]);
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    const int c = j & 1, n = c ^ 1;
    lds_issue_all<NB>(wa ^ (uint32_t)(16 * (j + 1)), tb ^ (uint32_t)(16 * (j + 1)), a[n], b[n]);
    ws_mfma_step<NB>(a[c], b[c], acc, issue, 2 * (j + 1));
    lds_landed<NB>(a[n], b[n]);
  }
}
template <int NB>
__device__ __forceinline__ void ws_compute_tail(f32x16 (&acc)[2][4], u32x4 (&a)[2][2], u32x4 (&b)[2][4]) {
  ws_mfma_step<NB>(a[1], b[1], acc, [](int, int) {}, 0);
}

// One K slab for a wave with NB (0..2) token fragments: 4 k-steps of 2 x NB MFMAs (small tiles are bound by the
// loads, not by LDS latency).  `issue(lo, hi)` enqueues this wave's LDS-direct loads number [lo, hi) of 8 for the
// slab being prefetched, spread between the MFMA groups.
template <int NB, typename Issue>
__device__ __forceinline__ void ws_compute(uint32_t wa, uint32_t tb, f32x16 (&acc)[2][4], Issue issue) {
  static_assert(NB < kPipeMinNB, "larger tiles take ws_compute_piped");
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // k-step j: the lane's chunk sits at byte offset o ^ (16 j) of its row
    const uint32_t wj = wa ^ (uint32_t)(16 * j), tj = tb ^ (uint32_t)(16 * j);
    u32x4 a[2], b[2];
    lds_read_a2_b<NB>(wj, tj, a, b);
#pragma unroll
    for (int f = 0; f < NB; ++f)
#pragma unroll
      for (int i = 0; i < 2; ++i)
        acc[i][f] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[f]), acc[i][f], 0, 0, 0);
    issue(2 * j, 2 * j + 2);
  }
}

// ------------------------------------------------------------------------------------------
// Work items and their claiming.
struct WsItem {
  int slot, m0, g, c, off, bts;  // slot < 0: no work left anywhere
  int wait_hi;                   // home-list items: counter value at which every item of this item's cohort is claimed
  int mode;                      // two-product launches: which product the item belongs to
};
#define EW_NO_ITEM WsItem{-1, 0, 0, 0, 0, 0, 0, 0}

// Work-list state of wave 0: lane i < 8 keeps list (home + i) % 8 -- its item total, its entry count
// and the last counter value seen (a lower bound: counters only grow).
struct WsLists {
  int total, n_ent, cnt;
  int tot0;  // two-product launches: items of the first product (they come first)
};

struct WsEnt {  // one plan entry
  int slot, nch, base, bts, c, off;
};

struct WsSched {       // what a workgroup needs to claim items; only wave 0 uses lists / pending
  int32_t* counters;
  int home;
  WsLists lists;
  int pending_t;       // list (relative to home) an asynchronous claim was issued on, -1: none
  int pending_w;       // its result, in lane pending_t (valid once the wave's vector-memory counter has drained)
};

__device__ __forceinline__ WsLists ws_lists_init(const WsArgs& a, const int32_t* counters, int home) {
  const int lane = threadIdx.x & 63;
  WsLists l{0, 0, 0, 0};
  if (lane < 8) {
    const int x = (home + lane) & 7;
    l.total = a.plan[8 + x] * a.groups;
    l.n_ent = a.plan[x];
    l.cnt = __hip_atomic_load(&counters[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return l;
}

__device__ __forceinline__ WsLists ws_lists_init2(const WsArgs2& aa, const int32_t* counters, int home) {
  const int lane = threadIdx.x & 63;
  WsLists l{0, 0, 0, 0};
  if (lane < 8) {
    const int x = (home + lane) & 7;
    const int chunks = aa.m[0].plan[8 + x];
    l.tot0 = chunks * aa.m[0].groups;
    l.total = l.tot0 + chunks * aa.m[1].groups;
    l.n_ent = aa.m[0].plan[x];
    l.cnt = __hip_atomic_load(&counters[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return l;
}

// Lane's entry of a list's entries [e0, e0 + 64).
__device__ __forceinline__ WsEnt ws_entries_load(const WsArgs& a, int x, int n, int e0) {
  const int e = e0 + (int)(threadIdx.x & 63);
  WsEnt v{0, 1, 0, 0, 0, 0};
  if (e < n) {
    const int32_t* en = a.plan + kPlanHdr + kEnt * (x * a.cap + e);
    v.slot = en[0]; v.nch = en[1]; v.base = en[2]; v.bts = en[3]; v.c = en[4]; v.off = en[5];
  }
  return v;
}

// Item number w of list x (whole wave): all lanes search the list's entries in parallel.  `first` holds the
// entries [0, 64) as loaded by ws_entries_load (so that the load can be issued ahead of time).
__device__ __forceinline__ WsItem ws_lookup(const WsArgs& a, int x, int w, int tot, int n, bool is_home, WsEnt first) {
  const int lane = threadIdx.x & 63;
  WsItem it = EW_NO_ITEM;
  for (int e0 = 0; e0 < n; e0 += 64) {
    const WsEnt v = e0 == 0 ? first : ws_entries_load(a, x, n, e0);
    const bool hit = e0 + lane < n && v.base * a.groups <= w && w < (v.base + v.nch) * a.groups;
    const unsigned long long m = __ballot(hit);
    if (m) {
      const int src = __ffsll((long long)m) - 1;
      const int b0 = __shfl(v.base, src, 64), chunks = __shfl(v.nch, src, 64);
      const int i = w - b0 * a.groups;
      it.slot = __shfl(v.slot, src, 64);
      it.bts = __shfl(v.bts, src, 64);
      it.m0 = (i % chunks) * it.bts;
      it.g = i / chunks;
      it.c = __shfl(v.c, src, 64);
      it.off = __shfl(v.off, src, 64);
      // the cohort this item starts with: 32 consecutive items of its entry (one per CU of the XCD)
      it.wait_hi = is_home ? min(min(b0 * a.groups + (i / 32 + 1) * 32, (b0 + chunks) * a.groups), tot) : 0;
      return it;
    }
  }
  return it;  // not reached: every claimed item lies in exactly one entry
}

// Claims the next work item for this workgroup (whole wave): the home list first, then the others
// (work stealing).  One lane claims with an atomic, then the entry search: two memory round trips.
__device__ __forceinline__ WsItem ws_fetch(const WsArgs& a, WsSched& sc) {
  const int lane = threadIdx.x & 63;
  WsLists& l = sc.lists;
  for (;;) {
    const unsigned long long avail = __ballot(lane < 8 && l.cnt < l.total);
    if (!avail) return EW_NO_ITEM;
    const int t = __ffsll((long long)avail) - 1;
    int w = 0;
    if (lane == t) {
      w = atomicAdd(&sc.counters[(sc.home + t) & 7], 1);
      l.cnt = w + 1;
    }
    w = __shfl(w, t, 64);
    const int tot = __shfl(l.total, t, 64), n = __shfl(l.n_ent, t, 64);
    if (w >= tot) continue;  // lost the race for the last items of this list (its cnt is now >= total)
    const int x = (sc.home + t) & 7;
    return ws_lookup(a, x, w, tot, n, t == 0, ws_entries_load(a, x, n, 0));
  }
}

// The item wave 0 left in LDS, in scalar registers (wait_hi stays with wave 0, the only one to use it).
__device__ __forceinline__ WsItem ws_item_from_lds(const int32_t* s_next, int wait_hi) {
  WsItem it;
  it.slot = __builtin_amdgcn_readfirstlane(s_next[0]);
  it.m0 = __builtin_amdgcn_readfirstlane(s_next[1]);
  it.g = __builtin_amdgcn_readfirstlane(s_next[2]);
  it.c = __builtin_amdgcn_readfirstlane(s_next[3]);
  it.off = __builtin_amdgcn_readfirstlane(s_next[4]);
  it.bts = __builtin_amdgcn_readfirstlane(s_next[5]);
  it.mode = __builtin_amdgcn_readfirstlane(s_next[6]);
  it.wait_hi = __builtin_amdgcn_readfirstlane(wait_hi);
  return it;
}

// The claim in two halves, so that its first memory round trip hides behind an item's last K slab: the atomic is
// issued without waiting for its result ...
__device__ __forceinline__ void ws_claim_issue(WsSched& sc) {
  const int lane = threadIdx.x & 63;
  const unsigned long long avail = __ballot(lane < 8 && sc.lists.cnt < sc.lists.total);
  sc.pending_t = avail ? __ffsll((long long)avail) - 1 : -1;
  if (lane == sc.pending_t)
    sc.pending_w = __hip_atomic_fetch_add(&sc.counters[(sc.home + sc.pending_t) & 7], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// ... and picked up later in two steps: the entries of the list the claim went to are fetched (their load in flight
// while the caller does something else), then the item is looked up.  If that list ran out in the meantime, the
// ordinary claim takes over.
__device__ __forceinline__ WsEnt ws_claim_entries(const WsArgs& a, const WsSched& sc) {
  if (sc.pending_t < 0) return WsEnt{0, 1, 0, 0, 0, 0};
  return ws_entries_load(a, (sc.home + sc.pending_t) & 7, __shfl(sc.lists.n_ent, sc.pending_t, 64), 0);
}
__device__ __forceinline__ WsItem ws_claim_finish(const WsArgs& a, WsSched& sc, WsEnt first) {
  const int t = sc.pending_t;
  sc.pending_t = -1;
  if (t < 0) return ws_fetch(a, sc);
  const int lane = threadIdx.x & 63;
  if (lane == t) sc.lists.cnt = sc.pending_w + 1;
  const int w = __shfl(sc.pending_w, t, 64);
  const int tot = __shfl(sc.lists.total, t, 64), n = __shfl(sc.lists.n_ent, t, 64);
  if (w >= tot) return ws_fetch(a, sc);
  return ws_lookup(a, (sc.home + t) & 7, w, tot, n, t == 0, first);
}

// The same for a two-product launch: item number w of a list belongs to the first product if w < tot0.
__device__ __forceinline__ WsItem ws_lookup2(const WsArgs2& aa, int x, int w, int tot0, int n, WsEnt first) {
  const int mode = w >= tot0 ? 1 : 0;
  WsItem it = ws_lookup(aa.m[mode], x, w - mode * tot0, 0, n, false, first);
  it.mode = mode;
  return it;
}
__device__ __forceinline__ WsItem ws_fetch2(const WsArgs2& aa, WsSched& sc) {
  const int lane = threadIdx.x & 63;
  WsLists& l = sc.lists;
  for (;;) {
    const unsigned long long avail = __ballot(lane < 8 && l.cnt < l.total);
    if (!avail) return EW_NO_ITEM;
    const int t = __ffsll((long long)avail) - 1;
    int w = 0;
    if (lane == t) {
      w = atomicAdd(&sc.counters[(sc.home + t) & 7], 1);
      l.cnt = w + 1;
    }
    w = __shfl(w, t, 64);
    const int tot = __shfl(l.total, t, 64), tot0 = __shfl(l.tot0, t, 64), n = __shfl(l.n_ent, t, 64);
    if (w >= tot) continue;
    const int x = (sc.home + t) & 7;
    return ws_lookup2(aa, x, w, tot0, n, ws_entries_load(aa.m[0], x, n, 0));
  }
}
__device__ __forceinline__ WsItem ws_claim_finish2(const WsArgs2& aa, WsSched& sc, WsEnt first) {
  const int t = sc.pending_t;
  sc.pending_t = -1;
  if (t < 0) return ws_fetch2(aa, sc);
  const int lane = threadIdx.x & 63;
  if (lane == t) sc.lists.cnt = sc.pending_w + 1;
  const int w = __shfl(sc.pending_w, t, 64);
  const int tot = __shfl(sc.lists.total, t, 64), tot0 = __shfl(sc.lists.tot0, t, 64), n = __shfl(sc.lists.n_ent, t, 64);
  if (w >= tot) return ws_fetch2(aa, sc);
  return ws_lookup2(aa, (sc.home + t) & 7, w, tot0, n, first);
}

// ------------------------------------------------------------------------------------------
// LDS of a workgroup: the two operand rings during an item's K loop, the output tile between two items.
template <int MODE, int NF>
struct WsCfg {
  static constexpr int BT = 32 * NF;                  // tokens per chunk
  static constexpr int TSTAGE = BT * 128;             // bytes of one token slab
  static constexpr int WSTAGE = 256 * 128;            // bytes of one weight slab
  static constexpr int TST = NF == 8 ? 2 : 3;         // token ring depth
  static constexpr int WST = NF <= 2 ? 4 : 3;         // weight ring depth (NF = 8: the two rings fill all 160 KB)
  static constexpr int FB = MODE == 0 ? 128 : 256;    // output features per workgroup
  static constexpr int FA = MODE == 0 ? 16 : 32;      // output features per A fragment
  static constexpr int RINGS = WST * WSTAGE + TST * TSTAGE;
  // Output tile [BT rows][FB features] bf16 staged for coalesced stores.  The row pitch is 8 bytes more than the
  // row, i.e. 2 banks: the 32 rows a half wave writes 8 bytes each to then cover all 64 banks exactly once.
  static constexpr int OPITCH = FB * 2 + 8;
  static constexpr int OTILE = BT * OPITCH;
  // Decode shapes (NF < 8) are a pure weight stream: their output tile is a few rows, stored straight from the
  // registers, the next item is claimed while the current one streams and kept beyond the rings.  The 256-row
  // shape stages its tile in LDS and claims late; the next item sits behind the tile.
  static constexpr bool EARLY = NF < 8;
  static constexpr int NEXT_OFF = EARLY ? RINGS : (OTILE + 15) / 16 * 16;   // the next item, handed from wave 0 to the others
  static constexpr int LDS = RINGS > NEXT_OFF + 32 ? RINGS : NEXT_OFF + 32;
  static_assert(LDS <= 160 * 1024, "LDS budget of a CU");
};

// Source rows (tokens for MODE 0, activation rows for MODE 1) of the lane's eight token-load instructions for an
// item: instruction i covers chunk rows L0 + 32 i (rows past the chunk's end: clamped duplicates, outputs masked).
template <int MODE>
__device__ __forceinline__ void ws_gather_rows(const WsArgs& a, const WsItem& it, int L0, int (&src)[8]) {
  const int rc = min(it.bts, it.c - it.m0);
  // a shared expert's rows are the tokens in order (item-uniform branch)
  const bool shared = MODE == 0 && it.slot >= a.P;
  const int first = it.off + it.m0 - (shared ? a.rows_routed + (it.slot - a.P) * a.sh_rows : 0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = first + min(L0 + 32 * i, rc - 1);
    if (MODE == 0 && !shared)
      src[i] = (a.por ? a.por[row] : row) / a.k;
    else
      src[i] = row;
  }
}

// One work item of one workgroup: K loop, then the hand-over to the next item.  NFL = live 32-token fragments of
// the chunk.  Every wave issues a compile-time number of loads per slab, so the waits can be counted.
//   tsrc   source rows of this item's token loads (ws_gather_rows), overwritten with the next item's
//   returns the next item (claimed by wave 0 behind this item's last slab)
//   M2     a two-product launch (aa = its arguments, a = aa->m[MODE]); decode shapes only
template <int MODE, int NF, int NFL, bool M2 = false>
__device__ __forceinline__ WsItem ws_body(const WsArgs& a, unsigned char* s_lds, const WsItem& cur, int (&tsrc)[8], WsSched& sc,
                                          const WsArgs2* aa = nullptr) {
  using C = WsCfg<MODE, NF>;
  static_assert(!M2 || C::EARLY, "two-product launches exist for the decode shapes");
  constexpr int NLD_T = NFL;                         // token load instructions per token wave and slab (8 rows each)
  // A chunk with few live fragments needs less LDS per token slab: spend the rest on ring depth
  // (token rows that miss L2 take longer to arrive than one slab takes to multiply).
  constexpr int TSTAGE = NFL * 4096;
  constexpr int TST = (C::TST * C::TSTAGE) / TSTAGE < 4 ? (C::TST * C::TSTAGE) / TSTAGE : 4;
  constexpr int NB0 = (NFL + 1) / 2, NB1 = NFL / 2;  // token fragments of the waves with p = 0 / p = 1
  unsigned char* s_w = s_lds;
  unsigned char* s_t = s_lds + C::WST * C::WSTAGE;
  const int s = cur.slot, g = cur.g, off_m0 = cur.off + cur.m0, rc = min(cur.bts, cur.c - cur.m0);
  const int K = a.K, NOUT = a.NOUT, nk = K >> 6;
  // Decode shapes: every item starts its walk over K at a slab of its own (a function of the item, so results do not
  // depend on which workgroup runs it).  The workgroups stream different slots in step, and slots lie a whole number
  // of MiB apart: walking them all from slab 0 made every workgroup ask the same memory channels at the same time
  // (measured: 7 to 14 % slower).  The 256-row shape keeps slab 0: its workgroups share operands in L2 only while
  // they walk in step, and measured 2 % slower with any rotation.
  const int rot = NF == 8 ? 0 : (s * 5 + g * 3) % nk;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the role branches scalar
  const int r32 = lane & 31, h = lane >> 5;
  const bool is_w = wave < 4;  // waves 0-3 load weights, waves 4-7 load tokens
  const int lw = wave & 3;

  // ---- LDS-direct load sources.  Instruction q = lw + 4i of a slab covers LDS rows [8q, 8q+8):
  // lane l -> row L = 8q + l/8, physical chunk l%8, i.e. logical chunk (l%8) ^ swz(L); swz(L)
  // depends on L mod 16 only, so it is the same for all of a lane's instructions (rows 32 apart).
  const int L0 = 8 * lw + (lane >> 3);
  const uint32_t lc16 = (uint32_t)(((lane & 7) ^ swz(L0)) << 4);
  // weights: LDS row L -> slot row.  MODE 0 keeps A-fragment order (16 gate rows, then the 16
  // matching up rows), so 32 LDS rows further on is 16 features further on: a constant stride.
  const unsigned char* wbase = reinterpret_cast<const unsigned char*>(
      s < a.P ? a.w + (size_t)s * a.slot_stride : a.w_sh + (size_t)(s - a.P) * a.slot_stride);
  uint32_t w_off0;
  int w_first_feat;  // feature of this wave's first instruction (wave-uniform up to the low 4 bits)
  if (MODE == 0) {
    w_first_feat = g * 128 + (L0 >> 5) * 16;
    w_off0 = (uint32_t)(((L0 & 16) ? NOUT : 0) + w_first_feat + (L0 & 15)) * (uint32_t)(K * 2) + lc16;
  } else {
    w_first_feat = g * 256 + 8 * lw;
    w_off0 = (uint32_t)(g * 256 + L0) * (uint32_t)(K * 2) + lc16;
  }
  const uint32_t w_stride = (uint32_t)(MODE == 0 ? 16 : 32) * (uint32_t)(K * 2);
  const int w_fstep = MODE == 0 ? 16 : 32;
  // tokens: gathered rows, one offset per instruction
  uint32_t t_off[NLD_T];
#pragma unroll
  for (int i = 0; i < NLD_T; ++i) t_off[i] = is_w ? 0u : (uint32_t)tsrc[i] * (uint32_t)(K * 2) + lc16;
  const unsigned char* xbase = reinterpret_cast<const unsigned char*>(a.x);
  const uint32_t my_stage = is_w ? C::WSTAGE : TSTAGE;
  const int my_depth = is_w ? C::WST : TST;
  unsigned char* my_ring = (is_w ? s_w : s_t) + lw * 1024;

  // Loads number [lo, hi) of one slab of this wave: a weight wave has 8, a token wave NLD_T.
  auto issue = [&](int kt, int slot, int lo, int hi) {
    const size_t kofs = (size_t)((min(kt, nk - 1) + rot) % nk) * 128;
    unsigned char* dst = my_ring + slot * my_stage;
    if (is_w) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (i < lo || i >= hi) continue;
        // a fragment past the last feature (partial last group) re-reads the wave's first rows; never stored
        const uint32_t o = w_off0 + (w_first_feat + i * w_fstep < NOUT ? i * w_stride : 0u);
        // Weights are read once and should not displace the token rows in L2.  Which cache-policy
        // bit does that best was measured: sc1 for the large-chunk (prefill) shape, where token
        // rows are re-read by every feature group (7 % faster than nt, 15 % than default); nt for
        // the decode shapes, which are a pure weight stream (5 % faster than sc1).
        if constexpr (NF == 8)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(wbase + kofs + o),
                                           (__attribute__((address_space(3))) void*)(dst + i * 4096), 16, 0, 16);
        else
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(wbase + kofs + o),
                                           (__attribute__((address_space(3))) void*)(dst + i * 4096), 16, 0, 2);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NLD_T; ++i) {
        if (i < lo || i >= hi) continue;
        // Two-product launches: the activation rows were written by other workgroups of this launch, with agent-scope
        // stores; agent-scope loads (sc1) read them at the point of coherence, past this XCD's L2 and the CU's L1.
        if constexpr (M2 && MODE == 1)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xbase + kofs + t_off[i]),
                                           (__attribute__((address_space(3))) void*)(dst + i * 4096), 16, 0, 16);
        else
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xbase + kofs + t_off[i]),
                                           (__attribute__((address_space(3))) void*)(dst + i * 4096), 16, 0, 0);
      }
    }
  };

  // ---- operand read addresses: lane reads row r32 of a fragment, logical chunk 4h + j in k-step j
  const int wr = wave >> 1, p = wave & 1;
  const uint32_t lane_off = (uint32_t)(r32 * 128 + (((4 * h) ^ swz(r32)) << 4));
  const uint32_t lds_w = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)s_w + wr * 8192 + lane_off;
  const uint32_t lds_t = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)s_t + p * 4096 + lane_off;

  f32x16 acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int f = 0; f < 4; ++f)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][f][e] = 0.f;

  if constexpr (M2 && MODE == 1) {
    // The chunk's activation rows are complete once every wave of every first-product item of the chunk has stored
    // its part.  Those items were claimed before this one (same list, lower numbers) by workgroups that never wait
    // while they work on them, so the count gets there; the time limit is a safety net that is never reached.
    if (!is_w) {
      const int32_t* flag = aa->done + off_m0;
      const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
      while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < aa->done_target &&
             __builtin_amdgcn_s_memrealtime() - t0 < (unsigned long long)aa->spin_ticks)
        __builtin_amdgcn_s_sleep(2);
      // No cache invalidation here (an agent-scope acquire would drop this XCD's whole L2, weights included): the
      // rows are read with agent-scope loads instead, see `issue`.  The loads are issued after this point.
      asm volatile("" ::: "memory");
    }
  }
  // prologue: slabs 0 .. depth-2 in flight
  for (int kt = 0; kt < my_depth - 1 && kt < nk; ++kt) issue(kt, kt, 0, 8);
  WsItem nx{-1, 0, 0, 0, 0, 0, 0};
  [[maybe_unused]] WsEnt claim_ent{0, 1, 0, 0, 0, 0};
  // The loop exists once per fragment count so that the accumulators stay in place (a branch on
  // p inside one loop makes the compiler shuffle all of them through copies every iteration).
  auto main_loop = [&](auto nb_tag) {
    constexpr int NB = decltype(nb_tag)::value;
    int my_slot = my_depth - 1;  // ring slot the next issued slab goes to
    int wslot = 0, tslot = 0;    // ring slots of the slab being multiplied
    [[maybe_unused]] u32x4 opa[2][2], opb[2][4];  // operand register sets of the pipelined (large-tile) loop
    for (int kt = 0; kt < nk; ++kt) {
      // This wave's loads of slab kt have landed once only the newer slabs are outstanding: depth-2
      // of them in the steady state, fewer in the item's last slabs, for which nothing is issued
      // any more.  The load counts per slab are compile-time constants, so the waits can be exact.
      {
        const int rem = nk - 1 - kt;
        const int newer = rem < my_depth - 2 ? rem : my_depth - 2;
        if (is_w) {
          if (newer >= 2) wait_vm<16>(); else if (newer == 1) wait_vm<8>(); else wait_vm<0>();
        } else {
          if (newer >= 2) wait_vm<2 * NLD_T>(); else if (newer == 1) wait_vm<NLD_T>(); else wait_vm<0>();
        }
      }
      // Everybody's part of slab kt has landed; everybody is done reading slab kt-1 (in the pipelined
      // loop its last operands sit in registers by now, their MFMAs follow this barrier).
      __builtin_amdgcn_s_barrier();
      // The last slab: nothing of this wave is in flight any more, so the claim of the next item can go out (wave 0)
      // and come back while the slab is multiplied.  Claiming this late keeps claim order close to finishing order:
      // workgroups that finish together get neighbouring items, which share operands (see k_ffn_ws).
      if constexpr (!C::EARLY) {
        if (kt == nk - 1 && wave == 0) ws_claim_issue(sc);
      } else if (wave == 0) {
        // Decode shapes: the claim goes out with the first slab and is picked up after the last one; the plan
        // entries it needs are fetched behind the last slab.  No wave ever waits for either.
        if (kt == 0) ws_claim_issue(sc);
        if (kt == nk - 1) claim_ent = ws_claim_entries(a, sc);
      }
      const int kt_next = kt + my_depth - 1, slot_next = my_slot;
      // Token loads go out first thing (their ring is the shallower one), the weight loads are spread between
      // the MFMA groups.  (Measured: any other split of the two streams over the slab runs at the same speed.)
      if (!is_w && kt_next < nk) issue(kt_next, slot_next, 0, 8);
      auto issue_w = [&](int lo, int hi) {
        if (kt_next >= nk) return;  // the item's last slabs are already in flight
        if (is_w) issue(kt_next, slot_next, lo, hi);
      };
      if constexpr (NB >= kPipeMinNB)
        ws_compute_piped<NB>(lds_w + wslot * C::WSTAGE, lds_t + tslot * TSTAGE, acc, opa, opb, kt > 0, issue_w);
      else
        ws_compute<NB>(lds_w + wslot * C::WSTAGE, lds_t + tslot * TSTAGE, acc, issue_w);
      my_slot = my_slot + 1 == my_depth ? 0 : my_slot + 1;
      wslot = wslot + 1 == C::WST ? 0 : wslot + 1;
      tslot = tslot + 1 == TST ? 0 : tslot + 1;
    }
    if constexpr (NB >= kPipeMinNB) ws_compute_tail<NB>(acc, opa, opb);
  };
  if (NB0 == NB1 || p == 0) main_loop(std::integral_constant<int, NB0>{});
  else main_loop(std::integral_constant<int, NB1>{});
  wait_vm<0>();  // no LDS-direct load may outlive its ring; the claim's result is in, too

  int32_t* s_next = reinterpret_cast<int32_t*>(s_lds + C::NEXT_OFF);
  auto publish = [&]() {  // wave 0 -> LDS
    if (wave == 0 && lane == 0) {
      s_next[0] = nx.slot; s_next[1] = nx.m0; s_next[2] = nx.g; s_next[3] = nx.c; s_next[4] = nx.off; s_next[5] = nx.bts;
      s_next[6] = nx.mode;
    }
  };
  auto take_next = [&]() {  // LDS -> every wave; the token waves fetch the next item's row map (in flight during the stores)
    nx = ws_item_from_lds(s_next, nx.wait_hi);
    int nsrc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (!is_w && nx.slot >= 0) {
      if constexpr (M2) {
        if (nx.mode == 0) ws_gather_rows<0>(aa->m[0], nx, L0, nsrc);
        else ws_gather_rows<1>(aa->m[1], nx, L0, nsrc);
      } else {
        ws_gather_rows<MODE>(a, nx, L0, nsrc);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) tsrc[i] = nsrc[i];
  };
  // Accumulator element e of lane l: A row 8*(e/4) + 4*(l/32) + e%4, token l%32.  `put(i, ff, q, o)`: four consecutive
  // features of token row (p + 2 ff) * 32 + l%32, starting at feature (wr*2 + i) * FA + 8 q + 4 (l/32) of the group.
  auto for_each_quad = [&](auto put) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int ff = 0; ff < 4; ++ff) {
        const int tr = (p + 2 * ff) * 32 + r32;
        if (ff < NB0 && tr < rc) {
          const f32x16& v = acc[i][ff];
          if (MODE == 0) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {  // A rows 8q + 4h + 0..3 are gate rows, +16 the matching up rows
              ushort4 o;
              o.x = f32_to_bf16(silu_f32(v[4 * q + 0]) * v[8 + 4 * q + 0]);
              o.y = f32_to_bf16(silu_f32(v[4 * q + 1]) * v[8 + 4 * q + 1]);
              o.z = f32_to_bf16(silu_f32(v[4 * q + 2]) * v[8 + 4 * q + 2]);
              o.w = f32_to_bf16(silu_f32(v[4 * q + 3]) * v[8 + 4 * q + 3]);
              put(i, tr, q, o);
            }
          } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              ushort4 o;
              o.x = f32_to_bf16(v[4 * q + 0]);
              o.y = f32_to_bf16(v[4 * q + 1]);
              o.z = f32_to_bf16(v[4 * q + 2]);
              o.w = f32_to_bf16(v[4 * q + 3]);
              put(i, tr, q, o);
            }
          }
        }
      }
  };
  if constexpr (C::EARLY) {
    // ---- hand-over, decode shapes: the next item (claimed during the K loop) goes to the other waves, then the few
    // output rows leave straight from the registers.  The barrier also keeps the next item's first loads out of
    // ring slots that a slower wave still reads.
    if (wave == 0) {
      if constexpr (M2) nx = ws_claim_finish2(*aa, sc, claim_ent);
      else nx = ws_claim_finish(a, sc, claim_ent);
    }
    publish();
    __syncthreads();
    take_next();
    for_each_quad([&](int i, int tr, int q, ushort4 o) {
      const int f0 = g * C::FB + (wr * 2 + i) * C::FA;
      if (f0 < NOUT) {
        uint16_t* dst = a.out + (size_t)(off_m0 + tr) * NOUT + f0 + 4 * h + 8 * q;
        if constexpr (M2 && MODE == 0) {
          // agent-scope store: written through to the point of coherence of the GPU's XCDs
          unsigned long long v;
          __builtin_memcpy(&v, &o, 8);
          __hip_atomic_store(reinterpret_cast<unsigned long long*>(dst), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
          *reinterpret_cast<ushort4*>(dst) = o;
        }
      }
    });
    if constexpr (M2 && MODE == 0) {
      // This wave's part of the chunk's activation rows is stored once its stores have been acknowledged; then it is
      // counted (every wave of every item counts, whether it had rows to store or not).  A release fence would also
      // write back this XCD's whole L2, which holds nothing of ours that anyone else reads.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      if (lane == 0) __hip_atomic_fetch_add(aa->done + off_m0, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  } else {
    // ---- hand-over, 256-row shape.  The output tile goes through LDS (the rings are dead now): a lane holds 4
    // consecutive features of one token per accumulator quad, which would be 8-byte stores scattered over 32 rows
    // per instruction (measured: 5 to 12 us per item for the second product that way).  Wave 0 completes the claim
    // it issued behind the last slab while the tile is written; the token waves fetch the next item's row map while
    // the tile is stored, 16 bytes per lane along the rows.
    WsEnt first{0, 1, 0, 0, 0, 0};
    if (wave == 0) first = ws_claim_entries(a, sc);  // in flight across the barrier and the tile write
    __syncthreads();  // every wave is done reading operands
    for_each_quad([&](int i, int tr, int q, ushort4 o) {
      *reinterpret_cast<ushort4*>(s_lds + tr * C::OPITCH + ((wr * 2 + i) * C::FA + 4 * h + 8 * q) * 2) = o;
    });
    if (wave == 0) nx = ws_claim_finish(a, sc, first);
    publish();
    __syncthreads();  // the tile and the next item are in LDS
    take_next();
    constexpr int CPR = C::FB / 8;  // 16-byte pieces per tile row
    uint16_t* obase = a.out + (size_t)off_m0 * NOUT + g * C::FB;
    for (int idx = tid; idx < rc * CPR; idx += kWsThreads) {
      const int row = idx / CPR, pc = idx % CPR;
      if (g * C::FB + pc * 8 < NOUT) {
        const uint2* src = reinterpret_cast<const uint2*>(s_lds + row * C::OPITCH + pc * 16);
        const uint2 lo = src[0], hi = src[1];
        *reinterpret_cast<uint4*>(obase + (size_t)row * NOUT + pc * 8) = make_uint4(lo.x, lo.y, hi.x, hi.y);
      }
    }
  }
  return nx;
}

// MODE 0: out = silu(x.Wg^T) * (x.Wu^T), Wg rows [0,NOUT), Wu rows [NOUT,2NOUT) of the slot.
// MODE 1: out = x.W^T, W rows [0,NOUT) of the slot.
// NF: 32-token fragments per row chunk (1, 2, 4 or 8); sizes the LDS rings and the plan's chunks.
template <int MODE, int NF>
__global__ __launch_bounds__(kWsThreads) void k_ffn_ws(WsArgs a) {
  using C = WsCfg<MODE, NF>;
  __shared__ __align__(1024) unsigned char s_lds[C::LDS];

  // Persistent workgroups: one per CU, each pulls (slot, chunk, feature group) items from the work
  // list of its own XCD and, once that is empty, from the others', so the grid drains evenly and
  // ends when every counter has run past its list.
  //
  // Items that share operands must start together to share them in L2: a workgroup streams 2 MB
  // per item through a 4 MB L2 that 32 CUs use, so a row fetched by one workgroup is gone a few
  // microseconds later.  Measured: with items of one duration the workgroups of an XCD stay in
  // step by themselves and the fabric traffic is 1.03x the compulsory bytes; with the ragged
  // chunk sizes of a real batch it was 1.6x.  Therefore
  //   * the next item is claimed when the current one is nearly finished -- behind its last K slab,
  //     which hides the claim's latency -- so claim order is finishing order and the workgroups
  //     that finish together get neighbouring items, i.e. the same slot;
  //   * optionally (wait_ticks > 0, a tuning aid; off by default because it no longer pays) a workgroup
  //     of the 256-row shape then waits, for at most wait_ticks, until all items of its cohort are
  //     claimed (the list counter says so), so that the group that will share rows starts as one.
  // That wait is bounded and nothing else ever waits for another workgroup, so every wave reaches
  // the exit whatever else runs on the GPU.
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  WsSched sc{a.plan + (MODE == 0 ? 16 : 24), (int)(blockIdx.x & 7), WsLists{0, 0, 0, 0}, -1, 0};
  int32_t* s_next = reinterpret_cast<int32_t*>(s_lds + C::NEXT_OFF);
  WsItem cur{-1, 0, 0, 0, 0, 0, 0};
  if (wave == 0) {
    sc.lists = ws_lists_init(a, sc.counters, sc.home);
    cur = ws_fetch(a, sc);
    if (lane == 0) {
      s_next[0] = cur.slot; s_next[1] = cur.m0; s_next[2] = cur.g; s_next[3] = cur.c; s_next[4] = cur.off; s_next[5] = cur.bts;
    }
  }
  __syncthreads();
  cur = ws_item_from_lds(s_next, cur.wait_hi);
  int tsrc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const int L0 = 8 * (wave & 3) + (lane >> 3);
  if (wave >= 4 && cur.slot >= 0) ws_gather_rows<MODE>(a, cur, L0, tsrc);
  while (cur.slot >= 0) {
    if (NF == 8 && wave == 0 && cur.wait_hi > 0 && a.wait_ticks > 0) {
      const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
      while (__hip_atomic_load(&sc.counters[sc.home], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < cur.wait_hi &&
             __builtin_amdgcn_s_memrealtime() - t0 < (unsigned long long)a.wait_ticks)
        __builtin_amdgcn_s_sleep(4);
    }
    __syncthreads();  // the previous item's tile has left LDS; the cohort (as far as it came together) starts
    const int rc = min(cur.bts, cur.c - cur.m0);
    const int nfl = (rc + 31) >> 5;
    WsItem nx{-1, 0, 0, 0, 0, 0, 0};
    switch (nfl) {
      case 1: nx = ws_body<MODE, NF, 1>(a, s_lds, cur, tsrc, sc); break;
      case 2: if constexpr (NF >= 2) nx = ws_body<MODE, NF, 2>(a, s_lds, cur, tsrc, sc); break;
      case 3: if constexpr (NF >= 4) nx = ws_body<MODE, NF, 3>(a, s_lds, cur, tsrc, sc); break;
      case 4: if constexpr (NF >= 4) nx = ws_body<MODE, NF, 4>(a, s_lds, cur, tsrc, sc); break;
      case 5: if constexpr (NF >= 8) nx = ws_body<MODE, NF, 5>(a, s_lds, cur, tsrc, sc); break;
      case 6: if constexpr (NF >= 8) nx = ws_body<MODE, NF, 6>(a, s_lds, cur, tsrc, sc); break;
      case 7: if constexpr (NF >= 8) nx = ws_body<MODE, NF, 7>(a, s_lds, cur, tsrc, sc); break;
      case 8: if constexpr (NF >= 8) nx = ws_body<MODE, NF, 8>(a, s_lds, cur, tsrc, sc); break;
      default: break;  // cannot happen for a plan built by k_plan_ws; nx.slot < 0 ends the loop
    }
    cur = nx;
  }
}

// Both products of a call in one launch, for the decode shapes (NF < 8), whose cost is the weight stream: a second
// launch would pay a second ramp-up (plan header, first claim, first slabs: several microseconds with nothing
// streaming) and the first product's tail, during which the compute units that have run out of items idle.  Here a
// workgroup that finds no first-product item left goes straight on to second-product items.  Such an item reads
// activation rows that first-product items of other workgroups write, so it waits until they are complete (done[]):
// every item it waits for was claimed earlier than itself, by a workgroup that is working on it or will once its
// current item is finished, and an item that is being worked on waits for nothing if it belongs to the first product.
// Following "waits for" from workgroup to workgroup, the claim time of the current item strictly decreases, so there
// is no cycle and every wait ends, whatever else runs on the GPU (workgroups that are not resident hold no claims).
template <int NF>
__global__ __launch_bounds__(kWsThreads) void k_ffn_ws2(WsArgs2 aa) {
  using C = WsCfg<0, NF>;
  static_assert(WsCfg<0, NF>::LDS == WsCfg<1, NF>::LDS && WsCfg<0, NF>::NEXT_OFF == WsCfg<1, NF>::NEXT_OFF, "one LDS layout");
  __shared__ __align__(1024) unsigned char s_lds[C::LDS];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  WsSched sc{aa.m[0].plan + 16, (int)(blockIdx.x & 7), WsLists{0, 0, 0, 0}, -1, 0};
  int32_t* s_next = reinterpret_cast<int32_t*>(s_lds + C::NEXT_OFF);
  WsItem cur = EW_NO_ITEM;
  if (wave == 0) {
    sc.lists = ws_lists_init2(aa, sc.counters, sc.home);
    cur = ws_fetch2(aa, sc);
    if (lane == 0) {
      s_next[0] = cur.slot; s_next[1] = cur.m0; s_next[2] = cur.g; s_next[3] = cur.c; s_next[4] = cur.off; s_next[5] = cur.bts;
      s_next[6] = cur.mode;
    }
  }
  __syncthreads();
  cur = ws_item_from_lds(s_next, 0);
  int tsrc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  const int L0 = 8 * (wave & 3) + (lane >> 3);
  if (wave >= 4 && cur.slot >= 0) {
    if (cur.mode == 0) ws_gather_rows<0>(aa.m[0], cur, L0, tsrc);
    else ws_gather_rows<1>(aa.m[1], cur, L0, tsrc);
  }
  while (cur.slot >= 0) {
    __syncthreads();
    const int rc = min(cur.bts, cur.c - cur.m0);
    const int nfl = (rc + 31) >> 5;
    WsItem nx = EW_NO_ITEM;
    if (cur.mode == 0) {
      switch (nfl) {
        case 1: nx = ws_body<0, NF, 1, true>(aa.m[0], s_lds, cur, tsrc, sc, &aa); break;
        case 2: if constexpr (NF >= 2) nx = ws_body<0, NF, 2, true>(aa.m[0], s_lds, cur, tsrc, sc, &aa); break;
        case 3: if constexpr (NF >= 4) nx = ws_body<0, NF, 3, true>(aa.m[0], s_lds, cur, tsrc, sc, &aa); break;
        case 4: if constexpr (NF >= 4) nx = ws_body<0, NF, 4, true>(aa.m[0], s_lds, cur, tsrc, sc, &aa); break;
        default: break;  // cannot happen for a plan built by ws_plan_build; nx.slot < 0 ends the loop
      }
    } else {
      switch (nfl) {
        case 1: nx = ws_body<1, NF, 1, true>(aa.m[1], s_lds, cur, tsrc, sc, &aa); break;
        case 2: if constexpr (NF >= 2) nx = ws_body<1, NF, 2, true>(aa.m[1], s_lds, cur, tsrc, sc, &aa); break;
        case 3: if constexpr (NF >= 4) nx = ws_body<1, NF, 3, true>(aa.m[1], s_lds, cur, tsrc, sc, &aa); break;
        case 4: if constexpr (NF >= 4) nx = ws_body<1, NF, 4, true>(aa.m[1], s_lds, cur, tsrc, sc, &aa); break;
        default: break;
      }
    }
    cur = nx;
  }
}

template <int MODE, int NF>
int launch_ws(const WsArgs& a, int n_cu, int max_tiles, hipStream_t st) {
  // never more workgroups than there can be items: a small call (shared experts at decode sizes)
  // leaves the other CUs to whatever runs beside it
  const long long max_items = (long long)max_tiles * a.groups;
  const int grid = max_items < n_cu ? (int)((max_items + 7) / 8 * 8) : n_cu;
  hipLaunchKernelGGL((k_ffn_ws<MODE, NF>), dim3(grid), dim3(kWsThreads), 0, st, a);
  EW_LAUNCH_CHECK("k_ffn_ws");
  return EW_OK;
}

// The per-product fields of the arguments: MODE 0 = gate/up + SwiGLU (H -> I), MODE 1 = down (I -> H).
template <int MODE>
void set_product(WsArgs& a, const void* x, const int32_t* por, const void* w, const void* w_sh, void* out, int H, int I) {
  a.x = (const uint16_t*)x; a.por = por; a.w = (const uint16_t*)w; a.w_sh = (const uint16_t*)w_sh; a.out = (uint16_t*)out;
  if (MODE == 0) {
    a.slot_stride = (size_t)2 * I * H; a.K = H; a.NOUT = I; a.groups = ceil_div(I, 128);
  } else {
    a.slot_stride = (size_t)H * I; a.K = I; a.NOUT = H; a.groups = ceil_div(H, 256);
  }
}

template <int NF>
int launch_both(WsArgs a, const void* x, const int32_t* por, const void* w13, const void* w2, const void* w13_sh,
                const void* w2_sh, void* act, void* y, int H, int I, int n_cu, int max_tiles, hipStream_t st) {
  set_product<0>(a, x, por, w13, w13_sh, act, H, I);
  int rc = launch_ws<0, NF>(a, n_cu, max_tiles, st);
  if (rc != EW_OK) return rc;
  set_product<1>(a, act, nullptr, w2, w2_sh, y, H, I);
  return launch_ws<1, NF>(a, n_cu, max_tiles, st);
}

}  // namespace

// Kernel shape for a call.  The host knows only totals: no slot has more than max_rows_per_slot rows
// (one per token), and rows / slots is what a slot gets on average if every slot is active.  The
// 256-row shape pays off only when slots are large; a 256-token decode batch spread over hundreds of
// slots is a weight stream like the smaller batches and takes the 128-row shape (any shape is correct
// for any counts: larger slots are cut into chunks).
int ffn_ws_frags(int max_rows_per_slot, int rows, int slots, int nf_override) {
  if (nf_override == 1 || nf_override == 2 || nf_override == 4 || nf_override == 8) return nf_override;
  if (max_rows_per_slot <= 32) return 1;
  if (max_rows_per_slot <= 64) return 2;
  if (max_rows_per_slot <= 128) return 4;
  return rows / (slots < 1 ? 1 : slots) >= 32 ? 8 : 4;
}

// Chunks per plan entry at most: 8 (a quarter of an XCD's workgroups per feature group), doubled until the
// entries of the worst case -- every possible slot active plus one more entry per ch * bt rows -- fit a plan.
static int ws_entry_chunks(int rows, int P, int bt) {
  const int max_active = P < rows ? P : rows;
  int ch = 8;
  while ((long long)max_active + rows / ((long long)ch * bt) > kPlanMaxEnt) ch *= 2;
  return ch;
}

static int ws_list_cap(int rows, int P) {
  // Entries per list at most.  A slot of c rows makes at most 1 + c / (ch * bt) entries, so a call makes at most
  // max_active + rows / (ch * bt) of them: never more than kPlanMaxEnt (choice of ch), nor than the figure for the
  // smallest chunk any kernel shape or tuning cap can ask for (bt = 32, ch = 8).
  const int max_active = P < rows ? P : rows;
  const long long worst = (long long)max_active + rows / 256;
  return ceil_div((int)(worst < kPlanMaxEnt ? worst : kPlanMaxEnt), 8) + 1;
}

// Calls of at most this many rows run their two products in one launch (decode shapes only); one counter per row.
constexpr int kMergeMaxRows = 16384;

size_t ffn_ws_plan_ints(int rows, int P, int nf) {
  (void)nf;
  return (size_t)kPlanHdr + (size_t)8 * kEnt * ws_list_cap(rows, P) + (size_t)(rows < kMergeMaxRows ? rows : kMergeMaxRows);
}

WsPlanShape ffn_ws_plan_shape(int rows, int slots, int nf, int chunk_frags, bool merge) {
  WsPlanShape sh;
  sh.nf = nf;
  sh.bt = 32 * (chunk_frags >= 1 && chunk_frags <= nf ? chunk_frags : nf);
  sh.ch = ws_entry_chunks(rows, slots, sh.bt);
  sh.cap = ws_list_cap(rows, slots);
  sh.n_done = merge && nf < 8 && rows <= kMergeMaxRows ? rows : 0;
  sh.done_off = kPlanHdr + 8 * kEnt * sh.cap;
  return sh;
}

int launch_ffn_ws_plan(const int32_t* counts, const int32_t* offsets, int P, int S, int T, int rows_routed, const WsPlanShape& sh,
                       int32_t* plan, hipStream_t st) {
  hipLaunchKernelGGL(k_plan_ws, dim3(1), dim3(512), 0, st, counts, offsets, P, S, T, rows_routed, sh, plan);
  EW_LAUNCH_CHECK("k_plan_ws");
  return EW_OK;
}

// Enqueues plan (unless plan_ready: the caller has had it built, with the same shape) + both products.  `plan` holds
// ffn_ws_plan_ints(rows, slots, nf) ints; H % 64 == 0, I % 64 == 0, I % 16 == 0, H % 32 == 0 and
// rows * max(H, I) * 2 < 2^32 are the caller's checks.
int launch_ffn_ws(const void* x, int rows_routed, int k, int H, int I, int P, int S, const WsPlanShape& sh, bool plan_ready,
                  const int32_t* counts, const int32_t* offsets, const int32_t* por, const void* w13, const void* w2,
                  const void* w13_sh, const void* w2_sh, void* act, void* y, int32_t* plan, int wait_ticks, hipStream_t st) {
  const int T = rows_routed / k;              // tokens = rows of each shared expert
  const int rows = rows_routed + S * T;
  const int slots = P + S;
  const int nf = sh.nf, bt = sh.bt, cap = sh.cap;
  // persistent grid: one workgroup per CU, a multiple of the 8 XCDs; the count is kept per device
  // (relaxed atomics: two threads racing on the first call store the same value)
  constexpr int kMaxDev = 64;
  static std::atomic<int> cu_of_dev[kMaxDev];
  int dev = 0;
  EW_HIP(hipGetDevice(&dev));
  int n_cu = dev >= 0 && dev < kMaxDev ? cu_of_dev[dev].load(std::memory_order_relaxed) : 0;
  if (n_cu == 0) {
    int v = 0;
    EW_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
    n_cu = v < 8 ? 8 : v / 8 * 8;
    if (dev >= 0 && dev < kMaxDev) cu_of_dev[dev].store(n_cu, std::memory_order_relaxed);
  }
  if (!plan_ready) {
    const int rc = launch_ffn_ws_plan(counts, offsets, P, S, T, rows_routed, sh, plan, st);
    if (rc != EW_OK) return rc;
  }
  const int max_active = slots < rows ? slots : rows;
  const int max_tiles = rows / bt + max_active;
  WsArgs a{};
  a.counts = counts; a.offsets = offsets; a.plan = plan; a.k = k; a.cap = cap; a.wait_ticks = wait_ticks;
  a.P = P; a.rows_routed = rows_routed; a.sh_rows = T > 0 ? T : 1;
  if (sh.n_done > 0) {
    WsArgs2 aa{};
    aa.m[0] = aa.m[1] = a;
    set_product<0>(aa.m[0], x, por, w13, w13_sh, act, H, I);
    set_product<1>(aa.m[1], act, nullptr, w2, w2_sh, y, H, I);
    aa.done = plan + sh.done_off;
    aa.done_target = 8 * aa.m[0].groups;
    aa.spin_ticks = 20000000u;  // 0.2 s
    const long long max_items = (long long)max_tiles * (aa.m[0].groups + aa.m[1].groups);
    const int grid = max_items < n_cu ? (int)((max_items + 7) / 8 * 8) : n_cu;
    switch (nf) {
      case 1: hipLaunchKernelGGL((k_ffn_ws2<1>), dim3(grid), dim3(kWsThreads), 0, st, aa); break;
      case 2: hipLaunchKernelGGL((k_ffn_ws2<2>), dim3(grid), dim3(kWsThreads), 0, st, aa); break;
      default: hipLaunchKernelGGL((k_ffn_ws2<4>), dim3(grid), dim3(kWsThreads), 0, st, aa); break;
    }
    EW_LAUNCH_CHECK("k_ffn_ws2");
    return EW_OK;
  }
  switch (nf) {
    case 1: return launch_both<1>(a, x, por, w13, w2, w13_sh, w2_sh, act, y, H, I, n_cu, max_tiles, st);
    case 2: return launch_both<2>(a, x, por, w13, w2, w13_sh, w2_sh, act, y, H, I, n_cu, max_tiles, st);
    case 4: return launch_both<4>(a, x, por, w13, w2, w13_sh, w2_sh, act, y, H, I, n_cu, max_tiles, st);
    default: return launch_both<8>(a, x, por, w13, w2, w13_sh, w2_sh, act, y, H, I, n_cu, max_tiles, st);
  }
}

}  // namespace ew
