// Work plan of the weight-stationary grouped-FFN kernel (k_ffn_ws): layout and the device routine that builds it.
// Shared by the FFN's own plan kernel and by the decode-sized permutation kernel, which can append the plan of the FFN
// call that follows it to its own launch.
#pragma once
#include <cstdint>
#include <hip/hip_runtime.h>

namespace ew {

// Work plan of one moe_grouped_ffn call, built on the device (the host never reads the counts).
//  * A slot with more than bt rows is cut into equal chunks (rounded up to whole 32-row fragments),
//    so all work items of a slot take the same time.
//  * A slot with more than `ch` chunks is cut further into entries of at most `ch` chunks each.  An
//    entry's items (chunk x feature group) are enumerated group-major, so the 32 workgroups of an XCD
//    that work through one entry hold about 32 / ch feature groups of ch chunks at any time: every
//    weight row they fetch serves ch of them and every token row 32 / ch of them out of the XCD's L2.
//    (A whole slot of 32 chunks per list made 32 workgroups share one feature group and nothing else:
//    every token row came from the fabric once per feature group.)
//  * Entries are ordered by chunk size, largest first (slot id, then position in the slot, break
//    ties), and dealt round-robin to 8 lists, one per XCD (workgroup b runs on XCD b % 8).  The
//    workgroups that share an entry's weights (different chunks) or its token rows (different feature
//    groups) thus run on the same XCD and meet in that XCD's L2 -- provided they start together, which
//    the kernel arranges (see k_ffn_ws); equal durations inside an entry and similar ones between
//    neighbours in the list keep them together.
//   plan[x]        x < 8   entries of list x
//   plan[8 + x]            row chunks of list x
//   plan[16 + x], plan[24 + x]   work counters of the two products (zeroed here, every call)
//   plan[32 + 6 (x cap + e)] ...  entry e of list x: slot, chunks, chunks of the list before it,
//                                 rows per chunk, rows of the entry, first row of the entry
//   plan[done_off + r]     calls whose two products share a launch: waves that have stored their part of the
//                          activation rows of the chunk that starts at sorted row r (zeroed here, every call)
constexpr int kPlanHdr = 32;
constexpr int kEnt = 6;
constexpr int kPlanMaxP = 2048;    // slots a plan can sort
constexpr int kPlanMaxEnt = 4096;  // entries a plan can hold (the host picks ch accordingly)

__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t t = (uint32_t)__shfl_up((int)v, o, 64);
    if (lane >= o) v += t;
  }
  return v;
}

// chunks and rows per chunk of a slot with c > 0 rows
__device__ __forceinline__ void chunking(int c, int bt, int& nch, int& bts) {
  nch = (c + bt - 1) / bt;
  bts = ((c + nch - 1) / nch + 31) & ~31;
}

// Shape of the plan and of the kernel that consumes it, chosen on the host from the call's dimensions.
struct WsPlanShape {
  int nf;        // 32-token fragments of the kernel shape (1, 2, 4, 8)
  int bt;        // rows per chunk at most
  int ch;        // chunks per entry at most
  int cap;       // entries per list at most
  int n_done;    // completion counters behind the lists, one per sorted row (0: the two products run as two launches)
  int done_off;  // where they start, in ints from the start of the plan
};

// Builds the plan from the slots' counts and offsets.  Slots P .. P+S-1 are the shared experts of the call, if any:
// each holds every token (sh_rows of them), and their rows follow the routed ones (first at sh_first).
// Called by every thread of a block of at least 512 threads (it contains barriers); the first 512 do the work.
// counts / offsets may have been written by this block before a barrier.
struct WsPlanLds {
  uint32_t sorted[kPlanMaxEnt];  // entries in processing order: slot | part << 16
  uint32_t wtot[8][8];           // per wave: entries per size class
  int base[9];                   // first position of each size class
  int32_t cnt[kPlanMaxP], off[kPlanMaxP];  // rows and first row of every slot (one global round trip)
};

// `have` (optional): the caller already holds the rows and first row of the routed slots 4 tid .. 4 tid + 3 of every
// working thread in have[0..3] / have[4..7] (then counts / offsets are not read).
__device__ __forceinline__ void ws_plan_build(const int32_t* counts, const int32_t* offsets, int P, int S, int sh_rows,
                                              int sh_first, const WsPlanShape sh, int32_t* __restrict__ plan, WsPlanLds& L,
                                              const int32_t* have = nullptr) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const bool worker = tid < 512;
  const int bt = sh.bt, ch = sh.ch, cap = sh.cap;
  for (int i = tid; i < sh.n_done; i += blockDim.x) plan[sh.done_off + i] = 0;
  // size class of a slot: 8 - (32-row fragments per chunk), i.e. 0 = largest chunks.  Thread t owns
  // slots 4t .. 4t+3, so thread order is slot order.
  int cls[4], nent[4];
  uint32_t mine[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
  uint32_t excl[8];
  if (worker) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int sl = 4 * tid + i;
      int c = 0, o = 0;
      if (sl < P) {
        c = have ? have[i] : counts[sl];
        o = have ? have[4 + i] : offsets[sl];
      } else if (sl < P + S) {
        c = sh_rows;
        o = sh_first + (sl - P) * sh_rows;
      }
      L.cnt[sl] = c;
      L.off[sl] = o;
      cls[i] = -1;
      nent[i] = 0;
      if (c > 0) {
        int nch, bts;
        chunking(c, bt, nch, bts);
        cls[i] = 8 - (bts >> 5);
        nent[i] = (nch + ch - 1) / ch;
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (cls[i] == k) mine[k] += (uint32_t)nent[i];
      }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const uint32_t inc = wave_incl_scan_u32(mine[k]);
      excl[k] = inc - mine[k];
      if (lane == 63) L.wtot[wave][k] = inc;
    }
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int k = 0; k < 8; ++k) {
      L.base[k] = run;
      for (int w = 0; w < 8; ++w) run += (int)L.wtot[w][k];
    }
    L.base[8] = run;
  }
  __syncthreads();
  if (worker) {
    int seen[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      int before = (int)excl[k];
      for (int w = 0; w < wave; ++w) before += (int)L.wtot[w][k];
      seen[k] = L.base[k] + before;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (cls[i] < 0) continue;
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (cls[i] == k) {
          for (int part = 0; part < nent[i]; ++part) L.sorted[seen[k]++] = (uint32_t)(4 * tid + i) | ((uint32_t)part << 16);
        }
    }
  }
  __syncthreads();
  if (!worker) return;
  // wave x builds list x from positions x, x + 8, ...
  const int n_total = L.base[8];
  const int x = wave;
  int32_t* list = plan + kPlanHdr + kEnt * x * cap;
  int n_chunks = 0, n_entries = 0;
  for (int e0 = 0; 8 * e0 + x < n_total; e0 += 64) {
    const int e = e0 + lane, pos = 8 * e + x;
    const bool ok = pos < n_total;
    int sl = 0, c = 0, nch = 0, bts = 0, first = 0;
    if (ok) {
      const uint32_t v = L.sorted[pos];
      sl = (int)(v & 0xFFFFu);
      int all;
      chunking(L.cnt[sl], bt, all, bts);
      first = (int)(v >> 16) * ch;                   // first chunk of this entry inside its slot
      nch = min(ch, all - first);
      c = min(L.cnt[sl] - first * bts, nch * bts);   // rows of this entry
    }
    const int incl = (int)wave_incl_scan_u32((uint32_t)nch);
    if (ok) {
      int32_t* en = list + kEnt * e;
      en[0] = sl;
      en[1] = nch;
      en[2] = n_chunks + incl - nch;
      en[3] = bts;
      en[4] = c;
      en[5] = L.off[sl] + first * bts;
    }
    n_chunks += __shfl(incl, 63, 64);
    n_entries += __popcll(__ballot(ok));
  }
  if (lane == 0) {
    plan[x] = n_entries;
    plan[8 + x] = n_chunks;
    plan[16 + x] = 0;
    plan[24 + x] = 0;
  }
}

}  // namespace ew
