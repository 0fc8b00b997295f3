/*
 * expertweave.h -- C ABI of the ExpertWeave MoE-layer hot path for AMD MI355X (gfx950).
 *
 * The path (paper arxiv 2508.17624, Sec. 2.1 and Sec. 4):
 *   router top-k -> batched rerouting through the ESFT expert map -> token permutation with
 *   per-slot counts/offsets -> grouped SwiGLU expert FFN over the unified base+adapter expert
 *   pool (the "virtual weight tensor") -> weighted un-permute (+ shared experts).
 *
 * Conventions
 *   - Every call returns 0 (EW_OK) or a negative EW_ERR_* code; ew_last_error() gives a
 *     thread-local message for the last failing call of the calling thread.
 *   - Pointers marked [dev] are device pointers valid on the current HIP device; [host] are host
 *     pointers.  All [dev] buffers are owned by the caller; the library never allocates
 *     activations.  Scratch comes from a caller-provided workspace whose size the matching
 *     *_workspace_bytes() query returns (align it to 256 bytes).
 *   - Kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *     and never synchronise; results are ready when the stream reaches them.
 *   - Shapes and pointers are checked on the host before any launch.  Values inside device
 *     arrays (adapter ids, expert ids, expert-map entries) are the caller's contract:
 *     0 <= adapter_id[t] <= N, 0 <= topk_ids < E, 0 <= expert_map < P.
 *   - Adapter ids: 0 = base model, a in 1..N = adapter a.  (The paper numbers adapters
 *     i = 0..N-1 and marks base tokens with -1; a = i+1.)
 *   - Slots: P = M + N*E_max.  Slot s < M is base expert s; adapter a owns slots
 *     [M + (a-1)*E_max, M + a*E_max), of which only the first e_a hold experts (Sec. 4.1).
 *   - Row-major everywhere.  Pair index p = t*k + j for token t and its j-th choice.
 */
#ifndef EXPERTWEAVE_H
#define EXPERTWEAVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  EW_OK = 0,
  EW_ERR_INVALID_ARG = -1, /* bad shape, null pointer, out-of-range scalar argument          */
  EW_ERR_OOM = -2,         /* the device runtime could not supply physical memory            */
  EW_ERR_VMM = -3,         /* a virtual-memory call (reserve/map/set-access/unmap) failed     */
  EW_ERR_STATE = -4,       /* call not valid in the pool's current state (e.g. double load)  */
  EW_ERR_WORKSPACE = -5,   /* workspace pointer null/misaligned or smaller than required     */
  EW_ERR_UNSUPPORTED = -6, /* shape outside what the kernels support (limits stated per call)*/
  EW_ERR_HIP = -7          /* any other HIP runtime error (launch failure, no device)        */
};

enum { EW_F32 = 0, EW_BF16 = 1 }; /* element type of tokens, expert weights and FFN outputs */

enum {
  EW_POOL_VMM = 0,    /* virtual weight tensor: pages mapped only under loaded experts (Sec. 4.2) */
  EW_POOL_PADDED = 1, /* the padding approach of Sec. 3.1: all P slots backed at creation         */
  EW_POOL_FAKE = 2,   /* host-memory backend (mmap/mprotect) for GPU-less tests; may be or-ed
                         with the other flags                                                     */
  EW_POOL_EAGER_UNMAP = 4 /* unmap a page the moment its last user is evicted; the default keeps
                         it mapped in place ("parked") until the pool needs it elsewhere          */
};

/* Thread-local message of the calling thread's last failing call ("" if none). Never NULL. */
const char* ew_last_error(void);
/* ABI version of this header: bumps whenever a signature changes. */
int ew_abi_version(void);

/* ===================================================================================== *
 * Expert pool: virtual weight tensors, physical page pool, ESFT expert map  (Sec. 4.1-4.2)
 * ===================================================================================== */

typedef struct ew_pool ew_pool; /* opaque; owns VA reservations, physical pages, page tables
                                   and the expert maps (device copies + host mirrors)        */

typedef struct ew_pool_stats {
  uint64_t page_bytes;        /* physical page size in use                                   */
  uint64_t bytes_virtual;     /* sum of reserved virtual ranges                              */
  uint64_t pages_mapped;      /* pages currently mapped into some virtual weight tensor      */
  uint64_t pages_free;        /* pages created and held by the pool, not mapped              */
  uint64_t pages_parked;      /* pages of evicted ranges still mapped at their old address    */
  uint64_t pages_created;     /* pages obtained from the runtime since creation              */
  uint64_t pages_released;    /* pages given back to the runtime since creation              */
  uint64_t pages_shared;      /* mapped pages used by more than one loaded expert range      */
  uint64_t bytes_experts;     /* bytes of expert weights currently loaded                    */
  uint64_t experts_loaded;    /* number of (layer, slot) entries holding an expert           */
  double   f_mem;             /* L*(M+N*E_max) / sum_l(M + sum_i e_i^(l)) over loaded adapters
                                 (Sec. 3.1); 0 if nothing is loaded                           */
} ew_pool_stats;

/* Create a pool for `num_layers` MoE layers on HIP device `device` (ignored for EW_POOL_FAKE).
 * For each layer two virtual weight tensors are reserved, unmapped (Sec. 4.2):
 *   W13 [P, 2I, H] (gate rows [0,I), then up rows [I,2I)), w13_bytes_per_expert per slot;
 *   W2  [P, H, I],                                        w2_bytes_per_expert  per slot.
 * page_bytes = 0 asks the runtime for its recommended granularity; otherwise it must be a
 * multiple of the minimum granularity (any multiple of 4096 for EW_POOL_FAKE).
 * prealloc_pages physical pages are created up front and kept in the free list.
 * Errors: INVALID_ARG, OOM, VMM, HIP.  On error *out is NULL and nothing is leaked. */
int expert_pool_create(ew_pool** out, int device, int num_layers, int M, int N, int E_max,
                       size_t w13_bytes_per_expert, size_t w2_bytes_per_expert,
                       size_t page_bytes, size_t prealloc_pages, int flags);

/* Unmaps and releases everything.  The caller guarantees no kernel still reads the pool. */
int expert_pool_destroy(ew_pool* pool);

/* Load one class's experts of one layer (Sec. 4.2, expert memory manager: a range of consecutive
 * experts is loaded at start_addr = base_addr + Delta * expert_size) and write its row of the
 * expert map (Sec. 4.1):
 *   adapter_id = 0: the base model; n must equal M and expert_ids (may be NULL) be 0..M-1.
 *   adapter_id = a in 1..N: n in 0..E_max tuned experts, expert_ids [host] strictly ascending
 *     in [0,M); the d-th of them goes to slot M+(a-1)*E_max+d and map[a][expert_ids[d]] is set
 *     to that slot; all other entries of row a stay identity.  n = 0 is legal (maps nothing).
 * w13 [n,2I,H] and w2 [n,H,I] are host or device pointers (may be NULL when n = 0, or to map
 * pages without filling them); they are copied on `stream` into the mapped range, and the
 * expert-map row is copied to the device on `stream`.  A page of this range that was evicted
 * earlier and is still parked in place is taken back as it is; other pages come from the pool's
 * free list, then from parked pages elsewhere (oldest first, unmapped and moved), then from the
 * runtime.  A page only partly covered by this range is shared with the neighbouring range
 * through a reference count.
 * Errors: INVALID_ARG; STATE if this (layer, adapter) is already loaded; OOM/VMM if pages
 * cannot be obtained or mapped -- then every page reference taken by this call is dropped again
 * (the pages return to the pool), reference counts and the expert map are left as before. */
int expert_pool_map(ew_pool* pool, int layer, int adapter_id, int n, const int32_t* expert_ids,
                    const void* w13, const void* w2, void* stream);

/* Evict (Sec. 4.2, unloading of a range): resets row adapter_id of the layer's expert map to
 * identity (copied to the device on `stream`, then the stream is synchronised) and drops the
 * range's page references.  Pages whose count reaches zero go back to the pool: parked in place
 * by default (no VMM call; see expert_pool_map and expert_pool_trim), or unmapped into the free
 * list at once for EW_POOL_EAGER_UNMAP pools.
 * The caller guarantees no kernel that may read those slots is still in flight.
 * Errors: INVALID_ARG; STATE if not loaded; VMM if an unmap failed -- the adapter is evicted all
 * the same (row reset, references dropped) and the pages that could not be unmapped stay parked. */
int expert_pool_unmap(ew_pool* pool, int layer, int adapter_id, void* stream);

/* Pointers a forward pass needs for one layer: base addresses of the two virtual weight
 * tensors, the expert map [N+1][M] int32 (device copy, or host memory for EW_POOL_FAKE) and
 * P.  Any out pointer may be NULL.  The addresses stay valid until expert_pool_destroy. */
int expert_pool_view(ew_pool* pool, int layer, void** w13_base, void** w2_base,
                     const int32_t** expert_map, int* num_slots);

/* Host mirror of one layer's expert map, [N+1][M] int32, copied into out [host]. */
int expert_pool_expert_map_host(ew_pool* pool, int layer, int32_t* out);

/* Eviction order for adapter churn (Sec. 4.2: adapters are loaded and unloaded at run time; the
 * policy itself is the serving engine's).  The pool keeps one logical clock: expert_pool_map stamps
 * the adapter it loads, expert_pool_touch stamps the n adapter ids [host] of a scheduled batch (all
 * with the same tick; id 0, the base model, is accepted and ignored by the victim search).
 * expert_pool_lru_victim writes the adapter (1..N) that is loaded in at least one layer and has the
 * oldest stamp, lower id on ties, or -1 if no adapter is loaded.  Nothing is unmapped: the caller
 * follows up with expert_pool_unmap per layer.  Errors: INVALID_ARG. */
int expert_pool_touch(ew_pool* pool, int n, const int32_t* adapter_ids);
int expert_pool_lru_victim(ew_pool* pool, int* adapter_id);

int expert_pool_stats(ew_pool* pool, ew_pool_stats* out);

/* Unmap every parked page into the free list, then give free pages back to the runtime until at
 * most keep_pages remain in the free list.  Errors: VMM (pages that failed stay parked / listed). */
int expert_pool_trim(ew_pool* pool, size_t keep_pages);

/* Test hooks of the EW_POOL_FAKE backend (STATE for other pools).
 * fail_at: the n-th (1-based, counted from now) call of kind `op` fails once;
 *   op: 0 = create physical page, 1 = map, 2 = unmap.  n = 0 disarms.
 * is_mapped: *out = 1 if the page holding byte `offset` of layer's tensor `which`
 *   (0 = W13, 1 = W2) is mapped. */
int expert_pool_fake_fail_at(ew_pool* pool, int op, int n);
int expert_pool_fake_is_mapped(ew_pool* pool, int layer, int which, size_t offset, int* out);

/* ===================================================================================== *
 * Hot path
 * ===================================================================================== */

/* Router top-k (Sec. 2.1: the learned router g(x) picks the k most relevant experts per token).
 *   logits   [dev] float32 [T, E]: gate scores, finite.
 *   topk_ids [dev] int32   [T, k]: the k experts with the largest logit, descending; equal
 *                                  logits (-0.0 == +0.0) ordered by lower index.
 *   topk_w   [dev] float32 [T, k]: softmax over all E logits (fp32, max-subtracted) of the chosen
 *                                  experts; divided by their sum if renormalize != 0.
 * Limits: 1 <= k <= E <= 1024.  T = 0 is a no-op.  Errors: INVALID_ARG, UNSUPPORTED, HIP. */
int moe_route_topk(const float* logits, int T, int E, int k, int renormalize,
                   int32_t* topk_ids, float* topk_w, void* stream);

/* Batched rerouting + dispatch bookkeeping (Sec. 4.1 TopK'(x) = {Pi[A(x), j]}, Sec. 4.3; Sec. 2.1:
 * tokens are replicated, permuted and grouped by their top-k ids).
 *   topk_ids   [dev] int32 [T, k]   base expert ids in [0, E)
 *   adapter_id [dev] int32 [T]      0 = base, 1..N
 *   expert_map [dev] int32 [N+1, E] row 0 identity (as written by expert_pool_map); entries < P
 *   slot_ids   [dev] int32 [T, k]   out: expert_map[adapter_id[t]][topk_ids[t, j]]
 *   counts     [dev] int32 [P]      out: pairs per slot
 *   offsets    [dev] int32 [P+1]    out: exclusive prefix sum of counts; offsets[P] = T*k
 *   pair_of_row[dev] int32 [T*k]    out: sorted row -> pair index; rows grouped by slot, pairs of
 *                                   one slot in ascending pair index (stable, hence unique)
 *   row_of_pair[dev] int32 [T*k]    out: inverse permutation (may be NULL to skip)
 * All integer; results are bit-exact and deterministic.
 * Limits: 1 <= k <= 64, 1 <= P <= 2048, T*k < 2^31.  T = 0 zero-fills counts/offsets.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
size_t moe_reroute_permute_workspace_bytes(int T, int k, int P);
int moe_reroute_permute(const int32_t* topk_ids, const int32_t* adapter_id,
                        const int32_t* expert_map, int T, int k, int E, int N, int P,
                        int32_t* slot_ids, int32_t* counts, int32_t* offsets,
                        int32_t* pair_of_row, int32_t* row_of_pair,
                        void* ws, size_t ws_bytes, void* stream);

/* moe_reroute_permute for callers that cannot allocate device memory or carry a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments
 * without the workspace, same outputs bit for bit.  Its scratch (the per-block histogram table) is
 * a device array built into the library, moe_reroute_permute_static_max_bytes() = 4 MiB per GPU,
 * held until the process ends; the call allocates nothing and frees nothing.
 * All calls on one GPU share that array: calls that overlap in time on one GPU (different
 * streams, different threads) race and must be serialised by the caller.  Nothing needs clearing
 * between calls.
 * Limits: as moe_reroute_permute, and moe_reroute_permute_workspace_bytes(T, k, P) must not
 * exceed moe_reroute_permute_static_max_bytes() -- e.g. T = 2^20, k = 6, P = 384 needs 0.75 MiB;
 * beyond that UNSUPPORTED is returned and nothing is launched.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
size_t moe_reroute_permute_static_max_bytes(void);
int moe_reroute_permute_static(const int32_t* topk_ids, const int32_t* adapter_id,
                               const int32_t* expert_map, int T, int k, int E, int N, int P,
                               int32_t* slot_ids, int32_t* counts, int32_t* offsets,
                               int32_t* pair_of_row, int32_t* row_of_pair, void* stream);

/* Fused router top-k + rerouting + permutation: same outputs as moe_route_topk followed by
 * moe_reroute_permute (bit-identical integers, identical weights), fewer launches.
 * Extra limit: E <= 1024.  Workspace: moe_reroute_permute_workspace_bytes(T, k, P). */
int moe_route_reroute_permute(const float* logits, const int32_t* adapter_id,
                              const int32_t* expert_map, int T, int E, int k, int N, int P,
                              int renormalize, int32_t* topk_ids, float* topk_w,
                              int32_t* slot_ids, int32_t* counts, int32_t* offsets,
                              int32_t* pair_of_row, int32_t* row_of_pair,
                              void* ws, size_t ws_bytes, void* stream);

/* Ablation baseline, not part of the hot path: batched rerouting as three separate canonical
 * operators -- broadcast the adapter id to every (token, choice) pair, compute the offset
 * adapter_id * E + topk_id, gather from the expert map -- each a launch and a pass over memory of its
 * own, as in the paper's ExpertWeave-SingleOp variant (Sec. 5.3).  Same slot_ids as
 * moe_reroute_permute, bit for bit; the permutation is then a separate moe_reroute_permute call
 * on slot_ids with an identity map.
 * Workspace: moe_reroute_singleop_workspace_bytes(T, k) (two int32 [T*k] temporaries).
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
size_t moe_reroute_singleop_workspace_bytes(int T, int k);
int moe_reroute_singleop(const int32_t* topk_ids, const int32_t* adapter_id, const int32_t* expert_map,
                         int T, int k, int E, int N, int32_t* slot_ids, void* ws, size_t ws_bytes,
                         void* stream);

/* Grouped SwiGLU expert FFN over the virtual weight tensors (Sec. 2.1: the grouped matrix
 * multiplication over the permuted tokens and the stacked expert weights; Sec. 4.1: executed on
 * the virtual weight tensor).  For every slot s with counts[s] > 0 and every sorted row r in
 * [offsets[s], offsets[s+1]):  t = pair_of_row[r] / k,
 *     y_sorted[r] = W2_s . ( silu(W1g_s . x_t) * (W1u_s . x_t) ),
 * W1g_s = rows [0,I) and W1u_s = rows [I,2I) of w13_base[s], W2_s = w2_base[s].
 * Slots with counts[s] == 0 are never dereferenced (they may be unmapped address space).
 *   x          [dev] dtype [*, H]: must hold every token pair_of_row[r] / k refers to
 *   T, k       T*k is the number of sorted rows and must equal offsets[P].  For rows that do not
 *              come from a top-k (shared experts: P = S slabs of all tokens) pass k = 1 and
 *              T = the row count, with pair_of_row[r] = the token of row r.
 *   counts, offsets, pair_of_row [dev] as produced by moe_reroute_permute; pair_of_row may be
 *              NULL, meaning row r is pair r
 *   w13_base   [dev] dtype [P, 2I, H]   w2_base [dev] dtype [P, H, I]
 *   y_sorted   [dev] dtype [T*k, H]
 * bf16: inputs bf16, fp32 accumulation on MFMA, the activation silu(g)*u is rounded to bf16
 * between the two products, y rounded to bf16.  f32: plain fp32 throughout.
 * Limits (bf16): H % 128 == 0 and I % 128 == 0.  Calls with T*k*max(H,I)*2 >= 2^32 bytes or
 * P > 2048 take an older, slower kernel, which also needs max(H, I) <= 5000.  T = 0 is a no-op.
 * Workspace: moe_grouped_ffn_workspace_bytes(T, k, H, I, P, dtype) with the same T and k.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
size_t moe_grouped_ffn_workspace_bytes(int T, int k, int H, int I, int P, int dtype);
int moe_grouped_ffn(const void* x, int dtype, int T, int k, int H, int I, int P,
                    const int32_t* counts, const int32_t* offsets, const int32_t* pair_of_row,
                    const void* w13_base, const void* w2_base, void* y_sorted,
                    void* ws, size_t ws_bytes, void* stream);

/* The routed experts and the model's S shared experts in one call.  Shared experts (Sec. 2.1: part of
 * the base model's MoE block, visited by every token whatever the router picks; the evaluated model
 * of Sec. 5.1 has two) are S further slots behind the P routed ones: slot P + s holds all T tokens
 * in order and reads its weights from w13_shared[s] / w2_shared[s] instead of the virtual tensors.
 * One launch then streams both kinds of expert; run separately, the few workgroups of the shared
 * experts either wait for the routed call or take its compute units.
 *     y_sorted[r]                 for r < T*k: as moe_grouped_ffn;
 *     y_sorted[T*k + s*T + t]   = W2sh_s . ( silu(W1g_sh_s . x_t) * (W1u_sh_s . x_t) ),
 * so y_sorted + T*k*H is the [S, T, H] shared_out operand of moe_unpermute.
 *   counts, offsets, pair_of_row [dev]: those of the P routed slots, exactly as for moe_grouped_ffn
 *   w13_shared [dev] bf16 [S, 2I, H]   w2_shared [dev] bf16 [S, H, I]
 *   y_sorted   [dev] bf16 [T*(k+S), H]
 * Limits: bf16 only, H % 128 == 0, I % 128 == 0, P + S <= 2048, T*(k+S)*max(H,I)*2 < 2^32 bytes;
 * anything else is UNSUPPORTED (make two moe_grouped_ffn calls instead).  T = 0 is a no-op.
 * Workspace: moe_grouped_ffn_workspace_bytes(T, k + S, H, I, P + S, dtype).
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
int moe_grouped_ffn_with_shared(const void* x, int dtype, int T, int k, int H, int I, int P, int S,
                                const int32_t* counts, const int32_t* offsets,
                                const int32_t* pair_of_row, const void* w13_base, const void* w2_base,
                                const void* w13_shared, const void* w2_shared, void* y_sorted,
                                void* ws, size_t ws_bytes, void* stream);

/* The last two calls split differently, for decode-sized batches where every launch counts: the
 * work plan that a grouped-FFN call builds from counts / offsets in a small launch of its own
 * (which slot chunks go to which group of compute units) is written by the permutation call
 * instead -- by its single-block kernel itself when the batch is small enough for that one --
 * and the FFN call starts streaming at once.
 *   moe_route_reroute_permute_plan: moe_route_reroute_permute, then the plan of the FFN call
 *     described by (T, k, H, I, P, S, dtype) into ffn_ws, that call's workspace (same size rule).
 *   moe_grouped_ffn_planned: moe_grouped_ffn (S = 0, shared pointers NULL) or
 *     moe_grouped_ffn_with_shared (S > 0) without its planning launch.  ws must be the ffn_ws of a
 *     moe_route_reroute_permute_plan call with the same T, k, H, I, P, S and dtype whose counts
 *     and offsets are the ones passed here, made earlier on the same stream with no other use of
 *     ws and no ew_tune_ffn call in between.  A plan serves one call (its work counters are used
 *     up by it).  Anything else computes garbage or nothing (no fault: a plan only names slots and
 *     rows inside the buffers of the call it was built for).
 * Limits: those of moe_grouped_ffn_with_shared (with S = 0 allowed); otherwise UNSUPPORTED.
 * Errors: INVALID_ARG, UNSUPPORTED, WORKSPACE, HIP. */
int moe_route_reroute_permute_plan(const float* logits, const int32_t* adapter_id,
                                   const int32_t* expert_map, int T, int E, int k, int N, int P,
                                   int renormalize, int32_t* topk_ids, float* topk_w,
                                   int32_t* slot_ids, int32_t* counts, int32_t* offsets,
                                   int32_t* pair_of_row, int32_t* row_of_pair, void* ws,
                                   size_t ws_bytes, int H, int I, int S, int dtype, void* ffn_ws,
                                   size_t ffn_ws_bytes, void* stream);
int moe_grouped_ffn_planned(const void* x, int dtype, int T, int k, int H, int I, int P, int S,
                            const int32_t* counts, const int32_t* offsets,
                            const int32_t* pair_of_row, const void* w13_base, const void* w2_base,
                            const void* w13_shared, const void* w2_shared, void* y_sorted, void* ws,
                            size_t ws_bytes, void* stream);

/* Combine and un-permute (Sec. 2.1: expert outputs are weighted with the router's weights and
 * put back into the original token order), plus the shared experts' contribution and
 * an optional residual stream (the layer's input when layers are stacked):
 *     out[t] = sum_{j<k} topk_w[t, j] * y_sorted[row_of_pair[t*k + j]] + sum_{s<S} shared_out[s][t]
 *              (+ residual[t])
 * accumulated in fp32: routed terms in ascending j, then shared in ascending s, then the residual.
 *   y_sorted [dev] dtype [T*k, H]; row_of_pair [dev] int32 [T*k]; topk_w [dev] float32 [T, k];
 *   shared_out [dev] dtype [num_shared, T, H] (the shared experts' outputs, one slab per shared
 *   expert, e.g. moe_grouped_ffn's y for P = num_shared, k = 1) or NULL; residual [dev] dtype
 *   [T, H] or NULL (may alias out only if it is the same pointer); out [dev] dtype [T, H].
 * Limits: k <= 64; H % 8 == 0 for bf16, H % 4 == 0 for f32.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
int moe_unpermute(const void* y_sorted, const int32_t* row_of_pair, const float* topk_w,
                  const void* shared_out, int num_shared, const void* residual, int T, int k, int H,
                  int dtype, void* out, void* stream);

/* Router scores g(x) = x . Wg^T (Sec. 2.1), fp32 accumulation, plus an optional per-class
 * additive bias (a property of synthetic traffic, not of the method):
 *     logits[t, e] = sum_h x[t, h] * Wg[e, h] + (bias ? bias[adapter_id[t]][e] : 0)
 *   x [dev] dtype [T, H]; Wg [dev] float32 [E, H]; adapter_id [dev] int32 [T] and
 *   bias [dev] float32 [N+1, E], both NULL or both set; logits [dev] float32 [T, E].
 * Limits: H % 4 == 0 (the matrix-core kernel runs for bf16 with H % 128 == 0).
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
int moe_gate_logits(const void* x, int dtype, const float* Wg, int T, int H, int E,
                    const int32_t* adapter_id, const float* bias, float* logits, void* stream);

/* Unit-gain RMS normalisation, out[t] = x[t] / sqrt(mean_h x[t][h]^2 + eps), fp32 arithmetic.
 * Not a step of the paper's method (Sec. 4.1: layers outside the MoE experts are left as they
 * are): an aid for chaining MoE layers as a pre-norm residual stack, h' = h + MoE(norm(h)), whose
 * activations would otherwise grow without bound with random-initialised experts.
 *   x [dev] dtype [T, H]; out [dev] dtype [T, H] (may be x).  Limits: H % 8 == 0 (bf16), % 4 (f32).
 * Errors: INVALID_ARG, UNSUPPORTED, HIP. */
int moe_rmsnorm(const void* x, int dtype, int T, int H, float eps, void* out, void* stream);

/* moe_unpermute and the moe_rmsnorm of its result in one launch, for stacked layers: `out` is the
 * next residual stream and `normed_out` (same shape and dtype, a different buffer) the next
 * layer's input.  Bit for bit what the two calls give (the norm is taken from the rounded `out`).
 * Arguments, limits and errors as for the two calls. */
int moe_unpermute_rmsnorm(const void* y_sorted, const int32_t* row_of_pair, const float* topk_w,
                          const void* shared_out, int num_shared, const void* residual, int T, int k,
                          int H, int dtype, void* out, float eps, void* normed_out, void* stream);

/* ===================================================================================== *
 * Measurement aids (not on the hot path): what the GPU sustains, timed by the caller with events
 * in the same run as the hot path, for quoting roofline fractions against achievable peaks.
 * ===================================================================================== */

/* Streams `bytes` (a multiple of 16; both buffers [dev], 16-byte aligned) with 16-byte accesses.
 * read_only != 0: every byte of src is read and consumed, dst (at least 16 bytes) is a sink that
 * is practically never written.  read_only == 0: plain copy src -> dst.
 * Errors: INVALID_ARG, HIP. */
int ew_probe_stream(const void* src, void* dst, size_t bytes, int read_only, void* stream);

/* Register-resident loop of the bf16 matrix-core instruction the grouped FFN uses
 * (v_mfma_f32_32x32x16_bf16, eight accumulators per wave, no memory access in the loop):
 * `workgroups` workgroups of 8 waves, `iters` rounds of 8 MFMAs per wave, i.e.
 * workgroups * 8 * iters * 8 * 32768 flop per launch.  random_operands != 0 fills the operands
 * with pseudo-random bf16 values instead of ones (the sustained clock depends on the data).
 * out [dev] uint64 [4 * workgroups]: per workgroup, shader-clock ticks and 100 MHz reference
 * ticks of its first wave's loop (their ratio gives the clock during the loop), and a checksum.
 * Errors: INVALID_ARG, HIP. */
int ew_probe_mfma_bf16(int workgroups, int iters, int random_operands, unsigned long long* out,
                       void* stream);

/* ===================================================================================== *
 * Tuning hooks for sweeps and tests.  Process-global and not thread-safe: not for serving code.
 * ===================================================================================== */

/* Kernel selection of moe_grouped_ffn(bf16).  Every argument: 0 = automatic.
 *   path                1 = register-streaming kernel, 2 = LDS-tiled GEMM kernel,
 *                       3 = LDS-direct streaming kernel (the automatic choice wherever it applies)
 *   stream_token_tiles  path 1: 16-token tiles per slot chunk (1 or 2)
 *   stream_threads      path 1: threads per block (a multiple of 64, at most 512)
 *   ws_frags            path 3: kernel shape, 32-token fragments per row chunk (1, 2, 4 or 8)
 *   ws_chunk_frags      path 3: cap on the fragments per row chunk (1..ws_frags)
 *   ws_wait_ticks       path 3: longest rendezvous wait of a workgroup for the other workgroups of
 *                       its slot, in 10 ns ticks; 0 = never wait, negative = automatic
 *   ws_two_launches     path 3, decode shapes (ws_frags < 8): non-zero = the two products as two
 *                       launches, as the 256-row shape always runs them; 0 = one launch for both */
void ew_tune_ffn(int path, int stream_token_tiles, int stream_threads, int ws_frags,
                 int ws_chunk_frags, int ws_wait_ticks, int ws_two_launches);

/* moe_reroute_permute / moe_route_reroute_permute: number of pairs (T*k) up to which the
 * single-block permutation runs (clamped to [0, 4096]; default 2048). */
void ew_tune_route(int small_pairs);

#ifdef __cplusplus
}
#endif
#endif /* EXPERTWEAVE_H */
