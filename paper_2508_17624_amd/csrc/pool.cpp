// Expert pool: virtual weight tensors, physical page pool, ESFT expert map.
//
// Paper Sec. 4.2: one contiguous *virtual* range per stacked weight tensor [P, H_out, H_in];
// physical pages of one fixed size back only the byte ranges of loaded experts; a page that a
// range covers only partly is shared with its neighbour and lives until its last user leaves
// (sub-page allocation with reference counting); evicted pages return to the pool and are reused.
// Sec. 4.1: the expert map Pi (one identity row for base tokens on top).
//
// Eviction is lazy by default: a page whose last user leaves stays mapped where it is ("parked").
// The expert-map row is reset first, so no token can reach it.  A parked page is reused in place
// when the same byte range is loaded again (no VMM call at all), is unmapped and moved when the
// pool needs a page elsewhere and its free list is empty (oldest parked page first), and is
// unmapped by expert_pool_trim.  Unmapping is by far the slowest VMM call (about a quarter of a
// millisecond per 2 MiB page measured on MI355X), so it is kept off the adapter-churn path.
// EW_POOL_EAGER_UNMAP restores unmap-at-evict.
//
// The VMM calls sit behind a small backend interface so the page/refcount logic runs on a
// GPU-less host too: HipVmm uses hipMemAddressReserve / hipMemCreate / hipMemMap /
// hipMemSetAccess / hipMemUnmap (the HIP counterparts of the paper's Table 2), FakeVmm uses
// mmap(PROT_NONE) + mprotect so that touching an unmapped slot faults on the host as well.
#include <sys/mman.h>

#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <vector>

#include "ew_internal.h"

namespace {

using ew::fail;

// ------------------------------------------------------------------------------------------
struct Backend {
  size_t page = 0;
  virtual ~Backend() {}
  // virt_total: bytes of address space the pool will reserve (sizes the default page)
  virtual int init(size_t requested_page, size_t virt_total) = 0;
  virtual int reserve(size_t bytes, void** va) = 0;
  virtual int unreserve(void* va, size_t bytes) = 0;
  virtual int create(uint64_t* h) = 0;
  virtual int release(uint64_t h) = 0;
  virtual int map(void* va, uint64_t h) = 0;
  virtual int unmap(void* va) = 0;
  virtual int copy_in(void* dst, const void* src, size_t n, void* stream) = 0;
  virtual int alloc_small(void** p, size_t n) = 0;
  virtual int free_small(void* p) = 0;
  virtual int sync(void* stream) = 0;
  virtual bool is_fake() const { return false; }
};

// ------------------------------------------------------------------------------------------
struct HipVmm final : Backend {
  int device;
  hipMemAllocationProp prop{};
  explicit HipVmm(int dev) : device(dev) {}

  int init(size_t requested_page, size_t virt_total) override {
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || device < 0 || device >= count)
      return fail(EW_ERR_HIP, "expert_pool_create: HIP device %d not available (%s)", device,
                  e == hipSuccess ? "index out of range" : hipGetErrorString(e));
    EW_HIP(hipSetDevice(device));
    int vmm = 0;
    EW_HIP(hipDeviceGetAttribute(&vmm, hipDeviceAttributeVirtualMemoryManagementSupported, device));
    if (!vmm) return fail(EW_ERR_VMM, "device %d reports no virtual memory management support", device);
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = device;
    size_t gmin = 0, grec = 0;
    EW_HIP(hipMemGetAllocationGranularity(&gmin, &prop, hipMemAllocationGranularityMinimum));
    EW_HIP(hipMemGetAllocationGranularity(&grec, &prop, hipMemAllocationGranularityRecommended));
    if (gmin == 0) gmin = 4096;
    if (grec < gmin) grec = gmin;
    // The runtime may recommend a granularity as small as 4 KiB, but every physical page is a
    // handle of its own and the driver runs out of them long before it runs out of memory;
    // 2 MiB (the size the paper quotes in Sec. 4.2) keeps a 100 GiB pool near 50K handles.
    // The driver also caps the number of live physical handles (allocation failed at about 32K
    // of them on MI355X / ROCm 7), so the default page doubles until a fully backed pool would
    // stay under 24K pages: 2 MiB for one layer of 384 slots, 8 MiB for 26 such layers.
    const size_t kDefaultPage = (size_t)2 << 20, kMaxPages = 24576;
    size_t def = grec > kDefaultPage ? grec : ew::align_up(kDefaultPage, gmin);
    while (virt_total / def > kMaxPages) def *= 2;
    page = requested_page ? requested_page : def;
    if (page % gmin) return fail(EW_ERR_INVALID_ARG, "page_bytes %zu is not a multiple of the granularity %zu", page, gmin);
    return EW_OK;
  }
  int reserve(size_t bytes, void** va) override {
    hipError_t e = hipMemAddressReserve(va, bytes, page, nullptr, 0);
    if (e != hipSuccess) return fail(EW_ERR_VMM, "hipMemAddressReserve(%zu): %s", bytes, hipGetErrorString(e));
    return EW_OK;
  }
  int unreserve(void* va, size_t bytes) override {
    hipError_t e = hipMemAddressFree(va, bytes);
    if (e != hipSuccess) return fail(EW_ERR_VMM, "hipMemAddressFree: %s", hipGetErrorString(e));
    return EW_OK;
  }
  int create(uint64_t* h) override {
    hipMemGenericAllocationHandle_t handle;
    hipError_t e = hipMemCreate(&handle, page, &prop, 0);
    if (e != hipSuccess) return fail(EW_ERR_OOM, "hipMemCreate(%zu): %s", page, hipGetErrorString(e));
    *h = (uint64_t)(uintptr_t)handle;
    return EW_OK;
  }
  int release(uint64_t h) override {
    hipError_t e = hipMemRelease((hipMemGenericAllocationHandle_t)(uintptr_t)h);
    if (e != hipSuccess) return fail(EW_ERR_VMM, "hipMemRelease: %s", hipGetErrorString(e));
    return EW_OK;
  }
  int map(void* va, uint64_t h) override {
    hipError_t e = hipMemMap(va, page, 0, (hipMemGenericAllocationHandle_t)(uintptr_t)h, 0);
    if (e != hipSuccess) return fail(EW_ERR_VMM, "hipMemMap: %s", hipGetErrorString(e));
    hipMemAccessDesc desc{};
    desc.location.type = hipMemLocationTypeDevice;
    desc.location.id = device;
    desc.flags = hipMemAccessFlagsProtReadWrite;
    e = hipMemSetAccess(va, page, &desc, 1);
    if (e != hipSuccess) {
      (void)hipMemUnmap(va, page);
      return fail(EW_ERR_VMM, "hipMemSetAccess: %s", hipGetErrorString(e));
    }
    return EW_OK;
  }
  int unmap(void* va) override {
    hipError_t e = hipMemUnmap(va, page);
    if (e != hipSuccess) return fail(EW_ERR_VMM, "hipMemUnmap: %s", hipGetErrorString(e));
    return EW_OK;
  }
  int copy_in(void* dst, const void* src, size_t n, void* stream) override {
    EW_HIP(hipMemcpyAsync(dst, src, n, hipMemcpyDefault, (hipStream_t)stream));
    return EW_OK;
  }
  int alloc_small(void** p, size_t n) override {
    EW_HIP(hipMalloc(p, n));
    return EW_OK;
  }
  int free_small(void* p) override {
    EW_HIP(hipFree(p));
    return EW_OK;
  }
  int sync(void* stream) override {
    EW_HIP(hipStreamSynchronize((hipStream_t)stream));
    return EW_OK;
  }
};

// ------------------------------------------------------------------------------------------
struct FakeVmm final : Backend {
  uint64_t next_handle = 1;
  int fail_op = -1, fail_countdown = 0;

  bool should_fail(int op) {
    if (op != fail_op || fail_countdown <= 0) return false;
    if (--fail_countdown == 0) {
      fail_op = -1;
      return true;
    }
    return false;
  }
  bool is_fake() const override { return true; }
  int init(size_t requested_page, size_t virt_total) override {
    page = requested_page ? requested_page : (size_t)(64 << 10);
    if (page % 4096) return fail(EW_ERR_INVALID_ARG, "page_bytes %zu is not a multiple of 4096", page);
    return EW_OK;
  }
  int reserve(size_t bytes, void** va) override {
    void* p = mmap(nullptr, bytes, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
    if (p == MAP_FAILED) return fail(EW_ERR_VMM, "fake reserve: mmap(%zu) failed", bytes);
    *va = p;
    return EW_OK;
  }
  int unreserve(void* va, size_t bytes) override {
    return munmap(va, bytes) == 0 ? EW_OK : fail(EW_ERR_VMM, "fake unreserve: munmap failed");
  }
  int create(uint64_t* h) override {
    if (should_fail(0)) return fail(EW_ERR_OOM, "fake create: injected failure");
    *h = next_handle++;
    return EW_OK;
  }
  int release(uint64_t) override { return EW_OK; }
  int map(void* va, uint64_t) override {
    if (should_fail(1)) return fail(EW_ERR_VMM, "fake map: injected failure");
    return mprotect(va, page, PROT_READ | PROT_WRITE) == 0 ? EW_OK : fail(EW_ERR_VMM, "fake map: mprotect failed");
  }
  int unmap(void* va) override {
    if (should_fail(2)) return fail(EW_ERR_VMM, "fake unmap: injected failure");
    (void)madvise(va, page, MADV_DONTNEED);
    return mprotect(va, page, PROT_NONE) == 0 ? EW_OK : fail(EW_ERR_VMM, "fake unmap: mprotect failed");
  }
  int copy_in(void* dst, const void* src, size_t n, void*) override {
    memcpy(dst, src, n);
    return EW_OK;
  }
  int alloc_small(void** p, size_t n) override {
    *p = malloc(n);
    return *p ? EW_OK : fail(EW_ERR_OOM, "fake alloc failed");
  }
  int free_small(void* p) override {
    free(p);
    return EW_OK;
  }
  int sync(void*) override { return EW_OK; }
};

// ------------------------------------------------------------------------------------------
struct Tensor {
  char* va = nullptr;
  size_t va_bytes = 0;
  size_t expert_bytes = 0;
  std::vector<int32_t> ref;      // users per page
  std::vector<uint64_t> handle;  // physical page mapped at each page index (valid while ref > 0 or parked)
  std::vector<uint64_t> parked;  // 0 = not parked, else the stamp of its entry in the pool's parked queue
};

struct ParkedRef {               // entry of the parked queue; stale once the page's stamp differs
  Tensor* t;
  size_t q;
  uint64_t stamp;
};

struct Layer {
  Tensor t[2];                    // 0 = W13, 1 = W2
  std::vector<int32_t> map_host;  // [N+1][M]
  int32_t* map_dev = nullptr;
  std::vector<int> loaded;        // per class 0..N: number of experts loaded, -1 = not loaded
};

}  // namespace

struct ew_pool {
  Backend* be = nullptr;
  int L = 0, M = 0, N = 0, E_max = 0, P = 0, flags = 0;
  std::vector<Layer> layers;
  std::vector<uint64_t> free_pages;
  std::deque<ParkedRef> parked;    // evicted pages still mapped at their old address, oldest first
  uint64_t pages_parked = 0, park_clock = 0;
  uint64_t pages_mapped = 0, pages_created = 0, pages_released = 0;
  std::vector<uint64_t> last_use;  // per class 0..N: tick of the last map or touch (eviction order)
  uint64_t tick = 0;
  std::mutex mu;
};

namespace {

struct DeviceGuard {  // makes the pool's device current for the duration of a call
  int prev = -1;
  bool active = false;
  explicit DeviceGuard(ew_pool* p) {
    if (p->be->is_fake()) return;
    if (hipGetDevice(&prev) == hipSuccess) {
      int dev = static_cast<HipVmm*>(p->be)->device;
      if (dev != prev) {
        (void)hipSetDevice(dev);
        active = true;
      }
    }
  }
  ~DeviceGuard() {
    if (active) (void)hipSetDevice(prev);
  }
};

void park_page(ew_pool* p, Tensor& t, size_t q) {
  t.parked[q] = ++p->park_clock;
  p->parked.push_back(ParkedRef{&t, q, t.parked[q]});
  ++p->pages_parked;
  // entries of pages that were reused in place are dropped lazily; keep the queue proportional
  if (p->parked.size() > 2 * p->pages_parked + 64) {
    std::deque<ParkedRef> live;
    for (const ParkedRef& r : p->parked)
      if (r.t->parked[r.q] == r.stamp) live.push_back(r);
    p->parked.swap(live);
  }
}

// Unmaps parked pages, oldest first, into the free list until `want` of them have moved or none
// is left.  A page whose unmap fails is still mapped, so it simply stays parked (at the back of
// the queue); the first such error is returned after the sweep.
int unpark_pages(ew_pool* p, size_t want, size_t* moved) {
  int first = EW_OK;
  *moved = 0;
  size_t budget = p->parked.size();
  while (*moved < want && budget-- > 0 && !p->parked.empty()) {
    ParkedRef r = p->parked.front();
    p->parked.pop_front();
    if (r.t->parked[r.q] != r.stamp) continue;  // stale: reused in place since
    int rc = p->be->unmap(r.t->va + r.q * p->be->page);
    if (rc != EW_OK) {
      if (first == EW_OK) first = rc;
      p->parked.push_back(r);
      continue;
    }
    p->free_pages.push_back(r.t->handle[r.q]);
    r.t->handle[r.q] = 0;
    r.t->parked[r.q] = 0;
    --p->pages_parked;
    ++*moved;
  }
  return first;
}

int acquire_page(ew_pool* p, uint64_t* h) {
  if (p->free_pages.empty() && p->pages_parked > 0) {
    size_t moved = 0;
    (void)unpark_pages(p, 1, &moved);  // on failure fall through to the runtime
  }
  if (!p->free_pages.empty()) {
    *h = p->free_pages.back();
    p->free_pages.pop_back();
    return EW_OK;
  }
  int rc = p->be->create(h);
  if (rc == EW_OK) ++p->pages_created;
  return rc;
}

inline void page_span(const Tensor& t, size_t page, int slot0, int n, size_t* q0, size_t* q1) {
  size_t b0 = (size_t)slot0 * t.expert_bytes, b1 = (size_t)(slot0 + n) * t.expert_bytes;
  *q0 = b0 / page;
  *q1 = (b1 - 1) / page + 1;  // exclusive
}

// Drops one reference from pages [q0, q1).  A page that reaches zero is parked (lazy pools) or
// unmapped into the free list (EW_POOL_EAGER_UNMAP); a page whose unmap fails is still mapped and
// is parked instead, so the page table stays true.  Keeps going on errors and reports the first.
int drop_pages(ew_pool* p, Tensor& t, size_t q0, size_t q1) {
  int first = EW_OK;
  const bool eager = (p->flags & EW_POOL_EAGER_UNMAP) != 0;
  for (size_t q = q0; q < q1; ++q) {
    if (--t.ref[q] == 0) {
      --p->pages_mapped;
      int rc = eager ? p->be->unmap(t.va + q * p->be->page) : EW_OK;
      if (eager && rc == EW_OK) {
        p->free_pages.push_back(t.handle[q]);
        t.handle[q] = 0;
      } else {
        if (rc != EW_OK && first == EW_OK) first = rc;
        park_page(p, t, q);
      }
    }
  }
  return first;
}

// Adds one reference to every page under slots [slot0, slot0+n), mapping pages that had none.
// On failure nothing changes.
int load_range(ew_pool* p, Tensor& t, int slot0, int n) {
  if (n <= 0) return EW_OK;
  size_t q0, q1;
  page_span(t, p->be->page, slot0, n, &q0, &q1);
  for (size_t q = q0; q < q1; ++q) {
    if (t.ref[q] == 0 && t.parked[q] != 0) {  // evicted earlier and still in place: take it back as it is
      t.parked[q] = 0;
      --p->pages_parked;
      ++p->pages_mapped;
    } else if (t.ref[q] == 0) {
      uint64_t h = 0;
      int rc = acquire_page(p, &h);
      if (rc == EW_OK) {
        rc = p->be->map(t.va + q * p->be->page, h);
        if (rc != EW_OK) p->free_pages.push_back(h);
      }
      if (rc != EW_OK) {
        char msg[512];
        snprintf(msg, sizeof(msg), "%s", ew_last_error());
        (void)drop_pages(p, t, q0, q);  // roll back what this call did
        return fail(rc, "%s (rolled back %zu pages)", msg, q - q0);
      }
      t.handle[q] = h;
      ++p->pages_mapped;
    }
    ++t.ref[q];
  }
  return EW_OK;
}

int unload_range(ew_pool* p, Tensor& t, int slot0, int n) {
  if (n <= 0) return EW_OK;
  size_t q0, q1;
  page_span(t, p->be->page, slot0, n, &q0, &q1);
  return drop_pages(p, t, q0, q1);
}

int slot0_of(const ew_pool* p, int adapter_id) { return adapter_id == 0 ? 0 : p->M + (adapter_id - 1) * p->E_max; }

void destroy_impl(ew_pool* p) {
  if (!p) return;
  if (p->be) {
    for (Layer& ly : p->layers) {
      for (Tensor& t : ly.t) {
        if (!t.va) continue;
        for (size_t q = 0; q < t.ref.size(); ++q)
          if (t.ref[q] > 0 || t.parked[q] != 0) {
            (void)p->be->unmap(t.va + q * p->be->page);
            p->free_pages.push_back(t.handle[q]);
          }
        (void)p->be->unreserve(t.va, t.va_bytes);
      }
      if (ly.map_dev) (void)p->be->free_small(ly.map_dev);
    }
    for (uint64_t h : p->free_pages) (void)p->be->release(h);
    delete p->be;
  }
  delete p;
}

int check_pool_layer(ew_pool* p, int layer, const char* who) {
  if (!p) return fail(EW_ERR_INVALID_ARG, "%s: pool is NULL", who);
  if (layer < 0 || layer >= p->L) return fail(EW_ERR_INVALID_ARG, "%s: layer %d outside [0,%d)", who, layer, p->L);
  return EW_OK;
}

}  // namespace

// ==========================================================================================
extern "C" int expert_pool_create(ew_pool** out, int device, int num_layers, int M, int N, int E_max,
                                  size_t w13_bytes, size_t w2_bytes, size_t page_bytes,
                                  size_t prealloc_pages, int flags) {
  if (!out) return fail(EW_ERR_INVALID_ARG, "expert_pool_create: out is NULL");
  *out = nullptr;
  if (num_layers < 1 || M < 1 || N < 0 || E_max < 0 || w13_bytes == 0 || w2_bytes == 0)
    return fail(EW_ERR_INVALID_ARG, "expert_pool_create: need num_layers>=1, M>=1, N>=0, E_max>=0, expert bytes>0");
  if (N > 0 && E_max < 1) return fail(EW_ERR_INVALID_ARG, "expert_pool_create: E_max must be >= 1 when N > 0");
  if (flags & ~(EW_POOL_PADDED | EW_POOL_FAKE | EW_POOL_EAGER_UNMAP)) return fail(EW_ERR_INVALID_ARG, "expert_pool_create: unknown flags 0x%x", flags);
  long long P = (long long)M + (long long)N * E_max;
  if (P > (1 << 20)) return fail(EW_ERR_INVALID_ARG, "expert_pool_create: P = %lld slots is too many", P);

  ew_pool* p = new (std::nothrow) ew_pool;
  if (!p) return fail(EW_ERR_OOM, "expert_pool_create: host allocation failed");
  p->L = num_layers; p->M = M; p->N = N; p->E_max = E_max; p->P = (int)P; p->flags = flags;
  p->last_use.assign(N + 1, 0);
  p->be = (flags & EW_POOL_FAKE) ? static_cast<Backend*>(new FakeVmm) : static_cast<Backend*>(new HipVmm(device));
  int rc = p->be->init(page_bytes, (size_t)num_layers * (size_t)P * (w13_bytes + w2_bytes));
  if (rc != EW_OK) { destroy_impl(p); return rc; }
  DeviceGuard guard(p);
  const size_t page = p->be->page;
  const size_t eb[2] = {w13_bytes, w2_bytes};
  p->layers.resize(num_layers);
  for (Layer& ly : p->layers) {
    for (int w = 0; w < 2; ++w) {
      Tensor& t = ly.t[w];
      t.expert_bytes = eb[w];
      t.va_bytes = ew::align_up((size_t)P * eb[w], page);
      void* va = nullptr;
      rc = p->be->reserve(t.va_bytes, &va);
      if (rc != EW_OK) { destroy_impl(p); return rc; }
      t.va = (char*)va;
      t.ref.assign(t.va_bytes / page, 0);
      t.handle.assign(t.va_bytes / page, 0);
      t.parked.assign(t.va_bytes / page, 0);
    }
    ly.map_host.resize((size_t)(N + 1) * M);
    for (int a = 0; a <= N; ++a)
      for (int e = 0; e < M; ++e) ly.map_host[(size_t)a * M + e] = e;
    ly.loaded.assign(N + 1, -1);
    void* d = nullptr;
    rc = p->be->alloc_small(&d, ly.map_host.size() * sizeof(int32_t));
    if (rc == EW_OK) {
      ly.map_dev = (int32_t*)d;
      rc = p->be->copy_in(d, ly.map_host.data(), ly.map_host.size() * sizeof(int32_t), nullptr);
    }
    if (rc != EW_OK) { destroy_impl(p); return rc; }
  }
  rc = p->be->sync(nullptr);
  for (size_t i = 0; rc == EW_OK && i < prealloc_pages; ++i) {
    uint64_t h;
    rc = p->be->create(&h);
    if (rc == EW_OK) { p->free_pages.push_back(h); ++p->pages_created; }
  }
  if (rc == EW_OK && (flags & EW_POOL_PADDED)) {
    // The padding approach: back every slot, used or not, for the pool's whole life.
    for (Layer& ly : p->layers)
      for (Tensor& t : ly.t)
        if (rc == EW_OK) rc = load_range(p, t, 0, p->P);
  }
  if (rc != EW_OK) { destroy_impl(p); return rc; }
  *out = p;
  return EW_OK;
}

extern "C" int expert_pool_destroy(ew_pool* pool) {
  if (!pool) return fail(EW_ERR_INVALID_ARG, "expert_pool_destroy: pool is NULL");
  {
    DeviceGuard guard(pool);
    (void)pool->be->sync(nullptr);
  }
  DeviceGuard guard(pool);
  Backend* be = pool->be;
  (void)be;
  destroy_impl(pool);
  return EW_OK;
}

extern "C" int expert_pool_map(ew_pool* p, int layer, int adapter_id, int n, const int32_t* expert_ids,
                               const void* w13, const void* w2, void* stream) {
  int rc = check_pool_layer(p, layer, "expert_pool_map");
  if (rc != EW_OK) return rc;
  if (adapter_id < 0 || adapter_id > p->N)
    return fail(EW_ERR_INVALID_ARG, "expert_pool_map: adapter_id %d outside [0,%d]", adapter_id, p->N);
  if (adapter_id == 0) {
    if (n != p->M) return fail(EW_ERR_INVALID_ARG, "expert_pool_map: the base model loads all M=%d experts, got n=%d", p->M, n);
    for (int e = 0; expert_ids && e < n; ++e)
      if (expert_ids[e] != e) return fail(EW_ERR_INVALID_ARG, "expert_pool_map: base expert_ids must be 0..M-1");
  } else {
    if (n < 0 || n > p->E_max) return fail(EW_ERR_INVALID_ARG, "expert_pool_map: n=%d outside [0,E_max=%d]", n, p->E_max);
    if (n > 0 && !expert_ids) return fail(EW_ERR_INVALID_ARG, "expert_pool_map: expert_ids is NULL");
    for (int d = 0; d < n; ++d) {
      if (expert_ids[d] < 0 || expert_ids[d] >= p->M)
        return fail(EW_ERR_INVALID_ARG, "expert_pool_map: expert id %d outside [0,%d)", expert_ids[d], p->M);
      if (d && expert_ids[d] <= expert_ids[d - 1])
        return fail(EW_ERR_INVALID_ARG, "expert_pool_map: expert_ids must be strictly ascending");
    }
  }
  std::lock_guard<std::mutex> lock(p->mu);
  DeviceGuard guard(p);
  Layer& ly = p->layers[layer];
  if (ly.loaded[adapter_id] >= 0)
    return fail(EW_ERR_STATE, "expert_pool_map: layer %d adapter %d is already loaded", layer, adapter_id);
  const int slot0 = slot0_of(p, adapter_id);
  rc = load_range(p, ly.t[0], slot0, n);
  if (rc != EW_OK) return rc;
  rc = load_range(p, ly.t[1], slot0, n);
  if (rc != EW_OK) {
    char msg[512];
    snprintf(msg, sizeof(msg), "%s", ew_last_error());
    (void)unload_range(p, ly.t[0], slot0, n);
    return fail(rc, "%s", msg);
  }
  const void* src[2] = {w13, w2};
  for (int w = 0; w < 2 && rc == EW_OK; ++w)
    if (n > 0 && src[w])
      rc = p->be->copy_in(ly.t[w].va + (size_t)slot0 * ly.t[w].expert_bytes, src[w], (size_t)n * ly.t[w].expert_bytes, stream);
  if (rc == EW_OK && adapter_id > 0) {
    int32_t* row = &ly.map_host[(size_t)adapter_id * p->M];
    for (int d = 0; d < n; ++d) row[expert_ids[d]] = slot0 + d;  // Pi[i, j] = Delta_i + delta_ij
    rc = p->be->copy_in(ly.map_dev + (size_t)adapter_id * p->M, row, p->M * sizeof(int32_t), stream);
    if (rc != EW_OK)
      for (int e = 0; e < p->M; ++e) row[e] = e;
  }
  if (rc != EW_OK) {
    char msg[512];
    snprintf(msg, sizeof(msg), "%s", ew_last_error());
    (void)p->be->sync(stream);
    (void)unload_range(p, ly.t[0], slot0, n);
    (void)unload_range(p, ly.t[1], slot0, n);
    return fail(rc, "%s", msg);
  }
  ly.loaded[adapter_id] = n;
  p->last_use[adapter_id] = ++p->tick;
  return EW_OK;
}

extern "C" int expert_pool_unmap(ew_pool* p, int layer, int adapter_id, void* stream) {
  int rc = check_pool_layer(p, layer, "expert_pool_unmap");
  if (rc != EW_OK) return rc;
  if (adapter_id < 0 || adapter_id > p->N)
    return fail(EW_ERR_INVALID_ARG, "expert_pool_unmap: adapter_id %d outside [0,%d]", adapter_id, p->N);
  std::lock_guard<std::mutex> lock(p->mu);
  DeviceGuard guard(p);
  Layer& ly = p->layers[layer];
  const int n = ly.loaded[adapter_id];
  if (n < 0) return fail(EW_ERR_STATE, "expert_pool_unmap: layer %d adapter %d is not loaded", layer, adapter_id);
  if (adapter_id > 0) {
    int32_t* row = &ly.map_host[(size_t)adapter_id * p->M];
    for (int e = 0; e < p->M; ++e) row[e] = e;
    rc = p->be->copy_in(ly.map_dev + (size_t)adapter_id * p->M, row, p->M * sizeof(int32_t), stream);
    if (rc != EW_OK) return rc;
  }
  rc = p->be->sync(stream);  // the identity row is in place before any page goes away
  if (rc != EW_OK) return rc;
  const int slot0 = slot0_of(p, adapter_id);
  int r0 = unload_range(p, ly.t[0], slot0, n);
  int r1 = unload_range(p, ly.t[1], slot0, n);
  ly.loaded[adapter_id] = -1;
  return r0 != EW_OK ? r0 : r1;
}

extern "C" int expert_pool_touch(ew_pool* p, int n, const int32_t* adapter_ids) {
  if (!p) return fail(EW_ERR_INVALID_ARG, "expert_pool_touch: pool is NULL");
  if (n < 0 || (n > 0 && !adapter_ids)) return fail(EW_ERR_INVALID_ARG, "expert_pool_touch: bad id list");
  for (int i = 0; i < n; ++i)
    if (adapter_ids[i] < 0 || adapter_ids[i] > p->N)
      return fail(EW_ERR_INVALID_ARG, "expert_pool_touch: adapter_id %d outside [0,%d]", adapter_ids[i], p->N);
  std::lock_guard<std::mutex> lock(p->mu);
  const uint64_t now = ++p->tick;  // one tick per call: the ids of one batch are equally recent
  for (int i = 0; i < n; ++i) p->last_use[adapter_ids[i]] = now;
  return EW_OK;
}

extern "C" int expert_pool_lru_victim(ew_pool* p, int* adapter_id) {
  if (!p || !adapter_id) return fail(EW_ERR_INVALID_ARG, "expert_pool_lru_victim: NULL argument");
  std::lock_guard<std::mutex> lock(p->mu);
  int best = -1;
  for (int a = 1; a <= p->N; ++a) {
    bool loaded = false;
    for (const Layer& ly : p->layers) loaded = loaded || ly.loaded[a] >= 0;
    if (loaded && (best < 0 || p->last_use[a] < p->last_use[best])) best = a;  // ties: lower id
  }
  *adapter_id = best;
  return EW_OK;
}

extern "C" int expert_pool_view(ew_pool* p, int layer, void** w13_base, void** w2_base,
                                const int32_t** expert_map, int* num_slots) {
  int rc = check_pool_layer(p, layer, "expert_pool_view");
  if (rc != EW_OK) return rc;
  Layer& ly = p->layers[layer];
  if (w13_base) *w13_base = ly.t[0].va;
  if (w2_base) *w2_base = ly.t[1].va;
  if (expert_map) *expert_map = ly.map_dev;
  if (num_slots) *num_slots = p->P;
  return EW_OK;
}

extern "C" int expert_pool_expert_map_host(ew_pool* p, int layer, int32_t* out) {
  int rc = check_pool_layer(p, layer, "expert_pool_expert_map_host");
  if (rc != EW_OK) return rc;
  if (!out) return fail(EW_ERR_INVALID_ARG, "expert_pool_expert_map_host: out is NULL");
  std::lock_guard<std::mutex> lock(p->mu);
  memcpy(out, p->layers[layer].map_host.data(), p->layers[layer].map_host.size() * sizeof(int32_t));
  return EW_OK;
}

extern "C" int expert_pool_stats(ew_pool* p, ew_pool_stats* out) {
  if (!p || !out) return fail(EW_ERR_INVALID_ARG, "expert_pool_stats: NULL argument");
  std::lock_guard<std::mutex> lock(p->mu);
  memset(out, 0, sizeof(*out));
  out->page_bytes = p->be->page;
  out->pages_mapped = p->pages_mapped;
  out->pages_free = p->free_pages.size();
  out->pages_parked = p->pages_parked;
  out->pages_created = p->pages_created;
  out->pages_released = p->pages_released;
  uint64_t used_slots = 0;
  bool any = false;
  for (const Layer& ly : p->layers) {
    for (const Tensor& t : ly.t) {
      out->bytes_virtual += t.va_bytes;
      for (int32_t r : t.ref)
        if (r > ((p->flags & EW_POOL_PADDED) ? 2 : 1)) ++out->pages_shared;
    }
    used_slots += p->M;
    for (int a = 0; a <= p->N; ++a) {
      if (ly.loaded[a] < 0) continue;
      any = true;
      out->experts_loaded += ly.loaded[a];
      out->bytes_experts += (uint64_t)ly.loaded[a] * (ly.t[0].expert_bytes + ly.t[1].expert_bytes);
      if (a > 0) used_slots += ly.loaded[a];
    }
  }
  out->f_mem = any ? (double)p->L * p->P / (double)used_slots : 0.0;
  return EW_OK;
}

extern "C" int expert_pool_trim(ew_pool* p, size_t keep_pages) {
  if (!p) return fail(EW_ERR_INVALID_ARG, "expert_pool_trim: pool is NULL");
  std::lock_guard<std::mutex> lock(p->mu);
  DeviceGuard guard(p);
  size_t moved = 0;
  int first = unpark_pages(p, (size_t)-1, &moved);
  while (p->free_pages.size() > keep_pages) {
    int rc = p->be->release(p->free_pages.back());
    p->free_pages.pop_back();
    ++p->pages_released;
    if (rc != EW_OK && first == EW_OK) first = rc;
  }
  return first;
}

extern "C" int expert_pool_fake_fail_at(ew_pool* p, int op, int n) {
  if (!p) return fail(EW_ERR_INVALID_ARG, "expert_pool_fake_fail_at: pool is NULL");
  if (!p->be->is_fake()) return fail(EW_ERR_STATE, "expert_pool_fake_fail_at: not a fake-backend pool");
  if (op < 0 || op > 2 || n < 0) return fail(EW_ERR_INVALID_ARG, "expert_pool_fake_fail_at: bad op/n");
  FakeVmm* f = static_cast<FakeVmm*>(p->be);
  f->fail_op = n ? op : -1;
  f->fail_countdown = n;
  return EW_OK;
}

extern "C" int expert_pool_fake_is_mapped(ew_pool* p, int layer, int which, size_t offset, int* out) {
  int rc = check_pool_layer(p, layer, "expert_pool_fake_is_mapped");
  if (rc != EW_OK) return rc;
  if (which < 0 || which > 1 || !out) return fail(EW_ERR_INVALID_ARG, "expert_pool_fake_is_mapped: bad argument");
  const Tensor& t = p->layers[layer].t[which];
  if (offset >= t.va_bytes) return fail(EW_ERR_INVALID_ARG, "expert_pool_fake_is_mapped: offset beyond the tensor");
  *out = t.ref[offset / p->be->page] > 0;
  return EW_OK;
}
