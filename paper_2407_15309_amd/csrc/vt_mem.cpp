// Region manager: per-request K and V virtual ranges backed by fixed-size physical chunks.
//
// Follows the paper's "vTensor Pool", "vTensor Operation" and "vTensor Scheduler": vAlloc reserves a range sized for
// the maximum sequence length and maps nothing; pAlloc takes idle chunks from the pool before asking
// the driver for new ones; Map attaches chunks at the next offsets of the range; Release unmaps and
// keeps everything for reuse (lazy deallocation); a chunk shared by several ranges is reference
// counted like a hard link.
#include <hip/hip_runtime.h>

#include <sys/mman.h>
#include <unistd.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "vt_internal.h"

namespace vt {

// ------------------------------------------------------------------------------------------------
// HIP backend: hipMemAddressReserve / hipMemCreate / hipMemMap / hipMemSetAccess
// ------------------------------------------------------------------------------------------------
class HipBackend final : public Backend {
 public:
  explicit HipBackend(int device) : device_(device), gran_(0) {
    std::memset(&prop_, 0, sizeof(prop_));
    prop_.type = hipMemAllocationTypePinned;
    prop_.location.type = hipMemLocationTypeDevice;
    prop_.location.id = device;
    std::memset(&access_, 0, sizeof(access_));
    access_.location.type = hipMemLocationTypeDevice;
    access_.location.id = device;
    access_.flags = hipMemAccessFlagsProtReadWrite;
  }
  int init() {
    size_t g = 0;
    if (hipMemGetAllocationGranularity(&g, &prop_, hipMemAllocationGranularityMinimum) != hipSuccess || g == 0)
      return VT_E_DRIVER;
    gran_ = g;
    return VT_OK;
  }
  int reserve(uint64_t size, uint64_t align, void** out) override {
    void* p = nullptr;
    if (hipMemAddressReserve(&p, size, align, nullptr, 0) != hipSuccess || !p) return VT_E_DRIVER;
    *out = p;
    return VT_OK;
  }
  int va_free(void* addr, uint64_t size) override {
    return hipMemAddressFree(addr, size) == hipSuccess ? VT_OK : VT_E_DRIVER;
  }
  int create(uint64_t size, void** handle) override {
    hipMemGenericAllocationHandle_t h;
    hipError_t e = hipMemCreate(&h, size, &prop_, 0);
    if (e == hipErrorOutOfMemory) {
      (void)hipGetLastError();
      return VT_E_OOM;
    }
    if (e != hipSuccess) return VT_E_DRIVER;
    *handle = (void*)h;
    return VT_OK;
  }
  int release(void* handle) override {
    return hipMemRelease((hipMemGenericAllocationHandle_t)handle) == hipSuccess ? VT_OK : VT_E_DRIVER;
  }
  int map(void* addr, uint64_t size, void* handle) override {
    if (hipMemMap(addr, size, 0, (hipMemGenericAllocationHandle_t)handle, 0) != hipSuccess) return VT_E_DRIVER;
    if (hipMemSetAccess(addr, size, &access_, 1) != hipSuccess) {
      (void)hipMemUnmap(addr, size);
      return VT_E_DRIVER;
    }
    return VT_OK;
  }
  int unmap(void* addr, uint64_t size) override {
    return hipMemUnmap(addr, size) == hipSuccess ? VT_OK : VT_E_DRIVER;
  }
  uint64_t granularity() const override { return gran_; }
  bool is_host() const override { return false; }

 private:
  int device_;
  uint64_t gran_;
  hipMemAllocationProp prop_;
  hipMemAccessDesc access_;
};

// ------------------------------------------------------------------------------------------------
// Host backend: PROT_NONE mmap as the reserved range, one memfd per chunk, MAP_FIXED to map.
// ------------------------------------------------------------------------------------------------
class HostBackend final : public Backend {
 public:
  HostBackend() {
    for (int i = 0; i < 4; ++i) fail_[i] = 0;
  }
  int reserve(uint64_t size, uint64_t align, void** out) override {
    if (trip(0)) return VT_E_DRIVER;
    uint64_t raw_size = size + align;
    void* raw = mmap(nullptr, raw_size, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
    if (raw == MAP_FAILED) return VT_E_DRIVER;
    uintptr_t a = ((uintptr_t)raw + align - 1) / align * align;
    raw_[(void*)a] = {raw, raw_size};
    *out = (void*)a;
    return VT_OK;
  }
  int va_free(void* addr, uint64_t) override {
    auto it = raw_.find(addr);
    if (it == raw_.end()) return VT_E_DRIVER;
    munmap(it->second.first, it->second.second);
    raw_.erase(it);
    return VT_OK;
  }
  int create(uint64_t size, void** handle) override {
    if (trip(1)) return VT_E_OOM;
    int fd = memfd_create("vt_chunk", 0);
    if (fd < 0) return VT_E_DRIVER;
    if (ftruncate(fd, (off_t)size) != 0) {
      close(fd);
      return VT_E_OOM;
    }
    *handle = (void*)(intptr_t)(fd + 1);  // never NULL
    return VT_OK;
  }
  int release(void* handle) override {
    close((int)(intptr_t)handle - 1);
    return VT_OK;
  }
  int map(void* addr, uint64_t size, void* handle) override {
    if (trip(2)) return VT_E_DRIVER;
    void* p = mmap(addr, size, PROT_READ | PROT_WRITE, MAP_SHARED | MAP_FIXED, (int)(intptr_t)handle - 1, 0);
    return p == addr ? VT_OK : VT_E_DRIVER;
  }
  int unmap(void* addr, uint64_t size) override {
    if (trip(3)) return VT_E_DRIVER;
    void* p = mmap(addr, size, PROT_NONE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE | MAP_FIXED, -1, 0);
    return p == addr ? VT_OK : VT_E_DRIVER;
  }
  uint64_t granularity() const override { return (uint64_t)sysconf(_SC_PAGESIZE); }
  bool is_host() const override { return true; }
  void fail_after(int op, int countdown) { fail_[op] = countdown; }

 private:
  bool trip(int op) {
    if (fail_[op] > 0 && --fail_[op] == 0) return true;
    return false;
  }
  std::map<void*, std::pair<void*, uint64_t>> raw_;
  int fail_[4];
};

Backend* make_hip_backend(int device, int* status) {
  HipBackend* b = new (std::nothrow) HipBackend(device);
  if (!b) {
    *status = VT_E_OOM;
    return nullptr;
  }
  *status = b->init();
  if (*status != VT_OK) {
    delete b;
    return nullptr;
  }
  return b;
}
Backend* make_host_backend() { return new (std::nothrow) HostBackend(); }
int host_backend_fail_after(Backend* b, int op, int countdown) {
  if (!b || !b->is_host() || op < 0 || op > 3 || countdown < 0) return VT_E_INVALID;
  static_cast<HostBackend*>(b)->fail_after(op, countdown);
  return VT_OK;
}

namespace {

struct Timer {
  explicit Timer(vt_ctx* c) : c_(c), t0_(std::chrono::steady_clock::now()) {}
  ~Timer() {
    c_->st.driver_ns += (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
                            std::chrono::steady_clock::now() - t0_).count();
  }
  vt_ctx* c_;
  std::chrono::steady_clock::time_point t0_;
};

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

int make_ctx(vt_ctx** out, Backend* be, int device, uint64_t chunk_bytes, uint64_t max_phys) {
  if (chunk_bytes == 0) chunk_bytes = 2ull << 20;
  if (chunk_bytes % be->granularity() != 0) {
    delete be;
    return VT_E_INVALID;
  }
  vt_ctx* c = new (std::nothrow) vt_ctx();
  if (!c) {
    delete be;
    return VT_E_OOM;
  }
  c->magic = VT_CTX_MAGIC;
  c->device = device;
  c->be = be;
  c->chunk_bytes = chunk_bytes;
  c->max_phys_bytes = max_phys;
  c->plan_target = 0;
  std::memset(&c->st, 0, sizeof(c->st));
  c->ws = nullptr;
  c->ws_bytes = 0;
  c->arrivals = nullptr;
  c->prefill_launches = 0;
  {
    const char* wide = std::getenv("VT_PREFILL_WIDE");
    c->prefill_wide = wide && wide[0] == '1';
  }
  c->n_cus = 256;
  c->profile = false;
  *out = c;
  return VT_OK;
}

// VA range of `size` bytes: free-list first, then the driver.
int take_va(vt_ctx* c, uint64_t size, char** out) {
  auto it = c->va_free.find(size);
  if (it != c->va_free.end() && !it->second.empty()) {
    *out = it->second.back();
    it->second.pop_back();
    c->st.va_reused++;
    return VT_OK;
  }
  void* p = nullptr;
  int rc;
  {
    Timer t(c);
    rc = c->be->reserve(size, c->chunk_bytes, &p);
  }
  if (rc != VT_OK) return rc;
  c->st.va_reserved_calls++;
  c->st.reserved_va_bytes += size;
  *out = (char*)p;
  return VT_OK;
}

void give_va(vt_ctx* c, uint64_t size, char* p) { c->va_free[size].push_back(p); }

// pAlloc(n): pool first, then new allocations.  On failure nothing is kept.
int take_chunks(vt_ctx* c, uint64_t n, std::vector<Chunk*>* out) {
  uint64_t from_pool = std::min<uint64_t>(n, c->pool.size());
  uint64_t to_create = n - from_pool;
  if (c->max_phys_bytes && c->st.phys_bytes + to_create * c->chunk_bytes > c->max_phys_bytes) return VT_E_OOM;
  std::vector<Chunk*> created;
  for (uint64_t i = 0; i < to_create; ++i) {
    void* h = nullptr;
    int rc;
    {
      Timer t(c);
      rc = c->be->create(c->chunk_bytes, &h);
    }
    if (rc != VT_OK) {
      for (Chunk* k : created) {
        c->be->release(k->handle);
        delete k;
      }
      return rc;
    }
    created.push_back(new Chunk{h, 0});
  }
  for (uint64_t i = 0; i < from_pool; ++i) {
    out->push_back(c->pool.back());
    c->pool.pop_back();
  }
  for (Chunk* k : created) out->push_back(k);
  c->st.chunks_reused += from_pool;
  c->st.chunks_created += to_create;
  c->st.create_calls += to_create;
  c->st.phys_bytes += to_create * c->chunk_bytes;
  c->st.chunks_pooled = c->pool.size();
  return VT_OK;
}

void pool_chunk(vt_ctx* c, Chunk* k) {
  c->pool.push_back(k);
  c->st.chunks_pooled = c->pool.size();
}

int unmap_one(vt_ctx* c, char* addr, Chunk* k) {
  int rc;
  {
    Timer t(c);
    rc = c->be->unmap(addr, c->chunk_bytes);
  }
  c->st.unmap_calls++;
  if (rc == VT_OK) {
    c->st.mapped_bytes -= c->chunk_bytes;
    if (--k->refs == 0) pool_chunk(c, k);
  }
  return rc;
}

int map_one(vt_ctx* c, char* addr, Chunk* k) {
  int rc;
  {
    Timer t(c);
    rc = c->be->map(addr, c->chunk_bytes, k->handle);
  }
  c->st.map_calls++;
  if (rc == VT_OK) {
    c->st.mapped_bytes += c->chunk_bytes;
    k->refs++;
  }
  return rc;
}

int new_region(vt_ctx* ctx, uint32_t hkv, uint32_t d, int dtype, uint64_t max_tokens, vt_kv** out) {
  if (!hkv || !d || !max_tokens || (dtype != VT_F16 && dtype != VT_BF16)) return VT_E_INVALID;
  uint64_t row = (uint64_t)hkv * d * 2;
  if (max_tokens > (~0ull >> 2) / row) return VT_E_INVALID;
  uint64_t cap = ceil_div(max_tokens * row, ctx->chunk_bytes) * ctx->chunk_bytes;
  char *kb = nullptr, *vb = nullptr;
  int rc = take_va(ctx, cap, &kb);
  if (rc != VT_OK) return rc;
  rc = take_va(ctx, cap, &vb);
  if (rc != VT_OK) {
    give_va(ctx, cap, kb);
    return rc;
  }
  vt_kv* kv = new (std::nothrow) vt_kv();
  if (!kv) {
    give_va(ctx, cap, kb);
    give_va(ctx, cap, vb);
    return VT_E_OOM;
  }
  kv->magic = VT_KV_MAGIC;
  kv->alive = true;
  kv->ctx = ctx;
  kv->n_kv_heads = hkv;
  kv->head_dim = d;
  kv->dtype = dtype;
  kv->row_bytes = row;
  kv->max_tokens = max_tokens;
  kv->capacity_bytes = cap;
  kv->len = 0;
  kv->k_base = kb;
  kv->v_base = vb;
  kv->shared_chunks = 0;
  ctx->regions.push_back(kv);
  ctx->st.live_regions++;
  *out = kv;
  return VT_OK;
}

int extend_locked(vt_kv* kv, uint64_t new_len) {
  vt_ctx* c = kv->ctx;
  if (new_len < kv->len) return VT_E_INVALID;
  if (new_len > kv->max_tokens) return VT_E_CAPACITY;
  uint64_t need = ceil_div(new_len * kv->row_bytes, c->chunk_bytes);
  uint64_t have = kv->k_chunks.size();
  if (need > have) {
    uint64_t add = need - have;
    std::vector<Chunk*> got;
    int rc = take_chunks(c, 2 * add, &got);
    if (rc != VT_OK) return rc;
    // Map K chunks then V chunks at the next offsets; undo everything on a failure.
    uint64_t done = 0;
    for (; done < 2 * add; ++done) {
      bool is_k = done < add;
      uint64_t idx = have + (is_k ? done : done - add);
      char* addr = (is_k ? kv->k_base : kv->v_base) + idx * c->chunk_bytes;
      rc = map_one(c, addr, got[done]);
      if (rc != VT_OK) break;
    }
    if (rc != VT_OK) {
      for (uint64_t i = 0; i < done; ++i) {
        bool is_k = i < add;
        uint64_t idx = have + (is_k ? i : i - add);
        char* addr = (is_k ? kv->k_base : kv->v_base) + idx * c->chunk_bytes;
        (void)unmap_one(c, addr, got[i]);  // returns the chunk to the pool
      }
      for (uint64_t i = done; i < 2 * add; ++i) pool_chunk(c, got[i]);
      return rc;
    }
    for (uint64_t i = 0; i < add; ++i) kv->k_chunks.push_back(got[i]);
    for (uint64_t i = 0; i < add; ++i) kv->v_chunks.push_back(got[add + i]);
  }
  kv->len = new_len;
  return VT_OK;
}

int release_locked(vt_kv* kv) {
  vt_ctx* c = kv->ctx;
  int worst = VT_OK;
  for (size_t i = 0; i < kv->k_chunks.size(); ++i) {
    int rc = unmap_one(c, kv->k_base + i * c->chunk_bytes, kv->k_chunks[i]);
    if (rc != VT_OK) worst = rc;
  }
  for (size_t i = 0; i < kv->v_chunks.size(); ++i) {
    int rc = unmap_one(c, kv->v_base + i * c->chunk_bytes, kv->v_chunks[i]);
    if (rc != VT_OK) worst = rc;
  }
  kv->k_chunks.clear();
  kv->v_chunks.clear();
  if (worst == VT_OK) {  // a range that failed to unmap is not handed out again
    give_va(c, kv->capacity_bytes, kv->k_base);
    give_va(c, kv->capacity_bytes, kv->v_base);
  }
  kv->alive = false;
  kv->len = 0;
  c->st.live_regions--;
  return worst;
}

int trim_locked(vt_ctx* c, uint64_t keep) {
  int worst = VT_OK;
  while (c->pool.size() > keep) {
    Chunk* k = c->pool.back();
    c->pool.pop_back();
    int rc;
    {
      Timer t(c);
      rc = c->be->release(k->handle);
    }
    c->st.release_calls++;
    if (rc != VT_OK) worst = rc;
    c->st.phys_bytes -= c->chunk_bytes;
    delete k;
  }
  c->st.chunks_pooled = c->pool.size();
  for (auto& kvp : c->va_free) {
    for (char* p : kvp.second) {
      int rc;
      {
        Timer t(c);
        rc = c->be->va_free(p, kvp.first);
      }
      c->st.va_free_calls++;
      if (rc != VT_OK) worst = rc;
      c->st.reserved_va_bytes -= kvp.first;
    }
    kvp.second.clear();
  }
  return worst;
}

}  // namespace
}  // namespace vt

using namespace vt;

extern "C" {

int vt_init(vt_ctx** out, int device, uint64_t chunk_bytes, uint64_t max_phys_bytes) {
  if (!out || device < 0) return VT_E_INVALID;
  int n = 0;
  if (hipGetDeviceCount(&n) != hipSuccess || device >= n) {
    (void)hipGetLastError();
    return VT_E_DRIVER;
  }
  if (hipSetDevice(device) != hipSuccess) return VT_E_DRIVER;
  int vmm = 0;
  if (hipDeviceGetAttribute(&vmm, hipDeviceAttributeVirtualMemoryManagementSupported, device) != hipSuccess || !vmm)
    return VT_E_UNSUPPORTED;
  int st = VT_OK;
  Backend* be = make_hip_backend(device, &st);
  if (!be) return st;
  int rc = make_ctx(out, be, device, chunk_bytes, max_phys_bytes);
  if (rc != VT_OK) return rc;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0)
    (*out)->n_cus = cus;
  if ((*out)->n_cus > kMaxPrefillGroups) (*out)->n_cus = kMaxPrefillGroups;
  void* arr = nullptr;
  if (hipMalloc(&arr, (size_t)kMaxPrefillGroups * 8) != hipSuccess ||
      hipMemset(arr, 0, (size_t)kMaxPrefillGroups * 8) != hipSuccess) {
    (void)hipGetLastError();
    if (arr) (void)hipFree(arr);
    vt_destroy(*out);
    *out = nullptr;
    return VT_E_OOM;
  }
  (*out)->arrivals = arr;
  // Address of this device's copy of the fixed scratch (the device is current).  A failure only disables
  // vt_attn_decode_static, which then reports VT_E_DRIVER.
  (void)static_scratch_init(device);
  return VT_OK;
}

int vt_init_host(vt_ctx** out, uint64_t chunk_bytes, uint64_t max_phys_bytes) {
  if (!out) return VT_E_INVALID;
  Backend* be = make_host_backend();
  if (!be) return VT_E_OOM;
  return make_ctx(out, be, -1, chunk_bytes, max_phys_bytes);
}

int vt_destroy(vt_ctx* ctx) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  int worst = VT_OK;
  {
    // queued extensions finish first; then the worker leaves
    std::unique_lock<std::mutex> lk(ctx->amu);
    ctx->astop = true;
  }
  ctx->acv_work.notify_all();
  if (ctx->aworker.joinable()) ctx->aworker.join();
  {
    std::lock_guard<std::mutex> g(ctx->mu);
    if (!ctx->be->is_host()) {
      (void)hipSetDevice(ctx->device);
      (void)hipDeviceSynchronize();  // no kernel may still read a range that is about to go
    }
    for (vt_kv* kv : ctx->regions) {
      if (kv->alive) {
        int rc = release_locked(kv);
        if (rc != VT_OK) worst = rc;
      }
    }
    int rc = trim_locked(ctx, 0);
    if (rc != VT_OK) worst = rc;
    for (vt_kv* kv : ctx->regions) {
      kv->magic = 0;
      delete kv;
    }
    ctx->regions.clear();
    for (auto& e : ctx->prof) {
      (void)hipEventDestroy((hipEvent_t)e.start);
      (void)hipEventDestroy((hipEvent_t)e.stop);
    }
    ctx->prof.clear();
    if (ctx->ws) (void)hipFree(ctx->ws);
    ctx->ws = nullptr;
    if (ctx->arrivals) (void)hipFree(ctx->arrivals);
    ctx->arrivals = nullptr;
    delete ctx->be;
    ctx->be = nullptr;
    ctx->magic = 0;
  }
  delete ctx;
  return worst;
}

int vt_reserve(vt_ctx* ctx, uint32_t n_kv_heads, uint32_t head_dim, int dtype, uint64_t max_tokens, vt_kv** out) {
  if (!ok_ctx(ctx) || !out) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(ctx->mu);
  return new_region(ctx, n_kv_heads, head_dim, dtype, max_tokens, out);
}

int vt_extend(vt_kv* kv, uint64_t new_len_tokens) {
  if (!ok_kv(kv)) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(kv->ctx->mu);
  return extend_locked(kv, new_len_tokens);
}

int vt_extend_batch(vt_kv* const* kvs, const uint64_t* new_lens, uint32_t n) {
  if (n == 0) return VT_OK;
  if (!kvs || !new_lens) return VT_E_INVALID;
  for (uint32_t i = 0; i < n; ++i)
    if (!ok_kv(kvs[i]) || kvs[i]->ctx != kvs[0]->ctx) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(kvs[0]->ctx->mu);
  for (uint32_t i = 0; i < n; ++i) {
    int rc = extend_locked(kvs[i], new_lens[i]);
    if (rc != VT_OK) return rc;
  }
  return VT_OK;
}

// Worker of the asynchronous extension: takes the queued requests in order and runs them like vt_extend_batch.
static void extend_worker(vt_ctx* c) {
  if (!c->be->is_host()) (void)hipSetDevice(c->device);
  for (;;) {
    vt::ExtendJob job;
    {
      std::unique_lock<std::mutex> lk(c->amu);
      c->acv_work.wait(lk, [&] { return c->astop || !c->ajobs.empty(); });
      if (c->ajobs.empty()) return;  // stop requested and nothing left
      job = std::move(c->ajobs.front());
      c->ajobs.pop_front();
    }
    int rc = VT_OK;
    {
      std::lock_guard<std::mutex> g(c->mu);
      for (size_t i = 0; i < job.kvs.size() && rc == VT_OK; ++i)
        rc = ok_kv(job.kvs[i]) ? extend_locked(job.kvs[i], job.lens[i]) : VT_E_INVALID;
    }
    {
      std::lock_guard<std::mutex> lk(c->amu);
      if (rc != VT_OK) c->afailed[job.ticket] = rc;
      c->adone = job.ticket;
    }
    c->acv_done.notify_all();
  }
}

int vt_extend_batch_async(vt_kv* const* kvs, const uint64_t* new_lens, uint32_t n, uint64_t* ticket) {
  if (!ticket || (n && (!kvs || !new_lens))) return VT_E_INVALID;
  if (n == 0) {
    *ticket = 0;
    return VT_OK;
  }
  for (uint32_t i = 0; i < n; ++i)
    if (!ok_kv(kvs[i]) || kvs[i]->ctx != kvs[0]->ctx) return VT_E_INVALID;
  vt_ctx* c = kvs[0]->ctx;
  vt::ExtendJob job;
  job.kvs.assign(kvs, kvs + n);
  job.lens.assign(new_lens, new_lens + n);
  {
    std::lock_guard<std::mutex> lk(c->amu);
    if (c->astop) return VT_E_INVALID;
    if (!c->aworker.joinable()) c->aworker = std::thread(extend_worker, c);
    job.ticket = c->anext++;
    *ticket = job.ticket;
    c->ajobs.push_back(std::move(job));
  }
  c->acv_work.notify_one();
  return VT_OK;
}

int vt_extend_wait(vt_ctx* ctx, uint64_t ticket) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  std::unique_lock<std::mutex> lk(ctx->amu);
  if (ticket >= ctx->anext) return VT_E_INVALID;
  ctx->acv_done.wait(lk, [&] { return ctx->adone >= ticket; });
  auto it = ctx->afailed.find(ticket);
  if (it == ctx->afailed.end()) return VT_OK;
  int rc = it->second;
  ctx->afailed.erase(it);
  return rc;
}

int vt_share_prefix(vt_kv* src, uint64_t n_tokens, uint64_t max_tokens, vt_kv** dst) {
  if (!ok_kv(src) || !dst) return VT_E_INVALID;
  vt_ctx* c = src->ctx;
  std::lock_guard<std::mutex> g(c->mu);
  if (n_tokens > src->len || n_tokens > max_tokens) return VT_E_INVALID;
  if ((n_tokens * src->row_bytes) % c->chunk_bytes != 0) return VT_E_INVALID;
  uint64_t n = n_tokens * src->row_bytes / c->chunk_bytes;
  vt_kv* kv = nullptr;
  int rc = new_region(c, src->n_kv_heads, src->head_dim, src->dtype, max_tokens, &kv);
  if (rc != VT_OK) return rc;
  uint64_t done = 0;
  for (; done < 2 * n; ++done) {
    bool is_k = done < n;
    uint64_t idx = is_k ? done : done - n;
    rc = map_one(c, (is_k ? kv->k_base : kv->v_base) + idx * c->chunk_bytes,
                 is_k ? src->k_chunks[idx] : src->v_chunks[idx]);
    if (rc != VT_OK) break;
    (is_k ? kv->k_chunks : kv->v_chunks).push_back(is_k ? src->k_chunks[idx] : src->v_chunks[idx]);
  }
  if (rc != VT_OK) {
    (void)release_locked(kv);
    return rc;
  }
  kv->len = n_tokens;
  kv->shared_chunks = n;
  *dst = kv;
  return VT_OK;
}

int vt_release(vt_kv* kv) {
  if (!ok_kv(kv)) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(kv->ctx->mu);
  return release_locked(kv);
}

int vt_trim(vt_ctx* ctx, uint64_t keep_pooled_chunks) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(ctx->mu);
  return trim_locked(ctx, keep_pooled_chunks);
}

int vt_query(const vt_kv* kv, vt_kv_info* out) {
  if (!ok_kv(kv) || !out) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(kv->ctx->mu);
  out->k_ptr = kv->k_base;
  out->v_ptr = kv->v_base;
  out->len = kv->len;
  out->max_tokens = kv->max_tokens;
  out->row_bytes = kv->row_bytes;
  out->chunk_bytes = kv->ctx->chunk_bytes;
  out->chunks_mapped = kv->k_chunks.size();
  out->capacity_bytes = kv->capacity_bytes;
  out->n_kv_heads = kv->n_kv_heads;
  out->head_dim = kv->head_dim;
  out->dtype = kv->dtype;
  out->shared_chunks = (int32_t)kv->shared_chunks;
  return VT_OK;
}

int vt_stats(const vt_ctx* ctx, vt_stats_t* out) {
  if (!ok_ctx(ctx) || !out) return VT_E_INVALID;
  std::lock_guard<std::mutex> g(const_cast<vt_ctx*>(ctx)->mu);
  *out = ctx->st;
  return VT_OK;
}

int vt_append(vt_kv* kv, const void* k_rows, const void* v_rows, uint64_t n_tokens, uint64_t at_token, void* stream) {
  if (!ok_kv(kv)) return VT_E_INVALID;
  if (n_tokens == 0) return VT_OK;
  if (!k_rows || !v_rows) return VT_E_INVALID;
  uint64_t len;
  {
    std::lock_guard<std::mutex> g(kv->ctx->mu);
    len = kv->len;
  }
  if (at_token > len || n_tokens > len - at_token) return VT_E_INVALID;
  uint64_t off = at_token * kv->row_bytes, bytes = n_tokens * kv->row_bytes;
  if (kv->ctx->be->is_host()) {
    std::memcpy(kv->k_base + off, k_rows, bytes);
    std::memcpy(kv->v_base + off, v_rows, bytes);
    return VT_OK;
  }
  // Rows are contiguous in the region, so an append is one linear copy per region.
  hipStream_t s = (hipStream_t)stream;
  if (hipMemcpyAsync(kv->k_base + off, k_rows, bytes, hipMemcpyDefault, s) != hipSuccess) return VT_E_DRIVER;
  if (hipMemcpyAsync(kv->v_base + off, v_rows, bytes, hipMemcpyDefault, s) != hipSuccess) return VT_E_DRIVER;
  return VT_OK;
}

int vt_set_plan_target(vt_ctx* ctx, uint64_t target_units) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  ctx->plan_target = target_units;
  return VT_OK;
}

int vt_host_fail_after(vt_ctx* ctx, int op, int countdown) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  return host_backend_fail_after(ctx->be, op, countdown);
}

const char* vt_strerror(int status) {
  switch (status) {
    case VT_OK: return "ok";
    case VT_E_INVALID: return "invalid argument or handle";
    case VT_E_CAPACITY: return "length exceeds the region's max_tokens";
    case VT_E_OOM: return "out of physical memory budget";
    case VT_E_DRIVER: return "HIP driver call failed";
    case VT_E_UNSUPPORTED: return "unsupported configuration";
    case VT_E_WORKSPACE: return "the call needs more scratch memory than the fixed buffer holds";
    default: return "unknown status";
  }
}

}  // extern "C"
