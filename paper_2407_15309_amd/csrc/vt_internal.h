// Internal declarations shared by the translation units of libvt.  Not part of the ABI.
#pragma once

#include <condition_variable>
#include <cstdint>
#include <deque>
#include <map>
#include <mutex>
#include <thread>
#include <vector>

#include "vt.h"

namespace vt {

// Driver-facing operations of the region manager.  Two implementations: HIP virtual memory management
// on a device, and host memory (mmap + memfd) for tests of the bookkeeping without a GPU.
struct Backend {
  virtual ~Backend() {}
  virtual int reserve(uint64_t size, uint64_t align, void** out) = 0;  // VA only
  virtual int va_free(void* addr, uint64_t size) = 0;
  virtual int create(uint64_t size, void** handle) = 0;                // one physical chunk
  virtual int release(void* handle) = 0;
  virtual int map(void* addr, uint64_t size, void* handle) = 0;        // also enables access
  virtual int unmap(void* addr, uint64_t size) = 0;
  virtual uint64_t granularity() const = 0;
  virtual bool is_host() const = 0;
};

Backend* make_hip_backend(int device, int* status);
Backend* make_host_backend();
int host_backend_fail_after(Backend* b, int op, int countdown);

struct Chunk {
  void* handle;
  int refs;  // number of live mappings
};

struct ProfEvent {
  void* start;  // hipEvent_t
  void* stop;
  int which;
};

// One queued vt_extend_batch_async request.
struct ExtendJob {
  uint64_t ticket;
  std::vector<vt_kv*> kvs;
  std::vector<uint64_t> lens;
};

}  // namespace vt

struct vt_kv {
  uint32_t magic;
  bool alive;
  vt_ctx* ctx;
  uint32_t n_kv_heads, head_dim;
  int32_t dtype;
  uint64_t row_bytes, max_tokens, capacity_bytes, len;
  char* k_base;
  char* v_base;
  uint64_t shared_chunks;
  std::vector<vt::Chunk*> k_chunks, v_chunks;
};

struct vt_ctx {
  uint32_t magic;
  int device;  // -1 on a host context
  vt::Backend* be;
  uint64_t chunk_bytes, max_phys_bytes;
  uint64_t plan_target;
  std::mutex mu;
  std::vector<vt::Chunk*> pool;                          // pSet: idle chunks
  std::map<uint64_t, std::vector<char*>> va_free;        // vSet: idle ranges by size
  std::vector<vt_kv*> regions;                           // every handle ever issued (freed at destroy)
  vt_stats_t st;
  void* ws;
  uint64_t ws_bytes;
  void* arrivals;             // device, kMaxPrefillGroups 8-byte words, zero at creation: arrival counts of the
                              // prefix-prefill items shared between workgroups, tagged with the launch number
  uint64_t prefill_launches;  // prefix-prefill launches on this context so far
  bool prefill_wide;          // VT_PREFILL_WIDE=1 when the context was created: head_dim 128 runs the 4-wavefront kernel
  int n_cus;
  bool profile;
  std::vector<vt::ProfEvent> prof;
  // Asynchronous extension (a worker thread that runs queued extensions in order, started on first use).
  std::mutex amu;
  std::condition_variable acv_work, acv_done;
  std::deque<vt::ExtendJob> ajobs;
  std::map<uint64_t, int> afailed;   // status of the tickets that failed
  uint64_t anext = 1, adone = 0;     // next ticket to hand out, last ticket finished
  bool astop = false;
  std::thread aworker;
};

constexpr uint32_t VT_CTX_MAGIC = 0x76544358u;
constexpr uint32_t VT_KV_MAGIC = 0x76544b56u;

namespace vt {

inline bool ok_ctx(const vt_ctx* c) { return c && c->magic == VT_CTX_MAGIC; }
inline bool ok_kv(const vt_kv* k) { return k && k->magic == VT_KV_MAGIC && k->alive && ok_ctx(k->ctx); }

constexpr int kMaxPrefillGroups = 1024;  // workgroups of a prefix-prefill launch (one per compute unit at most)
constexpr int kMaxPrefillBatch = 1024;  // requests per prefix-prefill launch (the item order lives in LDS)
constexpr int kMaxDecodeBatch = 4096;  // requests per decode launch (the tape prefix table lives in LDS)

// Integer plan of a decode call (see vt_plan in vt.h).
struct DecodePlan {
  uint32_t seg_len, n_seg, max_pieces;
  uint64_t n_units, ws_bytes;
};
int plan_decode(uint64_t target, const int32_t* lens, uint32_t batch, uint32_t hkv, uint32_t hq, uint32_t d,
                DecodePlan* out, int32_t* n_splits_out);

// Bytes of device workspace a decode launch needs: the tape prefix sums and the partial results.
uint64_t decode_workspace_bytes(uint32_t batch, uint32_t max_pieces, uint32_t hq, uint32_t d);

// Fixed scratch of the entry point that allocates nothing (the array lives in vt_decode.hip).  static_scratch_init
// looks up the current device's copy once (call with `device` current); static_scratch_ptr returns it, null if the
// look-up has not run or failed.
constexpr uint64_t kStaticScratchBytes = 32ull << 20;
int static_scratch_init(int device);
void* static_scratch_ptr(int device);

// Grows the context's device workspace to at least `bytes`.
int ensure_workspace(vt_ctx* ctx, uint64_t bytes);

// Event bracket around a kernel launch while profiling is enabled (no-ops otherwise).
void prof_begin(vt_ctx* ctx, int which, void* stream);
void prof_end(vt_ctx* ctx, void* stream);

// Kernel launchers (device code lives in the .hip files).
// `workspace`: device memory of at least plan.ws_bytes bytes.
int launch_decode(vt_ctx* ctx, const vt_decode_args* a, const DecodePlan& plan, void* stream, void* workspace,
                  bool allow_profile);
int launch_prefill(vt_ctx* ctx, const vt_prefill_args* a, void* stream);
int plan_prefill(const vt_ctx* ctx, const int32_t* cu_host, const int32_t* plens_host, uint32_t batch, uint32_t hq,
                 uint32_t hkv, uint32_t d, bool split, vt_prefill_plan* out, vt_prefill_piece* pieces,
                 uint64_t max_pieces, uint64_t* n_pieces);
int launch_append_batch(void* const* k_ptrs, void* const* v_ptrs, const int32_t* kv_lens, const void* k_rows,
                        const void* v_rows, uint32_t batch, uint32_t row_bytes, void* stream);

}  // namespace vt
