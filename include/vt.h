/*
 * vt.h - attention over per-request, virtually contiguous KV caches on MI355X (gfx950).
 *
 * C ABI of libvt.  Method: "vTensor" (arXiv 2407.15309).  A request's K cache and V cache are each
 * ONE contiguous virtual address range sized for the maximum sequence length; physical memory is
 * attached to the range in fixed-size chunks as the sequence grows (paper, "vTensor"), so the
 * attention kernels read plain arrays and need no page-table indirection.
 *
 * Conventions shared by every entry point
 *   - Returns a vt_status: 0 on success, negative on error.  Never throws, never aborts.  A call that
 *     fails leaves all library state as it was before the call; the exceptions are the calls that work through
 *     a list of requests (vt_extend_batch, vt_extend_batch_async), which stop at the first request that fails and
 *     keep the ones before it extended, as stated there.
 *   - "device" pointers are GPU addresses valid on the context's device; "host" pointers are ordinary
 *     process memory.  The library never takes ownership of caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The attention and append
 *     calls only enqueue work on it; they do not synchronise.  Region calls (reserve / extend /
 *     release / trim) are host-synchronous driver work and never touch bytes that are already mapped.
 *   - K/V layout: request b's K region is the row-major array [len_b, n_kv_heads, head_dim] of 16-bit
 *     elements, token stride n_kv_heads*head_dim elements; V likewise, in a separate region.
 *   - Query head h uses KV head h / (n_q_heads / n_kv_heads) (grouped-query attention, paper "KV Cache
 *     Optimization: GQA and MQA"; contiguous groups).
 *   - A vt_ctx may be used from several threads; region calls are serialised by an internal lock.
 *     Two attention calls on the same context must not overlap in time (they share one workspace).
 */
#ifndef VT_H_
#define VT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vt_ctx vt_ctx; /* owns the chunk pool (pSet), the VA free-list (vSet), the split-K workspace */
typedef struct vt_kv vt_kv;   /* one request's K region + V region (one layer); owned by its vt_ctx        */

typedef enum { VT_F16 = 1, VT_BF16 = 2 } vt_dtype;

typedef enum {
  VT_OK = 0,
  VT_E_INVALID = -1,     /* bad argument, stale handle, shrink request, empty KV in decode            */
  VT_E_CAPACITY = -2,    /* length beyond the region's max_tokens                                     */
  VT_E_OOM = -3,         /* physical budget (max_phys_bytes) or device memory exhausted               */
  VT_E_DRIVER = -4,      /* a HIP call failed                                                         */
  VT_E_UNSUPPORTED = -5, /* (dtype, head_dim, group size) combination without a kernel                */
  VT_E_WORKSPACE = -6    /* vt_attn_decode_static: the call needs more than the fixed scratch buffer  */
} vt_status;

typedef struct {
  void* k_ptr;              /* device base of the K region; constant for the handle's lifetime      */
  void* v_ptr;              /* device base of the V region                                          */
  uint64_t len;             /* token rows currently backed and valid                                */
  uint64_t max_tokens;
  uint64_t row_bytes;       /* n_kv_heads * head_dim * 2                                            */
  uint64_t chunk_bytes;
  uint64_t chunks_mapped;   /* per region (K and V always hold the same count)                      */
  uint64_t capacity_bytes;  /* per region: round_up(max_tokens*row_bytes, chunk_bytes)              */
  uint32_t n_kv_heads, head_dim;
  int32_t dtype;
  int32_t shared_chunks;    /* leading chunks that alias another request's memory (prefix sharing)  */
} vt_kv_info;

typedef struct {
  uint64_t reserved_va_bytes;   /* VA currently reserved from the driver (in use + free-listed)     */
  uint64_t mapped_bytes;        /* bytes currently mapped into live regions (aliases counted once per mapping) */
  uint64_t phys_bytes;          /* physical bytes currently held (mapped + pooled chunks)           */
  uint64_t chunks_created;      /* cumulative driver allocations                                    */
  uint64_t chunks_reused;       /* cumulative chunks taken from the pool instead                    */
  uint64_t chunks_pooled;       /* chunks idle in the pool now                                      */
  uint64_t va_reserved_calls, va_reused, create_calls, map_calls, unmap_calls, release_calls, va_free_calls;
  uint64_t driver_ns;           /* cumulative host time spent inside driver calls                   */
  uint64_t live_regions;
} vt_stats_t;

/* ---- context ------------------------------------------------------------------------------- */

/* Creates a context on HIP device `device`.  chunk_bytes: physical chunk size, 0 => 2 MiB (the paper's
 * "2 MB", "vTensor"); must be a multiple of the device's minimum allocation granularity.
 * max_phys_bytes: cap on physical bytes held by the context, 0 => no cap.  Paper: "vTensor Operation",
 * Allocation, GPU interface (reserve / create / map). */
int vt_init(vt_ctx** out, int device, uint64_t chunk_bytes, uint64_t max_phys_bytes);

/* Same bookkeeping over HOST memory (mmap/memfd stand-ins for reserve/create/map), for tests of the
 * region logic on machines without a GPU.  Attention calls on such a context return VT_E_UNSUPPORTED;
 * vt_append copies with memcpy.  chunk_bytes must be a multiple of the host page size. */
int vt_init_host(vt_ctx** out, uint64_t chunk_bytes, uint64_t max_phys_bytes);

/* Unmaps and frees everything the context holds (all regions, pooled chunks, VA ranges, workspace).
 * Every vt_kv* of the context is invalid afterwards.  Paper: "vTensor Operation", Deallocation (vFree, pFree at the
 * end of serving). */
int vt_destroy(vt_ctx* ctx);

/* ---- regions (paper, "vTensor Operation" and "vTensor Scheduler") ----------------------------- */

/* vAlloc: reserves the K and V virtual ranges for one request, sized for max_tokens rows; maps nothing
 * (len = 0).  A free-listed range of the same size is reused before the driver is asked for a new one.
 * Paper: "vTensor Operation", vAlloc; "vTensor Scheduler", Create. */
int vt_reserve(vt_ctx* ctx, uint32_t n_kv_heads, uint32_t head_dim, int dtype, uint64_t max_tokens, vt_kv** out);

/* Extend: makes rows [0, new_len) backed, mapping ceil(new_len*row_bytes/chunk) chunks per region, pool
 * first, then new allocations (pAlloc + Map).  Grow-only: new_len < len => VT_E_INVALID; new_len >
 * max_tokens => VT_E_CAPACITY; over budget => VT_E_OOM with nothing changed.  Base pointers never move
 * and mapped bytes are never touched.  Paper: "vTensor Operation", pAlloc / Map; "vTensor Scheduler", Extend. */
int vt_extend(vt_kv* kv, uint64_t new_len_tokens);

/* vt_extend for n requests in one call (one lock, one ABI crossing).  Stops at the first failure and
 * returns its status; requests before it stay extended, the failing one is unchanged. */
int vt_extend_batch(vt_kv* const* kvs /*host [n]*/, const uint64_t* new_lens /*host [n]*/, uint32_t n);

/* Asynchronous extension (paper, "vTensor Scheduler", Extend: allocation runs asynchronously and overlaps
 * computation; "FlexInfer Scheduler": the scheduler dispatches the extension for coming tokens ahead of the kernels that need it).  vt_extend_batch_async queues the same work as vt_extend_batch for a worker
 * thread of the context (requests run in the order queued) and returns at once with a ticket; the arrays are
 * copied.  vt_extend_wait blocks until that ticket and all earlier ones have run and returns the ticket's status
 * (VT_OK, or the error vt_extend_batch would have returned; later requests still run).  The driver's mapping calls
 * wait for the device work queued before them, which stalls a launching thread but not this worker.  The handles
 * must stay valid until the ticket has been waited for; vt_destroy runs what is still queued. */
int vt_extend_batch_async(vt_kv* const* kvs, const uint64_t* new_lens, uint32_t n, uint64_t* ticket);
int vt_extend_wait(vt_ctx* ctx, uint64_t ticket);

/* Prefix Match by aliasing: reserves a new request whose first ceil(n_tokens*row_bytes/chunk) chunks are
 * the SAME physical chunks as `src`'s (mapped a second time, reference counted; no copy, no new
 * memory), and sets its len to n_tokens.  n_tokens*row_bytes must be a multiple of chunk_bytes unless
 * the caller never appends to `dst` (appends beyond n_tokens would otherwise write into the shared
 * last chunk): a non-aligned n_tokens returns VT_E_INVALID.  Paper: "vTensor Scheduler", Prefix Record and
 * Match; "vTensor Pool", pSet reference counts. */
int vt_share_prefix(vt_kv* src, uint64_t n_tokens, uint64_t max_tokens, vt_kv** dst);

/* Release: unmaps the request's chunks into the pool (a shared chunk returns to the pool when its last
 * mapping goes), puts the VA ranges on the free-list; no device memory is freed (lazy deallocation).
 * The handle is invalid afterwards.  Paper: "vTensor Operation", Deallocation; "vTensor Scheduler", Release. */
int vt_release(vt_kv* kv);

/* pFree / vFree: really frees pooled chunks beyond `keep_pooled_chunks` and all free-listed VA ranges.
 * Paper: "vTensor Operation", Deallocation (explicit memory-emptying). */
int vt_trim(vt_ctx* ctx, uint64_t keep_pooled_chunks);

int vt_query(const vt_kv* kv, vt_kv_info* out);
int vt_stats(const vt_ctx* ctx, vt_stats_t* out);

/* KV-cache update: copies n_tokens rows [n_tokens, n_kv_heads, head_dim] from k_rows / v_rows (device
 * memory; host memory on a host context) into rows [at_token, at_token+n_tokens) of the regions, which
 * must already be backed (at_token + n_tokens <= len).  Enqueued on `stream`.  Paper: "LLM Inference"
 * (decode updates the KV cache). */
int vt_append(vt_kv* kv, const void* k_rows, const void* v_rows, uint64_t n_tokens, uint64_t at_token, void* stream);

/* One launch that writes one new row per request: row b of k_rows / v_rows (device [batch, n_kv_heads,
 * head_dim]) goes to token position kv_lens[b]-1 of request b's regions (i.e. call after the lengths
 * were advanced).  k_ptrs / v_ptrs / kv_lens are the same device arrays vt_attn_decode takes. */
int vt_append_batch(vt_ctx* ctx, void* const* k_ptrs, void* const* v_ptrs, const int32_t* kv_lens,
                    const void* k_rows, const void* v_rows, uint32_t batch, uint32_t n_kv_heads, uint32_t head_dim,
                    void* stream);

/* ---- attention ------------------------------------------------------------------------------ */

typedef struct {
  int32_t dtype;                 /* vt_dtype of q, out and the K/V regions                            */
  uint32_t batch, n_q_heads, n_kv_heads, head_dim;
  float scale;                   /* score scale, normally 1/sqrt(head_dim)                            */
  const void* q;                 /* device [batch, n_q_heads, head_dim]                               */
  void* out;                     /* device [batch, n_q_heads, head_dim], same dtype                   */
  const void* const* k_ptrs;     /* device [batch]: K region base of each request                     */
  const void* const* v_ptrs;     /* device [batch]: V region base                                     */
  const int32_t* kv_lens;        /* device [batch]: cached rows to attend over (>= 1)                 */
  const int32_t* kv_lens_host;   /* host   [batch]: the same values, read for planning                */
} vt_decode_args;

/* Integer work decomposition of a decode call ("tape split").  Per KV head, the requests' cached tokens laid
 * end to end form a tape of total = sum_b len_b tokens, cut into segments of span_tokens tokens; one wavefront
 * owns one (segment, kv head, sub-group of at most 16 of the head's query heads; two such sub-groups of one kv head
 * when the head has more than 16 query heads).  With slots = the plan target
 * (default 2048 wavefront slots) and U = n_kv_heads * ceil((n_q_heads / n_kv_heads) / 16):
 *   n_seg       = max(1, min(slots / U, ceil(total / 32)))
 *   span_tokens = round_up(ceil(total / n_seg), 32)
 *   pieces_b    = (T_b + len_b - 1) / span_tokens - T_b / span_tokens + 1,  T_b = tokens of the requests before b
 *   max_splits  = max_b pieces_b;   n_units = ceil(total / span_tokens) * U. */
typedef struct {
  uint32_t span_tokens;
  uint32_t max_splits;
  uint64_t n_units;
  uint64_t workspace_bytes;
} vt_plan;

/* Computes the plan vt_attn_decode will use; n_splits_out (host [batch], may be NULL) receives each
 * request's piece count. */
int vt_plan_decode(const vt_ctx* ctx, const int32_t* kv_lens_host, uint32_t batch, uint32_t n_kv_heads,
                   uint32_t n_q_heads, uint32_t head_dim, vt_plan* out, int32_t* n_splits_out);

/* Batched decode attention: out[b,h,:] = sum_j softmax_j(scale * <q[b,h,:], K_b[j,g(h),:]>) V_b[j,g(h),:]
 * over j in [0, kv_lens[b]).  Online softmax with fp32 accumulation over equal tape segments, followed by a merge of the requests that were cut.
 * Paper: "LLM Inference" (decode stage), "Decoding Kernel Evaluation".  The context's workspace is grown
 * on demand (growing it synchronises the device once; steady-state calls allocate nothing).
 * Errors: VT_E_INVALID for null pointers, n_q_heads % n_kv_heads != 0 or a host length < 1;
 * a non-finite scale; VT_E_UNSUPPORTED unless head_dim is 64 or 128, n_q_heads/n_kv_heads <= 256 and
 * batch <= 4096.  Any finite scale is taken (negative, zero). */
int vt_attn_decode(vt_ctx* ctx, const vt_decode_args* args, void* stream);

/* vt_attn_decode for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same result bits as vt_attn_decode, but the
 * tape table and the pieces' partial results live in a fixed device array that is part of the loaded library
 * (vt_static_scratch_bytes() bytes, 32 MiB, held by every GPU the library runs on until the process ends) instead
 * of the context's workspace.  The call allocates and frees nothing, on the host's device heap or through any
 * library, records no events (vt_profile_enable does not cover it) and only enqueues its two kernels on `stream`.
 * A call whose plan needs more (vt_plan_decode's workspace_bytes > vt_static_scratch_bytes(); e.g. batch 256
 * with 64 query heads cut three ways fits, batch 4096 with 64 query heads does not) returns VT_E_WORKSPACE and
 * launches nothing.  Nothing in the buffer has to start at zero: the merge reads only what the split pass of the
 * same call wrote.  All calls on one GPU share the one buffer, from every context and stream: two calls that
 * overlap in time on one GPU race on it; calls on one stream, or otherwise ordered, are safe.  Other errors as
 * vt_attn_decode; VT_E_DRIVER if the buffer's address could not be looked up when the context was created. */
int vt_attn_decode_static(vt_ctx* ctx, const vt_decode_args* args, void* stream);
uint64_t vt_static_scratch_bytes(void);

typedef struct {
  int32_t dtype;
  uint32_t batch, n_q_heads, n_kv_heads, head_dim;
  float scale;
  uint32_t total_new_tokens;     /* T = cu_seqlens[batch]                                             */
  const void* q_new;             /* device [T, n_q_heads, head_dim]; request b owns rows cu[b]..cu[b+1]-1 */
  void* out;                     /* device [T, n_q_heads, head_dim]                                   */
  const void* k_new;             /* device [T, n_kv_heads, head_dim], or NULL: the new rows are already */
  const void* v_new;             /*   in the regions at [prefix_len_b, prefix_len_b + N_b)            */
  const void* const* k_ptrs;     /* device [batch]                                                    */
  const void* const* v_ptrs;     /* device [batch]                                                    */
  const int32_t* cu_seqlens;     /* device [batch+1], cu[0] = 0                                       */
  const int32_t* prefix_lens;    /* device [batch]: cached rows each request's new tokens fully see   */
  const int32_t* cu_seqlens_host;   /* host copies of the two arrays above                            */
  const int32_t* prefix_lens_host;
} vt_prefill_args;

/* Prefix-prefill attention: new token i of request b (absolute position P_b + i) attends keys
 * 0 .. P_b + i of concat(cached prefix, new tokens): the whole prefix plus the new tokens causally.
 * FlashAttention-style tiling on MFMA with fp32 accumulation.  Paper: "Prefix Cache",
 * "Prefix-prefilling Kernel Evaluation".  Errors as vt_attn_decode; head_dim must be 128 or 64, batch <= 1024.
 * With head_dim 128 the kernel runs as eight wavefronts of 32 query rows (two per SIMD); a context created while the
 * environment holds VT_PREFILL_WIDE=1 runs it as four wavefronts of 64 rows instead (the shape head_dim 64 always
 * uses) - same results up to rounding order, kept so that the two can be timed against each other. */
int vt_attn_prefix_prefill(vt_ctx* ctx, const vt_prefill_args* args, void* stream);

/* Integer work decomposition of a prefix-prefill call.  An item is (request, kv head, token tile of
 * tb = 256 / (n_q_heads / n_kv_heads) new tokens); it sweeps the key tiles (64 keys) it sees.  Cached rows and new
 * rows are tiled separately when they come from different buffers (new_rows_in_cache = 0), as one run of rows
 * otherwise.  A tile is "fast" when all its 64 keys exist and every token of the token tile sees them (in the
 * sweep the fast tiles come first).  Work is counted in cost units - 8 per item, 2 per fast tile, 3 per other
 * tile - and group w of n_groups owns units [total_cost * w / n_groups, total_cost * (w+1) / n_groups) of
 * the items laid end to end (by request, kv head, token tile); a tile belongs to the owner of its first unit.
 * n_groups = clamp(total_cost / 64, 1, compute units).  One workgroup computes one group (which workgroup of the
 * launch takes which group is the kernel's business: it hands runs of consecutive groups to the same XCD).  The
 * pieces of an item shared by several groups meet in per-piece workspace slots (two per group) and the workgroup
 * that finishes its piece last merges them and writes the item's output. */
typedef struct {
  uint64_t total_cost;
  uint64_t n_tiles;
  uint32_t n_items;
  uint32_t n_groups;
  uint64_t workspace_bytes;
} vt_prefill_plan;

/* One contiguous run of tiles [tile_begin, tile_end) of an item's sweep, computed by one workgroup. */
typedef struct {
  uint32_t group, request, kv_head, token_tile;
  uint32_t tile_begin, tile_end;  /* in sweep order                                                   */
  uint32_t n_tiles, n_fast;       /* of the whole item                                                */
} vt_prefill_piece;

/* Computes the plan vt_attn_prefix_prefill will use for these lengths (host arrays as in vt_prefill_args).
 * pieces (host, may be NULL) receives up to max_pieces pieces in execution order; *n_pieces (may be NULL) their
 * total number.  Pure host computation; works on host contexts. */
int vt_plan_prefill(const vt_ctx* ctx, const int32_t* cu_seqlens_host, const int32_t* prefix_lens_host,
                    uint32_t batch, uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim,
                    int new_rows_in_cache, vt_prefill_plan* out, vt_prefill_piece* pieces, uint64_t max_pieces,
                    uint64_t* n_pieces);

/* Pre-sizes the context's workspace so that later attention calls never allocate. */
int vt_workspace_reserve(vt_ctx* ctx, uint64_t bytes);

/* ---- misc ------------------------------------------------------------------------------------ */

/* Kernel timing for benchmarks.  While enabled, vt_attn_decode brackets its split-pass kernel (which = 0)
 * and vt_attn_prefix_prefill its kernel (which = 1) with HIP events recorded on the caller's stream.
 * vt_profile_collect waits for the events recorded so far, returns their summed elapsed time and count
 * for `which`, and forgets them.  At most 4096 launches are kept between two collects. */
int vt_profile_enable(vt_ctx* ctx, int on);
int vt_profile_collect(vt_ctx* ctx, int which, double* total_ms, uint64_t* launches);

const char* vt_strerror(int status);

/* Tuning knob read by vt_plan_decode / vt_attn_decode: number of wavefront slots the tape is split for
 * (0 => default 2048 = 256 CUs x 8 resident wavefronts). */
int vt_set_plan_target(vt_ctx* ctx, uint64_t target_units);

/* Test hook (host contexts only): the `countdown`-th next driver stand-in call of kind `op`
 * (0 reserve, 1 create, 2 map, 3 unmap) fails once. */
int vt_host_fail_after(vt_ctx* ctx, int op, int countdown);

#ifdef __cplusplus
}
#endif
#endif /* VT_H_ */
