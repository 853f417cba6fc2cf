// Host side of the attention entry points: argument checks, the integer split plan, the workspace.
// Every arithmetic step of attention itself runs in the kernels (vt_decode.hip, vt_prefill.hip).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "vt_internal.h"

namespace vt {

constexpr uint64_t kDefaultWaveSlots = 2048;  // 256 CUs x 2 workgroups x 4 wavefronts

// Tape split.  Per KV head the requests' tokens laid end to end form a tape of total = sum_b L_b tokens.  With
// U = Hkv * ceil(G / 16) wavefronts per segment (a wavefront carries at most 16 query heads of one KV head), it is
// cut into n_seg = max(1, min(slots / U, ceil(total / 32))) segments of seg_len = round_up(ceil(total / n_seg), 32)
// tokens; one wavefront owns one (segment, kv head, 16-head sub-group).  Request b, starting at tape position T_b, is covered by
// pieces_b = (T_b + L_b - 1) / seg_len - T_b / seg_len + 1 segments.
int plan_decode(uint64_t slots, const int32_t* lens, uint32_t batch, uint32_t hkv, uint32_t hq, uint32_t d,
                DecodePlan* out, int32_t* n_splits_out) {
  if (!lens || !out || !hkv || !hq || !d || hq % hkv) return VT_E_INVALID;
  if (slots == 0) slots = kDefaultWaveSlots;
  const uint64_t units = (uint64_t)hkv * ((hq / hkv + 15) / 16);
  uint64_t total = 0;
  for (uint32_t b = 0; b < batch; ++b) {
    if (lens[b] < 1) return VT_E_INVALID;
    total += (uint64_t)lens[b];
  }
  if (total > 0x7fffffffull) return VT_E_UNSUPPORTED;
  uint64_t n_seg = std::min<uint64_t>(slots / units, (total + 31) / 32);
  if (n_seg < 1) n_seg = 1;
  uint64_t seg_len = total ? (total + n_seg - 1) / n_seg : 32;
  seg_len = (seg_len + 31) / 32 * 32;
  uint32_t mx = 0;
  uint64_t T = 0;
  for (uint32_t b = 0; b < batch; ++b) {
    const uint64_t L = (uint64_t)lens[b];
    const uint32_t pieces = (uint32_t)((T + L - 1) / seg_len - T / seg_len + 1);
    if (n_splits_out) n_splits_out[b] = (int32_t)pieces;
    mx = std::max(mx, pieces);
    T += L;
  }
  out->seg_len = (uint32_t)seg_len;
  out->n_seg = (uint32_t)n_seg;
  out->max_pieces = mx;
  out->n_units = (total + seg_len - 1) / seg_len * units;
  out->ws_bytes = decode_workspace_bytes(batch, mx, hq, d);
  return VT_OK;
}

int ensure_workspace(vt_ctx* ctx, uint64_t bytes) {
  if (bytes <= ctx->ws_bytes) return VT_OK;
  if (ctx->be->is_host()) return VT_E_UNSUPPORTED;
  uint64_t want = std::max<uint64_t>(bytes, 1ull << 20);
  want = (want + (1ull << 20) - 1) & ~((1ull << 20) - 1);
  void* p = nullptr;
  if (hipMalloc(&p, want) != hipSuccess) {
    (void)hipGetLastError();
    return VT_E_OOM;
  }
  if (ctx->ws) {
    (void)hipDeviceSynchronize();  // an earlier call may still be using the old buffer
    (void)hipFree(ctx->ws);
  }
  ctx->ws = p;
  ctx->ws_bytes = want;
  return VT_OK;
}

void prof_begin(vt_ctx* ctx, int which, void* stream) {
  if (!ctx->profile || ctx->prof.size() >= 4096) return;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return;
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    return;
  }
  ctx->prof.push_back(ProfEvent{(void*)a, (void*)b, which});
  (void)hipEventRecord(a, (hipStream_t)stream);
}

void prof_end(vt_ctx* ctx, void* stream) {
  if (!ctx->profile || ctx->prof.empty()) return;
  (void)hipEventRecord((hipEvent_t)ctx->prof.back().stop, (hipStream_t)stream);
}

static bool supported_dim(uint32_t d) { return d == 64 || d == 128; }

}  // namespace vt

using namespace vt;

extern "C" {

int vt_plan_decode(const vt_ctx* ctx, const int32_t* kv_lens_host, uint32_t batch, uint32_t n_kv_heads,
                   uint32_t n_q_heads, uint32_t head_dim, vt_plan* out, int32_t* n_splits_out) {
  if (!ok_ctx(ctx) || !out) return VT_E_INVALID;
  DecodePlan p;
  int rc = plan_decode(ctx->plan_target, kv_lens_host, batch, n_kv_heads, n_q_heads, head_dim, &p, n_splits_out);
  if (rc != VT_OK) return rc;
  out->span_tokens = p.seg_len;
  out->max_splits = p.max_pieces;
  out->n_units = p.n_units;
  out->workspace_bytes = p.ws_bytes;
  return VT_OK;
}

int vt_plan_prefill(const vt_ctx* ctx, const int32_t* cu_seqlens_host, const int32_t* prefix_lens_host, uint32_t batch,
                    uint32_t n_q_heads, uint32_t n_kv_heads, uint32_t head_dim, int new_rows_in_cache,
                    vt_prefill_plan* out, vt_prefill_piece* pieces, uint64_t max_pieces, uint64_t* n_pieces) {
  if (!ok_ctx(ctx) || !out) return VT_E_INVALID;
  if (batch && (!cu_seqlens_host || !prefix_lens_host)) return VT_E_INVALID;
  if (batch && cu_seqlens_host[0] != 0) return VT_E_INVALID;
  return plan_prefill(ctx, cu_seqlens_host, prefix_lens_host, batch, n_q_heads, n_kv_heads, head_dim,
                      new_rows_in_cache == 0, out, pieces, max_pieces, n_pieces);
}

int vt_profile_enable(vt_ctx* ctx, int on) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  ctx->profile = on != 0;
  return VT_OK;
}

int vt_profile_collect(vt_ctx* ctx, int which, double* total_ms, uint64_t* launches) {
  if (!ok_ctx(ctx) || !total_ms || !launches) return VT_E_INVALID;
  double sum = 0.0;
  uint64_t n = 0;
  std::vector<ProfEvent> keep;
  int rc = VT_OK;
  for (auto& e : ctx->prof) {
    if (e.which != which) {
      keep.push_back(e);
      continue;
    }
    float ms = 0.f;
    if (hipEventSynchronize((hipEvent_t)e.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, (hipEvent_t)e.start, (hipEvent_t)e.stop) == hipSuccess) {
      sum += ms;
      ++n;
    } else {
      (void)hipGetLastError();
      rc = VT_E_DRIVER;
    }
    (void)hipEventDestroy((hipEvent_t)e.start);
    (void)hipEventDestroy((hipEvent_t)e.stop);
  }
  ctx->prof.swap(keep);
  *total_ms = sum;
  *launches = n;
  return rc;
}

int vt_workspace_reserve(vt_ctx* ctx, uint64_t bytes) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  return ensure_workspace(ctx, bytes);
}

// Argument checks and the integer plan shared by the two decode entry points.  VT_OK with batch 0 means "nothing to do".
static int check_and_plan_decode(vt_ctx* ctx, const vt_decode_args* a, DecodePlan* plan) {
  if (!ok_ctx(ctx) || !a) return VT_E_INVALID;
  if (ctx->be->is_host()) return VT_E_UNSUPPORTED;
  if (a->batch == 0) return VT_OK;
  if (!a->q || !a->out || !a->k_ptrs || !a->v_ptrs || !a->kv_lens || !a->kv_lens_host) return VT_E_INVALID;
  if (!a->n_q_heads || !a->n_kv_heads || a->n_q_heads % a->n_kv_heads) return VT_E_INVALID;
  if (a->dtype != VT_F16 && a->dtype != VT_BF16) return VT_E_INVALID;
  if (!std::isfinite(a->scale)) return VT_E_INVALID;
  if (!supported_dim(a->head_dim) || a->n_q_heads / a->n_kv_heads > 256) return VT_E_UNSUPPORTED;
  if (a->batch > (uint32_t)kMaxDecodeBatch) return VT_E_UNSUPPORTED;
  return plan_decode(ctx->plan_target, a->kv_lens_host, a->batch, a->n_kv_heads, a->n_q_heads, a->head_dim, plan,
                     nullptr);
}

int vt_attn_decode(vt_ctx* ctx, const vt_decode_args* a, void* stream) {
  DecodePlan plan;
  int rc = check_and_plan_decode(ctx, a, &plan);
  if (rc != VT_OK || a->batch == 0) return rc;
  rc = ensure_workspace(ctx, plan.ws_bytes);
  if (rc != VT_OK) return rc;
  return launch_decode(ctx, a, plan, stream, ctx->ws, true);
}

int vt_attn_decode_static(vt_ctx* ctx, const vt_decode_args* a, void* stream) {
  DecodePlan plan;
  int rc = check_and_plan_decode(ctx, a, &plan);
  if (rc != VT_OK || a->batch == 0) return rc;
  if (plan.ws_bytes > kStaticScratchBytes) return VT_E_WORKSPACE;
  void* ws = static_scratch_ptr(ctx->device);
  if (!ws) return VT_E_DRIVER;  // the look-up at vt_init failed
  return launch_decode(ctx, a, plan, stream, ws, false);
}

uint64_t vt_static_scratch_bytes(void) { return kStaticScratchBytes; }

int vt_attn_prefix_prefill(vt_ctx* ctx, const vt_prefill_args* a, void* stream) {
  if (!ok_ctx(ctx) || !a) return VT_E_INVALID;
  if (ctx->be->is_host()) return VT_E_UNSUPPORTED;
  if (a->batch == 0 || a->total_new_tokens == 0) return VT_OK;
  if (!a->q_new || !a->out || !a->k_ptrs || !a->v_ptrs || !a->cu_seqlens || !a->prefix_lens || !a->cu_seqlens_host ||
      !a->prefix_lens_host)
    return VT_E_INVALID;
  if ((a->k_new == nullptr) != (a->v_new == nullptr)) return VT_E_INVALID;
  if (!a->n_q_heads || !a->n_kv_heads || a->n_q_heads % a->n_kv_heads) return VT_E_INVALID;
  if (a->dtype != VT_F16 && a->dtype != VT_BF16) return VT_E_INVALID;
  if (!supported_dim(a->head_dim)) return VT_E_UNSUPPORTED;
  if (!std::isfinite(a->scale)) return VT_E_INVALID;
  if (a->cu_seqlens_host[0] != 0 || (uint32_t)a->cu_seqlens_host[a->batch] != a->total_new_tokens) return VT_E_INVALID;
  for (uint32_t b = 0; b < a->batch; ++b)
    if (a->cu_seqlens_host[b + 1] < a->cu_seqlens_host[b] || a->prefix_lens_host[b] < 0) return VT_E_INVALID;
  return launch_prefill(ctx, a, stream);
}

int vt_append_batch(vt_ctx* ctx, void* const* k_ptrs, void* const* v_ptrs, const int32_t* kv_lens, const void* k_rows,
                    const void* v_rows, uint32_t batch, uint32_t n_kv_heads, uint32_t head_dim, void* stream) {
  if (!ok_ctx(ctx)) return VT_E_INVALID;
  if (ctx->be->is_host()) return VT_E_UNSUPPORTED;
  if (batch == 0) return VT_OK;
  if (!k_ptrs || !v_ptrs || !kv_lens || !k_rows || !v_rows || !n_kv_heads || !head_dim) return VT_E_INVALID;
  uint64_t row = (uint64_t)n_kv_heads * head_dim * 2;
  if (row % 16 != 0 || row > (1u << 30)) return VT_E_UNSUPPORTED;
  return launch_append_batch(k_ptrs, v_ptrs, kv_lens, k_rows, v_rows, batch, (uint32_t)row, stream);
}

}  // extern "C"
