// Batched decode attention over per-request contiguous K/V regions (gfx950).
//
// What is computed (paper Section 2.1, decode stage; Section 2.2.3 for grouped heads): for request b and
// query head h, out = sum_j softmax_j(scale <q, k_j>) v_j over the request's cached rows, K/V row j of
// KV head g living at base_b + (j*Hkv + g)*D.  Because a request's cache is one contiguous virtual
// range (paper Section 4.1) the kernel addresses rows by plain pointer arithmetic.
//
// Work decomposition: one wavefront per (request, kv head, span of `span` tokens); a workgroup holds
// the wavefronts of up to 4 adjacent kv heads of the same span so that concurrently issued loads
// cover adjacent 256 B pieces of the same token rows.  Each wavefront streams its span in tiles of 32
// tokens and keeps an online-softmax state (running max m, running sum l, fp32 accumulator) for all
// query heads of its group at once, so every K/V byte is read from HBM once per KV head.
//
// Matrix-core mapping (v_mfma_f32_16x16x32, one wavefront):
//   S^T[token, head]  = K_tile[16 tokens x D] * Q^T[D x 16 heads]      (A = K rows, B = Q, heads padded to 16)
//   O^T[d, head]     += V_tile^T[d x 32 tokens] * P^T[32 tokens x heads] (A = V^T, B = P)
// The result layout of the first product (lane holds one head column and four token rows per 16-token
// block) is exactly the B-operand layout of the second once the 32 tokens of a tile are assigned to the
// contraction slots in the order each lane already holds them, so P never moves between lanes.  V^T is
// produced without shared memory: a lane loads the same 16-byte column chunk of the 8 token rows of its
// contraction slots and transposes the 8x8 block of 16-bit values inside its own registers.  K goes
// through a wavefront-private LDS staging buffer so that the global loads stay fully coalesced
// (16 lanes x 16 B = one 256 B row piece) while the MFMA operand wants 16 different rows per 16 lanes.
//
// A second small kernel merges the per-span partial results with the usual log-sum-exp rule.
#include <hip/hip_runtime.h>

#include <cmath>

#include "vt_internal.h"

namespace vt {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

constexpr int kTile = 32;  // tokens per tile

template <int DT>
struct Elem;
template <>
struct Elem<VT_BF16> {
  static __device__ __forceinline__ f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  }
  static __device__ __forceinline__ u32x4 pack8(const float* p) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (__bf16)p[e];
    return __builtin_bit_cast(u32x4, v);
  }
  static __device__ __forceinline__ unsigned short cvt(float x) {
    __bf16 h = (__bf16)x;
    return __builtin_bit_cast(unsigned short, h);
  }
};
template <>
struct Elem<VT_F16> {
  static __device__ __forceinline__ f32x4 mfma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  }
  static __device__ __forceinline__ u32x4 pack8(const float* p) {
    f16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (_Float16)p[e];
    return __builtin_bit_cast(u32x4, v);
  }
  static __device__ __forceinline__ unsigned short cvt(float x) {
    _Float16 h = (_Float16)x;
    return __builtin_bit_cast(unsigned short, h);
  }
};

struct DecodeParams {
  const char* q;
  const char* const* k_ptrs;
  const char* const* v_ptrs;
  const int32_t* kv_lens;
  float* part_acc;  // [B][max_splits][Hq][D]
  float* part_m;    // [B][max_splits][Hq], running max of scale*log2(e)*score
  float* part_l;    // [B][max_splits][Hq]
  void* out;        // [B][Hq][D]
  uint32_t hq, hkv, group, span, max_splits;
  float scale_log2e;
};

// 8x8 transpose of 16-bit values held as 8 registers-of-8 (rows = tokens, columns = d) inside one lane.
// out[dd] holds column dd of the block: the 8 tokens' values of d = dd, in token-slot order.
__device__ __forceinline__ void transpose8x8(const u32x4* v, u32x4* out) {
#pragma unroll
  for (int dd = 0; dd < 8; ++dd) {
    const unsigned sel = (dd & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
    for (int w = 0; w < 4; ++w) out[dd][w] = __builtin_amdgcn_perm(v[2 * w + 1][dd >> 1], v[2 * w][dd >> 1], sel);
  }
}

template <int D>
struct Tile {
  static constexpr int CH = D / 8;         // 16-byte chunks per K/V head row
  static constexpr int TPL = 64 / CH;      // token rows covered by one wavefront-wide K load
  static constexpr int NLK = kTile / TPL;  // K loads per tile
  u32x4 k[NLK];
  u32x4 v[8];
};

template <int DT, int D, int W>
__global__ __launch_bounds__(64 * W) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_split_kernel(DecodeParams p) {
  using T = Tile<D>;
  constexpr int CH = T::CH, TPL = T::TPL, NLK = T::NLK;
  constexpr int KK = D / 32;             // MFMA k-steps of the score product
  constexpr int NM = D / 16;             // MFMAs (16 d-rows each) of the value product
  constexpr int RSB = D * 2 + 16;        // LDS row stride in bytes (16 B pad: conflict-free operand reads)
  __shared__ __attribute__((aligned(16))) char lds_all[W][kTile * RSB];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t g = blockIdx.x * W + wave, s = blockIdx.y, b = blockIdx.z;
  if (g >= p.hkv) return;
  const int L = p.kv_lens[b];
  const int t0 = (int)(s * p.span);
  if (t0 >= L) return;
  const int t1 = min(t0 + (int)p.span, L);
  char* lds = lds_all[wave];

  const int c16 = lane & 15, j = lane >> 4;
  const int cK = lane % CH, jK = lane / CH;
  const uint32_t row_bytes = p.hkv * D * 2;
  const char* kb = p.k_ptrs[b] + (size_t)g * D * 2 + cK * 16;
  const char* vb = p.v_ptrs[b] + (size_t)g * D * 2 + (c16 % CH) * 16;

  // Q as the B operand: lane (head c16, slot j) holds d-chunk 4*kk + j of its head; heads >= group are zero.
  u32x4 qf[KK];
  {
    const char* qh = p.q + ((size_t)b * p.hq + (size_t)g * p.group + c16) * D * 2;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      u32x4 z = {0u, 0u, 0u, 0u};
      qf[kk] = (c16 < (int)p.group) ? *(const u32x4*)(qh + (4 * kk + j) * 16) : z;
    }
  }

  f32x4 acc[NM];
#pragma unroll
  for (int m = 0; m < NM; ++m) acc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;

  auto load_tile = [&](T& t, int tile) {
    const int last = t1 - 1;
#pragma unroll
    for (int i = 0; i < NLK; ++i) {
      int tok = min(tile + i * TPL + jK, last);
      t.k[i] = *(const u32x4*)(kb + (size_t)tok * row_bytes);
    }
#pragma unroll
    for (int i8 = 0; i8 < 8; ++i8) {
      int tok = min(tile + (i8 & 3) + 4 * j + (i8 >> 2) * 16, last);
      t.v[i8] = *(const u32x4*)(vb + (size_t)tok * row_bytes);
    }
  };

  auto compute_tile = [&](const T& t, int tile) {
    // K tile -> LDS (coalesced layout) -> MFMA A-operand layout.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NLK; ++i) *(u32x4*)(lds + (i * TPL + jK) * RSB + cK * 16) = t.k[i];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    f32x4 sc[2];
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      sc[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        u32x4 kf = *(const u32x4*)(lds + (16 * hh + c16) * RSB + (4 * kk + j) * 16);
        sc[hh] = Elem<DT>::mfma(kf, qf[kk], sc[hh]);
      }
    }
    // Online softmax for head c16 over this lane's 8 tokens (4*j+i and 16+4*j+i) and, via two
    // cross-lane exchanges, over all 32 tokens of the tile.
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      int tok = tile + (e & 3) + 4 * j + (e >> 2) * 16;
      float v = sc[e >> 2][e & 3] * p.scale_log2e;
      x[e] = tok < t1 ? v : -INFINITY;
    }
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float pr[8], psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pr[e] = __builtin_amdgcn_exp2f(x[e] - m_new);
      psum += pr[e];
    }
    l_run = l_run * alpha + psum;
    const u32x4 pf = Elem<DT>::pack8(pr);
    // V^T operand by in-lane transpose, then O^T += V^T P^T.
    u32x4 vt[8];
    transpose8x8(t.v, vt);
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      u32x4 a;
      if constexpr (D == 128) {
        a = vt[m];
      } else {
        // D = 64: lanes c16 and c16+8 hold the same chunk; rows 0-7 take even columns, rows 8-15 odd ones.
#pragma unroll
        for (int w = 0; w < 4; ++w) a[w] = (c16 < 8) ? vt[2 * m][w] : vt[2 * m + 1][w];
      }
      acc[m] *= alpha;
      acc[m] = Elem<DT>::mfma(a, pf, acc[m]);
    }
  };

  T ta, tb;
  int tile = t0;
  load_tile(ta, tile);
  for (;;) {
    if (tile + kTile < t1) load_tile(tb, tile + kTile);
    compute_tile(ta, tile);
    tile += kTile;
    if (tile >= t1) break;
    if (tile + kTile < t1) load_tile(ta, tile + kTile);
    compute_tile(tb, tile);
    tile += kTile;
    if (tile >= t1) break;
  }

  // Partial result of this span: (m, l, acc) per head.
  l_run += __shfl_xor(l_run, 16);
  l_run += __shfl_xor(l_run, 32);
  if (c16 < (int)p.group) {
    const size_t pidx = ((size_t)b * p.max_splits + s) * p.hq + (size_t)g * p.group + c16;
    float* pa = p.part_acc + pidx * D;
    if constexpr (D == 128) {
      // acc[m][i] is d = 32*j + 8*i + m
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 lo = {acc[0][i], acc[1][i], acc[2][i], acc[3][i]};
        f32x4 hi = {acc[4][i], acc[5][i], acc[6][i], acc[7][i]};
        *(f32x4*)(pa + 32 * j + 8 * i) = lo;
        *(f32x4*)(pa + 32 * j + 8 * i + 4) = hi;
      }
    } else {
      // acc[m][i] is row r = 4*j + i of MFMA m: d = 8*(r % 8) + 2*m + r / 8
#pragma unroll
      for (int m = 0; m < NM; ++m)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          int r = 4 * j + i;
          pa[8 * (r & 7) + 2 * m + (r >> 3)] = acc[m][i];
        }
    }
    if (j == 0) {
      p.part_m[pidx] = m_run;
      p.part_l[pidx] = l_run;
    }
  }
}

// Merge of the per-span partials: M = max_s m_s; out = sum_s acc_s 2^(m_s-M) / sum_s l_s 2^(m_s-M).
template <int DT, int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeParams p) {
  const uint32_t h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
  const int L = p.kv_lens[b];
  const int n = min((L + (int)p.span - 1) / (int)p.span, (int)p.max_splits);
  const size_t base = (size_t)b * p.max_splits * p.hq + h;
  float M = -INFINITY;
  for (int s = 0; s < n; ++s) M = fmaxf(M, p.part_m[base + (size_t)s * p.hq]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < n; ++s) {
    const size_t idx = base + (size_t)s * p.hq;
    const float w = __builtin_amdgcn_exp2f(p.part_m[idx] - M);
    num += w * p.part_acc[idx * D + d];
    den += w * p.part_l[idx];
  }
  ((unsigned short*)p.out)[((size_t)b * p.hq + h) * D + d] = Elem<DT>::cvt(num / den);
}

__global__ void append_batch_kernel(char* const* k_ptrs, char* const* v_ptrs, const int32_t* kv_lens, const char* k_rows,
                                    const char* v_rows, uint32_t row_bytes) {
  const uint32_t b = blockIdx.x;
  const size_t dst = (size_t)(kv_lens[b] - 1) * row_bytes;
  const bool is_v = blockIdx.y != 0;
  char* base = (is_v ? v_ptrs[b] : k_ptrs[b]) + dst;
  const char* src = (is_v ? v_rows : k_rows) + (size_t)b * row_bytes;
  for (uint32_t off = threadIdx.x * 16; off < row_bytes; off += blockDim.x * 16)
    *(u32x4*)(base + off) = *(const u32x4*)(src + off);
}

template <int DT, int D>
int launch_decode_t(vt_ctx* ctx, const DecodeParams& p, uint32_t batch, hipStream_t st) {
  const uint32_t W = p.hkv % 4 == 0 ? 4 : (p.hkv % 2 == 0 ? 2 : 1);
  dim3 grid(p.hkv / W, p.max_splits, batch);
  prof_begin(ctx, 0, st);
  if (W == 4)
    hipLaunchKernelGGL((decode_split_kernel<DT, D, 4>), grid, dim3(256), 0, st, p);
  else if (W == 2)
    hipLaunchKernelGGL((decode_split_kernel<DT, D, 2>), grid, dim3(128), 0, st, p);
  else
    hipLaunchKernelGGL((decode_split_kernel<DT, D, 1>), grid, dim3(64), 0, st, p);
  prof_end(ctx, st);
  if (hipGetLastError() != hipSuccess) return VT_E_DRIVER;
  hipLaunchKernelGGL((decode_combine_kernel<DT, D>), dim3(p.hq, batch), dim3(D), 0, st, p);
  return hipGetLastError() == hipSuccess ? VT_OK : VT_E_DRIVER;
}

}  // namespace

int launch_decode(vt_ctx* ctx, const vt_decode_args* a, const DecodePlan& plan, void* stream) {
  DecodeParams p;
  p.q = (const char*)a->q;
  p.k_ptrs = (const char* const*)a->k_ptrs;
  p.v_ptrs = (const char* const*)a->v_ptrs;
  p.kv_lens = a->kv_lens;
  const size_t n_part = (size_t)a->batch * plan.max_splits * a->n_q_heads;
  p.part_acc = (float*)ctx->ws;
  p.part_m = p.part_acc + n_part * a->head_dim;
  p.part_l = p.part_m + n_part;
  p.out = a->out;
  p.hq = a->n_q_heads;
  p.hkv = a->n_kv_heads;
  p.group = a->n_q_heads / a->n_kv_heads;
  p.span = plan.span;
  p.max_splits = plan.max_splits;
  p.scale_log2e = a->scale * 1.4426950408889634f;
  hipStream_t st = (hipStream_t)stream;
  if (a->dtype == VT_BF16) {
    if (a->head_dim == 128) return launch_decode_t<VT_BF16, 128>(ctx, p, a->batch, st);
    if (a->head_dim == 64) return launch_decode_t<VT_BF16, 64>(ctx, p, a->batch, st);
  } else {
    if (a->head_dim == 128) return launch_decode_t<VT_F16, 128>(ctx, p, a->batch, st);
    if (a->head_dim == 64) return launch_decode_t<VT_F16, 64>(ctx, p, a->batch, st);
  }
  return VT_E_UNSUPPORTED;
}

int launch_append_batch(void* const* k_ptrs, void* const* v_ptrs, const int32_t* kv_lens, const void* k_rows,
                        const void* v_rows, uint32_t batch, uint32_t row_bytes, void* stream) {
  hipLaunchKernelGGL(append_batch_kernel, dim3(batch, 2), dim3(256), 0, (hipStream_t)stream, (char* const*)k_ptrs,
                     (char* const*)v_ptrs, kv_lens, (const char*)k_rows, (const char*)v_rows, row_bytes);
  return hipGetLastError() == hipSuccess ? VT_OK : VT_E_DRIVER;
}

}  // namespace vt
