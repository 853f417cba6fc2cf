// Prefix-prefill attention over per-request contiguous K/V regions (gfx950, MFMA).
//
// What is computed (paper Section 2.2.2, prefix cache; Section 6.2.2, prefix-prefilling kernel): new
// token i of request b sits at absolute position P_b + i and attends keys 0 .. P_b + i of
// concat(cached prefix rows, the new tokens' rows): the whole prefix without a mask, the new tokens
// causally.  Prefix rows are read straight from the request's virtually contiguous region (paper
// Section 4.1); the new tokens' rows come from k_new / v_new, or from the region itself when the caller
// has already appended them.
//
// Tiling: a workgroup of 4 wavefronts owns 256 query rows of one (request, kv head): the G query heads of
// the group for 256/G consecutive new tokens, so one K/V tile read serves every head of the group.  It
// sweeps the visible keys in tiles of 64.  Per tile, with v_mfma_f32_32x32x16:
//   S^T[key, row]  = K_tile[64 x D] * Q^T[D x 64 rows per wavefront]     (A = K from LDS, B = Q in registers)
//   O^T[d, row]   += V_tile^T[D x 64 keys] * P^T[64 keys x rows]         (A = V^T from LDS, B = P in registers)
// Keys run along the rows of S^T, so a softmax reduction over keys is 16 in-lane values plus one
// cross-lane exchange, and the result registers of the first product are, value for value, the B operand
// of the second once V^T is stored in LDS with its keys permuted into the order the lanes hold them.
// V is transposed once per tile by the whole workgroup on its way into LDS (registers, v_perm), not per
// wavefront.  The running maximum is only refreshed when a tile exceeds it by more than 2^8, which keeps
// the accumulator rescale off the common path; the final division by the running sum makes the result
// independent of which reference maximum was used.
#include <hip/hip_runtime.h>

#include <cmath>

#include "vt_internal.h"

namespace vt {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

constexpr int kBN = 64;          // keys per tile
constexpr int kRows = 256;       // query rows per workgroup (4 wavefronts x 64)
constexpr float kTau = 8.0f;     // lazy-rescale threshold in log2 units

template <int DT>
struct PElem;
template <>
struct PElem<VT_BF16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
  }
  static __device__ __forceinline__ u32x4 pack8(const float* p) {
    bf16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (__bf16)p[e];
    return __builtin_bit_cast(u32x4, v);
  }
  static __device__ __forceinline__ unsigned pack2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    bf16x2 v = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(unsigned, v);
  }
};
template <>
struct PElem<VT_F16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0,
                                                  0);
  }
  static __device__ __forceinline__ u32x4 pack8(const float* p) {
    f16x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (_Float16)p[e];
    return __builtin_bit_cast(u32x4, v);
  }
  static __device__ __forceinline__ unsigned pack2(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    f16x2 v = {(_Float16)a, (_Float16)b};
    return __builtin_bit_cast(unsigned, v);
  }
};

struct PrefillParams {
  const char* q;
  char* out;
  const char* k_new;  // may be null: new rows live in the regions
  const char* v_new;
  const char* const* k_ptrs;
  const char* const* v_ptrs;
  const int32_t* cu;
  const int32_t* plens;
  uint32_t batch, hq, hkv, group, tb;  // tb = new tokens per workgroup = 256 / group
  float scale_log2e;
};

template <int DT, int D>
__global__ __launch_bounds__(256) void prefill_kernel(PrefillParams p) {
  constexpr int CH = D / 8;            // 16-byte chunks per head row
  constexpr int KS = D / 16;           // k-steps of the score product
  constexpr int DB = D / 32;           // 32-row d blocks of the value product
  constexpr int RSK = D * 2 + 16;      // LDS row stride of the K tile [key][d]
  constexpr int RSV = kBN * 2 + 16;    // LDS row stride of the V^T tile [d][key slot]
  constexpr int KPASS = kBN * CH / 256;  // 16-byte K pieces per thread and tile
  constexpr int VITEMS = (kBN / 4) * CH; // (4 keys x 8 d) blocks of a V tile
  constexpr int VPASS = (VITEMS + 255) / 256;
  __shared__ __attribute__((aligned(16))) char lds_k[kBN * RSK];
  __shared__ __attribute__((aligned(16))) char lds_v[D * RSV];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, hi = lane >> 5;
  const int G = (int)p.group, tb = (int)p.tb;

  // Which (request, token tile) is this workgroup?  grid.x enumerates the tiles of all requests in order.
  int rem = blockIdx.x, b = 0, N = 0;
  for (;; ++b) {
    if (b >= (int)p.batch) return;
    N = p.cu[b + 1] - p.cu[b];
    const int nt = (N + tb - 1) / tb;
    if (rem < nt) break;
    rem -= nt;
  }
  const int g = blockIdx.y;
  const int cu_b = p.cu[b], P = p.plens[b];
  const int tok0 = rem * tb;
  const int ntok = min(tb, N - tok0);
  const int total_keys = P + tok0 + ntok;      // keys the last token of the tile sees
  const int nkt = (total_keys + kBN - 1) / kBN;
  const uint32_t row_bytes = p.hkv * D * 2;
  const char* kc = p.k_ptrs[b] + (size_t)g * D * 2;
  const char* vc = p.v_ptrs[b] + (size_t)g * D * 2;
  const bool split_src = p.k_new != nullptr;
  const char* kn = split_src ? p.k_new + (size_t)g * D * 2 : kc;
  const char* vn = split_src ? p.v_new + (size_t)g * D * 2 : vc;
  const int new_row0 = split_src ? cu_b - P : 0;   // key j >= P lives at row j + new_row0 of kn / vn

  // Query rows of this lane (one per 32-column block) and their causal limits.
  int lim[2], q_tok[2], q_head[2];
  bool q_valid[2];
  u32x4 qf[2][KS];
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const int r = wave * 64 + cb * 32 + col;
    const int t = r / G;
    q_head[cb] = r - t * G;
    q_valid[cb] = t < ntok;
    q_tok[cb] = min(t, ntok - 1);
    lim[cb] = P + tok0 + q_tok[cb];            // key j is visible iff j <= lim
    const char* qp = p.q + ((size_t)(cu_b + tok0 + q_tok[cb]) * p.hq + (size_t)g * G + q_head[cb]) * D * 2;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[cb][ks] = *(const u32x4*)(qp + (16 * ks + 8 * hi) * 2);
  }

  f32x16 acc[DB][2];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[db][cb][i] = 0.f;
  float m_used[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};

  // Staging registers: this thread's share of one K tile and one V tile.
  u32x4 kst[KPASS], vst[VPASS][4];
  const int last_key = total_keys - 1;
  auto key_ptr = [&](const char* cache, const char* fresh, int j) -> const char* {
    j = min(j, last_key);
    return j < P ? cache + (size_t)j * row_bytes : fresh + (size_t)(j + new_row0) * row_bytes;
  };
  auto load_tile = [&](int kt) {
    const int j0 = kt * kBN;
#pragma unroll
    for (int i = 0; i < KPASS; ++i) {
      const int it = tid + i * 256;
      kst[i] = *(const u32x4*)(key_ptr(kc, kn, j0 + it / CH) + (it % CH) * 16);
    }
#pragma unroll
    for (int i = 0; i < VPASS; ++i) {
      const int it = tid + i * 256;
      if (VITEMS % 256 == 0 || it < VITEMS) {
        const int kg = it / CH, c = it % CH;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) vst[i][kk] = *(const u32x4*)(key_ptr(vc, vn, j0 + 4 * kg + kk) + c * 16);
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < KPASS; ++i) {
      const int it = tid + i * 256;
      *(u32x4*)(lds_k + (it / CH) * RSK + (it % CH) * 16) = kst[i];
    }
#pragma unroll
    for (int i = 0; i < VPASS; ++i) {
      const int it = tid + i * 256;
      if (VITEMS % 256 == 0 || it < VITEMS) {
        const int kg = it / CH, c = it % CH;
        // keys 4kg..4kg+3 of the tile: block kg/8 of 32 keys; inside it key = 16*s + 8*x + 4*h + y sits at
        // slot 16*s + 8*h + 4*x + y, the order in which a lane of the score product holds its keys.
        const int k8 = kg & 7;
        const int pos = 32 * (kg >> 3) + 16 * (k8 >> 2) + 8 * (k8 & 1) + 4 * ((k8 >> 1) & 1);
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
          const unsigned sel = (dd & 1) ? 0x07060302u : 0x05040100u;
          u32x2 w;
          w[0] = __builtin_amdgcn_perm(vst[i][1][dd >> 1], vst[i][0][dd >> 1], sel);
          w[1] = __builtin_amdgcn_perm(vst[i][3][dd >> 1], vst[i][2][dd >> 1], sel);
          *(u32x2*)(lds_v + (8 * c + dd) * RSV + pos * 2) = w;
        }
      }
    }
  };

  load_tile(0);
  for (int kt = 0; kt < nkt; ++kt) {
    __syncthreads();
    store_tile();
    __syncthreads();
    if (kt + 1 < nkt) load_tile(kt + 1);
    const int j0 = kt * kBN;
    const bool need_mask = j0 + kBN - 1 > P + tok0;   // some (row, key) pair of this tile may be hidden

#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s[2];
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[cb][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const u32x4 kf = *(const u32x4*)(lds_k + (32 * kb + col) * RSK + (16 * ks + 8 * hi) * 2);
        s[0] = PElem<DT>::mfma(kf, qf[0][ks], s[0]);
        s[1] = PElem<DT>::mfma(kf, qf[1][ks], s[1]);
      }
      u32x4 pf[2][2];
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) {
        float x[16];
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          x[i] = s[cb][i] * p.scale_log2e;
          if (need_mask) {
            const int j = j0 + 32 * kb + 8 * (i >> 2) + 4 * hi + (i & 3);
            x[i] = j <= lim[cb] ? x[i] : -INFINITY;
          }
          tmax = fmaxf(tmax, x[i]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const bool grow = tmax > m_used[cb] + kTau;
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
          const float m_new = grow ? tmax : m_used[cb];
          const float alpha = __builtin_amdgcn_exp2f(m_used[cb] - m_new);
          m_used[cb] = m_new;
          l_run[cb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db) acc[db][cb] *= alpha;
        }
        float pr[16], psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          pr[i] = __builtin_amdgcn_exp2f(x[i] - m_used[cb]);
          psum += pr[i];
        }
        l_run[cb] += psum;
        pf[cb][0] = PElem<DT>::pack8(pr);
        pf[cb][1] = PElem<DT>::pack8(pr + 8);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const u32x4 vf = *(const u32x4*)(lds_v + (32 * db + col) * RSV + (32 * kb + 16 * s2 + 8 * hi) * 2);
          acc[db][0] = PElem<DT>::mfma(vf, pf[0][s2], acc[db][0]);
          acc[db][1] = PElem<DT>::mfma(vf, pf[1][s2], acc[db][1]);
        }
    }
  }

  // out[row, d] = acc / l.  acc[db][cb][i] is d = 32*db + 8*(i/4) + 4*hi + i%4 of the lane's query row.
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const float l_tot = l_run[cb] + __shfl_xor(l_run[cb], 32);
    if (!q_valid[cb]) continue;
    const float inv = 1.0f / l_tot;
    char* op = p.out + ((size_t)(cu_b + tok0 + q_tok[cb]) * p.hq + (size_t)g * G + q_head[cb]) * D * 2;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w;
        w[0] = PElem<DT>::pack2(acc[db][cb][4 * q4] * inv, acc[db][cb][4 * q4 + 1] * inv);
        w[1] = PElem<DT>::pack2(acc[db][cb][4 * q4 + 2] * inv, acc[db][cb][4 * q4 + 3] * inv);
        *(u32x2*)(op + (32 * db + 8 * q4 + 4 * hi) * 2) = w;
      }
  }
}

}  // namespace

int launch_prefill(vt_ctx* ctx, const vt_prefill_args* a, void* stream) {
  const uint32_t G = a->n_q_heads / a->n_kv_heads;
  if (G > (uint32_t)kRows) return VT_E_UNSUPPORTED;
  PrefillParams p;
  p.q = (const char*)a->q_new;
  p.out = (char*)a->out;
  p.k_new = (const char*)a->k_new;
  p.v_new = (const char*)a->v_new;
  p.k_ptrs = (const char* const*)a->k_ptrs;
  p.v_ptrs = (const char* const*)a->v_ptrs;
  p.cu = a->cu_seqlens;
  p.plens = a->prefix_lens;
  p.batch = a->batch;
  p.hq = a->n_q_heads;
  p.hkv = a->n_kv_heads;
  p.group = G;
  p.tb = kRows / G;
  p.scale_log2e = a->scale * 1.4426950408889634f;
  uint64_t tiles = 0;
  for (uint32_t b = 0; b < a->batch; ++b) {
    const uint32_t n = (uint32_t)(a->cu_seqlens_host[b + 1] - a->cu_seqlens_host[b]);
    tiles += (n + p.tb - 1) / p.tb;
  }
  if (tiles == 0) return VT_OK;
  if (tiles > 0x7fffffffull || a->n_kv_heads > 65535) return VT_E_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  dim3 grid((uint32_t)tiles, a->n_kv_heads);
  prof_begin(ctx, 1, st);
  if (a->dtype == VT_BF16 && a->head_dim == 128)
    hipLaunchKernelGGL((prefill_kernel<VT_BF16, 128>), grid, dim3(256), 0, st, p);
  else if (a->dtype == VT_BF16 && a->head_dim == 64)
    hipLaunchKernelGGL((prefill_kernel<VT_BF16, 64>), grid, dim3(256), 0, st, p);
  else if (a->dtype == VT_F16 && a->head_dim == 128)
    hipLaunchKernelGGL((prefill_kernel<VT_F16, 128>), grid, dim3(256), 0, st, p);
  else
    hipLaunchKernelGGL((prefill_kernel<VT_F16, 64>), grid, dim3(256), 0, st, p);
  prof_end(ctx, st);
  return hipGetLastError() == hipSuccess ? VT_OK : VT_E_DRIVER;
}

}  // namespace vt
