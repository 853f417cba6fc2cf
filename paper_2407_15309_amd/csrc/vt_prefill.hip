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
// of the second.
//
// Data movement: K and V tiles go from global memory straight into LDS (global_load_lds, 16 B per lane, no
// registers), double buffered, one workgroup barrier per tile.  Both tiles keep their natural [key][d]
// layout; the 16-byte chunks of a row are XOR-swizzled with the row number (applied to the global address,
// since the LDS side of such a load is fixed) so that the MFMA operand reads are bank-conflict free.  The
// V^T operand is read with the transposing LDS read (ds_read_b64_tr_b16): 16 lanes fetch a 4-key x 16-d
// block and each lane receives the 4 keys of its own d.
//
// The running maximum is only refreshed when a tile exceeds it by more than 2^8, which keeps the
// accumulator rescale off the common path; the final division by the running sum makes the result
// independent of which reference maximum was used.
#include <hip/hip_runtime.h>

#include <cmath>
#include <type_traits>

#include "vt_internal.h"

namespace vt {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kBN = 64;       // keys per tile
constexpr int kRows = 256;    // query rows per workgroup (4 wavefronts x 64)
constexpr float kTau = 8.0f;  // lazy-rescale threshold in log2 units

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
  // acc + both halves of a packed pair
  static __device__ __forceinline__ float add_pair(unsigned w, float acc) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, 0x3f803f80u), acc,
                                           false);
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
  static __device__ __forceinline__ float add_pair(unsigned w, float acc) {
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, w), __builtin_bit_cast(f16x2, 0x3c003c00u), acc, false);
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
  unsigned* counters;                  // [0] next work item, [1] workgroups that have left; zero between launches
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* gbl_ptr_t;

// 16 bytes per lane from global memory straight into LDS: lane l lands at lds_addr + 16*l (lds_addr uniform).
// Written as assembly so that these loads are invisible to the compiler's wait-count bookkeeping: it would
// otherwise guard operand reads of the tile buffers with waits for every outstanding load.  The kernel places
// its own waits (wait_loads) and barriers.  Two address forms: uniform base + 32-bit lane offset, or a 64-bit
// lane address.  (m0 is written here; nothing else in this file uses it.)
__device__ __forceinline__ void dma16(const char* base, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_off), "s"(base), "s"(lds_addr)
               : "memory");
}
__device__ __forceinline__ void dma16(const char* lane_addr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(lane_addr), "s"(lds_addr)
               : "memory");
}
// Marks a value that is the same in every lane as such (it then lives in scalar registers).
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ const char* uni(const char* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
  return (const char*)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t lds_addr_of(const char* p) {
  return (uint32_t)(size_t)(const __attribute__((address_space(3))) char*)p;
}

// Compile-time loop: f(integral_constant<int, I0>), ..., f(integral_constant<int, I1 - 1>).
template <int I0, int I1, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I0 < I1) {
    f(std::integral_constant<int, I0>{});
    static_for<I0 + 1, I1>(f);
  }
}

template <int DT, int D>
__global__ __launch_bounds__(256) void prefill_kernel(PrefillParams p) {
  constexpr int CH = D / 8;            // 16-byte chunks per head row
  constexpr int KS = D / 16;           // k-steps of the score product
  constexpr int DB = D / 32;           // 32-row d blocks of the value product
  constexpr int ROWB = D * 2;          // bytes per head row
  constexpr int RPL = 256 / ROWB;      // rows per 256-byte LDS bank line
  constexpr int RPI = 64 / CH;         // rows filled by one wavefront-wide load
  constexpr int TILEB = kBN * ROWB;    // bytes of one K (or V) tile
  constexpr int NLD = kBN / RPI / 4;   // loads per wavefront, tile and tensor
  // Four tile buffers (K tile, then V tile), separate arrays (not one array indexed by the buffer number) so
  // that the compiler can tell that the in-flight global-to-LDS loads of later tiles do not alias the operand
  // reads of the current one.  (Its bookkeeping of such loads distinguishes only a handful of arrays: with K
  // and V in arrays of their own the eighth one fell back to waiting for every outstanding load.)
  __shared__ __attribute__((aligned(1024))) char lds_t0[2 * TILEB];
  __shared__ __attribute__((aligned(1024))) char lds_t1[2 * TILEB];
  __shared__ __attribute__((aligned(1024))) char lds_t2[2 * TILEB];
  __shared__ __attribute__((aligned(1024))) char lds_t3[2 * TILEB];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, hi = lane >> 5;
  const int G = (int)p.group, tb = (int)p.tb;

  // Work items are (request, token tile, kv head).  The workgroups are persistent and take items from a device
  // counter, longest first: requests in descending order of prefix + new length, within a request the later
  // (longer) token tiles first, kv heads innermost.
  __shared__ int s_ord[kMaxPrefillBatch];      // s_ord[rank] = request
  __shared__ int s_pre[kMaxPrefillBatch + 1];  // items of the requests ranked before
  __shared__ int s_item;
  {
    const int B = (int)p.batch;
    for (int r = tid; r < B; r += 256) {
      const int key = p.plens[r] + p.cu[r + 1] - p.cu[r];
      int rank = 0;
      for (int u = 0; u < B; ++u) {
        const int ku = p.plens[u] + p.cu[u + 1] - p.cu[u];
        rank += (ku > key || (ku == key && u < r)) ? 1 : 0;
      }
      s_ord[rank] = r;
    }
    __syncthreads();
    if (tid == 0) {
      int n_before = 0;
      for (int rank = 0; rank < B; ++rank) {
        s_pre[rank] = n_before;
        const int r = s_ord[rank];
        n_before += ((p.cu[r + 1] - p.cu[r] + tb - 1) / tb) * (int)p.hkv;
      }
      s_pre[B] = n_before;
      s_item = (int)atomicAdd(&p.counters[0], 1u);
    }
    __syncthreads();
  }
  // (values read from LDS are the same in every lane; readfirstlane tells the compiler so, which keeps the
  // item's pointers and lengths in scalar registers)
  const int n_items = __builtin_amdgcn_readfirstlane(s_pre[p.batch]);
  int item = __builtin_amdgcn_readfirstlane(s_item);
  __syncthreads();
  for (; item < n_items;) {
  int next_item = 0;
  int b, rem, g, N;
  {
    int lo = 0, hi_r = (int)p.batch;  // last rank with s_pre[rank] <= item
    while (hi_r - lo > 1) {
      const int mid = (lo + hi_r) >> 1;
      if (s_pre[mid] <= item) lo = mid; else hi_r = mid;
    }
    lo = __builtin_amdgcn_readfirstlane(lo);
    b = __builtin_amdgcn_readfirstlane(s_ord[lo]);
    const int local = item - __builtin_amdgcn_readfirstlane(s_pre[lo]);
    N = uni(p.cu[b + 1] - p.cu[b]);
    const int nt = (N + tb - 1) / tb;
    g = local % (int)p.hkv;
    rem = nt - 1 - local / (int)p.hkv;
  }
  const int cu_b = uni(p.cu[b]), P = uni(p.plens[b]);
  const int tok0 = rem * tb;
  const int ntok = min(tb, N - tok0);
  const int total_keys = P + tok0 + ntok;      // keys the last token of the tile sees
  const int nkt = (total_keys + kBN - 1) / kBN;
  const uint32_t row_bytes = p.hkv * D * 2;
  const char* kc = uni(p.k_ptrs[b]) + (size_t)g * ROWB;
  const char* vc = uni(p.v_ptrs[b]) + (size_t)g * ROWB;
  const bool split_src = p.k_new != nullptr;
  const char* kn = split_src ? p.k_new + (size_t)g * ROWB : kc;
  const char* vn = split_src ? p.v_new + (size_t)g * ROWB : vc;
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
    const char* qp = p.q + ((size_t)(cu_b + tok0 + q_tok[cb]) * p.hq + (size_t)g * G + q_head[cb]) * ROWB;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[cb][ks] = *(const u32x4*)(qp + (16 * ks + 8 * hi) * 2);
  }
  // The Q operands stay in accumulation registers (MFMA reads its B operand from there as well), which leaves
  // the vector registers to the scores, the weights and the in-flight LDS operand reads.
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[cb][ks]));

  f32x16 acc[DB][2];
  float m_used[2], l_run[2];

  // Tile loads.  Load i of this wavefront fills LDS rows (4*wave + i)*RPI .. +RPI-1; the lane lands in row
  // ld_row + i*RPI (of the tile) at chunk position ld_pos and therefore fetches the chunk that the swizzle
  // assigns to that position.  K rows are swizzled with (row/RPL) % CH, V rows with 4*((row/RPL) % (CH/4)).
  const int last_key = total_keys - 1;
  // issue_part<i>: loads number i (one of K, one of V) of tile kt.  Every row chooses between the region and
  // the new rows, clamped to the last key.  The lane's row and chunk offsets are recomputed from the lane number
  // on every call (the asm hides the value from loop-invariant hoisting): keeping them live across the compute
  // phases costs vector registers the hot loop needs.  A tile's loads are issued a pair at a time between the
  // compute stages rather than back to back: the memory pipeline takes a 1 KiB load every 16 cycles or so, and
  // a wavefront that issues eight of them in a row (next to three other wavefronts doing the same) stalls.
  auto issue_part = [&](auto part, int kt, char* tile_k, char* tile_v) {
    constexpr int i = decltype(part)::value;
    unsigned l = (unsigned)lane;
    asm volatile("" : "+v"(l));
    const int row = wave * NLD * RPI + i * RPI + (int)(l / CH), ld_pos = (int)(l % CH);
    const uint32_t lk = (uint32_t)uni((int)lds_addr_of(tile_k) + (wave * NLD + i) * 1024);
    const uint32_t lv = (uint32_t)uni((int)lds_addr_of(tile_v) + (wave * NLD + i) * 1024);
    const int j = min(kt * kBN + row, last_key);
    const bool cached = j < P;
    const size_t ro = (size_t)(uint32_t)(cached ? j : j + new_row0) * row_bytes;
    dma16((cached ? kc : kn) + (ro + (uint32_t)((ld_pos ^ ((row / RPL) % CH)) * 16)), lk);
    dma16((cached ? vc : vn) + (ro + (uint32_t)((ld_pos ^ (4 * ((row / RPL) % (CH / 4)))) * 16)), lv);
  };
  auto issue_rest = [&](int kt, char* tile_k, char* tile_v) {  // parts 1 .. NLD-1
    issue_part(std::integral_constant<int, 1>{}, kt, tile_k, tile_v);
    if constexpr (NLD > 2) {
      issue_part(std::integral_constant<int, 2>{}, kt, tile_k, tile_v);
      issue_part(std::integral_constant<int, 3>{}, kt, tile_k, tile_v);
    }
  };
  auto issue_tile = [&](int kt, char* tile_k, char* tile_v) {
    issue_part(std::integral_constant<int, 0>{}, kt, tile_k, tile_v);
    issue_rest(kt, tile_k, tile_v);
  };
  static_assert(NLD == 2 || NLD == 4, "tile load split");

  // Operand reads of this lane.
  //  K operand (kb, ks): row 32*kb + col, chunk 2*ks + hi.
  //  V^T operand (db, kb, s2, h4): transposing read; inside its 16-lane group lane i supplies the address of
  //  key 32*kb + 16*s2 + 8*h4 + 4*hi + i/4, d = 32*db + 16*(col/16) + 4*(i%4), and receives the 4 keys
  //  (in order) of d = 32*db + col.
  const int kswz = ((col / RPL) % CH);  // K swizzle of row 32*kb + col (32 is a multiple of CH*RPL)
  const int vi = col & 15, vgi = col >> 4;
  const int v_key_lane = 4 * hi + (vi >> 2);           // + 32*kb + 16*s2 + 8*h4
  const int v_chunk_lane = 2 * vgi + ((vi & 3) >> 1);  // + 4*db
  const int v_within = 8 * (vi & 1);
  const float c = p.scale_log2e;

  // K operands of the 32-key block kb (one per k-step), and S^T block = K Q^T: 2*KS MFMAs.
  auto load_k = [&](const char* tk, int kb, u32x4* kf) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      kf[ks] = *(const u32x4*)(tk + (32 * kb + col) * ROWB + (((2 * ks + hi) ^ kswz) * 16));
  };
  auto mma_scores_cb = [&](const u32x4* kf, int cb, f32x16* s) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[cb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s[cb] = PElem<DT>::mfma(kf[ks], qf[cb][ks], s[cb]);
  };
  auto mma_scores = [&](const u32x4* kf, f32x16* s) {
    mma_scores_cb(kf, 0, s);
    mma_scores_cb(kf, 1, s);
  };
  auto scores = [&](const char* tk, int kb, f32x16* s) {
    u32x4 kf[KS];
    load_k(tk, kb, kf);
    mma_scores(kf, s);
  };
  // Softmax weights of a score block against the current reference maxima, rounded to the storage type (they
  // are the MFMA operand), and their sum added to the running sums.  The sum is taken over the rounded weights,
  // two per instruction (dot product of a packed pair with ones): the normaliser then matches the numerator
  // exactly, and the adds cost half as many instructions.
  auto weights_cb = [&](const f32x16* s, int cb, u32x4 (*pf)[2]) {
    float pr[16];
    const float nm = -m_used[cb];
#pragma unroll
    for (int i = 0; i < 16; ++i) pr[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[cb][i], c, nm));
    pf[cb][0] = PElem<DT>::pack8(pr);
    pf[cb][1] = PElem<DT>::pack8(pr + 8);
    float psum = 0.f, psum2 = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      psum = PElem<DT>::add_pair(pf[cb][0][w], psum);
      psum2 = PElem<DT>::add_pair(pf[cb][1][w], psum2);
    }
    l_run[cb] += psum + psum2;
  };
  auto weights = [&](const f32x16* s, u32x4 (*pf)[2]) {
    weights_cb(s, 0, pf);
    weights_cb(s, 1, pf);
  };
  // V^T operands of block kb (one per (d block, 16-key step)), and O^T += V^T P^T: 4*DB MFMAs.
  auto load_v_part = [&](const char* tv, int kb, u32x4* vf, int db0, int db1) {
#pragma unroll
    for (int db = db0; db < db1; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        s16x4 h[2];
#pragma unroll
        for (int h4 = 0; h4 < 2; ++h4) {
          const int key = 32 * kb + 16 * s2 + 8 * h4 + v_key_lane;
          const int chunk = (4 * db + v_chunk_lane) ^ (4 * ((key / RPL) % (CH / 4)));
          const char* a = tv + key * ROWB + chunk * 16 + v_within;
          h[h4] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a);
        }
        const u32x2 lo = __builtin_bit_cast(u32x2, h[0]), hi2 = __builtin_bit_cast(u32x2, h[1]);
        u32x4 f;
        f[0] = lo[0];
        f[1] = lo[1];
        f[2] = hi2[0];
        f[3] = hi2[1];
        vf[2 * db + s2] = f;
      }
  };
  auto load_v = [&](const char* tv, int kb, u32x4* vf) { load_v_part(tv, kb, vf, 0, DB); };
  auto mma_values = [&](const u32x4* vf, u32x4 (*pf)[2]) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        acc[db][0] = PElem<DT>::mfma(vf[2 * db + s2], pf[0][s2], acc[db][0]);
        acc[db][1] = PElem<DT>::mfma(vf[2 * db + s2], pf[1][s2], acc[db][1]);
      }
  };
  auto values = [&](const char* tv, int kb, u32x4 (*pf)[2]) {
    u32x4 vf[2 * DB];
    load_v(tv, kb, vf);
    mma_values(vf, pf);
  };
  // Column maxima of a score block (over the lane's 16 keys and its partner half), in exp2 units.
  auto block_max = [&](const f32x16* s, float* tmax) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
      float t = fmaxf(s[cb][0], s[cb][1]);
#pragma unroll
      for (int i = 2; i < 16; i += 2) t = fmaxf(t, fmaxf(s[cb][i], s[cb][i + 1]));
      tmax[cb] = fmaxf(t, __shfl_xor(t, 32)) * c;
    }
  };

  // Waits until at most `n` of this wavefront's global-to-LDS loads are outstanding.
  auto wait_loads = [](auto n) {
    constexpr int N = decltype(n)::value;
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
  };
  constexpr int VM = 2 * NLD;  // global-to-LDS loads per wavefront and tile
  // Tile pipeline.  Tile t lives in buffer t % 4.  While tile kt is computed, tiles kt+1 and kt+2 are in flight
  // or landed.  Every tile kt follows the same protocol.  Before its synchronisation point it issues loads
  // 1 and 2 of tile kt+2 (only load 1 when a tile has two loads per tensor).  At the synchronisation point the
  // wavefront waits until its own part of tile kt+1 has landed - loads complete in order, so it waits until at
  // most the SYNC_N loads issued after that tile's last one are outstanding - then, past the barrier, everyone's
  // part has landed and everyone is done with tile kt-1.  After it, it issues the last load of tile kt+2 (when
  // there are four) and load 0 of tile kt+3, which goes into the buffer of tile kt-1.  Past the last tile the
  // refills repeat tile nkt-1 (into buffers nobody reads), which keeps the count of outstanding loads, and with
  // it the wait, the same on every tile.  The barrier is the bare instruction: the fence of __syncthreads
  // would wait for all outstanding loads.
  constexpr int SYNC_N = NLD > 2 ? VM - 2 : VM;
  const std::integral_constant<int, 0> part0;
  const std::integral_constant<int, 1> part1;
  const std::integral_constant<int, 2> part2;
  const std::integral_constant<int, 3> part3;
  auto issue_before_sync = [&](int kt, char* gk, char* gv) {
    const int t2 = min(kt + 2, nkt - 1);
    issue_part(part1, t2, gk, gv);
    if constexpr (NLD > 2) issue_part(part2, t2, gk, gv);
  };
  auto sync_next = [&]() {
    wait_loads(std::integral_constant<int, SYNC_N>{});
    __builtin_amdgcn_s_barrier();
  };
  auto issue_after_sync = [&](int kt, char* gk, char* gv, char* fk, char* fv) {
    if constexpr (NLD > 2) issue_part(part3, min(kt + 2, nkt - 1), gk, gv);
    issue_part(part0, min(kt + 3, nkt - 1), fk, fv);
  };

  // One of the nine steps that turn a 32-key x 32-row score block (16 values per lane) into weights: step
  // j < 8 computes weights 2j and 2j+1, step j >= 1 packs the previous pair into word j-1 of the MFMA operand
  // and adds the pair (as rounded) to the partial sum.
  auto weight_step = [&](auto jc, const f32x16& sv, float nm, float* pr, u32x4* pw, float& ps) {
    constexpr int j = decltype(jc)::value;
    if constexpr (j < 8) {
      pr[2 * j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * j], c, nm));
      pr[2 * j + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * j + 1], c, nm));
    }
    if constexpr (j >= 1) {
      const unsigned w = PElem<DT>::pack2(pr[2 * j - 2], pr[2 * j - 1]);
      pw[(j - 1) / 4][(j - 1) % 4] = w;
      ps = PElem<DT>::add_pair(w, ps);
    }
  };
  // One transposing read of a V^T operand half: read r of block kb covers d block r/4, 16-key step (r/2)%2,
  // 8-key half r%2; operand 2*db + s2 is the pair of reads 2m, 2m+1.
  auto read_v = [&](auto rc, const char* tv, int kb) -> u32x2 {
    constexpr int r = decltype(rc)::value;
    constexpr int db = r / 4, s2 = (r / 2) % 2, h4 = r % 2;
    const int key = 32 * kb + 16 * s2 + 8 * h4 + v_key_lane;
    const int chunk = (4 * db + v_chunk_lane) ^ (4 * ((key / RPL) % (CH / 4)));
    const char* a = tv + key * ROWB + chunk * 16 + v_within;
    return __builtin_bit_cast(u32x2,
                              __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)a));
  };
  auto read_k = [&](auto ksc, const char* tk, int kb) -> u32x4 {
    constexpr int ks = decltype(ksc)::value;
    return *(const u32x4*)(tk + (32 * kb + col) * ROWB + (((2 * ks + hi) ^ kswz) * 16));
  };
  // MFMA i of the value product of one 32-key block: operand i/2, query column block i%2.
  auto pv_mfma = [&](auto ic, const u32x2* vh, u32x4 (*pf)[2]) {
    constexpr int i = decltype(ic)::value;
    constexpr int m = i / 2, cb = i % 2, db = m / 2, s2 = m % 2;
    u32x4 f;
    f[0] = vh[2 * m][0];
    f[1] = vh[2 * m][1];
    f[2] = vh[2 * m + 1][0];
    f[3] = vh[2 * m + 1][1];
    acc[db][cb] = PElem<DT>::mfma(f, pf[cb][s2], acc[db][cb]);
  };

  // Fast tile: every (row, key) pair visible, reference maxima fixed.  The instruction order is fixed by hand:
  // the code is a sequence of slots, each one MFMA followed by a share of the vector, LDS and load-issue work
  // that does not depend on it, and nothing moves between slots.  (Left to itself the scheduler puts long runs
  // of exponentials between the MFMAs and leaves the matrix pipeline idle; a single wavefront per SIMD has
  // nobody else to fill such gaps.)  Six stages; the scores are computed per 32-row half so that the weights
  // of one half can be worked out beside the scores of the next:
  //   A  S(block 0, rows 0-31)          | reads K block 1, issues loads of tile kt+2
  //   B  S(block 0, rows 32-63)         | weights of A's scores, reads first half of V block 0
  //   C  S(block 1, rows 0-31)          | weights of B's scores, reads second half of V block 0
  //   D  S(block 1, rows 32-63)         | weights of C's scores
  //   E  O += V(block 0) P(block 0)     | weights of D's scores, reads V block 1
  //   -- synchronisation point --
  //   F  O += V(block 1) P(block 1)     | issues loads of tiles kt+2 / kt+3, reads K block 0 of the next tile
  // ck/cv: this tile; nk: K of the next tile; gk/gv: buffer of tile kt+2; fk/fv: buffer of tile kt+3.  k0 holds K
  // block 0 of this tile on entry and of the next tile on exit.
  constexpr int NPV = 4 * DB;  // MFMAs of one value product; also the transposing reads of one V block
  static_assert(NPV == 2 * KS, "V reads are spread one per slot over two score stages");
  auto fast_tile = [&](int kt, const char* ck, const char* cv, const char* nk, char* gk, char* gv, char* fk,
                       char* fv, u32x4* k0) {
    f32x16 s0[2], s1[2];
    u32x4 p0[2][2], p1[2][2];
    u32x4 k1[KS];
    u32x2 v0h[NPV], v1h[NPV];
    float pr[16], ps;
    const float nm0 = -m_used[0], nm1 = -m_used[1];
    const int t2 = min(kt + 2, nkt - 1);
    auto zero = [](f32x16& x) {
#pragma unroll
      for (int i = 0; i < 16; ++i) x[i] = 0.f;
    };
    // A
    zero(s0[0]);
    static_for<0, KS>([&](auto i) {
      s0[0] = PElem<DT>::mfma(k0[i], qf[0][i], s0[0]);
      k1[i] = read_k(i, ck, 1);
      if constexpr (i == 0) issue_part(part1, t2, gk, gv);
      if constexpr (i == KS / 2 && NLD > 2) issue_part(part2, t2, gk, gv);
      __builtin_amdgcn_sched_barrier(0);
    });
    // B
    zero(s0[1]);
    ps = 0.f;
    static_for<0, KS>([&](auto i) {
      s0[1] = PElem<DT>::mfma(k0[i], qf[1][i], s0[1]);
      static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s0[0], nm0, pr, p0[0], ps); });
      v0h[i] = read_v(i, cv, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run[0] += ps;
    // C
    zero(s1[0]);
    ps = 0.f;
    static_for<0, KS>([&](auto i) {
      s1[0] = PElem<DT>::mfma(k1[i], qf[0][i], s1[0]);
      static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s0[1], nm1, pr, p0[1], ps); });
      v0h[KS + i] = read_v(std::integral_constant<int, KS + i>{}, cv, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run[1] += ps;
    // D
    zero(s1[1]);
    ps = 0.f;
    static_for<0, KS>([&](auto i) {
      s1[1] = PElem<DT>::mfma(k1[i], qf[1][i], s1[1]);
      static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s1[0], nm0, pr, p1[0], ps); });
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run[0] += ps;
    // E
    ps = 0.f;
    static_for<0, NPV>([&](auto i) {
      pv_mfma(i, v0h, p0);
      static_for<i * 9 / NPV, (i + 1) * 9 / NPV>([&](auto j) { weight_step(j, s1[1], nm1, pr, p1[1], ps); });
      v1h[i] = read_v(i, cv, 1);
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run[1] += ps;
    sync_next();
    // F
    static_for<0, NPV>([&](auto i) {
      pv_mfma(i, v1h, p1);
      if constexpr (i < KS) k0[i] = read_k(i, nk, 0);
      if constexpr (i == 0 && NLD > 2) issue_part(part3, t2, gk, gv);
      if constexpr (i == NPV / 2) issue_part(part0, min(kt + 3, nkt - 1), fk, fv);
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  auto buf_k = [&](int t) -> char* {
    const int m = t & 3;
    return m == 0 ? lds_t0 : (m == 1 ? lds_t1 : (m == 2 ? lds_t2 : lds_t3));
  };
  auto buf_v = [&](int t) -> char* { return buf_k(t) + TILEB; };

  // Generic tile: causal mask, classic online softmax (reference maxima follow the data, accumulators
  // rescaled when a maximum moves by more than kTau).
  auto generic_tile = [&](const char* tk, const char* tv, int j0) {
#pragma unroll 1
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s[2];
      scores(tk, kb, s);
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int j = j0 + 32 * kb + 8 * (i >> 2) + 4 * hi + (i & 3);
          s[cb][i] = j <= lim[cb] ? s[cb][i] : -INFINITY;
        }
      float tmax[2];
      block_max(s, tmax);
      const bool grow0 = tmax[0] > m_used[0] + kTau, grow1 = tmax[1] > m_used[1] + kTau;
      if (__builtin_amdgcn_ballot_w64(grow0 || grow1) != 0) {
        // The accumulators live in accumulation registers (the MFMAs read and write them there); this is the
        // only other code that touches them, so it goes through explicit moves.
#pragma unroll
        for (int cb = 0; cb < 2; ++cb) {
          const float m_new = (cb ? grow1 : grow0) ? tmax[cb] : m_used[cb];
          const float alpha = __builtin_amdgcn_exp2f(m_used[cb] - m_new);
          m_used[cb] = m_new;
          l_run[cb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              float t;
              asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n\tv_accvgpr_write_b32 %0, %1"
                           : "+a"(acc[db][cb][i]), "=&v"(t)
                           : "v"(alpha));
            }
        }
      }
      u32x4 pf[2][2];
      weights(s, pf);
      values(tv, kb, pf);
    }
  };

  // Tiles whose last key every row of the workgroup may see: kt*64 + 63 <= P + tok0.
  int nfast = min(nkt, (P + tok0 + 1) / kBN);
  for (int attempt = 0;; ++attempt) {
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][cb][i] = 0.f;
    m_used[0] = m_used[1] = -INFINITY;
    l_run[0] = l_run[1] = 0.f;

    issue_tile(0, lds_t0, lds_t0 + TILEB);
    issue_tile(min(1, nkt - 1), lds_t1, lds_t1 + TILEB);
    issue_part(part0, min(2, nkt - 1), lds_t2, lds_t2 + TILEB);
    wait_loads(std::integral_constant<int, VM + 2>{});
    __builtin_amdgcn_s_barrier();
    int kt = 0;
    if (nfast > 0) {
      // Reference maxima for the fast tiles: the column maxima of the first 32 keys (plus headroom when the
      // weights are fp16).  Rows whose later scores outgrow the representable range are caught below.
      u32x4 k0[KS];
      load_k(lds_t0, 0, k0);
      {
        f32x16 s[2];
        float tmax[2];
        mma_scores(k0, s);
        block_max(s, tmax);
        m_used[0] = tmax[0] + (DT == VT_F16 ? 4.0f : 0.0f);
        m_used[1] = tmax[1] + (DT == VT_F16 ? 4.0f : 0.0f);
      }
      for (;;) {
        fast_tile(kt, lds_t0, lds_t0 + TILEB, lds_t1, lds_t2, lds_t2 + TILEB, lds_t3, lds_t3 + TILEB, k0);
        if (++kt >= nfast) break;
        fast_tile(kt, lds_t1, lds_t1 + TILEB, lds_t2, lds_t3, lds_t3 + TILEB, lds_t0, lds_t0 + TILEB, k0);
        if (++kt >= nfast) break;
        fast_tile(kt, lds_t2, lds_t2 + TILEB, lds_t3, lds_t0, lds_t0 + TILEB, lds_t1, lds_t1 + TILEB, k0);
        if (++kt >= nfast) break;
        fast_tile(kt, lds_t3, lds_t3 + TILEB, lds_t0, lds_t1, lds_t1 + TILEB, lds_t2, lds_t2 + TILEB, k0);
        if (++kt >= nfast) break;
      }
    }
    for (; kt < nkt; ++kt) {
      issue_before_sync(kt, buf_k(kt + 2), buf_v(kt + 2));
      generic_tile(buf_k(kt), buf_v(kt), kt * kBN);
      sync_next();
      issue_after_sync(kt, buf_k(kt + 2), buf_v(kt + 2), buf_k(kt + 3), buf_v(kt + 3));
    }
    // drain the repeated refills before anything else is loaded into the buffers
    wait_loads(std::integral_constant<int, 0>{});
    if (attempt > 0 || nfast == 0) break;
    // Fixed reference maxima can overflow the weights when later scores are far larger than the first ones:
    // then some sum or accumulator is no longer finite and the whole workgroup redoes its rows the classic way.
    float chk = l_run[0] + l_run[1];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int cb = 0; cb < 2; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) chk += __builtin_fabsf(acc[db][cb][i]);
    if (!__syncthreads_or(!(chk < INFINITY))) break;
    nfast = 0;
  }

  // The next item is claimed only now: a workgroup that claimed it at the start would sit on it for the whole
  // current item while others idle at the end of the launch.  The atomic's latency hides behind the stores.
  if (tid == 0) next_item = (int)atomicAdd(&p.counters[0], 1u);

  // out[row, d] = acc / l.  acc[db][cb][i] is d = 32*db + 8*(i/4) + 4*hi + i%4 of the lane's query row.
#pragma unroll
  for (int cb = 0; cb < 2; ++cb) {
    const float l_tot = l_run[cb] + __shfl_xor(l_run[cb], 32);
    if (!q_valid[cb]) continue;
    const float inv = 1.0f / l_tot;
    char* op = p.out + ((size_t)(cu_b + tok0 + q_tok[cb]) * p.hq + (size_t)g * G + q_head[cb]) * ROWB;
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
  // next item (the barriers also keep the LDS tiles of this item safe from the next item's loads)
  __syncthreads();
  if (tid == 0) s_item = next_item;
  __syncthreads();
  item = __builtin_amdgcn_readfirstlane(s_item);
  }  // item loop

  // Leave the counters at zero for the next launch: the last workgroup out resets them.
  if (tid == 0) {
    const unsigned old = atomicAdd(&p.counters[1], 1u);
    if (old == gridDim.x - 1) {
      p.counters[0] = 0u;
      p.counters[1] = 0u;
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
  const uint64_t items = tiles * a->n_kv_heads;
  if (items > 0x7fffffffull || a->batch > (uint32_t)kMaxPrefillBatch || !ctx->counters) return VT_E_UNSUPPORTED;
  p.counters = (unsigned*)ctx->counters;
  hipStream_t st = (hipStream_t)stream;
  dim3 grid((uint32_t)(items < (uint64_t)ctx->n_cus ? items : (uint64_t)ctx->n_cus));
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
