// Batched decode attention over per-request contiguous K/V regions (gfx950).
//
// What is computed (paper "LLM Inference", decode stage; "KV Cache Optimization: GQA and MQA" for grouped
// heads): for request b and
// query head h, out = sum_j softmax_j(scale <q, k_j>) v_j over the request's cached rows, K/V row j of
// KV head g living at base_b + (j*Hkv + g)*D.  Because a request's cache is one contiguous virtual
// range (paper "vTensor") the kernel addresses rows by plain pointer arithmetic.
//
// Work decomposition ("tape" split).  For every KV head the cached tokens of all requests, laid end to end,
// form one tape of sum_b L_b tokens.  The tape is cut into n_seg equal segments of seg_len tokens and one
// wavefront owns one (segment, kv head): every wavefront reads the same number of tokens (no ragged tail
// however the lengths are distributed), reads them as one long sequential stream per region (which is what
// HBM likes), and the 4 wavefronts of a workgroup take 4 adjacent kv heads of the same segment, so the
// workgroup's loads cover 1 KiB contiguous per token row.  A segment may cross request boundaries: the part
// of a request inside a segment is a "piece".  A piece that is the whole request is normalised and written
// to the output directly; otherwise the wavefront stores (m, l, acc) per head for the piece and a small
// second kernel merges a request's pieces with the log-sum-exp rule.  A wavefront keeps the next tile's loads
// in flight at all times, across piece boundaries too.
//
// Matrix-core mapping (v_mfma_f32_16x16x32, one wavefront, tiles of 32 tokens):
//   S^T[token, head]  = K_tile[16 tokens x D] * Q^T[D x 16 heads]      (A = K rows, B = Q, heads padded to 16)
//   O^T[d, head]     += V_tile^T[d x 32 tokens] * P^T[32 tokens x heads] (A = V^T, B = P)
// All G query heads of the group ride in the N dimension, so every K/V byte is read from HBM once per KV
// head.  The result layout of the first product (lane holds one head column and four token rows per
// 16-token block) is exactly the B-operand layout of the second once the 32 tokens of a tile are assigned to
// the contraction slots in the order each lane already holds them, so P never moves between lanes.  V^T is
// produced without shared memory: a lane loads the same 16-byte column chunk of the 8 token rows of its
// contraction slots and transposes the 8x8 block of 16-bit values inside its own registers.  K goes
// through a wavefront-private LDS staging buffer so that the global loads stay fully coalesced
// (16 lanes x 16 B = one 256 B row piece) while the MFMA operand wants 16 different rows per 16 lanes.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

#include "vt_internal.h"

namespace vt {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

constexpr int kTile = 32;   // tokens per tile
constexpr int kWaves = 4;   // wavefronts per workgroup

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
  int32_t* tape;    // [B+1] exclusive prefix sums of kv_lens, written by workgroup 0 for the merge kernel
  float* part_acc;  // [B][max_pieces][Hq][D]
  float* part_m;    // [B][max_pieces][Hq], running max of scale*log2(e)*score
  float* part_l;    // [B][max_pieces][Hq]
  void* out;        // [B][Hq][D]
  uint32_t batch, hq, hkv, group, seg_len, max_pieces, n_seg;
  uint32_t sub;  // 16-head sub-groups per kv head (1 unless the group has more than 16 query heads)
  float scale_log2e;
};

// 8x8 transpose of 16-bit values held as 8 registers-of-8 (rows = tokens, columns = d) inside one lane.
// out[dd] holds column dd of the block: the 8 tokens' values of d = dd, in token-slot order.
// 16 bytes of K/V, read once: a global (not flat) load, so that it only counts as a vector-memory operation and
// the waits for LDS traffic do not wait for it as well, marked nontemporal (a plain streaming read of HBM reaches
// 6.3 TB/s on this chip, a nontemporal one 7.1 TB/s).
__device__ __forceinline__ u32x4 stream_load16(const char* p) {
  return __builtin_nontemporal_load((const __attribute__((address_space(1))) u32x4*)p);
}

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

// The part of one request that lies inside this wavefront's segment.  Fields are wavefront-uniform except the
// two lane base pointers.
struct Piece {
  bool valid;
  int b, t0, t1, index, count;  // tokens [t0, t1) of request b; piece `index` of `count`
  const char* kb;               // lane's K base: region + head offset + its 16-byte chunk
  const char* vb;
};

// NB: blocks of 16 query heads one wavefront carries (1, or 2 for groups of more than 16 heads: the second block
// reuses the tile's K rows in LDS and its transposed V registers, so the K/V head is read once for 32 heads; that
// variant needs more than 256 registers and runs one wavefront per SIMD).
template <int DT, int D, int NB>
__global__ __launch_bounds__(64 * kWaves) __attribute__((amdgpu_waves_per_eu(NB == 1 ? 2 : 1, NB == 1 ? 2 : 1))) void
decode_kernel(DecodeParams p) {
  using T = Tile<D>;
  constexpr int CH = T::CH, TPL = T::TPL, NLK = T::NLK;
  constexpr int KK = D / 32;       // MFMA k-steps of the score product
  constexpr int NM = D / 16;       // MFMAs (16 d-rows each) of the value product
  constexpr int RSB = D * 2 + 16;  // LDS row stride in bytes (the 16 B pad spreads the rows of an operand read over the
                                   // banks; the counters still show conflicts on about half of the LDS instructions,
                                   // which a kernel that waits for HBM does not feel)
  __shared__ __attribute__((aligned(16))) char lds_all[kWaves][kTile * RSB];
  __shared__ int tape[kMaxDecodeBatch + 1];  // tape[b] = tokens of the requests before b
  __shared__ int wave_tot[kWaves];
  // Region bases of the first requests, fetched beside the lengths: a piece of one of them starts its K/V loads
  // without a second round trip to memory for the pointers.
  constexpr int kPtrWin = 256;
  __shared__ const char* s_kp[kPtrWin];
  __shared__ const char* s_vp[kPtrWin];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int B = (int)p.batch, seg_len = (int)p.seg_len;

  // Exclusive prefix sum of the lengths, entries 0 .. B (entry B is the tape's total).  Thread t owns the `per`
  // consecutive entries t*per .. t*per + per - 1 with per = ceil((B + 1) / 256), so the 256 threads cover
  // 0 .. 256*per - 1 >= B whatever the batch (one entry per thread up to batch 255, 17 at the largest batch);
  // wavefront scan of the per-thread sums, then across wavefronts.
  {
    const int per = (B + 256) >> 8;
    if (tid < kPtrWin && tid < B) {
      s_kp[tid] = p.k_ptrs[tid];
      s_vp[tid] = p.v_ptrs[tid];
    }
    int sum = 0;
    for (int i = 0; i < per; ++i) {
      const int r = tid * per + i;
      sum += r < B ? p.kv_lens[r] : 0;
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int base = incl - sum;
    for (int w = 0; w < wave; ++w) base += wave_tot[w];
    for (int i = 0; i < per; ++i) {
      const int r = tid * per + i;
      if (r <= B) {
        tape[r] = base;
        if (blockIdx.x == 0) p.tape[r] = base;
      }
      base += r < B ? p.kv_lens[r] : 0;
    }
    __syncthreads();
  }
  const int total = tape[B];

  // This wavefront's (segment, kv head).
  const unsigned w_global = (unsigned)__builtin_amdgcn_readfirstlane((int)(blockIdx.x * kWaves + wave));
  // A wavefront carries at most 16 query heads (the N dimension of the MFMA).  A group of more than 16 is cut into
  // sub-groups of 16 that each get a wavefront of their own and read the same K/V head (the four wavefronts of a
  // workgroup are neighbours in this numbering, so the repeated reads meet in the caches).
  const unsigned wsub = (p.sub + NB - 1) / NB;            // wavefronts per (segment, kv head)
  const unsigned units_per_seg = p.hkv * wsub;
  const int sidx = (int)(w_global / units_per_seg);
  const int gv = (int)(w_global - (unsigned)sidx * units_per_seg);
  const int g = gv / (int)wsub;                           // kv head
  const int h0 = (gv - g * (int)wsub) * 16 * NB;          // first query head of this wavefront inside the group
  int n_heads[NB];                                        // query heads of each 16-head block this wavefront carries
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) n_heads[nb] = max(0, min(16, (int)p.group - h0 - 16 * nb));
  const int seg0 = sidx * seg_len;
  if (sidx >= (int)p.n_seg || seg0 >= total) return;
  const int seg1 = min(seg0 + seg_len, total);

  char* lds = lds_all[wave];
  const int c16 = lane & 15, j = lane >> 4;
  const int cK = lane % CH, jK = lane / CH;
  const uint32_t row_bytes = p.hkv * D * 2;

  auto make_piece = [&](Piece& d, int b) {
    d.valid = b < B && tape[b] < seg1;
    if (!d.valid) return;
    const int T0 = tape[b], L = tape[b + 1] - T0;
    d.b = b;
    d.t0 = max(seg0 - T0, 0);
    d.t1 = min(L, seg1 - T0);
    const int first = T0 / seg_len;
    d.index = sidx - first;
    d.count = (T0 + L - 1) / seg_len - first + 1;
    d.kb = (b < kPtrWin ? s_kp[b] : p.k_ptrs[b]) + (size_t)g * D * 2 + cK * 16;
    d.vb = (b < kPtrWin ? s_vp[b] : p.v_ptrs[b]) + (size_t)g * D * 2 + (c16 % CH) * 16;
  };

  Piece cur, nxt;
  {
    int lo = 0, hi = B;  // request containing tape position seg0: tape[lo] <= seg0 < tape[lo+1]
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (tape[mid] <= seg0) lo = mid; else hi = mid;
    }
    make_piece(cur, lo);
    make_piece(nxt, lo + 1);
  }

  u32x4 qf[NB][KK];
  f32x4 acc[NB][NM];
  float m_run[NB], l_run[NB];
  // Q as the B operand: lane (head c16, slot j) holds d-chunk 4*kk + j of its head; heads >= group are zero.
  auto begin_piece = [&](const Piece& d) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const char* qh = p.q + ((size_t)d.b * p.hq + (size_t)g * p.group + h0 + 16 * nb + c16) * D * 2;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        u32x4 z = {0u, 0u, 0u, 0u};
        qf[nb][kk] = (c16 < n_heads[nb]) ? *(const u32x4*)(qh + (4 * kk + j) * 16) : z;
      }
#pragma unroll
      for (int m = 0; m < NM; ++m) acc[nb][m] = f32x4{0.f, 0.f, 0.f, 0.f};
      m_run[nb] = -INFINITY;
      l_run[nb] = 0.f;
    }
  };

  auto load_tile = [&](T& t, const Piece& d, int tile) {
    const int last = d.t1 - 1;
#pragma unroll
    for (int i = 0; i < NLK; ++i) {
      const int tok = min(tile + i * TPL + jK, last);
      t.k[i] = stream_load16(d.kb + (size_t)tok * row_bytes);
    }
#pragma unroll
    for (int i8 = 0; i8 < 8; ++i8) {
      const int tok = min(tile + (i8 & 3) + 4 * j + (i8 >> 2) * 16, last);
      t.v[i8] = stream_load16(d.vb + (size_t)tok * row_bytes);
    }
  };

  auto compute_tile = [&](const T& t, int tile, int t1) {
    // K tile -> LDS (coalesced layout) -> MFMA A-operand layout.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < NLK; ++i) *(u32x4*)(lds + (i * TPL + jK) * RSB + cK * 16) = t.k[i];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    u32x4 vt[8];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      f32x4 sc[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        sc[hh] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const u32x4 kf = *(const u32x4*)(lds + (16 * hh + c16) * RSB + (4 * kk + j) * 16);
          sc[hh] = Elem<DT>::mfma(kf, qf[nb][kk], sc[hh]);
        }
      }
      // Online softmax for head c16 over this lane's 8 tokens (4*j+i and 16+4*j+i) and, via two
      // cross-lane exchanges, over all 32 tokens of the tile.
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int tok = tile + (e & 3) + 4 * j + (e >> 2) * 16;
        const float v = sc[e >> 2][e & 3] * p.scale_log2e;
        x[e] = tok < t1 ? v : -INFINITY;
      }
      float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      mx = fmaxf(mx, __shfl_xor(mx, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[nb], mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run[nb] - m_new);
      m_run[nb] = m_new;
      float pr[8], psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        pr[e] = __builtin_amdgcn_exp2f(x[e] - m_new);
        psum += pr[e];
      }
      l_run[nb] = l_run[nb] * alpha + psum;
      const u32x4 pf = Elem<DT>::pack8(pr);
      // V^T operand by in-lane transpose (once per tile, shared by the head blocks), then O^T += V^T P^T.
      if (nb == 0) transpose8x8(t.v, vt);
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
        acc[nb][m] *= alpha;
        acc[nb][m] = Elem<DT>::mfma(a, pf, acc[nb][m]);
      }
    }
  };

  // d index of accumulator element (m, i) of this lane.
  auto d_of = [&](int m, int i) -> int {
    if constexpr (D == 128) return 32 * j + 8 * i + m;
    const int r = 4 * j + i;
    return 8 * (r & 7) + 2 * m + (r >> 3);
  };

  auto end_piece = [&](const Piece& d) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float l_tot = l_run[nb] + __shfl_xor(l_run[nb], 16);
      l_tot += __shfl_xor(l_tot, 32);
      if (c16 >= n_heads[nb]) continue;
      const size_t head = (size_t)g * p.group + h0 + 16 * nb + c16;
      if (d.count == 1) {
        // The piece is the whole request: normalise and write the output row.
        const float inv = 1.0f / l_tot;
        unsigned short* o = (unsigned short*)p.out + ((size_t)d.b * p.hq + head) * D;
        if constexpr (D == 128) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float r[8];
#pragma unroll
            for (int m = 0; m < 8; ++m) r[m] = acc[nb][m][i] * inv;
            *(u32x4*)(o + 32 * j + 8 * i) = Elem<DT>::pack8(r);
          }
        } else {
#pragma unroll
          for (int m = 0; m < NM; ++m)
#pragma unroll
            for (int i = 0; i < 4; ++i) o[d_of(m, i)] = Elem<DT>::cvt(acc[nb][m][i] * inv);
        }
        continue;
      }
      const size_t pidx = ((size_t)d.b * p.max_pieces + d.index) * p.hq + head;
      float* pa = p.part_acc + pidx * D;
      if constexpr (D == 128) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 lo = {acc[nb][0][i], acc[nb][1][i], acc[nb][2][i], acc[nb][3][i]};
          f32x4 hi = {acc[nb][4][i], acc[nb][5][i], acc[nb][6][i], acc[nb][7][i]};
          *(f32x4*)(pa + 32 * j + 8 * i) = lo;
          *(f32x4*)(pa + 32 * j + 8 * i + 4) = hi;
        }
      } else {
#pragma unroll
        for (int m = 0; m < NM; ++m)
#pragma unroll
          for (int i = 0; i < 4; ++i) pa[d_of(m, i)] = acc[nb][m][i];
      }
      if (j == 0) {
        p.part_m[pidx] = m_run[nb];
        p.part_l[pidx] = l_tot;
      }
    }
  };

  T ta, tb;
  int tile = cur.t0;
  begin_piece(cur);
  load_tile(ta, cur, tile);
  bool running = true;
  // One phase: start the loads of the tile after this one (of this piece, else of the next piece), compute
  // this tile, and on the piece's last tile finish it and move to the next piece.
  auto phase = [&](T& now, T& next) {
    if (tile + kTile < cur.t1) {
      load_tile(next, cur, tile + kTile);
    } else if (nxt.valid) {
      load_tile(next, nxt, nxt.t0);
    }
    compute_tile(now, tile, cur.t1);
    tile += kTile;
    if (tile >= cur.t1) {
      end_piece(cur);
      if (!nxt.valid) {
        running = false;
        return;
      }
      cur = nxt;
      begin_piece(cur);
      tile = cur.t0;
      make_piece(nxt, cur.b + 1);
    }
  };
  while (running) {
    phase(ta, tb);
    if (!running) break;
    phase(tb, ta);
  }
}

// Merge of a request's pieces (requests with a single piece were written by the main kernel):
// M = max_s m_s; out = sum_s acc_s 2^(m_s-M) / sum_s l_s 2^(m_s-M).
// One workgroup of W wavefronts per (request, query head).  A long request at a small batch is cut into hundreds of
// pieces, and walking them one after the other is a chain of memory round trips: wavefront w takes pieces w, w+W,
// ..., four of them in flight at a time, each lane D/64 of the row's values, keeps a running maximum with rescaled
// sums, and the wavefronts' results meet in LDS.
template <int DT, int D, int W>
__global__ __launch_bounds__(64 * W) void decode_combine_kernel(DecodeParams p) {
  constexpr int E = D / 64;  // values per lane
  __shared__ float s_m[W], s_den[W];
  __shared__ float s_num[W][D];
  const uint32_t h = blockIdx.x, b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int T0 = p.tape[b], L = p.tape[b + 1] - T0, seg_len = (int)p.seg_len;
  const int n = min((T0 + L - 1) / seg_len - T0 / seg_len + 1, (int)p.max_pieces);
  if (n <= 1) return;
  const size_t base = (size_t)b * p.max_pieces * p.hq + h;
  float M = -INFINITY, den = 0.f, num[E];
#pragma unroll
  for (int e = 0; e < E; ++e) num[e] = 0.f;
  for (int s = wave; s < n; s += 4 * W) {
    float m4[4], l4[4], a4[4][E];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int su = s + u * W;
      const bool valid = su < n;
      const size_t idx = base + (size_t)(valid ? su : s) * p.hq;
      m4[u] = valid ? p.part_m[idx] : -INFINITY;
      l4[u] = p.part_l[idx];
#pragma unroll
      for (int e = 0; e < E; ++e) a4[u][e] = p.part_acc[idx * D + lane * E + e];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (m4[u] == -INFINITY) continue;  // (no such piece; every real piece holds at least one token)
      const float m_new = fmaxf(M, m4[u]);
      const float keep = __builtin_amdgcn_exp2f(M - m_new), w = __builtin_amdgcn_exp2f(m4[u] - m_new);
      M = m_new;
      den = den * keep + w * l4[u];
#pragma unroll
      for (int e = 0; e < E; ++e) num[e] = num[e] * keep + w * a4[u][e];
    }
  }
  if (lane == 0) {
    s_m[wave] = M;
    s_den[wave] = den;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) s_num[wave][lane * E + e] = num[e];
  __syncthreads();
  if (wave != 0) return;
  float Mx = -INFINITY;
#pragma unroll
  for (int w = 0; w < W; ++w) Mx = fmaxf(Mx, s_m[w]);
  float dsum = 0.f, nsum[E];
#pragma unroll
  for (int e = 0; e < E; ++e) nsum[e] = 0.f;
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const float wt = s_m[w] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(s_m[w] - Mx);
    dsum += wt * s_den[w];
#pragma unroll
    for (int e = 0; e < E; ++e) nsum[e] += wt * s_num[w][lane * E + e];
  }
  unsigned short* o = (unsigned short*)p.out + ((size_t)b * p.hq + h) * D + lane * E;
#pragma unroll
  for (int e = 0; e < E; ++e) o[e] = Elem<DT>::cvt(nsum[e] / dsum);
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

constexpr uint64_t kTapeBytes = ((uint64_t)(kMaxDecodeBatch + 1) * sizeof(int32_t) + 255) & ~255ull;

// Scratch of vt_attn_decode_static: the same layout as the context workspace (tape table, then the pieces'
// partial results), in device memory that belongs to the loaded code object, so the call allocates nothing.  Every
// GPU the library runs on holds its own copy until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels get the looked-up device address as an argument.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];  // per device: address of its copy of `scratch` (null = not looked up yet)

}  // namespace

int static_scratch_init(int device) {
  if (device < 0 || device >= kMaxDevices) return VT_E_UNSUPPORTED;
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (g_scratch_ptr[device]) return VT_OK;
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
    (void)hipGetLastError();
    return VT_E_DRIVER;
  }
  g_scratch_ptr[device] = ptr;
  return VT_OK;
}

void* static_scratch_ptr(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> g(g_scratch_mu);
  return g_scratch_ptr[device];
}

uint64_t decode_workspace_bytes(uint32_t batch, uint32_t max_pieces, uint32_t hq, uint32_t d) {
  return kTapeBytes + (uint64_t)batch * max_pieces * hq * (d + 2) * sizeof(float);
}

int launch_decode(vt_ctx* ctx, const vt_decode_args* a, const DecodePlan& plan, void* stream, void* workspace,
                  bool allow_profile) {
  if (a->batch > (uint32_t)kMaxDecodeBatch) return VT_E_UNSUPPORTED;
  DecodeParams p;
  p.q = (const char*)a->q;
  p.k_ptrs = (const char* const*)a->k_ptrs;
  p.v_ptrs = (const char* const*)a->v_ptrs;
  p.kv_lens = a->kv_lens;
  char* ws = (char*)workspace;
  p.tape = (int32_t*)ws;
  const size_t n_part = (size_t)a->batch * plan.max_pieces * a->n_q_heads;
  p.part_acc = (float*)(ws + kTapeBytes);
  p.part_m = p.part_acc + n_part * a->head_dim;
  p.part_l = p.part_m + n_part;
  p.out = a->out;
  p.batch = a->batch;
  p.hq = a->n_q_heads;
  p.hkv = a->n_kv_heads;
  p.group = a->n_q_heads / a->n_kv_heads;
  p.sub = (p.group + 15) / 16;
  p.seg_len = plan.seg_len;
  p.max_pieces = plan.max_pieces;
  p.n_seg = plan.n_seg;
  p.scale_log2e = a->scale * 1.4426950408889634f;
  hipStream_t st = (hipStream_t)stream;
  // Groups of more than 16 query heads: one wavefront carries two 16-head blocks of a kv head.
  const uint32_t nb = p.sub > 1 ? 2 : 1;
  const uint64_t waves = (uint64_t)plan.n_seg * a->n_kv_heads * ((p.sub + nb - 1) / nb);
  const uint32_t blocks = (uint32_t)((waves + kWaves - 1) / kWaves);
  const dim3 cgrid(p.hq, a->batch);
  const bool combine = plan.max_pieces > 1;
  if (allow_profile) prof_begin(ctx, 0, st);
#define VT_LAUNCH(DT, DD)                                                                        \
  do {                                                                                           \
    if (nb == 1)                                                                                 \
      hipLaunchKernelGGL((decode_kernel<DT, DD, 1>), dim3(blocks), dim3(64 * kWaves), 0, st, p); \
    else                                                                                         \
      hipLaunchKernelGGL((decode_kernel<DT, DD, 2>), dim3(blocks), dim3(64 * kWaves), 0, st, p); \
    if (allow_profile) prof_end(ctx, st);                                                        \
    if (combine && plan.max_pieces <= 4)                                                         \
      hipLaunchKernelGGL((decode_combine_kernel<DT, DD, 1>), cgrid, dim3(64), 0, st, p);         \
    else if (combine && plan.max_pieces <= 16)                                                   \
      hipLaunchKernelGGL((decode_combine_kernel<DT, DD, 4>), cgrid, dim3(256), 0, st, p);        \
    else if (combine)                                                                            \
      hipLaunchKernelGGL((decode_combine_kernel<DT, DD, 16>), cgrid, dim3(1024), 0, st, p);      \
  } while (0)
  if (a->dtype == VT_BF16 && a->head_dim == 128)
    VT_LAUNCH(VT_BF16, 128);
  else if (a->dtype == VT_BF16 && a->head_dim == 64)
    VT_LAUNCH(VT_BF16, 64);
  else if (a->dtype == VT_F16 && a->head_dim == 128)
    VT_LAUNCH(VT_F16, 128);
  else if (a->dtype == VT_F16 && a->head_dim == 64)
    VT_LAUNCH(VT_F16, 64);
  else
    return VT_E_UNSUPPORTED;
#undef VT_LAUNCH
  return hipGetLastError() == hipSuccess ? VT_OK : VT_E_DRIVER;
}

int launch_append_batch(void* const* k_ptrs, void* const* v_ptrs, const int32_t* kv_lens, const void* k_rows,
                        const void* v_rows, uint32_t batch, uint32_t row_bytes, void* stream) {
  hipLaunchKernelGGL(append_batch_kernel, dim3(batch, 2), dim3(256), 0, (hipStream_t)stream, (char* const*)k_ptrs,
                     (char* const*)v_ptrs, kv_lens, (const char*)k_rows, (const char*)v_rows, row_bytes);
  return hipGetLastError() == hipSuccess ? VT_OK : VT_E_DRIVER;
}

}  // namespace vt
